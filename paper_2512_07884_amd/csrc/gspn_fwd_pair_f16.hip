// Two-channel kernel of the 128x128 maps, f16 storage (see gspn_fwd_pair.hip).
#include "gspn_fwd_pair_impl.hpp"

namespace gspn {

hipError_t launch_pair_f16(const FwdParams& p, bool reverse, hipStream_t s) { return launch_pair_typed<f16_t>(p, reverse, s); }

}  // namespace gspn
