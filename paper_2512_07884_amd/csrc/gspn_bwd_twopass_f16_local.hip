// Reverse sweep of the two-pass backward scan on the forward tile machinery, fp16 storage, GSPN-local and logits
// (see gspn_bwd_twopass.hip).
#include "gspn_fwd_tile_impl.hpp"

namespace gspn {

hipError_t launch_reverse_sweep_f16_local(const FwdParams& p, hipStream_t s) { return launch_reverse_sweep_part<f16_t, true>(p, s); }

}  // namespace gspn
