// Forward tile kernels, one translation unit of six (see gspn_fwd_tile.hip).
#include "gspn_fwd_tile_impl.hpp"

namespace gspn {

hipError_t launch_fwd_tile_f16_local(const FwdParams& p, hipStream_t s) { return launch_fwd_tile_part<f16_t, true>(p, s); }

}  // namespace gspn
