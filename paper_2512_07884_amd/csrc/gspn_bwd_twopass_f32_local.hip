// Reverse sweep of the two-pass backward scan on the forward tile machinery, f32 storage, GSPN-local and logits calls
// (see gspn_bwd_twopass.hip).
#include "gspn_fwd_tile_impl.hpp"

namespace gspn {

hipError_t launch_reverse_sweep_f32_local(const FwdParams& p, hipStream_t s) { return launch_reverse_sweep_part<float, true>(p, s); }

}  // namespace gspn
