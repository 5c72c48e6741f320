// Forward tile kernels: host-side choice of the instantiation.  The kernels live in gspn_fwd_tile_impl.hpp and are
// compiled in six translation units, by storage type and by family (global scan / GSPN-local and logits).
#include "gspn_fwd_tile_impl.hpp"

namespace gspn {

hipError_t launch_fwd_tile_f32_global(const FwdParams& p, hipStream_t s);
hipError_t launch_fwd_tile_f32_local(const FwdParams& p, hipStream_t s);
hipError_t launch_fwd_tile_bf16_global(const FwdParams& p, hipStream_t s);
hipError_t launch_fwd_tile_bf16_local(const FwdParams& p, hipStream_t s);
hipError_t launch_fwd_tile_f16_global(const FwdParams& p, hipStream_t s);
hipError_t launch_fwd_tile_f16_local(const FwdParams& p, hipStream_t s);

bool fwd_tile_applicable(const FwdParams& p, int dtype) { return plan_tile(p, dtype).ok; }

hipError_t launch_fwd_tile(const FwdParams& p, int dtype, hipStream_t s) {
    const bool local = p.kchunk > 0 || p.logits;
    if (dtype == 0) return local ? launch_fwd_tile_f32_local(p, s) : launch_fwd_tile_f32_global(p, s);
    if (dtype == 1) return local ? launch_fwd_tile_bf16_local(p, s) : launch_fwd_tile_bf16_global(p, s);
    return local ? launch_fwd_tile_f16_local(p, s) : launch_fwd_tile_f16_global(p, s);
}

}  // namespace gspn
