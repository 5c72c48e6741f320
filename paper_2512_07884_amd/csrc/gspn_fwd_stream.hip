// Stream kernels (maps too large for an on-chip output tile): host-side dispatch.  The kernels live in
// gspn_fwd_stream_impl.hpp and are compiled in two translation units, by storage type.
#include "gspn_fwd_stream_impl.hpp"

namespace gspn {

hipError_t launch_stream_f32(const FwdParams& p, hipStream_t s, bool reverse);
hipError_t launch_stream_bf16(const FwdParams& p, hipStream_t s, bool reverse);

bool fwd_stream_applicable(const FwdParams& p, int dtype) { return plan_stream(p, dtype).ok; }
bool reverse_sweep_stream_applicable(const FwdParams& p, int dtype) { return plan_stream(p, dtype).ok; }

hipError_t launch_fwd_stream(const FwdParams& p, int dtype, hipStream_t s) {
    return dtype == 0 ? launch_stream_f32(p, s, false) : launch_stream_bf16(p, s, false);
}

hipError_t launch_reverse_sweep_stream(const FwdParams& p, int dtype, hipStream_t s) {
    return dtype == 0 ? launch_stream_f32(p, s, true) : launch_stream_bf16(p, s, true);
}

}  // namespace gspn
