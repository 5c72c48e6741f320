// Whole-line variant of the stream kernel (16-bit storage): host-side dispatch.  The kernels live in
// gspn_fwd_stream_staged_impl.hpp and are compiled in six translation units, by storage type and family (global scan /
// GSPN-local / weights as logits).
#include "gspn_fwd_stream_staged_impl.hpp"

namespace gspn {

hipError_t launch_stream_staged_bf16(const FwdParams& p, bool reverse, hipStream_t s);
hipError_t launch_stream_staged_f16(const FwdParams& p, bool reverse, hipStream_t s);
hipError_t launch_stream_staged_bf16_local(const FwdParams& p, bool reverse, hipStream_t s);
hipError_t launch_stream_staged_f16_local(const FwdParams& p, bool reverse, hipStream_t s);
hipError_t launch_stream_staged_bf16_logits(const FwdParams& p, bool reverse, hipStream_t s);
hipError_t launch_stream_staged_f16_logits(const FwdParams& p, bool reverse, hipStream_t s);

bool stream_staged_applicable(const FwdParams& p, int dtype) { return staged_shape_ok(p, dtype); }

hipError_t launch_stream_staged(const FwdParams& p, int dtype, bool reverse, hipStream_t s) {
    if (!staged_shape_ok(p, dtype)) return hipErrorInvalidValue;
    if (p.logits) return dtype == 1 ? launch_stream_staged_bf16_logits(p, reverse, s) : launch_stream_staged_f16_logits(p, reverse, s);
    if (p.kchunk > 0) return dtype == 1 ? launch_stream_staged_bf16_local(p, reverse, s) : launch_stream_staged_f16_local(p, reverse, s);
    return dtype == 1 ? launch_stream_staged_bf16(p, reverse, s) : launch_stream_staged_f16(p, reverse, s);
}

}  // namespace gspn
