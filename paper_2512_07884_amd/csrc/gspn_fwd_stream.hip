// Stream kernels (maps too large for an on-chip output tile): host-side dispatch.  The kernels live in
// gspn_fwd_stream_impl.hpp and are compiled in three translation units, by storage type.
#include "gspn_fwd_stream_impl.hpp"

namespace gspn {

hipError_t launch_stream_f32(const FwdParams& p, hipStream_t s, bool reverse);
hipError_t launch_stream_bf16(const FwdParams& p, hipStream_t s, bool reverse);
hipError_t launch_stream_f16(const FwdParams& p, hipStream_t s, bool reverse);
// 16-bit storage (global scan, GSPN-local, logits): horizontal phases with whole-line requests
// (gspn_fwd_stream_staged.hip)
bool stream_staged_applicable(const FwdParams& p, int dtype);
hipError_t launch_stream_staged(const FwdParams& p, int dtype, bool reverse, hipStream_t s);

// maps of up to 2048 rows (reverse sweep: 1024) / lines of up to 2048 positions, global scan: two launches
// (gspn_fwd_stream_big.hip)
bool stream_big_applicable(const FwdParams& p, int dtype, bool reverse);
hipError_t launch_stream_big(const FwdParams& p, int dtype, bool reverse, hipStream_t s);

bool fwd_stream_applicable(const FwdParams& p, int dtype) { return plan_stream(p, dtype).ok || stream_big_applicable(p, dtype, false); }
bool reverse_sweep_stream_applicable(const FwdParams& p, int dtype) { return plan_stream(p, dtype).ok || stream_big_applicable(p, dtype, true); }

static hipError_t launch_stream_general(const FwdParams& p, int dtype, hipStream_t s, bool reverse) {
    if (dtype == 0) return launch_stream_f32(p, s, reverse);
    return dtype == 1 ? launch_stream_bf16(p, s, reverse) : launch_stream_f16(p, s, reverse);
}

hipError_t launch_fwd_stream(const FwdParams& p, int dtype, hipStream_t s) {
    if (!plan_stream(p, dtype).ok) return launch_stream_big(p, dtype, false, s);
    if (staged_stream_enabled() && stream_staged_applicable(p, dtype)) return launch_stream_staged(p, dtype, false, s);
    return launch_stream_general(p, dtype, s, false);
}

hipError_t launch_reverse_sweep_stream(const FwdParams& p, int dtype, hipStream_t s) {
    if (!plan_stream(p, dtype).ok) return launch_stream_big(p, dtype, true, s);
    if (staged_stream_enabled() && stream_staged_applicable(p, dtype)) return launch_stream_staged(p, dtype, true, s);
    return launch_stream_general(p, dtype, s, true);
}

}  // namespace gspn
