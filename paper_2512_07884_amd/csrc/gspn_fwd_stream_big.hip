// Maps beyond 512 rows (two launches: vertical pair, horizontal pair): host-side dispatch.  The kernels live in
// gspn_fwd_stream_big_impl.hpp and are compiled in three translation units: the global scan with normalised weights, the
// GSPN-local calls, and the calls with the weights as logits.
#include "gspn_fwd_stream_big_impl.hpp"

namespace gspn {

hipError_t launch_stream_big_global(const FwdParams& p, int dtype, bool reverse, hipStream_t s);
hipError_t launch_stream_big_local(const FwdParams& p, int dtype, bool reverse, hipStream_t s);
hipError_t launch_stream_big_logits(const FwdParams& p, int dtype, bool reverse, hipStream_t s);

// reverse: as the first pass of the two-pass backward (maps of up to 1024 rows only)
bool stream_big_applicable(const FwdParams& p, int dtype, bool reverse) {
    const BigPlan t = plan_big(p, dtype);
    return t.ok && !(reverse && t.two_rows);
}

hipError_t launch_stream_big(const FwdParams& p, int dtype, bool reverse, hipStream_t s) {
    if (p.logits) return launch_stream_big_logits(p, dtype, reverse, s);
    return p.kchunk > 0 ? launch_stream_big_local(p, dtype, reverse, s) : launch_stream_big_global(p, dtype, reverse, s);
}

}  // namespace gspn
