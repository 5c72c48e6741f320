// Maps beyond 512 rows (two launches: vertical pair, horizontal pair): host-side dispatch.  The kernels live in
// gspn_fwd_stream_big_impl.hpp and are compiled in two translation units: the global scan with normalised weights, and
// the GSPN-local and logits calls.
#include "gspn_fwd_stream_big_impl.hpp"

namespace gspn {

hipError_t launch_stream_big_global(const FwdParams& p, int dtype, bool reverse, hipStream_t s);
hipError_t launch_stream_big_local(const FwdParams& p, int dtype, bool reverse, hipStream_t s);

// reverse: as the first pass of the two-pass backward (maps of up to 1024 rows only)
bool stream_big_applicable(const FwdParams& p, int dtype, bool reverse) {
    const BigPlan t = plan_big(p, dtype);
    return t.ok && !(reverse && t.two_rows);
}

hipError_t launch_stream_big(const FwdParams& p, int dtype, bool reverse, hipStream_t s) {
    return (p.kchunk > 0 || p.logits) ? launch_stream_big_local(p, dtype, reverse, s) : launch_stream_big_global(p, dtype, reverse, s);
}

}  // namespace gspn
