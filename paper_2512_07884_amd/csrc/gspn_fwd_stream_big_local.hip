// Maps beyond 512 rows, GSPN-local calls (see gspn_fwd_stream_big.hip).
#include "gspn_fwd_stream_big_impl.hpp"

namespace gspn {

hipError_t launch_stream_big_local(const FwdParams& p, int dtype, bool reverse, hipStream_t s) {
    return launch_big_family<true, false>(p, dtype, reverse, s);
}

}  // namespace gspn
