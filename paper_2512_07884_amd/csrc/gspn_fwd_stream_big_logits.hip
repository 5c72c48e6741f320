// Maps beyond 512 rows, calls with the weights as logits (see gspn_fwd_stream_big.hip).
#include "gspn_fwd_stream_big_impl.hpp"

namespace gspn {

hipError_t launch_stream_big_logits(const FwdParams& p, int dtype, bool reverse, hipStream_t s) {
    return launch_big_family<true, true>(p, dtype, reverse, s);
}

}  // namespace gspn
