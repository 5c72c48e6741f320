// Stream kernels, fp16 storage (see gspn_fwd_stream.hip).
#include "gspn_fwd_stream_impl.hpp"

namespace gspn {

hipError_t launch_stream_f16(const FwdParams& p, hipStream_t s, bool reverse) {
    return reverse ? launch_stream_part<f16_t, true>(p, s) : launch_stream_part<f16_t, false>(p, s);
}

}  // namespace gspn
