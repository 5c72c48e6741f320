// Stream kernels, f32 storage (see gspn_fwd_stream.hip).
#include "gspn_fwd_stream_impl.hpp"

namespace gspn {

hipError_t launch_stream_f32(const FwdParams& p, hipStream_t s, bool reverse) {
    return reverse ? launch_stream_part<float, true>(p, s) : launch_stream_part<float, false>(p, s);
}

}  // namespace gspn
