// Whole-line variant of the stream kernel, f16 storage, global scan (see gspn_fwd_stream_staged.hip).
#include "gspn_fwd_stream_staged_impl.hpp"

namespace gspn {

hipError_t launch_stream_staged_f16(const FwdParams& p, bool reverse, hipStream_t s) { return launch_stream_staged_family<f16_t, false>(p, reverse, s); }

}  // namespace gspn
