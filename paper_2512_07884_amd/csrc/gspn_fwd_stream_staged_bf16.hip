// Whole-line variant of the stream kernel, bf16 storage (see gspn_fwd_stream_staged.hip).
#include "gspn_fwd_stream_staged_impl.hpp"

namespace gspn {

hipError_t launch_stream_staged_bf16(const FwdParams& p, bool reverse, hipStream_t s) { return launch_stream_staged_typed<bf16_t>(p, reverse, s); }

}  // namespace gspn
