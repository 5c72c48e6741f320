// Whole-line variant of the stream kernel, bf16 storage, weights as logits (see gspn_fwd_stream_staged.hip).
#include "gspn_fwd_stream_staged_impl.hpp"

namespace gspn {

hipError_t launch_stream_staged_bf16_logits(const FwdParams& p, bool reverse, hipStream_t s) { return launch_stream_staged_family<bf16_t, true, true>(p, reverse, s); }

}  // namespace gspn
