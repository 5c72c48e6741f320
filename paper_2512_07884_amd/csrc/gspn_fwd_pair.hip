// Two-channel kernel of the 128x128 maps in 16-bit storage: host-side dispatch.  The kernel lives in
// gspn_fwd_pair_impl.hpp and is compiled in two translation units, by storage type.
#include "gspn_fwd_pair_impl.hpp"

namespace gspn {

hipError_t launch_pair_bf16(const FwdParams& p, bool reverse, hipStream_t s);
hipError_t launch_pair_f16(const FwdParams& p, bool reverse, hipStream_t s);

bool fwd_pair_applicable(const FwdParams& p, int dtype) { return pair_shape_ok(p, dtype); }

hipError_t launch_fwd_pair(const FwdParams& p, int dtype, hipStream_t s) {
    if (!pair_shape_ok(p, dtype)) return hipErrorInvalidValue;
    return dtype == 1 ? launch_pair_bf16(p, false, s) : launch_pair_f16(p, false, s);
}

bool reverse_sweep_pair_applicable(const FwdParams& p, int dtype) { return pair_shape_ok(p, dtype) && p.hs; }

hipError_t launch_reverse_sweep_pair(const FwdParams& p, int dtype, hipStream_t s) {
    if (!reverse_sweep_pair_applicable(p, dtype)) return hipErrorInvalidValue;
    return dtype == 1 ? launch_pair_bf16(p, true, s) : launch_pair_f16(p, true, s);
}

}  // namespace gspn
