// Chooses the kernel family for a call.  Host code only.
#include "gspn_common.hpp"

namespace gspn {

enum FwdPlan { FWD_GENERIC = 0 };
enum BwdPlan { BWD_GENERIC = 0 };

static FwdPlan choose_fwd(const FwdParams&, int) { return FWD_GENERIC; }
static BwdPlan choose_bwd(const BwdParams&, int) { return BWD_GENERIC; }

hipError_t launch_fwd(const FwdParams& p, int dtype, hipStream_t s) {
    switch (choose_fwd(p, dtype)) {
        default: return launch_fwd_generic(p, dtype, s);
    }
}

hipError_t launch_bwd(const BwdParams& p, int dtype, hipStream_t s) {
    switch (choose_bwd(p, dtype)) {
        default: return launch_bwd_generic(p, dtype, s);
    }
}

const char* fwd_plan_name(const FwdParams& p, int dtype) {
    switch (choose_fwd(p, dtype)) {
        default: return "generic";
    }
}

const char* bwd_plan_name(const BwdParams& p, int dtype) {
    switch (choose_bwd(p, dtype)) {
        default: return "generic";
    }
}

}  // namespace gspn
