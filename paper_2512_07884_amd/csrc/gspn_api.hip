// C ABI of libgspn: argument validation and dispatch.  See include/gspn.h.
#include "../../include/gspn.h"
#include "gspn_common.hpp"

using namespace gspn;

static_assert(GSPN_PROXY_STATIC_MAX_FLOATS == PROXY_SCRATCH_FLOATS, "the header states the size of the static workspace");

namespace {

inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

int check_common(int B, int C, int H, int W, int G, unsigned dir_mask, int dtype, unsigned flags) {
    if (B < 1 || C < 1 || H < 1 || W < 1 || G < 1) return GSPN_ERR_SHAPE;
    if (C % G != 0) return GSPN_ERR_SHAPE;
    if (dir_mask == 0 || dir_mask > 15u) return GSPN_ERR_SHAPE;
    if (dtype != GSPN_F32 && dtype != GSPN_BF16 && dtype != GSPN_F16) return GSPN_ERR_DTYPE;
    if (flags & ~(unsigned)GSPN_FLAG_SHARED_PARAMS) return GSPN_ERR_UNSUPPORTED;
    if (H > GSPN_MAX_LINE || W > GSPN_MAX_LINE) return GSPN_ERR_UNSUPPORTED;
    // plane offsets inside a (batch, channel) image are 32-bit in the kernels
    if ((long long)H * W * 3 >= (1ll << 31)) return GSPN_ERR_UNSUPPORTED;
    return GSPN_OK;
}

// a stretch at least as long as both axes is the global scan: 0 for the kernels
int effective_kchunk(int kchunk, int H, int W) { return (kchunk >= H && kchunk >= W) ? 0 : kchunk; }

}  // namespace

extern "C" {

static int scan_fwd_any(const void* x, const void* w, const void* lam, const void* u,
                        void* y, void* h_save,
                        int B, int C, int H, int W, int G, int kchunk, int logits,
                        unsigned dir_mask, int dtype, unsigned flags, void* stream) {
    if (!x || !w || !lam || !u || !y) return GSPN_ERR_NULL;
    int st = check_common(B, C, H, W, G, dir_mask, dtype, flags);
    if (st != GSPN_OK) return st;
    if (kchunk < 1) return GSPN_ERR_SHAPE;
    if (logits && (H > GSPN_MAX_LINE_LOGITS || W > GSPN_MAX_LINE_LOGITS)) return GSPN_ERR_UNSUPPORTED;
    if (misaligned(x) || misaligned(w) || misaligned(lam) || misaligned(u) || misaligned(y) ||
        (h_save && misaligned(h_save)))
        return GSPN_ERR_ALIGN;
    FwdParams p = {};
    p.x = x; p.w = w; p.lam = lam; p.u = u; p.y = y; p.hs = h_save;
    p.B = B; p.C = C; p.H = H; p.W = W; p.G = G; p.cpg = C / G;
    p.mask = dir_mask; p.shared = (flags & GSPN_FLAG_SHARED_PARAMS) ? 1 : 0;
    p.kchunk = effective_kchunk(kchunk, H, W);
    p.logits = logits;
    hipError_t e = launch_fwd(p, dtype, (hipStream_t)stream);
    return e == hipSuccess ? GSPN_OK : GSPN_ERR_HIP;
}

int gspn_scan_fwd_transposed(const void* x, const void* xt, const void* w, const void* lam, const void* u, void* y,
                             int B, int C, int H, int W, int G,
                             unsigned dir_mask, int dtype, unsigned flags, void* stream) {
    if (!x || !xt || !w || !lam || !u || !y) return GSPN_ERR_NULL;
    int st = check_common(B, C, H, W, G, dir_mask, dtype, flags);
    if (st != GSPN_OK) return st;
    if (misaligned(x) || misaligned(xt) || misaligned(w) || misaligned(lam) || misaligned(u) || misaligned(y))
        return GSPN_ERR_ALIGN;
    FwdParams p = {};
    p.x = x; p.xt = xt; p.w = w; p.lam = lam; p.u = u; p.y = y; p.hs = nullptr;
    p.B = B; p.C = C; p.H = H; p.W = W; p.G = G; p.cpg = C / G;
    p.mask = dir_mask; p.shared = (flags & GSPN_FLAG_SHARED_PARAMS) ? 1 : 0;
    hipError_t e = launch_fwd(p, dtype, (hipStream_t)stream);
    return e == hipSuccess ? GSPN_OK : GSPN_ERR_HIP;
}

int gspn_scan_fwd_unfused(const void* x, const void* w, const void* lam, const void* u, void* y, void* h_save,
                          void* workspace, unsigned long long workspace_bytes,
                          int B, int C, int H, int W, int G,
                          unsigned dir_mask, int dtype, unsigned flags, void* stream) {
    if (!x || !w || !lam || !u || !y || !workspace) return GSPN_ERR_NULL;
    int st = check_common(B, C, H, W, G, dir_mask, dtype, flags);
    if (st != GSPN_OK) return st;
    if (misaligned(x) || misaligned(w) || misaligned(lam) || misaligned(u) || misaligned(y) || misaligned(workspace) ||
        (h_save && misaligned(h_save)))
        return GSPN_ERR_ALIGN;
    if (workspace_bytes < unfused_workspace_bytes(B, C, H, W)) return GSPN_ERR_SHAPE;
    FwdParams p = {};
    p.x = x; p.w = w; p.lam = lam; p.u = u; p.y = y; p.hs = h_save;
    p.B = B; p.C = C; p.H = H; p.W = W; p.G = G; p.cpg = C / G;
    p.mask = dir_mask; p.shared = (flags & GSPN_FLAG_SHARED_PARAMS) ? 1 : 0;
    hipError_t e = launch_fwd_unfused(p, dtype, workspace, (hipStream_t)stream);
    return e == hipSuccess ? GSPN_OK : GSPN_ERR_HIP;
}

unsigned long long gspn_unfused_workspace_bytes(int B, int C, int H, int W) {
    if (B < 1 || C < 1 || H < 1 || W < 1) return 0;
    return unfused_workspace_bytes(B, C, H, W);
}

const char* gspn_fwd_transposed_plan(int B, int C, int H, int W, int G, unsigned dir_mask, int dtype, unsigned flags) {
    if (check_common(B, C, H, W, G, dir_mask, dtype, flags) != GSPN_OK) return "invalid";
    FwdParams p = {};
    p.xt = (const void*)16;
    p.B = B; p.C = C; p.H = H; p.W = W; p.G = G; p.cpg = C / G; p.mask = dir_mask;
    p.shared = (flags & GSPN_FLAG_SHARED_PARAMS) ? 1 : 0;
    return fwd_plan_name(p, dtype);
}

int gspn_scan_fwd_local(const void* x, const void* w, const void* lam, const void* u,
                        void* y, void* h_save,
                        int B, int C, int H, int W, int G, int kchunk,
                        unsigned dir_mask, int dtype, unsigned flags, void* stream) {
    return scan_fwd_any(x, w, lam, u, y, h_save, B, C, H, W, G, kchunk, 0, dir_mask, dtype, flags, stream);
}

int gspn_scan_fwd_logits(const void* x, const void* z, const void* lam, const void* u,
                         void* y, void* h_save,
                         int B, int C, int H, int W, int G, int kchunk,
                         unsigned dir_mask, int dtype, unsigned flags, void* stream) {
    return scan_fwd_any(x, z, lam, u, y, h_save, B, C, H, W, G, kchunk, 1, dir_mask, dtype, flags, stream);
}

int gspn_scan_fwd(const void* x, const void* w, const void* lam, const void* u,
                  void* y, void* h_save,
                  int B, int C, int H, int W, int G,
                  unsigned dir_mask, int dtype, unsigned flags, void* stream) {
    return gspn_scan_fwd_local(x, w, lam, u, y, h_save, B, C, H, W, G, GSPN_MAX_LINE, dir_mask, dtype, flags, stream);
}

static int scan_bwd_any(const void* gy, const void* x, const void* w, const void* lam, const void* u,
                        const void* h_save,
                        void* gx, void* gw, void* glam, void* gu,
                        int B, int C, int H, int W, int G, int kchunk, int logits,
                        unsigned dir_mask, int dtype, unsigned flags, void* stream) {
    if (!gy || !x || !w || !lam || !u || !h_save || !gx || !gw || !glam || !gu) return GSPN_ERR_NULL;
    int st = check_common(B, C, H, W, G, dir_mask, dtype, flags);
    if (st != GSPN_OK) return st;
    if (kchunk < 1) return GSPN_ERR_SHAPE;
    if (logits && (H > GSPN_MAX_LINE_LOGITS || W > GSPN_MAX_LINE_LOGITS)) return GSPN_ERR_UNSUPPORTED;
    if (misaligned(gy) || misaligned(x) || misaligned(w) || misaligned(lam) || misaligned(u) ||
        misaligned(h_save) || misaligned(gx) || misaligned(gw) || misaligned(glam) || misaligned(gu))
        return GSPN_ERR_ALIGN;
    BwdParams p;
    p.gy = gy; p.x = x; p.w = w; p.lam = lam; p.u = u; p.hs = h_save;
    p.gx = gx; p.gw = gw; p.glam = glam; p.gu = gu;
    p.B = B; p.C = C; p.H = H; p.W = W; p.G = G; p.cpg = C / G;
    p.mask = dir_mask; p.shared = (flags & GSPN_FLAG_SHARED_PARAMS) ? 1 : 0;
    p.kchunk = effective_kchunk(kchunk, H, W);
    p.logits = logits;
    hipError_t e = launch_bwd(p, dtype, (hipStream_t)stream);
    return e == hipSuccess ? GSPN_OK : GSPN_ERR_HIP;
}

int gspn_scan_bwd_local(const void* gy, const void* x, const void* w, const void* lam, const void* u,
                        const void* h_save,
                        void* gx, void* gw, void* glam, void* gu,
                        int B, int C, int H, int W, int G, int kchunk,
                        unsigned dir_mask, int dtype, unsigned flags, void* stream) {
    return scan_bwd_any(gy, x, w, lam, u, h_save, gx, gw, glam, gu, B, C, H, W, G, kchunk, 0, dir_mask, dtype, flags, stream);
}

int gspn_scan_bwd_logits(const void* gy, const void* x, const void* z, const void* lam, const void* u,
                         const void* h_save,
                         void* gx, void* gz, void* glam, void* gu,
                         int B, int C, int H, int W, int G, int kchunk,
                         unsigned dir_mask, int dtype, unsigned flags, void* stream) {
    return scan_bwd_any(gy, x, z, lam, u, h_save, gx, gz, glam, gu, B, C, H, W, G, kchunk, 1, dir_mask, dtype, flags, stream);
}

int gspn_scan_bwd(const void* gy, const void* x, const void* w, const void* lam, const void* u,
                  const void* h_save,
                  void* gx, void* gw, void* glam, void* gu,
                  int B, int C, int H, int W, int G,
                  unsigned dir_mask, int dtype, unsigned flags, void* stream) {
    return gspn_scan_bwd_local(gy, x, w, lam, u, h_save, gx, gw, glam, gu, B, C, H, W, G, GSPN_MAX_LINE,
                               dir_mask, dtype, flags, stream);
}

static const char* fwd_plan_any(int B, int C, int H, int W, int G, int kchunk, int logits, unsigned dir_mask, int dtype,
                                unsigned flags, int has_h_save) {
    if (check_common(B, C, H, W, G, dir_mask, dtype, flags) != GSPN_OK || kchunk < 1) return "invalid";
    if (logits && (H > GSPN_MAX_LINE_LOGITS || W > GSPN_MAX_LINE_LOGITS)) return "invalid";
    FwdParams p = {};
    p.logits = logits;
    p.B = B; p.C = C; p.H = H; p.W = W; p.G = G; p.cpg = C / G; p.mask = dir_mask;
    p.shared = (flags & GSPN_FLAG_SHARED_PARAMS) ? 1 : 0;
    p.kchunk = effective_kchunk(kchunk, H, W);
    p.hs = has_h_save ? (void*)16 : nullptr;
    return fwd_plan_name(p, dtype);
}

const char* gspn_fwd_local_plan(int B, int C, int H, int W, int G, int kchunk, unsigned dir_mask, int dtype,
                                unsigned flags, int has_h_save) {
    return fwd_plan_any(B, C, H, W, G, kchunk, 0, dir_mask, dtype, flags, has_h_save);
}
const char* gspn_fwd_logits_plan(int B, int C, int H, int W, int G, int kchunk, unsigned dir_mask, int dtype,
                                 unsigned flags, int has_h_save) {
    return fwd_plan_any(B, C, H, W, G, kchunk, 1, dir_mask, dtype, flags, has_h_save);
}

static const char* bwd_plan_any(int B, int C, int H, int W, int G, int kchunk, int logits, unsigned dir_mask, int dtype,
                                unsigned flags) {
    if (check_common(B, C, H, W, G, dir_mask, dtype, flags) != GSPN_OK || kchunk < 1) return "invalid";
    if (logits && (H > GSPN_MAX_LINE_LOGITS || W > GSPN_MAX_LINE_LOGITS)) return "invalid";
    BwdParams p = {};
    p.logits = logits;
    p.B = B; p.C = C; p.H = H; p.W = W; p.G = G; p.cpg = C / G; p.mask = dir_mask;
    p.shared = (flags & GSPN_FLAG_SHARED_PARAMS) ? 1 : 0;
    p.kchunk = effective_kchunk(kchunk, H, W);
    return bwd_plan_name(p, dtype);
}

const char* gspn_bwd_local_plan(int B, int C, int H, int W, int G, int kchunk, unsigned dir_mask, int dtype,
                                unsigned flags) {
    return bwd_plan_any(B, C, H, W, G, kchunk, 0, dir_mask, dtype, flags);
}
const char* gspn_bwd_logits_plan(int B, int C, int H, int W, int G, int kchunk, unsigned dir_mask, int dtype,
                                 unsigned flags) {
    return bwd_plan_any(B, C, H, W, G, kchunk, 1, dir_mask, dtype, flags);
}

const char* gspn_fwd_plan(int B, int C, int H, int W, int G, unsigned dir_mask, int dtype, unsigned flags,
                          int has_h_save) {
    return gspn_fwd_local_plan(B, C, H, W, G, GSPN_MAX_LINE, dir_mask, dtype, flags, has_h_save);
}

const char* gspn_bwd_plan(int B, int C, int H, int W, int G, unsigned dir_mask, int dtype, unsigned flags) {
    return gspn_bwd_local_plan(B, C, H, W, G, GSPN_MAX_LINE, dir_mask, dtype, flags);
}

int gspn_proxy_project(const void* in, const void* P, void* out, int B, int K, int M, int H, int W, int dtype,
                       void* stream) {
    if (!in || !P || !out) return GSPN_ERR_NULL;
    if (B < 1 || K < 1 || M < 1 || H < 1 || W < 1) return GSPN_ERR_SHAPE;
    if (dtype != GSPN_F32 && dtype != GSPN_BF16 && dtype != GSPN_F16) return GSPN_ERR_DTYPE;
    if (H > GSPN_MAX_LINE || W > GSPN_MAX_LINE) return GSPN_ERR_UNSUPPORTED;
    if ((long long)H * W >= (1ll << 31)) return GSPN_ERR_UNSUPPORTED;
    if (misaligned(in) || misaligned(P) || misaligned(out)) return GSPN_ERR_ALIGN;
    hipError_t e = launch_proxy_project(in, P, out, B, K, M, H * W, dtype, (hipStream_t)stream);
    return e == hipSuccess ? GSPN_OK : GSPN_ERR_HIP;
}

int gspn_proxy_project_bwd(const void* gout, const void* in, const void* P, void* gin, float* gP, float* partial,
                           int B, int K, int M, int H, int W, int dtype, void* stream) {
    if (!gout || !in || !P || (!gin && !gP) || (gP && !partial)) return GSPN_ERR_NULL;
    if (B < 1 || K < 1 || M < 1 || H < 1 || W < 1) return GSPN_ERR_SHAPE;
    if (dtype != GSPN_F32 && dtype != GSPN_BF16 && dtype != GSPN_F16) return GSPN_ERR_DTYPE;
    if (H > GSPN_MAX_LINE || W > GSPN_MAX_LINE) return GSPN_ERR_UNSUPPORTED;
    if ((long long)H * W >= (1ll << 31) || (long long)M * K >= (1ll << 31)) return GSPN_ERR_UNSUPPORTED;
    if (misaligned(gout) || misaligned(in) || misaligned(P) || misaligned(gin) || misaligned(gP) || misaligned(partial))
        return GSPN_ERR_ALIGN;
    hipError_t e = launch_proxy_project_bwd(gout, in, P, gin, gP, partial, B, K, M, H * W, dtype, (hipStream_t)stream);
    return e == hipSuccess ? GSPN_OK : GSPN_ERR_HIP;
}

int gspn_proxy_project_bwd_static(const void* gout, const void* in, const void* P, void* gin, float* gP,
                                  int B, int K, int M, int H, int W, int dtype, void* stream) {
    if (!gout || !in || !P || (!gin && !gP)) return GSPN_ERR_NULL;
    if (B < 1 || K < 1 || M < 1 || H < 1 || W < 1) return GSPN_ERR_SHAPE;
    if (dtype != GSPN_F32 && dtype != GSPN_BF16 && dtype != GSPN_F16) return GSPN_ERR_DTYPE;
    if (H > GSPN_MAX_LINE || W > GSPN_MAX_LINE) return GSPN_ERR_UNSUPPORTED;
    if ((long long)H * W >= (1ll << 31) || (long long)M * K >= (1ll << 31)) return GSPN_ERR_UNSUPPORTED;
    if (gP && (long long)B * M * K > (long long)GSPN_PROXY_STATIC_MAX_FLOATS) return GSPN_ERR_UNSUPPORTED;
    if (misaligned(gout) || misaligned(in) || misaligned(P) || misaligned(gin) || misaligned(gP)) return GSPN_ERR_ALIGN;
    hipError_t e = launch_proxy_project_bwd_static(gout, in, P, gin, gP, B, K, M, H * W, dtype, (hipStream_t)stream);
    return e == hipSuccess ? GSPN_OK : GSPN_ERR_HIP;
}

const char* gspn_proxy_plan(int B, int K, int M, int H, int W, int dtype) {
    if (B < 1 || K < 1 || M < 1 || H < 1 || W < 1 || (dtype != GSPN_F32 && dtype != GSPN_BF16 && dtype != GSPN_F16)) return "invalid";
    if (H > GSPN_MAX_LINE || W > GSPN_MAX_LINE || (long long)H * W >= (1ll << 31)) return "invalid";
    return proxy_mfma_applicable(B, K, M, H * W, dtype) ? "mfma" : "fma";
}

const char* gspn_status_string(int status) {
    switch (status) {
        case GSPN_OK: return "ok";
        case GSPN_ERR_NULL: return "a required pointer is NULL";
        case GSPN_ERR_SHAPE: return "bad shape: dimensions and kchunk must be >= 1, C divisible by G, dir_mask in 1..15";
        case GSPN_ERR_DTYPE: return "dtype must be GSPN_F32, GSPN_BF16 or GSPN_F16";
        case GSPN_ERR_ALIGN: return "pointers must be 16-byte aligned";
        case GSPN_ERR_UNSUPPORTED: return "unsupported: line longer than GSPN_MAX_LINE (GSPN_MAX_LINE_LOGITS with logits), unknown flag, or B*M*K beyond the static workspace";
        case GSPN_ERR_HIP: return "HIP launch failed";
        default: return "unknown status";
    }
}

int gspn_version(void) { return 300; }   // 0.3.0: testing aids read once (gspn_reload_env)

void gspn_reload_env(void) { reload_env_knobs(); }

}  // extern "C"
