// COMPARATOR, NOT A PRODUCT PATH.  The scan the way the first GSPN implementation ran it, as the paper describes it
// (Sec. 3.3; the step-by-step figure and Table 1 of Sec. 5.1): one small kernel launch PER LINE and per direction, the
// hidden state of the previous line handed from launch to launch through global memory, no fusion over lines or
// directions.  It exists so that the fused kernels can be measured against the structure they replace on the same
// hardware (bench.py --unfused); the dispatcher never selects it.
//
// Per launch (direction d, scan step t): every (image, channel, position j) computes Eq. 1 for its element from the
// previous line in the caller's workspace, stores its state into the other half of the workspace and adds u*h to y
// (first direction of the call: stores it).  States travel in fp32; y is accumulated in storage precision direction by
// direction, like the other kernels that merge through global memory.
#include "gspn_common.hpp"

namespace gspn {
namespace {

template <typename T>
__global__ void __launch_bounds__(256) line_step_kernel(FwdParams p, float* h_prev, float* h_cur, int d, int t, int first_dir) {
    const DirGeom gm = dir_geom(d, p.H, p.W);
    const int L = gm.L;
    const size_t n = (size_t)p.B * p.C * L;
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n) return;
    const int j = (int)(idx % L);
    const size_t bc = idx / L;
    const int c = (int)(bc % p.C), b = (int)(bc / p.C);
    const int g = c / p.cpg;
    const int HW = p.H * p.W;
    const int line = gm.reversed ? gm.S - 1 - t : t;
    const size_t pix = (size_t)line * gm.stride_s + (size_t)j * gm.stride_j;
    const size_t planes = (size_t)p.B * p.C;
    const size_t slot_c = p.shared ? 0 : (size_t)d * planes * HW;
    const size_t slot_w = p.shared ? 0 : (size_t)d * p.B * p.G * 3 * HW;
    const size_t plane = bc * HW;
    const T* X = (const T*)p.x + plane;
    const T* LAM = (const T*)p.lam + slot_c + plane;
    const T* U = (const T*)p.u + slot_c + plane;
    const T* Wt = (const T*)p.w + slot_w + ((size_t)b * p.G + g) * 3 * HW;
    float h = ldf(LAM + pix) * ldf(X + pix);
    if (t > 0) {
        // an out-of-line neighbour contributes 0 whatever weight is stored for it
        const float* hp = h_prev + bc * L;
        const float l = j > 0 ? hp[j - 1] : 0.f, m = hp[j], r = j + 1 < L ? hp[j + 1] : 0.f;
        const float w0 = j > 0 ? ldf(Wt + pix) : 0.f, w1 = ldf(Wt + HW + pix), w2 = j + 1 < L ? ldf(Wt + 2 * (size_t)HW + pix) : 0.f;
        h = fmaf(w0, l, fmaf(w1, m, fmaf(w2, r, h)));
    }
    h_cur[bc * L + j] = h;
    T* Y = (T*)p.y + plane;
    const float yv = ldf(U + pix) * h;
    stf(Y + pix, first_dir ? yv : ldf(Y + pix) + yv);
    if (p.hs) stf((T*)p.hs + (size_t)d * planes * HW + plane + pix, h);
}

}  // namespace

size_t unfused_workspace_bytes(int B, int C, int H, int W) {
    return (size_t)2 * B * C * (H > W ? H : W) * sizeof(float);
}

hipError_t launch_fwd_unfused(const FwdParams& p, int dtype, void* workspace, hipStream_t s) {
    float* buf0 = (float*)workspace;
    float* buf1 = buf0 + (size_t)p.B * p.C * (p.H > p.W ? p.H : p.W);
    int first_dir = 1;
    for (int d = 0; d < 4; ++d) {
        if (!((p.mask >> d) & 1u)) continue;
        const DirGeom gm = dir_geom(d, p.H, p.W);
        const size_t n = (size_t)p.B * p.C * gm.L;
        const size_t blocks = (n + 255) / 256;
        if (blocks > 0x7fffffffull) return hipErrorInvalidValue;
        for (int t = 0; t < gm.S; ++t) {
            float* prev = (t & 1) ? buf0 : buf1;
            float* cur = (t & 1) ? buf1 : buf0;
            if (dtype == 0) hipLaunchKernelGGL((line_step_kernel<float>), dim3((unsigned)blocks), dim3(256), 0, s, p, prev, cur, d, t, first_dir);
            else if (dtype == 1) hipLaunchKernelGGL((line_step_kernel<bf16_t>), dim3((unsigned)blocks), dim3(256), 0, s, p, prev, cur, d, t, first_dir);
            else hipLaunchKernelGGL((line_step_kernel<f16_t>), dim3((unsigned)blocks), dim3(256), 0, s, p, prev, cur, d, t, first_dir);
        }
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        first_dir = 0;
    }
    return hipSuccess;
}

}  // namespace gspn
