// Generic GSPN scan kernels: any H, W up to GSPN_MAX_LINE, any group layout.
//
// One workgroup owns one (batch, channel) plane in the forward pass -- one
// (batch, group) in the backward pass -- and walks every requested direction,
// line by line, inside a single launch (the fused-loop structure of Sec. 4.1).
// The previous line's state lives in LDS (two ping-pong lines) so a position can
// read its three neighbours (Sec. 3.2); one barrier per line.  The merged
// outputs (y, gx) are accumulated in place, direction after direction, by the
// workgroup that owns the plane, so no atomics and no zero-fill are needed and
// the summation order is fixed.
//
// This is the fallback for shapes the specialised kernels do not take; it makes
// no attempt at coalescing the horizontal directions.
#include "gspn_common.hpp"

namespace gspn {

template <typename T>
__global__ void __launch_bounds__(256) fwd_generic_kernel(FwdParams p) {
    extern __shared__ float lds[];
    const int H = p.H, W = p.W, HW = H * W;
    const int Lmax = H > W ? H : W;
    const size_t plane_cnt = (size_t)p.B * p.C;
    const T* X = (const T*)p.x;
    const T* WT = (const T*)p.w;
    const T* LAM = (const T*)p.lam;
    const T* U = (const T*)p.u;
    T* Y = (T*)p.y;
    T* HS = (T*)p.hs;

    for (size_t item = blockIdx.x; item < plane_cnt; item += gridDim.x) {
        const int b = (int)(item / p.C), c = (int)(item % p.C), g = c / p.cpg;
        const size_t pc = item * HW;
        bool first = true;
        for (int d = 0; d < 4; ++d) {
            if (!((p.mask >> d) & 1u)) continue;
            const DirGeom q = dir_geom(d, H, W);
            const size_t slot_c = p.shared ? 0 : (size_t)d * plane_cnt * HW;
            const size_t slot_w = p.shared ? 0 : (size_t)d * p.B * p.G * 3 * HW;
            // transposed-horizontal layout: x, w, lam, u of directions 2 and 3 are stored [..][W][H]
            const bool tr = p.xt != nullptr && d >= 2;
            const T* xp = (tr ? (const T*)p.xt : X) + pc;
            const T* lp = LAM + slot_c + pc;
            const T* up = U + slot_c + pc;
            const T* wp = WT + slot_w + ((size_t)b * p.G + g) * 3 * HW;
            T* yp = Y + pc;
            T* hp = HS ? HS + (size_t)d * plane_cnt * HW + pc : nullptr;
            float* prev = lds;
            float* cur = lds + Lmax;
            for (int t = 0; t < q.S; ++t) {
                const int line = q.reversed ? q.S - 1 - t : t;
                const int base = line * q.stride_s;
                const bool starts = starts_stretch(t, q.S, q.reversed, p.kchunk);
                for (int j = threadIdx.x; j < q.L; j += blockDim.x) {
                    const int offy = base + j * q.stride_j;               // in the image (y)
                    const int off = tr ? line * q.L + j : offy;          // in the inputs
                    float h = ldf(lp + off) * ldf(xp + off);
                    if (!starts) {   // first line (of the scan, of a stretch): state before it is zero, its weights are not read
                        const bool out0 = j == 0, out2 = j + 1 == q.L;     // no neighbour there: that tap is never read
                        float w0 = out0 ? 0.f : ldf(wp + off), w1 = ldf(wp + HW + off), w2 = out2 ? 0.f : ldf(wp + 2 * HW + off);
                        if (p.logits) softmax3(w0, w1, w2, out0, out2);
                        h = fmaf(w1, prev[j], h);
                        if (!out0) h = fmaf(w0, prev[j - 1], h);
                        if (!out2) h = fmaf(w2, prev[j + 1], h);
                    }
                    cur[j] = h;
                    float yv = ldf(up + off) * h;
                    if (!first) yv += ldf(yp + offy);
                    stf(yp + offy, yv);
                    if (hp) stf(hp + off, h);
                }
                __syncthreads();   // line t complete (LDS) and, after the last line, y visible to the block
                float* tmp = prev; prev = cur; cur = tmp;
            }
            first = false;
        }
    }
}

template <typename T>
__global__ void __launch_bounds__(256) bwd_generic_kernel(BwdParams p) {
    extern __shared__ float lds[];
    const int H = p.H, W = p.W, HW = H * W;
    const int Lmax = H > W ? H : W;
    const size_t plane_cnt = (size_t)p.B * p.C;
    const size_t group_cnt = (size_t)p.B * p.G;
    const T* GY = (const T*)p.gy;
    const T* X = (const T*)p.x;
    const T* WT = (const T*)p.w;
    const T* LAM = (const T*)p.lam;
    const T* U = (const T*)p.u;
    const T* HS = (const T*)p.hs;
    T* GX = (T*)p.gx;
    T* GW = (T*)p.gw;
    T* GLAM = (T*)p.glam;
    T* GU = (T*)p.gu;

    for (size_t item = blockIdx.x; item < group_cnt; item += gridDim.x) {
        const int b = (int)(item / p.G), g = (int)(item % p.G);
        for (int ci = 0; ci < p.cpg; ++ci) {
            const size_t pc = ((size_t)b * p.C + (size_t)g * p.cpg + ci) * HW;
            bool first = true;
            for (int d = 0; d < 4; ++d) {
                if (!((p.mask >> d) & 1u)) continue;
                const DirGeom q = dir_geom(d, H, W);
                const size_t out_c = (size_t)d * plane_cnt * HW;
                const size_t out_w = (size_t)d * group_cnt * 3 * HW;
                const size_t slot_c = p.shared ? 0 : out_c;
                const size_t slot_w = p.shared ? 0 : out_w;
                const T* gyp = GY + pc;
                const T* xp = X + pc;
                const T* lp = LAM + slot_c + pc;
                const T* up = U + slot_c + pc;
                const T* hp = HS + out_c + pc;
                const T* wp = WT + slot_w + item * 3 * HW;
                T* gxp = GX + pc;
                T* glp = GLAM + out_c + pc;
                T* gup = GU + out_c + pc;
                T* gwp = GW + out_w + item * 3 * HW;
                float* enext = lds;         // e of scan step t+1
                float* ecur = lds + Lmax;
                // weights as logits: the normalised taps of the current line and of the next one (scan order)
                float* wcur = lds + 2 * Lmax;
                float* wnext = lds + 5 * Lmax;
                const bool last_channel = ci == p.cpg - 1;
                for (int t = q.S - 1; t >= 0; --t) {
                    const int base = (q.reversed ? q.S - 1 - t : t) * q.stride_s;
                    const int step = q.reversed ? -q.stride_s : q.stride_s;   // to the next line in scan order
                    const bool starts = starts_stretch(t, q.S, q.reversed, p.kchunk);
                    const bool next_starts = t + 1 < q.S && starts_stretch(t + 1, q.S, q.reversed, p.kchunk);
                    if (p.logits) {
                        // this line's taps, normalised (0 where nothing is read: the line has no predecessor)
                        for (int j = threadIdx.x; j < q.L; j += blockDim.x) {
                            const int off = base + j * q.stride_j;
                            const bool out0 = j == 0, out2 = j + 1 == q.L;
                            float w0 = 0.f, w1 = 0.f, w2 = 0.f;
                            if (!starts) {
                                w0 = out0 ? 0.f : ldf(wp + off); w1 = ldf(wp + HW + off); w2 = out2 ? 0.f : ldf(wp + 2 * HW + off);
                                softmax3(w0, w1, w2, out0, out2);
                            }
                            wcur[j] = w0; wcur[Lmax + j] = w1; wcur[2 * Lmax + j] = w2;
                        }
                        __syncthreads();
                    }
                    for (int j = threadIdx.x; j < q.L; j += blockDim.x) {
                        const int off = base + j * q.stride_j;
                        const float gyv = ldf(gyp + off);
                        float e = ldf(up + off) * gyv;
                        if (t + 1 < q.S && !next_starts) {   // transposed tridiagonal of the next line (of the same stretch)
                            const int offn = off + step;
                            if (p.logits) {
                                e = fmaf(wnext[Lmax + j], enext[j], e);
                                if (j > 0) e = fmaf(wnext[2 * Lmax + j - 1], enext[j - 1], e);
                                if (j + 1 < q.L) e = fmaf(wnext[j + 1], enext[j + 1], e);
                            } else {
                                e = fmaf(ldf(wp + HW + offn), enext[j], e);
                                if (j > 0) e = fmaf(ldf(wp + 2 * HW + offn - q.stride_j), enext[j - 1], e);
                                if (j + 1 < q.L) e = fmaf(ldf(wp + offn + q.stride_j), enext[j + 1], e);
                            }
                        }
                        ecur[j] = e;
                        stf(glp + off, ldf(xp + off) * e);
                        stf(gup + off, gyv * ldf(hp + off));
                        float gxv = ldf(lp + off) * e;
                        if (!first) gxv += ldf(gxp + off);
                        stf(gxp + off, gxv);
                        const int offp = off - step;   // same position on the previous line
                        float v[3];
                        #pragma unroll
                        for (int k = 0; k < 3; ++k) {
                            const int jj = j + k - 1;
                            v[k] = 0.f;
                            if (!starts && jj >= 0 && jj < q.L) v[k] = e * ldf(hp + offp + (k - 1) * q.stride_j);
                            if (ci > 0) v[k] += ldf(gwp + k * HW + off);
                        }
                        // weights as logits: the sum over the group's channels goes through the softmax once, at the end
                        if (p.logits && last_channel) softmax3_grad(v[0], v[1], v[2], wcur[j], wcur[Lmax + j], wcur[2 * Lmax + j]);
                        #pragma unroll
                        for (int k = 0; k < 3; ++k) stf(gwp + k * HW + off, v[k]);
                    }
                    __syncthreads();
                    float* tmp = enext; enext = ecur; ecur = tmp;
                    tmp = wnext; wnext = wcur; wcur = tmp;
                }
                first = false;
            }
        }
    }
}

static int pick_block(int L) { return L <= 64 ? 64 : (L <= 128 ? 128 : 256); }

hipError_t launch_fwd_generic(const FwdParams& p, int dtype, hipStream_t s) {
    const int Lmax = p.H > p.W ? p.H : p.W;
    const size_t items = (size_t)p.B * p.C;
    const unsigned grid = (unsigned)(items < 65536 ? items : 65536);
    const int block = pick_block(Lmax);
    const size_t shmem = 2 * (size_t)Lmax * sizeof(float);
    void (*k)(FwdParams) = dtype == 0 ? fwd_generic_kernel<float> : fwd_generic_kernel<bf16_t>;
    if (shmem > 48 * 1024) {                                 // long lines: ask for the LDS explicitly
        const hipError_t e = allow_dynamic_lds((const void*)k, 160 * 1024);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(k, dim3(grid), dim3(block), shmem, s, p);
    return hipGetLastError();
}

hipError_t launch_bwd_generic(const BwdParams& p, int dtype, hipStream_t s) {
    const int Lmax = p.H > p.W ? p.H : p.W;
    const size_t items = (size_t)p.B * p.G;
    const unsigned grid = (unsigned)(items < 65536 ? items : 65536);
    const int block = pick_block(Lmax);
    const size_t shmem = (p.logits ? 8 : 2) * (size_t)Lmax * sizeof(float);
    if (shmem > 128 * 1024) return hipErrorInvalidValue;      // checked by the caller (GSPN_MAX_LINE_LOGITS)
    void (*k)(BwdParams) = dtype == 0 ? bwd_generic_kernel<float> : bwd_generic_kernel<bf16_t>;
    if (shmem > 48 * 1024) {                                 // long lines: ask for the LDS explicitly
        const hipError_t e = allow_dynamic_lds((const void*)k, 160 * 1024);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(k, dim3(grid), dim3(block), shmem, s, p);
    return hipGetLastError();
}

}  // namespace gspn
