// Generic GSPN scan kernels: any H, W up to GSPN_MAX_LINE, any group layout.
//
// One workgroup owns one (batch, channel) plane in the forward pass -- one
// (batch, group) in the backward pass -- and walks every requested direction,
// line by line, inside a single launch (the fused-loop structure of Sec. 4.1).
// The previous line's state lives in LDS (two ping-pong lines) so a position can
// read its three neighbours (Sec. 3.2); one barrier per line.  The merged
// outputs (y, gx) are accumulated direction after direction by the workgroup that
// owns the plane -- y of a bf16 plane that fits in an fp32 LDS tile, everything
// else in place in global memory -- so no atomics and no zero-fill are needed and
// the summation order is fixed.
//
// This is the fallback for shapes the specialised kernels do not take; it makes
// no attempt at coalescing the horizontal directions.
#include "gspn_common.hpp"

namespace gspn {

// TILE: the merged output of the plane is accumulated in an fp32 LDS tile behind the two line buffers and meets the
// storage type once (planes that fit); otherwise it is accumulated in place in global memory, one rounding per direction.
template <typename T, bool TILE>
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
    float* acc = lds + 2 * Lmax;

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
                    if constexpr (TILE) {
                        if (!first) yv += acc[offy];
                        acc[offy] = yv;
                    } else {
                        if (!first) yv += ldf(yp + offy);
                        stf(yp + offy, yv);
                    }
                    if (hp) stf(hp + off, h);
                }
                __syncthreads();   // line t complete (LDS) and, after the last line, y visible to the block
                float* tmp = prev; prev = cur; cur = tmp;
            }
            first = false;
        }
        if constexpr (TILE) {
            for (int i = threadIdx.x; i < HW; i += blockDim.x) stf(Y + pc + i, acc[i]);
            __syncthreads();       // the tile is free for the next plane
        }
    }
}

// Backward: one workgroup per (batch, group).  Directions are the outer loop; inside a direction the channels of the
// group are walked in batches of `nc` whose error lines e_{t+1} fit in LDS side by side, so that the scan steps are the
// middle loop and the channels the inner one: the sum over the group's channels that gw needs (chain rule on Eq. 1 with
// the shared weights of Sec. 4.2) is then taken in fp32 registers, position by position, and meets the storage type
// once per batch (one batch unless lines are very long), and a line costs one barrier for all its channels.
template <typename T>
__global__ void __launch_bounds__(256) bwd_generic_kernel(BwdParams p, int nc) {
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
    // LDS: e of scan step t+1 and of step t for the nc channels of the batch, then (weights as logits) the normalised
    // taps of the current line and of the next one in scan order
    float* ebuf0 = lds;
    float* ebuf1 = lds + (size_t)nc * Lmax;
    float* wbuf0 = lds + 2 * (size_t)nc * Lmax;
    float* wbuf1 = wbuf0 + 3 * Lmax;

    for (size_t item = blockIdx.x; item < group_cnt; item += gridDim.x) {
        const int b = (int)(item / p.G), g = (int)(item % p.G);
        const size_t pc0 = ((size_t)b * p.C + (size_t)g * p.cpg) * HW;      // first channel of the group
        bool first = true;                                                   // first direction: gx is overwritten
        for (int d = 0; d < 4; ++d) {
            if (!((p.mask >> d) & 1u)) continue;
            const DirGeom q = dir_geom(d, H, W);
            const size_t out_c = (size_t)d * plane_cnt * HW;
            const size_t out_w = (size_t)d * group_cnt * 3 * HW;
            const size_t slot_c = p.shared ? 0 : out_c;
            const size_t slot_w = p.shared ? 0 : out_w;
            const T* wp = WT + slot_w + item * 3 * HW;
            T* gwp = GW + out_w + item * 3 * HW;
            const int step = q.reversed ? -q.stride_s : q.stride_s;          // to the next line in scan order
            for (int c0 = 0; c0 < p.cpg; c0 += nc) {
                const int n_here = min(nc, p.cpg - c0);
                const bool last_batch = c0 + n_here == p.cpg;
                float* enext = ebuf0;
                float* ecur = ebuf1;
                float* wcur = wbuf0;
                float* wnext = wbuf1;
                for (int t = q.S - 1; t >= 0; --t) {
                    const int base = (q.reversed ? q.S - 1 - t : t) * q.stride_s;
                    const bool starts = starts_stretch(t, q.S, q.reversed, p.kchunk);
                    const bool next_starts = t + 1 < q.S && starts_stretch(t + 1, q.S, q.reversed, p.kchunk);
                    const bool carry = t + 1 < q.S && !next_starts;         // e of the next line (same stretch) comes in
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
                        const int offp = off - step;                        // same position on the previous line
                        // transposed tridiagonal of the next line: position j is read by tap 1 of j, tap 2 of j-1, tap 0 of j+1
                        float tc = 0.f, tl = 0.f, tr = 0.f;
                        if (carry) {
                            if (p.logits) {
                                tc = wnext[Lmax + j];
                                if (j > 0) tl = wnext[2 * Lmax + j - 1];
                                if (j + 1 < q.L) tr = wnext[j + 1];
                            } else {
                                const int offn = off + step;
                                tc = ldf(wp + HW + offn);
                                if (j > 0) tl = ldf(wp + 2 * HW + offn - q.stride_j);
                                if (j + 1 < q.L) tr = ldf(wp + offn + q.stride_j);
                            }
                        }
                        float v[3] = {0.f, 0.f, 0.f};                       // gw of this position, summed over the batch in fp32
                        for (int ci = 0; ci < n_here; ++ci) {
                            const size_t pc = pc0 + (size_t)(c0 + ci) * HW;
                            const float* en = enext + (size_t)ci * Lmax;
                            const float gyv = ldf(GY + pc + off);
                            float e = ldf(U + slot_c + pc + off) * gyv;
                            if (carry) {
                                e = fmaf(tc, en[j], e);
                                if (j > 0) e = fmaf(tl, en[j - 1], e);
                                if (j + 1 < q.L) e = fmaf(tr, en[j + 1], e);
                            }
                            ecur[(size_t)ci * Lmax + j] = e;
                            const T* hp = HS + out_c + pc;
                            stf(GLAM + out_c + pc + off, ldf(X + pc + off) * e);
                            stf(GU + out_c + pc + off, gyv * ldf(hp + off));
                            float gxv = ldf(LAM + slot_c + pc + off) * e;
                            if (!first) gxv += ldf(GX + pc + off);
                            stf(GX + pc + off, gxv);
                            if (!starts) {
                                v[1] = fmaf(e, ldf(hp + offp), v[1]);
                                if (j > 0) v[0] = fmaf(e, ldf(hp + offp - q.stride_j), v[0]);
                                if (j + 1 < q.L) v[2] = fmaf(e, ldf(hp + offp + q.stride_j), v[2]);
                            }
                        }
                        if (c0 > 0) {
#pragma unroll
                            for (int k = 0; k < 3; ++k) v[k] += ldf(gwp + k * HW + off);
                        }
                        // weights as logits: the sum over the group's channels goes through the softmax once, at the end
                        if (p.logits && last_batch) softmax3_grad(v[0], v[1], v[2], wcur[j], wcur[Lmax + j], wcur[2 * Lmax + j]);
#pragma unroll
                        for (int k = 0; k < 3; ++k) stf(gwp + k * HW + off, v[k]);
                    }
                    __syncthreads();
                    float* tmp = enext; enext = ecur; ecur = tmp;
                    tmp = wnext; wnext = wcur; wcur = tmp;
                }
            }
            first = false;
        }
    }
}

static int pick_block(int L) { return L <= 64 ? 64 : (L <= 128 ? 128 : 256); }

hipError_t launch_fwd_generic(const FwdParams& p, int dtype, hipStream_t s) {
    const int Lmax = p.H > p.W ? p.H : p.W;
    const size_t items = (size_t)p.B * p.C;
    const unsigned grid = (unsigned)(items < 65536 ? items : 65536);
    const int block = pick_block(Lmax);
    const size_t lines = 2 * (size_t)Lmax * sizeof(float);
    // the fp32 tile of the merged output, when the plane fits beside the line buffers (one rounding of y instead of
    // one per direction; in fp32 storage the in-place sum is already exact to the storage type)
    const size_t with_tile = lines + (size_t)p.H * p.W * sizeof(float);
    const bool tile = dtype != 0 && with_tile <= 160 * 1024;
    const size_t shmem = tile ? with_tile : lines;
    void (*k)(FwdParams) = dtype == 0 ? fwd_generic_kernel<float, false>
                           : dtype == 1 ? (tile ? fwd_generic_kernel<bf16_t, true> : fwd_generic_kernel<bf16_t, false>)
                                        : (tile ? fwd_generic_kernel<f16_t, true> : fwd_generic_kernel<f16_t, false>);
    if (shmem > 48 * 1024) {                                 // ask for the LDS explicitly
        const hipError_t e = allow_dynamic_lds((const void*)k, 160 * 1024);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(k, dim3(grid), dim3(block), shmem, s, p);
    return hipGetLastError();
}

// channels of a group whose error lines share the LDS in the backward kernel: all of them when they fit in 96 KB
static int bwd_batch(const BwdParams& p, int Lmax) {
    const size_t budget = 96 * 1024 / sizeof(float);
    const size_t taps = p.logits ? 6 * (size_t)Lmax : 0;
    size_t nc = budget > taps ? (budget - taps) / (2 * (size_t)Lmax) : 0;
    if (nc < 1) nc = 1;
    return nc < (size_t)p.cpg ? (int)nc : p.cpg;
}

hipError_t launch_bwd_generic(const BwdParams& p, int dtype, hipStream_t s) {
    const int Lmax = p.H > p.W ? p.H : p.W;
    const size_t items = (size_t)p.B * p.G;
    const unsigned grid = (unsigned)(items < 65536 ? items : 65536);
    const int block = pick_block(Lmax);
    const int nc = bwd_batch(p, Lmax);
    const size_t shmem = (2 * (size_t)nc + (p.logits ? 6 : 0)) * (size_t)Lmax * sizeof(float);
    if (shmem > 160 * 1024) return hipErrorInvalidValue;      // checked by the caller (GSPN_MAX_LINE_LOGITS)
    void (*k)(BwdParams, int) = dtype == 0 ? bwd_generic_kernel<float> : dtype == 1 ? bwd_generic_kernel<bf16_t> : bwd_generic_kernel<f16_t>;
    if (shmem > 48 * 1024) {                                 // ask for the LDS explicitly
        const hipError_t e = allow_dynamic_lds((const void*)k, 160 * 1024);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(k, dim3(grid), dim3(block), shmem, s, p, nc);
    return hipGetLastError();
}

}  // namespace gspn
