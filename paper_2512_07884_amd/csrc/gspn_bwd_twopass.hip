// Backward GSPN scan in two passes, for maps beyond the reach of the single-launch backward kernels (more than 64
// lines per scan, weight groups that do not fit one workgroup: the 128x128 diffusion shape with 64 channels per group).
//
// The paper gives no algorithm for the backward pass (Sec. 5.1 has timings only); this is the chain rule on Eq. 1-2
// (Sec. 3.2) with the shared weights of Sec. 4.2, split where the sum over the channels of a group comes in:
//
//   pass 1, per channel: e_t = u_t*gy_t + T_{t+1}^T e_{t+1} is the forward recurrence run against the scan order with the
//           tridiagonal transposed, and gx = sum_d lam_d*e_d is its merged output -- so it runs on the forward kernels: the
//           plane kernel on small maps, the tile kernels, the stream kernel beyond the LDS tile (reverse-sweep
//           instantiations: gy as x, u as lam, lam as u, gx as y), which also save e per direction, into the buffer of glam;
//   pass 2, per (direction, image, group) and pixel: gw[k] = sum over the group's channels of e[j] * h_{t-1}[j+k-1] has no
//           recurrence left: one thread per few adjacent pixels walks the channels, accumulates the three taps in fp32
//           registers, and on the way turns the saved e into glam = x*e in place and writes gu = gy*h.
//
// GSPN-local (Sec. 3.2) cuts both passes at the stretch boundaries; with the weights given as logits pass 1 normalises
// them as it reads them and pass 2 sends the channel sum through the softmax of its pixel.
//
// No scratch memory and no atomics: every output element has one writer, the channel sum has a fixed order.  In bf16
// storage e passes through storage precision between the passes (one rounding more on glam and on the terms of gw,
// whose sum is still accumulated in fp32).
#include "gspn_tile_common.hpp"

namespace gspn {

hipError_t launch_reverse_sweep_f32(const FwdParams& p, hipStream_t s);
hipError_t launch_reverse_sweep_bf16(const FwdParams& p, hipStream_t s);
hipError_t launch_reverse_sweep_f32_local(const FwdParams& p, hipStream_t s);     // GSPN-local and logits calls
hipError_t launch_reverse_sweep_bf16_local(const FwdParams& p, hipStream_t s);
hipError_t launch_reverse_sweep_f16(const FwdParams& p, hipStream_t s);
hipError_t launch_reverse_sweep_f16_local(const FwdParams& p, hipStream_t s);
hipError_t launch_reverse_sweep_plane(const FwdParams& p, int dtype, hipStream_t s);     // small maps: whole planes through LDS
bool reverse_sweep_plane_applicable(const FwdParams& p, int dtype);
hipError_t launch_reverse_sweep_stream(const FwdParams& p, int dtype, hipStream_t s);    // maps beyond the LDS tile
bool reverse_sweep_stream_applicable(const FwdParams& p, int dtype);
hipError_t launch_reverse_sweep_pair(const FwdParams& p, int dtype, hipStream_t s);      // 128x128 bf16, two channels per workgroup
bool reverse_sweep_pair_applicable(const FwdParams& p, int dtype);
hipError_t launch_reverse_sweep_chunk(const FwdParams& p, int dtype, hipStream_t s);     // GSPN-local, one workgroup per stretch
bool reverse_sweep_chunk_applicable(const FwdParams& p, int dtype);

namespace {

// VEC adjacent elements of storage, widened to fp32 (p aligned to VEC elements).  ONCE: nothing reads these lines again
// (non-temporal request: the caches give them up first, which leaves more room for x and gy, which the workgroups of all four directions read)
template <typename T, int VEC, bool ONCE = false> __device__ __forceinline__ void ldv(const T* p, float (&out)[VEC]) {
    if constexpr (VEC == 1) {
        out[0] = ldf(p);
    } else {
        constexpr int NB = VEC * (int)sizeof(T);
        uint32_t r[NB / 4];
        if constexpr (NB == 4) r[0] = ONCE ? __builtin_nontemporal_load((const uint32_t*)p) : *(const uint32_t*)p;
        else if constexpr (NB == 8) { const u32x2 v = ONCE ? __builtin_nontemporal_load((const u32x2*)p) : *(const u32x2*)p; r[0] = v.x; r[1] = v.y; }
        else {
#pragma unroll
            for (int i = 0; i < NB / 16; ++i) {
                const u32x4 v = ONCE ? __builtin_nontemporal_load((const u32x4*)p + i) : ((const u32x4*)p)[i];
                r[4 * i] = v.x; r[4 * i + 1] = v.y; r[4 * i + 2] = v.z; r[4 * i + 3] = v.w;
            }
        }
#pragma unroll
        for (int v = 0; v < VEC; ++v) out[v] = elem<T>(r, v);
    }
}
template <typename T, int VEC, bool ONCE = false> __device__ __forceinline__ void stv(T* p, const float (&in)[VEC]) {
    if constexpr (VEC == 1) {
        stf(p, in[0]);
    } else {
        constexpr int NB = VEC * (int)sizeof(T);
        uint32_t r[NB / 4];
        pack<T, VEC>(in, r);
        if constexpr (NB == 4) { if constexpr (ONCE) __builtin_nontemporal_store(r[0], (uint32_t*)p); else *(uint32_t*)p = r[0]; }
        else if constexpr (NB == 8) { const u32x2 v = {r[0], r[1]}; if constexpr (ONCE) __builtin_nontemporal_store(v, (u32x2*)p); else *(u32x2*)p = v; }
        else {
#pragma unroll
            for (int i = 0; i < NB / 16; ++i) {
                const u32x4 v = {r[4 * i], r[4 * i + 1], r[4 * i + 2], r[4 * i + 3]};
                if constexpr (ONCE) __builtin_nontemporal_store(v, (u32x4*)p + i); else ((u32x4*)p)[i] = v;
            }
        }
    }
}

// h of the previous scan line as the three taps of VEC adjacent pixels see it.  `row` = the image row to read (NULL: it
// does not exist), j0 = first column of the pixels, `shift` = column offset of the tap (-1, 0, +1); 0 outside the image.
// SHUF: the pixel blocks of neighbouring lanes are neighbours in the row (the blocks of a row divide a wave), so the element beside the block comes from the neighbouring lane's registers instead of a request of its own.
template <typename T, int VEC, bool SHUF>
__device__ __forceinline__ void tap_window(const T* row, int j0, int W, int shift, const float (&centre)[VEC], float (&out)[VEC]) {
    if (shift == 0) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) out[v] = centre[v];
    } else if (shift < 0) {
        float edge;
        if constexpr (SHUF) { const float nb = from_lane_below(centre[VEC - 1]); edge = j0 > 0 ? nb : 0.f; }
        else edge = (row && j0 > 0) ? ldf(row + j0 - 1) : 0.f;
#pragma unroll
        for (int v = 0; v < VEC; ++v) out[v] = v > 0 ? centre[v - 1] : edge;
    } else {
        float edge;
        if constexpr (SHUF) { const float nb = from_lane_above(centre[0]); edge = j0 + VEC < W ? nb : 0.f; }
        else edge = (row && j0 + VEC < W) ? ldf(row + j0 + VEC) : 0.f;
#pragma unroll
        for (int v = 0; v < VEC; ++v) out[v] = v < VEC - 1 ? centre[v + 1] : edge;
    }
}

template <typename T, int VEC, bool SHUF>
__global__ void __launch_bounds__(256) bwd_finish_kernel(BwdParams p, int ndirs) {
    const int H = p.H, W = p.W, HW = H * W;
    const int npb = HW / VEC;
    const size_t per_dir = (size_t)p.B * p.G * npb;
    // workgroup -> (direction, block of pixels): the workgroups that work on the same pixels in the different
    // directions read the same x and gy; they get indices 8 apart, which the dispatcher hands to the same XCD one
    // after the other, so that those re-reads meet in one L2
    const unsigned wg = blockIdx.x;
    int dsel = (int)((wg / 8) % (unsigned)ndirs);
    const unsigned blk = (wg / (8 * (unsigned)ndirs)) * 8 + (wg % 8);
    const size_t rem = (size_t)blk * blockDim.x + threadIdx.x;
    if (rem >= per_dir) return;
    const int bg = (int)(rem / npb);
    const int pix0 = (int)(rem - (size_t)bg * npb) * VEC;
    int d = 0;
    for (;; ++d)                                               // the dsel-th direction of the mask
        if ((p.mask >> d) & 1u) { if (dsel == 0) break; --dsel; }
    const int b = bg / p.G, g = bg - b * p.G;
    const int i = pix0 / W, j0 = pix0 - i * W;                 // VEC divides W: the pixels share a row
    const size_t planes = (size_t)p.B * p.C, groups = (size_t)p.B * p.G;
    const T* X = (const T*)p.x;
    const T* GY = (const T*)p.gy;
    const T* HS = (const T*)p.hs + (size_t)d * planes * HW;
    T* GL = (T*)p.glam + (size_t)d * planes * HW;              // holds e on entry
    T* GU = (T*)p.gu + (size_t)d * planes * HW;
    T* GW = (T*)p.gw + ((size_t)d * groups + bg) * 3 * HW;
    // where the previous scan line is: a row up / down (vertical scans, taps along the columns) or a column left / right
    // (horizontal scans, taps along the rows)
    const bool vert = d < 2;
    const int drow = vert ? ((d & 1) ? 1 : -1) : 0;
    const int dcol = vert ? 0 : ((d & 1) ? 1 : -1);

    float a0[VEC], a1[VEC], a2[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) { a0[v] = 0.f; a1[v] = 0.f; a2[v] = 0.f; }
    // GSPN-local (Sec. 3.2): a pixel on a line that starts a stretch has no previous line (its taps were never read)
    bool starts[VEC], first_step[VEC];      // first_step: the first line of the whole scan (no previous line either)
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
        const int r = vert ? i : j0 + v, S = vert ? H : W;        // image line along the scan axis
        starts[v] = p.kchunk > 0 && starts_stretch((d & 1) ? S - 1 - r : r, S, d & 1, p.kchunk);
        first_step[v] = ((d & 1) ? S - 1 - r : r) == 0;
    }

    for (int ci = 0; ci < p.cpg; ++ci) {
        const size_t plane = ((size_t)b * p.C + (size_t)g * p.cpg + ci) * HW;
        float e[VEC], xv[VEC], gyv[VEC], hc[VEC];
        ldv<T, VEC, true>(GL + plane + pix0, e);
        ldv<T, VEC>(X + plane + pix0, xv);
        ldv<T, VEC>(GY + plane + pix0, gyv);
        ldv<T, VEC>(HS + plane + pix0, hc);
        float t0[VEC], t1[VEC], t2[VEC];
        if (vert) {
            const int ip = i + drow;
            const T* row = (ip >= 0 && ip < H) ? HS + plane + (size_t)ip * W : nullptr;
            float hv[VEC];
#pragma unroll
            for (int v = 0; v < VEC; ++v) hv[v] = 0.f;
            if (row) ldv<T, VEC>(row + j0, hv);
            tap_window<T, VEC, SHUF>(row, j0, W, -1, hv, t0);
            tap_window<T, VEC, SHUF>(row, j0, W, 0, hv, t1);
            tap_window<T, VEC, SHUF>(row, j0, W, 1, hv, t2);
        } else {
            float hv[VEC];
#pragma unroll
            for (int k = 0; k < 3; ++k) {
                const int ir = i + k - 1;
                const T* row = (ir >= 0 && ir < H) ? HS + plane + (size_t)ir * W : nullptr;
#pragma unroll
                for (int v = 0; v < VEC; ++v) hv[v] = k == 1 ? hc[v] : 0.f;      // the pixels' own row is in registers already
                if (k != 1 && row) ldv<T, VEC>(row + j0, hv);
                tap_window<T, VEC, SHUF>(row, j0, W, dcol, hv, k == 0 ? t0 : (k == 1 ? t1 : t2));
            }
        }
        float gl[VEC], gu[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            const float ev = starts[v] ? 0.f : e[v];
            a0[v] = fmaf(ev, t0[v], a0[v]);
            a1[v] = fmaf(ev, t1[v], a1[v]);
            a2[v] = fmaf(ev, t2[v], a2[v]);
            gl[v] = xv[v] * e[v];
            gu[v] = gyv[v] * hc[v];
        }
        stv<T, VEC, true>(GL + plane + pix0, gl);
        stv<T, VEC, true>(GU + plane + pix0, gu);
    }
    if (p.logits) {
        // the weights were given as logits: the sum over the group's channels goes through the softmax of its pixel once
        const T* Z = (const T*)p.w + ((p.shared ? (size_t)0 : (size_t)d * groups) + bg) * 3 * HW;
        float z0[VEC], z1[VEC], z2[VEC];
        ldv<T, VEC>(Z + pix0, z0);
        ldv<T, VEC>(Z + HW + pix0, z1);
        ldv<T, VEC>(Z + 2 * (size_t)HW + pix0, z2);
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            const int pos = vert ? j0 + v : i, L = vert ? W : H;      // position on the line
            // a line without a predecessor never reads its logits: whatever they hold (NaN, Inf) stays out and
            // their gradient is an exact 0
            const bool unread = starts[v] || first_step[v];
            z0[v] = unread ? 0.f : z0[v]; z1[v] = unread ? 0.f : z1[v]; z2[v] = unread ? 0.f : z2[v];
            a0[v] = unread ? 0.f : a0[v]; a1[v] = unread ? 0.f : a1[v]; a2[v] = unread ? 0.f : a2[v];
            softmax3(z0[v], z1[v], z2[v], pos == 0, pos == L - 1);
            softmax3_grad(a0[v], a1[v], a2[v], z0[v], z1[v], z2[v]);
        }
    }
    stv<T, VEC>(GW + pix0, a0);
    stv<T, VEC>(GW + HW + pix0, a1);
    stv<T, VEC>(GW + 2 * (size_t)HW + pix0, a2);
}

FwdParams reverse_sweep_params(const BwdParams& p) {
    FwdParams f = {};
    f.x = p.gy; f.w = p.w; f.lam = p.u; f.u = p.lam; f.y = p.gx; f.hs = p.glam;
    f.B = p.B; f.C = p.C; f.H = p.H; f.W = p.W; f.G = p.G; f.cpg = p.cpg;
    f.mask = p.mask; f.shared = p.shared; f.kchunk = p.kchunk; f.logits = p.logits; f.xt = nullptr;
    return f;
}

template <typename T, int VEC>
hipError_t launch_finish(const BwdParams& p, int ndirs, hipStream_t s) {
    const size_t per_dir = (size_t)p.B * p.G * (p.H * p.W / VEC);
    const size_t blocks = ((per_dir + 255) / 256 + 7) / 8 * 8 * ndirs;      // per direction: a multiple of 8 workgroups
    if (blocks > 0x7fffffffull) return hipErrorInvalidValue;
    // a lane's neighbours hold the neighbouring blocks of its row when the blocks of a row divide a wave (a wave starts at a
    // multiple of 64 blocks: workgroups are 256 threads, planes whole rows), so that no row continues in another wave
    const int bpr = p.W / VEC;
    if (VEC > 1 && 64 % bpr == 0)
        hipLaunchKernelGGL((bwd_finish_kernel<T, VEC, true>), dim3((unsigned)blocks), dim3(256), 0, s, p, ndirs);
    else
        hipLaunchKernelGGL((bwd_finish_kernel<T, VEC, false>), dim3((unsigned)blocks), dim3(256), 0, s, p, ndirs);
    return hipGetLastError();
}

}  // namespace

bool bwd_twopass_applicable(const BwdParams& p, int dtype) {
    if ((size_t)p.B * p.G * ((size_t)p.H * p.W) * 4 / 256 > 0x7fffffffull) return false;
    const FwdParams f = reverse_sweep_params(p);
    return reverse_sweep_plane_applicable(f, dtype) || fwd_tile_applicable(f, dtype) || reverse_sweep_stream_applicable(f, dtype) ||
           (chunk_kernels_enabled() && reverse_sweep_chunk_applicable(f, dtype));
}

hipError_t launch_bwd_twopass(const BwdParams& p, int dtype, hipStream_t s) {
    if (!bwd_twopass_applicable(p, dtype)) return hipErrorInvalidValue;
    const FwdParams f = reverse_sweep_params(p);
    hipError_t e;
    if (chunk_kernels_enabled() && reverse_sweep_chunk_applicable(f, dtype)) {
        e = launch_reverse_sweep_chunk(f, dtype, s);
    } else if (reverse_sweep_plane_applicable(f, dtype)) {
        e = launch_reverse_sweep_plane(f, dtype, s);
    } else if (pair_kernels_enabled() && reverse_sweep_pair_applicable(f, dtype)) {
        e = launch_reverse_sweep_pair(f, dtype, s);
    } else if (fwd_tile_applicable(f, dtype)) {
        const bool local = p.kchunk > 0 || p.logits;
        if (dtype == 0) e = local ? launch_reverse_sweep_f32_local(f, s) : launch_reverse_sweep_f32(f, s);
        else if (dtype == 1) e = local ? launch_reverse_sweep_bf16_local(f, s) : launch_reverse_sweep_bf16(f, s);
        else e = local ? launch_reverse_sweep_f16_local(f, s) : launch_reverse_sweep_f16(f, s);
    } else {
        e = launch_reverse_sweep_stream(f, dtype, s);
    }
    if (e != hipSuccess) return e;
    int ndirs = 0;
    for (int d = 0; d < 4; ++d) ndirs += (p.mask >> d) & 1u;
    if (dtype == 0) {
        if (p.W % 8 == 0) return launch_finish<float, 8>(p, ndirs, s);
        if (p.W % 4 == 0) return launch_finish<float, 4>(p, ndirs, s);
        if (p.W % 2 == 0) return launch_finish<float, 2>(p, ndirs, s);
        return launch_finish<float, 1>(p, ndirs, s);
    }
    if (dtype == 2) {
        if (p.W % 8 == 0) return launch_finish<f16_t, 8>(p, ndirs, s);
        if (p.W % 4 == 0) return launch_finish<f16_t, 4>(p, ndirs, s);
        if (p.W % 2 == 0) return launch_finish<f16_t, 2>(p, ndirs, s);
        return launch_finish<f16_t, 1>(p, ndirs, s);
    }
    if (p.W % 8 == 0) return launch_finish<bf16_t, 8>(p, ndirs, s);
    if (p.W % 4 == 0) return launch_finish<bf16_t, 4>(p, ndirs, s);
    if (p.W % 2 == 0) return launch_finish<bf16_t, 2>(p, ndirs, s);
    return launch_finish<bf16_t, 1>(p, ndirs, s);
}

}  // namespace gspn
