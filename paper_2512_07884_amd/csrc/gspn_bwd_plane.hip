// Backward GSPN scan for very small feature maps (fp32 or 16-bit storage, H, W <= 32: the 28x28
// training stage): every tensor crosses the memory system exactly once, as whole planes.
//
// The paper gives timings but no algorithm for the backward pass (Sec. 5.1); this is the chain rule
// on Eq. 1-2 (Sec. 3.2) with the shared weights of Sec. 4.2.  Per direction, with e_s = dL/dh_s and
// s the scan step:
//     e_s[j]  = u_s[j]*gy_s[j] + w2_{s+1}[j-1]*e_{s+1}[j-1] + w1_{s+1}[j]*e_{s+1}[j] + w0_{s+1}[j+1]*e_{s+1}[j+1]
//     gu_s = gy_s*h_s,  glam_s = x_s*e_s,  gx_s += lam_s*e_s (summed over directions)
//     gw_s[k][j] = sum over the channels of the group of e_s[j] * h_{s-1}[j+k-1]      (0 for s = 0)
//
// A plane of at most 32x32 fp32 is 4 KB, so a wave can hold a whole directional sweep of two
// channels in registers: lane = position on the line (lanes 0-31 one channel, 32-63 the next),
// register index = scan step.  Planes are read from global memory as flat, fully coalesced 16 B
// per lane copies, dropped into a per-wave LDS buffer and read back "transposed" (position per
// lane, step per register) with an address pattern that encodes the direction; results that are
// elementwise in the plane (gu = gy*h, glam = x*e, gx += lam*e) are formed in the flat layout, so
// the only transposes are u*gy, w0, w1, w2 and h on the way in and e on the way out.  The sweep
// itself is 100% register + DPP work, unrolled over the scan steps.
//
// gw: a wave keeps 3 x steps accumulators in registers while it walks the channel pairs it owns
// (directions are the outer loop), the two halves of the wave and then the waves of the workgroup
// are summed through LDS in a fixed order, and the group's gw leaves the workgroup once per
// direction: stored when the workgroup holds the whole weight group, added atomically onto a
// zero-filled gw when the group is split over two workgroups (two addends commute: still bitwise
// reproducible).  With one channel per group (per-channel weights of Eq. 1) every sweep writes
// its own gw.  gx is merged over the directions in an LDS tile owned pair-wise by single waves.
//
// Lines of at most 16 / 8 positions (14x14, 7x7: the last stages of a classifier) put four / eight
// channels side by side in a wave instead of two.  There a plane need not be a whole number of 16 B
// chunks: only the wave's channels together are, and the group's three weight planes (and their
// gradients) move as one block in the widest pieces its alignment allows.
#include "gspn_tile_common.hpp"
#include <stdlib.h>

namespace gspn {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4a __attribute__((ext_vector_type(4), may_alias));
typedef float f32a __attribute__((may_alias));

struct BwdPlaneArgs {
    BwdParams p;
    int K;             // channels per workgroup (a multiple of the channels per wave)
    int shared_group;  // 1: the K channels share one weight group; 0: one weight group per channel
    int gsplit;        // workgroups per weight group; 2: gw is accumulated atomically
    int nwaves;
    int wlw;           // four / eight channels per wave: bytes per request of the group's weight block (16, 8, 4, 2)
    uint32_t seg[4];   // per direction: bit s set <=> scan step s starts a stretch (bit 0 always)
};

// one piece of `ew` elements (a power of two, at most E) to storage
template <typename T, int E> __device__ __forceinline__ void store_piece(T* dst, const float (&v)[E], int ew) {
    if constexpr (sizeof(T) == 4) {
        if (ew == 4) { const u32x4 c = {__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])}; *(u32x4*)dst = c; }
        else if (ew == 2) { const u32x2 c = {__float_as_uint(v[0]), __float_as_uint(v[1])}; *(u32x2*)dst = c; }
        else *(float*)dst = v[0];
    } else {
        if (ew == 8) { const u32x4 c = {pack_word<T>(v[0], v[1]), pack_word<T>(v[2], v[3]), pack_word<T>(v[4], v[5]), pack_word<T>(v[6], v[7])}; *(u32x4*)dst = c; }
        else if (ew == 4) { const u32x2 c = {pack_word<T>(v[0], v[1]), pack_word<T>(v[2], v[3])}; *(u32x2*)dst = c; }
        else if (ew == 2) *(uint32_t*)dst = pack_word<T>(v[0], v[1]);
        else stf(dst, v[0]);
    }
}

// widening / narrowing of one 16 B chunk of storage (E = 4 fp32 or 8 bf16 elements)
template <typename T, int E> __device__ __forceinline__ void chunk_unpack(const u32x4& c, float (&v)[E]) {
    if constexpr (sizeof(T) == 4) {
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = __uint_as_float(c[e]);
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) { v[2 * e] = word_lo<T>(c[e]); v[2 * e + 1] = word_hi<T>(c[e]); }
    }
}
template <typename T, int E> __device__ __forceinline__ u32x4 chunk_pack(const float (&v)[E]) {
    u32x4 c;
    if constexpr (sizeof(T) == 4) {
#pragma unroll
        for (int e = 0; e < 4; ++e) c[e] = __float_as_uint(v[e]);
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) c[e] = pack_word<T>(v[2 * e], v[2 * e + 1]);
    }
    return c;
}

// SMAX: scan steps held in registers; CPW: channels per wave, on 64 / CPW lanes each; LOCAL: GSPN-local;
// LOGITS: w holds raw logits (normalised here, Sec. 3.2) and gw receives the gradient w.r.t. them
template <typename T, int SMAX, int CPW, bool SHARED, bool LOCAL, bool LOGITS>
__global__ void __launch_bounds__((SHARED && SMAX < 32) ? 384 : 256, (SHARED && SMAX == 32) ? 1 : 2)
bwd_plane_kernel(BwdPlaneArgs a) {
    static_assert(CPW == 2 || SHARED, "more than two channels per wave: shared weights only");
    static_assert(SMAX * CPW <= 64, "a line per channel");
    constexpr int E = 16 / (int)sizeof(T);                    // elements per 16 B chunk of storage
    constexpr int LPC = 64 / CPW;                             // lanes per channel
    constexpr int NCH = (CPW * SMAX * SMAX / E + 63) / 64;    // chunks per lane for the planes of the wave's channels
    extern __shared__ float lds[];
    const BwdParams& p = a.p;
    const int H = p.H, W = p.W, HW = H * W;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int half = lane / LPC, i = lane % LPC;               // channel of the wave, position on the line
    const int wgs_per_image = p.C / a.K;
    const int b = blockIdx.x / wgs_per_image;
    const int c_first = (blockIdx.x - b * wgs_per_image) * a.K;
    const int pairs = a.K / CPW;                               // sets of CPW channels ("pairs" when CPW = 2)
    const int n16p = HW / E, n16 = CPW * HW / E;               // chunks per plane (CPW = 2 only) / per set
    const size_t planes = (size_t)p.B * p.C, groups = (size_t)p.B * p.G;
    constexpr bool shared_group = SHARED;
    const bool atomic = a.gsplit > 1;                          // fp32 storage only (checked on the host)

    float* tile = lds;                                         // [K][HW] merged gx (fp32)
    float* wave_bufs = lds + a.K * HW;                         // per wave: X (CPW planes), H (CPW planes), fp32
    f32a* bufX = wave_bufs + wave * 2 * CPW * HW;
    f32a* bufH = bufX + CPW * HW;

    // chunk q = k*64 + lane of a contiguous pair of planes covers elements [E*q, E*q + E)
    bool vq[NCH];        // chunk inside the pair
    bool vq1[NCH];       // chunk inside the first plane
    uint32_t wq[NCH];    // byte offset of the chunk in a weight tensor (per-channel groups: planes 3*HW apart)
#pragma unroll
    for (int k = 0; k < NCH; ++k) {
        const int q = k * 64 + lane;
        vq[k] = q < n16;
        vq1[k] = q < n16p;
        wq[k] = (uint32_t)((shared_group || q < n16p) ? 16 * q : 3 * HW * (int)sizeof(T) + 16 * (q - n16p));
    }
    // global memory is reached through buffer resources: uniform base, per-lane byte offset 16*lane,
    // uniform chunk offset k*1024 -- no per-lane 64-bit addresses to keep in registers
    const uint32_t voff = (uint32_t)lane * 16u;
    auto ldg = [&](rsrc_t rs, uint32_t vo, int so, float (&v)[E]) {
        chunk_unpack<T, E>(__builtin_amdgcn_raw_buffer_load_b128(rs, vo, so, 0), v);
    };
    auto stg = [&](rsrc_t rs, uint32_t vo, int so, const float (&v)[E]) {
        st_b128<CP_STREAM>(rs, vo + (uint32_t)so, chunk_pack<T, E>(v));     // whole offset in the vector offset (see st_b128)
    };
    // the planes of a channel's own tensors are read once, the gradients written once: non-temporal (CP_STREAM)
    auto ldg_own = [&](rsrc_t rs, uint32_t vo, int so, float (&v)[E]) {
        chunk_unpack<T, E>(__builtin_amdgcn_raw_buffer_load_b128(rs, vo, so, CP_STREAM), v);
    };
    auto zero = [&](float (&v)[E]) {
#pragma unroll
        for (int e = 0; e < E; ++e) v[e] = 0.f;
    };
    auto load_pair = [&](const T* base, float (&st)[NCH][E]) {
        const rsrc_t rs = make_rsrc(base);
#pragma unroll
        for (int k = 0; k < NCH; ++k) {
            zero(st[k]);
            if (vq[k]) ldg_own(rs, voff, k * 1024, st[k]);
        }
    };
    auto load_w = [&](const T* base, float (&st)[NCH][E]) {
        const rsrc_t rs = make_rsrc(base);
#pragma unroll
        for (int k = 0; k < NCH; ++k) {
            zero(st[k]);
            if constexpr (SHARED) { if (vq1[k]) ldg(rs, voff, k * 1024, st[k]); }
            else { if (vq[k]) ldg(rs, wq[k], 0, st[k]); }
        }
    };
    // flat fp32 planes in LDS: chunk q sits at floats [E*q, E*q + E)
    auto lds_put = [&](f32a* buf, int q, const float (&v)[E]) {
#pragma unroll
        for (int j = 0; j < E / 4; ++j) {
            const f32x4 t = {v[4 * j], v[4 * j + 1], v[4 * j + 2], v[4 * j + 3]};
            *(f32x4a*)(buf + E * q + 4 * j) = t;
        }
    };
    auto lds_get = [&](const f32a* buf, int q, float (&v)[E]) {
#pragma unroll
        for (int j = 0; j < E / 4; ++j) {
            const f32x4 t = *(const f32x4a*)(buf + E * q + 4 * j);
            v[4 * j] = t.x; v[4 * j + 1] = t.y; v[4 * j + 2] = t.z; v[4 * j + 3] = t.w;
        }
    };
    auto to_lds = [&](f32a* buf, const float (&st)[NCH][E], bool one_plane) {
#pragma unroll
        for (int k = 0; k < NCH; ++k)
            if (one_plane ? vq1[k] : vq[k]) lds_put(buf, k * 64 + lane, st[k]);
    };

    // the wave's pairs start with gx = 0
    for (int pair = wave; pair < pairs; pair += a.nwaves) {
        f32a* tp = tile + (size_t)CPW * pair * HW;
        float z[E];
        zero(z);
#pragma unroll
        for (int k = 0; k < NCH; ++k)
            if (vq[k]) lds_put(tp, k * 64 + lane, z);
    }

    for (int d = 0; d < 4; ++d) {
        if (!((p.mask >> d) & 1u)) continue;
        // element (position j, scan step s) of a plane sits at float offset j*ps + s0 + s*ss
        const bool vert = d < 2, rev = (d & 1) != 0;
        const int S = vert ? H : W, L = vert ? W : H;
        const int ps = vert ? 1 : W;
        const int ss = vert ? (rev ? -W : W) : (rev ? -1 : 1);
        const int s0 = vert ? (rev ? (H - 1) * W : 0) : (rev ? W - 1 : 0);
        const bool active = i < L;
        const int ic = active ? i : L - 1;
        const bool first = i == 0, last = i == L - 1;
        const int tb = half * HW + ic * ps + s0;               // this lane's element at scan step 0
        const int tbw = shared_group ? ic * ps + s0 : tb;      // same, in a weight plane
        const size_t out_c = (size_t)d * planes * HW, out_w = (size_t)d * groups * 3 * HW;
        const size_t slot_c = p.shared ? 0 : out_c, slot_w = p.shared ? 0 : out_w;
        const uint32_t starts = LOCAL ? a.seg[d] : 1u;         // scan steps without a predecessor

        // walking a line's scan steps in LDS: one running index, pinned in a register after every step so
        // that the compiler keeps a single address instead of one per step; it stops at the last step
        auto next = [&](int& idx, int s) {
            idx += (s + 1 < S) ? ss : 0;
            asm volatile("" : "+v"(idx));
        };

        float gw0[SMAX], gw1[SMAX], gw2[SMAX];
#pragma unroll
        for (int s = 0; s < SMAX; ++s) { gw0[s] = 0.f; gw1[s] = 0.f; gw2[s] = 0.f; }

        // Four / eight channels per wave: the group's three weight planes as one block of 3*HW elements, fetched in
        // pieces of a.wlw bytes (the block's start is a multiple of its size, so a piece that divides the size is
        // aligned), through the wave's LDS buffer into registers by scan step; `at` = this lane's element at step 0
        auto weight_block = [&](const T* wp, int at, float (&w0r)[SMAX], float (&w1r)[SMAX], float (&w2r)[SMAX]) {
            const int ew = a.wlw / (int)sizeof(T);
            const rsrc_t rs = make_rsrc(wp);
            for (int c = lane; c * ew < 3 * HW; c += 64) {
                const uint32_t bo = (uint32_t)(c * ew * (int)sizeof(T));
                u32x4 v = {0, 0, 0, 0};
                if (a.wlw == 16) v = __builtin_amdgcn_raw_buffer_load_b128(rs, bo, 0, 0);
                else if (a.wlw == 8) { const u32x2 t = __builtin_amdgcn_raw_buffer_load_b64(rs, bo, 0, 0); v[0] = t.x; v[1] = t.y; }
                else if (a.wlw == 4) v[0] = __builtin_amdgcn_raw_buffer_load_b32(rs, bo, 0, 0);
                else v[0] = (uint32_t)(uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rs, bo, 0, 0);
                float f[E];
                chunk_unpack<T, E>(v, f);
#pragma unroll
                for (int j = 0; j < E; ++j)
                    if (j < ew) bufX[c * ew + j] = f[j];
            }
#pragma unroll
            for (int s = 0, idx = at; s < SMAX; ++s) {
                w0r[s] = bufX[idx]; w1r[s] = bufX[idx + HW]; w2r[s] = bufX[idx + 2 * HW];
                next(idx, s);
            }
        };
        // LOGITS: softmax over the taps whose neighbour exists, per scan step; step 0 has no predecessor: no weight
        auto normalise = [&](float (&w0r)[SMAX], float (&w1r)[SMAX], float (&w2r)[SMAX]) {
#pragma unroll
            for (int s = 1; s < SMAX; ++s) softmax3(w0r[s], w1r[s], w2r[s], first, last);
            w0r[0] = 0.f; w1r[0] = 0.f; w2r[0] = 0.f;
        };
        for (int pair = wave; pair < pairs; pair += a.nwaves) {
            const int c0 = c_first + CPW * pair;
            const size_t pc = ((size_t)b * p.C + c0) * HW;
            const int g = c0 / p.cpg;
            const size_t wg = ((size_t)b * p.G + g) * 3 * HW;
            const T* gyp = (const T*)p.gy + pc;
            const T* xp = (const T*)p.x + pc;
            const T* lp = (const T*)p.lam + slot_c + pc;
            const T* up = (const T*)p.u + slot_c + pc;
            const T* hp = (const T*)p.hs + out_c + pc;
            const T* wp = (const T*)p.w + slot_w + wg;
            const rsrc_t glb = make_rsrc((T*)p.glam + out_c + pc);
            const rsrc_t gub = make_rsrc((T*)p.gu + out_c + pc);
            T* gwp = (T*)p.gw + out_w + wg;

            float sa[NCH][E], sb[NCH][E], sc[NCH][E];
            load_pair(gyp, sa);
            load_pair(hp, sb);
            load_pair(up, sc);
            // gu = gy*h in the flat layout; h goes to LDS for the weight gradients
#pragma unroll
            for (int k = 0; k < NCH; ++k) {
                if (vq[k]) {
                    float t[E];
#pragma unroll
                    for (int e = 0; e < E; ++e) t[e] = sa[k][e] * sb[k][e];
                    stg(gub, voff, k * 1024, t);
                }
            }
            to_lds(bufH, sb, false);
            if constexpr (CPW == 2) load_w(wp, sb);             // w0
            // seed u*gy, flat -> per-lane line positions
#pragma unroll
            for (int k = 0; k < NCH; ++k)
#pragma unroll
                for (int e = 0; e < E; ++e) sc[k][e] *= sa[k][e];
            to_lds(bufX, sc, false);
            if constexpr (CPW == 2) load_w(wp + HW, sa);        // w1
            float e[SMAX];
#pragma unroll
            for (int s = 0, idx = tb; s < SMAX; ++s) {
                const float v = bufX[idx];                    // unconditional read of a valid address, then select
                e[s] = active ? v : 0.f;
                next(idx, s);
            }
            float w0r[SMAX], w1r[SMAX], w2r[SMAX];
            if constexpr (CPW == 2) {
                load_w(wp + 2 * HW, sc);                        // w2
                to_lds(bufX, sb, shared_group);
#pragma unroll
                for (int s = 0, idx = tbw; s < SMAX; ++s) { w0r[s] = bufX[idx]; next(idx, s); }
                to_lds(bufX, sa, shared_group);
#pragma unroll
                for (int s = 0, idx = tbw; s < SMAX; ++s) { w1r[s] = bufX[idx]; next(idx, s); }
                to_lds(bufX, sc, shared_group);
#pragma unroll
                for (int s = 0, idx = tbw; s < SMAX; ++s) { w2r[s] = bufX[idx]; next(idx, s); }
            } else {
                weight_block(wp, tbw, w0r, w1r, w2r);
            }

            if constexpr (LOGITS) normalise(w0r, w1r, w2r);     // what was loaded are logits
            if constexpr (LOCAL) {
                // GSPN-local: nothing flows into the first line of a stretch -- its weights count as 0, and so
                // does the line before it where the weight gradients read it (h in LDS serves nothing else)
#pragma unroll
                for (int s = 1, idx = tb; s < SMAX; ++s) {
                    const bool z = (starts >> s) & 1u;
                    w0r[s] = z ? 0.f : w0r[s]; w1r[s] = z ? 0.f : w1r[s]; w2r[s] = z ? 0.f : w2r[s];
                    if (s < S) { if (z && active) bufH[idx] = 0.f; }     // h of scan step s-1
                    next(idx, s);
                }
            }
            // the sweep, against the scan order; the weights of scan step 0 are never used
#pragma unroll
            for (int s = SMAX - 2; s >= 0; --s) {
                if (s + 1 < S) {
                    const float en = e[s + 1];
                    const float q0 = w0r[s + 1] * en, q1 = w1r[s + 1] * en, q2 = w2r[s + 1] * en;
                    float lin = from_lane_below(q2), rin = from_lane_above(q0);
                    lin = first ? 0.f : lin;                    // no neighbour outside the line, whatever is stored
                    rin = last ? 0.f : rin;
                    const float v = e[s] + lin + q1 + rin;
                    e[s] = active ? v : 0.f;
                }
            }
            // x and lam are requested only now: while the weights are live there are no registers to park them in
            __builtin_amdgcn_sched_barrier(0);
            load_pair(xp, sb);
            load_pair(lp, sa);
            // weight gradients: e_s[j] * h_{s-1}[j-1, j, j+1]
            if constexpr (SHARED) {
#pragma unroll
                for (int s = 1, idx = tb; s < SMAX; ++s) {
                    if (s < S) {
                        const float hm = bufH[idx];             // h of scan step s-1
                        next(idx, s);
                        float hl = from_lane_below(hm), hr = from_lane_above(hm);
                        hl = first ? 0.f : hl;
                        hr = last ? 0.f : hr;
                        gw0[s] = fmaf(e[s], hl, gw0[s]);
                        gw1[s] = fmaf(e[s], hm, gw1[s]);
                        gw2[s] = fmaf(e[s], hr, gw2[s]);
                    }
                }
            }
            // e back to the flat layout: glam = x*e, gx += lam*e
#pragma unroll
            for (int s = 0, idx = tb; s < SMAX; ++s) {
                if (s < S) { if (active) bufX[idx] = e[s]; }
                next(idx, s);
            }
            f32a* tp = tile + (size_t)CPW * pair * HW;
#pragma unroll
            for (int k = 0; k < NCH; ++k) {
                if (vq[k]) {
                    const int q = k * 64 + lane;
                    float ef[E], acc[E], gl[E];
                    lds_get(bufX, q, ef);
                    lds_get(tp, q, acc);
#pragma unroll
                    for (int j = 0; j < E; ++j) { gl[j] = sb[k][j] * ef[j]; acc[j] = fmaf(sa[k][j], ef[j], acc[j]); }
                    stg(glb, voff, k * 1024, gl);
                    lds_put(tp, q, acc);
                }
            }
            if constexpr (!SHARED) {
                // one group per channel: this sweep's gw is complete; one tap at a time through the LDS buffer
                float dot[LOGITS ? SMAX : 1];                   // LOGITS: sum over the taps of w * gw, per scan step
                if constexpr (LOGITS) {
                    dot[0] = 0.f;
#pragma unroll
                    for (int s = 1, idh = tb; s < SMAX; ++s) {
                        const float hm = bufH[idh];             // h of scan step s-1
                        next(idh, s);
                        float hl = from_lane_below(hm), hr = from_lane_above(hm);
                        hl = first ? 0.f : hl;
                        hr = last ? 0.f : hr;
                        dot[s] = e[s] * fmaf(w0r[s], hl, fmaf(w1r[s], hm, w2r[s] * hr));
                    }
                }
#pragma unroll
                for (int t = 0; t < 3; ++t) {
#pragma unroll
                    for (int s = 0, idx = tb, idh = tb; s < SMAX; ++s) {
                        if (s < S) {
                            float v = 0.f;
                            if (s > 0) {
                                const float hm = bufH[idh];     // h of scan step s-1
                                next(idh, s);
                                float hn = t == 0 ? from_lane_below(hm) : (t == 2 ? from_lane_above(hm) : hm);
                                if (t == 0) hn = first ? 0.f : hn;
                                if (t == 2) hn = last ? 0.f : hn;
                                v = e[s] * hn;
                                if constexpr (LOGITS) v = (t == 0 ? w0r[s] : (t == 1 ? w1r[s] : w2r[s])) * (v - dot[s]);
                            }
                            if (active) bufX[idx] = v;
                        }
                        next(idx, s);
                    }
                    const rsrc_t gwb = make_rsrc(gwp + t * HW);
#pragma unroll
                    for (int k = 0; k < NCH; ++k) {
                        if (vq[k]) {
                            float v[E];
                            lds_get(bufX, k * 64 + lane, v);
                            stg(gwb, wq[k], 0, v);
                        }
                    }
                }
            }
        }

        if constexpr (SHARED && LOGITS) {
            // The softmax gradient is linear in gw: it is applied to this lane's partial sums before they are
            // added up.  The group's weights are fetched once more for it (keeping them in registers across
            // the loop above would cost more than this one fetch per direction).
            const int g = c_first / p.cpg;
            const T* wp = (const T*)p.w + slot_w + ((size_t)b * p.G + g) * 3 * HW;
            float w0r[SMAX], w1r[SMAX], w2r[SMAX];
            if constexpr (CPW == 2) {
                float st[NCH][E];
#pragma unroll
                for (int t = 0; t < 3; ++t) {
                    load_w(wp + t * HW, st);
                    to_lds(bufX, st, true);
#pragma unroll
                    for (int s = 0, idx = ic * ps + s0; s < SMAX; ++s) {
                        const float v = bufX[idx];
                        if (t == 0) w0r[s] = v; else if (t == 1) w1r[s] = v; else w2r[s] = v;
                        next(idx, s);
                    }
                }
            } else {
                weight_block(wp, ic * ps + s0, w0r, w1r, w2r);
            }
            normalise(w0r, w1r, w2r);
#pragma unroll
            for (int s = 0; s < SMAX; ++s) {
                // a step that starts a stretch has gw = 0 already; its weights count as 0 as well
                const bool z = LOCAL && ((starts >> s) & 1u);
                softmax3_grad(gw0[s], gw1[s], gw2[s], z ? 0.f : w0r[s], z ? 0.f : w1r[s], z ? 0.f : w2r[s]);
            }
        }
        if constexpr (SHARED && CPW > 2) {
            // sum over the channels of each wave, then over the waves (fixed order); the three taps are one block
            const int g = c_first / p.cpg;
            T* gwp = (T*)p.gw + out_w + ((size_t)b * p.G + g) * 3 * HW;
#pragma unroll
            for (int s = 0, idx = ic * ps + s0; s < SMAX; ++s) {
                float v0 = gw0[s], v1 = gw1[s], v2 = gw2[s];
#pragma unroll
                for (int m = 32; m >= LPC; m >>= 1) {
                    const int src = ((lane ^ m) & 63) << 2;
                    v0 += __int_as_float(__builtin_amdgcn_ds_bpermute(src, __float_as_int(v0)));
                    v1 += __int_as_float(__builtin_amdgcn_ds_bpermute(src, __float_as_int(v1)));
                    v2 += __int_as_float(__builtin_amdgcn_ds_bpermute(src, __float_as_int(v2)));
                }
                if (s < S) { if (active && half == 0) { bufX[idx] = v0; bufX[idx + HW] = v1; bufX[idx + 2 * HW] = v2; } }
                next(idx, s);
            }
            lds_barrier();
            const int ew = a.wlw / (int)sizeof(T);
            for (int el = (int)threadIdx.x * ew; el < 3 * HW; el += (int)blockDim.x * ew) {
                float acc[E];
#pragma unroll
                for (int j = 0; j < E; ++j) {
                    acc[j] = 0.f;
                    if (j < ew) {
                        acc[j] = wave_bufs[el + j];
                        for (int wv = 1; wv < a.nwaves; ++wv) acc[j] += wave_bufs[wv * 2 * CPW * HW + el + j];
                    }
                }
                if constexpr (sizeof(T) == 4) {
                    if (atomic) {
#pragma unroll
                        for (int j = 0; j < E; ++j)
                            if (j < ew) atomicAdd((float*)gwp + el + j, acc[j]);
                    } else {
                        store_piece<T, E>(gwp + el, acc, ew);
                    }
                } else {
                    store_piece<T, E>(gwp + el, acc, ew);
                }
            }
            lds_barrier();
        } else if constexpr (SHARED) {
            // sum over the two halves of each wave, then over the waves (fixed order), one tap at a time
            const int g = c_first / p.cpg;
            T* gwp = (T*)p.gw + out_w + ((size_t)b * p.G + g) * 3 * HW;
#pragma unroll
            for (int t = 0; t < 3; ++t) {
#pragma unroll
                for (int s = 0, idx = ic * ps + s0; s < SMAX; ++s) {
                    float v = t == 0 ? gw0[s] : (t == 1 ? gw1[s] : gw2[s]);
                    v += __int_as_float(__builtin_amdgcn_ds_bpermute(((lane ^ 32) & 63) << 2, __float_as_int(v)));
                    if (s < S) { if (active && half == 0) bufX[idx] = v; }
                    next(idx, s);
                }
                lds_barrier();
                for (int q = threadIdx.x; q < n16p; q += blockDim.x) {
                    float acc[E];
                    lds_get(wave_bufs, q, acc);
                    for (int wv = 1; wv < a.nwaves; ++wv) {
                        float o[E];
                        lds_get(wave_bufs + wv * 4 * HW, q, o);
#pragma unroll
                        for (int j = 0; j < E; ++j) acc[j] += o[j];
                    }
                    T* dst = gwp + t * HW + E * q;
                    if constexpr (sizeof(T) == 4) {
                        if (atomic) {
#pragma unroll
                            for (int j = 0; j < E; ++j) atomicAdd((float*)dst + j, acc[j]);
                        } else {
                            *(u32x4*)dst = chunk_pack<T, E>(acc);
                        }
                    } else {
                        *(u32x4*)dst = chunk_pack<T, E>(acc);
                    }
                }
                lds_barrier();
            }
        }
    }

    // merged gx of the wave's pairs: written once, coalesced
    for (int pair = wave; pair < pairs; pair += a.nwaves) {
        const f32a* tp = tile + (size_t)CPW * pair * HW;
        const rsrc_t gxb = make_rsrc((T*)p.gx + ((size_t)b * p.C + c_first + CPW * pair) * HW);
#pragma unroll
        for (int k = 0; k < NCH; ++k) {
            if (vq[k]) {
                float v[E];
                lds_get(tp, k * 64 + lane, v);
                stg(gxb, voff, k * 1024, v);
            }
        }
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
static constexpr int PLANE_LDS_BUDGET = 160 * 1024;

struct PlanePlan { bool ok; int K, shared_group, gsplit, nwaves, smax, cpw, wlw; size_t lds; };

static size_t plane_lds(int K, int nwaves, int HW, int cpw) {
    return (size_t)(K + 2 * cpw * nwaves) * HW * sizeof(float);
}

// waves per workgroup: the most (up to `cap`) that share the channel sets evenly and whose buffers fit
static int plane_waves(int K, int HW, int cap, int cpw) {
    const int sets = K / cpw;
    for (int n = cap; n > 1; --n)
        if (sets % n == 0 && plane_lds(K, n, HW, cpw) <= (size_t)PLANE_LDS_BUDGET) return n;
    return 1;
}

static PlanePlan plan_plane(const BwdParams& p, int dtype) {
    PlanePlan t = {};
    const int es = dtype == 0 ? 4 : 2, E = 16 / es;             // elements per 16 B of storage
    if (p.H < 2 || p.W < 2 || p.H > 32 || p.W > 32) return t;
    const int HW = p.H * p.W;
    const int m = p.H > p.W ? p.H : p.W;
    // channels per wave: eight / four when the lines are short enough, the group divides evenly and the
    // channels together are whole 16 B chunks; else two, which needs whole chunks per plane
    auto fits = [&](int cpw) { return (64 / cpw) >= m && p.cpg % cpw == 0 && ((size_t)cpw * HW * es) % 16 == 0; };
    if (p.cpg > 1 && fits(8)) { t.cpw = 8; t.smax = 8; }
    else if (p.cpg > 1 && fits(4)) { t.cpw = 4; t.smax = 16; }
    else {
        if (HW % E) return t;
        t.cpw = 2; t.smax = m <= 16 ? 16 : (m <= 28 ? 28 : 32);
    }
    const size_t wblock = (size_t)3 * HW * es;
    t.wlw = wblock % 16 == 0 ? 16 : wblock % 8 == 0 ? 8 : wblock % 4 == 0 ? 4 : 2;
    const int cap_shared = t.smax < 32 ? 6 : 4;                 // the 32-step variant needs more registers per wave
    if (p.cpg == 1) {
        t.shared_group = 0; t.gsplit = 1;
        t.K = (p.C % 8 == 0) ? 8 : ((p.C % 4 == 0) ? 4 : 2);
        if (p.C % t.K) return t;
    } else {
        if (p.cpg % 2) return t;
        t.shared_group = 1; t.gsplit = 1; t.K = p.cpg;
        const bool few = (size_t)p.B * p.G < 256;               // fewer workgroups than compute units
        // a split group adds into gw atomically, which needs fp32 storage
        if (dtype == 0 && (plane_lds(t.K, plane_waves(t.K, HW, cap_shared, t.cpw), HW, t.cpw) > (size_t)PLANE_LDS_BUDGET || few) &&
            t.K % (2 * t.cpw) == 0) {
            t.K /= 2; t.gsplit = 2;
        }
    }
    t.nwaves = plane_waves(t.K, HW, t.shared_group ? cap_shared : 4, t.cpw);
    t.lds = plane_lds(t.K, t.nwaves, HW, t.cpw);
    if (t.lds > (size_t)PLANE_LDS_BUDGET) return t;
    if ((size_t)p.B * (p.C / t.K) > 0x7fffffffull) return t;
    t.ok = true;
    return t;
}

bool bwd_plane_applicable(const BwdParams& p, int dtype) { return plan_plane(p, dtype).ok; }

template <typename T, int SMAX, int CPW, bool SHARED, bool LOCAL, bool LOGITS>
static hipError_t launch_plane_k(const BwdPlaneArgs& a, const PlanePlan& t, hipStream_t s) {
    auto k = bwd_plane_kernel<T, SMAX, CPW, SHARED, LOCAL, LOGITS>;
    hipError_t e = allow_dynamic_lds((const void*)k, PLANE_LDS_BUDGET);
    if (e != hipSuccess) return e;
    const dim3 grid((unsigned)((size_t)a.p.B * (a.p.C / a.K))), block(64 * a.nwaves);
    hipLaunchKernelGGL(k, grid, block, t.lds, s, a);
    return hipGetLastError();
}

// GSPN-local (Sec. 3.2) runs on instantiations of its own, so that the global scan carries none of it
template <typename T, int SMAX, int CPW, bool SHARED>
static hipError_t launch_plane(const BwdPlaneArgs& a, const PlanePlan& t, hipStream_t s) {
    // weights as logits always run the local instantiation (a global scan is one stretch: only step 0 starts one)
    if (a.p.logits) return launch_plane_k<T, SMAX, CPW, SHARED, true, true>(a, t, s);
    return a.p.kchunk > 0 ? launch_plane_k<T, SMAX, CPW, SHARED, true, false>(a, t, s)
                          : launch_plane_k<T, SMAX, CPW, SHARED, false, false>(a, t, s);
}

template <typename T>
static hipError_t launch_plane_t(const BwdPlaneArgs& a, const PlanePlan& t, hipStream_t s) {
    if (t.cpw == 8) return launch_plane<T, 8, 8, true>(a, t, s);
    if (t.cpw == 4) return launch_plane<T, 16, 4, true>(a, t, s);
    if (t.shared_group) {
        if (t.smax == 16) return launch_plane<T, 16, 2, true>(a, t, s);
        if (t.smax == 28) return launch_plane<T, 28, 2, true>(a, t, s);
        return launch_plane<T, 32, 2, true>(a, t, s);
    }
    if (t.smax == 16) return launch_plane<T, 16, 2, false>(a, t, s);
    if (t.smax == 28) return launch_plane<T, 28, 2, false>(a, t, s);
    return launch_plane<T, 32, 2, false>(a, t, s);
}

hipError_t launch_bwd_plane(const BwdParams& p, int dtype, hipStream_t s) {
    const PlanePlan t = plan_plane(p, dtype);
    if (!t.ok) return hipErrorInvalidValue;
    BwdPlaneArgs a;
    a.p = p; a.K = t.K; a.shared_group = t.shared_group; a.gsplit = t.gsplit; a.nwaves = t.nwaves; a.wlw = t.wlw;
    for (int d = 0; d < 4; ++d) a.seg[d] = (uint32_t)stretch_start_bits(d < 2 ? p.H : p.W, d & 1, p.kchunk, true);
    if (t.gsplit > 1) {
        // gw of the requested directions is accumulated atomically: clear it first, on the same stream
        const size_t per_dir = (size_t)p.B * p.G * 3 * p.H * p.W * sizeof(float);
        for (int d = 0; d < 4;) {                               // one fill per run of consecutive directions
            if (!((p.mask >> d) & 1u)) { ++d; continue; }
            int d1 = d;
            while (d1 < 4 && ((p.mask >> d1) & 1u)) ++d1;
            hipError_t e = launch_zero_fill((char*)p.gw + d * per_dir, (size_t)(d1 - d) * per_dir, s);
            if (e != hipSuccess) return e;
            d = d1;
        }
    }
    if (dtype == 2) return launch_plane_t<f16_t>(a, t, s);
    return dtype == 0 ? launch_plane_t<float>(a, t, s) : launch_plane_t<bf16_t>(a, t, s);
}

}  // namespace gspn
