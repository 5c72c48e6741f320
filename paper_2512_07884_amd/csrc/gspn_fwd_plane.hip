// Forward GSPN scan for small feature maps (lines of at most 64 positions, planes of at most 8 KB in
// storage precision: 56x56 bf16, 28x28 fp32, ...): every tensor is read from global memory exactly
// once per use as flat, fully coalesced 16 B-per-lane plane copies, and the scans run out of LDS.
//
// Per (channel, direction) the recurrence of Eq. 1 (Sec. 3.2)
//     h_s[j] = w0_s[j] h_{s-1}[j-1] + w1_s[j] h_{s-1}[j] + w2_s[j] h_{s-1}[j+1] + lam_s[j] x_s[j]
// is walked by one wave: lane = position j on the line (two channels side by side when a line fits
// in 32 lanes), the previous line's neighbours come from DPP whole-wave shifts, and the per-step
// operands a = lam*x, w0, w1, w2 are read from fp32 planes in LDS through an address walk whose stride
// encodes the direction (+-pitch for the vertical scans, +-1 for the horizontal ones), so that one
// code path serves all four directions.  h overwrites a in place; afterwards the plane is read back
// in the flat layout for y += u*h (Eq. 2 and the sum merge of the four passes, accumulated in
// registers and rounded once) and, when asked for, h_save.
//
// What this saves over line-by-line loading: x is loaded once for all directions and stays in
// registers; with channel-shared weights (Sec. 4.2) the three weight planes of a direction are
// loaded ONCE per workgroup into LDS and read by all its channels; every request is a complete
// cache line.  Rows in LDS have an odd pitch so that both access orientations are conflict-free.
//
// Maps whose rows are not whole 16 B chunks (7x7, 14x14, 28x28 bf16: the later stages of a classifier) take
// the FLAT variant: LDS planes without padding, so that a chunk's place in LDS is its place in memory and
// chunks may run over row and channel ends; 2, 4 or 8 channels side by side in a wave (32, 16 or 8 lanes
// each) so that the wave's channels together are whole chunks; weights fetched in the widest pieces their
// alignment allows.
#include "gspn_tile_common.hpp"
#include <stdlib.h>

namespace gspn {

namespace {

typedef float pf32a __attribute__((may_alias));
typedef __attribute__((address_space(3))) pf32a plds_f32;
extern __shared__ float plane_lds[];

__device__ __forceinline__ uint32_t plds_base() {
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)plane_lds;
}
__device__ __forceinline__ float plds_ld(uint32_t a) { return *(const plds_f32*)(uintptr_t)a; }
__device__ __forceinline__ void plds_st(uint32_t a, float v) { *(plds_f32*)(uintptr_t)a = v; }
typedef float pf32x4a __attribute__((ext_vector_type(4), may_alias));
typedef __attribute__((address_space(3))) pf32x4a plds_f32x4;
__device__ __forceinline__ pf32x4a plds_ld4(uint32_t a) { return *(const plds_f32x4*)(uintptr_t)a; }
__device__ __forceinline__ void plds_st4(uint32_t a, pf32x4a v) { *(plds_f32x4*)(uintptr_t)a = v; }

// element e of a 16 B chunk of storage, widened to fp32
template <typename T> __device__ __forceinline__ float chunk_elem(const u32x4& c, int e) {
    if constexpr (sizeof(T) == 4) return __uint_as_float(c[e]);
    else return (e & 1) ? word_hi<T>(c[e >> 1]) : word_lo<T>(c[e >> 1]);
}
template <typename T> __device__ __forceinline__ u32x4 chunk_pack(const float* v) {
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

}  // namespace

struct FwdPlaneArgs {
    FwdParams p;
    int K;        // channels per workgroup
    int cpw;      // channels per wave (1, 2, 4 or 8): each takes 64 / cpw lanes
    int lsh;      // log2 of the lanes per channel
    int nwaves;
    int pitch;    // LDS row pitch in floats (odd; W in the flat variant)
    int wlw;      // flat variant, shared weights: bytes per weight request (16, 8, 4 or 2)
    uint64_t seg[4];   // per direction: bit r set <=> image line r of the scan axis starts a stretch in scan order
};

// WPRE (shared weights): the workgroup has enough threads to hold a direction's weights in registers
// (WSH chunks per thread), so they are requested a direction ahead; otherwise they are fetched in place.
// FLAT: planes in LDS are unpadded and the wave's channels contiguous (see the head of the file).
// LOCAL: GSPN-local (Sec. 3.2), on instantiations of its own so that the global scan carries none of it.
// BWD: the reverse sweep of the backward pass (first pass of the two-pass backward scan) on the same machinery: the
// caller passes gy as x, u as lam, lam as u, gx as y and the buffer that receives e as hs; every direction is walked
// against its scan order, and a position multiplies its state by the taps of the line swept before and hands the
// products to the positions those taps read from (e_t = u_t*gy_t + T_{t+1}^T e_{t+1}).  The taps that are stored as 0
// (out-of-line neighbours, GSPN-local: lines that start a stretch) are the ones that must pass nothing on here too.
// NCHT: 16 B chunks per lane the register arrays are sized for (8: the wave's channels hold at most 8 KB; 4: small maps
// of the flat variant, which then has the registers to give its LDS planes an odd pitch too -- every element's place is
// tracked through two bit masks per chunk)
template <typename T, bool SAVE, bool SHARED, bool WPRE, bool FLAT, bool LOCAL, bool BWD = false, int NCHT = 8>
__global__ void __launch_bounds__(SHARED ? 512 : 256) fwd_plane_kernel(FwdPlaneArgs a) {
    static_assert(!(FLAT && WPRE), "the flat variant fetches its weights in place");
    static_assert(NCHT == 8 || (NCHT == 4 && FLAT), "the short register arrays are for small maps of the flat variant");
    constexpr bool PADFLAT = FLAT && NCHT == 4;    // flat variant with padded LDS planes
    static_assert(!BWD || SAVE, "the reverse sweep saves its state");
    constexpr int E = 16 / (int)sizeof(T);        // elements per 16 B chunk
    constexpr int NCH = NCHT;                     // chunks per lane
    constexpr int WSH = 4;                        // weight chunks per thread (shared weights)
    const FwdParams& p = a.p;
    const int H = p.H, W = p.W, HW = H * W, P = a.pitch;
    const int HP = (FLAT && !PADFLAT) ? HW : (H * P + 3) & ~3;   // floats per plane region in LDS (16 B granules when padded)
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int cpw = a.cpw;
    const int half = lane >> a.lsh;                    // which of the wave's channels this lane works on
    const int i = lane & ((1 << a.lsh) - 1);           // position on the line
    const int wgs_per_image = p.C / a.K;
    const unsigned item = xcd_contiguous_item(blockIdx.x, gridDim.x);
    const int b = item / wgs_per_image;
    const int c_first = (item - b * wgs_per_image) * a.K;
    const int c0 = c_first + wave * cpw;                               // first channel of this wave
    const size_t planes = (size_t)p.B * p.C, groups = (size_t)p.B * p.G;
    const size_t pc = ((size_t)b * p.C + c0) * HW;
    const int n16 = cpw * HW / E;                                      // 16 B chunks of the wave's channels
    const int n16p = HW / E;                                           // ... of one plane

    // LDS (floats).  Weights are kept interleaved, [H][P][4] = (w0, w1, w2, unused) per position, so that a scan
    // step fetches its three taps with one 16 B read.  Shared weights: one such region for the direction,
    // then per wave [cpw][H][P] a/h.  Per-channel weights: per wave [cpw] weight regions, then [cpw][H][P] a/h.
    const uint32_t base = plds_base();
    const uint32_t wreg = SHARED ? base : base + 4u * (uint32_t)(wave * cpw * 5 * HP);
    const uint32_t ahreg = SHARED ? base + 4u * (uint32_t)(4 * HP + wave * cpw * HP)
                                  : wreg + 4u * (uint32_t)(cpw * 4 * HP);

    // flat layout: chunk q = k*64 + lane covers elements [q*E, q*E + E) of the wave's channels
    bool vq[NCH];
    int rc[NCH];          // row*P + col of the chunk's first element (padded flat variant: plus its channel's region)
    int ch[NCH];          // channel of the wave (0 / 1) the chunk belongs to
    int row0[NCH], col0[NCH];
    // padded flat variant: a chunk may run over the end of a row and of a channel: bit e set <=> element e of the chunk is
    // the last of its row / of its channel, i.e. the next element's place in LDS is further by the row / region padding
    uint32_t rowend[NCH], chend[NCH];
#pragma unroll
    for (int k = 0; k < NCH; ++k) {
        const int q = k * 64 + lane;
        vq[k] = q < n16;
        const int idx0 = vq[k] ? q * E : 0;
        rowend[k] = 0; chend[k] = 0;
        if constexpr (PADFLAT) {
            const int c = idx0 / HW, rem = idx0 - c * HW;
            int row = rem / W, col = rem - row * W;
            ch[k] = 0; rc[k] = c * HP + row * P + col; row0[k] = 0; col0[k] = 0;
#pragma unroll
            for (int e = 0; e < E; ++e) {
                if (++col == W) {
                    col = 0; rowend[k] |= 1u << e;
                    if (++row == H) { row = 0; chend[k] |= 1u << e; }
                }
            }
        } else if constexpr (FLAT) {
            ch[k] = 0; rc[k] = idx0; row0[k] = 0; col0[k] = 0;     // LDS offset = offset in memory
        } else {
            ch[k] = idx0 >= HW ? 1 : 0;
            const int rem = idx0 - ch[k] * HW;
            const int row = rem / W;
            rc[k] = row * P + (rem - row * W);
            row0[k] = row; col0[k] = rem - row * W;
        }
    }
    const uint32_t flat = (uint32_t)lane * 16u;
    const uint32_t row_pad4 = 4u * (uint32_t)(P - W), ch_pad4 = 4u * (uint32_t)(HP - H * P);   // padded flat variant: bytes skipped at a row / channel end
    auto ldg = [&](rsrc_t rs, uint32_t vo, int so) -> u32x4 { return __builtin_amdgcn_raw_buffer_load_b128(rs, vo, so, 0); };
    // x, lam, u: each line is asked for once by the whole launch (CP_STREAM: the caches give it up first)
    auto load_planes = [&](const T* basep, u32x4 (&st)[NCH]) {
        const rsrc_t rs = make_rsrc(basep);
#pragma unroll
        for (int k = 0; k < NCH; ++k) {
            u32x4 v = {0, 0, 0, 0};
            if (vq[k]) v = __builtin_amdgcn_raw_buffer_load_b128(rs, flat, k * 1024, CP_STREAM);
            st[k] = v;
        }
    };

    // shared weights: the three planes of a direction are 3*n16p chunks, dealt round-robin to the threads
    const int nthreads = blockDim.x;
    bool wv[WSH];
    int wl[WSH];          // LDS float offset of the chunk's first element in the weight region (tap included)
    int wrow[WSH], wcol[WSH], wtap[WSH];
    uint32_t wgo[WSH];    // byte offset of the chunk from the group's first weight plane
    if constexpr (SHARED && WPRE) {
#pragma unroll
        for (int j = 0; j < WSH; ++j) {
            const int c = (int)threadIdx.x + j * nthreads;
            wv[j] = c < 3 * n16p;
            const int cc = wv[j] ? c : 0;
            const int tap = cc / n16p;
            const int idx0 = (cc - tap * n16p) * E;
            const int row = idx0 / W;
            wl[j] = 4 * (row * P + (idx0 - row * W)) + tap;
            wrow[j] = row; wcol[j] = idx0 - row * W; wtap[j] = tap;
            wgo[j] = (uint32_t)((tap * HW + idx0) * (int)sizeof(T));
        }
    }
    auto load_wshare = [&](const T* wbase, u32x4 (&st)[WSH]) {
        const rsrc_t rs = make_rsrc(wbase);
#pragma unroll
        for (int j = 0; j < WSH; ++j) {
            u32x4 v = {0, 0, 0, 0};
            if (wv[j]) v = ldg(rs, wgo[j], 0);
            st[j] = v;
        }
    };

    u32x4 xs[NCH];
    load_planes((const T*)p.x + pc, xs);
    float y[NCH][E];
#pragma unroll
    for (int k = 0; k < NCH; ++k)
#pragma unroll
        for (int e = 0; e < E; ++e) y[k][e] = 0.f;

    // directions in scan order; operands of the first one are requested here, later ones a direction ahead
    int d = 0;
    while (d < 4 && !((p.mask >> d) & 1u)) ++d;
    const int g = c_first / p.cpg;                                     // shared weights: the workgroup's group
    auto slot_c = [&](int dd) { return p.shared ? (size_t)0 : (size_t)dd * planes * HW; };
    auto wptr = [&](int dd, int grp) {
        return (const T*)p.w + (p.shared ? (size_t)0 : (size_t)dd * groups * 3 * HW) + ((size_t)b * p.G + grp) * 3 * HW;
    };
    u32x4 ls[NCH], us[NCH], wsh[WSH];
    if (d < 4) {
        load_planes((const T*)p.lam + slot_c(d) + pc, ls);
        if constexpr (SHARED && WPRE) load_wshare(wptr(d, g), wsh);
    }

    while (d < 4) {
        int dn = d + 1;
        while (dn < 4 && !((p.mask >> dn) & 1u)) ++dn;
        // element (position j, scan step s) of a plane sits at float offset j*ps + s0 + s*ss
        const bool vert = d < 2, rev = ((d & 1) != 0) != BWD;       // (the reverse sweep walks against the scan order)
        const int S = vert ? H : W, L = vert ? W : H;
        const int ps = vert ? 1 : P;
        const int ss4 = 4 * (vert ? (rev ? -P : P) : (rev ? -1 : 1));
        const int s0 = vert ? (rev ? (H - 1) * P : 0) : (rev ? W - 1 : 0);
        const bool active = i < L;
        const int ic = active ? i : L - 1;
        const bool first = i == 0, last = i == L - 1;
        const int tpos = ic * ps + s0;
        // GSPN-local (Sec. 3.2): a line that starts a stretch has no predecessor, so its three taps are stored as 0
        // like the out-of-line ones, and the sweep restarts from lam*x there without knowing about stretches.
        // The prefetching variant has no registers to spare for the test where the weights are written: it clears
        // those lines in a pass of its own afterwards.
        constexpr bool LOCAL_PASS = LOCAL && WPRE;
        // weights given as logits: a tap that takes no part is stored as -inf and the three are normalised in LDS
        const float masked = p.logits ? -__builtin_huge_valf() : 0.f;
        const uint64_t starts = LOCAL ? a.seg[d] : 0ull;
        auto no_pred = [&](int row, int col) { return LOCAL && !LOCAL_PASS && ((starts >> (vert ? row : col)) & 1ull) != 0; };

        // ---- operands into LDS
        if constexpr (FLAT) {
            if constexpr (SHARED) lds_barrier();           // every wave is done with the previous direction's weights
            // The block to bring in: the group's three planes (the threads of the workgroup share the work) or
            // the three planes of each of the wave's channels, which are contiguous in memory.  A request may run
            // over the end of a row, a plane or a channel: the place of every element is tracked on its own.
            const int nel = SHARED ? 3 * HW : cpw * 3 * HW;
            const int lw = SHARED ? a.wlw : 16;
            const int ew = lw / (int)sizeof(T);            // elements per request; divides nel (host)
            const int t0 = SHARED ? (int)threadIdx.x : lane, tn = SHARED ? nthreads : 64;
            const rsrc_t rs = make_rsrc(wptr(d, SHARED ? g : c0));
            for (int c = t0; c * ew < nel; c += tn) {
                const int idx0 = c * ew;
                const uint32_t bo = (uint32_t)(idx0 * (int)sizeof(T));
                u32x4 v = {0, 0, 0, 0};
                if (lw == 16) v = ldg(rs, bo, 0);
                else if (lw == 8) { const u32x2 t = __builtin_amdgcn_raw_buffer_load_b64(rs, bo, 0, 0); v[0] = t.x; v[1] = t.y; }
                else if (lw == 4) v[0] = __builtin_amdgcn_raw_buffer_load_b32(rs, bo, 0, 0);
                else v[0] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b16(rs, bo, 0, 0);
                int chn = idx0 / (3 * HW);
                int r = idx0 - chn * 3 * HW;
                int tap = r / HW;
                r -= tap * HW;
                int row = r / W, col = r - row * W;
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    if (e < ew) {
                        // a tap that points outside the line is stored as 0, whatever the tensor holds there
                        const int pos = vert ? col : row;
                        const bool outside = (tap == 0 && pos == 0) || (tap == 2 && pos == L - 1) || no_pred(row, col);
                        plds_st(wreg + 4u * (uint32_t)(chn * 4 * HP + 4 * (row * P + col) + tap),
                                outside ? masked : chunk_elem<T>(v, e));
                        if (++col == W) { col = 0; if (++row == H) { row = 0; if (++tap == 3) { tap = 0; ++chn; } } }
                    }
                }
            }
        } else if constexpr (SHARED) {
            lds_barrier();                                 // every wave is done with the previous direction's weights
            if constexpr (WPRE) {
#pragma unroll
                for (int j = 0; j < WSH; ++j) {
                    if (wv[j]) {
#pragma unroll
                        for (int e = 0; e < E; ++e) {
                            // a tap that points outside the line is stored as 0, whatever the tensor holds there
                            const int pos = vert ? wcol[j] + e : wrow[j];
                            const bool outside = (wtap[j] == 0 && pos == 0) || (wtap[j] == 2 && pos == L - 1) ||
                                                 no_pred(wrow[j], wcol[j] + e);
                            plds_st(wreg + 4u * (uint32_t)(wl[j] + 4 * e), outside ? masked : chunk_elem<T>(wsh[j], e));
                        }
                    }
                }
            } else {
                // small workgroups: fetched here, without the head start
                const rsrc_t rs = make_rsrc(wptr(d, g));
                for (int c = (int)threadIdx.x; c < 3 * n16p; c += nthreads) {
                    const int tap = c / n16p;
                    const int idx0 = (c - tap * n16p) * E;
                    const int row = idx0 / W, col = idx0 - row * W;
                    const u32x4 v = ldg(rs, (uint32_t)((tap * HW + idx0) * (int)sizeof(T)), 0);
#pragma unroll
                    for (int e = 0; e < E; ++e) {
                        const int pos = vert ? col + e : row;
                        const bool outside = (tap == 0 && pos == 0) || (tap == 2 && pos == L - 1) || no_pred(row, col + e);
                        plds_st(wreg + 4u * (uint32_t)(4 * (row * P + col + e) + tap), outside ? masked : chunk_elem<T>(v, e));
                    }
                }
            }
        } else {
            // the wave's own channels: three planes each, 3*HW elements apart per channel
#pragma unroll
            for (int t = 0; t < 3; ++t) {
                const rsrc_t rs = make_rsrc(wptr(d, c0) + (size_t)t * HW);
                u32x4 wt[NCH];
#pragma unroll
                for (int k = 0; k < NCH; ++k) {
                    u32x4 v = {0, 0, 0, 0};
                    if (vq[k]) v = ldg(rs, (uint32_t)(((ch[k] * 2 * HW) + (k * 64 + lane) * E) * (int)sizeof(T)), 0);
                    wt[k] = v;
                }
#pragma unroll
                for (int k = 0; k < NCH; ++k) {
                    if (vq[k]) {
                        const uint32_t o = wreg + 4u * (uint32_t)(ch[k] * 4 * HP + 4 * rc[k] + t);
#pragma unroll
                        for (int e = 0; e < E; ++e) {
                            const int pos = vert ? col0[k] + e : row0[k];
                            const bool outside = (t == 0 && pos == 0) || (t == 2 && pos == L - 1) || no_pred(row0[k], col0[k] + e);
                            plds_st(o + 16u * e, outside ? masked : chunk_elem<T>(wt[k], e));
                        }
                    }
                }
            }
        }
        // a = lam * x
#pragma unroll
        for (int k = 0; k < NCH; ++k) {
            if (vq[k]) {
                uint32_t o = ahreg + 4u * (uint32_t)(ch[k] * HP + rc[k]);
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    if constexpr (PADFLAT) {
                        plds_st(o, chunk_elem<T>(ls[k], e) * chunk_elem<T>(xs[k], e));
                        o += 4u + (((rowend[k] >> e) & 1u) ? row_pad4 : 0u) + (((chend[k] >> e) & 1u) ? ch_pad4 : 0u);
                    } else {
                        plds_st(o + 4u * e, chunk_elem<T>(ls[k], e) * chunk_elem<T>(xs[k], e));
                    }
                }
            }
        }
        // requests for after the sweep (u) and for the next direction (lam, shared weights)
        load_planes((const T*)p.u + slot_c(d) + pc, us);
        if (dn < 4) {
            load_planes((const T*)p.lam + slot_c(dn) + pc, ls);
            if constexpr (SHARED && WPRE) load_wshare(wptr(dn, g), wsh);
        }
        if constexpr (SHARED) lds_barrier();               // weights of this direction are in place (LDS only: the
                                                           // requests above stay in flight across the barrier)

        if (p.logits) {
            // Sec. 3.2 normalisation: softmax over the taps of a position that take part (the others hold -inf);
            // a line without predecessor (GSPN-local: first line of a stretch) gets three zeros
            const int nreg = SHARED ? 1 : cpw;             // weight regions: the group's, or the wave's own
            const int t0 = SHARED ? (int)threadIdx.x : lane, tn = SHARED ? nthreads : 64;
            // (padding positions are normalised like the rest: what they hold is never read)
            const float inv_hp = 1.0f / (float)HP, inv_p = 1.0f / (float)P;
            for (int idx = t0; idx < nreg * HP; idx += tn) {
                const uint32_t o = wreg + 16u * (uint32_t)idx;
                pf32x4a z = plds_ld4(o);
                const float m = fmaxf(z.y, fmaxf(z.x, z.z));
                bool none = m == -__builtin_huge_valf();
                if constexpr (LOCAL) {
                    // (row, column) of the position; the float quotients are exact at these sizes (idx < 2^16, P <= 65)
                    const int chn = (int)(((float)idx + 0.5f) * inv_hp), pos = idx - chn * HP;
                    const int row = (int)(((float)pos + 0.5f) * inv_p), col = pos - row * P;
                    none = none || ((starts >> ((vert ? row : col) & 63)) & 1ull) != 0;
                }
                const float e0 = __expf(z.x - m), e1 = __expf(z.y - m), e2 = __expf(z.z - m);
                const float r = 1.0f / (e0 + e1 + e2);
                z.x = none ? 0.f : e0 * r; z.y = none ? 0.f : e1 * r; z.z = none ? 0.f : e2 * r; z.w = 0.f;
                plds_st4(o, z);
            }
            if constexpr (SHARED) lds_barrier();
        } else if constexpr (LOCAL_PASS) {
            for (int r = 0; r < S; ++r) {
                if (!((starts >> r) & 1ull)) continue;
                for (int j = (int)threadIdx.x; j < L; j += nthreads) {
                    const uint32_t o = wreg + 16u * (uint32_t)(vert ? r * P + j : j * P + r);
                    plds_st(o, 0.f); plds_st(o + 4u, 0.f); plds_st(o + 8u, 0.f);
                }
            }
            lds_barrier();
        }

        // ---- the scan: h overwrites a
        {
            uint32_t aad = ahreg + 4u * (uint32_t)(half * HP + tpos);
            uint32_t wad = wreg + 16u * (uint32_t)((SHARED ? 0 : half * HP) + tpos);
            float h = plds_ld(aad);                        // scan step 0: no previous line, its weights are never read
            pf32x4a wp = plds_ld4(wad);                    // BWD: taps of the line swept before
            // lanes past the end of the line walk the last position's operands; what they compute is never
            // stored, and the selects below keep it out of the line
            auto step = [&]() {
                aad += (uint32_t)ss4; wad += (uint32_t)(4 * ss4);
                const float av = plds_ld(aad);
                const pf32x4a w = plds_ld4(wad);
                if constexpr (BWD) {
                    float lin = from_lane_below(wp.z * h), rin = from_lane_above(wp.x * h);
                    lin = first ? 0.f : lin;
                    rin = last ? 0.f : rin;
                    h = fmaf(wp.y, h, av) + (lin + rin);
                    wp = w;
                } else {
                    float hl = from_lane_below(h), hr = from_lane_above(h);
                    hl = first ? 0.f : hl;                 // no neighbour outside the line (its weight is stored as 0)
                    hr = last ? 0.f : hr;
                    h = fmaf(w.x, hl, fmaf(w.y, h, fmaf(w.z, hr, av)));
                }
                if (active) plds_st(aad, h);
            };
            // four steps per trip: their operand reads do not depend on h and are issued together
            int s = 1;
            for (; s + 7 < S; s += 8) { step(); step(); step(); step(); step(); step(); step(); step(); }
            for (; s + 3 < S; s += 4) { step(); step(); step(); step(); }
            for (; s < S; ++s) step();
        }

        // ---- back in the flat layout: y += u*h, optional h_save
        {
            const rsrc_t hb = make_rsrc(SAVE ? (T*)p.hs + (size_t)d * planes * HW + pc : (T*)p.y);
#pragma unroll
            for (int k = 0; k < NCH; ++k) {
                if (vq[k]) {
                    uint32_t o = ahreg + 4u * (uint32_t)(ch[k] * HP + rc[k]);
                    float hv[E];
#pragma unroll
                    for (int e = 0; e < E; ++e) {
                        if constexpr (PADFLAT) {
                            hv[e] = plds_ld(o);
                            o += 4u + (((rowend[k] >> e) & 1u) ? row_pad4 : 0u) + (((chend[k] >> e) & 1u) ? ch_pad4 : 0u);
                        } else {
                            hv[e] = plds_ld(o + 4u * e);
                        }
                        y[k][e] = fmaf(chunk_elem<T>(us[k], e), hv[e], y[k][e]);
                    }
                    if constexpr (SAVE) st_b128<CP_STREAM>(hb, flat + k * 1024, chunk_pack<T>(hv));
                }
            }
        }
        d = dn;
    }

    // merged output, rounded once
    {
        const rsrc_t yb = make_rsrc((T*)p.y + pc);
#pragma unroll
        for (int k = 0; k < NCH; ++k)
            if (vq[k]) st_b128<CP_STREAM>(yb, flat + k * 1024, chunk_pack<T>(y[k]));
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
static constexpr int FPLANE_LDS_BUDGET = 160 * 1024;

struct FwdPlanePlan { bool ok, flat, small; int K, cpw, lsh, nwaves, pitch, shared_group, wlw; size_t lds; };

// waves per workgroup and LDS bytes, given the channels per wave and the bytes of one fp32 plane region
static bool plan_fwd_plane_waves(const FwdParams& p, FwdPlanePlan& t, size_t hp) {
    if (p.cpg == 1) {
        t.shared_group = 0;
        // per wave: cpw * (4 weight + 1 a/h) planes; aim at 4 waves per workgroup
        int nw = 4;
        while (nw > 1 && (p.C % (nw * t.cpw) || (size_t)nw * t.cpw * 5 * hp > (size_t)FPLANE_LDS_BUDGET)) --nw;
        if (p.C % (nw * t.cpw) || (size_t)nw * t.cpw * 5 * hp > (size_t)FPLANE_LDS_BUDGET) return false;
        t.nwaves = nw; t.K = nw * t.cpw;
        t.lds = (size_t)nw * t.cpw * 5 * hp;
    } else {
        t.shared_group = 1;
        // the most waves (up to 8) whose channels divide the group and whose planes fit beside the weights
        int nw = 8;
        for (; nw >= 1; --nw) {
            if ((p.cpg / t.cpw) % nw) continue;
            if ((4 + (size_t)nw * t.cpw) * hp > (size_t)FPLANE_LDS_BUDGET) continue;
            break;
        }
        if (nw < 1) return false;
        t.nwaves = nw; t.K = nw * t.cpw;
        t.lds = (4 + (size_t)nw * t.cpw) * hp;
    }
    return (size_t)p.B * (p.C / t.K) <= 0x7fffffffull;
}

static FwdPlanePlan plan_fwd_plane(const FwdParams& p, int dtype) {
    FwdPlanePlan t = {};
    const int es = dtype == 0 ? 4 : 2, E = 16 / es;
    if (p.H < 2 || p.W < 2 || p.H > 64 || p.W > 64) return t;
    if (p.xt) return t;                                    // transposed-horizontal layout: tile and generic kernels
    const int HW = p.H * p.W;
    const int m = p.H > p.W ? p.H : p.W;
    if (p.W % E == 0) {
        // padded planes, one or two channels per wave
        t.cpw = m <= 32 ? 2 : 1;
        if ((size_t)t.cpw * HW * es > 8192) {
            if (t.cpw == 2 && (size_t)HW * es <= 8192) t.cpw = 1; else return t;
        }
        if (p.cpg == 1 ? p.C % t.cpw : p.cpg % t.cpw) t.cpw = 1;
        t.lsh = t.cpw == 2 ? 5 : 6;
        t.pitch = p.W | 1;
        const size_t hp = (((size_t)p.H * t.pitch + 3) & ~(size_t)3) * sizeof(float);   // one plane region in LDS
        t.ok = plan_fwd_plane_waves(p, t, hp);
        return t;
    }
    // flat planes: the most channels per wave (each on 64 / cpw lanes) that are whole 16 B chunks together
    t.flat = true;
    int lsh = 3;
    while ((1 << lsh) < m) ++lsh;
    for (; lsh <= 6; ++lsh) {
        const int cpw = 64 >> lsh;
        if ((size_t)cpw * HW * es % 16 || (size_t)cpw * HW * es > 8192) continue;
        if (p.cpg == 1 ? p.C % cpw : p.cpg % cpw) continue;
        t.cpw = cpw; t.lsh = lsh;
        break;
    }
    if (!t.cpw) return t;
    // small maps (at most four 16 B chunks per lane) get an odd pitch like the padded variant; larger ones keep rows packed
    t.small = (size_t)t.cpw * HW * es <= 4 * 64 * 16;
    t.pitch = t.small ? (p.W | 1) : p.W;
    // shared weights: the widest request that divides a group's block (its start is a multiple of its size)
    const size_t wblock = (size_t)3 * HW * es;
    t.wlw = wblock % 16 == 0 ? 16 : wblock % 8 == 0 ? 8 : wblock % 4 == 0 ? 4 : 2;
    t.ok = plan_fwd_plane_waves(p, t, t.small ? (((size_t)p.H * t.pitch + 3) & ~(size_t)3) * sizeof(float) : (size_t)HW * sizeof(float));
    return t;
}

bool fwd_plane_applicable(const FwdParams& p, int dtype) { return plan_fwd_plane(p, dtype).ok; }

template <typename T, bool SAVE, bool SHARED, bool WPRE, bool FLAT, bool LOCAL, bool BWD, int NCH>
static hipError_t launch_fplane_kn(const FwdPlaneArgs& a, const FwdPlanePlan& t, hipStream_t s) {
    auto k = fwd_plane_kernel<T, SAVE, SHARED, WPRE, FLAT, LOCAL, BWD, NCH>;
    hipError_t e = allow_dynamic_lds((const void*)k, FPLANE_LDS_BUDGET);
    if (e != hipSuccess) return e;
    const dim3 grid((unsigned)((size_t)a.p.B * (a.p.C / a.K))), block(64 * a.nwaves);
    hipLaunchKernelGGL(k, grid, block, t.lds, s, a);
    return hipGetLastError();
}

template <typename T, bool SAVE, bool SHARED, bool WPRE, bool FLAT, bool LOCAL, bool BWD = false>
static hipError_t launch_fplane_kl(const FwdPlaneArgs& a, const FwdPlanePlan& t, hipStream_t s) {
    if constexpr (FLAT) {
        if (t.small) return launch_fplane_kn<T, SAVE, SHARED, WPRE, FLAT, LOCAL, BWD, 4>(a, t, s);
    }
    return launch_fplane_kn<T, SAVE, SHARED, WPRE, FLAT, LOCAL, BWD, 8>(a, t, s);
}

template <typename T, bool SAVE, bool SHARED, bool WPRE, bool FLAT>
static hipError_t launch_fplane_k(const FwdPlaneArgs& a, const FwdPlanePlan& t, hipStream_t s) {
    return a.p.kchunk > 0 ? launch_fplane_kl<T, SAVE, SHARED, WPRE, FLAT, true>(a, t, s)
                          : launch_fplane_kl<T, SAVE, SHARED, WPRE, FLAT, false>(a, t, s);
}

template <typename T, bool SAVE, bool SHARED>
static hipError_t launch_fplane(const FwdPlaneArgs& a, const FwdPlanePlan& t, hipStream_t s) {
    if (t.flat) return launch_fplane_k<T, SAVE, SHARED, false, true>(a, t, s);
    if constexpr (SHARED) {
        const int E = 16 / (int)sizeof(T);
        const bool wpre = 3 * (a.p.H * a.p.W / E) <= 4 * 64 * a.nwaves;   // WSH chunks per thread
        return wpre ? launch_fplane_k<T, SAVE, true, true, false>(a, t, s)
                    : launch_fplane_k<T, SAVE, true, false, false>(a, t, s);
    } else {
        return launch_fplane_k<T, SAVE, false, false, false>(a, t, s);
    }
}

template <typename T>
static hipError_t launch_fplane_t(const FwdPlaneArgs& a, const FwdPlanePlan& t, hipStream_t s) {
    if (a.p.hs) return t.shared_group ? launch_fplane<T, true, true>(a, t, s) : launch_fplane<T, true, false>(a, t, s);
    return t.shared_group ? launch_fplane<T, false, true>(a, t, s) : launch_fplane<T, false, false>(a, t, s);
}

// reverse sweep (first pass of the two-pass backward scan): the same choice of variant, state always saved
template <typename T, bool SHARED, bool WPRE, bool FLAT>
static hipError_t launch_fplane_rev_k(const FwdPlaneArgs& a, const FwdPlanePlan& t, hipStream_t s) {
    return a.p.kchunk > 0 ? launch_fplane_kl<T, true, SHARED, WPRE, FLAT, true, true>(a, t, s)
                          : launch_fplane_kl<T, true, SHARED, WPRE, FLAT, false, true>(a, t, s);
}
template <typename T, bool SHARED>
static hipError_t launch_fplane_rev(const FwdPlaneArgs& a, const FwdPlanePlan& t, hipStream_t s) {
    if (t.flat) return launch_fplane_rev_k<T, SHARED, false, true>(a, t, s);
    if constexpr (SHARED) {
        const int E = 16 / (int)sizeof(T);
        const bool wpre = 3 * (a.p.H * a.p.W / E) <= 4 * 64 * a.nwaves;   // WSH chunks per thread
        return wpre ? launch_fplane_rev_k<T, true, true, false>(a, t, s) : launch_fplane_rev_k<T, true, false, false>(a, t, s);
    } else {
        return launch_fplane_rev_k<T, false, false, false>(a, t, s);
    }
}

bool reverse_sweep_plane_applicable(const FwdParams& p, int dtype) { return plan_fwd_plane(p, dtype).ok; }

// p holds gy as x, u as lam, lam as u, gx as y and the buffer that receives e as hs
hipError_t launch_reverse_sweep_plane(const FwdParams& p, int dtype, hipStream_t s) {
    const FwdPlanePlan t = plan_fwd_plane(p, dtype);
    if (!t.ok || !p.hs) return hipErrorInvalidValue;
    FwdPlaneArgs a;
    a.p = p; a.K = t.K; a.cpw = t.cpw; a.lsh = t.lsh; a.nwaves = t.nwaves; a.pitch = t.pitch; a.wlw = t.wlw;
    for (int d = 0; d < 4; ++d) a.seg[d] = stretch_start_bits(d < 2 ? p.H : p.W, d & 1, p.kchunk, false);
    if (dtype == 0) return t.shared_group ? launch_fplane_rev<float, true>(a, t, s) : launch_fplane_rev<float, false>(a, t, s);
    if (dtype == 2) return t.shared_group ? launch_fplane_rev<f16_t, true>(a, t, s) : launch_fplane_rev<f16_t, false>(a, t, s);
    return t.shared_group ? launch_fplane_rev<bf16_t, true>(a, t, s) : launch_fplane_rev<bf16_t, false>(a, t, s);
}

hipError_t launch_fwd_plane(const FwdParams& p, int dtype, hipStream_t s) {
    const FwdPlanePlan t = plan_fwd_plane(p, dtype);
    if (!t.ok) return hipErrorInvalidValue;
    FwdPlaneArgs a;
    a.p = p; a.K = t.K; a.cpw = t.cpw; a.lsh = t.lsh; a.nwaves = t.nwaves; a.pitch = t.pitch; a.wlw = t.wlw;
    for (int d = 0; d < 4; ++d) a.seg[d] = stretch_start_bits(d < 2 ? p.H : p.W, d & 1, p.kchunk, false);
    if (dtype == 2) return launch_fplane_t<f16_t>(a, t, s);
    return dtype == 0 ? launch_fplane_t<float>(a, t, s) : launch_fplane_t<bf16_t>(a, t, s);
}

}  // namespace gspn
