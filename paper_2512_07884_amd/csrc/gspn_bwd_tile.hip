// Backward GSPN scan for small feature maps (fp32 or bf16 storage, H <= 64, W <= 128): all directions in
// one launch, wave-owned lines in registers, the merged gradient gx accumulated in an fp32 LDS tile.
//
// The paper gives timings but no algorithm for the backward pass (Sec. 5.1); this is the chain rule
// on Eq. 1-2 (Sec. 3.2) with the shared weights of Sec. 4.2.  Per direction, sweeping the lines
// against the scan order, with e_t = dL/dh_t:
//     q_k[j]  = w_k[t+1][j] * e_{t+1}[j]                       (k = 0, 1, 2; 0 past the last line)
//     e_t[j]  = u_t[j]*gy_t[j] + q_2[j-1] + q_1[j] + q_0[j+1]    (transposed tridiagonal)
//     gu_t = gy_t*h_t,  glam_t = x_t*e_t,  gx_t += lam_t*e_t (summed over directions)
//     gw_t[k][j] = sum over the channels of the group of e_t[j] * h_{t-1}[j+k-1]
// so the cross-lane traffic per line is q_2 from the lane below, q_0 from the lane above and the
// two shifted copies of h_{t-1} (DPP whole-wave shifts), as in the forward kernel.
//
// Work split: one workgroup owns K consecutive channels of one image.  A wave owns one direction
// and walks its lines against the scan order; for every line it loops over its "rounds" (packs of
// channels that sit side by side in the wave).  The carried state e of each round lives in a few
// hundred bytes of LDS, the weights of the previous line stay in registers for all rounds, and gw
// is summed over the rounds in registers, then over the side-by-side channels with cross-lane
// reads, and leaves the wave once per line: stored directly when the workgroup holds the whole
// weight group, added atomically onto a zero-filled gw when the group is split over two
// workgroups (two addends commute, so the result stays bitwise reproducible).  With one channel
// per group (the per-channel weights of Eq. 1) every wave has a single round and every lane
// stores its own gw.
#include "gspn_tile_common.hpp"
#include <stdlib.h>

namespace gspn {

struct BwdTileArgs {
    BwdParams p;
    int K;            // channels per workgroup
    int pitch;        // gx tile row pitch in floats (odd)
    int lplv, pv;     // vertical phases: lanes per line, channels side by side
    int ph;           // horizontal phases: channels side by side (one image row per lane, H lanes per line)
    int shared_group; // 1: the K channels share one weight group; 0: one weight group per channel
    int gsplit;       // workgroups per weight group (shared_group only); > 1: gw is accumulated atomically
    int seq_parts;    // > 1: a group is covered by this many launches, one slice of K channels each
    int seq_index;    // which slice this launch covers; slices after the first add onto the stored gw
    int nwaves;
    int est_floats;   // LDS floats per wave for the carried state of its rounds
};

// lane-wise sum over the `slots` channel slots that sit `stride` lanes apart (this lane is in slot
// `slot`); the total is valid in slot 0
__device__ __forceinline__ float slot_sum(float v, int slots, int stride, int lane, int slot) {
    for (int s = 1; s < slots; s <<= 1) {
        const int src = lane + s * stride;
        const float o = __int_as_float(__builtin_amdgcn_ds_bpermute((src & 63) << 2, __float_as_int(v)));
        v += (slot + s < slots) ? o : 0.f;
    }
    return v;
}

__device__ __forceinline__ void gw_out(rsrc_t rs, char* base, uint32_t voff, int so, float v, bool atomic) {
    if (atomic) atomicAdd((float*)(base + so + voff), v);
    else __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), rs, voff, __builtin_amdgcn_readfirstlane(so), 0);
}

// gw of one line leaves the wave: plain store, or (later launches over the same group) stored value + v
template <typename T, int V>
__device__ __forceinline__ void gw_store(rsrc_t rs, uint32_t voff, int so, const float (&v)[V], bool add) {
    constexpr int NB = V * (int)sizeof(T);
    uint32_t o[NB / 4];
    float t[V];
#pragma unroll
    for (int k = 0; k < V; ++k) t[k] = v[k];
    if (add) {
        ld_buf<NB>(rs, voff, so, o);
#pragma unroll
        for (int k = 0; k < V; ++k) t[k] += elem<T>(o, k);
    }
    pack<T, V>(t, o);
    st_buf<NB>(rs, voff, so, o);
}

// ---------------------------------------------------------------------------
// vertical directions: lines are image rows, 2 adjacent columns per lane
// ---------------------------------------------------------------------------
// LOCAL: GSPN-local (Sec. 3.2), on instantiations of its own so that the global scan carries none of it
// LOGITS (with LOCAL): w holds raw logits (normalised as they are consumed) and gw receives the gradient w.r.t. them
template <typename T, int PF, bool REV, bool LOCAL, bool LOGITS>
__device__ __forceinline__ void bwd_vertical(const BwdTileArgs& a, float* tile, float* est, int b, int c_first,
                                             int pk0, int rounds, int lane, int split) {
    constexpr int V = 2;
    constexpr int NB = V * (int)sizeof(T);
    constexpr int NR = NB / 4;
    constexpr int d = REV ? 1 : 0;
    const BwdParams& p = a.p;
    const int H = p.H, W = p.W, HW = H * W;
    const int pl = lane / a.lplv, i = lane - pl * a.lplv;
    const bool active = pl < a.pv;
    const int plc = active ? pl : 0, ic = active ? i : 0;
    const bool first = ic == 0, last = ic == a.lplv - 1;
    const size_t planes = (size_t)p.B * p.C, groups = (size_t)p.B * p.G;
    const size_t out_c = (size_t)d * planes * HW, out_w = (size_t)d * groups * 3 * HW;
    const size_t slot_c = p.shared ? 0 : out_c, slot_w = p.shared ? 0 : out_w;
    const int row_bytes = W * (int)sizeof(T);
    const size_t plane_bytes = (size_t)HW * sizeof(T);
    const size_t img0 = ((size_t)b * p.C + c_first) * HW;          // first channel of the workgroup
    const int g_first = c_first / p.cpg;
    const uint32_t voff = (uint32_t)((plc * HW + ic * V) * (int)sizeof(T));
    const uint32_t voff_w = (uint32_t)(((a.shared_group ? 0 : plc) * 3 * HW + ic * V) * (int)sizeof(T));
    const rsrc_t gyb = make_rsrc((const char*)p.gy + img0 * sizeof(T));
    const rsrc_t xb = make_rsrc((const char*)p.x + img0 * sizeof(T));
    const rsrc_t lb = make_rsrc((const char*)p.lam + (slot_c + img0) * sizeof(T));
    const rsrc_t ub = make_rsrc((const char*)p.u + (slot_c + img0) * sizeof(T));
    const rsrc_t hb = make_rsrc((const char*)p.hs + (out_c + img0) * sizeof(T));
    const rsrc_t glb = make_rsrc((char*)p.glam + (out_c + img0) * sizeof(T));
    const rsrc_t gub = make_rsrc((char*)p.gu + (out_c + img0) * sizeof(T));
    const size_t wgrp = ((size_t)b * p.G + g_first) * 3 * HW;
    const char* wbase = (const char*)p.w + (slot_w + wgrp) * sizeof(T);
    char* gwbase = (char*)p.gw + (out_w + wgrp) * sizeof(T);
    const rsrc_t w0b = make_rsrc(wbase), w1b = make_rsrc(wbase + plane_bytes), w2b = make_rsrc(wbase + 2 * plane_bytes);
    const rsrc_t g0b = make_rsrc(gwbase), g1b = make_rsrc(gwbase + plane_bytes), g2b = make_rsrc(gwbase + 2 * plane_bytes);

    if (!active) return;

    // sweep line n is scan step H-1-n: image row H-1-n (top->bottom scan) or n (bottom->top scan)
    const int sstep = REV ? row_bytes : -row_bytes;
    const int so0 = REV ? 0 : (H - 1) * row_bytes;
    const int tstep = REV ? a.pitch : -a.pitch;
    const int round_bytes = HW * (int)sizeof(T) * a.pv;             // next round = pv channels further
    const int wround_bytes = a.shared_group ? 0 : 3 * round_bytes;  // per-channel groups: weights move with the round
    const int tile_round = a.pv * H * a.pitch;
    float* tp0 = tile + pk0 * tile_round + (plc * H + (REV ? 0 : H - 1)) * a.pitch + ic * V;
    float* es = est + lane * V;                                     // carried state of round r: es[r * 128 + v]
    const bool atomic = a.gsplit > 1;

    struct Item { uint32_t gy[NR], x[NR], l[NR], u[NR], h[NR], hm[NR], w0[NR], w1[NR], w2[NR]; };
    const int nitems = H * rounds;
    int in = 0, ir = 0;                       // (line, round) of the next item to request
    auto issue = [&](Item& s) {
        const int so = so0 + in * sstep + (pk0 + ir) * round_bytes;
        const int som = so0 + (in + 1 < H ? in + 1 : in) * sstep + (pk0 + ir) * round_bytes;   // h of the next sweep line
        const int sow = so0 + in * sstep + (pk0 + ir) * wround_bytes;
        ld_buf<NB>(gyb, voff, so, s.gy);
        ld_buf<NB>(xb, voff, so, s.x);
        ld_buf<NB>(lb, voff, so, s.l);
        ld_buf<NB>(ub, voff, so, s.u);
        ld_buf<NB>(hb, voff, so, s.h);
        ld_buf<NB>(hb, voff, som, s.hm);
        ld_buf<NB>(w0b, voff_w, sow, s.w0);
        ld_buf<NB>(w1b, voff_w, sow, s.w1);
        ld_buf<NB>(w2b, voff_w, sow, s.w2);
        // advance; past the end the last item is requested again (redundant, in bounds)
        if (in * rounds + ir + 1 < nitems) { if (++ir == rounds) { ir = 0; ++in; } }
    };

    Item slot[PF];
#pragma unroll
    for (int k = 0; k < PF; ++k) issue(slot[k]);
    for (int r = 0; r < rounds; ++r) { es[r * 128] = 0.f; es[r * 128 + 1] = 0.f; }

    float wp0[V] = {0.f, 0.f}, wp1[V] = {0.f, 0.f}, wp2[V] = {0.f, 0.f};   // weights of the previous sweep line
    float wn0[V], wn1[V], wn2[V];                                           // weights of this line (for the next)
    float gw0[V] = {0.f, 0.f}, gw1[V] = {0.f, 0.f}, gw2[V] = {0.f, 0.f};
    int n = 0, r = 0;
    int until_split = split;
    // launches after the first over a group: sums of the line whose stored gw is on its way, and where they go
    float pend0[V] = {0.f, 0.f}, pend1[V] = {0.f, 0.f}, pend2[V] = {0.f, 0.f};
    uint32_t old0[NR], old1[NR], old2[NR];
    int pend_so = -1;
    auto flush_pending = [&]() {
        uint32_t o[NR];
#pragma unroll
        for (int v = 0; v < V; ++v) { pend0[v] += elem<T>(old0, v); pend1[v] += elem<T>(old1, v); pend2[v] += elem<T>(old2, v); }
        pack<T, V>(pend0, o); st_buf<NB>(g0b, voff_w, pend_so, o);
        pack<T, V>(pend1, o); st_buf<NB>(g1b, voff_w, pend_so, o);
        pack<T, V>(pend2, o); st_buf<NB>(g2b, voff_w, pend_so, o);
    };
    StretchWalkBack walk;
    if constexpr (LOCAL) walk.init(H, REV, p.kchunk);
    bool no_prev = false;                     // this scan step has no line before it: its gw is 0, nothing flows into it
    for (int it0 = 0; it0 < nitems; it0 += PF) {
#pragma unroll
        for (int k = 0; k < PF; ++k) {
            if (it0 + k < nitems) {
                const Item& cur = slot[k];
                if (r == 0) {
                    if (until_split == 0) lds_barrier();
                    --until_split;
                    // scan step 0 (GSPN-local: the first line of a stretch)
                    if constexpr (LOCAL) no_prev = walk.start(n == H - 1);
                    else no_prev = n == H - 1;
                }
                const float en0 = es[r * 128], en1 = es[r * 128 + 1];
                const float q00 = wp0[0] * en0, q01 = wp0[1] * en1;
                const float q10 = wp1[0] * en0, q11 = wp1[1] * en1;
                const float q20 = wp2[0] * en0, q21 = wp2[1] * en1;
                float lin = from_lane_below(q21), rin = from_lane_above(q00);
                lin = first ? 0.f : lin;
                rin = last ? 0.f : rin;
                const float gy0 = elem<T>(cur.gy, 0), gy1 = elem<T>(cur.gy, 1);
                const float e0 = fmaf(elem<T>(cur.u, 0), gy0, lin + q10 + q01);
                const float e1 = fmaf(elem<T>(cur.u, 1), gy1, q20 + q11 + rin);
                es[r * 128] = e0; es[r * 128 + 1] = e1;
                const int so = so0 + n * sstep + (pk0 + r) * round_bytes;
                {
                    float gl[V] = {elem<T>(cur.x, 0) * e0, elem<T>(cur.x, 1) * e1};
                    float gu[V] = {gy0 * elem<T>(cur.h, 0), gy1 * elem<T>(cur.h, 1)};
                    uint32_t o[NR];
                    pack<T, V>(gl, o); st_buf<NB>(glb, voff, so, o);
                    pack<T, V>(gu, o); st_buf<NB>(gub, voff, so, o);
                }
                float* tpr = tp0 + n * tstep + r * tile_round;
                tpr[0] += elem<T>(cur.l, 0) * e0;       // exclusive owner of these tile elements in this half
                tpr[1] += elem<T>(cur.l, 1) * e1;
                // weight gradients of this line: e_t[j] * h_{t-1}[j-1, j, j+1]
                const float hm0 = no_prev ? 0.f : elem<T>(cur.hm, 0), hm1 = no_prev ? 0.f : elem<T>(cur.hm, 1);
                float hl = from_lane_below(hm1), hr = from_lane_above(hm0);
                hl = first ? 0.f : hl;
                hr = last ? 0.f : hr;
                gw0[0] = fmaf(e0, hl, gw0[0]);  gw0[1] = fmaf(e1, hm0, gw0[1]);
                gw1[0] = fmaf(e0, hm0, gw1[0]); gw1[1] = fmaf(e1, hm1, gw1[1]);
                gw2[0] = fmaf(e0, hm1, gw2[0]); gw2[1] = fmaf(e1, hr, gw2[1]);
#pragma unroll
                for (int v = 0; v < V; ++v) { wn0[v] = elem<T>(cur.w0, v); wn1[v] = elem<T>(cur.w1, v); wn2[v] = elem<T>(cur.w2, v); }
                if constexpr (LOGITS) {
#pragma unroll
                    for (int v = 0; v < V; ++v) softmax3(wn0[v], wn1[v], wn2[v], first && v == 0, last && v == V - 1);
                }
                if constexpr (LOCAL) {
#pragma unroll
                    for (int v = 0; v < V; ++v) { wn0[v] = no_prev ? 0.f : wn0[v]; wn1[v] = no_prev ? 0.f : wn1[v]; wn2[v] = no_prev ? 0.f : wn2[v]; }
                }
                issue(slot[k]);
                if (++r == rounds) {
                    // end of the line: gw leaves the wave, this line's weights become the previous line's
                    const int sow = so0 + n * sstep + pk0 * wround_bytes;
                    if constexpr (LOGITS) {
                        // gradient w.r.t. the logits: linear in gw, applied to the partial sums of this lane
#pragma unroll
                        for (int v = 0; v < V; ++v) softmax3_grad(gw0[v], gw1[v], gw2[v], wn0[v], wn1[v], wn2[v]);
                    }
                    if (a.shared_group) {
#pragma unroll
                        for (int v = 0; v < V; ++v) {
                            gw0[v] = slot_sum(gw0[v], a.pv, a.lplv, lane, pl);
                            gw1[v] = slot_sum(gw1[v], a.pv, a.lplv, lane, pl);
                            gw2[v] = slot_sum(gw2[v], a.pv, a.lplv, lane, pl);
                        }
                    }
                    if (!a.shared_group || pl == 0) {
                        if (sizeof(T) == 4 && atomic) {
#pragma unroll
                            for (int v = 0; v < V; ++v) {
                                gw_out(g0b, gwbase, voff_w + 4 * v, sow, gw0[v], true);
                                gw_out(g1b, gwbase + plane_bytes, voff_w + 4 * v, sow, gw1[v], true);
                                gw_out(g2b, gwbase + 2 * plane_bytes, voff_w + 4 * v, sow, gw2[v], true);
                            }
                        } else if (a.seq_index > 0) {
                            // a later launch over the same group adds onto the stored gw: the stored values of this line
                            // are requested here and added a line later, when they have arrived behind that line's work
                            if (pend_so >= 0) flush_pending();
#pragma unroll
                            for (int v = 0; v < V; ++v) { pend0[v] = gw0[v]; pend1[v] = gw1[v]; pend2[v] = gw2[v]; }
                            ld_buf<NB>(g0b, voff_w, sow, old0);
                            ld_buf<NB>(g1b, voff_w, sow, old1);
                            ld_buf<NB>(g2b, voff_w, sow, old2);
                            pend_so = sow;
                        } else {
                            gw_store<T, V>(g0b, voff_w, sow, gw0, false);
                            gw_store<T, V>(g1b, voff_w, sow, gw1, false);
                            gw_store<T, V>(g2b, voff_w, sow, gw2, false);
                        }
                    }
#pragma unroll
                    for (int v = 0; v < V; ++v) {
                        gw0[v] = 0.f; gw1[v] = 0.f; gw2[v] = 0.f;
                        wp0[v] = wn0[v]; wp1[v] = wn1[v]; wp2[v] = wn2[v];
                    }
                    r = 0; ++n;
                }
            }
        }
    }
    if (pend_so >= 0 && (!a.shared_group || pl == 0)) flush_pending();
}

// ---------------------------------------------------------------------------
// horizontal directions: lines are image columns, one image row per lane, the sweep is read in
// chunks of CS columns (16 B per row and tensor: 4 of fp32, 8 of bf16; 4 of bf16 for odd widths; 56 B / 112 B --
// 28 columns of bf16 / fp32 -- for rows that are multiples of 112 B in workgroups of at most four waves)
// ---------------------------------------------------------------------------
// DB = false: one item buffer (for bursts too large to hold twice); the next item is requested when the current one
// has been consumed
template <typename T, bool REV, int CS, bool LOCAL, bool LOGITS, bool DB = true>
struct BwdHorizontal {
    static constexpr int NB = CS * (int)sizeof(T);
    static constexpr int NR = NB / 4;
    struct Item { uint32_t gy[NR], x[NR], l[NR], u[NR], h[NR], w0[NR], w1[NR], w2[NR], hm; };
    rsrc_t gyb, xb, lb, ub, hb, glb, gub, w0b, w1b, w2b, g0b, g1b, g2b;
    char* gwbase;
    size_t plane_bytes;
    uint32_t voff, voff_w;
    int W, nchunks, rounds, pk0, round_bytes, wround_bytes, tile_round, pitch, ph, H, lane, pl;
    float* trow;
    float* es;
    bool active, first, last, shared_group, atomic, gw_add;
    int in, ir;                    // (chunk, round) of the next item to request
    int m, r;                      // (chunk, round) of the next item to consume
    float wc0, wc1, wc2;           // weights at the previous sweep position (last element of the previous chunk)
    float gw0[CS], gw1[CS], gw2[CS];
    StretchWalkBack walk;          // GSPN-local only
    unsigned starts;               // GSPN-local: bit k set <=> the element of the current chunk visited k-th starts a stretch
    Item buf0, buf1;

    __device__ __forceinline__ void init(const BwdTileArgs& a, float* tile, float* est, int d, int b, int c_first,
                                         int pk0_, int rounds_, int lane_) {
        const BwdParams& p = a.p;
        H = p.H; W = p.W;
        const int HW = H * W;
        lane = lane_;
        pl = lane / H;
        const int i = lane - pl * H;
        active = pl < a.ph;
        const int plc = active ? pl : 0, ic = active ? i : 0;
        first = ic == 0; last = ic == H - 1;
        shared_group = a.shared_group != 0; atomic = a.gsplit > 1; gw_add = a.seq_index > 0;
        ph = a.ph; pk0 = pk0_; rounds = rounds_; pitch = a.pitch;
        const size_t planes = (size_t)p.B * p.C, groups = (size_t)p.B * p.G;
        const size_t out_c = (size_t)d * planes * HW, out_w = (size_t)d * groups * 3 * HW;
        const size_t slot_c = p.shared ? 0 : out_c, slot_w = p.shared ? 0 : out_w;
        plane_bytes = (size_t)HW * sizeof(T);
        const size_t img0 = ((size_t)b * p.C + c_first) * HW;
        const int g_first = c_first / p.cpg;
        voff = (uint32_t)((plc * HW + ic * W) * (int)sizeof(T));
        voff_w = (uint32_t)(((shared_group ? 0 : plc) * 3 * HW + ic * W) * (int)sizeof(T));
        gyb = make_rsrc((const char*)p.gy + img0 * sizeof(T));
        xb = make_rsrc((const char*)p.x + img0 * sizeof(T));
        lb = make_rsrc((const char*)p.lam + (slot_c + img0) * sizeof(T));
        ub = make_rsrc((const char*)p.u + (slot_c + img0) * sizeof(T));
        hb = make_rsrc((const char*)p.hs + (out_c + img0) * sizeof(T));
        glb = make_rsrc((char*)p.glam + (out_c + img0) * sizeof(T));
        gub = make_rsrc((char*)p.gu + (out_c + img0) * sizeof(T));
        const size_t wgrp = ((size_t)b * p.G + g_first) * 3 * HW;
        const char* wbase = (const char*)p.w + (slot_w + wgrp) * sizeof(T);
        gwbase = (char*)p.gw + (out_w + wgrp) * sizeof(T);
        w0b = make_rsrc(wbase); w1b = make_rsrc(wbase + plane_bytes); w2b = make_rsrc(wbase + 2 * plane_bytes);
        g0b = make_rsrc(gwbase); g1b = make_rsrc(gwbase + plane_bytes); g2b = make_rsrc(gwbase + 2 * plane_bytes);
        nchunks = W / CS;
        round_bytes = HW * (int)sizeof(T) * a.ph;
        wround_bytes = shared_group ? 0 : 3 * round_bytes;
        tile_round = a.ph * H * a.pitch;
        trow = tile + pk0 * tile_round + (plc * H + ic) * a.pitch;
        es = est + lane;
        in = 0; ir = 0; m = 0; r = 0;
        wc0 = 0.f; wc1 = 0.f; wc2 = 0.f;
#pragma unroll
        for (int e = 0; e < CS; ++e) { gw0[e] = 0.f; gw1[e] = 0.f; gw2[e] = 0.f; }
        starts = 0;
        if constexpr (LOCAL) walk.init(W, REV, p.kchunk);
    }

    // Sweep chunk c covers the columns the backward pass visits c-th: the scan left->right is swept
    // from the right (chunk 0 = the last CS columns, visited in descending order), right->left from the left.
    __device__ __forceinline__ int chunk_col(int c) const { return (REV ? c : nchunks - 1 - c) * CS; }

    __device__ __forceinline__ void issue(Item& s) {
        const int c0 = chunk_col(in);
        const int so = c0 * (int)sizeof(T) + (pk0 + ir) * round_bytes;
        const int sow = c0 * (int)sizeof(T) + (pk0 + ir) * wround_bytes;
        // column the sweep visits right after this chunk (h of scan step t-1 for the chunk's last element)
        int cn = REV ? c0 + CS : c0 - 1;
        cn = cn < 0 ? 0 : (cn > W - 1 ? W - 1 : cn);
        ld_buf<NB>(gyb, voff, so, s.gy);
        ld_buf<NB>(xb, voff, so, s.x);
        ld_buf<NB>(lb, voff, so, s.l);
        ld_buf<NB>(ub, voff, so, s.u);
        ld_buf<NB>(hb, voff, so, s.h);
        {
            const int soh = __builtin_amdgcn_readfirstlane(cn * (int)sizeof(T) + (pk0 + ir) * round_bytes);
            if constexpr (sizeof(T) == 4) s.hm = __builtin_amdgcn_raw_buffer_load_b32(hb, voff, soh, 0);
            else s.hm = (uint32_t)__builtin_amdgcn_raw_buffer_load_b16(hb, voff, soh, 0) << 16;   // widened: fp32 bits
        }
        ld_buf<NB>(w0b, voff_w, sow, s.w0);
        ld_buf<NB>(w1b, voff_w, sow, s.w1);
        ld_buf<NB>(w2b, voff_w, sow, s.w2);
        if (in * rounds + ir + 1 < nchunks * rounds) { if (++ir == rounds) { ir = 0; ++in; } }
    }

    __device__ __forceinline__ void compute(const Item& s) {
        const int c0 = chunk_col(m);
        const bool last_chunk = m == nchunks - 1;
        if constexpr (LOCAL) {
            if (r == 0) {                                         // once per chunk, the same for all its rounds
                starts = 0;
#pragma unroll
                for (int k = 0; k < CS; ++k) starts |= (walk.start(last_chunk && k == CS - 1) ? 1u : 0u) << k;
            }
        }
        float e = es[r * 64];
        float gl[CS], gu[CS];
        float w0p = wc0, w1p = wc1, w2p = wc2;
        float wk0[LOGITS ? CS : 1], wk1[LOGITS ? CS : 1], wk2[LOGITS ? CS : 1];   // LOGITS: this chunk's normalised weights
#pragma unroll
        for (int k = 0; k < CS; ++k) {
            const int ix = REV ? k : CS - 1 - k;                  // element of the chunk visited k-th
            const int ixn = REV ? k + 1 : CS - 2 - k;             // element visited next (h of scan step t-1)
            const float q0 = w0p * e, q1 = w1p * e, q2 = w2p * e;
            float lin = from_lane_below(q2), rin = from_lane_above(q0);
            lin = first ? 0.f : lin;
            rin = last ? 0.f : rin;
            const float gy = elem<T>(s.gy, ix);
            e = fmaf(elem<T>(s.u, ix), gy, lin + q1 + rin);
            gl[ix] = elem<T>(s.x, ix) * e;
            gu[ix] = gy * elem<T>(s.h, ix);
            trow[r * tile_round + c0 + ix] += elem<T>(s.l, ix) * e;
            float hm = (k == CS - 1) ? __uint_as_float(s.hm) : elem<T>(s.h, ixn);
            if (k == CS - 1) hm = last_chunk ? 0.f : hm;          // scan step 0 has no predecessor: gw = 0
            if constexpr (LOCAL) hm = ((starts >> k) & 1u) ? 0.f : hm;   // nor has the first line of a stretch
            float hl = from_lane_below(hm), hr = from_lane_above(hm);
            hl = first ? 0.f : hl;
            hr = last ? 0.f : hr;
            gw0[ix] = fmaf(e, hl, gw0[ix]);
            gw1[ix] = fmaf(e, hm, gw1[ix]);
            gw2[ix] = fmaf(e, hr, gw2[ix]);
            w0p = elem<T>(s.w0, ix); w1p = elem<T>(s.w1, ix); w2p = elem<T>(s.w2, ix);
            if constexpr (LOGITS) softmax3(w0p, w1p, w2p, first, last);
            if constexpr (LOCAL) {
                const bool z = (starts >> k) & 1u;                // nothing flows into the first line of a stretch
                w0p = z ? 0.f : w0p; w1p = z ? 0.f : w1p; w2p = z ? 0.f : w2p;
            }
            if constexpr (LOGITS) { wk0[ix] = w0p; wk1[ix] = w1p; wk2[ix] = w2p; }
        }
        es[r * 64] = e;
        {
            const int so = c0 * (int)sizeof(T) + (pk0 + r) * round_bytes;
            uint32_t o[NR];
            pack<T, CS>(gl, o); st_buf<NB>(glb, voff, so, o);
            pack<T, CS>(gu, o); st_buf<NB>(gub, voff, so, o);
        }
        if (++r == rounds) {
            const int sow = c0 * (int)sizeof(T) + pk0 * wround_bytes;
            if constexpr (LOGITS) {
                // gradient w.r.t. the logits: linear in gw, applied to the partial sums of this lane
#pragma unroll
                for (int ix = 0; ix < CS; ++ix) softmax3_grad(gw0[ix], gw1[ix], gw2[ix], wk0[ix], wk1[ix], wk2[ix]);
            }
            if (shared_group) {
#pragma unroll
                for (int ix = 0; ix < CS; ++ix) {
                    gw0[ix] = slot_sum(gw0[ix], ph, H, lane, pl);
                    gw1[ix] = slot_sum(gw1[ix], ph, H, lane, pl);
                    gw2[ix] = slot_sum(gw2[ix], ph, H, lane, pl);
                }
            }
            if (!shared_group || pl == 0) {
                if (atomic) {
#pragma unroll
                    for (int ix = 0; ix < CS; ++ix) {
                        atomicAdd((float*)(gwbase + sow + voff_w + 4 * ix), gw0[ix]);
                        atomicAdd((float*)(gwbase + plane_bytes + sow + voff_w + 4 * ix), gw1[ix]);
                        atomicAdd((float*)(gwbase + 2 * plane_bytes + sow + voff_w + 4 * ix), gw2[ix]);
                    }
                } else {
                    gw_store<T, CS>(g0b, voff_w, sow, gw0, gw_add);
                    gw_store<T, CS>(g1b, voff_w, sow, gw1, gw_add);
                    gw_store<T, CS>(g2b, voff_w, sow, gw2, gw_add);
                }
            }
#pragma unroll
            for (int ix = 0; ix < CS; ++ix) { gw0[ix] = 0.f; gw1[ix] = 0.f; gw2[ix] = 0.f; }
            wc0 = w0p; wc1 = w1p; wc2 = w2p;     // weights at the last position visited in this chunk
            r = 0; ++m;
        }
    }

    __device__ __forceinline__ void prologue() {
        if (!active) return;
        for (int q = 0; q < rounds; ++q) es[q * 64] = 0.f;
        issue(buf0);
    }

    // items [begin, end) of the flattened (chunk, round) sequence; buffer (item & 1) holds item `begin`
    __device__ __forceinline__ void run(int begin, int end) {
        if (!active) return;
        if constexpr (!DB) {
            for (int it = begin; it < end; ++it) { compute(buf0); issue(buf0); }   // (past the end: the last item again)
            return;
        }
        for (int it = begin; it < end; ++it) {
            if ((it & 1) == 0) { issue(buf1); compute(buf0); }
            else               { issue(buf0); compute(buf1); }
        }
    }
};

template <typename T, int PF, int MAXW, int HCS, bool LOCAL, bool LOGITS>
__global__ void __launch_bounds__(64 * MAXW) bwd_tile_kernel(BwdTileArgs a) {
    static_assert(LOCAL || !LOGITS, "logits run on the local instantiations (a global scan is one stretch)");
    extern __shared__ float lds[];
    const BwdParams& p = a.p;
    const int H = p.H, W = p.W, HW = H * W;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // one workgroup per K channels; when a group is covered by several launches, this one takes slice seq_index
    const int blocks_per_image = p.C / (a.K * a.seq_parts);
    const int b = blockIdx.x / blocks_per_image;
    const int c_first = ((blockIdx.x - b * blocks_per_image) * a.seq_parts + a.seq_index) * a.K;
    float* tile = lds;
    const int tile_floats = a.K * H * a.pitch;
    float* est = lds + tile_floats + wave * a.est_floats;

    for (int i = threadIdx.x; i < tile_floats; i += blockDim.x) tile[i] = 0.f;
    lds_barrier();

    // one wave per (direction, set of rounds): with a shared weight group a wave takes all packs of
    // its direction (so that gw is summed inside the wave), otherwise one pack per wave
    const int packs_v = a.K / a.pv, packs_h = a.K / a.ph;
    {
        const int nd = ((p.mask >> 0) & 1) + ((p.mask >> 1) & 1);
        const int tasks = a.shared_group ? nd : packs_v * nd;
        if (nd > 0 && wave < tasks) {
            const int slot = a.shared_group ? 0 : wave / nd;
            const int dsel = a.shared_group ? wave : wave - slot * nd;
            const int d = (nd == 2) ? dsel : ((p.mask & 1) ? 0 : 1);
            const int rounds = a.shared_group ? packs_v : 1;
            // the wave sweeping the top->bottom scan starts at the bottom rows, the other at the top rows
            const int split = nd == 2 ? (d == 0 ? (H + 1) / 2 : H - (H + 1) / 2) : -1;
            if (d == 0) bwd_vertical<T, PF, false, LOCAL, LOGITS>(a, tile, est, b, c_first, slot, rounds, lane, split);
            else bwd_vertical<T, PF, true, LOCAL, LOGITS>(a, tile, est, b, c_first, slot, rounds, lane, split);
        } else if (nd == 2) {
            lds_barrier();
        }
    }
    {
        const int has_lr = (p.mask >> 2) & 1, has_rl = (p.mask >> 3) & 1;
        const int nd = has_lr + has_rl;
        const int tasks = a.shared_group ? nd : packs_h * nd;
        const bool busy = nd > 0 && wave < tasks;
        const int slot = (busy && !a.shared_group) ? wave / nd : 0;
        const int dsel = a.shared_group ? wave : wave - slot * nd;
        const int d = (nd == 2) ? 2 + dsel : (has_lr ? 2 : 3);
        const int rounds = a.shared_group ? packs_h : 1;
        const int nchunks = W / HCS;
        const int half_lr = (nchunks + 1) / 2, half_rl = nchunks - half_lr;
        if (nd == 0) {
            lds_barrier();
        } else if (d == 2) {
            BwdHorizontal<T, false, HCS, LOCAL, LOGITS, (HCS * sizeof(T) < 56)> hp;
            if (busy) { hp.init(a, tile, est, 2, b, c_first, slot, rounds, lane); hp.prologue(); }
            lds_barrier();
            if (busy) hp.run(0, (nd == 2 ? half_lr : nchunks) * rounds);
            if (nd == 2) {
                lds_barrier();
                if (busy) hp.run(half_lr * rounds, nchunks * rounds);
            }
        } else {
            BwdHorizontal<T, true, HCS, LOCAL, LOGITS, (HCS * sizeof(T) < 56)> hp;
            if (busy) { hp.init(a, tile, est, 3, b, c_first, slot, rounds, lane); hp.prologue(); }
            lds_barrier();
            if (busy) hp.run(0, (nd == 2 ? half_rl : nchunks) * rounds);
            if (nd == 2) {
                lds_barrier();
                if (busy) hp.run(half_rl * rounds, nchunks * rounds);
            }
        }
    }
    lds_barrier();

    // merged gx: written once, coalesced
    {
        T* GX = (T*)p.gx + ((size_t)b * p.C + c_first) * HW;
        const int rows = a.K * H;
        const int nw = blockDim.x >> 6;
        for (int rr = wave; rr < rows; rr += nw) {
            const float* tr = tile + rr * a.pitch;
            T* yr = GX + (size_t)rr * W;
            for (int j = lane * 2; j < W; j += 128) {
                float v[2] = {tr[j], tr[j + 1]};
                uint32_t o[2 * sizeof(T) / 4];
                pack<T, 2>(v, o);
                st_raw<2 * sizeof(T)>((char*)(yr + j), o);
            }
        }
    }
}

// zero fill (used instead of a memset node so that the call can be captured in a HIP graph)
__global__ void __launch_bounds__(256) zero_fill_kernel(uint32_t* p, size_t n16) {
    u32x4* q = (u32x4*)p;
    const u32x4 z = {0, 0, 0, 0};
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x) q[i] = z;
}

hipError_t launch_zero_fill(void* p, size_t bytes, hipStream_t s) {
    const size_t n16 = bytes / 16;
    const unsigned blocks = (unsigned)((n16 + 255) / 256 < 2048 ? (n16 + 255) / 256 : 2048);
    if (blocks == 0) return hipSuccess;
    hipLaunchKernelGGL(zero_fill_kernel, dim3(blocks), dim3(256), 0, s, (uint32_t*)p, n16);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
static constexpr int BWD_LDS_BUDGET = 160 * 1024;

struct BwdPlan { bool ok; int K, pitch, lplv, pv, ph, shared_group, gsplit, seq_parts, nwaves, est_floats; size_t lds; };

static BwdPlan plan_bwd(const BwdParams& p, int dtype) {
    BwdPlan t = {};
    if (p.W % 4 || p.W / 2 > 64 || p.H > 64 || p.H < 2) return t;
    t.pitch = p.W | 1;
    t.lplv = p.W / 2; t.pv = 64 / t.lplv;
    t.ph = 64 / p.H;
    const int lcm = (t.pv % t.ph == 0) ? t.pv : ((t.ph % t.pv == 0) ? t.ph : t.pv * t.ph);
    const size_t per_channel = (size_t)p.H * t.pitch * sizeof(float);
    const int dirs_v = ((p.mask >> 0) & 1) + ((p.mask >> 1) & 1), dirs_h = ((p.mask >> 2) & 1) + ((p.mask >> 3) & 1);
    const size_t hw4 = (size_t)p.H * p.W * 4;
    if (p.cpg == 1) {
        // one weight group per channel: the smallest workgroup that fills the lanes in both phases
        t.shared_group = 0; t.gsplit = 1; t.seq_parts = 1;
        const int K = lcm;
        if (p.C % K) return t;
        const int wv = (K / t.pv) * dirs_v, wh = (K / t.ph) * dirs_h;
        t.nwaves = wv > wh ? wv : wh;
        if (t.nwaves < 1) t.nwaves = 1;
        if (t.nwaves > 8) return t;
        t.K = K;
        t.est_floats = 128;
    } else {
        // shared weights: the whole group (or half of it) in one workgroup, one wave per direction
        t.shared_group = 1;
        int K = p.cpg, gs = 1;
        const size_t wgs = (size_t)p.B * p.G;
        // a group too large for LDS is covered by two launches, the second adding onto the stored gw (in the horizontal
        // phases a lane's gw elements are a row pitch apart: atomics there were measured at four times the cost of this
        // read-add-write, 1210 against 300 us for the horizontal pair of 56x56x96 fp32); a group that fits, fp32
        // storage, too few groups to fill the chip: split over two workgroups that add into gw atomically
        int seq = 1;
        if (K * per_channel > (size_t)BWD_LDS_BUDGET - 16384) {
            if (K % (2 * lcm) == 0) { K /= 2; seq = 2; }
        } else if (dtype == 0 && wgs < 384 && K % (2 * lcm) == 0) { K /= 2; gs = 2; }
        if (K % lcm || K * per_channel > (size_t)BWD_LDS_BUDGET - 16384) return t;
        t.K = K; t.gsplit = gs; t.seq_parts = seq;
        t.nwaves = dirs_v > dirs_h ? dirs_v : dirs_h;
        if (t.nwaves < 1) t.nwaves = 1;
        const int rv = K / t.pv, rh = K / t.ph;
        t.est_floats = (rv * 128 > rh * 64) ? rv * 128 : rh * 64;
    }
    t.lds = t.K * per_channel + (size_t)t.nwaves * t.est_floats * sizeof(float);
    if (t.lds > (size_t)BWD_LDS_BUDGET) return t;
    if ((size_t)t.K * hw4 >= (1ull << 31) || (size_t)t.K * 3 * hw4 >= (1ull << 31)) return t;
    if ((size_t)p.B * (p.C / t.K) > 0x7fffffffull) return t;
    t.ok = true;
    return t;
}

bool bwd_tile_applicable(const BwdParams& p, int dtype) { return plan_bwd(p, dtype).ok; }

hipError_t launch_bwd_tile(const BwdParams& p, int dtype, hipStream_t s) {
    const BwdPlan t = plan_bwd(p, dtype);
    if (!t.ok) return hipErrorInvalidValue;
    BwdTileArgs a;
    a.p = p; a.K = t.K; a.pitch = t.pitch; a.lplv = t.lplv; a.pv = t.pv; a.ph = t.ph;
    a.shared_group = t.shared_group; a.gsplit = t.gsplit; a.nwaves = t.nwaves; a.est_floats = t.est_floats;
    a.seq_parts = t.seq_parts; a.seq_index = 0;
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
    const dim3 grid((unsigned)((size_t)p.B * (p.C / (t.K * t.seq_parts)))), block(64 * t.nwaves);
    // horizontal phases read 8 columns per row and request when the width allows (bf16: 16 B; fp32: 32 B, which
    // needs more registers than 8 waves per workgroup leave, so only workgroups of up to 4 waves take it)
    const bool wide = p.W % 8 == 0;
    // rows that are multiples of 112 B (56 columns of bf16; 28, 56 of fp32) or of 64 / 128 B (32 columns), workgroups
    // of up to 4 waves: 56 / 64 B (bf16) or 112 / 128 B (fp32) per row and request -- the whole register file of a SIMD
    // goes to the one wave it runs
    const bool big = t.nwaves <= 4 && !p.logits;
    const bool burst28 = big && (p.W * (dtype == 0 ? 4 : 2)) % 112 == 0, burst32 = big && !burst28 && p.W % 32 == 0;
    void (*k)(BwdTileArgs);
    if (burst28) {
        if (p.kchunk > 0) k = dtype == 0 ? bwd_tile_kernel<float, 8, 4, 28, true, false> : bwd_tile_kernel<bf16_t, 8, 4, 28, true, false>;
        else k = dtype == 0 ? bwd_tile_kernel<float, 8, 4, 28, false, false> : bwd_tile_kernel<bf16_t, 8, 4, 28, false, false>;
    } else if (burst32) {
        if (p.kchunk > 0) k = dtype == 0 ? bwd_tile_kernel<float, 8, 4, 32, true, false> : bwd_tile_kernel<bf16_t, 8, 4, 32, true, false>;
        else k = dtype == 0 ? bwd_tile_kernel<float, 8, 4, 32, false, false> : bwd_tile_kernel<bf16_t, 8, 4, 32, false, false>;
    } else if (p.logits) {
        if (dtype == 0) k = (wide && t.nwaves <= 4) ? bwd_tile_kernel<float, 4, 4, 8, true, true> : bwd_tile_kernel<float, 4, 8, 4, true, true>;
        else k = wide ? bwd_tile_kernel<bf16_t, 4, 8, 8, true, true> : bwd_tile_kernel<bf16_t, 4, 8, 4, true, true>;
    } else if (p.kchunk > 0) {
        if (dtype == 0) k = (wide && t.nwaves <= 4) ? bwd_tile_kernel<float, 4, 4, 8, true, false> : bwd_tile_kernel<float, 4, 8, 4, true, false>;
        else k = wide ? bwd_tile_kernel<bf16_t, 4, 8, 8, true, false> : bwd_tile_kernel<bf16_t, 4, 8, 4, true, false>;
    } else {
        if (dtype == 0) k = (wide && t.nwaves <= 4) ? bwd_tile_kernel<float, 4, 4, 8, false, false> : bwd_tile_kernel<float, 4, 8, 4, false, false>;
        else k = wide ? bwd_tile_kernel<bf16_t, 4, 8, 8, false, false> : bwd_tile_kernel<bf16_t, 4, 8, 4, false, false>;
    }
    hipError_t e = allow_dynamic_lds((const void*)k, BWD_LDS_BUDGET);
    if (e != hipSuccess) return e;
    for (int part = 0; part < t.seq_parts; ++part) {          // same stream: the launches run one after the other
        a.seq_index = part;
        hipLaunchKernelGGL(k, grid, block, t.lds, s, a);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace gspn
