// Forward GSPN scan for feature maps whose fp32 output tile fits in LDS (gfx950: 160 KB per CU).
//
// One workgroup owns K consecutive channels of one batch image and runs all requested
// directions over them inside one launch (Sec. 4.1 "single kernel": the loop over lines
// is inside the kernel; here the loop over the four directions of Sec. 3.2 is too).
//
//  * A wave owns whole lines: each lane keeps V adjacent positions of the current line's
//    hidden state in registers (several channels side by side when a line is shorter than
//    the wave), so the three-neighbour read of Eq. 1 is two cross-lane DPP shifts per line
//    plus in-lane register moves.  No LDS, no barrier on the recurrence itself.
//  * Vertical directions: a line is an image row, the lane's V positions are contiguous in
//    memory, one vector load per tensor per line, PF lines prefetched ahead in registers.
//  * Horizontal directions: a line is an image column; the lane's V positions are V image
//    rows, and each lane reads its rows in bursts of CS scan steps (16..32 B), double
//    buffered in registers.
//  * The merged output y = sum_d u_d*h_d (Eq. 2 + sum merge) is accumulated in an fp32 LDS
//    tile by plain read-modify-write (every element has one owner wave between two barriers)
//    and written once, coalesced, rounded once to the storage type.  x is read once per
//    direction and the weight planes of a group once per channel (the two-channel kernel for
//    128x128 bf16 maps shares both within a workgroup).
//  * Accumulation order per output element is fixed (vertical pair first -- its two
//    contributions commute --, then the horizontal pair split at mid-scan by a barrier so
//    that the two waves never touch the same element in the same half), so results are
//    bitwise reproducible.
#pragma once
#include "gspn_tile_common.hpp"
#include <stdlib.h>

namespace gspn {

struct TileArgs {
    FwdParams p;
    int K;        // channels per workgroup (divides C)
    int pitch;    // LDS tile row pitch in floats (odd)
    int lplv, pv; // vertical phases: lanes per line, channels side by side in a wave
    int lplh, ph; // horizontal phases
    int nwaves;
    int parts;    // row-split horizontal phases: waves per line (each owns H/parts image rows)
};

// ---------------------------------------------------------------------------
// vertical direction (d = 0 top->bottom, 1 bottom->top): lines are image rows
// ---------------------------------------------------------------------------
// LOGITS (with LOCAL): w holds raw logits, normalised as they are consumed (softmax3)
// HT: the same pass for a horizontal direction (2 left->right, 3 right->left) whose w, lam, u (and h_save) slots
// and x are stored transposed, [..][W][H]: lines are image columns, contiguous in memory, and the pass differs
// from the vertical one only in the roles of H and W and in how it walks the (row-major) output tile
// BWD: the reverse sweep of the backward pass over the same machinery (see line_update_transposed): the caller passes gy
// as x, u as lam, lam as u, gx as y and the buffer that receives e as h_save; the wave that walks the rows downwards
// (REV = false) then works on the parameters of the bottom->top scan and the other way round, and the taps it applies
// are those of the line it swept before.
template <typename T, int V, int PF, bool REV, bool SAVE, bool LOCAL, bool LOGITS, bool HT = false, bool BWD = false>
__device__ __forceinline__ void vertical_pass(const TileArgs& a, float* tile, int b, int c_first, int pk,
                                              int lane, int split) {
    static_assert(!BWD || (SAVE && !HT), "the reverse sweep saves e and takes the standard layout");
    constexpr int NB = V * (int)sizeof(T);
    constexpr int NR = NB / 4;
    constexpr int d = HT ? (REV ? 3 : 2) : ((REV != BWD) ? 1 : 0);
    const FwdParams& p = a.p;
    const int H = p.H, W = p.W, HW = H * W;
    const int S = HT ? W : H, LL = HT ? H : W;                 // scan steps, positions per line
    const int lpl = HT ? a.lplh : a.lplv, pp = HT ? a.ph : a.pv;
    const int pl = lane / lpl, i = lane - pl * lpl;
    const int c_pack = c_first + pk * pp;                      // first channel of this wave's pack
    const int n_here = min(pp, a.K - pk * pp);
    const bool active = pl < n_here;
    const int plc = active ? pl : 0, ic = active ? i : 0;
    const int c = c_pack + plc;
    const int g = c / p.cpg, g0 = c_pack / p.cpg;
    const bool first = ic == 0, last = ic == lpl - 1;
    const size_t planes = (size_t)p.B * p.C;
    const size_t slot_c = p.shared ? 0 : (size_t)d * planes * HW;
    const size_t slot_w = p.shared ? 0 : (size_t)d * p.B * p.G * 3 * HW;
    const size_t plane0 = ((size_t)b * p.C + c_pack) * HW;      // uniform
    const uint32_t voff = (uint32_t)((plc * HW + ic * V) * (int)sizeof(T));
    const uint32_t voff_w = (uint32_t)(((g - g0) * 3 * HW + ic * V) * (int)sizeof(T));
    const int row_bytes = LL * (int)sizeof(T);
    const size_t plane_bytes = (size_t)HW * sizeof(T);
    const char* wbase = (const char*)p.w + (slot_w + ((size_t)b * p.G + g0) * 3 * HW) * sizeof(T);
    const rsrc_t xb = make_rsrc((const char*)(HT ? p.xt : p.x) + plane0 * sizeof(T));
    const rsrc_t lb = make_rsrc((const char*)p.lam + (slot_c + plane0) * sizeof(T));
    const rsrc_t ub = make_rsrc((const char*)p.u + (slot_c + plane0) * sizeof(T));
    const rsrc_t w0b = make_rsrc(wbase), w1b = make_rsrc(wbase + plane_bytes), w2b = make_rsrc(wbase + 2 * plane_bytes);
    const rsrc_t hb = make_rsrc(SAVE ? (char*)p.hs + ((size_t)d * planes * HW + plane0) * sizeof(T) : (char*)p.y);

    if (!active) return;   // the whole pass runs with unused lanes masked off (their DPP reads see 0)

    // scan step t works on image row t (top->bottom) or H-1-t (bottom->top); everything below walks
    // byte / float offsets by a constant signed stride per step, so a step costs no address arithmetic
    // beyond one scalar add (global) and one vector add (LDS)
    const int sstep = REV ? -row_bytes : row_bytes;
    const int so0 = REV ? (S - 1) * row_bytes : 0;
    // tile element of (scan step s, position j of the line): row s, column j -- transposed passes: row j, column s
    const int tstep = HT ? (REV ? -1 : 1) : (REV ? -a.pitch : a.pitch);
    const int tvs = HT ? a.pitch : 1;                          // from one of the lane's positions to the next
    float* tp = HT ? tile + ((pk * pp + plc) * H + ic * V) * a.pitch + (REV ? W - 1 : 0)
                   : tile + ((pk * pp + plc) * H + (REV ? H - 1 : 0)) * a.pitch + ic * V;   // scan step 0

    struct Line { uint32_t x[NR], l[NR], u[NR], w0[NR], w1[NR], w2[NR]; };
    Line slot[PF];
    auto issue = [&](Line& s, int so) {
        ld_buf<NB>(xb, voff, so, s.x);
        ld_buf<NB>(lb, voff, so, s.l);
        ld_buf<NB>(ub, voff, so, s.u);
        ld_buf<NB>(w0b, voff_w, so, s.w0);
        ld_buf<NB>(w1b, voff_w, so, s.w1);
        ld_buf<NB>(w2b, voff_w, so, s.w2);
    };
    // the ring starts with scan steps 0..PF-1 (clamped to the last step of short scans: redundant but in
    // bounds); issued unconditionally so that every path into the loops has the same loads in flight
#pragma unroll
    for (int k = 0; k < PF; ++k) issue(slot[k], so0 + min(k, S - 1) * sstep);

    float h[V];
#pragma unroll
    for (int v = 0; v < V; ++v) h[v] = 0.f;
    int so_cur = so0;            // byte offset of the row of the current step (for h_save)
    int until_split = split;     // steps left before the mid-scan barrier (negative: none)

    // `scan_start`: this is scan step 0, whose weights are never used (the stored values may be
    // anything): they are replaced by 0 so the (zero) initial state contributes exactly 0.  GSPN-local
    // (Sec. 3.2): the same at the first line of every stretch, where the carried state counts as 0 too.
    StretchWalk walk;
    if constexpr (LOCAL) walk.init(S, REV, p.kchunk);
    float wp0[V], wp1[V], wp2[V];            // BWD: taps of the line swept before (none before the first: 0)
#pragma unroll
    for (int v = 0; v < V; ++v) { wp0[v] = 0.f; wp1[v] = 0.f; wp2[v] = 0.f; }
    StretchWalkBack bwalk;                   // BWD, GSPN-local: the scan steps from the last one down
    if constexpr (BWD && LOCAL) bwalk.init(S, d & 1, p.kchunk);
    int sweep_t = 0;
    auto step = [&](const Line& cur, bool maybe_start, bool scan_start) {
        if (until_split == 0) lds_barrier();
        --until_split;
        if constexpr (BWD) {
            // GSPN-local: a line that starts a stretch takes nothing from the line before it in scan order, so its
            // taps hand nothing on to the line swept next
            bool starts = false;
            if constexpr (LOCAL) starts = bwalk.start(sweep_t == S - 1);
            ++sweep_t;
            float av[V], uv[V];
#pragma unroll
            for (int v = 0; v < V; ++v) { av[v] = elem<T>(cur.l, v) * elem<T>(cur.x, v); uv[v] = elem<T>(cur.u, v); }
            line_update_transposed<V>(h, av, wp0, wp1, wp2, first, last);
#pragma unroll
            for (int v = 0; v < V; ++v) {
                float c0 = elem<T>(cur.w0, v), c1 = elem<T>(cur.w1, v), c2 = elem<T>(cur.w2, v);
                if constexpr (LOGITS) softmax3(c0, c1, c2, first && v == 0, last && v == V - 1);
                // a tap that points outside the line takes nothing, whatever the tensor holds there
                wp0[v] = ((first && v == 0) || starts) ? 0.f : c0;
                wp1[v] = starts ? 0.f : c1;
                wp2[v] = ((last && v == V - 1) || starts) ? 0.f : c2;
                tp[v * tvs] += uv[v] * h[v];
            }
            tp += tstep;
            uint32_t hr[NR];
            pack<T, V>(h, hr);
            st_buf<NB, CP_STREAM>(hb, voff, so_cur, hr);
            so_cur += sstep;
            return;
        }
        if constexpr (LOCAL) {
            maybe_start = true;
            scan_start = walk.start();
            if (scan_start) {
#pragma unroll
                for (int v = 0; v < V; ++v) h[v] = 0.f;
            }
        }
        float av[V], w0[V], w1[V], w2[V], uv[V];
#pragma unroll
        for (int v = 0; v < V; ++v) {
            av[v] = elem<T>(cur.l, v) * elem<T>(cur.x, v);
            w0[v] = elem<T>(cur.w0, v); w1[v] = elem<T>(cur.w1, v); w2[v] = elem<T>(cur.w2, v);
            uv[v] = elem<T>(cur.u, v);
            if constexpr (LOGITS) softmax3(w0[v], w1[v], w2[v], first && v == 0, last && v == V - 1);
            if (maybe_start) {
                w0[v] = scan_start ? 0.f : w0[v]; w1[v] = scan_start ? 0.f : w1[v]; w2[v] = scan_start ? 0.f : w2[v];
            }
        }
        line_update<V>(h, av, w0, w1, w2, first, last);
#pragma unroll
        for (int v = 0; v < V; ++v) tp[v * tvs] += uv[v] * h[v];   // exclusive owner of these elements in this half
        tp += tstep;
        if constexpr (SAVE) {
            uint32_t hr[NR];
            pack<T, V>(h, hr);
            st_buf<NB, CP_STREAM>(hb, voff, so_cur, hr);
            so_cur += sstep;
        }
    };

    // Hot loop: blocks of PF steps while the line PF steps ahead always exists.  Straight-line code:
    // slot k is consumed and at once refilled, so the register ring is static and the hardware
    // load counter can be waited on by count (never drained).
    int t0 = 0;
    int so_next = so0 + PF * sstep;      // byte offset of the next line to request
    for (; t0 + 2 * PF <= S; t0 += PF) {
#pragma unroll
        for (int k = 0; k < PF; ++k) {
            step(slot[k], k == 0, t0 == 0);
            issue(slot[k], so_next);
            so_next += sstep;
            __builtin_amdgcn_sched_barrier(0);   // keep the consume/refill interleaving as written
        }
    }
    // Last full block: refills are clamped to the last line (redundant, in bounds), then the tail.
    if (t0 + PF <= S) {
#pragma unroll
        for (int k = 0; k < PF; ++k) {
            step(slot[k], k == 0, t0 == 0);
            issue(slot[k], so0 + min(t0 + k + PF, S - 1) * sstep);
            __builtin_amdgcn_sched_barrier(0);
        }
        t0 += PF;
    }
#pragma unroll
    for (int k = 0; k < PF; ++k)
        if (t0 + k < S) step(slot[k], k == 0, t0 == 0);
}

// ---------------------------------------------------------------------------
// horizontal direction (d = 2 left->right, 3 right->left): lines are image columns;
// the lane's V positions are V consecutive image rows.  Scan steps [c_begin*CS, c_end*CS).
// ---------------------------------------------------------------------------
template <typename T, int V, int CS>
struct HBuf { uint32_t x[V][CS * sizeof(T) / 4], l[V][CS * sizeof(T) / 4], u[V][CS * sizeof(T) / 4],
              w0[V][CS * sizeof(T) / 4], w1[V][CS * sizeof(T) / 4], w2[V][CS * sizeof(T) / 4]; };

// DB = true: two chunk buffers, the next chunk is loaded while the current one is consumed.
// DB = false: one buffer (for chunks too large to hold twice); the next chunk is requested as soon
// as the current one is consumed and other waves of the CU cover the wait.
template <typename T, int V, int CS, bool REV, bool SAVE, bool DB, bool LOCAL, bool LOGITS, bool BWD = false>
struct HorizontalPass {
    static constexpr int NB = CS * (int)sizeof(T);
    static constexpr int NR = NB / 4;
    rsrc_t xb, lb, ub, wb, hb;
    uint32_t voff, voff_w;
    int row_bytes, plane_bytes, nchunks, W;
    float* trow;
    int pitch;
    bool active, first, last;
    float h[V];
    float wp0[V], wp1[V], wp2[V];   // BWD: taps of the column swept before
    StretchWalk walk;   // GSPN-local only
    StretchWalkBack bwalk;   // ... in the reverse sweep
    HBuf<T, V, CS> buf0, buf1;

    __device__ __forceinline__ void init(const TileArgs& a, float* tile, int d, int b, int c_first, int pk, int lane) {
        const FwdParams& p = a.p;
        const int H = p.H, HW = H * p.W;
        W = p.W;
        const int pl = lane / a.lplh, i = lane - pl * a.lplh;
        const int c_pack = c_first + pk * a.ph;
        const int n_here = min(a.ph, a.K - pk * a.ph);
        active = pl < n_here;
        const int plc = active ? pl : 0, ic = active ? i : 0;
        const int c = c_pack + plc;
        const int g = c / p.cpg, g0 = c_pack / p.cpg;
        first = ic == 0; last = ic == a.lplh - 1;
        const size_t planes = (size_t)p.B * p.C;
        const size_t slot_c = p.shared ? 0 : (size_t)d * planes * HW;
        const size_t slot_w = p.shared ? 0 : (size_t)d * p.B * p.G * 3 * HW;
        const size_t plane0 = ((size_t)b * p.C + c_pack) * HW;
        voff = (uint32_t)((plc * HW + ic * V * W) * (int)sizeof(T));
        voff_w = (uint32_t)(((g - g0) * 3 * HW + ic * V * W) * (int)sizeof(T));
        xb = make_rsrc((const char*)p.x + plane0 * sizeof(T));
        lb = make_rsrc((const char*)p.lam + (slot_c + plane0) * sizeof(T));
        ub = make_rsrc((const char*)p.u + (slot_c + plane0) * sizeof(T));
        wb = make_rsrc((const char*)p.w + (slot_w + ((size_t)b * p.G + g0) * 3 * HW) * sizeof(T));
        hb = make_rsrc(SAVE ? (char*)p.hs + ((size_t)d * planes * HW + plane0) * sizeof(T) : (char*)p.y);
        row_bytes = W * (int)sizeof(T);
        plane_bytes = HW * (int)sizeof(T);
        nchunks = W / CS;
        pitch = a.pitch;
        trow = tile + ((pk * a.ph + plc) * H + ic * V) * a.pitch;
#pragma unroll
        for (int v = 0; v < V; ++v) { h[v] = 0.f; wp0[v] = 0.f; wp1[v] = 0.f; wp2[v] = 0.f; }
        if constexpr (LOCAL && !BWD) walk.init(W, REV, p.kchunk);
        if constexpr (LOCAL && BWD) bwalk.init(W, d & 1, p.kchunk);
    }

    // byte offset of chunk c (in scan order) inside a row
    __device__ __forceinline__ int chunk_col(int c) const { return (REV ? nchunks - 1 - c : c) * CS; }

    __device__ __forceinline__ void issue(HBuf<T, V, CS>& s, int c) {
        const int co = chunk_col(c) * (int)sizeof(T);
#pragma unroll
        for (int v = 0; v < V; ++v) {
            const int o = co + v * row_bytes;
            ld_buf<NB>(xb, voff, o, s.x[v]);
            ld_buf<NB>(lb, voff, o, s.l[v]);
            ld_buf<NB>(ub, voff, o, s.u[v]);
            ld_buf<NB>(wb, voff_w, o, s.w0[v]);
            ld_buf<NB>(wb, voff_w, plane_bytes + o, s.w1[v]);
            ld_buf<NB>(wb, voff_w, 2 * plane_bytes + o, s.w2[v]);
        }
    }

    __device__ __forceinline__ void compute(const HBuf<T, V, CS>& s, int c) {
        const int col0 = chunk_col(c);
        float hs[V][CS];
#pragma unroll
        for (int k = 0; k < CS; ++k) {
            const int e = REV ? CS - 1 - k : k;       // element inside the chunk, compile-time
            float av[V], w0[V], w1[V], w2[V];
            if constexpr (BWD) {
                bool starts = false;                  // GSPN-local: this column starts a stretch in scan order
                if constexpr (LOCAL) starts = bwalk.start(c == nchunks - 1 && k == CS - 1);
#pragma unroll
                for (int v = 0; v < V; ++v) av[v] = elem<T>(s.l[v], e) * elem<T>(s.x[v], e);
                line_update_transposed<V>(h, av, wp0, wp1, wp2, first, last);
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    float c0 = elem<T>(s.w0[v], e), c1 = elem<T>(s.w1[v], e), c2 = elem<T>(s.w2[v], e);
                    if constexpr (LOGITS) softmax3(c0, c1, c2, first && v == 0, last && v == V - 1);
                    wp0[v] = ((first && v == 0) || starts) ? 0.f : c0;
                    wp1[v] = starts ? 0.f : c1;
                    wp2[v] = ((last && v == V - 1) || starts) ? 0.f : c2;
                    trow[v * pitch + col0 + e] += elem<T>(s.u[v], e) * h[v];
                    hs[v][e] = h[v];
                }
                continue;
            }
            // first line of the scan (GSPN-local: of a stretch): its weights are never read, the state before it is 0
            bool start = (c == 0) && (k == 0);
            if constexpr (LOCAL) start = walk.start();
#pragma unroll
            for (int v = 0; v < V; ++v) {
                av[v] = elem<T>(s.l[v], e) * elem<T>(s.x[v], e);
                w0[v] = elem<T>(s.w0[v], e); w1[v] = elem<T>(s.w1[v], e); w2[v] = elem<T>(s.w2[v], e);
                if constexpr (LOGITS) softmax3(w0[v], w1[v], w2[v], first && v == 0, last && v == V - 1);
                if (LOCAL || k == 0) { w0[v] = start ? 0.f : w0[v]; w1[v] = start ? 0.f : w1[v]; w2[v] = start ? 0.f : w2[v]; }
                if constexpr (LOCAL) h[v] = start ? 0.f : h[v];
            }
            line_update<V>(h, av, w0, w1, w2, first, last);
#pragma unroll
            for (int v = 0; v < V; ++v) trow[v * pitch + col0 + e] += elem<T>(s.u[v], e) * h[v];
            if constexpr (SAVE) {
#pragma unroll
                for (int v = 0; v < V; ++v) hs[v][e] = h[v];
            }
        }
        if constexpr (SAVE) {
#pragma unroll
            for (int v = 0; v < V; ++v) {
                uint32_t r[NR];
                pack<T, CS>(hs[v], r);
                st_buf<NB, CP_STREAM>(hb, voff, col0 * (int)sizeof(T) + v * row_bytes, r);
            }
        }
    }

    __device__ __forceinline__ void prologue() { if (active) issue(buf0, 0); }

    // chunks [c_begin, c_end); the buffer for chunk c_begin already holds it or is being loaded.
    // Unused lanes are masked off for the whole loop (their DPP reads see 0).
    __device__ __forceinline__ void run(int c_begin, int c_end) {
        if (!active) return;
        if constexpr (!DB) {
            for (int c = c_begin; c < c_end; ++c) {
                compute(buf0, c);
                issue(buf0, c + 1 < nchunks ? c + 1 : c);     // clamped: redundant but in bounds at the end
            }
            return;
        }
        for (int c = c_begin; c < c_end; ++c) {
            const int cn = c + 1 < nchunks ? c + 1 : c;      // clamped: redundant but in bounds at the end
            if ((c & 1) == 0) {
                issue(buf1, cn);
                compute(buf0, c);
            } else {
                issue(buf0, cn);
                compute(buf1, c);
            }
        }
    }
};

// ---------------------------------------------------------------------------
// horizontal direction for lines longer than a wave can hold at one row per lane: the H image
// rows of a line are split over `parts` waves (each lane owns ONE row, so a whole 128 B memory
// line per row and tensor fits in registers and every line is fetched exactly once).  The
// waves of a line run in lock step, one workgroup barrier per scan step, and pass the state of
// their edge rows to each other through a two-slot LDS mailbox (slot = parity of the step).
// Because every step is its own barrier interval, the two directions never own the same tile
// column at the same time and no mid-scan split is needed.
// ---------------------------------------------------------------------------
template <typename T, int CS, bool REV, bool SAVE, bool LOCAL, bool LOGITS, bool BWD = false>
struct HorizontalSplitPass {
    static constexpr int NB = CS * (int)sizeof(T);
    static constexpr int NR = NB / 4;
    rsrc_t xb, lb, ub, w0b, w1b, w2b, hb;
    uint32_t voff;
    int nchunks;
    float* trow;        // this lane's row of the channel's tile
    float* mb_out;      // where this lane publishes its state (edge lanes only), parity 0
    const float* mb_up; // edge state of the part above (its last row), parity 0
    const float* mb_dn; // edge state of the part below (its first row), parity 0
    bool active, edge, top_lane, bot_lane, has_up, has_dn, img_first, img_last;
    float h;
    float wp0, wp1, wp2;   // BWD: taps of the column swept before
    StretchWalk walk;   // GSPN-local only
    StretchWalkBack bwalk;   // ... in the reverse sweep
    uint32_t bx[NR], bl[NR], bu[NR], b0[NR], b1[NR], b2[NR];

    // mailbox layout: [task = channel * 2 + direction slot][part][side: 0 first row, 1 last row][parity]
    __device__ __forceinline__ void init(const TileArgs& a, float* tile, float* mailbox, int d, int dslot, int b,
                                         int c_first, int kc, int part, int lane) {
        const FwdParams& p = a.p;
        const int H = p.H, W = p.W, HW = H * W;
        const int rp = H / a.parts;                       // rows per part (<= 64)
        active = lane < rp;
        const int lr = active ? lane : 0;
        const int row = part * rp + lr;
        const int c = c_first + kc;
        const int g = c / p.cpg;
        top_lane = lr == 0; bot_lane = lr == rp - 1;
        edge = active && (top_lane || bot_lane);
        has_up = part > 0; has_dn = part < a.parts - 1;
        img_first = top_lane && !has_up; img_last = bot_lane && !has_dn;
        const size_t planes = (size_t)p.B * p.C;
        const size_t slot_c = p.shared ? 0 : (size_t)d * planes * HW;
        const size_t slot_w = p.shared ? 0 : (size_t)d * p.B * p.G * 3 * HW;
        const size_t plane0 = ((size_t)b * p.C + c) * HW;
        const size_t plane_bytes = (size_t)HW * sizeof(T);
        const char* wbase = (const char*)p.w + (slot_w + ((size_t)b * p.G + g) * 3 * HW) * sizeof(T);
        voff = (uint32_t)(row * W * (int)sizeof(T));
        xb = make_rsrc((const char*)p.x + plane0 * sizeof(T));
        lb = make_rsrc((const char*)p.lam + (slot_c + plane0) * sizeof(T));
        ub = make_rsrc((const char*)p.u + (slot_c + plane0) * sizeof(T));
        w0b = make_rsrc(wbase); w1b = make_rsrc(wbase + plane_bytes); w2b = make_rsrc(wbase + 2 * plane_bytes);
        hb = make_rsrc(SAVE ? (char*)p.hs + ((size_t)d * planes * HW + plane0) * sizeof(T) : (char*)p.y);
        nchunks = W / CS;
        trow = tile + (kc * H + row) * a.pitch;
        float* task = mailbox + ((kc * 2 + dslot) * a.parts) * 4;
        mb_out = task + part * 4 + (bot_lane ? 2 : 0);
        mb_up = task + (has_up ? part - 1 : part) * 4 + 2;
        mb_dn = task + (has_dn ? part + 1 : part) * 4 + 0;
        h = 0.f; wp0 = 0.f; wp1 = 0.f; wp2 = 0.f;
        if constexpr (LOCAL && !BWD) walk.init(W, REV, p.kchunk);
        if constexpr (LOCAL && BWD) bwalk.init(W, d & 1, p.kchunk);
    }

    __device__ __forceinline__ int chunk_col(int c) const { return (REV ? nchunks - 1 - c : c) * CS; }

    __device__ __forceinline__ void issue(int c) {
        const int so = chunk_col(c) * (int)sizeof(T);
        ld_buf<NB>(xb, voff, so, bx);
        ld_buf<NB>(lb, voff, so, bl);
        ld_buf<NB>(ub, voff, so, bu);
        ld_buf<NB>(w0b, voff, so, b0);
        ld_buf<NB>(w1b, voff, so, b1);
        ld_buf<NB>(w2b, voff, so, b2);
    }

    // one chunk of CS scan steps; `s0` = scan step of its first column (for the mailbox parity)
    __device__ __forceinline__ void compute(int c) {
        const int col0 = chunk_col(c);
        float hs[CS];
#pragma unroll
        for (int k = 0; k < CS; ++k) {
            const int e = REV ? CS - 1 - k : k;
            constexpr int dummy = 0; (void)dummy;
            const int par = k & 1;                           // CS is even: parity of the scan step
            // edge state the neighbouring parts published in the previous step
            const float pu = mb_up[par ^ 1];
            const float pd = mb_dn[par ^ 1];
            const float yold = trow[col0 + e];               // read early: one LDS round trip per step, not three
            if constexpr (BWD) {
                // the edge rows publish the products that cross into the neighbouring part: tap 0 of a part's first row
                // reads the row above it, tap 2 of its last row the row below
                const float q0 = wp0 * h, q2 = wp2 * h;
                float up = from_lane_below(q2), dn = from_lane_above(q0);
                up = top_lane ? (has_up ? pu : 0.f) : up;
                dn = bot_lane ? (has_dn ? pd : 0.f) : dn;
                h = fmaf(wp1, h, elem<T>(bl, e) * elem<T>(bx, e)) + (up + dn);
                bool starts = false;                      // GSPN-local: this column starts a stretch in scan order
                if constexpr (LOCAL) starts = bwalk.start(c == nchunks - 1 && k == CS - 1);
                float c0 = elem<T>(b0, e), c1 = elem<T>(b1, e), c2 = elem<T>(b2, e);
                if constexpr (LOGITS) softmax3(c0, c1, c2, img_first, img_last);
                wp0 = (img_first || starts) ? 0.f : c0;
                wp1 = starts ? 0.f : c1;
                wp2 = (img_last || starts) ? 0.f : c2;
                if (edge) mb_out[par] = bot_lane ? wp2 * h : wp0 * h;
                trow[col0 + e] = fmaf(elem<T>(bu, e), h, yold);
                hs[e] = h;
                lds_barrier();
                continue;
            }
            bool start = (c == 0) && (k == 0);
            if constexpr (LOCAL) start = walk.start();
            float w0 = elem<T>(b0, e), w1 = elem<T>(b1, e), w2 = elem<T>(b2, e);
            if constexpr (LOGITS) softmax3(w0, w1, w2, img_first, img_last);
            if (LOCAL || k == 0) { w0 = start ? 0.f : w0; w1 = start ? 0.f : w1; w2 = start ? 0.f : w2; }
            const float av = elem<T>(bl, e) * elem<T>(bx, e);
            float up = from_lane_below(h), dn = from_lane_above(h);
            up = top_lane ? (has_up ? pu : 0.f) : up;
            dn = bot_lane ? (has_dn ? pd : 0.f) : dn;
            w0 = img_first ? 0.f : w0;
            w2 = img_last ? 0.f : w2;
            h = fmaf(w0, up, fmaf(w1, h, fmaf(w2, dn, av)));
            if (edge) mb_out[par] = h;
            trow[col0 + e] = fmaf(elem<T>(bu, e), h, yold);
            if constexpr (SAVE) hs[e] = h;
            lds_barrier();
        }
        if constexpr (SAVE) {
            uint32_t r[NR];
            pack<T, CS>(hs, r);
            st_buf<NB, CP_STREAM>(hb, voff, col0 * (int)sizeof(T), r);
        }
    }

    __device__ __forceinline__ void prologue() { if (active) issue(0); }

    __device__ __forceinline__ void run() {
        // unused lanes are masked off for the whole loop; the wave still executes every barrier
        if (active) {
            for (int c = 0; c < nchunks; ++c) {
                compute(c);
                issue(c + 1 < nchunks ? c + 1 : c);     // clamped: redundant but in bounds at the end
            }
        }
    }
};

// BWD: the first pass of the backward scan for maps beyond the backward kernels' reach (see vertical_pass): the wave
// that sweeps in the orientation of scan direction d works on the parameters of the opposite direction d ^ 1
template <typename T, int VV, int VH, int CS, bool DB, int PF, bool SAVE, int MAXW, bool LOCAL, bool LOGITS, bool BWD = false>
__global__ void __launch_bounds__(64 * MAXW) fwd_tile_kernel(TileArgs a) {
    static_assert(LOCAL || !LOGITS, "logits run on the local instantiations (a global scan is one stretch)");
    static_assert(!BWD || VH != 3, "the reverse sweep takes the standard layout");
    extern __shared__ float tile[];
    const FwdParams& p = a.p;
    const int H = p.H, W = p.W, HW = H * W;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int blocks_per_image = p.C / a.K;
    const unsigned item = xcd_contiguous_item(blockIdx.x, gridDim.x);
    const int b = item / blocks_per_image;
    const int c_first = (item - b * blocks_per_image) * a.K;

    // tile, followed (row-split horizontal phases only) by the mailbox: both start at zero
    const int tile_floats = a.K * H * a.pitch;
    const int lds_floats = tile_floats + (VH == 0 ? a.K * 2 * a.parts * 4 : 0);
    for (int i = threadIdx.x; i < lds_floats; i += blockDim.x) tile[i] = 0.f;
    lds_barrier();

    // Every element of the LDS tile has exactly one owner wave between two barriers, so plain
    // read-modify-write is safe and the order of the four additions per element is fixed.
    // ---- vertical pair: one wave per (pack, direction).  The top->bottom wave takes rows
    // [0, ceil(H/2)) before the mid barrier and the rest after it; the bottom->top wave the complement.
    {
        const int nd = ((p.mask >> 0) & 1) + ((p.mask >> 1) & 1);
        const int packs = (a.K + a.pv - 1) / a.pv;
        if (nd > 0 && wave < packs * nd) {
            const int pk = wave / nd;
            const int d = (nd == 2) ? (wave - pk * nd) : ((p.mask & 1) ? 0 : 1);
            const bool down = (d == 0) != BWD;                 // this wave walks the rows from the top
            const int split = nd == 2 ? (down ? (H + 1) / 2 : H - (H + 1) / 2) : -1;
            if (down) vertical_pass<T, VV, PF, false, SAVE, LOCAL, LOGITS, false, BWD>(a, tile, b, c_first, pk, lane, split);
            else vertical_pass<T, VV, PF, true, SAVE, LOCAL, LOGITS, false, BWD>(a, tile, b, c_first, pk, lane, split);
        } else if (nd == 2) {
            lds_barrier();
        }
    }

    // ---- horizontal pair, split at mid-scan (chunk granularity) the same way
    {
        const int has_lr = (p.mask >> 2) & 1, has_rl = (p.mask >> 3) & 1;
        const int nd = has_lr + has_rl;
        const int packs = (a.K + a.ph - 1) / a.ph;
        const int nchunks = W / CS;
        const int half_lr = (nchunks + 1) / 2;            // chunks the left->right wave does before the barrier
        const int half_rl = nchunks - half_lr;            // chunks the right->left wave does before the barrier
        const bool busy = nd > 0 && wave < packs * nd;
        const int pk = busy ? wave / nd : 0;
        const int d = (nd == 2) ? 2 + (wave - pk * nd) : (has_lr ? 2 : 3);
        if constexpr (VH == 3) {
            // transposed storage of the horizontal directions: the vertical pass with the roles of H and W swapped;
            // the left->right wave takes columns [0, ceil(W/2)) before the mid barrier, the other wave the complement
            lds_barrier();                                  // vertical phase complete
            if (busy) {
                const int split = nd == 2 ? (d == 2 ? (W + 1) / 2 : W - (W + 1) / 2) : -1;
                if (d == 2) vertical_pass<T, VV, PF, false, SAVE, LOCAL, LOGITS, true>(a, tile, b, c_first, pk, lane, split);
                else vertical_pass<T, VV, PF, true, SAVE, LOCAL, LOGITS, true>(a, tile, b, c_first, pk, lane, split);
            } else if (nd == 2) {
                lds_barrier();
            }
        } else if constexpr (VH == 0) {
            // row-split variant: wave -> (channel, direction, part); one barrier per scan step for everybody
            const int ntask = a.K * nd * a.parts;
            const bool work = nd > 0 && wave < ntask;
            const int part = work ? wave % a.parts : 0;
            const int cd = work ? wave / a.parts : 0;
            const int kc = cd / (nd > 0 ? nd : 1);
            const int dslot = cd - kc * (nd > 0 ? nd : 1);
            const int dd = (nd == 2) ? 2 + dslot : (has_lr ? 2 : 3);
            float* mailbox = tile + tile_floats;
            if (nd == 0) {
                lds_barrier();
            } else if (work && (dd == 2) != BWD) {             // this wave walks the columns from the left
                HorizontalSplitPass<T, CS, false, SAVE, LOCAL, LOGITS, BWD> hp;
                hp.init(a, tile, mailbox, dd, dslot, b, c_first, kc, part, lane);
                hp.prologue();
                lds_barrier();
                hp.run();
            } else if (work) {
                HorizontalSplitPass<T, CS, true, SAVE, LOCAL, LOGITS, BWD> hp;
                hp.init(a, tile, mailbox, dd, dslot, b, c_first, kc, part, lane);
                hp.prologue();
                lds_barrier();
                hp.run();
            } else {
                lds_barrier();
                for (int st = 0; st < W; ++st) lds_barrier();    // idle wave: keep the barrier count
            }
        } else if (nd == 0) {
            lds_barrier();
        } else if ((d == 2) != BWD) {                       // this wave walks the columns from the left
            HorizontalPass<T, VH, CS, false, SAVE, DB, LOCAL, LOGITS, BWD> hp;
            if (busy) { hp.init(a, tile, d, b, c_first, pk, lane); hp.prologue(); }
            lds_barrier();                                  // vertical phase complete (first loads already in flight)
            if (busy) hp.run(0, nd == 2 ? half_lr : nchunks);
            if (nd == 2) {
                lds_barrier();
                if (busy) hp.run(half_lr, nchunks);
            }
        } else {
            HorizontalPass<T, VH, CS, true, SAVE, DB, LOCAL, LOGITS, BWD> hp;
            if (busy) { hp.init(a, tile, d, b, c_first, pk, lane); hp.prologue(); }
            lds_barrier();
            if (busy) hp.run(0, nd == 2 ? half_rl : nchunks);
            if (nd == 2) {
                lds_barrier();
                if (busy) hp.run(half_rl, nchunks);
            }
        }
    }
    lds_barrier();

    // ---- write the merged tile out once, coalesced, rounded once to the storage type
    {
        T* Y = (T*)p.y + ((size_t)b * p.C + c_first) * HW;
        const int rows = a.K * H;
        const int nw = blockDim.x >> 6;
        for (int r = wave; r < rows; r += nw) {
            const float* tr = tile + r * a.pitch;
            T* yr = Y + (size_t)r * W;
            for (int j = lane * 2; j < W; j += 128) {
                float v[2] = {tr[j], tr[j + 1]};
                uint32_t o[2 * sizeof(T) / 4];
                pack<T, 2>(v, o);
                st_raw<2 * sizeof(T)>((char*)(yr + j), o);
            }
        }
    }
}

// ---------------------------------------------------------------------------
// host side: applicability, tiling choice, launch
// ---------------------------------------------------------------------------
static constexpr int TILE_PF = 8;     // lines kept in flight per wave in the vertical phases
static constexpr int LDS_BUDGET = 160 * 1024;

// Horizontal-phase variants: rows per lane, scan steps per burst, double buffered or not.
//   bursts of 112 B (a whole row of 56 bf16 / 28 fp32, half a row of 56 fp32 / 112 bf16), one row per lane,
//   single buffer;
//   64 B bursts (one L2 sector per row and tensor), two rows per lane, single buffer;
//   16 B bursts, two rows per lane, double buffered: any width that is a multiple of 16 B.
enum HVariant { H_ROW = 0, H_SECTOR = 1, H_SMALL = 2, H_SPLIT = 3, H_TRANSPOSED = 4 };

struct TilePlan { bool ok; int hv, vv, vh, cs, K, pitch, lplv, pv, lplh, ph, nwaves, parts; size_t lds; };

static TilePlan plan_tile(const FwdParams& p, int dtype) {
    TilePlan t = {};
    const int es = dtype == 0 ? 4 : 2;
    // two positions per lane in the vertical passes.  Measured and not adopted on 128x128 in the transposed layout:
    // four positions per lane with half as many waves (0.233 -> 0.294 ms); reading the tile elements of a step one
    // step ahead (0.232 -> 0.229 ms there, 0.299 -> 0.306 ms in the standard layout)
    const int vv = 2;
    if (p.W % vv || p.W / vv > 64) return t;
    // a map of one row has no mid-scan meeting of the vertical pair (the barrier that separates the two halves sits
    // before a step both waves take): such maps run the generic kernel
    if (p.H < 2) return t;
    const int row_bytes = p.W * es;
    int hv;
    const int parts = (p.H + 63) / 64;
    if (p.xt) {
        // horizontal directions stored transposed: they run the vertical machinery, two image rows per lane
        if (p.hs || p.H % vv || p.H / vv > 64) return t;
        hv = H_TRANSPOSED;
    }
    else if (row_bytes % 112 == 0 && row_bytes <= 224 && p.H <= 64) hv = H_ROW;
    else if (row_bytes % 128 == 0 && p.H > 64 && p.H % parts == 0 && p.H / parts >= 2) hv = H_SPLIT;
    else if (row_bytes % 64 == 0) hv = H_SECTOR;
    else if (row_bytes % 16 == 0) hv = H_SMALL;
    else return t;
    const int vh = hv == H_ROW ? 1 : (hv == H_SPLIT ? 0 : 2);      // image rows per lane (0: one row, rows split over waves)
    const int cs = hv == H_ROW ? 112 / es : (hv == H_SPLIT ? 128 / es : (hv == H_SECTOR ? 64 / es : 16 / es));
    if (vh > 0 && (p.H % vh || p.H / vh > 64)) return t;
    t.hv = hv; t.vv = vv; t.vh = vh; t.cs = cs; t.parts = hv == H_SPLIT ? parts : 1;
    t.pitch = p.W | 1;
    t.lplv = p.W / vv; t.pv = 64 / t.lplv;
    t.lplh = vh > 0 ? p.H / vh : 64; t.ph = vh > 0 ? 64 / t.lplh : 1;
    const size_t per_channel = (size_t)p.H * t.pitch * sizeof(float) + (hv == H_SPLIT ? 2 * parts * 4 * sizeof(float) : 0);
    // channels per workgroup: the smallest count that fills the lanes of a wave in both phases
    // (several small workgroups per CU overlap each other's barriers and load waits better than
    // one large one), dividing C, fitting LDS, with at most 8 waves (fp16 storage: 4 -- its widening and rounding
    // instructions hold more registers than the shifts of bf16, and the 128 registers per lane of an eight-wave
    // workgroup do not take them without spilling)
    const int max_waves = dtype == 2 ? 4 : 8;
    const int dirs_v = ((p.mask >> 0) & 1) + ((p.mask >> 1) & 1), dirs_h = ((p.mask >> 2) & 1) + ((p.mask >> 3) & 1);
    const int want = t.pv > t.ph ? t.pv : t.ph;
    int best = 0;
    for (int K = 1; K <= p.C && K <= 64; ++K) {
        if (p.C % K) continue;
        if (K * per_channel > (size_t)LDS_BUDGET) break;
        const int wv = ((K + t.pv - 1) / t.pv) * dirs_v, wh = ((K + t.ph - 1) / t.ph) * dirs_h * t.parts;
        const int nw = wv > wh ? wv : wh;
        if (nw > max_waves) continue;
        best = K;
        if (K >= want && K % t.pv == 0 && K % t.ph == 0) break;
    }
    if (!best) return t;
    t.K = best;
    {
        const int wv = ((best + t.pv - 1) / t.pv) * dirs_v, wh = ((best + t.ph - 1) / t.ph) * dirs_h * t.parts;
        t.nwaves = wv > wh ? wv : wh;
        if (t.nwaves < 1) t.nwaves = 1;
    }
    t.lds = best * per_channel;
    if ((size_t)p.B * (p.C / best) > 0x7fffffffull) return t;
    if ((size_t)t.pv * p.H * p.W * es >= (1ull << 31) || (size_t)p.G * 3 * p.H * p.W * es >= (1ull << 31)) return t;
    t.ok = true;
    return t;
}


template <typename T, int VV, int VH, int CS, bool DB, int PF, bool SAVE, int MAXW, bool LOCAL, bool LOGITS, bool BWD = false>
static hipError_t launch_one_l(const TileArgs& a, const TilePlan& t, hipStream_t s) {
    const dim3 grid((unsigned)((size_t)a.p.B * (a.p.C / a.K))), block(64 * t.nwaves);
    auto k = fwd_tile_kernel<T, VV, VH, CS, DB, PF, SAVE, MAXW, LOCAL, LOGITS, BWD>;
    hipError_t e = allow_dynamic_lds((const void*)k, LDS_BUDGET);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k, grid, block, t.lds, s, a);
    return hipGetLastError();
}

// One translation unit per (storage type, family): LOC = false instantiates the kernels of the global scan, LOC = true
// those of GSPN-local (Sec. 3.2) and of the weights-as-logits calls, so that the global scan carries none of their
// bookkeeping and the library builds in parallel.
template <typename T, int VV, int VH, int CS, bool DB, int PF, bool SAVE, int MAXW, bool LOC>
static hipError_t launch_one(const TileArgs& a, const TilePlan& t, hipStream_t s) {
    if constexpr (LOC) {
        // weights as logits always run a local instantiation (a global scan is one stretch)
        if (a.p.logits) return launch_one_l<T, VV, VH, CS, DB, PF, SAVE, MAXW, true, true>(a, t, s);
        return launch_one_l<T, VV, VH, CS, DB, PF, SAVE, MAXW, true, false>(a, t, s);
    } else {
        return launch_one_l<T, VV, VH, CS, DB, PF, SAVE, MAXW, false, false>(a, t, s);
    }
}

// storage type -> the dtype code of the planners
template <typename T> constexpr int dtype_code() { return sizeof(T) == 4 ? 0 : (__is_same(T, f16_t) ? 2 : 1); }

template <typename T, int VV, int VH, int CS, bool DB, int PF, bool LOC>
static hipError_t launch_cfg(const TileArgs& a, const TilePlan& t, bool save, hipStream_t s) {
    if (t.nwaves <= 4)
        return save ? launch_one<T, VV, VH, CS, DB, PF, true, 4, LOC>(a, t, s)
                    : launch_one<T, VV, VH, CS, DB, PF, false, 4, LOC>(a, t, s);
    if constexpr (__is_same(T, f16_t)) return hipErrorInvalidValue;      // (never planned: see plan_tile)
    else
        return save ? launch_one<T, VV, VH, CS, DB, PF, true, 8, LOC>(a, t, s)
                    : launch_one<T, VV, VH, CS, DB, PF, false, 8, LOC>(a, t, s);
}

template <typename T, bool LOC>
static hipError_t launch_fwd_tile_part(const FwdParams& p, hipStream_t s) {
    constexpr int ES = (int)sizeof(T);
    const TilePlan t = plan_tile(p, dtype_code<T>());
    if (!t.ok) return hipErrorInvalidValue;
    TileArgs a;
    a.p = p; a.K = t.K; a.pitch = t.pitch; a.lplv = t.lplv; a.pv = t.pv; a.lplh = t.lplh; a.ph = t.ph;
    a.nwaves = t.nwaves; a.parts = t.parts;
    const bool save = p.hs != nullptr;
    // scan steps per burst of the horizontal variants: 128 B, a whole row of 112 B, 64 B, 16 B
    if (t.hv == H_TRANSPOSED) return launch_cfg<T, 2, 3, 2, false, TILE_PF, LOC>(a, t, save, s);
    if (t.hv == H_SPLIT) return launch_cfg<T, 2, 0, 128 / ES, false, TILE_PF, LOC>(a, t, save, s);
    if (t.hv == H_ROW) return launch_cfg<T, 2, 1, 112 / ES, false, TILE_PF, LOC>(a, t, save, s);
    if (t.hv == H_SECTOR) return launch_cfg<T, 2, 2, 64 / ES, false, TILE_PF, LOC>(a, t, save, s);
    return launch_cfg<T, 2, 2, 16 / ES, true, TILE_PF, LOC>(a, t, save, s);
}

// First pass of the two-pass backward scan (gspn_bwd_twopass.hip): p holds gy as x, u as lam, lam as u, gx as y and
// the buffer that receives e as hs.  One translation unit per storage type.
template <typename T, int VV, int VH, int CS, bool DB, int PF, int MAXW, bool LOC>
static hipError_t launch_one_reverse(const TileArgs& a, const TilePlan& t, hipStream_t s) {
    if constexpr (LOC) {
        if (a.p.logits) return launch_one_l<T, VV, VH, CS, DB, PF, true, MAXW, true, true, true>(a, t, s);
        return launch_one_l<T, VV, VH, CS, DB, PF, true, MAXW, true, false, true>(a, t, s);
    } else {
        return launch_one_l<T, VV, VH, CS, DB, PF, true, MAXW, false, false, true>(a, t, s);
    }
}

template <typename T, int VV, int VH, int CS, bool DB, int PF, bool LOC>
static hipError_t launch_cfg_reverse(const TileArgs& a, const TilePlan& t, hipStream_t s) {
    if (t.nwaves <= 4) return launch_one_reverse<T, VV, VH, CS, DB, PF, 4, LOC>(a, t, s);
    if constexpr (__is_same(T, f16_t)) return hipErrorInvalidValue;      // (never planned: see plan_tile)
    else return launch_one_reverse<T, VV, VH, CS, DB, PF, 8, LOC>(a, t, s);
}

// LOC as in launch_one: the GSPN-local and logits calls on instantiations (and in translation units) of their own
template <typename T, bool LOC>
static hipError_t launch_reverse_sweep_part(const FwdParams& p, hipStream_t s) {
    constexpr int ES = (int)sizeof(T);
    const TilePlan t = plan_tile(p, dtype_code<T>());
    if (!t.ok || t.hv == H_TRANSPOSED || !p.hs || LOC != (p.kchunk > 0 || p.logits)) return hipErrorInvalidValue;
    TileArgs a;
    a.p = p; a.K = t.K; a.pitch = t.pitch; a.lplv = t.lplv; a.pv = t.pv; a.lplh = t.lplh; a.ph = t.ph;
    a.nwaves = t.nwaves; a.parts = t.parts;
    if (t.hv == H_SPLIT) return launch_cfg_reverse<T, 2, 0, 128 / ES, false, TILE_PF, LOC>(a, t, s);
    if (t.hv == H_ROW) return launch_cfg_reverse<T, 2, 1, 112 / ES, false, TILE_PF, LOC>(a, t, s);
    if (t.hv == H_SECTOR) return launch_cfg_reverse<T, 2, 2, 64 / ES, false, TILE_PF, LOC>(a, t, s);
    return launch_cfg_reverse<T, 2, 2, 16 / ES, true, TILE_PF, LOC>(a, t, s);
}

}  // namespace gspn
