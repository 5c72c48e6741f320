// Forward GSPN scan for feature maps too large for an on-chip output tile (e.g. 512x512,
// 256x1024): one workgroup per (image, channel) plane, all directions inside one launch
// (Sec. 4.1: the loop over lines is inside the kernel), wave-owned lines in registers with DPP
// neighbour exchange, and the merged output y = sum_d u_d*h_d (Eq. 2 + sum merge of the four
// passes of Sec. 3.2) accumulated in place in global memory, direction after direction, by the
// workgroup that owns the plane (fixed order, no atomics, no zero fill).  In bf16 storage the
// running sum is rounded once per direction.  The global scan can save its hidden states (h_save), and
// the same kernel runs the reverse sweep of the two-pass backward scan (template flags SAVE, BWD).
//
//  * Vertical directions: a line is an image row of W = 64*V positions held by ONE wave (V
//    contiguous positions per lane, 16..32 B vector loads), PF lines prefetched in registers.  The
//    two vertical waves split the rows: each first STORES its half of y, then, after a barrier,
//    READ-MODIFY-WRITES the other half.
//  * Horizontal directions: a line is an image column of H positions split over H/64 waves (one
//    image row per lane), lock-stepped with one workgroup barrier per scan step and an LDS
//    mailbox for the edge rows; every lane reads its row in 128 B bursts (one cache line per tensor)
//    and read-modify-writes its 128 B of y per burst.  The two horizontal directions run one
//    after the other.
#pragma once
#include "gspn_tile_common.hpp"
#include <stdlib.h>

namespace gspn {

struct StreamArgs {
    FwdParams p;
    int parts;     // waves per image column in the horizontal phases (H / 64)
    int nwaves;
};

// ---------------------------------------------------------------------------
// vertical direction, one wave per line
// ---------------------------------------------------------------------------
// LOCAL: GSPN-local (Sec. 3.2), on instantiations of its own so that the global scan carries none of it
// LOGITS (with LOCAL): w holds raw logits, normalised as they are consumed (softmax3)
// BWD: the reverse sweep of the backward pass (first pass of the two-pass backward scan): the caller passes gy as x, u as
// lam, lam as u, gx as y and the buffer that receives e as hs; the wave that walks the rows downwards then works on the
// parameters of the bottom->top scan and the other way round, applies the taps of the line it swept before
// (line_update_transposed) and stores its state per line
// SAVE: the state of every line is stored per direction (h_save of the forward call; e of the reverse sweep)
template <typename T, int V, int PF, bool REV, bool LOCAL, bool LOGITS, bool BWD = false, bool SAVE = BWD>
struct VStream {
    static_assert(!BWD || SAVE, "the reverse sweep saves its state");
    static constexpr int NB = V * (int)sizeof(T);
    static constexpr int NR = NB / 4;
    // more than 16 bytes per lane: as runs of 16 bytes, 1 KB apart, so that every request covers whole lines, each once
    static constexpr int RUNS = NB > 16 ? NB / 16 : 1;
    // x, lam, u are read once by the launch
    static constexpr int CP_OWN = CP_STREAM;
    struct Line { uint32_t x[NR], l[NR], u[NR], w0[NR], w1[NR], w2[NR], y[NR]; };
    rsrc_t xb, lb, ub, w0b, w1b, w2b, yb, hb;
    uint32_t voff;
    int H, row_bytes;
    bool first, last;
    float h[V];
    float wp0[BWD ? V : 1], wp1[BWD ? V : 1], wp2[BWD ? V : 1];   // BWD: taps of the line swept before
    StretchWalk walk;   // GSPN-local only
    StretchWalkBack bwalk;   // ... in the reverse sweep

    __device__ __forceinline__ void init(const FwdParams& p, int b, int c, int lane) {
        constexpr int d = (REV != BWD) ? 1 : 0;
        H = p.H;
        if constexpr (LOCAL && !BWD) walk.init(p.H, REV, p.kchunk);
        if constexpr (LOCAL && BWD) bwalk.init(p.H, d & 1, p.kchunk);
        const int W = p.W, HW = H * W;
        const int g = c / p.cpg;
        const size_t planes = (size_t)p.B * p.C;
        const size_t slot_c = p.shared ? 0 : (size_t)d * planes * HW;
        const size_t slot_w = p.shared ? 0 : (size_t)d * p.B * p.G * 3 * HW;
        const size_t plane0 = ((size_t)b * p.C + c) * HW;
        const size_t plane_bytes = (size_t)HW * sizeof(T);
        const char* wbase = (const char*)p.w + (slot_w + ((size_t)b * p.G + g) * 3 * HW) * sizeof(T);
        row_bytes = W * (int)sizeof(T);
        voff = (uint32_t)(lane * (RUNS > 1 ? 16 : NB));
        first = lane == 0; last = lane == 63;
        xb = make_rsrc((const char*)p.x + plane0 * sizeof(T));
        lb = make_rsrc((const char*)p.lam + (slot_c + plane0) * sizeof(T));
        ub = make_rsrc((const char*)p.u + (slot_c + plane0) * sizeof(T));
        w0b = make_rsrc(wbase); w1b = make_rsrc(wbase + plane_bytes); w2b = make_rsrc(wbase + 2 * plane_bytes);
        yb = make_rsrc((char*)p.y + plane0 * sizeof(T));
        hb = make_rsrc(SAVE ? (char*)p.hs + ((size_t)d * planes * HW + plane0) * sizeof(T) : (char*)p.y);
#pragma unroll
        for (int v = 0; v < V; ++v) h[v] = 0.f;
        if constexpr (BWD) {
#pragma unroll
            for (int v = 0; v < V; ++v) { wp0[v] = 0.f; wp1[v] = 0.f; wp2[v] = 0.f; }
        }
    }

    __device__ __forceinline__ int row_off(int t) const { return (REV ? H - 1 - t : t) * row_bytes; }
    template <int CP = 0> __device__ __forceinline__ void ld_line(rsrc_t rs, int so, uint32_t* r) const {
        if constexpr (RUNS > 1) ld_runs<NB, CP>(rs, voff, so, r); else ld_buf<NB, CP>(rs, voff, so, r);
    }
    template <int CP = 0> __device__ __forceinline__ void st_line(rsrc_t rs, int so, const uint32_t* r) const {
        if constexpr (RUNS > 1) st_runs<NB, CP>(rs, voff, so, r); else st_buf<NB, CP>(rs, voff, so, r);
    }
    __device__ __forceinline__ void update(const float (&av)[V], const float (&w0)[V], const float (&w1)[V], const float (&w2)[V]) {
        if constexpr (RUNS > 1) line_update_runs<V, RUNS>(h, av, w0, w1, w2, first, last);
        else line_update<V>(h, av, w0, w1, w2, first, last);
    }
    __device__ __forceinline__ void update_transposed(const float (&av)[V]) {
        if constexpr (RUNS > 1) line_update_transposed_runs<V, RUNS>(h, av, wp0, wp1, wp2, first, last);
        else line_update_transposed<V>(h, av, wp0, wp1, wp2, first, last);
    }

    // scan steps [t_begin, t_end); RMW: y already holds the other directions' sum for these rows
    template <bool RMW>
    __device__ __forceinline__ void run(int t_begin, int t_end) {
        Line slot[PF];
        auto issue = [&](Line& s, int t) {
            const int so = row_off(t < t_end ? t : t_end - 1);    // clamped: redundant but in bounds
            ld_line<CP_OWN>(xb, so, s.x);
            ld_line<CP_OWN>(lb, so, s.l);
            ld_line<CP_OWN>(ub, so, s.u);
            ld_line(w0b, so, s.w0);
            ld_line(w1b, so, s.w1);
            ld_line(w2b, so, s.w2);
            if constexpr (RMW) ld_line(yb, so, s.y);
        };
        if (t_begin >= t_end) return;
        // line after line, as the loop below requests them: the compiler would otherwise group the requests by tensor,
        // count few requests behind the first line's on entry to the loop, and wait for (nearly) all of them at its head
#pragma unroll
        for (int k = 0; k < PF; ++k) { issue(slot[k], t_begin + k); __builtin_amdgcn_sched_barrier(0); }
        // one line: ring slot k holds it; its slot takes line t + PF
        auto line = [&](int t, int k) __attribute__((always_inline)) {
            const Line& cur = slot[k];
            float av[V], w0[V], w1[V], w2[V], yv[V];
            if constexpr (BWD) {
                // GSPN-local: a line that starts a stretch takes nothing from the line before it in scan
                // order, so its taps hand nothing on to the line swept next
                bool starts = false;
                if constexpr (LOCAL) starts = bwalk.start(t == H - 1);
#pragma unroll
                for (int v = 0; v < V; ++v) av[v] = elem<T>(cur.l, v) * elem<T>(cur.x, v);
                update_transposed(av);
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    float c0 = elem<T>(cur.w0, v), c1 = elem<T>(cur.w1, v), c2 = elem<T>(cur.w2, v);
                    if constexpr (LOGITS) softmax3(c0, c1, c2, first && v == 0, last && v == V - 1);
                    // a tap that points outside the line takes nothing, whatever the tensor holds there
                    wp0[v] = ((first && v == 0) || starts) ? 0.f : c0;
                    wp1[v] = starts ? 0.f : c1;
                    wp2[v] = ((last && v == V - 1) || starts) ? 0.f : c2;
                    yv[v] = elem<T>(cur.u, v) * h[v];
                    if constexpr (RMW) yv[v] += elem<T>(cur.y, v);
                }
                uint32_t o[NR];
                pack<T, V>(yv, o);
                st_line(yb, row_off(t), o);
                pack<T, V>(h, o);
                st_line<CP_STREAM>(hb, row_off(t), o);
                issue(slot[k], t + PF);
                return;
            }
            // scan step 0 (only ever in ring slot 0): its weights are never used (the stored values may be
            // anything); GSPN-local: the same for the first line of every stretch, any slot
            bool start = t == 0;
            if constexpr (LOCAL) start = walk.start();
#pragma unroll
            for (int v = 0; v < V; ++v) {
                av[v] = elem<T>(cur.l, v) * elem<T>(cur.x, v);
                w0[v] = elem<T>(cur.w0, v); w1[v] = elem<T>(cur.w1, v); w2[v] = elem<T>(cur.w2, v);
                if constexpr (LOGITS) softmax3(w0[v], w1[v], w2[v], first && v == 0, last && v == V - 1);
                if (LOCAL || k == 0) { w0[v] = start ? 0.f : w0[v]; w1[v] = start ? 0.f : w1[v]; w2[v] = start ? 0.f : w2[v]; }
                if constexpr (LOCAL) h[v] = start ? 0.f : h[v];
            }
            update(av, w0, w1, w2);
#pragma unroll
            for (int v = 0; v < V; ++v) {
                yv[v] = elem<T>(cur.u, v) * h[v];
                if constexpr (RMW) yv[v] += elem<T>(cur.y, v);
            }
            uint32_t o[NR];
            pack<T, V>(yv, o);
            st_line(yb, row_off(t), o);
            if constexpr (SAVE) {
                pack<T, V>(h, o);
                st_line<CP_STREAM>(hb, row_off(t), o);      // h_save: nothing in this call reads it
            }
            issue(slot[k], t + PF);
        };
        // whole groups of PF lines without a test inside (a way out of the middle of a group would reach the loop's back
        // edge with few requests counted behind the next line's, and the compiler would wait for nearly all of them at
        // the head of every group), then the lines left over
        const int t_main = t_begin + (t_end - t_begin) / PF * PF;
        for (int t0 = t_begin; t0 < t_main; t0 += PF) {
#pragma unroll
            for (int k = 0; k < PF; ++k) { line(t0 + k, k); __builtin_amdgcn_sched_barrier(0); }   // one line after the other
        }
#pragma unroll
        for (int k = 0; k < PF; ++k)
            if (t_main + k < t_end) line(t_main + k, k);
    }
};

// ---------------------------------------------------------------------------
// horizontal direction, the rows of the image split over `parts` waves, one row per lane
// ---------------------------------------------------------------------------
// A chunk (CS scan steps: NB = 64 or 128 bytes of every row) is requested so that NB / 16 neighbouring lanes share an image
// row -- an instruction then touches 16 or 8 lines instead of the 64 it touches when every lane asks for its own row; the
// vector cache looks a line up once per lane group, and that rate bounded the row-per-lane requests -- and turned into
// the row-per-lane order through an LDS block of the wave's own (64 rows of NB + 16 bytes).  The chunk of y stays in that
// block while the chunk is worked on, so that no register holds it, and the registers of the other tensors take the next
// chunk's requests as their columns are consumed (128 registers per lane are enough for 64 B of a row per tensor).  y and
// the saved states leave through the block, in request order.
template <typename T, int CS, bool REV, bool LOCAL, bool LOGITS, bool BWD = false, bool SAVE = BWD>
struct HStream {
    static_assert(!BWD || SAVE, "the reverse sweep saves its state");
    static constexpr int NB = CS * (int)sizeof(T);
    static constexpr int NR = NB / 4;
    static constexpr int LPR = NB / 16;          // lanes per row, = instructions per chunk of a tensor
    static constexpr int RPI = 64 / LPR;         // rows per instruction
    static constexpr int PITCHU = LPR + 1;       // 16-byte units between two rows of the staging block
    static constexpr int STAGE_BYTES = 64 * PITCHU * 16;
    u32x4* g_wr;                                 // staging: where this lane drops the registers of instruction 0
    u32x4* g_rd;                                 // staging: this lane's row
    uint32_t voff_g;                             // request order: byte offset of (row l / LPR, piece l % LPR) in the plane
    int istep_g;                                 // bytes between the rows of two instructions
    rsrc_t xb, lb, ub, w0b, w1b, w2b, yb, hb;
    float wp0, wp1, wp2;   // BWD: taps of the column swept before
    StretchWalkBack bwalk; // BWD, GSPN-local
    int nchunks;
    float* mb_out;
    const float* mb_up;
    const float* mb_dn;
    bool edge, top_lane, bot_lane, has_up, has_dn, img_first, img_last;
    float h;
    StretchWalk walk;   // GSPN-local only
    uint32_t bx[NR], bl[NR], bu[NR], b0[NR], b1[NR], b2[NR], by[NR];

    __device__ __forceinline__ void init(const FwdParams& p, float* mailbox, int parts, int b, int c, int part, int lane) {
        constexpr int d = (REV != BWD) ? 3 : 2;
        const int H = p.H, W = p.W, HW = H * W;
        const int g = c / p.cpg;
        top_lane = lane == 0; bot_lane = lane == 63;
        edge = top_lane || bot_lane;
        has_up = part > 0; has_dn = part < parts - 1;
        img_first = top_lane && !has_up; img_last = bot_lane && !has_dn;
        const size_t planes = (size_t)p.B * p.C;
        const size_t slot_c = p.shared ? 0 : (size_t)d * planes * HW;
        const size_t slot_w = p.shared ? 0 : (size_t)d * p.B * p.G * 3 * HW;
        const size_t plane0 = ((size_t)b * p.C + c) * HW;
        const size_t plane_bytes = (size_t)HW * sizeof(T);
        const char* wbase = (const char*)p.w + (slot_w + ((size_t)b * p.G + g) * 3 * HW) * sizeof(T);
        xb = make_rsrc((const char*)p.x + plane0 * sizeof(T));
        lb = make_rsrc((const char*)p.lam + (slot_c + plane0) * sizeof(T));
        ub = make_rsrc((const char*)p.u + (slot_c + plane0) * sizeof(T));
        w0b = make_rsrc(wbase); w1b = make_rsrc(wbase + plane_bytes); w2b = make_rsrc(wbase + 2 * plane_bytes);
        yb = make_rsrc((char*)p.y + plane0 * sizeof(T));
        hb = make_rsrc(SAVE ? (char*)p.hs + ((size_t)d * planes * HW + plane0) * sizeof(T) : (char*)p.y);
        wp0 = 0.f; wp1 = 0.f; wp2 = 0.f;
        nchunks = W / CS;
        // mailbox: [part][side: 0 first row, 1 last row][parity]
        mb_out = mailbox + part * 4 + (bot_lane ? 2 : 0);
        mb_up = mailbox + (has_up ? part - 1 : part) * 4 + 2;
        mb_dn = mailbox + (has_dn ? part + 1 : part) * 4 + 0;
        h = 0.f;
        if constexpr (LOCAL && !BWD) walk.init(W, REV, p.kchunk);
        if constexpr (LOCAL && BWD) bwalk.init(W, d & 1, p.kchunk);
        voff_g = (uint32_t)(((part * 64 + lane / LPR) * W) * (int)sizeof(T) + 16 * (lane % LPR));
        istep_g = RPI * W * (int)sizeof(T);
    }
    // `stage` = the wave's own block of STAGE_BYTES
    __device__ __forceinline__ void use_staging(char* stage, int lane) {
        g_wr = (u32x4*)stage + PITCHU * (lane / LPR) + (lane % LPR);
        g_rd = (u32x4*)stage + PITCHU * lane;
    }

    __device__ __forceinline__ int chunk_col(int c) const { return (REV ? nchunks - 1 - c : c) * CS; }

    // x, lam, u are read once: where a request covers whole lines (128 B of a row) it carries the non-temporal bit
    static constexpr int CP_OWN = NB == 128 ? CP_STREAM : 0;
    template <int CP = 0>
    __device__ __forceinline__ void ld_chunk(rsrc_t rs, int so, uint32_t (&r)[NR]) const {
#pragma unroll
        for (int i = 0; i < LPR; ++i) {
            const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, voff_g, __builtin_amdgcn_readfirstlane(so + i * istep_g), CP);
            r[4 * i] = v.x; r[4 * i + 1] = v.y; r[4 * i + 2] = v.z; r[4 * i + 3] = v.w;
        }
    }
    // instruction i of a chunk alone, into the registers 4i..4i+3
    template <int CP = 0>
    __device__ __forceinline__ void ld_piece(rsrc_t rs, int so, int i, uint32_t (&r)[NR]) const {
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, voff_g, __builtin_amdgcn_readfirstlane(so + i * istep_g), CP);
        r[4 * i] = v.x; r[4 * i + 1] = v.y; r[4 * i + 2] = v.z; r[4 * i + 3] = v.w;
    }
    // The 16 bytes (EPP columns) of a row that scan step k completes are consumed: their registers take an
    // instruction of the next chunk, so that it arrives while this one is worked on.  Not y, whose registers hold the
    // chunk's output until it is stored, nor -- with SAVE -- x, whose registers hold the states.
    static constexpr int EPP = 16 / (int)sizeof(T);
    __device__ __forceinline__ void refill(int c, int k) {
        if ((k % EPP) == EPP - 1 && c + 1 < nchunks) {
            __builtin_amdgcn_sched_barrier(0);       // not before the step that reads these registers last
            const int e = REV ? CS - 1 - k : k;
            const int q = e / EPP;
            const int so = chunk_col(c + 1) * (int)sizeof(T);
            if constexpr (!SAVE) ld_piece<CP_OWN>(xb, so, q, bx);
            ld_piece<CP_OWN>(lb, so, q, bl);
            ld_piece<CP_OWN>(ub, so, q, bu);
            ld_piece(w0b, so, q, b0);
            ld_piece(w1b, so, q, b1);
            ld_piece(w2b, so, q, b2);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    // request order -> row order, in place
    __device__ __forceinline__ void to_rows(uint32_t (&r)[NR]) const {
#pragma unroll
        for (int i = 0; i < LPR; ++i) { const u32x4 v = {r[4 * i], r[4 * i + 1], r[4 * i + 2], r[4 * i + 3]}; g_wr[RPI * PITCHU * i] = v; }
        __builtin_amdgcn_sched_barrier(0);     // the reads below take the registers the writes above have released
#pragma unroll
        for (int q = 0; q < LPR; ++q) { const u32x4 v = g_rd[q]; r[4 * q] = v.x; r[4 * q + 1] = v.y; r[4 * q + 2] = v.z; r[4 * q + 3] = v.w; }
        __builtin_amdgcn_sched_barrier(0);
    }
    template <int CP = 0>
    __device__ __forceinline__ void st_chunk(rsrc_t rs, int so, const uint32_t (&r)[NR]) const {
#pragma unroll
        for (int q = 0; q < LPR; ++q) { const u32x4 v = {r[4 * q], r[4 * q + 1], r[4 * q + 2], r[4 * q + 3]}; g_rd[q] = v; }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < LPR; ++i) st_b128<CP>(rs, voff_g + (uint32_t)(so + i * istep_g), g_wr[RPI * PITCHU * i]);
        __builtin_amdgcn_sched_barrier(0);
    }

    template <bool RMW>
    __device__ __forceinline__ void issue(int c) {
        const int so = chunk_col(c) * (int)sizeof(T);
        ld_chunk<CP_OWN>(xb, so, bx);
        ld_chunk<CP_OWN>(lb, so, bl);
        ld_chunk<CP_OWN>(ub, so, bu);
        ld_chunk(w0b, so, b0);
        ld_chunk(w1b, so, b1);
        ld_chunk(w2b, so, b2);
        if constexpr (RMW) ld_chunk(yb, so, by);
    }

    template <bool RMW>
    __device__ __forceinline__ void compute(int c) {
        // the six operand tensors into row order; the chunk of y into the staging block, where it stays while the chunk is
        // worked on (a lane reads and writes the words of its own row there)
        uint32_t* const yrow = (uint32_t*)g_rd;
        to_rows(bx); to_rows(bl); to_rows(bu); to_rows(b0); to_rows(b1); to_rows(b2);
        if constexpr (RMW) {
#pragma unroll
            for (int i = 0; i < LPR; ++i) { const u32x4 v = {by[4 * i], by[4 * i + 1], by[4 * i + 2], by[4 * i + 3]}; g_wr[RPI * PITCHU * i] = v; }
            __builtin_amdgcn_sched_barrier(0);
        }
        float ypair = 0.f;                                   // bf16: first element of the pair being assembled
        float epair = 0.f;                                   // SAVE: the same for the saved state
        uint32_t yw = 0;                                     // bf16: the word of y the pair adds to
        // step k has produced yv = u * h for element e: add it to y and keep the state (SAVE: x of this element is
        // consumed, its word takes h)
        auto emit = [&](int k, int e, float yv) __attribute__((always_inline)) {
            if constexpr (sizeof(T) == 4) {
                if constexpr (RMW) yv += __uint_as_float(yrow[e]);
                yrow[e] = __float_as_uint(yv);
                if constexpr (SAVE) bx[e] = __float_as_uint(h);
            } else {
                // elements e and e^1 share a word; the pair is complete on every second step
                if ((k & 1) == 0) {
                    ypair = yv; epair = h;
                    if constexpr (RMW) yw = yrow[e >> 1];
                } else {
                    float lo = (e & 1) ? ypair : yv, hi = (e & 1) ? yv : ypair;
                    if constexpr (RMW) { lo += word_lo<T>(yw); hi += word_hi<T>(yw); }
                    yrow[e >> 1] = pack_word<T>(lo, hi);
                    if constexpr (SAVE) bx[e >> 1] = pack_word<T>((e & 1) ? epair : h, (e & 1) ? h : epair);
                }
            }
        };
#pragma unroll
        for (int k = 0; k < CS; ++k) {
            const int e = REV ? CS - 1 - k : k;
            const int par = k & 1;                           // CS is even: parity of the scan step
            const float pu = mb_up[par ^ 1];
            const float pd = mb_dn[par ^ 1];
            if constexpr (BWD) {
                // the edge rows publish the products that cross into the neighbouring part: tap 0 of a part's first row
                // reads the row above it, tap 2 of its last row the row below
                const float q0 = wp0 * h, q2 = wp2 * h;
                float up = from_lane_below(q2), dn = from_lane_above(q0);
                up = top_lane ? (has_up ? pu : 0.f) : up;
                dn = bot_lane ? (has_dn ? pd : 0.f) : dn;
                h = fmaf(wp1, h, elem<T>(bl, e) * elem<T>(bx, e)) + (up + dn);
                bool starts = false;                     // GSPN-local: this column starts a stretch in scan order
                if constexpr (LOCAL) starts = bwalk.start(c == nchunks - 1 && k == CS - 1);
                float c0 = elem<T>(b0, e), c1 = elem<T>(b1, e), c2 = elem<T>(b2, e);
                if constexpr (LOGITS) softmax3(c0, c1, c2, img_first, img_last);
                wp0 = (img_first || starts) ? 0.f : c0;
                wp1 = starts ? 0.f : c1;
                wp2 = (img_last || starts) ? 0.f : c2;
                // y takes u * e and e replaces the words of x (= gy, consumed), element by element
                emit(k, e, elem<T>(bu, e) * h);
                if (edge) mb_out[par] = bot_lane ? wp2 * h : wp0 * h;
                refill(c, k);
                lds_barrier();
                continue;
            }
            bool start = (c == 0) && (k == 0);               // scan step 0: its weights are never used
            if constexpr (LOCAL) start = walk.start();       // ... nor those of a stretch's first line
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
            emit(k, e, elem<T>(bu, e) * h);
            if (edge) mb_out[par] = h;
            refill(c, k);
            lds_barrier();
        }
        // the chunk of y is in the staging block, in row order: it leaves in request order
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < LPR; ++i)
            st_b128(yb, voff_g + (uint32_t)(chunk_col(c) * (int)sizeof(T) + i * istep_g), g_wr[RPI * PITCHU * i]);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (SAVE) st_chunk<CP_STREAM>(hb, chunk_col(c) * (int)sizeof(T), bx);
    }

    template <bool RMW>
    __device__ __forceinline__ void run() {
        issue<RMW>(0);
        for (int c = 0; c < nchunks; ++c) {
            compute<RMW>(c);
            // the other tensors of the next chunk were requested as this one was consumed
            if (c + 1 < nchunks) {
                const int so = chunk_col(c + 1) * (int)sizeof(T);
                if constexpr (SAVE) ld_chunk<CP_OWN>(xb, so, bx);
                if constexpr (RMW) ld_chunk(yb, so, by);
            }
        }
    }
};

// BWD: first pass of the two-pass backward scan (see VStream); the wave that sweeps in the orientation of scan direction d
// works on the parameters of the opposite direction d ^ 1
template <typename T, int V, int CS, int PF, bool LOCAL, bool LOGITS, bool BWD = false, bool SAVE = BWD>
__global__ void __launch_bounds__(512) fwd_stream_kernel(StreamArgs a) {
    static_assert(LOCAL || !LOGITS, "logits run on the local instantiations (a global scan is one stretch)");
    __shared__ float mailbox[8 * 4];
    using HS = HStream<T, CS, false, LOCAL, LOGITS, BWD, SAVE>;
    __shared__ __attribute__((aligned(16))) char stage[8 * HS::STAGE_BYTES];      // horizontal phases: a block per wave
    const FwdParams& p = a.p;
    const int H = p.H, W = p.W;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const unsigned item = xcd_contiguous_item(blockIdx.x, gridDim.x);
    const int b = item / p.C, c = item - b * p.C;
    bool wrote = false;          // does y already hold a partial sum?  (uniform over the workgroup)

    // ---- vertical pair (waves 0 and 1)
    {
        const int has_tb = (p.mask >> 0) & 1, has_bt = (p.mask >> 1) & 1;
        const int nd = has_tb + has_bt;
        if (nd == 2) {
            const int split = (H + 1) / 2;          // top->bottom wave: rows [0, split) first; bottom->top: rows [split, H)
            if (wave == 0) {
                VStream<T, V, PF, false, LOCAL, LOGITS, BWD, SAVE> v; v.init(p, b, c, lane);
                v.template run<false>(0, split);
                __syncthreads();
                v.template run<true>(split, H);
            } else if (wave == 1) {
                VStream<T, V, PF, true, LOCAL, LOGITS, BWD, SAVE> v; v.init(p, b, c, lane);
                v.template run<false>(0, H - split);
                __syncthreads();
                v.template run<true>(H - split, H);
            } else {
                __syncthreads();
            }
            wrote = true;
        } else if (nd == 1) {
            if (wave == 0) {
                if ((has_tb != 0) != BWD) { VStream<T, V, PF, false, LOCAL, LOGITS, BWD, SAVE> v; v.init(p, b, c, lane); v.template run<false>(0, H); }
                else                      { VStream<T, V, PF, true, LOCAL, LOGITS, BWD, SAVE> v;  v.init(p, b, c, lane); v.template run<false>(0, H); }
            }
            wrote = true;
        }
    }

    // ---- horizontal directions, one after the other; waves 0..parts-1 hold the rows
    for (int dsel = 0; dsel < 2; ++dsel) {
        if (!((p.mask >> (2 + dsel)) & 1)) continue;
        if (threadIdx.x < 32) mailbox[threadIdx.x] = 0.f;
        __syncthreads();                        // y of the previous phase visible, mailbox cleared
        if (wave < a.parts) {
            if ((dsel == 0) != BWD) {                    // columns walked from the left
                HStream<T, CS, false, LOCAL, LOGITS, BWD, SAVE> hs; hs.init(p, mailbox, a.parts, b, c, wave, lane);
                hs.use_staging(stage + wave * HS::STAGE_BYTES, lane);
                if (wrote) hs.template run<true>(); else hs.template run<false>();
            } else {
                HStream<T, CS, true, LOCAL, LOGITS, BWD, SAVE> hs; hs.init(p, mailbox, a.parts, b, c, wave, lane);
                hs.use_staging(stage + wave * HS::STAGE_BYTES, lane);
                if (wrote) hs.template run<true>(); else hs.template run<false>();
            }
        } else {
            for (int st = 0; st < W; ++st) lds_barrier();    // idle wave: keep the barrier count
        }
        wrote = true;
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
struct StreamPlan { bool ok; int v, parts, nwaves; };

static StreamPlan plan_stream(const FwdParams& p, int dtype) {
    StreamPlan t = {};
    if (p.xt) return t;                                    // transposed-horizontal layout: tile and generic kernels
    if (p.W % 64 || p.H % 64) return t;
    const int v = p.W / 64;
    if (dtype != 0 && !(v == 4 || v == 8 || v == 16)) return t;
    if (dtype == 0 && !(v == 4 || v == 8)) return t;
    const int parts = p.H / 64;
    if (parts < 1 || parts > 8) return t;
    const int es = dtype == 0 ? 4 : 2;
    if ((size_t)p.H * p.W * es >= (1ull << 31)) return t;
    if ((size_t)p.B * p.C > 0x7fffffffull) return t;
    t.v = v; t.parts = parts; t.nwaves = parts > 2 ? parts : 2;
    t.ok = true;
    return t;
}

template <typename T, int V, int CS, int PF>
static hipError_t launch_stream(const StreamArgs& a, hipStream_t s) {
    const dim3 grid((unsigned)((size_t)a.p.B * a.p.C)), block(64 * a.nwaves);
    if (a.p.hs) {
        if (a.p.logits) hipLaunchKernelGGL((fwd_stream_kernel<T, V, CS, PF, true, true, false, true>), grid, block, 0, s, a);
        else if (a.p.kchunk > 0) hipLaunchKernelGGL((fwd_stream_kernel<T, V, CS, PF, true, false, false, true>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((fwd_stream_kernel<T, V, CS, PF, false, false, false, true>), grid, block, 0, s, a);
    }
    else if (a.p.logits) hipLaunchKernelGGL((fwd_stream_kernel<T, V, CS, PF, true, true>), grid, block, 0, s, a);
    else if (a.p.kchunk > 0) hipLaunchKernelGGL((fwd_stream_kernel<T, V, CS, PF, true, false>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((fwd_stream_kernel<T, V, CS, PF, false, false>), grid, block, 0, s, a);
    return hipGetLastError();
}

template <typename T, int V, int CS, int PF>
static hipError_t launch_stream_reverse(const StreamArgs& a, hipStream_t s) {
    const dim3 grid((unsigned)((size_t)a.p.B * a.p.C)), block(64 * a.nwaves);
    if (a.p.logits) hipLaunchKernelGGL((fwd_stream_kernel<T, V, CS, PF, true, true, true>), grid, block, 0, s, a);
    else if (a.p.kchunk > 0) hipLaunchKernelGGL((fwd_stream_kernel<T, V, CS, PF, true, false, true>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((fwd_stream_kernel<T, V, CS, PF, false, false, true>), grid, block, 0, s, a);
    return hipGetLastError();
}

// One translation unit per storage type.  REVERSE: first pass of the two-pass backward scan on maps beyond the tile
// kernels (p holds gy as x, u as lam, lam as u, gx as y and the buffer that receives e as hs).
template <typename T, bool REVERSE>
static hipError_t launch_stream_part(const FwdParams& p, hipStream_t s) {
    constexpr bool F32 = sizeof(T) == 4;
    const StreamPlan t = plan_stream(p, F32 ? 0 : 1);
    if (!t.ok || (REVERSE && !p.hs)) return hipErrorInvalidValue;
    StreamArgs a;
    a.p = p; a.parts = t.parts; a.nwaves = t.nwaves;
    if constexpr (F32) {
        if (t.v == 4) return REVERSE ? launch_stream_reverse<T, 4, 32, 4>(a, s) : launch_stream<T, 4, 32, 4>(a, s);
        return REVERSE ? launch_stream_reverse<T, 8, 32, 2>(a, s) : launch_stream<T, 8, 32, 2>(a, s);
    } else {
        if (t.v == 4) return REVERSE ? launch_stream_reverse<T, 4, 64, 4>(a, s) : launch_stream<T, 4, 64, 4>(a, s);
        if (t.v == 8) return REVERSE ? launch_stream_reverse<T, 8, 64, 4>(a, s) : launch_stream<T, 8, 64, 4>(a, s);
        return REVERSE ? launch_stream_reverse<T, 16, 64, 2>(a, s) : launch_stream<T, 16, 64, 2>(a, s);
    }
}

}  // namespace gspn
