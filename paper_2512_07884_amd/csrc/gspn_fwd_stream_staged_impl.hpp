// Forward GSPN scan for maps in 16-bit storage (T = bf16_t or f16_t) too large for an on-chip output tile (512x512, 256x1024; H and W multiples of 64, at
// most 512 rows): the stream kernel of gspn_fwd_stream_impl.hpp with its horizontal phases rebuilt around whole-line
// requests.  One workgroup per (image, channel) plane, all directions inside one launch (Sec. 4.1), the merged output
// y = sum_d u_d h_d (Eq. 2) accumulated in place in global memory by the workgroup that owns the plane.
//
//  * Vertical pair: as in the stream kernel (one wave per direction, a whole image row per wave, PF rows in flight).
//  * Horizontal directions (a scan step is an image column): a wave owns 64 image rows, one row per lane; the waves of a
//    column run in lock step (one LDS-only barrier per scan step, edge rows through a two-slot LDS mailbox).  A chunk is
//    64 scan steps of the six tensors in registers.  It is requested so that eight lanes share a row (each request
//    covers eight whole 128-byte lines, each line is asked for once: one row per lane would touch 64 lines per
//    request, and rows of 1 KB put them all into a few sets of the vector cache) and is turned into the row-per-lane
//    order through a 9 KB LDS block of the wave's own.  When the columns 8q..8q+7 of a chunk have been consumed their
//    registers take instruction q of the next chunk, so the next chunk arrives while this one is worked on.
//  * The chunk of y a wave adds to sits in a second LDS block of its own: it arrives and leaves in whole lines and is
//    updated in place, two columns per word, as the scan steps produce them (one rounding to storage per direction).
//  * Maps of at most 256 rows with an even number of chunks run both horizontal directions at the same time, each on
//    the half of the columns the other one is not working on.
//  * SAVE stores the hidden states per direction (h_save); BWD is the reverse sweep of the two-pass backward scan on the
//    same machinery (gy as x, u as lam, lam as u, gx as y, e into hs; see gspn_bwd_twopass.hip); LOCAL confines the
//    propagation to stretches of kchunk lines (GSPN-local, Sec. 3.2).
#pragma once
#include "gspn_fwd_stream_impl.hpp"
#include <utility>

namespace gspn {
namespace {

template <int... I, typename F> __device__ __forceinline__ void static_for_impl(std::integer_sequence<int, I...>, F& f) {
    (f(std::integral_constant<int, I>{}), ...);
}
// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>), written out by the front end (the scan steps of a
// chunk index registers)
template <int N, typename F> __device__ __forceinline__ void static_for(F f) { static_for_impl(std::make_integer_sequence<int, N>{}, f); }

constexpr int CS = 64;                            // scan steps per chunk (128 bytes per row)
constexpr int SPITCH = 9;                         // 16-byte units between two rows of an LDS block (128 bytes + 16)
constexpr int BLOCK_B = 64 * SPITCH * 16;         // 64 rows of 128 bytes
constexpr int MAILBOX_FLOATS = 2 * 8 * 4;         // [direction slot][part][side][parity]
constexpr int LDS_BYTES = 8 * 2 * BLOCK_B + MAILBOX_FLOATS * 4;

// the stretch bookkeeping of GSPN-local, or nothing at all: the global scan's instantiations carry no trace of it
template <bool ON> struct WalkIf {
    StretchWalk w;
    __device__ __forceinline__ void init(int S, int reversed, int kchunk) { w.init(S, reversed, kchunk); }
    __device__ __forceinline__ bool start() { return w.start(); }
};
template <> struct WalkIf<false> {
    __device__ __forceinline__ void init(int, int, int) {}
    __device__ __forceinline__ bool start() { return false; }
};
template <bool ON> struct WalkBackIf {
    StretchWalkBack w;
    __device__ __forceinline__ void init(int S, int reversed, int kchunk) { w.init(S, reversed, kchunk); }
    __device__ __forceinline__ bool start(bool at_step0) { return w.start(at_step0); }
};
template <> struct WalkBackIf<false> {
    __device__ __forceinline__ void init(int, int, int) {}
    __device__ __forceinline__ bool start(bool) { return false; }
};

template <int CP = 0> __device__ __forceinline__ u32x4 ld128(rsrc_t rs, uint32_t voff, int soff) {
    return __builtin_amdgcn_raw_buffer_load_b128(rs, voff, __builtin_amdgcn_readfirstlane(soff), CP);
}

// One horizontal direction for the wave that owns rows 64 * part .. of the plane.  Chunks [0, nchunks) in scan order;
// `sync_at`: chunk before which the whole workgroup meets (the two directions swap halves there; -1: never);
// `rmw_from`: first chunk (in scan order) whose y already holds a partial sum.
template <typename T, bool REV, bool SAVE, bool BWD, bool LOCAL, bool LOGITS>
__device__ __forceinline__ void horizontal_rows(const FwdParams& p, char* blk_a, char* blk_b, float* mailbox, int parts, int b, int c,
                                                int dslot, int part, int lane, int sync_at, int rmw_from) {
    constexpr int d = (REV != BWD) ? 3 : 2;
    const int H = p.H, W = p.W, HW = H * W;
    const int row_bytes = W * 2, nchunks = W / CS;
    const int g = c / p.cpg;
    const bool top_lane = lane == 0, bot_lane = lane == 63;
    const bool has_up = part > 0, has_dn = part < parts - 1;
    const bool img_first = top_lane && !has_up, img_last = bot_lane && !has_dn;
    rsrc_t xb, lb, ub, w0b, w1b, w2b, yb, hb;
    {
        const size_t planes = (size_t)p.B * p.C;
        const size_t slot_c = p.shared ? 0 : (size_t)d * planes * HW;
        const size_t slot_w = p.shared ? 0 : (size_t)d * p.B * p.G * 3 * HW;
        const size_t plane0 = ((size_t)b * p.C + c) * HW;
        const size_t plane_bytes = (size_t)HW * 2;
        const char* wbase = (const char*)p.w + (slot_w + ((size_t)b * p.G + g) * 3 * HW) * 2;
        xb = make_rsrc((const char*)p.x + plane0 * 2);
        lb = make_rsrc((const char*)p.lam + (slot_c + plane0) * 2);
        ub = make_rsrc((const char*)p.u + (slot_c + plane0) * 2);
        w0b = make_rsrc(wbase); w1b = make_rsrc(wbase + plane_bytes); w2b = make_rsrc(wbase + 2 * plane_bytes);
        yb = make_rsrc((char*)p.y + plane0 * 2);
        hb = make_rsrc(SAVE ? (char*)p.hs + ((size_t)d * planes * HW + plane0) * 2 : (char*)p.y);
    }
    // mailbox: [direction slot][part][parity] pairs (what the part above published for this part's first row, what the
    // part below published for its last row): a wave reads its own pair with one request; its last row writes into the
    // pair of the part below, its first row into the pair of the part above
    float* const task = mailbox + dslot * 8 * 4;
    const f32x2_hw* const mb_in = (const f32x2_hw*)(task + part * 4);
    float* const mb_out = bot_lane ? task + (part + 1) * 4 : task + (part - 1) * 4 + 1;
    const bool publishes = (bot_lane && has_dn) || (top_lane && has_up);
    // request order: lane -> (row l / 8 of an instruction's eight rows, bytes 16 * (l % 8) ..); instruction i: rows 8i..
    const uint32_t voff = (uint32_t)(((part * 64 + (lane >> 3)) * W + 8 * (lane & 7)) * 2);
    const int istep = 8 * row_bytes;
    // LDS blocks, rows 144 bytes apart: where this lane drops instruction 0's registers (instruction i: 8 rows further),
    // and this lane's own row
    u32x4* const wr_a = (u32x4*)blk_a + SPITCH * (lane >> 3) + (lane & 7);
    u32x4* const rd_a = (u32x4*)blk_a + SPITCH * lane;
    u32x4* const wr_b = (u32x4*)blk_b + SPITCH * (lane >> 3) + (lane & 7);
    uint32_t* const yrow = (uint32_t*)((u32x4*)blk_b + SPITCH * lane);

    uint32_t bx[32], bl[32], bu[32], b0[32], b1[32], b2[32], ty[32];
    auto col_bytes = [&](int c_) { return (REV ? nchunks - 1 - c_ : c_) * CS * 2; };
    auto issue1 = [&](rsrc_t rs, int cb, int i, uint32_t (&r)[32]) {
        const u32x4 v = ld128(rs, voff, cb + i * istep);
        r[4 * i] = v.x; r[4 * i + 1] = v.y; r[4 * i + 2] = v.z; r[4 * i + 3] = v.w;
    };
    // ... of a tensor this launch reads once (x, lam, u)
    auto issue1s = [&](rsrc_t rs, int cb, int i, uint32_t (&r)[32]) {
        const u32x4 v = ld128<CP_STREAM>(rs, voff, cb + i * istep);
        r[4 * i] = v.x; r[4 * i + 1] = v.y; r[4 * i + 2] = v.z; r[4 * i + 3] = v.w;
    };
    // instruction q of chunk c_ for the six tensors (their registers 4q..4q+3 are free at that point)
    auto issue_slot = [&](int c_, int q) {
        const int cb = col_bytes(c_);
        issue1s(xb, cb, q, bx); issue1s(lb, cb, q, bl);
        issue1(w0b, cb, q, b0); issue1(w1b, cb, q, b1); issue1(w2b, cb, q, b2);
        issue1s(ub, cb, q, bu);
    };
    auto issue_y = [&](int c_) {
        const int cb = col_bytes(c_);
#pragma unroll
        for (int i = 0; i < 8; ++i) issue1(yb, cb, i, ty);
    };
    auto to_rows = [&](uint32_t (&r)[32]) {
#pragma unroll
        for (int i = 0; i < 8; ++i) { const u32x4 v = {r[4 * i], r[4 * i + 1], r[4 * i + 2], r[4 * i + 3]}; wr_a[8 * SPITCH * i] = v; }
        __builtin_amdgcn_sched_barrier(0);     // the reads below take the registers the writes above have released
#pragma unroll
        for (int q = 0; q < 8; ++q) { const u32x4 v = rd_a[q]; r[4 * q] = v.x; r[4 * q + 1] = v.y; r[4 * q + 2] = v.z; r[4 * q + 3] = v.w; }
        __builtin_amdgcn_sched_barrier(0);
    };

    float h = 0.f, wp0 = 0.f, wp1 = 0.f, wp2 = 0.f;
    // GSPN-local (Sec. 3.2): the wave walks in the scan order of direction REV ? 3 : 2 (forward) or against that of
    // direction REV ? 2 : 3 (reverse sweep); a column that starts a stretch takes nothing from the column before it
    WalkIf<LOCAL && !BWD> walk;
    WalkBackIf<LOCAL && BWD> bwalk;
    walk.init(W, REV ? 1 : 0, p.kchunk);
    bwalk.init(W, REV ? 0 : 1, p.kchunk);
#pragma unroll
    for (int q = 0; q < 8; ++q) issue_slot(0, q);
    if (0 >= rmw_from && 0 != sync_at) issue_y(0);
    for (int ch = 0; ch < nchunks; ++ch) {
        const bool rmw = ch >= rmw_from;
        const int col0 = (REV ? nchunks - 1 - ch : ch) * CS;
        if (ch == sync_at) {
            __syncthreads();                     // every wave's stores of y are complete: the two directions swap halves
            if (rmw) issue_y(ch);                // (could not be asked for before the other direction had written it)
        }
        // the chunk of y this wave adds to: whole lines into the second block (requested while the chunk before was
        // worked on), or zeros
        if (rmw) {
#pragma unroll
            for (int i = 0; i < 8; ++i) { const u32x4 v = {ty[4 * i], ty[4 * i + 1], ty[4 * i + 2], ty[4 * i + 3]}; wr_b[8 * SPITCH * i] = v; }
        } else {
            const u32x4 z = {0, 0, 0, 0};
#pragma unroll
            for (int i = 0; i < 8; ++i) wr_b[8 * SPITCH * i] = z;
        }
        __builtin_amdgcn_sched_barrier(0);
        to_rows(bx); to_rows(bl); to_rows(b0); to_rows(b1); to_rows(b2); to_rows(bu);
        const bool y_ahead = ch + 1 < nchunks && ch + 1 >= rmw_from && ch + 1 != sync_at;

        float cpair = 0.f, hpair = 0.f;          // first element of the pair of columns that share a word
        uint32_t yw = 0;
        uint32_t hq[4];                          // SAVE: the states of the eight columns being worked on
        static_for<CS>([&](auto kc_) __attribute__((always_inline)) {
            constexpr int k = decltype(kc_)::value;
            constexpr int e = REV ? CS - 1 - k : k;
            constexpr int par = k & 1;
            const f32x2_hw pin = mb_in[par ^ 1];                 // edge states the neighbouring parts published in the previous step
            const float pu = pin.x, pd = pin.y;
            if ((k & 1) == 0) yw = yrow[e >> 1];
            const float av = elem<T>(bl, e) * elem<T>(bx, e);
            float c0 = elem<T>(b0, e), c1 = elem<T>(b1, e), c2 = elem<T>(b2, e);
            // raw logits: normalised here over the taps whose neighbour row exists (Sec. 3.2)
            if constexpr (LOGITS) softmax3(c0, c1, c2, img_first, img_last);
            if constexpr (BWD) {
                // the edge rows publish the products that cross into the neighbouring part: tap 0 of a part's first row
                // reads the row above it, tap 2 of its last row the row below
                const float q0 = wp0 * h, q2 = wp2 * h;
                float up = from_lane_below(q2), dn = from_lane_above(q0);
                up = top_lane ? (has_up ? pu : 0.f) : up;
                dn = bot_lane ? (has_dn ? pd : 0.f) : dn;
                h = fmaf(wp1, h, av) + (up + dn);
                bool starts = false;
                if constexpr (LOCAL) starts = bwalk.start(ch == nchunks - 1 && k == CS - 1);     // hands nothing on to the column swept next
                wp0 = (img_first || starts) ? 0.f : c0;
                wp1 = starts ? 0.f : c1;
                wp2 = (img_last || starts) ? 0.f : c2;
                if (publishes) mb_out[par * 2] = bot_lane ? wp2 * h : wp0 * h;
            } else {
                if (LOCAL || k == 0) {
                    bool start = ch == 0 && k == 0;              // scan step 0: its weights are never read
                    if constexpr (LOCAL) start = walk.start();      // ... nor those of a stretch's first column
                    c0 = start ? 0.f : c0; c1 = start ? 0.f : c1; c2 = start ? 0.f : c2;
                    if constexpr (LOCAL) h = start ? 0.f : h;
                }
                float up = from_lane_below(h), dn = from_lane_above(h);
                up = top_lane ? (has_up ? pu : 0.f) : up;
                dn = bot_lane ? (has_dn ? pd : 0.f) : dn;
                c0 = img_first ? 0.f : c0;
                c2 = img_last ? 0.f : c2;
                h = fmaf(c0, up, fmaf(c1, h, fmaf(c2, dn, av)));
                if (publishes) mb_out[par * 2] = h;
            }
            const float cv = elem<T>(bu, e) * h;
            if ((k & 1) == 0) { cpair = cv; hpair = h; }
            else {
                // columns e and e ^ 1 are complete: their word of y takes both
                const float clo = (e & 1) ? cpair : cv, chi = (e & 1) ? cv : cpair;
                yrow[e >> 1] = pack_word<T>(word_lo<T>(yw) + clo, word_hi<T>(yw) + chi);
                if constexpr (SAVE) hq[(e >> 1) & 3] = pack_word<T>((e & 1) ? hpair : h, (e & 1) ? h : hpair);
            }
            if constexpr (SAVE) {
                // eight columns of states are complete: they wait in the first block (idle while a chunk is worked on)
                if ((k & 7) == 7) { const u32x4 v = {hq[0], hq[1], hq[2], hq[3]}; rd_a[e >> 3] = v; }
            }
            lds_barrier();
            if ((k & 7) == 7) {
                // columns 8q..8q+7 are consumed: their registers take instruction q of the next chunk
                if (ch + 1 < nchunks) issue_slot(ch + 1, e >> 3);
                // ... and towards the end of the chunk the next chunk of y is asked for, unless the other direction is
                // still to write it
                if (k == (BWD ? 55 : 47) && y_ahead) issue_y(ch + 1);
                __builtin_amdgcn_sched_barrier(0);
            }
        });
        // the chunk of y (and of the states) leaves in whole lines
#pragma unroll
        for (int i = 0; i < 8; ++i) st_b128(yb, voff + (uint32_t)(col0 * 2 + i * istep), wr_b[8 * SPITCH * i]);
        if constexpr (SAVE) {
#pragma unroll
            for (int i = 0; i < 8; ++i) st_b128<CP_STREAM>(hb, voff + (uint32_t)(col0 * 2 + i * istep), wr_a[8 * SPITCH * i]);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// The same for TWO channels of one weight group (Sec. 4.2: they share the weights), one after the other chunk by chunk:
// a chunk of the weights is requested and turned into row order once and serves both channels' 64 scan steps.  The
// registers of x, lam, u take, as they are consumed, channel B's chunk while channel A is worked on and channel A's next
// chunk while channel B is; those of the weights take the next chunk while channel B is worked on.  y of both channels
// already holds the vertical pair's sum.  Maps of 512 rows run one direction at a time (all eight waves hold rows,
// sync_at < 0); maps of 256 rows both at once, four waves each (direction slot dslot), each first on the half of the
// columns it starts in and, after the workgroup has met before chunk sync_at, on the other half.
template <typename T, bool REV, bool SAVE, bool BWD, bool LOCAL, bool LOGITS>
__device__ __forceinline__ void horizontal_rows2(const FwdParams& p, char* blk_a, char* blk_b, float* mailbox, int parts, int b, int c,
                                                 int dslot, int part, int lane, int sync_at) {
    constexpr int d = (REV != BWD) ? 3 : 2;
    const int H = p.H, W = p.W, HW = H * W;
    const int row_bytes = W * 2, nchunks = W / CS;
    const int g = c / p.cpg;
    const bool top_lane = lane == 0, bot_lane = lane == 63;
    const bool has_up = part > 0, has_dn = part < parts - 1;
    const bool img_first = top_lane && !has_up, img_last = bot_lane && !has_dn;
    rsrc_t xb, lb, ub, yb, hb, w0b, w1b, w2b;       // channel A's planes; channel B's are the next ones in memory
    const int plane_b = HW * 2;
    {
        const size_t planes = (size_t)p.B * p.C;
        const size_t slot_c = p.shared ? 0 : (size_t)d * planes * HW;
        const size_t slot_w = p.shared ? 0 : (size_t)d * p.B * p.G * 3 * HW;
        const size_t plane0 = ((size_t)b * p.C + c) * HW;
        const size_t plane_bytes = (size_t)HW * 2;
        const char* wbase = (const char*)p.w + (slot_w + ((size_t)b * p.G + g) * 3 * HW) * 2;
        xb = make_rsrc((const char*)p.x + plane0 * 2);
        lb = make_rsrc((const char*)p.lam + (slot_c + plane0) * 2);
        ub = make_rsrc((const char*)p.u + (slot_c + plane0) * 2);
        yb = make_rsrc((char*)p.y + plane0 * 2);
        hb = make_rsrc(SAVE ? (char*)p.hs + ((size_t)d * planes * HW + plane0) * 2 : (char*)p.y);
        w0b = make_rsrc(wbase); w1b = make_rsrc(wbase + plane_bytes); w2b = make_rsrc(wbase + 2 * plane_bytes);
    }
    const uint32_t voff = (uint32_t)(((part * 64 + (lane >> 3)) * W + 8 * (lane & 7)) * 2);
    const int istep = 8 * row_bytes;
    u32x4* const wr_a = (u32x4*)blk_a + SPITCH * (lane >> 3) + (lane & 7);
    u32x4* const rd_a = (u32x4*)blk_a + SPITCH * lane;
    u32x4* const wr_b = (u32x4*)blk_b + SPITCH * (lane >> 3) + (lane & 7);
    uint32_t* const yrow = (uint32_t*)((u32x4*)blk_b + SPITCH * lane);
    const bool publishes = (bot_lane && has_dn) || (top_lane && has_up);

    uint32_t bx[32], bl[32], bu[32], b0[32], b1[32], b2[32], ty[32];
    auto col_bytes = [&](int c_) { return (REV ? nchunks - 1 - c_ : c_) * CS * 2; };
    auto issue1 = [&](rsrc_t rs, int cb, int i, uint32_t (&r)[32]) {
        const u32x4 v = ld128(rs, voff, cb + i * istep);
        r[4 * i] = v.x; r[4 * i + 1] = v.y; r[4 * i + 2] = v.z; r[4 * i + 3] = v.w;
    };
    // ... of a tensor this launch reads once (x, lam, u)
    auto issue1s = [&](rsrc_t rs, int cb, int i, uint32_t (&r)[32]) {
        const u32x4 v = ld128<CP_STREAM>(rs, voff, cb + i * istep);
        r[4 * i] = v.x; r[4 * i + 1] = v.y; r[4 * i + 2] = v.z; r[4 * i + 3] = v.w;
    };
    // chan: 0 = channel A, 1 = channel B
    auto issue_own = [&](int chan, int c_, int q) {
        const int cb = col_bytes(c_) + chan * plane_b;
        issue1s(xb, cb, q, bx); issue1s(lb, cb, q, bl); issue1s(ub, cb, q, bu);
    };
    auto issue_w = [&](int c_, int q) {
        const int cb = col_bytes(c_);
        issue1(w0b, cb, q, b0); issue1(w1b, cb, q, b1); issue1(w2b, cb, q, b2);
    };
    auto issue_y = [&](int chan, int c_) {
        const int cb = col_bytes(c_) + chan * plane_b;
#pragma unroll
        for (int i = 0; i < 8; ++i) issue1(yb, cb, i, ty);
    };
    auto to_rows = [&](uint32_t (&r)[32]) {
#pragma unroll
        for (int i = 0; i < 8; ++i) { const u32x4 v = {r[4 * i], r[4 * i + 1], r[4 * i + 2], r[4 * i + 3]}; wr_a[8 * SPITCH * i] = v; }
        __builtin_amdgcn_sched_barrier(0);     // the reads below take the registers the writes above have released
#pragma unroll
        for (int q = 0; q < 8; ++q) { const u32x4 v = rd_a[q]; r[4 * q] = v.x; r[4 * q + 1] = v.y; r[4 * q + 2] = v.z; r[4 * q + 3] = v.w; }
        __builtin_amdgcn_sched_barrier(0);
    };

    // GSPN-local: the two channels take the same 64 steps of a chunk, so both start from the walk's state at the chunk's
    // first step, and the state after them is kept once channel B is through
    WalkIf<LOCAL && !BWD> walk;
    WalkBackIf<LOCAL && BWD> bwalk;
    walk.init(W, REV ? 1 : 0, p.kchunk);
    bwalk.init(W, REV ? 0 : 1, p.kchunk);
    float hA = 0.f, hB = 0.f;
    float wpA0 = 0.f, wpA1 = 0.f, wpA2 = 0.f, wpB0 = 0.f, wpB1 = 0.f, wpB2 = 0.f;     // BWD: taps of the column swept before, per channel

    // the 64 scan steps of one channel (second: channel B, uniform over the workgroup) on chunk ch
    auto steps = [&](const bool second, int ch) __attribute__((always_inline)) {
        float h = second ? hB : hA;
        float wp0 = second ? wpB0 : wpA0, wp1 = second ? wpB1 : wpA1, wp2 = second ? wpB2 : wpA2;
        auto wk = walk;
        auto bwk = bwalk;
        // mailbox: [channel][part][parity] pairs, as in horizontal_rows
        float* const task = mailbox + (dslot * 2 + (second ? 1 : 0)) * parts * 4;
        const f32x2_hw* const mb_in = (const f32x2_hw*)(task + part * 4);
        float* const mb_out = bot_lane ? task + (part + 1) * 4 : task + (part - 1) * 4 + 1;
        // what the registers of x, lam, u take as they are consumed: channel B's same chunk, or channel A's next one
        const int next_chan = second ? 0 : 1, next_chunk = second ? ch + 1 : ch;
        const bool more = next_chunk < nchunks;
        float cpair = 0.f, hpair = 0.f;          // first element of the pair of columns that share a word
        uint32_t yw = 0;
        uint32_t hq[4];                          // SAVE: the states of the eight columns being worked on
        static_for<CS>([&](auto kc_) __attribute__((always_inline)) {
            constexpr int k = decltype(kc_)::value;
            constexpr int e = REV ? CS - 1 - k : k;
            constexpr int par = k & 1;
            const f32x2_hw pin = mb_in[par ^ 1];                 // edge states the neighbouring parts published in the previous step
            const float pu = pin.x, pd = pin.y;
            if ((k & 1) == 0) yw = yrow[e >> 1];
            const float av = elem<T>(bl, e) * elem<T>(bx, e);
            float c0 = elem<T>(b0, e), c1 = elem<T>(b1, e), c2 = elem<T>(b2, e);
            // raw logits: normalised here over the taps whose neighbour row exists (Sec. 3.2)
            if constexpr (LOGITS) softmax3(c0, c1, c2, img_first, img_last);
            if constexpr (BWD) {
                const float q0 = wp0 * h, q2 = wp2 * h;
                float up = from_lane_below(q2), dn = from_lane_above(q0);
                up = top_lane ? (has_up ? pu : 0.f) : up;
                dn = bot_lane ? (has_dn ? pd : 0.f) : dn;
                h = fmaf(wp1, h, av) + (up + dn);
                bool starts = false;
                if constexpr (LOCAL) starts = bwk.start(ch == nchunks - 1 && k == CS - 1);     // hands nothing on to the column swept next
                wp0 = (img_first || starts) ? 0.f : c0;
                wp1 = starts ? 0.f : c1;
                wp2 = (img_last || starts) ? 0.f : c2;
                if (publishes) mb_out[par * 2] = bot_lane ? wp2 * h : wp0 * h;
            } else {
                if (LOCAL || k == 0) {
                    bool start = ch == 0 && k == 0;              // scan step 0: its weights are never read
                    if constexpr (LOCAL) start = wk.start();      // ... nor those of a stretch's first column
                    c0 = start ? 0.f : c0; c1 = start ? 0.f : c1; c2 = start ? 0.f : c2;
                    if constexpr (LOCAL) h = start ? 0.f : h;
                }
                float up = from_lane_below(h), dn = from_lane_above(h);
                up = top_lane ? (has_up ? pu : 0.f) : up;
                dn = bot_lane ? (has_dn ? pd : 0.f) : dn;
                c0 = img_first ? 0.f : c0;
                c2 = img_last ? 0.f : c2;
                h = fmaf(c0, up, fmaf(c1, h, fmaf(c2, dn, av)));
                if (publishes) mb_out[par * 2] = h;
            }
            const float cv = elem<T>(bu, e) * h;
            if ((k & 1) == 0) { cpair = cv; hpair = h; }
            else {
                const float clo = (e & 1) ? cpair : cv, chi = (e & 1) ? cv : cpair;
                yrow[e >> 1] = pack_word<T>(word_lo<T>(yw) + clo, word_hi<T>(yw) + chi);
                if constexpr (SAVE) hq[(e >> 1) & 3] = pack_word<T>((e & 1) ? hpair : h, (e & 1) ? h : hpair);
            }
            if constexpr (SAVE) {
                if ((k & 7) == 7) { const u32x4 v = {hq[0], hq[1], hq[2], hq[3]}; rd_a[e >> 3] = v; }
            }
            lds_barrier();
            if ((k & 7) == 7) {
                // columns 8q..8q+7 are consumed: the registers of x, lam, u take instruction q of the other channel's chunk,
                // those of the weights, once channel B is done with them, instruction q of the next chunk
                if (more) issue_own(next_chan, next_chunk, e >> 3);
                if (second && more) issue_w(next_chunk, e >> 3);
                // (channel A's next chunk of y cannot be asked for while the other direction is still to write it)
                if (k == (BWD ? 55 : 47) && more && !(second && next_chunk == sync_at)) issue_y(next_chan, next_chunk);
                __builtin_amdgcn_sched_barrier(0);
            }
        });
        if (second) { hB = h; wpB0 = wp0; wpB1 = wp1; wpB2 = wp2; walk = wk; bwalk = bwk; }
        else { hA = h; wpA0 = wp0; wpA1 = wp1; wpA2 = wp2; }
    };
    auto y_to_block = [&]() {
#pragma unroll
        for (int i = 0; i < 8; ++i) { const u32x4 v = {ty[4 * i], ty[4 * i + 1], ty[4 * i + 2], ty[4 * i + 3]}; wr_b[8 * SPITCH * i] = v; }
        __builtin_amdgcn_sched_barrier(0);
    };
    auto store_chunk = [&](int chan, int col0) {
        const uint32_t at = voff + (uint32_t)(col0 * 2 + chan * plane_b);
#pragma unroll
        for (int i = 0; i < 8; ++i) st_b128(yb, at + (uint32_t)(i * istep), wr_b[8 * SPITCH * i]);
        if constexpr (SAVE) {
#pragma unroll
            for (int i = 0; i < 8; ++i) st_b128<CP_STREAM>(hb, at + (uint32_t)(i * istep), wr_a[8 * SPITCH * i]);
        }
        __builtin_amdgcn_sched_barrier(0);
    };

#pragma unroll
    for (int q = 0; q < 8; ++q) { issue_own(0, 0, q); issue_w(0, q); }
    issue_y(0, 0);
    for (int ch = 0; ch < nchunks; ++ch) {
        const int col0 = (REV ? nchunks - 1 - ch : ch) * CS;
        for (int chan = 0; chan < 2; ++chan) {
            if (chan == 0 && ch == sync_at) {
                __syncthreads();                 // every wave's stores of y are complete: the two directions swap halves
                issue_y(0, ch);
            }
            y_to_block();
            to_rows(bx); to_rows(bl);
            if (chan == 0) { to_rows(b0); to_rows(b1); to_rows(b2); }      // channel B: the weights are in row order already
            to_rows(bu);
            steps(chan == 1, ch);
            store_chunk(chan, col0);
        }
    }
}

template <typename T, int V, int PF, bool SAVE, bool BWD, bool LOCAL, bool LOGITS>
__global__ void __launch_bounds__(512) fwd_stream_staged_kernel(StreamArgs a) {
    extern __shared__ char lds[];
    float* mailbox = (float*)(lds + 8 * 2 * BLOCK_B);
    const FwdParams& p = a.p;
    const int H = p.H, W = p.W;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const unsigned item = xcd_contiguous_item(blockIdx.x, gridDim.x);
    const int b = item / p.C, c = item - b * p.C;
    bool wrote = false;          // does y already hold a partial sum?  (uniform over the workgroup)

    // ---- vertical pair (waves 0 and 1): each wave first stores its half of y, then adds to the other half
    {
        const int has_tb = (p.mask >> 0) & 1, has_bt = (p.mask >> 1) & 1;
        const int nd = has_tb + has_bt;
        if (nd == 2) {
            const int split = (H + 1) / 2;
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

    // ---- horizontal directions
    const int has_lr = (p.mask >> 2) & 1, has_rl = (p.mask >> 3) & 1;
    const int nchunks = W / CS;
    const int parts = a.parts;
    char* const blk_a = lds + wave * 2 * BLOCK_B;
    char* const blk_b = blk_a + BLOCK_B;
    const int never = 1 << 30;
    if (has_lr && has_rl && 2 * parts <= 8 && nchunks % 2 == 0) {
        // both at once: wave -> (direction slot, part); each direction first works on the half of the columns it
        // starts in, then, after the workgroup has met, on the other half (which then holds a partial sum)
        if (threadIdx.x < MAILBOX_FLOATS) mailbox[threadIdx.x] = 0.f;
        __syncthreads();                        // y of the vertical pair complete, mailbox cleared
        const int dslot = wave / parts, part = wave - dslot * parts;
        const int rmw_from = wrote ? 0 : nchunks / 2;
        if (wave >= 2 * parts) {
            for (int ch = 0; ch < nchunks; ++ch) {
                if (ch == nchunks / 2) __syncthreads();
                for (int st = 0; st < CS; ++st) lds_barrier();      // idle wave: keep the barrier count
            }
        } else if ((dslot == 0) != BWD) {
            horizontal_rows<T, false, SAVE, BWD, LOCAL, LOGITS>(p, blk_a, blk_b, mailbox, parts, b, c, dslot, part, lane, nchunks / 2, rmw_from);
        } else {
            horizontal_rows<T, true, SAVE, BWD, LOCAL, LOGITS>(p, blk_a, blk_b, mailbox, parts, b, c, dslot, part, lane, nchunks / 2, rmw_from);
        }
    } else {
        // one after the other; waves 0..parts-1 hold the rows
        for (int dsel = 0; dsel < 2; ++dsel) {
            if (!((p.mask >> (2 + dsel)) & 1)) continue;
            if (threadIdx.x < MAILBOX_FLOATS) mailbox[threadIdx.x] = 0.f;
            __syncthreads();                    // y of the previous phase complete, mailbox cleared
            const int rmw_from = wrote ? 0 : never;
            if (wave >= parts) {
                for (int st = 0; st < W; ++st) lds_barrier();       // idle wave: keep the barrier count
            } else if ((dsel == 0) != BWD) {
                horizontal_rows<T, false, SAVE, BWD, LOCAL, LOGITS>(p, blk_a, blk_b, mailbox, parts, b, c, 0, wave, lane, never, rmw_from);
            } else {
                horizontal_rows<T, true, SAVE, BWD, LOCAL, LOGITS>(p, blk_a, blk_b, mailbox, parts, b, c, 0, wave, lane, never, rmw_from);
            }
            wrote = true;
        }
    }
}

// Two channels of a weight group per workgroup on maps of 512 or 256 rows, all four directions: the vertical pairs of both
// channels at the same time (waves 0, 1 and 2, 3), then the horizontal directions one after the other with the weights
// shared (horizontal_rows2).
template <typename T, int V, int PF, bool SAVE, bool BWD, bool LOCAL, bool LOGITS>
__global__ void __launch_bounds__(512) fwd_stream_staged2_kernel(StreamArgs a) {
    extern __shared__ char lds[];
    float* mailbox = (float*)(lds + 8 * 2 * BLOCK_B);
    const FwdParams& p = a.p;
    const int H = p.H;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const unsigned item = xcd_contiguous_item(blockIdx.x, gridDim.x);
    const int pairs = p.C / 2;
    const int b = item / pairs, c = (item - b * pairs) * 2;

    // ---- vertical pairs: each wave first stores its half of its channel's y, then adds to the other half
    {
        const int split = (H + 1) / 2;
        const int cv = c + (wave >> 1);
        if (wave < 4 && (wave & 1) == 0) {
            VStream<T, V, PF, false, LOCAL, LOGITS, BWD, SAVE> v; v.init(p, b, cv, lane);
            v.template run<false>(0, split);
            __syncthreads();
            v.template run<true>(split, H);
        } else if (wave < 4) {
            VStream<T, V, PF, true, LOCAL, LOGITS, BWD, SAVE> v; v.init(p, b, cv, lane);
            v.template run<false>(0, H - split);
            __syncthreads();
            v.template run<true>(H - split, H);
        } else {
            __syncthreads();
        }
    }

    // ---- horizontal directions, one after the other; wave = part
    char* const blk_a = lds + wave * 2 * BLOCK_B;
    char* const blk_b = blk_a + BLOCK_B;
    if (a.parts == 8) {
        for (int dsel = 0; dsel < 2; ++dsel) {
            if (threadIdx.x < MAILBOX_FLOATS) mailbox[threadIdx.x] = 0.f;
            __syncthreads();                    // y of the previous phase complete, mailbox cleared
            if ((dsel == 0) != BWD) horizontal_rows2<T, false, SAVE, BWD, LOCAL, LOGITS>(p, blk_a, blk_b, mailbox, 8, b, c, 0, wave, lane, -1);
            else horizontal_rows2<T, true, SAVE, BWD, LOCAL, LOGITS>(p, blk_a, blk_b, mailbox, 8, b, c, 0, wave, lane, -1);
        }
    } else {
        // 256 rows: both directions at once, wave -> (direction slot, part)
        if (threadIdx.x < MAILBOX_FLOATS) mailbox[threadIdx.x] = 0.f;
        __syncthreads();                        // y of the vertical pair complete, mailbox cleared
        const int nchunks = p.W / CS;
        const int dslot = wave >> 2, part = wave & 3;
        if ((dslot == 0) != BWD) horizontal_rows2<T, false, SAVE, BWD, LOCAL, LOGITS>(p, blk_a, blk_b, mailbox, 4, b, c, dslot, part, lane, nchunks / 2);
        else horizontal_rows2<T, true, SAVE, BWD, LOCAL, LOGITS>(p, blk_a, blk_b, mailbox, 4, b, c, dslot, part, lane, nchunks / 2);
    }
}

template <typename T, int V, int PF, bool LOCAL, bool LOGITS>
static hipError_t launch_staged(const StreamArgs& a, bool reverse, hipStream_t s) {
    const dim3 grid((unsigned)((size_t)a.p.B * a.p.C)), block(512);
    const void* k = reverse ? (const void*)fwd_stream_staged_kernel<T, V, PF, true, true, LOCAL, LOGITS>
                  : a.p.hs  ? (const void*)fwd_stream_staged_kernel<T, V, PF, true, false, LOCAL, LOGITS>
                            : (const void*)fwd_stream_staged_kernel<T, V, PF, false, false, LOCAL, LOGITS>;
    hipError_t e = allow_dynamic_lds(k, LDS_BYTES);
    if (e != hipSuccess) return e;
    if (reverse) hipLaunchKernelGGL((fwd_stream_staged_kernel<T, V, PF, true, true, LOCAL, LOGITS>), grid, block, LDS_BYTES, s, a);
    else if (a.p.hs) hipLaunchKernelGGL((fwd_stream_staged_kernel<T, V, PF, true, false, LOCAL, LOGITS>), grid, block, LDS_BYTES, s, a);
    else hipLaunchKernelGGL((fwd_stream_staged_kernel<T, V, PF, false, false, LOCAL, LOGITS>), grid, block, LDS_BYTES, s, a);
    return hipGetLastError();
}

}  // namespace

template <typename T, int V, int PF, bool LOCAL, bool LOGITS>
static hipError_t launch_staged2(const StreamArgs& a, bool reverse, hipStream_t s) {
    const dim3 grid((unsigned)((size_t)a.p.B * (a.p.C / 2))), block(512);
    const void* k = reverse ? (const void*)fwd_stream_staged2_kernel<T, V, PF, true, true, LOCAL, LOGITS>
                  : a.p.hs  ? (const void*)fwd_stream_staged2_kernel<T, V, PF, true, false, LOCAL, LOGITS>
                            : (const void*)fwd_stream_staged2_kernel<T, V, PF, false, false, LOCAL, LOGITS>;
    hipError_t e = allow_dynamic_lds(k, LDS_BYTES);
    if (e != hipSuccess) return e;
    if (reverse) hipLaunchKernelGGL((fwd_stream_staged2_kernel<T, V, PF, true, true, LOCAL, LOGITS>), grid, block, LDS_BYTES, s, a);
    else if (a.p.hs) hipLaunchKernelGGL((fwd_stream_staged2_kernel<T, V, PF, true, false, LOCAL, LOGITS>), grid, block, LDS_BYTES, s, a);
    else hipLaunchKernelGGL((fwd_stream_staged2_kernel<T, V, PF, false, false, LOCAL, LOGITS>), grid, block, LDS_BYTES, s, a);
    return hipGetLastError();
}

// two channels of a group per workgroup: maps of 512 or 256 rows, all four directions, an even number of channels per
// group -- and more planes than the chip has compute units: a compute unit holds one workgroup of these kernels, so with
// fewer planes the pairing would leave half of the units it could fill idle (measured, one image of 512x512 in bf16:
// 128 channels 0.784 ms paired / 0.455 ms one channel per workgroup, 256 channels 0.822 / 0.504 ms, 512 channels
// 0.965 / 1.058 ms)
constexpr size_t CHIP_CUS = 256;
static bool two_channels_ok(const FwdParams& p, const StreamPlan& t) {
    const bool rows_ok = t.parts == 8 || (t.parts == 4 && (p.W / CS) % 2 == 0);
    return stream_two_channels_enabled() && rows_ok && p.mask == 15u && p.cpg % 2 == 0 && p.C % 2 == 0 &&
           ((size_t)p.B * p.C > CHIP_CUS || stream_two_channels_forced());
}

// 16-bit storage, every shape the stream plan takes
static bool staged_shape_ok(const FwdParams& p, int dtype) {
    return dtype != 0 && plan_stream(p, dtype).ok;
}

template <typename T, bool LOCAL, bool LOGITS = false>
static hipError_t launch_stream_staged_family(const FwdParams& p, bool reverse, hipStream_t s) {
    const StreamPlan t = plan_stream(p, 1);
    if (!t.ok || !staged_shape_ok(p, 1) || (reverse && !p.hs)) return hipErrorInvalidValue;
    StreamArgs a;
    a.p = p; a.parts = t.parts; a.nwaves = 8;
    if (two_channels_ok(p, t)) {
        if (t.v == 4) return launch_staged2<T, 4, 4, LOCAL, LOGITS>(a, reverse, s);
        if (t.v == 8) return launch_staged2<T, 8, 4, LOCAL, LOGITS>(a, reverse, s);
        return launch_staged2<T, 16, 2, LOCAL, LOGITS>(a, reverse, s);
    }
    if (t.v == 4) return launch_staged<T, 4, 4, LOCAL, LOGITS>(a, reverse, s);
    if (t.v == 8) return launch_staged<T, 8, 4, LOCAL, LOGITS>(a, reverse, s);
    return launch_staged<T, 16, 2, LOCAL, LOGITS>(a, reverse, s);
}

}  // namespace gspn
