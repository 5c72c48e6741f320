// Forward GSPN scan for 128x128 maps in 16-bit storage (T = bf16_t or f16_t) whose weight groups hold an even number of channels (the
// diffusion-latent shape): one workgroup of four waves owns TWO channels of one weight group and runs the four
// directions of Sec. 3.2 over them inside one launch (Sec. 4.1), built around how few bytes a compute unit can pull
// through its vector cache per unit time and around a register file of 512 registers per lane for a single wave:
//
//  * Vertical pair (rows are contiguous in memory): one wave per (channel, walk) runs the recurrence of Eq. 1 down or up
//    the rows, two columns per lane, neighbours by DPP.  It requests the rows of its own x, lam, u itself (256
//    contiguous bytes per request, four bands of four rows in flight); the weights of a walk serve both channels
//    (Sec. 4.2: the channels of a group share them), so its two waves request half of a band's weight rows each and
//    hand them to each other through a small LDS ring.  One barrier per band.
//  * Horizontal pair (a scan step is an image column): one wave per (channel, direction) holds all 128 image rows, two
//    adjacent rows per lane, so the three-neighbour read of Eq. 1 is two DPP shifts and in-lane moves and no wave
//    ever waits for another inside a chunk.  A chunk is 64 scan steps of the six tensors (12 x 32 registers per lane).
//    It is requested so that eight lanes share a row (each request covers eight whole 128-byte lines, each line is
//    asked for once) and turned into the row-per-lane order through an 18 KB LDS block of the wave's own.
//  * The merged output y = sum_d u_d h_d (Eq. 2) is accumulated in LDS, one 32 KB tile per channel in storage
//    precision (a 32-bit word holds two adjacent columns; even rows fill the first half of a tile, odd rows the
//    second, rows 65 words apart, so that the row-wise and the column-wise walk are both bank-conflict free), and copied
//    out once at the end.  The running sum is therefore rounded to storage after each of the four additions an element
//    receives (bf16: at most 4 * 2^-8 of the largest partial sum in the worst case, about 5e-3 of max|y| observed), which
//    is what frees the LDS for the staging above.
//  * The launch has one workgroup per compute unit (its LDS holds one); a workgroup works through its share of the
//    channel pairs and has the first requests of the next pair on their way before the current one is finished.
//  * SAVE stores the hidden states per direction (h_save); BWD is the reverse sweep of the two-pass backward scan on the
//    same machinery (gy as x, u as lam, lam as u, gx as y, e into hs; see gspn_bwd_twopass.hip); LOCAL confines the
//    propagation to stretches of kchunk lines (GSPN-local, Sec. 3.2); LOGITS takes the weights as raw logits.
#pragma once
#include "gspn_tile_common.hpp"
#include <utility>

namespace gspn {
namespace {

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>), written out by the front end: the scan steps of a chunk
// index registers, so they must be distinct code whatever the optimiser's unrolling limits say
template <int... I, typename F> __device__ __forceinline__ void static_for_impl(std::integer_sequence<int, I...>, F& f) {
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F> __device__ __forceinline__ void static_for(F f) { static_for_impl(std::make_integer_sequence<int, N>{}, f); }

constexpr int PH = 128, PW = 128;                 // rows, columns
constexpr int HW = PH * PW;
constexpr int ROW_B = PW * 2;                     // bytes per image row
constexpr int PLANE_B = HW * 2;
constexpr int TPITCH = PW / 2 + 1;                // words between two rows of an output tile (odd: see above)
constexpr int TILE_WORDS = PH * TPITCH;           // one channel's output tile, two columns per word
constexpr int VBAND = 4;                          // rows per band of the vertical pair
constexpr int VNBANDS = PH / VBAND;
constexpr int VPF = 4;                            // bands of a chain's own tensors in flight
constexpr int VSLOT_B = 2 * 3 * VBAND * ROW_B;    // weight ring slot: three taps of two walks, one band
constexpr int SPITCH = 9;                         // 16-byte units between two rows of a staging block (128 bytes + 16)
constexpr int STAGE_B = PH * SPITCH * 16;         // horizontal pair: 128 rows of 128 bytes per wave
constexpr int REGION_B = 2 * VSLOT_B > 4 * STAGE_B ? 2 * VSLOT_B : 4 * STAGE_B;
constexpr int CS = 64;                            // scan steps per chunk of the horizontal pair (128 bytes per row)
constexpr int LDS_BYTES = 2 * TILE_WORDS * 4 + REGION_B;
constexpr size_t PERSIST_WGS = 256;               // compute units of the chip this is written for

template <int CP = 0> __device__ __forceinline__ u32x4 ld128(rsrc_t rs, uint32_t voff, int soff) {
    return __builtin_amdgcn_raw_buffer_load_b128(rs, voff, __builtin_amdgcn_readfirstlane(soff), CP);
}
// where image row r sits in an output tile (in rows of TPITCH words)
__device__ __forceinline__ int tile_row(int r) { return (r >> 1) + (PH / 2) * (r & 1); }

// ---------------------------------------------------------------------------
// vertical pair: one wave = the chain of one (channel, walk), two columns per lane
// ---------------------------------------------------------------------------
// The wave requests the rows of its own x, lam, u itself, one 4-byte-per-lane request per row (256 contiguous bytes:
// two whole lines), VPF bands of VBAND rows ahead in registers.  The three weight planes of a walk serve both channels
// (Sec. 4.2): the two waves of a walk request half of a band's rows each and hand them to each other through an LDS
// ring of two slots (slot = [walk][tap][VBAND rows] of 256 bytes), one workgroup barrier per band.  A walk's first 64
// rows are rows of the output tile nobody has touched yet; its last 64 hold what the opposite walk of the same channel
// left there more than a band ago.
// ahead() is called once, V_AHEAD bands before the end (the wave's own requests for what comes next).
// The tensors of one chain behind buffer resources.
struct ChainRefs { rsrc_t xb, lb, ub, w0b, w1b, w2b, hb; };
template <bool UP, bool SAVE, bool BWD>
__device__ __forceinline__ ChainRefs chain_refs(const FwdParams& p, int b, int c) {
    constexpr int d = BWD ? (UP ? 0 : 1) : (UP ? 1 : 0);                      // the parameters this chain works on
    const int g = c / p.cpg;
    const size_t planes = (size_t)p.B * p.C;
    const size_t slot_c = p.shared ? 0 : (size_t)d * planes * HW;
    const size_t slot_w = p.shared ? 0 : (size_t)d * p.B * p.G * 3 * HW;
    const size_t plane0 = ((size_t)b * p.C + c) * HW;
    const char* wbase = (const char*)p.w + (slot_w + ((size_t)b * p.G + g) * 3 * HW) * 2;
    ChainRefs r;
    r.xb = make_rsrc((const char*)p.x + plane0 * 2);
    r.lb = make_rsrc((const char*)p.lam + (slot_c + plane0) * 2);
    r.ub = make_rsrc((const char*)p.u + (slot_c + plane0) * 2);
    r.w0b = make_rsrc(wbase); r.w1b = make_rsrc(wbase + PLANE_B); r.w2b = make_rsrc(wbase + 2 * PLANE_B);
    r.hb = make_rsrc(SAVE ? (char*)p.hs + ((size_t)d * planes * HW + plane0) * 2 : (char*)p.y);
    return r;
}
// image row of step k of band s
template <bool UP> __device__ __forceinline__ int chain_row(int s, int k) { return UP ? PH - 1 - (s * VBAND + k) : s * VBAND + k; }
template <int CP = 0> __device__ __forceinline__ uint32_t ld32(rsrc_t rs, uint32_t voff, int row) {
    return __builtin_amdgcn_raw_buffer_load_b32(rs, voff, __builtin_amdgcn_readfirstlane(row * ROW_B), CP);
}
// band s of the chain's own tensors
// lam and u of a direction are read by one chain only: their lines go with CP_STREAM, so that the weights, which all
// channels of the group read, stay in the L2 longer (diff128 0.194 -> 0.186 ms).  Not x, which the horizontal pair reads
// a second time 25 us later; not with h_save and not in the reverse sweep: there a backward call follows, or the
// forward call came just before, and what the 256 MB last-level cache still holds of lam and u is worth more
// (train128: forward 0.243 -> 0.231 ms but the backward call after it 0.500 -> 0.511 ms).
template <bool SAVE, bool BWD> constexpr int cp_lam_u() { return (SAVE || BWD) ? 0 : CP_STREAM; }
template <bool UP, int CP>
__device__ __forceinline__ void issue_own(const ChainRefs& t, uint32_t voff, int s, uint32_t (&x)[VBAND], uint32_t (&l)[VBAND], uint32_t (&u)[VBAND]) {
#pragma unroll
    for (int k = 0; k < VBAND; ++k) {
        const int row = chain_row<UP>(s, k);
        x[k] = ld32(t.xb, voff, row); l[k] = ld32<CP>(t.lb, voff, row); u[k] = ld32<CP>(t.ub, voff, row);
    }
}
// steps kc * VBAND/2 .. of band s: this wave's share of the weight rows
template <bool UP>
__device__ __forceinline__ void issue_w(const ChainRefs& t, uint32_t voff, int kc, int s, uint32_t (&w)[3][VBAND / 2]) {
#pragma unroll
    for (int k = 0; k < VBAND / 2; ++k) {
        const int row = chain_row<UP>(s, kc * (VBAND / 2) + k);
        w[0][k] = ld32(t.w0b, voff, row); w[1][k] = ld32(t.w1b, voff, row); w[2][k] = ld32(t.w2b, voff, row);
    }
}
// ... into the ring slot of band s: word (walk * 3 + tap) * VBAND * 64 + step * 64 + lane
template <bool UP>
__device__ __forceinline__ void drop_w(char* region, int kc, int lane, int s, const uint32_t (&w)[3][VBAND / 2]) {
    uint32_t* to = (uint32_t*)(region + (s & 1) * VSLOT_B) + ((UP ? 1 : 0) * 3) * VBAND * 64 + kc * (VBAND / 2) * 64 + lane;
#pragma unroll
    for (int k = 0; k < VBAND / 2; ++k) {
        to[k * 64] = w[0][k]; to[VBAND * 64 + k * 64] = w[1][k]; to[2 * VBAND * 64 + k * 64] = w[2][k];
    }
}

// The first requests of a chain, in the order the band loop would have made them (weights of band s + 3, then own
// tensors of band s + 4, band after band), so that the counters the compiler keeps for requests in flight look the same
// on entry to the loop as on its back edge and it waits for no more than it has to.  Touches no LDS: a workgroup calls
// it for its next pair of channels while the horizontal pair of the current one is still at work.
// FROM, TO: the requests are numbered 0..4 (own 0, weights 0, own 1, weights 1, own 2); where registers are short the
// early call makes the first of them only and the chain makes the others when it starts.
template <bool UP, bool SAVE, bool BWD, int FROM, int TO>
__device__ __forceinline__ void chain_request_first(const FwdParams& p, int b, int c, int kc, int lane,
                                                    uint32_t (&xr)[VPF][VBAND], uint32_t (&lr)[VPF][VBAND], uint32_t (&ur)[VPF][VBAND],
                                                    uint32_t (&wr)[2][3][VBAND / 2]) {
    static_assert(VPF == 4, "written out for four bands in flight");
    const ChainRefs t = chain_refs<UP, false, BWD>(p, b, c);
    const uint32_t voff = (uint32_t)(lane * 4);
    if constexpr (FROM <= 0 && 0 < TO) issue_own<UP, cp_lam_u<SAVE, BWD>()>(t, voff, 0, xr[0], lr[0], ur[0]);
    if constexpr (FROM <= 1 && 1 < TO) issue_w<UP>(t, voff, kc, 0, wr[0]);
    if constexpr (FROM <= 2 && 2 < TO) issue_own<UP, cp_lam_u<SAVE, BWD>()>(t, voff, 1, xr[1], lr[1], ur[1]);
    if constexpr (FROM <= 3 && 3 < TO) issue_w<UP>(t, voff, kc, 1, wr[1]);
    if constexpr (FROM <= 4 && 4 < TO) issue_own<UP, cp_lam_u<SAVE, BWD>()>(t, voff, 2, xr[2], lr[2], ur[2]);
}
// how many of them are made early: all five in the plain forward scan; with h_save / in the reverse sweep the
// horizontal tasks hold more registers (the states on their way out), and one or two is what fits beside them
// (with the logits normalised on the way in, the forward call with h_save has no register left for even one)
// a line is a whole wave here, so the lane shifts deliver the zeros at its ends (see line_update); the GSPN-local forward
// call with h_save in fp16 storage keeps the explicit selects: without them its register allocation went to scratch memory
template <typename T, bool SAVE, bool BWD, bool LOCAL> constexpr bool wave_line() { return !(__is_same(T, f16_t) && SAVE && !BWD && LOCAL); }

template <bool SAVE, bool BWD, bool LOGITS = false> constexpr int early_requests() { return SAVE ? (BWD ? 2 : (LOGITS ? 0 : 1)) : 5; }

// ... and the chain itself, after chain_request_first() for the same (b, c).
// ahead() is called once, V_AHEAD bands before the end (the wave's own requests for what comes next).
// LOCAL: GSPN-local (Sec. 3.2): the propagation is confined to stretches of p.kchunk scan lines; a line that starts a
// stretch takes nothing from the line before it (forward) and hands nothing on to the line swept next (reverse sweep).
// LOGITS: w holds raw logits, normalised as they are read (the three taps of a position through softmax3, a tap that points
// outside the line left out); on the LOCAL instantiations only, where a global scan is one stretch
template <typename T, bool UP, bool SAVE, bool BWD, bool LOCAL, bool LOGITS, typename F>
__device__ __forceinline__ void vertical_chain(const FwdParams& p, char* region, uint32_t* tile, int b, int c, int kc, int lane,
                                               uint32_t (&xr)[VPF][VBAND], uint32_t (&lr)[VPF][VBAND], uint32_t (&ur)[VPF][VBAND],
                                               uint32_t (&wr)[2][3][VBAND / 2], F& ahead) {
    constexpr int walk = UP ? 1 : 0;
    constexpr int V_AHEAD = VPF;
    static_assert(VNBANDS % VPF == 0 && VBAND % 2 == 0, "band loop unrolled by the ring depth; two waves share a band's weight rows");
    const bool first = lane == 0, last = lane == 63;
    const ChainRefs t = chain_refs<UP, SAVE, BWD>(p, b, c);
    const uint32_t voff = (uint32_t)(lane * 4);

    float h[2] = {0.f, 0.f};
    float wp0[2] = {0.f, 0.f}, wp1[2] = {0.f, 0.f}, wp2[2] = {0.f, 0.f};     // BWD: taps of the row swept before
    // the chain walks in the scan order of direction UP ? 1 : 0 (forward) or against that of direction UP ? 0 : 1
    StretchWalk stretch;
    StretchWalkBack bstretch;
    if constexpr (LOCAL && !BWD) stretch.init(PH, UP ? 1 : 0, p.kchunk);
    if constexpr (LOCAL && BWD) bstretch.init(PH, UP ? 0 : 1, p.kchunk);

    // one band: `slot` = its place in the own ring, `wslot` = where the weight rows of band s + 1 wait in registers
    auto band = [&](int s, int slot, int wslot, bool more_own, bool more_w) __attribute__((always_inline)) {
        if (s + 1 < VNBANDS) drop_w<UP>(region, kc, lane, s + 1, wr[wslot]);  // for the band after this one
        if (more_w) issue_w<UP>(t, voff, kc, s + 3, wr[wslot]);
        const uint32_t* cw = (const uint32_t*)(region + (s & 1) * VSLOT_B) + (walk * 3) * VBAND * 64 + lane;
        // everything the band needs from LDS is requested before its first row is worked on: the writes to the tile below
        // would otherwise fence the reads of the following rows (LDS against LDS)
        uint32_t t0[VBAND], t1[VBAND], t2[VBAND], ow[VBAND];
#pragma unroll
        for (int k = 0; k < VBAND; ++k) { t0[k] = cw[k * 64]; t1[k] = cw[VBAND * 64 + k * 64]; t2[k] = cw[2 * VBAND * 64 + k * 64]; }
        // the band's four image rows sit at fixed distances in the tile (tile_row of a multiple of four plus 0..3): one
        // address per band, the rows through constant offsets -- in the calls that save states (measured: train128
        // backward 0.469 -> 0.459 ms; the plain forward scan is 1.5 % faster with an address per row, 0.178 / 0.175 ms)
        uint32_t* const band_tile = tile + (UP ? PH / 2 - 2 - 2 * s : 2 * s) * TPITCH + lane;
        auto tile_word = [&](int k) -> uint32_t& {
            if constexpr (SAVE) return band_tile[tile_row(UP ? VBAND - 1 - k : k) * TPITCH];
            else return tile[tile_row(chain_row<UP>(s, k)) * TPITCH + lane];
        };
        if (s >= VNBANDS / 2) {
#pragma unroll
            for (int k = 0; k < VBAND; ++k) ow[k] = tile_word(k);
        } else {
#pragma unroll
            for (int k = 0; k < VBAND; ++k) ow[k] = 0;
        }
#pragma unroll
        for (int k = 0; k < VBAND; ++k) {
            const int row = chain_row<UP>(s, k);
            float c0[2] = {word_lo<T>(t0[k]), word_hi<T>(t0[k])}, c1[2] = {word_lo<T>(t1[k]), word_hi<T>(t1[k])}, c2[2] = {word_lo<T>(t2[k]), word_hi<T>(t2[k])};
            if constexpr (LOGITS) { softmax3(c0[0], c1[0], c2[0], first, false); softmax3(c0[1], c1[1], c2[1], false, last); }
            const uint32_t xw = xr[slot][k], lw = lr[slot][k], uw = ur[slot][k];
            float av[2] = {word_lo<T>(lw) * word_lo<T>(xw), word_hi<T>(lw) * word_hi<T>(xw)};
            if constexpr (BWD) {
                line_update_transposed<2, wave_line<T, SAVE, BWD, LOCAL>()>(h, av, wp0, wp1, wp2, first, last);
                bool starts = false;
                if constexpr (LOCAL) starts = bstretch.start(s == VNBANDS - 1 && k == VBAND - 1);
                // the taps this row hands on to the row swept next; a tap that points outside the line takes nothing,
                // whatever the tensor holds there
                wp0[0] = (first || starts) ? 0.f : c0[0]; wp0[1] = starts ? 0.f : c0[1];
                wp1[0] = starts ? 0.f : c1[0]; wp1[1] = starts ? 0.f : c1[1];
                wp2[0] = starts ? 0.f : c2[0]; wp2[1] = (last || starts) ? 0.f : c2[1];
            } else {
                if (LOCAL || k == 0) {
                    // scan step 0 (GSPN-local: the first line of a stretch): its weights are never read (they may hold
                    // anything) and the state before it is 0
                    bool start = s == 0 && k == 0;
                    if constexpr (LOCAL) start = stretch.start();
#pragma unroll
                    for (int v = 0; v < 2; ++v) {
                        c0[v] = start ? 0.f : c0[v]; c1[v] = start ? 0.f : c1[v]; c2[v] = start ? 0.f : c2[v];
                        if constexpr (LOCAL) h[v] = start ? 0.f : h[v];
                    }
                }
                line_update<2, wave_line<T, SAVE, BWD, LOCAL>()>(h, av, c0, c1, c2, first, last);
            }
            const float y0 = word_lo<T>(uw) * h[0], y1 = word_hi<T>(uw) * h[1];
            tile_word(k) = pack_word<T>(word_lo<T>(ow[k]) + y0, word_hi<T>(ow[k]) + y1);
            if constexpr (SAVE) {
                const uint32_t hw = pack_word<T>(h[0], h[1]);
                __builtin_amdgcn_raw_buffer_store_b32(hw, t.hb, voff, __builtin_amdgcn_readfirstlane(row * ROW_B), CP_STREAM);
            }
        }
        if (more_own) issue_own<UP, cp_lam_u<SAVE, BWD>()>(t, voff, s + VPF, xr[slot], lr[slot], ur[slot]);
        lds_barrier();
    };

    chain_request_first<UP, SAVE, BWD, early_requests<SAVE, BWD, LOGITS>(), 5>(p, b, c, kc, lane, xr, lr, ur, wr);
    // the rest of the first requests: band 0 of the weights goes to the ring (it takes the place band "s + 1" has in
    // the loop), its registers take band 2
    drop_w<UP>(region, kc, lane, 0, wr[0]);
    issue_w<UP>(t, voff, kc, 2, wr[0]);
    issue_own<UP, cp_lam_u<SAVE, BWD>()>(t, voff, 3, xr[3], lr[3], ur[3]);
    lds_barrier();
    // weight registers: band s + 1 waits in wr[(s + 1) & 1]; once dropped, the same registers take band s + 3
    for (int s0 = 0; s0 < VNBANDS - V_AHEAD; s0 += VPF) {
#pragma unroll
        for (int q = 0; q < VPF; ++q) band(s0 + q, q, (q + 1) & 1, true, s0 + q + 3 < VNBANDS);
    }
    ahead();
#pragma unroll
    for (int q = 0; q < VPF; ++q) band(VNBANDS - VPF + q, q, (q + 1) & 1, false, VNBANDS - VPF + q + 3 < VNBANDS);
}

// ---------------------------------------------------------------------------
// horizontal pair: one wave = the 128 image rows of one (channel, direction), rows 2l and 2l+1 in lane l
// ---------------------------------------------------------------------------
// A chunk of a tensor (128 rows x 128 bytes) is requested in sixteen instructions of eight rows each (lane -> row l / 8
// of the instruction, bytes 16 * (l % 8) ..), so every request covers whole lines.  The registers of a chunk are two
// arrays of 32 per tensor: in row order, array a holds row 2l + a (registers 4q..4q+3 = columns 8q..8q+7).  The turn
// from request order into row order goes through the wave's staging block, whose rows are 144 bytes apart: conflict
// free for the writers (eight lanes fill one row) and for every eight neighbouring readers.
struct ChunkIO {
    uint32_t voff;          // request order: byte offset of (row l / 8, column group l % 8) inside the plane
    u32x4* wr;              // staging: where this lane drops the registers of the instruction for rows 0..7; rows 8i..: + 8 i rows
    u32x4* rd;              // staging: this lane's two rows (the second one SPITCH units further)

    __device__ __forceinline__ void init(char* stage, int lane) {
        voff = (uint32_t)(((lane >> 3) * PW + 8 * (lane & 7)) * 2);
        wr = (u32x4*)stage + SPITCH * (lane >> 3) + (lane & 7);
        rd = (u32x4*)stage + SPITCH * 2 * lane;
    }
    // rows 8i..8i+7 of a chunk whose first column sits col_bytes into the row, into registers 4 * slot ..
    // CP: CP_STREAM for the tensors no other workgroup reads (x, lam, u)
    template <int CP = 0>
    __device__ __forceinline__ void issue1(rsrc_t rs, int col_bytes, int i, int slot, uint32_t (&r)[32]) const {
        const u32x4 v = ld128<CP>(rs, voff, col_bytes + i * 8 * ROW_B);
        r[4 * slot] = v.x; r[4 * slot + 1] = v.y; r[4 * slot + 2] = v.z; r[4 * slot + 3] = v.w;
    }
    // ... and from there to their place in a staging block
    __device__ __forceinline__ void drop1(u32x4* to, int i, int slot, const uint32_t (&r)[32]) const {
        const u32x4 v = {r[4 * slot], r[4 * slot + 1], r[4 * slot + 2], r[4 * slot + 3]};
        to[8 * SPITCH * i] = v;
    }
    __device__ __forceinline__ void read_rows(uint32_t (&r0)[32], uint32_t (&r1)[32]) const {
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const u32x4 v = rd[q], w = rd[SPITCH + q];
            r0[4 * q] = v.x; r0[4 * q + 1] = v.y; r0[4 * q + 2] = v.z; r0[4 * q + 3] = v.w;
            r1[4 * q] = w.x; r1[4 * q + 1] = w.y; r1[4 * q + 2] = w.z; r1[4 * q + 3] = w.w;
        }
    }
    __device__ __forceinline__ void write_rows(u32x4* to, const uint32_t (&r0)[32], const uint32_t (&r1)[32]) const {
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const u32x4 v = {r0[4 * q], r0[4 * q + 1], r0[4 * q + 2], r0[4 * q + 3]};
            const u32x4 w = {r1[4 * q], r1[4 * q + 1], r1[4 * q + 2], r1[4 * q + 3]};
            to[q] = v; to[SPITCH + q] = w;
        }
    }
    // ... and back, for stores that cover whole lines: the staging block holds a chunk in row order
    template <int CP = 0>
    __device__ __forceinline__ void store_staged(rsrc_t rs, int col_bytes) const {
#pragma unroll
        for (int i = 0; i < 16; ++i) st_b128<CP>(rs, voff + (uint32_t)(col_bytes + i * 8 * ROW_B), wr[8 * SPITCH * i]);
    }
};

// One workgroup's work as wave `wave` sees it: its share of the vertical pair, then its (channel, direction) task of
// the horizontal pair.  What keeps the requests of that task few and always in flight:
//  * the two channels of the workgroup share the weights: the task of channel k requests rows 64k..64k+63 of the weight
//    chunk only, and the two tasks drop what they fetched into both staging blocks on the way to the row order;
//  * when the columns 8q..8q+7 of a chunk have been consumed their registers take two instructions of the next chunk,
//    so the next chunk arrives while this one is worked on and no register is added;
//  * (without h_save) the task that walks from the left and the one that walks from the right hand each other their
//    chunk of x at half time instead of fetching it a second time;
//  * the first chunk is requested while the vertical pair is still at work.
//  * a workgroup works through several pairs of channels, and requests the first bands of the next pair's vertical
//    chains (has_next: image nb, channels nc0, nc0 + 1) before the last chunk of this pair's horizontal tasks is worked
//    on -- otherwise nothing would be on its way to the compute unit from there until the next pair's first rows arrive.
// xr, lr, ur, wr: the first bands of THIS pair's vertical chain on entry (chain_request_first), of the next pair's on exit.
template <typename T, bool REV, bool SAVE, bool BWD, bool LOCAL, bool LOGITS>
__device__ __forceinline__ void pair_body(const FwdParams& p, uint32_t* tiles, char* region, int b, int c0, int wave, int lane,
                                          bool has_next, int nb, int nc0,
                                          uint32_t (&xr)[VPF][VBAND], uint32_t (&lr)[VPF][VBAND], uint32_t (&ur)[VPF][VBAND],
                                          uint32_t (&wr)[2][3][VBAND / 2]) {
    constexpr int d = (REV != BWD) ? 3 : 2;
    constexpr bool UP = REV != BWD;            // the vertical chain of the wave: direction slot 0 walks the rows downwards
    constexpr bool SWAP_X = !SAVE;             // with h_save the staging blocks collect the states while a chunk is worked on
    const int kc = wave >> 1;                  // channel of the horizontal task; its direction slot is wave & 1
    const int twin = kc;
    const bool first = lane == 0, last = lane == 63;      // the lane holds image row 0 / row 127
    rsrc_t xb, lb, ub, w0b, w1b, w2b, hb;
    {
        const int c = c0 + kc, g = c / p.cpg;
        const size_t planes = (size_t)p.B * p.C;
        const size_t slot_c = p.shared ? 0 : (size_t)d * planes * HW;
        const size_t slot_w = p.shared ? 0 : (size_t)d * p.B * p.G * 3 * HW;
        const size_t plane0 = ((size_t)b * p.C + c) * HW;
        const char* wbase = (const char*)p.w + (slot_w + ((size_t)b * p.G + g) * 3 * HW) * 2;
        xb = make_rsrc((const char*)p.x + plane0 * 2);
        lb = make_rsrc((const char*)p.lam + (slot_c + plane0) * 2);
        ub = make_rsrc((const char*)p.u + (slot_c + plane0) * 2);
        w0b = make_rsrc(wbase); w1b = make_rsrc(wbase + PLANE_B); w2b = make_rsrc(wbase + 2 * PLANE_B);
        hb = make_rsrc(SAVE ? (char*)p.hs + ((size_t)d * planes * HW + plane0) * 2 : (char*)p.y);
    }
    // rows 2l and 2l+1 of the channel's tile
    uint32_t* const trow = tiles + kc * TILE_WORDS + lane * TPITCH;
    constexpr int TODD = (PH / 2) * TPITCH;
    ChunkIO io;
    io.init(region + wave * STAGE_B, lane);
    // the same place as io.wr in the staging block of the other channel's task; this lane's rows in the staging block of
    // the task that walks the other way
    u32x4* const wr_twin = (u32x4*)((char*)io.wr + ((wave ^ 2) - wave) * STAGE_B);
    u32x4* const rd_mirror = (u32x4*)((char*)io.rd + ((wave ^ 1) - wave) * STAGE_B);

    // the chunk: per tensor, array 0 = the lane's even row, array 1 = its odd row
    uint32_t bx0[32], bx1[32], bl0[32], bl1[32], bu0[32], bu1[32], b00[32], b01[32], b10[32], b11[32], b20[32], b21[32];
    // byte offset of chunk c_ (in scan order) inside a row
    auto col_bytes = [&](int c_) { return (REV ? 1 - c_ : c_) * CS * 2; };
    // Requests of chunk c_ into the registers 4q..4q+3 of both arrays, which are free at that point.  q is the f-th
    // set to come free; it takes instructions 2f and 2f+1 of x, lam, u; of the weights this task requests rows
    // 64 * twin + 8j .. (j = 0..7) only, two instructions into every second set (the same registers for both channels' tasks)
    auto issue_slot = [&](int c_, int q, bool with_x) {
        const int cb = col_bytes(c_);
        const int f = REV ? 7 - q : q;
        if (with_x) { io.issue1(xb, cb, 2 * f, q, bx0); io.issue1(xb, cb, 2 * f + 1, q, bx1); }
        io.issue1<cp_lam_u<SAVE, BWD>()>(lb, cb, 2 * f, q, bl0); io.issue1<cp_lam_u<SAVE, BWD>()>(lb, cb, 2 * f + 1, q, bl1);
        if ((f & 1) == 0) {
            const int i = 8 * twin + f;
            io.issue1(w0b, cb, i, q, b00); io.issue1(w0b, cb, i + 1, q, b01);
            io.issue1(w1b, cb, i, q, b10); io.issue1(w1b, cb, i + 1, q, b11);
            io.issue1(w2b, cb, i, q, b20); io.issue1(w2b, cb, i + 1, q, b21);
        }
        io.issue1<cp_lam_u<SAVE, BWD>()>(ub, cb, 2 * f, q, bu0); io.issue1<cp_lam_u<SAVE, BWD>()>(ub, cb, 2 * f + 1, q, bu1);
    };
    auto prefetch = [&]() {
#pragma unroll
        for (int q = 0; q < 8; ++q) issue_slot(0, q, true);
    };
    // a tensor of the task's own from request order to row order
    auto to_rows = [&](uint32_t (&r0)[32], uint32_t (&r1)[32]) {
#pragma unroll
        for (int f = 0; f < 8; ++f) {
            const int q = REV ? 7 - f : f;
            io.drop1(io.wr, 2 * f, q, r0); io.drop1(io.wr, 2 * f + 1, q, r1);
        }
        __builtin_amdgcn_sched_barrier(0);     // the reads below take the registers the writes above have released
        io.read_rows(r0, r1);
        __builtin_amdgcn_sched_barrier(0);
    };
    // a weight chunk: both channels' tasks drop their half of the rows into both staging blocks
    auto share_rows = [&](uint32_t (&r0)[32], uint32_t (&r1)[32]) {
#pragma unroll
        for (int f = 0; f < 8; f += 2) {
            const int q = REV ? 7 - f : f;
            u32x4* const mine = io.wr + 64 * SPITCH * twin;
            u32x4* const theirs = wr_twin + 64 * SPITCH * twin;
            io.drop1(mine, f, q, r0); io.drop1(mine, f + 1, q, r1);
            io.drop1(theirs, f, q, r0); io.drop1(theirs, f + 1, q, r1);
        }
        lds_barrier();
        io.read_rows(r0, r1);
        lds_barrier();                           // before the next tensor lands in the staging blocks
    };

    // ---- vertical pair: the wave runs the chain of its channel that walks the rows downwards (direction slot 0) or
    // upwards (slot 1), and requests the first chunk of its horizontal task on the way
    vertical_chain<T, UP, SAVE, BWD, LOCAL, LOGITS>(p, region, tiles + kc * TILE_WORDS, b, c0 + kc, kc, lane, xr, lr, ur, wr, prefetch);

    // ---- horizontal pair
    float h[2] = {0.f, 0.f};
    float wp0[2] = {0.f, 0.f}, wp1[2] = {0.f, 0.f}, wp2[2] = {0.f, 0.f};     // BWD: taps of the column swept before
    // the task walks in the scan order of direction REV ? 3 : 2 (forward) or against that of direction REV ? 2 : 3
    StretchWalk walk;
    StretchWalkBack bwalk;
    if constexpr (LOCAL && !BWD) walk.init(PW, REV ? 1 : 0, p.kchunk);
    if constexpr (LOCAL && BWD) bwalk.init(PW, REV ? 0 : 1, p.kchunk);
    for (int ch = 0; ch < 2; ++ch) {
        const int col0 = (REV ? 1 - ch : ch) * CS;
        // registers from request order to row order
        if (SWAP_X && ch == 1) {
            io.write_rows(rd_mirror, bx0, bx1);  // my chunk of x is the one the opposite walk needs now
            lds_barrier();
            io.read_rows(bx0, bx1);
            __builtin_amdgcn_sched_barrier(0);
        } else {
            to_rows(bx0, bx1);
        }
        to_rows(bl0, bl1);
        to_rows(bu0, bu1);
        lds_barrier();                           // every task is done with its own staging block
        share_rows(b00, b01);
        share_rows(b10, b11);
        share_rows(b20, b21);
        __builtin_amdgcn_sched_barrier(0);

        // nothing is left to request for this pair: the next pair's vertical chains start theirs
        if (ch == 1 && has_next) chain_request_first<UP, SAVE, BWD, 0, early_requests<SAVE, BWD, LOGITS>()>(p, nb, nc0 + kc, kc, lane, xr, lr, ur, wr);

        float cpair[2] = {0.f, 0.f}, hpair[2] = {0.f, 0.f};    // first element of the pair of columns that share a word
        uint32_t yw[2] = {0, 0};
        uint32_t hq[2][4];                       // SAVE: the states of the eight columns being worked on
        static_for<CS>([&](auto kc_) __attribute__((always_inline)) {
            constexpr int k = decltype(kc_)::value;
            constexpr int e = REV ? CS - 1 - k : k;
            uint32_t* tw = trow + ((col0 + e) >> 1);
            if ((k & 1) == 0) { yw[0] = tw[0]; yw[1] = tw[TODD]; }
            float av[2] = {elem<T>(bl0, e) * elem<T>(bx0, e), elem<T>(bl1, e) * elem<T>(bx1, e)};
            float c0[2] = {elem<T>(b00, e), elem<T>(b01, e)};
            float c1[2] = {elem<T>(b10, e), elem<T>(b11, e)};
            float c2[2] = {elem<T>(b20, e), elem<T>(b21, e)};
            if constexpr (LOGITS) { softmax3(c0[0], c1[0], c2[0], first, false); softmax3(c0[1], c1[1], c2[1], false, last); }
            if constexpr (BWD) {
                line_update_transposed<2, wave_line<T, SAVE, BWD, LOCAL>()>(h, av, wp0, wp1, wp2, first, last);
                bool starts = false;
                if constexpr (LOCAL) starts = bwalk.start(ch == 1 && k == CS - 1);
                // the taps this column hands on to the column swept next; a tap that points outside the line takes nothing
                wp0[0] = (first || starts) ? 0.f : c0[0]; wp0[1] = starts ? 0.f : c0[1];
                wp1[0] = starts ? 0.f : c1[0]; wp1[1] = starts ? 0.f : c1[1];
                wp2[0] = starts ? 0.f : c2[0]; wp2[1] = (last || starts) ? 0.f : c2[1];
            } else {
                if (LOCAL || k == 0) {
                    bool start = ch == 0 && k == 0;              // scan step 0: its weights are never read
                    if constexpr (LOCAL) start = walk.start();   // ... nor those of a stretch's first line
#pragma unroll
                    for (int v = 0; v < 2; ++v) {
                        c0[v] = start ? 0.f : c0[v]; c1[v] = start ? 0.f : c1[v]; c2[v] = start ? 0.f : c2[v];
                        if constexpr (LOCAL) h[v] = start ? 0.f : h[v];
                    }
                }
                line_update<2, wave_line<T, SAVE, BWD, LOCAL>()>(h, av, c0, c1, c2, first, last);
            }
            const float cv[2] = {elem<T>(bu0, e) * h[0], elem<T>(bu1, e) * h[1]};
            if ((k & 1) == 0) { cpair[0] = cv[0]; cpair[1] = cv[1]; hpair[0] = h[0]; hpair[1] = h[1]; }
            else {
                // columns e and e ^ 1 are complete: their words of the tile take both
#pragma unroll
                for (int v = 0; v < 2; ++v) {
                    const float clo = (e & 1) ? cpair[v] : cv[v], chi = (e & 1) ? cv[v] : cpair[v];
                    tw[v * TODD] = pack_word<T>(word_lo<T>(yw[v]) + clo, word_hi<T>(yw[v]) + chi);
                    if constexpr (SAVE) hq[v][(e >> 1) & 3] = pack_word<T>((e & 1) ? hpair[v] : h[v], (e & 1) ? h[v] : hpair[v]);
                }
            }
            if constexpr (SAVE) {
                // eight columns of states are complete: they wait in the staging block (idle while a chunk is worked on)
                if ((k & 7) == 7) {
                    const u32x4 v0 = {hq[0][0], hq[0][1], hq[0][2], hq[0][3]}, v1 = {hq[1][0], hq[1][1], hq[1][2], hq[1][3]};
                    io.rd[e >> 3] = v0; io.rd[SPITCH + (e >> 3)] = v1;
                }
            }
            __builtin_amdgcn_sched_barrier(0);       // one scan step after the other: nothing is gained by mixing them, registers are lost
            if ((k & 7) == 7 && ch == 0) {
                // columns 8q..8q+7 are consumed: their registers take the next chunk's requests (x: unless it is swapped)
                issue_slot(1, e >> 3, !SWAP_X);
                __builtin_amdgcn_sched_barrier(0);
            }
        });
        if constexpr (SAVE) io.store_staged<CP_STREAM>(hb, col0 * 2);
    }

    // ---- the tiles hold the rounded output: copy them out, one row per request
    lds_barrier();
    {
        // sixteen rows at a time: all their LDS reads are on their way before the first store needs its word
        const rsrc_t yb = make_rsrc((char*)p.y + ((size_t)b * p.C + c0) * PLANE_B);
        const uint32_t voff = (uint32_t)(lane * 4);
        constexpr int GROUP = 16;
        for (int r0 = wave; r0 < 2 * PH; r0 += 4 * GROUP) {
            uint32_t v[GROUP];
#pragma unroll
            for (int i = 0; i < GROUP; ++i) {
                const int r = r0 + 4 * i, ch = r >> 7, row = r & (PH - 1);
                v[i] = tiles[ch * TILE_WORDS + tile_row(row) * TPITCH + lane];
            }
#pragma unroll
            for (int i = 0; i < GROUP; ++i)
                __builtin_amdgcn_raw_buffer_store_b32(v[i], yb, voff, __builtin_amdgcn_readfirstlane((r0 + 4 * i) * ROW_B), CP_STREAM);
        }
    }
}

// The pairs of channels a workgroup works through: items blockIdx.x, blockIdx.x + gridDim.x, ... of B * C/2, dealt so
// that the workgroups running at any one time hold neighbouring channels of few weight groups per XCD.
template <typename T, bool REV, bool SAVE, bool BWD, bool LOCAL, bool LOGITS>
__device__ __forceinline__ void pair_loop(const FwdParams& p, uint32_t* tiles, char* region, int wave, int lane) {
    constexpr bool UP = REV != BWD;
    const int kc = wave >> 1;
    const unsigned pairs = (unsigned)(p.C / 2), total = (unsigned)p.B * pairs;
    const unsigned rounds = (total + gridDim.x - 1) / gridDim.x;
    auto item_of = [&](unsigned round, int& b, int& c0) {
        // the last round may be short: its items are dealt as a launch of their own
        const unsigned in_round = round + 1 < rounds ? gridDim.x : total - round * gridDim.x;
        const unsigned item = round * gridDim.x + xcd_contiguous_item(blockIdx.x, in_round);
        b = (int)(item / pairs);
        c0 = (int)(item - (unsigned)b * pairs) * 2;
    };
    uint32_t xr[VPF][VBAND], lr[VPF][VBAND], ur[VPF][VBAND], wr[2][3][VBAND / 2];
    int b, c0;
    item_of(0, b, c0);
    chain_request_first<UP, SAVE, BWD, 0, early_requests<SAVE, BWD, LOGITS>()>(p, b, c0 + kc, kc, lane, xr, lr, ur, wr);
    for (unsigned round = 0; round < rounds; ++round) {
        // a workgroup beyond the end of a short last round has nothing left
        const bool has_next = round + 1 < rounds && (round + 2 < rounds || blockIdx.x < total - (round + 1) * gridDim.x);
        int nb = b, nc0 = c0;
        if (has_next) item_of(round + 1, nb, nc0);
        pair_body<T, REV, SAVE, BWD, LOCAL, LOGITS>(p, tiles, region, b, c0, wave, lane, has_next, nb, nc0, xr, lr, ur, wr);
        if (!has_next) break;
        b = nb; c0 = nc0;
    }
}

template <typename T, bool SAVE, bool BWD, bool LOCAL, bool LOGITS>
__global__ void __launch_bounds__(256) fwd_pair_kernel(FwdParams p) {
    static_assert(LOCAL || !LOGITS, "logits run on the local instantiations (a global scan is one stretch)");
    extern __shared__ uint32_t lds[];
    uint32_t* tiles = lds;
    char* region = (char*)(lds + 2 * TILE_WORDS);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // wave -> horizontal task (channel = wave / 2, direction slot = wave % 2); the task of direction slot 0 walks the
    // columns from the left in the forward scan and from the right in the reverse sweep
    if (((wave & 1) == 0) != BWD) pair_loop<T, false, SAVE, BWD, LOCAL, LOGITS>(p, tiles, region, wave, lane);
    else pair_loop<T, true, SAVE, BWD, LOCAL, LOGITS>(p, tiles, region, wave, lane);
}

static bool pair_shape_ok(const FwdParams& p, int dtype) {
    if ((dtype != 1 && dtype != 2) || p.H != PH || p.W != PW) return false;
    if (p.mask != 15u || p.xt) return false;
    if (p.cpg % 2 || p.C % 2) return false;
    if ((size_t)p.B * (p.C / 2) > 0x7fffffffull) return false;
    return true;
}

template <typename T, bool SAVE, bool BWD, bool LOCAL, bool LOGITS>
static hipError_t launch_pair_as(const FwdParams& p, hipStream_t s) {
    auto k = fwd_pair_kernel<T, SAVE, BWD, LOCAL, LOGITS>;
    hipError_t e = allow_dynamic_lds((const void*)k, LDS_BYTES);
    if (e != hipSuccess) return e;
    // one workgroup fits a compute unit (LDS): as many workgroups as the chip has compute units, each working through
    // its share of the pairs
    const size_t total = (size_t)p.B * (p.C / 2);
    hipLaunchKernelGGL(k, dim3((unsigned)(total < PERSIST_WGS ? total : PERSIST_WGS)), dim3(256), LDS_BYTES, s, p);
    return hipGetLastError();
}

template <typename T, bool SAVE, bool BWD>
static hipError_t launch_pair(const FwdParams& p, hipStream_t s) {
    if (p.logits) return launch_pair_as<T, SAVE, BWD, true, true>(p, s);
    return p.kchunk > 0 ? launch_pair_as<T, SAVE, BWD, true, false>(p, s) : launch_pair_as<T, SAVE, BWD, false, false>(p, s);
}

// T = bf16_t or f16_t; reverse: the reverse sweep of the two-pass backward (p as gspn_bwd_twopass.hip sets it up)
template <typename T>
static hipError_t launch_pair_typed(const FwdParams& p, bool reverse, hipStream_t s) {
    if (reverse) return launch_pair<T, true, true>(p, s);
    return p.hs ? launch_pair<T, true, false>(p, s) : launch_pair<T, false, false>(p, s);
}

}  // namespace
}  // namespace gspn
