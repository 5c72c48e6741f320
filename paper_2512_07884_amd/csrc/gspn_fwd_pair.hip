// Forward GSPN scan for 128x128 maps in bf16 storage whose weight groups hold an even number of channels (the
// diffusion-latent shape): one workgroup of four waves owns TWO channels of one weight group and runs the four
// directions of Sec. 3.2 over them inside one launch (Sec. 4.1), built around how few bytes a compute unit can pull
// through its vector cache per unit time and around a register file of 512 registers per lane for a single wave:
//
//  * Vertical pair (rows are contiguous in memory): two waves copy whole bands of eight rows -- x, lam, u of each
//    (channel, direction) chain and the three weight planes of each direction -- from memory into an LDS ring with
//    16-byte-per-lane requests (every request is whole cache lines, two bands in flight per wave), and two waves run
//    the recurrences of Eq. 1 out of that ring: one wave per walk (rows downwards / upwards), both channels side by
//    side in it, two columns per lane, neighbours by DPP.  The weights of a band are fetched and read once for the
//    two channels (Sec. 4.2: the channels of a group share them).  One barrier per band.
//  * Horizontal pair (a scan step is an image column): one wave per (channel, direction) holds all 128 image rows, two
//    adjacent rows per lane, so the three-neighbour read of Eq. 1 is two DPP shifts and in-lane moves and no wave
//    ever waits for another inside a chunk.  A chunk is 64 scan steps of the six tensors (12 x 32 registers per lane).
//    It is requested so that eight lanes share a row (each request covers eight whole 128-byte lines, each line is
//    asked for once) and turned into the row-per-lane order through an 18 KB LDS block of the wave's own.
//  * The merged output y = sum_d u_d h_d (Eq. 2) is accumulated in LDS, one 32 KB tile per channel in storage
//    precision (a 32-bit word holds two adjacent columns; even rows fill the first half of a tile, odd rows the
//    second, rows 65 words apart, so that the row-wise and the column-wise walk are both bank-conflict free), and copied
//    out once at the end.  The running sum is therefore rounded to bf16 after each of the four additions an element
//    receives (at most 4 * 2^-8 of the largest partial sum in the worst case, about 5e-3 of max|y| observed), which
//    is what frees the LDS for the staging above.
//  * SAVE stores the hidden states per direction (h_save); BWD is the reverse sweep of the two-pass backward scan on the
//    same machinery (gy as x, u as lam, lam as u, gx as y, e into hs; see gspn_bwd_twopass.hip).
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
constexpr int BAND = 8;                           // rows per band of the vertical pair
constexpr int NBANDS = PH / BAND;
constexpr int UNIT_B = 1024;                      // one 16-byte-per-lane request of a wave
constexpr int BAND_B = BAND * ROW_B;              // one tensor's band: two units
constexpr int NTB = 4 * 3 + 2 * 3;                // tensor bands per ring slot: (x, lam, u) of four chains, three taps of two walks
constexpr int SLOT_B = NTB * BAND_B;              // 36 KB
constexpr int SPITCH = 9;                         // 16-byte units between two rows of a staging block (128 bytes + 16)
constexpr int STAGE_B = PH * SPITCH * 16;         // horizontal pair: 128 rows of 128 bytes per wave
constexpr int REGION_B = 2 * SLOT_B > 4 * STAGE_B ? 2 * SLOT_B : 4 * STAGE_B;
constexpr int CS = 64;                            // scan steps per chunk of the horizontal pair (128 bytes per row)
constexpr int LDS_BYTES = 2 * TILE_WORDS * 4 + REGION_B;

__device__ __forceinline__ float lo16(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float hi16(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ u32x4 ld128(rsrc_t rs, uint32_t voff, int soff) {
    return __builtin_amdgcn_raw_buffer_load_b128(rs, voff, __builtin_amdgcn_readfirstlane(soff), 0);
}
// where image row r sits in an output tile (in rows of TPITCH words)
__device__ __forceinline__ int tile_row(int r) { return (r >> 1) + (PH / 2) * (r & 1); }

// ---------------------------------------------------------------------------
// vertical pair, loader waves: band s of every tensor -> ring slot s & 1
// ---------------------------------------------------------------------------
// Tensor band tb of a slot (2 KB at byte tb * 2048): 0..11 are x, lam, u of chain 0..3 (chain = channel * 2 + walk,
// walk 0 = rows downwards), 12..17 the taps 0..2 of the two walks.  Loader j copies half j of every tensor band.  A chain
// that walks the rows upwards takes its bands from the bottom of the plane.
template <bool BWD>
struct BandLoader {
    const char* src[NTB];
    uint32_t off_dn, off_up;      // this lane's byte offset into band 0 of a plane for the two walks
    uint32_t lds_off;
    u32x4 ra[NTB], rb[NTB];

    __device__ __forceinline__ void init(const FwdParams& p, int b, int c0, int j, int lane) {
        const int g = c0 / p.cpg;
        const size_t planes = (size_t)p.B * p.C;
        off_dn = (uint32_t)(j * UNIT_B + lane * 16);
        off_up = off_dn + (uint32_t)((NBANDS - 1) * BAND_B);
        lds_off = off_dn;
#pragma unroll
        for (int tb = 0; tb < NTB; ++tb) {
            if (tb < 12) {
                const int chain = tb / 3, tensor = tb - chain * 3, ch = chain >> 1, walk = chain & 1;
                const int d = BWD ? 1 - walk : walk;               // the parameters this chain works on
                const size_t slot_c = p.shared ? 0 : (size_t)d * planes * HW;
                const size_t plane = ((size_t)b * p.C + c0 + ch) * HW;
                src[tb] = tensor == 0 ? (const char*)p.x + plane * 2
                        : tensor == 1 ? (const char*)p.lam + (slot_c + plane) * 2
                                      : (const char*)p.u + (slot_c + plane) * 2;
            } else {
                const int t = tb - 12, walk = t / 3, tap = t - walk * 3;
                const int d = BWD ? 1 - walk : walk;
                const size_t slot_w = p.shared ? 0 : (size_t)d * p.B * p.G * 3 * HW;
                src[tb] = (const char*)p.w + (slot_w + (((size_t)b * p.G + g) * 3 + tap) * HW) * 2;
            }
        }
    }
    static __device__ __forceinline__ constexpr bool walks_up(int tb) { return tb < 12 ? ((tb / 3) & 1) != 0 : (tb - 12) / 3 != 0; }
    __device__ __forceinline__ void issue(u32x4 (&r)[NTB], int s) {
        const uint32_t dn = off_dn + (uint32_t)(s * BAND_B), up = off_up - (uint32_t)(s * BAND_B);
#pragma unroll
        for (int tb = 0; tb < NTB; ++tb) r[tb] = *(const u32x4*)(src[tb] + (walks_up(tb) ? up : dn));
    }
    __device__ __forceinline__ void drop(const u32x4 (&r)[NTB], char* slot) {
#pragma unroll
        for (int tb = 0; tb < NTB; ++tb) *(u32x4*)(slot + lds_off + tb * BAND_B) = r[tb];
    }
    // tail() is called once, when the last band is on its way to LDS (the wave's own requests for what comes next)
    template <typename F>
    __device__ __forceinline__ void run(char* region, F& tail) {
        issue(ra, 0);
        issue(rb, 1);
        drop(ra, region);
        issue(ra, 2);
        lds_barrier();
        for (int s = 0; s < NBANDS - 4; s += 2) {
            // while the chains work on band s (slot 0), band s + 1 goes to slot 1 and band s + 3 is requested
            drop(rb, region + SLOT_B);
            issue(rb, s + 3);
            lds_barrier();
            drop(ra, region);
            issue(ra, s + 4);
            lds_barrier();
        }
        // the last four bands: nothing is left to request after the last one
        drop(rb, region + SLOT_B);
        issue(rb, NBANDS - 1);
        lds_barrier();
        drop(ra, region);
        lds_barrier();
        drop(rb, region + SLOT_B);
        tail();
        lds_barrier();
        lds_barrier();
    }
};

// ---------------------------------------------------------------------------
// vertical pair, compute waves: the two channels' chains of one walk out of the ring
// ---------------------------------------------------------------------------
// ahead() is called once, V_AHEAD bands before the end (the wave's own requests for what comes next)
template <bool UP, bool SAVE, bool BWD, typename F>
__device__ __forceinline__ void vertical_chains(const FwdParams& p, const char* region, uint32_t* tiles, int b, int c0, int lane, F& ahead) {
    constexpr int d = BWD ? (UP ? 0 : 1) : (UP ? 1 : 0);
    constexpr int V_AHEAD = 4;
    const bool first = lane == 0, last = lane == 63;
    const size_t planes = (size_t)p.B * p.C;
    // SAVE: the two channels' planes of h_save are adjacent in memory
    const rsrc_t hb = make_rsrc(SAVE ? (char*)p.hs + ((size_t)d * planes * HW + ((size_t)b * p.C + c0) * HW) * 2 : (char*)p.y);
    const uint32_t voff = (uint32_t)(lane * 4);
    float h[2][2] = {{0.f, 0.f}, {0.f, 0.f}};
    float wp0[2] = {0.f, 0.f}, wp1[2] = {0.f, 0.f}, wp2[2] = {0.f, 0.f};     // BWD: taps of the row swept before
    lds_barrier();                                                            // band 0 is in slot 0
    auto band = [&](int s) {
        const char* slot = region + (s & 1) * SLOT_B;
        const uint32_t* cw = (const uint32_t*)(slot + (12 + (UP ? 3 : 0)) * BAND_B) + lane;
        // everything the band needs from LDS is requested before the first row is worked on: the writes to the tiles
        // below would otherwise fence the reads of the following rows (LDS against LDS), and this wave has its SIMD to
        // itself, so nothing else would cover their latency
        uint32_t t0[BAND], t1[BAND], t2[BAND], xw[2][BAND], lw[2][BAND], uw[2][BAND], ow[2][BAND];
#pragma unroll
        for (int k = 0; k < BAND; ++k) {
            const int r = UP ? BAND - 1 - k : k;                              // row inside the band
            t0[k] = cw[r * 64]; t1[k] = cw[BAND_B / 4 + r * 64]; t2[k] = cw[2 * (BAND_B / 4) + r * 64];
#pragma unroll
            for (int ch = 0; ch < 2; ++ch) {
                const uint32_t* cx = (const uint32_t*)(slot + (ch * 2 + (UP ? 1 : 0)) * 3 * BAND_B) + lane;
                xw[ch][k] = cx[r * 64]; lw[ch][k] = cx[BAND_B / 4 + r * 64]; uw[ch][k] = cx[2 * (BAND_B / 4) + r * 64];
            }
        }
        if (s >= NBANDS / 2) {
            // second half of a walk: these rows hold what the other walk left
#pragma unroll
            for (int k = 0; k < BAND; ++k) {
                const int row = UP ? PH - 1 - (s * BAND + k) : s * BAND + k;
#pragma unroll
                for (int ch = 0; ch < 2; ++ch) ow[ch][k] = tiles[ch * TILE_WORDS + tile_row(row) * TPITCH + lane];
            }
        } else {
#pragma unroll
            for (int k = 0; k < BAND; ++k) { ow[0][k] = 0; ow[1][k] = 0; }
        }
#pragma unroll
        for (int k = 0; k < BAND; ++k) {
            const int row = UP ? PH - 1 - (s * BAND + k) : s * BAND + k;      // image row
            float c0[2] = {lo16(t0[k]), hi16(t0[k])}, c1[2] = {lo16(t1[k]), hi16(t1[k])}, c2[2] = {lo16(t2[k]), hi16(t2[k])};
            if constexpr (!BWD) {
                if (k == 0) {
                    // scan step 0: its weights are never read (they may hold anything) and the state before it is 0
                    const bool start = s == 0;
#pragma unroll
                    for (int v = 0; v < 2; ++v) { c0[v] = start ? 0.f : c0[v]; c1[v] = start ? 0.f : c1[v]; c2[v] = start ? 0.f : c2[v]; }
                }
            }
#pragma unroll
            for (int ch = 0; ch < 2; ++ch) {
                float av[2] = {lo16(lw[ch][k]) * lo16(xw[ch][k]), hi16(lw[ch][k]) * hi16(xw[ch][k])};
                if constexpr (BWD) line_update_transposed<2>(h[ch], av, wp0, wp1, wp2, first, last);
                else line_update<2>(h[ch], av, c0, c1, c2, first, last);
                const float y0 = lo16(uw[ch][k]) * h[ch][0], y1 = hi16(uw[ch][k]) * h[ch][1];
                // the first half of a walk writes rows nobody has touched yet (ow = 0); the second half adds to what the
                // other walk left
                tiles[ch * TILE_WORDS + tile_row(row) * TPITCH + lane] = pack_bf16x2(lo16(ow[ch][k]) + y0, hi16(ow[ch][k]) + y1);
                if constexpr (SAVE) {
                    const uint32_t hw = pack_bf16x2(h[ch][0], h[ch][1]);
                    __builtin_amdgcn_raw_buffer_store_b32(hw, hb, voff, __builtin_amdgcn_readfirstlane(ch * PLANE_B + row * ROW_B), 0);
                }
            }
            if constexpr (BWD) {
                // the taps this row hands on to the row swept next; a tap that points outside the line takes nothing,
                // whatever the tensor holds there
                wp0[0] = first ? 0.f : c0[0]; wp0[1] = c0[1];
                wp1[0] = c1[0]; wp1[1] = c1[1];
                wp2[0] = c2[0]; wp2[1] = last ? 0.f : c2[1];
            }
        }
        lds_barrier();
    };
    for (int s = 0; s < NBANDS - V_AHEAD; ++s) band(s);
    ahead();
    for (int s = NBANDS - V_AHEAD; s < NBANDS; ++s) band(s);
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
    __device__ __forceinline__ void issue1(rsrc_t rs, int col_bytes, int i, int slot, uint32_t (&r)[32]) const {
        const u32x4 v = ld128(rs, voff, col_bytes + i * 8 * ROW_B);
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
    __device__ __forceinline__ void store_staged(rsrc_t rs, int col_bytes) const {
#pragma unroll
        for (int i = 0; i < 16; ++i) st_b128(rs, voff + (uint32_t)(col_bytes + i * 8 * ROW_B), wr[8 * SPITCH * i]);
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
template <bool REV, bool SAVE, bool BWD>
__device__ __forceinline__ void pair_body(const FwdParams& p, uint32_t* tiles, char* region, int b, int c0, int wave, int lane) {
    constexpr int d = (REV != BWD) ? 3 : 2;
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
        io.issue1(lb, cb, 2 * f, q, bl0); io.issue1(lb, cb, 2 * f + 1, q, bl1);
        if ((f & 1) == 0) {
            const int i = 8 * twin + f;
            io.issue1(w0b, cb, i, q, b00); io.issue1(w0b, cb, i + 1, q, b01);
            io.issue1(w1b, cb, i, q, b10); io.issue1(w1b, cb, i + 1, q, b11);
            io.issue1(w2b, cb, i, q, b20); io.issue1(w2b, cb, i + 1, q, b21);
        }
        io.issue1(ub, cb, 2 * f, q, bu0); io.issue1(ub, cb, 2 * f + 1, q, bu1);
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

    // ---- vertical pair: wave 0 walks the rows downwards, wave 1 upwards (both channels each), waves 2 and 3 feed the
    // ring; everybody requests the first chunk of its horizontal task on the way
    if (wave >= 2) {
        BandLoader<BWD> ld;
        ld.init(p, b, c0, wave - 2, lane);
        ld.run(region, prefetch);
    } else {
        if (wave & 1) vertical_chains<true, SAVE, BWD>(p, region, tiles, b, c0, lane, prefetch);
        else vertical_chains<false, SAVE, BWD>(p, region, tiles, b, c0, lane, prefetch);
    }

    // ---- horizontal pair
    float h[2] = {0.f, 0.f};
    float wp0[2] = {0.f, 0.f}, wp1[2] = {0.f, 0.f}, wp2[2] = {0.f, 0.f};     // BWD: taps of the column swept before
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

        float cpair[2] = {0.f, 0.f}, hpair[2] = {0.f, 0.f};    // first element of the pair of columns that share a word
        uint32_t yw[2] = {0, 0};
        uint32_t hq[2][4];                       // SAVE: the states of the eight columns being worked on
        static_for<CS>([&](auto kc_) __attribute__((always_inline)) {
            constexpr int k = decltype(kc_)::value;
            constexpr int e = REV ? CS - 1 - k : k;
            uint32_t* tw = trow + ((col0 + e) >> 1);
            if ((k & 1) == 0) { yw[0] = tw[0]; yw[1] = tw[TODD]; }
            float av[2] = {elem<bf16_t>(bl0, e) * elem<bf16_t>(bx0, e), elem<bf16_t>(bl1, e) * elem<bf16_t>(bx1, e)};
            float c0[2] = {elem<bf16_t>(b00, e), elem<bf16_t>(b01, e)};
            float c1[2] = {elem<bf16_t>(b10, e), elem<bf16_t>(b11, e)};
            float c2[2] = {elem<bf16_t>(b20, e), elem<bf16_t>(b21, e)};
            if constexpr (BWD) {
                line_update_transposed<2>(h, av, wp0, wp1, wp2, first, last);
                // the taps this column hands on to the column swept next; a tap that points outside the line takes nothing
                wp0[0] = first ? 0.f : c0[0]; wp0[1] = c0[1];
                wp1[0] = c1[0]; wp1[1] = c1[1];
                wp2[0] = c2[0]; wp2[1] = last ? 0.f : c2[1];
            } else {
                if (k == 0) {
                    const bool start = ch == 0;                  // scan step 0: its weights are never read
#pragma unroll
                    for (int v = 0; v < 2; ++v) { c0[v] = start ? 0.f : c0[v]; c1[v] = start ? 0.f : c1[v]; c2[v] = start ? 0.f : c2[v]; }
                }
                line_update<2>(h, av, c0, c1, c2, first, last);
            }
            const float cv[2] = {elem<bf16_t>(bu0, e) * h[0], elem<bf16_t>(bu1, e) * h[1]};
            if ((k & 1) == 0) { cpair[0] = cv[0]; cpair[1] = cv[1]; hpair[0] = h[0]; hpair[1] = h[1]; }
            else {
                // columns e and e ^ 1 are complete: their words of the tile take both
#pragma unroll
                for (int v = 0; v < 2; ++v) {
                    const float clo = (e & 1) ? cpair[v] : cv[v], chi = (e & 1) ? cv[v] : cpair[v];
                    tw[v * TODD] = pack_bf16x2(lo16(yw[v]) + clo, hi16(yw[v]) + chi);
                    if constexpr (SAVE) hq[v][(e >> 1) & 3] = pack_bf16x2((e & 1) ? hpair[v] : h[v], (e & 1) ? h[v] : hpair[v]);
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
        if constexpr (SAVE) io.store_staged(hb, col0 * 2);
    }
}

template <bool SAVE, bool BWD>
__global__ void __launch_bounds__(256) fwd_pair_kernel(FwdParams p) {
    extern __shared__ uint32_t lds[];
    uint32_t* tiles = lds;
    char* region = (char*)(lds + 2 * TILE_WORDS);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int pairs = p.C / 2;
    const unsigned item = xcd_contiguous_item(blockIdx.x, gridDim.x);
    const int b = item / pairs;
    const int c0 = (item - b * pairs) * 2;

    // wave -> horizontal task (channel = wave / 2, direction slot = wave % 2); the task of direction slot 0 walks the
    // columns from the left in the forward scan and from the right in the reverse sweep
    if (((wave & 1) == 0) != BWD) pair_body<false, SAVE, BWD>(p, tiles, region, b, c0, wave, lane);
    else pair_body<true, SAVE, BWD>(p, tiles, region, b, c0, wave, lane);

    // ---- the tiles hold the rounded output: copy them out, one row per request
    lds_barrier();
    {
        char* Y = (char*)p.y + ((size_t)b * p.C + c0) * PLANE_B;
        for (int r = wave; r < 2 * PH; r += 4) {
            const int ch = r >> 7, row = r & (PH - 1);
            const uint32_t v = tiles[ch * TILE_WORDS + tile_row(row) * TPITCH + lane];
            *(uint32_t*)(Y + (size_t)r * ROW_B + lane * 4) = v;
        }
    }
}

bool pair_shape_ok(const FwdParams& p, int dtype) {
    if (dtype != 1 || p.H != PH || p.W != PW) return false;
    if (p.mask != 15u || p.kchunk > 0 || p.logits || p.xt) return false;
    if (p.cpg % 2 || p.C % 2) return false;
    if ((size_t)p.B * (p.C / 2) > 0x7fffffffull) return false;
    return true;
}

template <bool SAVE, bool BWD>
hipError_t launch_pair(const FwdParams& p, hipStream_t s) {
    auto k = fwd_pair_kernel<SAVE, BWD>;
    hipError_t e = allow_dynamic_lds((const void*)k, LDS_BYTES);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k, dim3((unsigned)((size_t)p.B * (p.C / 2))), dim3(256), LDS_BYTES, s, p);
    return hipGetLastError();
}

}  // namespace

bool fwd_pair_applicable(const FwdParams& p, int dtype) { return pair_shape_ok(p, dtype); }

hipError_t launch_fwd_pair(const FwdParams& p, int dtype, hipStream_t s) {
    if (!pair_shape_ok(p, dtype)) return hipErrorInvalidValue;
    return p.hs ? launch_pair<true, false>(p, s) : launch_pair<false, false>(p, s);
}

bool reverse_sweep_pair_applicable(const FwdParams& p, int dtype) { return pair_shape_ok(p, dtype) && p.hs; }

hipError_t launch_reverse_sweep_pair(const FwdParams& p, int dtype, hipStream_t s) {
    if (!reverse_sweep_pair_applicable(p, dtype)) return hipErrorInvalidValue;
    return launch_pair<true, true>(p, s);
}

}  // namespace gspn
