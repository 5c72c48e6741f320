// Forward GSPN scan for 128x128 maps in bf16 storage whose weight groups hold an even number of channels (the
// diffusion-latent shape): one workgroup of eight waves owns TWO channels of one weight group and runs the four
// directions of Sec. 3.2 over them inside one launch (Sec. 4.1), built around how few bytes a compute unit can pull
// through its vector cache per unit time:
//
//  * Vertical pair (rows are contiguous in memory): four waves copy whole bands of eight rows -- x, lam, u of each
//    (channel, direction) chain and the three weight planes of each direction -- from memory into an LDS ring with
//    16-byte-per-lane requests (every request is whole cache lines, two bands in flight per wave), and four waves run
//    the recurrences of Eq. 1 out of that ring, two columns per lane, neighbours by DPP.  The weights of a band are
//    fetched once for the two channels (Sec. 4.2: the channels of a group share them).  One barrier per band.
//  * Horizontal pair (a scan step is an image column): every wave owns 64 image rows of one (channel, direction),
//    one row per lane, and holds a chunk of 64 scan steps of its six tensors in registers.  A chunk is requested so
//    that eight lanes share a row (each request covers eight whole 128-byte lines, each line is asked for once) and is
//    turned into the row-per-lane order through a 9 KB LDS block of the wave's own; the two waves of a column pass
//    their edge rows through a two-slot LDS mailbox whose entries carry the scan step they belong to, so each pair
//    of waves keeps step by itself (no workgroup barrier inside a chunk: the four pairs of a workgroup run apart
//    and fill each other's waits).
//  * The merged output y = sum_d u_d h_d (Eq. 2) is accumulated in LDS, one 32 KB tile per channel in storage
//    precision (a 32-bit word holds two adjacent columns; rows are 65 words apart so that both the row-wise and the
//    column-wise walk are bank-conflict free), and copied out once at the end.  The running sum is therefore rounded
//    to bf16 after each of the four additions an element receives (at most 4 * 2^-8 of the largest partial sum in the
//    worst case, about 5e-3 of max|y| observed), which is what frees the LDS for the staging above.
//  * SAVE stores the hidden states per direction (h_save); BWD is the reverse sweep of the two-pass backward scan on the
//    same machinery (gy as x, u as lam, lam as u, gx as y, e into hs; see gspn_bwd_twopass.hip).
#include "gspn_tile_common.hpp"

namespace gspn {
namespace {

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
constexpr int NTB = 4 * 3 + 2 * 3;                // tensor bands per ring slot: (x, lam, u) of four chains, three taps of two directions
constexpr int SLOT_B = NTB * BAND_B;              // 36 KB
constexpr int UNITS_PER_LOADER = NTB * 2 / 4;     // four loader waves
constexpr int SPITCH = 9;                         // 16-byte units between two rows of a staging block (128 bytes + 16)
constexpr int STAGE_B = 64 * SPITCH * 16;         // horizontal pair: 64 rows of 128 bytes per wave
constexpr int REGION_B = 2 * SLOT_B > 8 * STAGE_B ? 2 * SLOT_B : 8 * STAGE_B;
constexpr int CS = 64;                            // scan steps per chunk of the horizontal pair (128 bytes per row)
constexpr int MAILBOX_FLOATS = 2 * 2 * 2 * 2 * 2;  // [channel][direction][part][parity] x (value, scan step)
constexpr int SPIN_LIMIT = 1 << 16;               // polls of a mailbox entry before a wave gives up waiting (never reached: the partner always writes)
constexpr int LDS_BYTES = 2 * TILE_WORDS * 4 + REGION_B + MAILBOX_FLOATS * 4;

__device__ __forceinline__ float lo16(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float hi16(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ u32x4 ld128(rsrc_t rs, uint32_t voff, int soff) {
    return __builtin_amdgcn_raw_buffer_load_b128(rs, voff, __builtin_amdgcn_readfirstlane(soff), 0);
}

// ---------------------------------------------------------------------------
// vertical pair, loader waves: band s of every tensor -> ring slot s & 1
// ---------------------------------------------------------------------------
// Unit u of a slot (1 KB at byte u * 1024) is half `u & 1` of tensor band `u >> 1`: tensor bands 0..11 are x, lam, u of
// chain 0..3 (chain = channel * 2 + walk, walk 0 = rows downwards), 12..17 the taps 0..2 of the two walks.  Loader j
// copies units j, j + 4, ...  A chain that walks the rows upwards takes its bands from the bottom of the plane.
template <bool BWD>
struct BandLoader {
    rsrc_t rs[UNITS_PER_LOADER];
    int up[UNITS_PER_LOADER];
    int half_off;
    uint32_t voff, lds_off;
    u32x4 ra[UNITS_PER_LOADER], rb[UNITS_PER_LOADER];

    __device__ __forceinline__ void init(const FwdParams& p, int b, int c0, int j, int lane) {
        const int g = c0 / p.cpg;
        const size_t planes = (size_t)p.B * p.C;
        half_off = (j & 1) * UNIT_B;
        voff = (uint32_t)(lane * 16);
        lds_off = (uint32_t)(j * UNIT_B + lane * 16);
#pragma unroll
        for (int k = 0; k < UNITS_PER_LOADER; ++k) {
            const int tb = (j >> 1) + 2 * k;
            const char* base;
            int walk;
            if (tb < 12) {
                const int chain = tb / 3, tensor = tb - chain * 3, ch = chain >> 1;
                walk = chain & 1;
                const int d = BWD ? 1 - walk : walk;               // the parameters this chain works on
                const size_t slot_c = p.shared ? 0 : (size_t)d * planes * HW;
                const size_t plane = ((size_t)b * p.C + c0 + ch) * HW;
                base = tensor == 0 ? (const char*)p.x + plane * 2
                     : tensor == 1 ? (const char*)p.lam + (slot_c + plane) * 2
                                   : (const char*)p.u + (slot_c + plane) * 2;
            } else {
                const int t = tb - 12;
                walk = t / 3;
                const int tap = t - walk * 3;
                const int d = BWD ? 1 - walk : walk;
                const size_t slot_w = p.shared ? 0 : (size_t)d * p.B * p.G * 3 * HW;
                base = (const char*)p.w + (slot_w + (((size_t)b * p.G + g) * 3 + tap) * HW) * 2;
            }
            rs[k] = make_rsrc(base);
            up[k] = walk;
        }
    }
    __device__ __forceinline__ void issue(u32x4 (&r)[UNITS_PER_LOADER], int s) {
        s = s < NBANDS ? s : NBANDS - 1;                           // clamped: redundant but in bounds at the end
#pragma unroll
        for (int k = 0; k < UNITS_PER_LOADER; ++k)
            r[k] = ld128(rs[k], voff, (up[k] ? NBANDS - 1 - s : s) * BAND_B + half_off);
    }
    __device__ __forceinline__ void drop(const u32x4 (&r)[UNITS_PER_LOADER], char* slot) {
#pragma unroll
        for (int k = 0; k < UNITS_PER_LOADER; ++k) *(u32x4*)(slot + lds_off + k * 4 * UNIT_B) = r[k];
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
// vertical pair, compute waves: one (channel, walk) chain out of the ring
// ---------------------------------------------------------------------------
// ahead() is called once, V_AHEAD bands before the end (the wave's own requests for what comes next)
template <bool UP, bool SAVE, bool BWD, typename F>
__device__ __forceinline__ void vertical_chain(const FwdParams& p, const char* region, uint32_t* tile, int b, int c, int chain, int lane, F& ahead) {
    constexpr int d = BWD ? (UP ? 0 : 1) : (UP ? 1 : 0);
    const bool first = lane == 0, last = lane == 63;
    const size_t planes = (size_t)p.B * p.C;
    const rsrc_t hb = make_rsrc(SAVE ? (char*)p.hs + ((size_t)d * planes * HW + ((size_t)b * p.C + c) * HW) * 2 : (char*)p.y);
    constexpr int V_AHEAD = 4;
    const uint32_t voff = (uint32_t)(lane * 4);
    float h[2] = {0.f, 0.f};
    float wp0[2] = {0.f, 0.f}, wp1[2] = {0.f, 0.f}, wp2[2] = {0.f, 0.f};     // BWD: taps of the row swept before
    lds_barrier();                                                            // band 0 is in slot 0
    auto band = [&](int s) {
        const char* slot = region + (s & 1) * SLOT_B;
        const uint32_t* cx = (const uint32_t*)(slot + chain * 3 * BAND_B) + lane;
        const uint32_t* cw = (const uint32_t*)(slot + (12 + (UP ? 3 : 0)) * BAND_B) + lane;
#pragma unroll
        for (int k = 0; k < BAND; ++k) {
            const int r = UP ? BAND - 1 - k : k;                              // row inside the band
            const int row = UP ? PH - 1 - (s * BAND + k) : s * BAND + k;      // image row
            const uint32_t xw = cx[r * 64], lw = cx[BAND_B / 4 + r * 64], uw = cx[2 * (BAND_B / 4) + r * 64];
            const uint32_t t0 = cw[r * 64], t1 = cw[BAND_B / 4 + r * 64], t2 = cw[2 * (BAND_B / 4) + r * 64];
            float av[2] = {lo16(lw) * lo16(xw), hi16(lw) * hi16(xw)};
            float c0[2] = {lo16(t0), hi16(t0)}, c1[2] = {lo16(t1), hi16(t1)}, c2[2] = {lo16(t2), hi16(t2)};
            if constexpr (BWD) {
                line_update_transposed<2>(h, av, wp0, wp1, wp2, first, last);
                // a tap that points outside the line takes nothing, whatever the tensor holds there
                wp0[0] = first ? 0.f : c0[0]; wp0[1] = c0[1];
                wp1[0] = c1[0]; wp1[1] = c1[1];
                wp2[0] = c2[0]; wp2[1] = last ? 0.f : c2[1];
            } else {
                if (k == 0) {
                    // scan step 0: its weights are never read (they may hold anything) and the state before it is 0
                    const bool start = s == 0;
#pragma unroll
                    for (int v = 0; v < 2; ++v) { c0[v] = start ? 0.f : c0[v]; c1[v] = start ? 0.f : c1[v]; c2[v] = start ? 0.f : c2[v]; }
                }
                line_update<2>(h, av, c0, c1, c2, first, last);
            }
            const float y0 = lo16(uw) * h[0], y1 = hi16(uw) * h[1];
            uint32_t* tw = tile + row * TPITCH + lane;
            // the first half of a walk writes rows nobody has touched yet; the second half adds to what the other walk left
            if (s < NBANDS / 2) *tw = pack_bf16x2(y0, y1);
            else { const uint32_t o = *tw; *tw = pack_bf16x2(lo16(o) + y0, hi16(o) + y1); }
            if constexpr (SAVE) {
                const uint32_t hw = pack_bf16x2(h[0], h[1]);
                __builtin_amdgcn_raw_buffer_store_b32(hw, hb, voff, __builtin_amdgcn_readfirstlane(row * ROW_B), 0);
            }
            // two rows at a time: the chunk the wave has requested for its horizontal task lives in registers meanwhile
            if (k & 1) __builtin_amdgcn_sched_barrier(0);
        }
        lds_barrier();
    };
    for (int s = 0; s < NBANDS - V_AHEAD; ++s) band(s);
    ahead();
    for (int s = NBANDS - V_AHEAD; s < NBANDS; ++s) band(s);
}

// ---------------------------------------------------------------------------
// horizontal pair: one wave = 64 image rows of one (channel, direction), one row per lane
// ---------------------------------------------------------------------------
// A chunk of a tensor (64 rows x 128 bytes) is requested in eight instructions of eight rows each (lane -> row l / 8 of
// the instruction, bytes 16 * (l % 8) ..), so every request covers whole lines, instruction i into registers 4i..4i+3.
// to_rows() turns the registers from that order into "lane = row, registers 4q..4q+3 = columns 8q..8q+7" through the
// wave's staging block, whose rows are 144 bytes apart: conflict free for the writers (eight lanes fill one row) and
// for every sixteen neighbouring readers.
struct ChunkIO {
    uint32_t voff;          // load order: byte offset of (row l / 8, column group l % 8) inside the plane
    u32x4* wr;              // staging: where this lane drops instruction 0's registers; instruction i: 8 rows further
    u32x4* rd;              // staging: this lane's row

    __device__ __forceinline__ void init(char* stage, int part, int lane) {
        voff = (uint32_t)(((part * 64 + (lane >> 3)) * PW + 8 * (lane & 7)) * 2);
        wr = (u32x4*)stage + SPITCH * (lane >> 3) + (lane & 7);
        rd = (u32x4*)stage + SPITCH * lane;
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
    __device__ __forceinline__ void read_row(uint32_t (&r)[32]) const {
#pragma unroll
        for (int q = 0; q < 8; ++q) { const u32x4 v = rd[q]; r[4 * q] = v.x; r[4 * q + 1] = v.y; r[4 * q + 2] = v.z; r[4 * q + 3] = v.w; }
    }
    __device__ __forceinline__ void write_row(u32x4* to, const uint32_t (&r)[32]) const {
#pragma unroll
        for (int q = 0; q < 8; ++q) { const u32x4 v = {r[4 * q], r[4 * q + 1], r[4 * q + 2], r[4 * q + 3]}; to[q] = v; }
    }
    __device__ __forceinline__ void to_rows(uint32_t (&r)[32]) const {
#pragma unroll
        for (int i = 0; i < 8; ++i) drop1(wr, i, i, r);
        __builtin_amdgcn_sched_barrier(0);     // the reads below take the registers the writes above have released
        read_row(r);
        __builtin_amdgcn_sched_barrier(0);
    }
    // ... and back, for stores that cover whole lines: the staging block holds a chunk in row order
    __device__ __forceinline__ void store_staged(rsrc_t rs, int col_bytes) const {
#pragma unroll
        for (int i = 0; i < 8; ++i) st_b128(rs, voff + (uint32_t)(col_bytes + i * 8 * ROW_B), wr[8 * SPITCH * i]);
    }
};

// One workgroup's work as wave `wave` sees it: its share of the vertical pair, then its (channel, direction, part) task
// of the horizontal pair.  What keeps the requests of that task few and always in flight:
//  * the two channels of the workgroup share the weights: the task of channel k requests rows 32k..32k+31 of its part's
//    weight chunk only, and the two tasks drop what they fetched into both staging blocks on the way to the row order;
//  * when the columns 8q..8q+7 of a chunk have been consumed their registers take instruction q of the next chunk, so
//    the next chunk arrives while this one is worked on and no register is added;
//  * (without h_save) the task that walks from the left and the one that walks from the right over the same rows hand
//    each other their chunk of x at half time instead of fetching it a second time;
//  * the first chunk is requested while the vertical pair is still at work.
template <bool REV, bool SAVE, bool BWD>
__device__ __forceinline__ void pair_body(const FwdParams& p, uint32_t* tiles, char* region, float* mailbox, int b, int c0, int wave, int lane) {
    constexpr int d = (REV != BWD) ? 3 : 2;
    constexpr bool SWAP_X = !SAVE;             // with h_save the staging blocks collect the states while a chunk is worked on
    const int kc = wave >> 2, dslot = (wave >> 1) & 1, part = wave & 1;
    const int twin = kc;
    const bool top_lane = lane == 0, bot_lane = lane == 63;
    const bool has_up = part > 0, has_dn = part < 1;
    const bool img_first = top_lane && !has_up, img_last = bot_lane && !has_dn;
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
    // mailbox: [task = channel * 2 + direction slot][part][parity] entries of (edge value, scan step it belongs to); part 0
    // publishes its last row and reads the first row of part 1, and the other way round
    u32x2* const task = (u32x2*)mailbox + (kc * 2 + dslot) * 4;
    u32x2* const mb_out = task + part * 2;
    const volatile u32x2* const mb_in = task + (1 - part) * 2;
    const bool publishes = part == 0 ? bot_lane : top_lane;
    uint32_t* const trow = tiles + kc * TILE_WORDS + (part * 64 + lane) * TPITCH;
    ChunkIO io;
    io.init(region + wave * STAGE_B, part, lane);
    // the same place as io.wr in the staging block of the other channel's task; this lane's row in the staging block of
    // the task that walks the other way
    u32x4* const wr_twin = (u32x4*)((char*)io.wr + ((wave ^ 4) - wave) * STAGE_B);
    u32x4* const rd_mirror = (u32x4*)((char*)io.rd + ((wave ^ 2) - wave) * STAGE_B);

    uint32_t bx[32], bl[32], bu[32], b0[32], b1[32], b2[32];
    // byte offset of chunk c_ (in scan order) inside a row
    auto col_bytes = [&](int c_) { return (REV ? 1 - c_ : c_) * CS * 2; };
    // Requests of chunk c_ into the registers 4q..4q+3, which are free at that point: instruction q of x, lam, u; of the
    // weights this task requests rows 32 * twin + 8j .. (j = 0..3) only, into every second set of registers in the
    // order in which the sets come free (the same registers for both channels' tasks)
    auto w_slot = [&](int j) { return REV ? 7 - 2 * j : 2 * j; };
    auto issue_slot = [&](int c_, int q, bool with_x) {
        const int cb = col_bytes(c_);
        const int f = REV ? 7 - q : q;           // q is the f-th set to come free
        if (with_x) io.issue1(xb, cb, q, q, bx);
        io.issue1(lb, cb, q, q, bl);
        if ((f & 1) == 0) {
            const int i = 4 * twin + (f >> 1);
            io.issue1(w0b, cb, i, q, b0); io.issue1(w1b, cb, i, q, b1); io.issue1(w2b, cb, i, q, b2);
        }
        io.issue1(ub, cb, q, q, bu);
    };
    auto prefetch = [&]() {
#pragma unroll
        for (int q = 0; q < 8; ++q) issue_slot(0, q, true);
    };
    // the weight chunk of this part: both channels' tasks drop their half of the rows into both staging blocks
    auto share_rows = [&](uint32_t (&r)[32]) {
#pragma unroll
        for (int j = 0; j < 4; ++j) { io.drop1(io.wr + 32 * SPITCH * twin, j, w_slot(j), r); io.drop1(wr_twin + 32 * SPITCH * twin, j, w_slot(j), r); }
        lds_barrier();
        io.read_row(r);
        lds_barrier();                           // before the next tensor lands in the staging blocks
    };

    // ---- vertical pair: waves 0..3 run the chains (channel = wave / 2, walk = wave % 2), waves 4..7 feed the ring;
    // everybody requests the first chunk of its horizontal task on the way
    if (wave >= 4) {
        BandLoader<BWD> ld;
        ld.init(p, b, c0, wave - 4, lane);
        ld.run(region, prefetch);
    } else {
        uint32_t* tile = tiles + (wave >> 1) * TILE_WORDS;
        if (wave & 1) vertical_chain<true, SAVE, BWD>(p, region, tile, b, c0 + (wave >> 1), wave, lane, prefetch);
        else vertical_chain<false, SAVE, BWD>(p, region, tile, b, c0 + (wave >> 1), wave, lane, prefetch);
    }

    // ---- horizontal pair
    float h = 0.f, wp0 = 0.f, wp1 = 0.f, wp2 = 0.f;
    for (int ch = 0; ch < 2; ++ch) {
        const int col0 = (REV ? 1 - ch : ch) * CS;
        // registers from request order to row order
        if (SWAP_X && ch == 1) {
            io.write_row(rd_mirror, bx);         // my chunk of x is the one the opposite walk needs now
            lds_barrier();
            io.read_row(bx);
            __builtin_amdgcn_sched_barrier(0);
        } else {
            io.to_rows(bx);
        }
        io.to_rows(bl);
        io.to_rows(bu);
        lds_barrier();                           // every task is done with its own staging block
        share_rows(b0);
        share_rows(b1);
        share_rows(b2);
        __builtin_amdgcn_sched_barrier(0);

        float cpair = 0.f, hpair = 0.f;          // first element of the pair of columns that share a word
        uint32_t yw = 0;
        uint32_t hq[4];                          // SAVE: the states of the eight columns being worked on
#pragma unroll
        for (int k = 0; k < CS; ++k) {
            const int e = REV ? CS - 1 - k : k;
            // what the other part's edge row published in the previous scan step (none before the first one)
            const int step = ch * CS + k + 1;
            float pv = 0.f;
            if (ch > 0 || k > 0) {
                u32x2 m;
                int spins = 0;
                do { m = mb_in[(k & 1) ^ 1]; } while (__builtin_amdgcn_readfirstlane((int)m.y) != step - 1 && ++spins < SPIN_LIMIT);
                pv = __uint_as_float(m.x);
            }
            const float pu = pv, pd = pv;
            uint32_t* tw = trow + ((col0 + e) >> 1);
            if ((k & 1) == 0) yw = *tw;
            const float av = elem<bf16_t>(bl, e) * elem<bf16_t>(bx, e);
            float c0 = elem<bf16_t>(b0, e), c1 = elem<bf16_t>(b1, e), c2 = elem<bf16_t>(b2, e);
            if constexpr (BWD) {
                // the edge rows publish the products that cross into the neighbouring part: tap 0 of a part's first row
                // reads the row above it, tap 2 of its last row the row below
                const float q0 = wp0 * h, q2 = wp2 * h;
                float up = from_lane_below(q2), dn = from_lane_above(q0);
                up = top_lane ? (has_up ? pu : 0.f) : up;
                dn = bot_lane ? (has_dn ? pd : 0.f) : dn;
                h = fmaf(wp1, h, av) + (up + dn);
                wp0 = img_first ? 0.f : c0;
                wp1 = c1;
                wp2 = img_last ? 0.f : c2;
                if (publishes) { const u32x2 m = {__float_as_uint(bot_lane ? wp2 * h : wp0 * h), (uint32_t)step}; mb_out[k & 1] = m; }
            } else {
                if (k == 0) {
                    const bool start = ch == 0;                  // scan step 0: its weights are never read
                    c0 = start ? 0.f : c0; c1 = start ? 0.f : c1; c2 = start ? 0.f : c2;
                }
                float up = from_lane_below(h), dn = from_lane_above(h);
                up = top_lane ? (has_up ? pu : 0.f) : up;
                dn = bot_lane ? (has_dn ? pd : 0.f) : dn;
                c0 = img_first ? 0.f : c0;
                c2 = img_last ? 0.f : c2;
                h = fmaf(c0, up, fmaf(c1, h, fmaf(c2, dn, av)));
                if (publishes) { const u32x2 m = {__float_as_uint(h), (uint32_t)step}; mb_out[k & 1] = m; }
            }
            const float cv = elem<bf16_t>(bu, e) * h;
            if ((k & 1) == 0) { cpair = cv; hpair = h; }
            else {
                // columns e and e ^ 1 are complete: their word of the tile takes both
                const float clo = (e & 1) ? cpair : cv, chi = (e & 1) ? cv : cpair;
                *tw = pack_bf16x2(lo16(yw) + clo, hi16(yw) + chi);
                if constexpr (SAVE) hq[(e >> 1) & 3] = pack_bf16x2((e & 1) ? hpair : h, (e & 1) ? h : hpair);
            }
            if constexpr (SAVE) {
                // eight columns of states are complete: they wait in the staging block (idle while a chunk is worked on)
                if ((k & 7) == 7) { const u32x4 v = {hq[0], hq[1], hq[2], hq[3]}; io.rd[e >> 3] = v; }
            }
            __builtin_amdgcn_sched_barrier(0);       // one scan step after the other: nothing is gained by mixing them, registers are lost
            if ((k & 7) == 7 && ch == 0) {
                // columns 8q..8q+7 are consumed: their registers take instruction q of the next chunk (x: unless it is swapped)
                issue_slot(1, e >> 3, !SWAP_X);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if constexpr (SAVE) io.store_staged(hb, col0 * 2);
    }
}

template <bool SAVE, bool BWD>
__global__ void __launch_bounds__(512) fwd_pair_kernel(FwdParams p) {
    extern __shared__ uint32_t lds[];
    uint32_t* tiles = lds;
    char* region = (char*)(lds + 2 * TILE_WORDS);
    float* mailbox = (float*)(region + REGION_B);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int pairs = p.C / 2;
    const unsigned item = xcd_contiguous_item(blockIdx.x, gridDim.x);
    const int b = item / pairs;
    const int c0 = (item - b * pairs) * 2;

    if (threadIdx.x < MAILBOX_FLOATS) mailbox[threadIdx.x] = 0.f;         // scan steps count from 1: no entry is valid yet

    // wave -> horizontal task (channel = wave / 4, direction slot = (wave / 2) % 2, part = wave % 2); the task of
    // direction slot 0 walks the columns from the left in the forward scan and from the right in the reverse sweep
    if ((((wave >> 1) & 1) == 0) != BWD) pair_body<false, SAVE, BWD>(p, tiles, region, mailbox, b, c0, wave, lane);
    else pair_body<true, SAVE, BWD>(p, tiles, region, mailbox, b, c0, wave, lane);

    // ---- the tiles hold the rounded output: copy them out, one row per request
    lds_barrier();
    {
        char* Y = (char*)p.y + ((size_t)b * p.C + c0) * PLANE_B;
        for (int r = wave; r < 2 * PH; r += 8) {
            const uint32_t v = tiles[r * TPITCH + lane];
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
    hipLaunchKernelGGL(k, dim3((unsigned)((size_t)p.B * (p.C / 2))), dim3(512), LDS_BYTES, s, p);
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
