// Forward GSPN scan (global, normalised weights) on maps beyond the stream kernel's reach: up to 2048 image rows and
// lines of up to 2048 positions -- the 1024x1024 shapes of the paper's scaling experiments
// (Sec. 5.1) and high-resolution generation (App. B).  Same structure as the stream kernel (one workgroup per
// (image, channel) plane, wave-owned lines in registers, y merged in place in global memory in a fixed order by the
// plane's owner), split into two launches because the two halves want different workgroup shapes:
//   1. vertical pair: two waves per plane, each holding a whole image row (up to 64 B per lane and tensor), which
//      needs the register file of a small workgroup;
//   2. horizontal pair: one image row per lane, so 1024 rows are sixteen waves in lock-step (one workgroup barrier per
//      scan step, edge rows through an LDS mailbox), which leaves 128 registers per lane: 64 B of every row per
//      request.
//      request.  Beyond 1024 rows a lane holds two adjacent rows and 16 B of each per request (forward only).
// Launch 2 reads the y of launch 1 (stream order).  h_save and, up to 1024 rows, the reverse sweep of the two-pass
// backward run on the same kernels (template flags SAVE, BWD), and so do, up to 1024 rows, GSPN-local and logits calls
// (LOCAL, LOGITS: the stretch bookkeeping and the softmax of the line objects, as in the stream kernel).
#pragma once
#include "gspn_fwd_stream_impl.hpp"

namespace gspn {

namespace {

template <typename T, int V, int PF, bool BWD, bool SAVE, bool LOCAL, bool LOGITS>
__global__ void __launch_bounds__(128) stream_big_vertical_kernel(FwdParams p) {
    static_assert(LOCAL || !LOGITS, "logits run on the local instantiations (a global scan is one stretch)");
    const int H = p.H;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const unsigned item = xcd_contiguous_item(blockIdx.x, gridDim.x);
    const int b = item / p.C, c = item - b * p.C;
    const int has_tb = (p.mask >> 0) & 1, has_bt = (p.mask >> 1) & 1;
    if (has_tb + has_bt == 2) {
        // each wave first stores its half of y, then, after a barrier, read-modify-writes the other half
        const int split = (H + 1) / 2;
        if (wave == 0) {
            VStream<T, V, PF, false, LOCAL, LOGITS, BWD, SAVE> v; v.init(p, b, c, lane);
            v.template run<false>(0, split);
            __syncthreads();
            v.template run<true>(split, H);
        } else {
            VStream<T, V, PF, true, LOCAL, LOGITS, BWD, SAVE> v; v.init(p, b, c, lane);
            v.template run<false>(0, H - split);
            __syncthreads();
            v.template run<true>(H - split, H);
        }
    } else if (wave == 0) {
        if ((has_tb != 0) != BWD) { VStream<T, V, PF, false, LOCAL, LOGITS, BWD, SAVE> v; v.init(p, b, c, lane); v.template run<false>(0, H); }
        else                      { VStream<T, V, PF, true, LOCAL, LOGITS, BWD, SAVE> v;  v.init(p, b, c, lane); v.template run<false>(0, H); }
    }
}

constexpr int BIG_WAVES = 16;

// wrote: y already holds the sum of the vertical directions
template <typename T, int CS, bool BWD, bool SAVE, bool LOCAL, bool LOGITS>
__global__ void __launch_bounds__(64 * BIG_WAVES) stream_big_horizontal_kernel(StreamArgs a, int wrote_in) {
    __shared__ float mailbox[BIG_WAVES * 4];
    using HS = HStream<T, CS, false, LOCAL, LOGITS, BWD, SAVE>;
    __shared__ __attribute__((aligned(16))) char stage[BIG_WAVES * HS::STAGE_BYTES];
    const FwdParams& p = a.p;
    const int W = p.W;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const unsigned item = xcd_contiguous_item(blockIdx.x, gridDim.x);
    const int b = item / p.C, c = item - b * p.C;
    bool wrote = wrote_in != 0;
    for (int dsel = 0; dsel < 2; ++dsel) {
        if (!((p.mask >> (2 + dsel)) & 1)) continue;
        if (threadIdx.x < BIG_WAVES * 4) mailbox[threadIdx.x] = 0.f;
        __syncthreads();                        // y of the previous direction visible, mailbox cleared
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
// maps of more than 1024 rows: two adjacent image rows per lane, forward scan only
// ---------------------------------------------------------------------------
// The same lock-step (one barrier per scan step, the edge rows of a wave through the mailbox), with the rows 2l and 2l+1
// of a wave's 128 in lane l; 128 registers per lane then hold 16 B of every row per request.
template <typename T, bool REV, bool SAVE>
struct HStream2 {
    static constexpr int CS = 16 / (int)sizeof(T);
    rsrc_t xb, lb, ub, w0b, w1b, w2b, yb, hb;
    uint32_t voff[2];
    int nchunks;
    float* mb_out;
    const float* mb_up;
    const float* mb_dn;
    bool edge, top_lane, bot_lane, has_up, has_dn, img_first, img_last;
    float h[2];
    uint32_t bx[2][4], bl[2][4], bu[2][4], b0[2][4], b1[2][4], b2[2][4], by[2][4];

    __device__ __forceinline__ void init(const FwdParams& p, float* mailbox, int parts, int b, int c, int part, int lane) {
        constexpr int d = REV ? 3 : 2;
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
#pragma unroll
        for (int r = 0; r < 2; ++r) voff[r] = (uint32_t)((part * 128 + 2 * lane + r) * W * (int)sizeof(T));
        xb = make_rsrc((const char*)p.x + plane0 * sizeof(T));
        lb = make_rsrc((const char*)p.lam + (slot_c + plane0) * sizeof(T));
        ub = make_rsrc((const char*)p.u + (slot_c + plane0) * sizeof(T));
        w0b = make_rsrc(wbase); w1b = make_rsrc(wbase + plane_bytes); w2b = make_rsrc(wbase + 2 * plane_bytes);
        yb = make_rsrc((char*)p.y + plane0 * sizeof(T));
        hb = make_rsrc(SAVE ? (char*)p.hs + ((size_t)d * planes * HW + plane0) * sizeof(T) : (char*)p.y);
        nchunks = W / CS;
        // mailbox: [part][side: 0 first row, 1 last row][parity]
        mb_out = mailbox + part * 4 + (bot_lane ? 2 : 0);
        mb_up = mailbox + (has_up ? part - 1 : part) * 4 + 2;
        mb_dn = mailbox + (has_dn ? part + 1 : part) * 4 + 0;
        h[0] = 0.f; h[1] = 0.f;
    }
    __device__ __forceinline__ int chunk_col(int c) const { return (REV ? nchunks - 1 - c : c) * CS; }

    template <bool RMW>
    __device__ __forceinline__ void issue(int c) {
        const int so = chunk_col(c) * (int)sizeof(T);
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            ld_buf<16>(xb, voff[r], so, bx[r]);
            ld_buf<16>(lb, voff[r], so, bl[r]);
            ld_buf<16>(ub, voff[r], so, bu[r]);
            ld_buf<16>(w0b, voff[r], so, b0[r]);
            ld_buf<16>(w1b, voff[r], so, b1[r]);
            ld_buf<16>(w2b, voff[r], so, b2[r]);
            if constexpr (RMW) ld_buf<16>(yb, voff[r], so, by[r]);
        }
    }

    template <bool RMW>
    __device__ __forceinline__ void compute(int c) {
        float ypair[2] = {0.f, 0.f}, epair[2] = {0.f, 0.f};      // bf16: first element of the pair being assembled
#pragma unroll
        for (int k = 0; k < CS; ++k) {
            const int e = REV ? CS - 1 - k : k;
            const int par = k & 1;                               // CS is even: parity of the scan step
            const float pu = mb_up[par ^ 1];
            const float pd = mb_dn[par ^ 1];
            const bool start = (c == 0) && (k == 0);             // scan step 0: its weights are never used
            float w0[2], w1[2], w2[2], av[2];
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                w0[r] = elem<T>(b0[r], e); w1[r] = elem<T>(b1[r], e); w2[r] = elem<T>(b2[r], e);
                if (k == 0) { w0[r] = start ? 0.f : w0[r]; w1[r] = start ? 0.f : w1[r]; w2[r] = start ? 0.f : w2[r]; }
                av[r] = elem<T>(bl[r], e) * elem<T>(bx[r], e);
            }
            float up = from_lane_below(h[1]), dn = from_lane_above(h[0]);
            up = top_lane ? (has_up ? pu : 0.f) : up;
            dn = bot_lane ? (has_dn ? pd : 0.f) : dn;
            // a tap that points outside the image takes nothing, whatever the tensor holds there
            w0[0] = img_first ? 0.f : w0[0];
            w2[1] = img_last ? 0.f : w2[1];
            const float n0 = fmaf(w0[0], up, fmaf(w1[0], h[0], fmaf(w2[0], h[1], av[0])));
            const float n1 = fmaf(w0[1], h[0], fmaf(w1[1], h[1], fmaf(w2[1], dn, av[1])));
            h[0] = n0; h[1] = n1;
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                float yv = elem<T>(bu[r], e) * h[r];
                if constexpr (RMW) yv += elem<T>(by[r], e);
                if constexpr (sizeof(T) == 4) {
                    by[r][e] = __float_as_uint(yv);
                    if constexpr (SAVE) bx[r][e] = __float_as_uint(h[r]);     // x of this element is consumed: its word takes h
                } else {
                    // elements e and e^1 share a word; the pair is complete on every second step
                    if ((k & 1) == 0) { ypair[r] = yv; epair[r] = h[r]; }
                    else {
                        by[r][e >> 1] = pack_word<T>((e & 1) ? ypair[r] : yv, (e & 1) ? yv : ypair[r]);
                        if constexpr (SAVE) bx[r][e >> 1] = pack_word<T>((e & 1) ? epair[r] : h[r], (e & 1) ? h[r] : epair[r]);
                    }
                }
            }
            if (edge) mb_out[par] = bot_lane ? h[1] : h[0];
            lds_barrier();
        }
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            st_buf<16>(yb, voff[r], chunk_col(c) * (int)sizeof(T), by[r]);
            if constexpr (SAVE) st_buf<16, CP_STREAM>(hb, voff[r], chunk_col(c) * (int)sizeof(T), bx[r]);
        }
    }

    template <bool RMW>
    __device__ __forceinline__ void run() {
        issue<RMW>(0);
        for (int c = 0; c < nchunks; ++c) {
            compute<RMW>(c);
            issue<RMW>(c + 1 < nchunks ? c + 1 : c);        // clamped: redundant but in bounds at the end
        }
    }
};

template <typename T, bool SAVE>
__global__ void __launch_bounds__(64 * BIG_WAVES) stream_big_horizontal2_kernel(StreamArgs a, int wrote_in) {
    __shared__ float mailbox[BIG_WAVES * 4];
    const FwdParams& p = a.p;
    const int W = p.W;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const unsigned item = xcd_contiguous_item(blockIdx.x, gridDim.x);
    const int b = item / p.C, c = item - b * p.C;
    bool wrote = wrote_in != 0;
    for (int dsel = 0; dsel < 2; ++dsel) {
        if (!((p.mask >> (2 + dsel)) & 1)) continue;
        if (threadIdx.x < BIG_WAVES * 4) mailbox[threadIdx.x] = 0.f;
        __syncthreads();                        // y of the previous direction visible, mailbox cleared
        if (wave < a.parts) {
            if (dsel == 0) {
                HStream2<T, false, SAVE> hs; hs.init(p, mailbox, a.parts, b, c, wave, lane);
                if (wrote) hs.template run<true>(); else hs.template run<false>();
            } else {
                HStream2<T, true, SAVE> hs; hs.init(p, mailbox, a.parts, b, c, wave, lane);
                if (wrote) hs.template run<true>(); else hs.template run<false>();
            }
        } else {
            for (int st = 0; st < W; ++st) lds_barrier();    // idle wave: keep the barrier count
        }
        wrote = true;
    }
}

struct BigPlan { bool ok; int v, parts; bool two_rows; };

static BigPlan plan_big(const FwdParams& p, int dtype) {
    BigPlan t = {};
    if (p.xt) return t;
    if (p.W % 64 || p.H % 64) return t;
    const int v = p.W / 64;
    if (!(v == 4 || v == 8 || v == 16 || v == 32)) return t;
    int parts = p.H / 64;
    if (parts > BIG_WAVES) {
        // two rows per lane: up to 2048 rows, in whole blocks of 128
        if (p.H % 128 || p.H / 128 > BIG_WAVES) return t;
        if (p.kchunk > 0 || p.logits) return t;                 // (the two-row form is the global scan with normalised weights)
        parts = p.H / 128;
        t.two_rows = true;
    }
    if (parts < 1) return t;
    const int es = dtype == 0 ? 4 : 2;
    if ((size_t)p.H * p.W * es >= (1ull << 31)) return t;
    if ((size_t)p.B * p.C > 0x7fffffffull) return t;
    t.v = v; t.parts = parts; t.ok = true;
    return t;
}

template <typename T, int V, int PF, bool BWD, bool SAVE, bool LOCAL, bool LOGITS>
static hipError_t launch_vertical(const FwdParams& p, hipStream_t s) {
    hipLaunchKernelGGL((stream_big_vertical_kernel<T, V, PF, BWD, SAVE, LOCAL, LOGITS>), dim3((unsigned)((size_t)p.B * p.C)), dim3(128), 0, s, p);
    return hipGetLastError();
}

template <typename T, bool BWD, bool SAVE, bool LOCAL, bool LOGITS>
static hipError_t launch_big(const FwdParams& p, const BigPlan& t, hipStream_t s) {
    constexpr int CS = 64 / (int)sizeof(T);                     // 64 B of a row per request
    const bool vertical = (p.mask & 3u) != 0, horizontal = (p.mask & 12u) != 0;
    hipError_t e = hipSuccess;
    if (vertical) {
        switch (t.v) {
            case 4: e = launch_vertical<T, 4, 4, BWD, SAVE, LOCAL, LOGITS>(p, s); break;
            case 8: e = launch_vertical<T, 8, 4, BWD, SAVE, LOCAL, LOGITS>(p, s); break;
            case 16: e = launch_vertical<T, 16, sizeof(T) == 4 ? 2 : 4, BWD, SAVE, LOCAL, LOGITS>(p, s); break;
            default: e = launch_vertical<T, 32, sizeof(T) == 4 ? 1 : 2, BWD, SAVE, LOCAL, LOGITS>(p, s); break;
        }
        if (e != hipSuccess) return e;
    }
    if (horizontal) {
        StreamArgs a;
        a.p = p; a.parts = t.parts; a.nwaves = BIG_WAVES;
        const dim3 grid((unsigned)((size_t)p.B * p.C)), block(64 * BIG_WAVES);
        if (t.two_rows) {
            if constexpr (BWD || LOCAL) return hipErrorInvalidValue;
            else hipLaunchKernelGGL((stream_big_horizontal2_kernel<T, SAVE>), grid, block, 0, s, a, vertical ? 1 : 0);
        } else {
            hipLaunchKernelGGL((stream_big_horizontal_kernel<T, CS, BWD, SAVE, LOCAL, LOGITS>), grid, block, 0, s, a, vertical ? 1 : 0);
        }
        e = hipGetLastError();
    }
    return e;
}

// the three roles of a launch (forward, forward with h_save, reverse sweep) for one storage type and family
template <typename T, bool LOCAL, bool LOGITS>
static hipError_t launch_big_roles(const FwdParams& p, const BigPlan& t, bool reverse, hipStream_t s) {
    if (reverse) return launch_big<T, true, true, LOCAL, LOGITS>(p, t, s);
    return p.hs ? launch_big<T, false, true, LOCAL, LOGITS>(p, t, s) : launch_big<T, false, false, LOCAL, LOGITS>(p, t, s);
}
template <bool LOCAL, bool LOGITS>
static hipError_t launch_big_family(const FwdParams& p, int dtype, bool reverse, hipStream_t s) {
    const BigPlan t = plan_big(p, dtype);
    if (!t.ok || (reverse && (!p.hs || t.two_rows))) return hipErrorInvalidValue;
    if (dtype == 0) return launch_big_roles<float, LOCAL, LOGITS>(p, t, reverse, s);
    if (dtype == 2) return launch_big_roles<f16_t, LOCAL, LOGITS>(p, t, reverse, s);
    return launch_big_roles<bf16_t, LOCAL, LOGITS>(p, t, reverse, s);
}

}  // namespace
}  // namespace gspn
