// Forward GSPN scan (global, normalised weights) on maps beyond the stream kernel's reach: up to 1024 image rows and
// lines of up to 1024 (fp32) / 2048 (bf16) positions -- the 1024x1024 shapes of the paper's scaling experiments
// (Sec. 5.1) and high-resolution generation (App. B).  Same structure as the stream kernel (one workgroup per
// (image, channel) plane, wave-owned lines in registers, y merged in place in global memory in a fixed order by the
// plane's owner), split into two launches because the two halves want different workgroup shapes:
//   1. vertical pair: two waves per plane, each holding a whole image row (up to 64 B per lane and tensor), which
//      needs the register file of a small workgroup;
//   2. horizontal pair: one image row per lane, so 1024 rows are sixteen waves in lock-step (one workgroup barrier per
//      scan step, edge rows through an LDS mailbox), which leaves 128 registers per lane: 64 B of every row per
//      request.
// Launch 2 reads the y of launch 1 (stream order).  h_save and the reverse sweep of the two-pass backward run on the
// same kernels (template flags SAVE, BWD).  GSPN-local and logits calls on these maps take the generic kernels.
#include "gspn_fwd_stream_impl.hpp"

namespace gspn {

namespace {

template <typename T, int V, int PF, bool BWD, bool SAVE>
__global__ void __launch_bounds__(128) stream_big_vertical_kernel(FwdParams p) {
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
            VStream<T, V, PF, false, false, false, BWD, SAVE> v; v.init(p, b, c, lane);
            v.template run<false>(0, split);
            __syncthreads();
            v.template run<true>(split, H);
        } else {
            VStream<T, V, PF, true, false, false, BWD, SAVE> v; v.init(p, b, c, lane);
            v.template run<false>(0, H - split);
            __syncthreads();
            v.template run<true>(H - split, H);
        }
    } else if (wave == 0) {
        if ((has_tb != 0) != BWD) { VStream<T, V, PF, false, false, false, BWD, SAVE> v; v.init(p, b, c, lane); v.template run<false>(0, H); }
        else                      { VStream<T, V, PF, true, false, false, BWD, SAVE> v;  v.init(p, b, c, lane); v.template run<false>(0, H); }
    }
}

constexpr int BIG_WAVES = 16;

// wrote: y already holds the sum of the vertical directions
template <typename T, int CS, bool BWD, bool SAVE>
__global__ void __launch_bounds__(64 * BIG_WAVES) stream_big_horizontal_kernel(StreamArgs a, int wrote_in) {
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
            if ((dsel == 0) != BWD) {                    // columns walked from the left
                HStream<T, CS, false, false, false, BWD, SAVE> hs; hs.init(p, mailbox, a.parts, b, c, wave, lane);
                if (wrote) hs.template run<true>(); else hs.template run<false>();
            } else {
                HStream<T, CS, true, false, false, BWD, SAVE> hs; hs.init(p, mailbox, a.parts, b, c, wave, lane);
                if (wrote) hs.template run<true>(); else hs.template run<false>();
            }
        } else {
            for (int st = 0; st < W; ++st) lds_barrier();    // idle wave: keep the barrier count
        }
        wrote = true;
    }
}

struct BigPlan { bool ok; int v, parts; };

BigPlan plan_big(const FwdParams& p, int dtype) {
    BigPlan t = {};
    if (p.xt || p.kchunk > 0 || p.logits) return t;
    if (p.W % 64 || p.H % 64) return t;
    const int v = p.W / 64;
    if (!(v == 4 || v == 8 || v == 16 || (dtype == 1 && v == 32))) return t;
    const int parts = p.H / 64;
    if (parts < 1 || parts > BIG_WAVES) return t;
    const int es = dtype == 0 ? 4 : 2;
    if ((size_t)p.H * p.W * es >= (1ull << 31)) return t;
    if ((size_t)p.B * p.C > 0x7fffffffull) return t;
    t.v = v; t.parts = parts; t.ok = true;
    return t;
}

template <typename T, int V, int PF, bool BWD, bool SAVE>
hipError_t launch_vertical(const FwdParams& p, hipStream_t s) {
    hipLaunchKernelGGL((stream_big_vertical_kernel<T, V, PF, BWD, SAVE>), dim3((unsigned)((size_t)p.B * p.C)), dim3(128), 0, s, p);
    return hipGetLastError();
}

template <typename T, bool BWD, bool SAVE>
hipError_t launch_big(const FwdParams& p, const BigPlan& t, hipStream_t s) {
    constexpr int CS = 64 / (int)sizeof(T);                     // 64 B of a row per request
    const bool vertical = (p.mask & 3u) != 0, horizontal = (p.mask & 12u) != 0;
    hipError_t e = hipSuccess;
    if (vertical) {
        switch (t.v) {
            case 4: e = launch_vertical<T, 4, 4, BWD, SAVE>(p, s); break;
            case 8: e = launch_vertical<T, 8, 4, BWD, SAVE>(p, s); break;
            case 16: e = launch_vertical<T, 16, sizeof(T) == 4 ? 2 : 4, BWD, SAVE>(p, s); break;
            default:
                if constexpr (sizeof(T) == 2) { e = launch_vertical<T, 32, 2, BWD, SAVE>(p, s); break; }
                return hipErrorInvalidValue;
        }
        if (e != hipSuccess) return e;
    }
    if (horizontal) {
        StreamArgs a;
        a.p = p; a.parts = t.parts; a.nwaves = BIG_WAVES;
        hipLaunchKernelGGL((stream_big_horizontal_kernel<T, CS, BWD, SAVE>), dim3((unsigned)((size_t)p.B * p.C)), dim3(64 * BIG_WAVES), 0, s,
                           a, vertical ? 1 : 0);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace

bool stream_big_applicable(const FwdParams& p, int dtype) { return plan_big(p, dtype).ok; }

hipError_t launch_stream_big(const FwdParams& p, int dtype, bool reverse, hipStream_t s) {
    const BigPlan t = plan_big(p, dtype);
    if (!t.ok || (reverse && !p.hs)) return hipErrorInvalidValue;
    if (dtype == 0) {
        if (reverse) return launch_big<float, true, true>(p, t, s);
        return p.hs ? launch_big<float, false, true>(p, t, s) : launch_big<float, false, false>(p, t, s);
    }
    if (reverse) return launch_big<bf16_t, true, true>(p, t, s);
    return p.hs ? launch_big<bf16_t, false, true>(p, t, s) : launch_big<bf16_t, false, false>(p, t, s);
}

}  // namespace gspn
