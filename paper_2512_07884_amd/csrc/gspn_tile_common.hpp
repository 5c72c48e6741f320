// Device helpers shared by the register-resident ("tile") scan kernels for gfx950:
// buffer-addressed vector loads/stores, storage <-> fp32 element access, whole-wave DPP shifts and
// the LDS-only workgroup barrier.
#pragma once
#include "gspn_common.hpp"

namespace gspn {

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// ---- buffer addressing: a tensor is reached through a buffer resource (uniform base in SGPRs),
// a uniform byte offset (SGPR) and a per-lane byte offset (VGPR), so that stepping from line to
// line costs scalar adds only.  Offsets stay below 2^31 (checked on the host).
typedef __amdgpu_buffer_rsrc_t rsrc_t;
__device__ __forceinline__ rsrc_t make_rsrc(const void* base) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, 0x7fffffff, 0x00020000);
}
// CP: the cache-policy bits of the request.  CP_STREAM marks data this launch reads exactly once ("nt", non-temporal):
// the caches then give such lines up first, and what several workgroups read again -- the weights of a group
// (Sec. 4.2), which every channel of the group asks for -- stays in the L2 longer (measured on a 512x512 map with 32
// channels per group: 1.07 -> 0.96 ms).  Only for requests that cover each 128-byte line once: a line that a later
// request of the same wave touches again would be fetched twice.
constexpr int CP_STREAM = 2;
template <int NB, int CP = 0> __device__ __forceinline__ void ld_buf(rsrc_t rs, uint32_t voff, int soff, uint32_t* r) {
    soff = __builtin_amdgcn_readfirstlane(soff);   // wave-uniform by construction: keep it in an SGPR
    if constexpr (NB == 4) { r[0] = __builtin_amdgcn_raw_buffer_load_b32(rs, voff, soff, CP); }
    else if constexpr (NB == 8) { u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rs, voff, soff, CP); r[0] = v.x; r[1] = v.y; }
    else {
        static_assert(NB % 8 == 0, "vector width");
#pragma unroll
        for (int i = 0; i < NB / 16; ++i) {
            u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, voff + 16 * i, soff, CP);
            r[4 * i] = v.x; r[4 * i + 1] = v.y; r[4 * i + 2] = v.z; r[4 * i + 3] = v.w;
        }
        if constexpr (NB % 16 != 0) {                  // bursts of 8 (mod 16) bytes: the rest as one 8 B request
            u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rs, voff + (NB / 16) * 16, soff, CP);
            r[NB / 4 - 2] = v.x; r[NB / 4 - 1] = v.y;
        }
    }
}
// A store of more than 8 bytes must not be followed directly by a VALU write of its data registers.
// The compiler inserts the wait state only when the store's scalar offset is not a register (measured
// on gfx950: with an SGPR offset and the data registers rewritten by the next instruction, the upper
// half of the stored 16 B was corrupted now and then).  16 B stores therefore carry their whole
// offset in the vector offset and pass 0 as the scalar one.
template <int CP = 0> __device__ __forceinline__ void st_b128(rsrc_t rs, uint32_t voff, u32x4 v) {
    __builtin_amdgcn_raw_buffer_store_b128(v, rs, voff, 0, CP);
}
template <int NB, int CP = 0> __device__ __forceinline__ void st_buf(rsrc_t rs, uint32_t voff, int soff, const uint32_t* r) {
    if constexpr (NB == 4) { __builtin_amdgcn_raw_buffer_store_b32(r[0], rs, voff, __builtin_amdgcn_readfirstlane(soff), CP); }
    else if constexpr (NB == 8) {
        u32x2 v = {r[0], r[1]};
        __builtin_amdgcn_raw_buffer_store_b64(v, rs, voff, __builtin_amdgcn_readfirstlane(soff), CP);
    } else {
        static_assert(NB % 8 == 0, "vector width");
        const uint32_t vo = voff + (uint32_t)soff;
#pragma unroll
        for (int i = 0; i < NB / 16; ++i) {
            u32x4 v = {r[4 * i], r[4 * i + 1], r[4 * i + 2], r[4 * i + 3]};
            st_b128<CP>(rs, vo + 16 * i, v);
        }
        if constexpr (NB % 16 != 0) {
            u32x2 v = {r[NB / 4 - 2], r[NB / 4 - 1]};
            __builtin_amdgcn_raw_buffer_store_b64(v, rs, vo + (NB / 16) * 16, 0, CP);
        }
    }
}
template <int NB> __device__ __forceinline__ void st_raw(char* p, const uint32_t* r) {
    if constexpr (NB == 4) { *(uint32_t*)p = r[0]; }
    else { u32x2 v = {r[0], r[1]}; *(u32x2*)p = v; }
}

// element e of a packed register vector, widened to fp32 (e is a compile-time constant after unrolling)
template <typename T> __device__ __forceinline__ float elem(const uint32_t* r, int e) {
    if constexpr (sizeof(T) == 4) return __uint_as_float(r[e]);
    else return (e & 1) ? word_hi<T>(r[e >> 1]) : word_lo<T>(r[e >> 1]);
}
// pack V fp32 values into storage registers (round to nearest even for the 16-bit types)
template <typename T, int V> __device__ __forceinline__ void pack(const float* v, uint32_t* r) {
    if constexpr (sizeof(T) == 4) {
#pragma unroll
        for (int i = 0; i < V; ++i) r[i] = __float_as_uint(v[i]);
    } else {
        static_assert(V % 2 == 0, "vectors of 16-bit values hold an even number of elements");
#pragma unroll
        for (int i = 0; i < V / 2; ++i)
            r[i] = pack_word<T>(v[2 * i], v[2 * i + 1]);
    }
}

// whole-wave shift by one lane; lanes without a source read 0
__device__ __forceinline__ float from_lane_below(float v) {   // lane i <- lane i-1
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x138, 0xf, 0xf, true));
}
__device__ __forceinline__ float from_lane_above(float v) {   // lane i <- lane i+1
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x130, 0xf, 0xf, true));
}

// Workgroup index -> work item, for kernels whose neighbouring items read the same weight planes.
// The dispatcher deals workgroups to the chip's 8 XCDs (each with an L2 of its own) round-robin by
// index, so items i, i+1, ... would land in 8 different L2s and every L2 would fetch every group's
// weights.  This bijection on [0, n) gives XCD k the contiguous range of items
// [k*n/8 ..), so the channels of one group (Sec. 3.2: they share w) meet in one L2.
__device__ __forceinline__ unsigned xcd_contiguous_item(unsigned wg, unsigned n) {
    constexpr unsigned XCDS = 8;
    const unsigned k = wg % XCDS, j = wg / XCDS;
    const unsigned q = n / XCDS, r = n % XCDS;
    return k * q + (k < r ? k : r) + j;
}

// Workgroup barrier that orders LDS traffic only: the wave's own LDS operations are complete
// before it arrives, and the compiler may not move memory operations across it.  Unlike
// __syncthreads() it does not wait for the global loads in flight (the prefetch rings keep running).
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// One line of Eq. 1 for the lane's V positions.  `first`/`last`: the lane holds the first/last
// positions of its line, whose outer neighbour does not exist: both the neighbour value and its
// weight are forced to 0 so that nothing stored for it (NaN, Inf) can leak in.
// WAVE_LINE: the line spans the whole wave (first = lane 0, last = lane 63), so the lane shifts themselves deliver the
// zeros at its ends and only the weights need the selects.
template <int V, bool WAVE_LINE = false>
__device__ __forceinline__ void line_update(float (&h)[V], const float (&a)[V], const float (&w0)[V],
                                            const float (&w1)[V], const float (&w2)[V], bool first, bool last) {
    float lin = from_lane_below(h[V - 1]);
    float rin = from_lane_above(h[0]);
    if constexpr (!WAVE_LINE) {
        lin = first ? 0.f : lin;
        rin = last ? 0.f : rin;
    }
    const float wl = first ? 0.f : w0[0];
    const float wr = last ? 0.f : w2[V - 1];
    float hn[V];
#pragma unroll
    for (int v = 0; v < V; ++v) {
        const float l = v == 0 ? lin : h[v - 1];
        const float r = v == V - 1 ? rin : h[v + 1];
        const float c0 = v == 0 ? wl : w0[v];
        const float c2 = v == V - 1 ? wr : w2[v];
        hn[v] = fmaf(c0, l, fmaf(w1[v], h[v], fmaf(c2, r, a[v])));
    }
#pragma unroll
    for (int v = 0; v < V; ++v) h[v] = hn[v];
}

// The same for the reverse sweep of the backward pass, e_t = a_t + T_{t+1}^T e_{t+1} (chain rule on Eq. 1): every position
// multiplies its own state by the three taps of the line swept before (`wp*`, the line after it in scan order) and hands
// the products to the positions those taps read from.  h holds e of that line on entry and of this line on exit.
template <int V, bool WAVE_LINE = false>
__device__ __forceinline__ void line_update_transposed(float (&h)[V], const float (&a)[V], const float (&wp0)[V],
                                                       const float (&wp1)[V], const float (&wp2)[V], bool first, bool last) {
    float q0[V], q2[V];
#pragma unroll
    for (int v = 0; v < V; ++v) { q0[v] = wp0[v] * h[v]; q2[v] = wp2[v] * h[v]; }
    float lin = from_lane_below(q2[V - 1]);      // tap 2 of position j-1 reads position j
    float rin = from_lane_above(q0[0]);          // tap 0 of position j+1 reads position j
    if constexpr (!WAVE_LINE) {
        lin = first ? 0.f : lin;
        rin = last ? 0.f : rin;
    }
    float hn[V];
#pragma unroll
    for (int v = 0; v < V; ++v) {
        const float l = v == 0 ? lin : q2[v - 1];
        const float r = v == V - 1 ? rin : q0[v + 1];
        hn[v] = fmaf(wp1[v], h[v], a[v]) + (l + r);
    }
#pragma unroll
    for (int v = 0; v < V; ++v) h[v] = hn[v];
}

// ---- a line whose lane holds RUNS separate runs of V / RUNS adjacent positions, run i of lane l at positions
// (i * 64 + l) * V / RUNS ..: every 16-byte request of the wave then covers 1 KB of whole lines, each line once, where V
// adjacent positions per lane of more than 16 bytes make every request touch twice or four times as many lines in part.
// Between the runs the neighbour of lane 0 / lane 63 is the end of the run before / after, held by lane 63 / lane 0.
template <int NB, int CP = 0> __device__ __forceinline__ void ld_runs(rsrc_t rs, uint32_t voff, int soff, uint32_t* r) {
    static_assert(NB % 16 == 0, "runs of 16 bytes");
    soff = __builtin_amdgcn_readfirstlane(soff);
#pragma unroll
    for (int i = 0; i < NB / 16; ++i) {
        u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, voff + 1024 * i, soff, CP);
        r[4 * i] = v.x; r[4 * i + 1] = v.y; r[4 * i + 2] = v.z; r[4 * i + 3] = v.w;
    }
}
template <int NB, int CP = 0> __device__ __forceinline__ void st_runs(rsrc_t rs, uint32_t voff, int soff, const uint32_t* r) {
    static_assert(NB % 16 == 0, "runs of 16 bytes");
    const uint32_t vo = voff + (uint32_t)soff;
#pragma unroll
    for (int i = 0; i < NB / 16; ++i) {
        u32x4 v = {r[4 * i], r[4 * i + 1], r[4 * i + 2], r[4 * i + 3]};
        st_b128<CP>(rs, vo + 1024 * i, v);
    }
}
__device__ __forceinline__ float lane_value(float v, int lane) {      // lane: compile-time constant
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}
// what the positions at the ends of the runs see beside them: lin[i] left of run i, rin[i] right of it; `left_of` /
// `right_of`: the values the neighbours would read from this lane's run ends
template <int RUNS>
__device__ __forceinline__ void run_neighbours(const float (&ends_hi)[RUNS], const float (&ends_lo)[RUNS], bool first, bool last,
                                               float (&lin)[RUNS], float (&rin)[RUNS]) {
#pragma unroll
    for (int i = 0; i < RUNS; ++i) { lin[i] = from_lane_below(ends_hi[i]); rin[i] = from_lane_above(ends_lo[i]); }
#pragma unroll
    for (int i = RUNS - 1; i > 0; --i) { const float s = lane_value(ends_hi[i - 1], 63); lin[i] = first ? s : lin[i]; }
#pragma unroll
    for (int i = 0; i < RUNS - 1; ++i) { const float s = lane_value(ends_lo[i + 1], 0); rin[i] = last ? s : rin[i]; }
    lin[0] = first ? 0.f : lin[0];
    rin[RUNS - 1] = last ? 0.f : rin[RUNS - 1];
}
template <int V, int RUNS>
__device__ __forceinline__ void line_update_runs(float (&h)[V], const float (&a)[V], const float (&w0)[V],
                                                 const float (&w1)[V], const float (&w2)[V], bool first, bool last) {
    constexpr int E = V / RUNS;
    float hi[RUNS], lo[RUNS], lin[RUNS], rin[RUNS];
#pragma unroll
    for (int i = 0; i < RUNS; ++i) { hi[i] = h[i * E + E - 1]; lo[i] = h[i * E]; }
    run_neighbours<RUNS>(hi, lo, first, last, lin, rin);
    const float wl = first ? 0.f : w0[0];
    const float wr = last ? 0.f : w2[V - 1];
    float hn[V];
#pragma unroll
    for (int v = 0; v < V; ++v) {
        const float l = v % E == 0 ? lin[v / E] : h[v - 1];
        const float r = v % E == E - 1 ? rin[v / E] : h[v + 1];
        const float c0 = v == 0 ? wl : w0[v];
        const float c2 = v == V - 1 ? wr : w2[v];
        hn[v] = fmaf(c0, l, fmaf(w1[v], h[v], fmaf(c2, r, a[v])));
    }
#pragma unroll
    for (int v = 0; v < V; ++v) h[v] = hn[v];
}
template <int V, int RUNS>
__device__ __forceinline__ void line_update_transposed_runs(float (&h)[V], const float (&a)[V], const float (&wp0)[V],
                                                            const float (&wp1)[V], const float (&wp2)[V], bool first, bool last) {
    constexpr int E = V / RUNS;
    float q0[V], q2[V];
#pragma unroll
    for (int v = 0; v < V; ++v) { q0[v] = wp0[v] * h[v]; q2[v] = wp2[v] * h[v]; }
    float hi[RUNS], lo[RUNS], lin[RUNS], rin[RUNS];
#pragma unroll
    for (int i = 0; i < RUNS; ++i) { hi[i] = q2[i * E + E - 1]; lo[i] = q0[i * E]; }
    run_neighbours<RUNS>(hi, lo, first, last, lin, rin);
    float hn[V];
#pragma unroll
    for (int v = 0; v < V; ++v) {
        const float l = v % E == 0 ? lin[v / E] : q2[v - 1];
        const float r = v % E == E - 1 ? rin[v / E] : q0[v + 1];
        hn[v] = fmaf(wp1[v], h[v], a[v]) + (l + r);
    }
#pragma unroll
    for (int v = 0; v < V; ++v) h[v] = hn[v];
}

}  // namespace gspn
