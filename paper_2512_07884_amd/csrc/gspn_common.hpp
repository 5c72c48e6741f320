// Shared device helpers and launch parameter blocks for the GSPN scan kernels (gfx950).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <mutex>

namespace gspn {

typedef uint16_t bf16_t;  // raw bfloat16 bit pattern

// ---- storage <-> fp32 ------------------------------------------------------
__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// round-to-nearest-even, NaN stays NaN: gfx950 converts in hardware (v_cvt_pk_bf16_f32, two values per
// instruction), which is what these casts compile to
typedef __bf16 bf16x2_hw __attribute__((ext_vector_type(2)));
typedef float f32x2_hw __attribute__((ext_vector_type(2)));
__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return __builtin_bit_cast(bf16_t, (__bf16)f); }
// two values into one 32-bit word: `lo` in bits 0-15, `hi` in bits 16-31
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    const f32x2_hw v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_hw));
}


// IEEE binary16 storage: a type of its own, so that overloads and templates tell it from bf16.  Conversions are the
// hardware's (v_cvt_f32_f16 / v_cvt_f16_f32: round to nearest even, subnormals kept, beyond 65504 -> inf).
struct f16_t { uint16_t bits; };
typedef _Float16 f16x2_hw __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float f16_to_f32(f16_t v) { return (float)__builtin_bit_cast(_Float16, v.bits); }
__device__ __forceinline__ f16_t f32_to_f16(float f) { f16_t r; r.bits = __builtin_bit_cast(uint16_t, (_Float16)f); return r; }
__device__ __forceinline__ uint32_t pack_f16x2(float lo, float hi) {
    const f32x2_hw v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2_hw));
}

// a 32-bit word of two 16-bit storage values (T = bf16_t or f16_t): the value in bits 0-15 / bits 16-31, and the way back
template <typename T> __device__ __forceinline__ float word_lo(uint32_t w) {
    if constexpr (__is_same(T, f16_t)) { f16_t v; v.bits = (uint16_t)w; return f16_to_f32(v); }
    else return __uint_as_float(w << 16);
}
template <typename T> __device__ __forceinline__ float word_hi(uint32_t w) {
    if constexpr (__is_same(T, f16_t)) { f16_t v; v.bits = (uint16_t)(w >> 16); return f16_to_f32(v); }
    else return __uint_as_float(w & 0xffff0000u);
}
template <typename T> __device__ __forceinline__ uint32_t pack_word(float lo, float hi) {
    if constexpr (__is_same(T, f16_t)) return pack_f16x2(lo, hi);
    else return pack_bf16x2(lo, hi);
}

__device__ __forceinline__ float ldf(const float* p) { return *p; }
__device__ __forceinline__ float ldf(const bf16_t* p) { return bf16_to_f32(*p); }
__device__ __forceinline__ float ldf(const f16_t* p) { return f16_to_f32(*p); }
__device__ __forceinline__ void stf(float* p, float v) { *p = v; }
__device__ __forceinline__ void stf(bf16_t* p, float v) { *p = f32_to_bf16(v); }
__device__ __forceinline__ void stf(f16_t* p, float v) { *p = f32_to_f16(v); }

// ---- weights from raw logits (Sec. 3.2: the weights are normalised so that every row of T_i sums to 1) ----
// Softmax over the three taps of one position, in place.  A tap whose neighbour lies outside the line
// (out0: tap 0, out2: tap 2) takes no part and gets weight 0, whatever its logit holds.
__device__ __forceinline__ void softmax3(float& z0, float& z1, float& z2, bool out0, bool out2) {
    const float ninf = -__builtin_huge_valf();
    z0 = out0 ? ninf : z0;
    z2 = out2 ? ninf : z2;
    const float m = fmaxf(z1, fmaxf(z0, z2));
    // hardware exp2 on x * log2(e): the rounding of the product is a relative error |x| * 6e-8 on a term of size
    // e^x (x <= 0 here), at most 2.2e-8 absolute on a weight
    const float e0 = __expf(z0 - m), e1 = __expf(z1 - m), e2 = __expf(z2 - m);   // exp(-inf) = 0
    const float r = 1.0f / (e0 + e1 + e2);
    z0 = e0 * r; z1 = e1 * r; z2 = e2 * r;
}
// Gradient w.r.t. the logits from the gradient w.r.t. the normalised weights, in place: linear in g, so it
// may be applied to partial sums over channels.  w = 0 (masked tap, line without predecessor) gives 0.
__device__ __forceinline__ void softmax3_grad(float& g0, float& g1, float& g2, float w0, float w1, float w2) {
    const float dot = fmaf(w0, g0, fmaf(w1, g1, w2 * g2));
    g0 = w0 * (g0 - dot); g1 = w1 * (g1 - dot); g2 = w2 * (g2 - dot);
}

// ---- direction geometry ----------------------------------------------------
// Direction d scans S lines of length L.  Element (scan step t, position j) of a
// [H][W] plane sits at  line(t)*stride_s + j*stride_j  with line(t) = t or S-1-t.
struct DirGeom {
    int S, L, stride_s, stride_j, reversed;
};
__host__ __device__ __forceinline__ DirGeom dir_geom(int d, int H, int W) {
    DirGeom g;
    if (d < 2) { g.S = H; g.L = W; g.stride_s = W; g.stride_j = 1; }
    else       { g.S = W; g.L = H; g.stride_s = 1; g.stride_j = W; }
    g.reversed = d & 1;
    return g;
}

// ---- GSPN-local (Sec. 3.2): propagation confined to stretches of kchunk lines ------------------
// The scan axis is cut at image lines 0, kchunk, 2*kchunk, ... (the same cut for a direction and its
// reverse).  A line that starts a stretch in scan order has no predecessor: its state is lambda*x and
// its weights are never read.  kchunk <= 0 means one stretch (the global scan).
// t = scan step (0 = first line visited), S = lines along the scan axis.
__host__ __device__ __forceinline__ bool starts_stretch(int t, int S, int reversed, int kchunk) {
    if (t == 0) return true;
    if (kchunk <= 0) return false;
    const int r = reversed ? S - 1 - t : t;               // image line
    return reversed ? (r + 1) % kchunk == 0 : r % kchunk == 0;
}
// bit i set <=> line i starts a stretch in scan order; i is the scan step (by_step) or the image line.  S <= 64.
inline uint64_t stretch_start_bits(int S, int reversed, int kchunk, bool by_step) {
    uint64_t m = 0;
    for (int t = 0; t < S && t < 64; ++t)
        if (starts_stretch(t, S, reversed, kchunk)) m |= 1ull << (by_step ? t : (reversed ? S - 1 - t : t));
    return m;
}

// The same predicate as a running counter for kernels that walk the scan steps in order: `start()` is
// called once per scan step and tells whether that step starts a stretch (uniform scalar work only).
struct StretchWalk {
    int until, gap, k;
    // S lines along the scan axis; kchunk >= 1
    __device__ __forceinline__ void init(int S, int reversed, int kchunk) {
        if (kchunk <= 0) kchunk = 1 << 30;                // the global scan is one stretch
        k = kchunk;
        until = 0;                                        // scan step 0 starts a stretch
        gap = (reversed && S % kchunk) ? S % kchunk : kchunk;   // a reversed scan begins with the short last stretch
    }
    __device__ __forceinline__ bool start() {
        const bool s = until == 0;
        if (s) { until = gap; gap = k; }
        --until;
        return s;
    }
};

// ... and for kernels that walk the scan steps against the scan order (backward sweeps): `start(at_step0)`
// is called once per scan step, from the last one down to step 0.
struct StretchWalkBack {
    int phase, k, rev;
    __device__ __forceinline__ void init(int S, int reversed, int kchunk) {
        if (kchunk <= 0) kchunk = 1 << 30;                // the global scan is one stretch
        k = kchunk; rev = reversed;
        // position of the last scan step inside its stretch, counted so that 0 = "starts a stretch"
        phase = reversed ? 1 % kchunk : (S - 1) % kchunk;
    }
    __device__ __forceinline__ bool start(bool at_step0) {
        const bool s = phase == 0 || at_step0;
        if (rev) phase = (phase + 1 == k) ? 0 : phase + 1;
        else phase = (phase == 0) ? k - 1 : phase - 1;
        return s;
    }
};

struct FwdParams {
    const void* x; const void* w; const void* lam; const void* u;
    void* y; void* hs;
    int B, C, H, W, G, cpg;
    unsigned mask;
    int shared;   // 1: w/lam/u have a single direction slot
    int kchunk;   // GSPN-local stretch length; 0: global scan
    int logits;   // 1: w holds raw logits, normalised on the way in (softmax3)
    const void* xt;   // transposed-horizontal layout: x stored [B][C][W][H]; NULL otherwise.  Slots 2 and 3 of
                      // w, lam, u are then stored transposed as well ([..][W][H])
};

struct BwdParams {
    const void* gy; const void* x; const void* w; const void* lam; const void* u; const void* hs;
    void* gx; void* gw; void* glam; void* gu;
    int B, C, H, W, G, cpg;
    unsigned mask;
    int shared;
    int kchunk;   // GSPN-local stretch length; 0: global scan
    int logits;   // 1: w holds raw logits and gw receives the gradient w.r.t. them
};

// Raises a kernel's dynamic-LDS limit (up to the 160 KB of a gfx950 CU) once per (kernel, device).
// Later calls are a table lookup, so that a launch made while the stream is being captured issues
// no attribute call.  Host only.
inline hipError_t allow_dynamic_lds(const void* kernel, int bytes) {
    struct Seen { const void* kernel; int device; };
    static Seen seen[512];
    static int n = 0;
    static std::mutex mu;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> guard(mu);
    for (int i = 0; i < n; ++i)
        if (seen[i].kernel == kernel && seen[i].device == dev) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e != hipSuccess) return e;
    if (n < 512) seen[n++] = Seen{kernel, dev};
    return hipSuccess;
}

// launchers implemented by the kernel files; return hipError_t of the launch
hipError_t launch_fwd_generic(const FwdParams& p, int dtype, hipStream_t s);
hipError_t launch_bwd_generic(const BwdParams& p, int dtype, hipStream_t s);
hipError_t launch_fwd_tile(const FwdParams& p, int dtype, hipStream_t s);
bool fwd_tile_applicable(const FwdParams& p, int dtype);
hipError_t launch_fwd_plane(const FwdParams& p, int dtype, hipStream_t s);
bool fwd_plane_applicable(const FwdParams& p, int dtype);
hipError_t launch_fwd_stream(const FwdParams& p, int dtype, hipStream_t s);
bool fwd_stream_applicable(const FwdParams& p, int dtype);
hipError_t launch_fwd_pair(const FwdParams& p, int dtype, hipStream_t s);
bool fwd_pair_applicable(const FwdParams& p, int dtype);
// GSPN-local with one workgroup per (plane, stretch): for calls with few planes (gspn_fwd_chunk.hip)
hipError_t launch_fwd_chunk(const FwdParams& p, int dtype, hipStream_t s);
bool fwd_chunk_applicable(const FwdParams& p, int dtype);
hipError_t launch_bwd_tile(const BwdParams& p, int dtype, hipStream_t s);
bool bwd_tile_applicable(const BwdParams& p, int dtype);
hipError_t launch_bwd_plane(const BwdParams& p, int dtype, hipStream_t s);
bool bwd_plane_applicable(const BwdParams& p, int dtype);
hipError_t launch_bwd_twopass(const BwdParams& p, int dtype, hipStream_t s);
bool bwd_twopass_applicable(const BwdParams& p, int dtype);
// clears `bytes` (a multiple of 16) of device memory with a kernel on stream s (no memset node: capturable)
hipError_t launch_zero_fill(void* p, size_t bytes, hipStream_t s);

// the per-line-launch comparator (gspn_unfused.hip): never dispatched to, timed against the fused kernels by bench.py
size_t unfused_workspace_bytes(int B, int C, int H, int W);
hipError_t launch_fwd_unfused(const FwdParams& p, int dtype, void* workspace, hipStream_t s);

// compressive proxy projection (gspn_proxy.hip): out[b][m][n] = sum_k P[m][k] in[b][k][n]
hipError_t launch_proxy_project(const void* in, const void* P, void* out, int B, int K, int M, int N, int dtype, hipStream_t s);
bool proxy_mfma_applicable(int B, int K, int M, int N, int dtype);
// ... and its gradients: gin[b][k][n] = sum_m P[m][k] gout[b][m][n] (NULL: skipped); gP[m][k] = sum_{b,n} gout[b][m][n] in[b][k][n]
// (fp32, NULL: skipped; partial = B*M*K floats of the caller's)
hipError_t launch_proxy_project_bwd(const void* gout, const void* in, const void* P, void* gin, float* gP, float* partial,
                                    int B, int K, int M, int N, int dtype, hipStream_t s);

// ... with the per-image sums in a static device array of PROXY_SCRATCH_FLOATS floats (B*M*K must fit): no workspace argument
constexpr size_t PROXY_SCRATCH_FLOATS = (size_t)1 << 20;   // 4 MiB per GPU
hipError_t launch_proxy_project_bwd_static(const void* gout, const void* in, const void* P, void* gin, float* gP,
                                           int B, int K, int M, int N, int dtype, hipStream_t s);

// dispatch (gspn_dispatch.hip): picks the kernel family for the arguments
hipError_t launch_fwd(const FwdParams& p, int dtype, hipStream_t s);
hipError_t launch_bwd(const BwdParams& p, int dtype, hipStream_t s);
const char* fwd_plan_name(const FwdParams& p, int dtype);
const char* bwd_plan_name(const BwdParams& p, int dtype);
bool staged_stream_enabled();  // false while GSPN_STREAM_NO_STAGED=1 keeps the whole-line stream kernel out (testing aid)
bool pair_kernels_enabled();   // false while GSPN_FWD_NO_PAIR=1 keeps the two-channel kernels out (testing aid)
bool stream_two_channels_forced();   // true while GSPN_STREAM_TWO_CHANNELS=1 pairs the channels whatever the number of planes (testing aid)
bool stream_two_channels_enabled();  // false while GSPN_STREAM_ONE_CHANNEL=1 keeps the stream kernel that shares a group's weights between two channels out (testing aid)
bool chunk_kernels_enabled();  // false while GSPN_FWD_NO_CHUNK=1 keeps the per-stretch kernels of GSPN-local out (testing aid)
void reload_env_knobs();   // re-reads the GSPN_* testing aids from the environment (they are read once otherwise)

}  // namespace gspn
