// Compressive proxy projections (Sec. 4.2, "Compressive Proxy Dimension"): the 1x1 convolutions over the channel
// axis that take x from C channels down to C_proxy before the scan and back up to C after it,
//
//     out[b][m][n] = sum_k P[m][k] * in[b][k][n]        n = pixel (h*W + w), contiguous
//
// i.e. per image a dense [M x K] by [K x N] product with N = H*W: down-projection M = C_proxy, K = C; back up
// M = C, K = C_proxy.  This is the one dense contraction around the scan, so it runs on the matrix cores in bf16
// (v_mfma_f32_32x32x16_bf16, or 32x32x8 when K is not a multiple of 16; fp32 accumulation); with C_proxy << C it moves far more bytes than it computes and
// is bound by reading `in` (down) or writing `out` (up) once.
//
// Mapping: one wave owns a tile of 32 output channels x 256 pixels.  The MFMA wants both operands packed along
// k, while `in` is contiguous along n: each lane loads, for its k-rows (lanes 0-31 the first half of the k-step,
// lanes 32-63 the second), 16 B = 8 consecutive pixels (a wave reads whole 512 B row segments), and regroups them in registers
// with byte permutes into eight k-packed B operands, one per pixel of its eight.  Eight MFMAs per k-step then give
// each lane, per output row it holds, eight consecutive pixels: the result leaves as 16 B stores of whole segments.
// Shapes the MFMA path does not take (fp32 storage, K or N not multiples of 8) run a plain FMA kernel.
#include "gspn_tile_common.hpp"

namespace gspn {

namespace {

typedef short bf16x4_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef _Float16 f16x4_t __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));

// one 32x32 matrix-core step over 8 / 16 k values of 16-bit operands (T = bf16_t or f16_t; the two formats share the
// operand layout), fp32 accumulation
template <typename T> __device__ __forceinline__ f32x16_t mfma_k8(const u32x2& a, const u32x2& b, const f32x16_t& c) {
    if constexpr (__is_same(T, f16_t)) return __builtin_amdgcn_mfma_f32_32x32x8f16(__builtin_bit_cast(f16x4_t, a), __builtin_bit_cast(f16x4_t, b), c, 0, 0, 0);
    else return __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(__builtin_bit_cast(bf16x4_t, a), __builtin_bit_cast(bf16x4_t, b), c, 0, 0, 0);
}
template <typename T> __device__ __forceinline__ f32x16_t mfma_k16(const u32x4& a, const u32x4& b, const f32x16_t& c) {
    if constexpr (__is_same(T, f16_t)) return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
    else return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

// KS = k values per MFMA: 8 (v_mfma_f32_32x32x8_bf16_1k) or 16 (v_mfma_f32_32x32x16_bf16, K a multiple of 16).
// A lane feeds KS/2 consecutive k: lanes 0-31 the first half of the k-step, lanes 32-63 the second.
// PT: the matrix is applied transposed, out[b][m][n] = sum_k P[k][m] * in[b][k][n] with P stored [K][M] (the gradient of
// the projection w.r.t. its input): a lane then gathers its KS/2 values of P with 2-byte loads a row apart (P is small
// and stays in cache).
template <typename T, int KS, bool PT = false>
__global__ void __launch_bounds__(256) proxy_mfma_kernel(const T* __restrict__ in, const T* __restrict__ P,
                                                         T* __restrict__ out, int B, int K, int M, int N,
                                                         int ntiles, int mtiles) {
    constexpr int KL = KS / 2;                                 // k-rows per lane and k-step
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    // work item -> (image, pixel tile, row tile), row tile fastest: the waves of a workgroup take the row tiles of
    // one pixel tile (they read the same `in`, which then comes out of L1) or, with a single row tile,
    // neighbouring pixel tiles
    const long item = (long)blockIdx.x * 4 + wave;
    const long per_image = (long)ntiles * mtiles;
    if (item >= (long)B * per_image) return;
    const int b = (int)(item / per_image);
    const int rem = (int)(item - (long)b * per_image);
    const int nt = rem / mtiles, mt = rem - nt * mtiles;
    const int jl = lane & 31, kh = lane >> 5;                  // pixel group of the lane, which half of the k-step
    const int n_lane = nt * 256 + jl * 8;                      // first of the lane's eight pixels
    const bool n_ok = n_lane < N;                              // N is a multiple of 8: all eight or none
    const int m_lane = mt * 32 + jl;                           // row of P this lane feeds as the A operand
    const bool m_ok = m_lane < M;

    const rsrc_t inb = make_rsrc(in + (size_t)b * K * N);
    const rsrc_t pb = make_rsrc(P);
    f32x16_t acc[8];
#pragma unroll
    for (int v = 0; v < 8; ++v)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[v][r] = 0.f;

    struct Step { u32x4 q[KL]; uint32_t pa[KL / 2]; };         // the lane's k-rows of `in`; P[m_lane][its k values]
    auto fetch = [&](int k0, Step& t) {
        const int kr = k0 + KL * kh;
#pragma unroll
        for (int kk = 0; kk < KL; ++kk) {
            t.q[kk] = u32x4{0, 0, 0, 0};
            if (n_ok) t.q[kk] = __builtin_amdgcn_raw_buffer_load_b128(inb, (uint32_t)(((size_t)(kr + kk) * N + n_lane) * 2), 0, 0);
        }
#pragma unroll
        for (int i = 0; i < KL / 2; ++i) t.pa[i] = 0;
        if (m_ok && PT) {
#pragma unroll
            for (int i = 0; i < KL / 2; ++i) {
                const uint32_t lo = (uint32_t)__builtin_amdgcn_raw_buffer_load_b16(pb, (uint32_t)(((size_t)(kr + 2 * i) * M + m_lane) * 2), 0, 0);
                const uint32_t hi = (uint32_t)__builtin_amdgcn_raw_buffer_load_b16(pb, (uint32_t)(((size_t)(kr + 2 * i + 1) * M + m_lane) * 2), 0, 0);
                t.pa[i] = (lo & 0xffffu) | (hi << 16);
            }
        } else if (m_ok) {
            const uint32_t po = (uint32_t)(((size_t)m_lane * K + kr) * 2);
            if constexpr (KS == 8) { const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(pb, po, 0, 0); t.pa[0] = v.x; t.pa[1] = v.y; }
            else { const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(pb, po, 0, 0); t.pa[0] = v.x; t.pa[1] = v.y; t.pa[2] = v.z; t.pa[3] = v.w; }
        }
    };
    auto multiply = [&](const Step& t) {
#pragma unroll
        for (int v = 0; v < 8; ++v) {
            // pixel v of the lane's eight, its k values packed in pairs: element v sits in word v/2, half v%2
            const uint32_t sel = (v & 1) ? 0x07060302u : 0x05040100u;
            uint32_t bb[KL / 2];
#pragma unroll
            for (int i = 0; i < KL / 2; ++i) bb[i] = __builtin_amdgcn_perm(t.q[2 * i + 1][v >> 1], t.q[2 * i][v >> 1], sel);
            if constexpr (KS == 8) {
                const u32x2 av = {t.pa[0], t.pa[1]}, bv = {bb[0], bb[1]};
                acc[v] = mfma_k8<T>(av, bv, acc[v]);
            } else {
                const u32x4 av = {t.pa[0], t.pa[1], t.pa[2], t.pa[3]}, bv = {bb[0], bb[1], bb[2], bb[3]};
                acc[v] = mfma_k16<T>(av, bv, acc[v]);
            }
        }
    };
    // the operands of the next k-step are requested before the current one is multiplied (past the end the last
    // step is requested again: redundant, in bounds, never multiplied)
    Step cur, nxt;
    const int last = K - KS;
    fetch(0, cur);
    for (int k0 = 0; k0 < K; k0 += KS) {
        fetch(min(k0 + KS, last), nxt);
        multiply(cur);
        cur = nxt;
    }

    // accumulator register r of a lane: output row 8*(r/4) + 4*(lane/32) + r%4 of the tile, column = the lane's pixel
    if (!n_ok) return;
    const rsrc_t ob = make_rsrc(out + (size_t)b * M * N);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int m = mt * 32 + 8 * (r >> 2) + 4 * kh + (r & 3);
        if (m < M) {
            const u32x4 o = {pack_word<T>(acc[0][r], acc[1][r]), pack_word<T>(acc[2][r], acc[3][r]),
                             pack_word<T>(acc[4][r], acc[5][r]), pack_word<T>(acc[6][r], acc[7][r])};
            st_b128(ob, (uint32_t)(((size_t)m * N + n_lane) * 2), o);
        }
    }
}

// any shape, any storage type: one thread per pixel, eight output channels at a time
template <typename T, bool PT = false>
__global__ void __launch_bounds__(256) proxy_fma_kernel(const T* __restrict__ in, const T* __restrict__ P, T* __restrict__ out,
                                                        int B, int K, int M, int N) {
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (long)B * N) return;
    const int b = (int)(idx / N), n = (int)(idx - (long)b * N);
    const T* x = in + (size_t)b * K * N + n;
    T* y = out + (size_t)b * M * N + n;
    for (int m0 = 0; m0 < M; m0 += 8) {
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        for (int k = 0; k < K; ++k) {
            const float xv = ldf(x + (size_t)k * N);
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (m0 + j < M) acc[j] = fmaf(ldf(PT ? P + (size_t)k * M + (m0 + j) : P + (size_t)(m0 + j) * K + k), xv, acc[j]);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (m0 + j < M) stf(y + (size_t)(m0 + j) * N, acc[j]);
    }
}

// ---- gradient w.r.t. the matrix: gP[m][k] = sum over b, n of gout[b][m][n] * in[b][k][n] ----------------------------
// Both operands are contiguous along the contraction axis n, which is what the matrix cores want.  One workgroup per
// (image, 32 x 32 tile of gP); its NW waves take interleaved 16-pixel steps of n and add their accumulators through
// LDS in wave order; the per-image sums go to the caller's workspace and a small kernel adds the images in order, so the
// result does not depend on scheduling.  NW = 8 where four waves per tile would leave the chip short of loads in flight.
template <typename T, int NW>
__global__ void __launch_bounds__(64 * NW) proxy_gradw_mfma_kernel(const T* __restrict__ gout, const T* __restrict__ in,
                                                               float* __restrict__ partial, int K, int M, int N,
                                                               int mtiles, int ktiles) {
    __shared__ float red[NW][16][64];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int per_image = mtiles * ktiles;
    const int b = blockIdx.x / per_image;
    const int rem = blockIdx.x - b * per_image;
    const int mt = rem / ktiles, kt = rem - mt * ktiles;
    const int jl = lane & 31, nh = lane >> 5;                  // row of the operand this lane feeds; which 8 of the 16 pixels
    const int m_lane = mt * 32 + jl, k_lane = kt * 32 + jl;
    const bool m_ok = m_lane < M, k_ok = k_lane < K;
    const rsrc_t gb = make_rsrc(gout + ((size_t)b * M + mt * 32) * N);      // the tile's 32 rows of gout / of in
    const rsrc_t ib = make_rsrc(in + ((size_t)b * K + kt * 32) * N);
    const uint32_t row_off = (uint32_t)((size_t)jl * N * 2);
    f32x16_t acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    // four 16-pixel steps per trip: their eight loads are requested together (N is a multiple of 16; steps past the end
    // load nothing and multiply zeros)
    for (int n0 = wave * 16; n0 < N; n0 += 64 * NW) {
        u32x4 av[4], bv[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int n = n0 + 16 * NW * q;
            const uint32_t off = row_off + (uint32_t)((n + 8 * nh) * 2);
            av[q] = u32x4{0, 0, 0, 0}; bv[q] = u32x4{0, 0, 0, 0};
            if (m_ok && n < N) av[q] = __builtin_amdgcn_raw_buffer_load_b128(gb, off, 0, 0);
            if (k_ok && n < N) bv[q] = __builtin_amdgcn_raw_buffer_load_b128(ib, off, 0, 0);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q)
            acc = mfma_k16<T>(av[q], bv[q], acc);
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) red[wave][r][lane] = acc[r];
    __syncthreads();
    // accumulator register r of a lane: row 8*(r/4) + 4*(lane/32) + r%4 of the tile (m), column lane%32 (k)
    for (int idx = threadIdx.x; idx < 16 * 64; idx += 64 * NW) {
        const int r = idx >> 6, l = idx & 63;
        float v = red[0][r][l];
#pragma unroll
        for (int w = 1; w < NW; ++w) v += red[w][r][l];
        const int m = mt * 32 + 8 * (r >> 2) + 4 * (l >> 5) + (r & 3), k = kt * 32 + (l & 31);
        if (m < M && k < K) partial[((size_t)b * M + m) * K + k] = v;
    }
}

// any shape, any storage type: a workgroup owns 8 rows x 32 columns of gP for one image and walks n in chunks of 64
// staged through LDS (coalesced loads along n; pitch 65 keeps the per-thread walks conflict-free)
template <typename T>
__global__ void __launch_bounds__(256) proxy_gradw_fma_kernel(const T* __restrict__ gout, const T* __restrict__ in,
                                                              float* __restrict__ partial, int K, int M, int N,
                                                              int mtiles, int ktiles) {
    __shared__ float gs[8][65], xs[32][65];
    const int per_image = mtiles * ktiles;
    const int b = blockIdx.x / per_image;
    const int rem = blockIdx.x - b * per_image;
    const int mt = rem / ktiles, kt = rem - mt * ktiles;
    const int tm = threadIdx.x >> 5, tk = threadIdx.x & 31;    // this thread's element of the tile
    const int col = threadIdx.x & 63, row4 = threadIdx.x >> 6; // loader: pixel inside the chunk, row group
    float acc = 0.f;
    for (int n0 = 0; n0 < N; n0 += 64) {
        const int n = n0 + col;
#pragma unroll
        for (int r = row4; r < 8; r += 4) {
            const int m = mt * 8 + r;
            gs[r][col] = (m < M && n < N) ? ldf(gout + ((size_t)b * M + m) * N + n) : 0.f;
        }
#pragma unroll
        for (int r = row4; r < 32; r += 4) {
            const int k = kt * 32 + r;
            xs[r][col] = (k < K && n < N) ? ldf(in + ((size_t)b * K + k) * N + n) : 0.f;
        }
        __syncthreads();
#pragma unroll 8
        for (int j = 0; j < 64; ++j) acc = fmaf(gs[tm][j], xs[tk][j], acc);
        __syncthreads();
    }
    const int m = mt * 8 + tm, k = kt * 32 + tk;
    if (m < M && k < K) partial[((size_t)b * M + m) * K + k] = acc;
}

// gP = the per-image sums added in image order
__global__ void __launch_bounds__(256) proxy_gradw_sum_kernel(const float* __restrict__ partial, float* __restrict__ gP, int B, int MK) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= MK) return;
    float v = 0.f;
    // sixteen images requested at a time (the loads do not depend on the sum), then added in order
    for (int b0 = 0; b0 < B; b0 += 16) {
        float t[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) t[j] = b0 + j < B ? partial[(size_t)(b0 + j) * MK + i] : 0.f;
#pragma unroll
        for (int j = 0; j < 16; ++j) if (b0 + j < B) v += t[j];
    }
    gP[i] = v;
}

}  // namespace

bool proxy_mfma_applicable(int B, int K, int M, int N, int dtype) {
    if (dtype == 0 || K % 8 || N % 8) return false;
    // 32-bit byte offsets inside one image of `in` / `out` and inside P
    return (size_t)K * N * 2 < (1ull << 31) && (size_t)M * N * 2 < (1ull << 31) && (size_t)M * K * 2 < (1ull << 31);
}

// out = P in (PT = false) or P^T in (PT = true: the gradient w.r.t. the projection's input) in storage type T
template <typename T, bool PT>
static hipError_t launch_project_as(const void* in, const void* P, void* out, int B, int K, int M, int N, bool mfma, hipStream_t s) {
    if constexpr (sizeof(T) == 2) {
        if (mfma) {
            const int ntiles = (N + 255) / 256, mtiles = (M + 31) / 32;
            const long items = (long)B * ntiles * mtiles;
            if ((items + 3) / 4 > 0x7fffffffl) return hipErrorInvalidValue;
            const dim3 grid((unsigned)((items + 3) / 4)), block(256);
            if (K % 16 == 0)
                hipLaunchKernelGGL((proxy_mfma_kernel<T, 16, PT>), grid, block, 0, s, (const T*)in, (const T*)P, (T*)out, B, K, M, N, ntiles, mtiles);
            else
                hipLaunchKernelGGL((proxy_mfma_kernel<T, 8, PT>), grid, block, 0, s, (const T*)in, (const T*)P, (T*)out, B, K, M, N, ntiles, mtiles);
            return hipGetLastError();
        }
    }
    const long threads = (long)B * N;
    if ((threads + 255) / 256 > 0x7fffffffl) return hipErrorInvalidValue;
    const dim3 grid((unsigned)((threads + 255) / 256)), block(256);
    hipLaunchKernelGGL((proxy_fma_kernel<T, PT>), grid, block, 0, s, (const T*)in, (const T*)P, (T*)out, B, K, M, N);
    return hipGetLastError();
}

hipError_t launch_proxy_project(const void* in, const void* P, void* out, int B, int K, int M, int N, int dtype,
                                hipStream_t s) {
    const bool mfma = proxy_mfma_applicable(B, K, M, N, dtype);
    if (dtype == 0) return launch_project_as<float, false>(in, P, out, B, K, M, N, false, s);
    if (dtype == 1) return launch_project_as<bf16_t, false>(in, P, out, B, K, M, N, mfma, s);
    return launch_project_as<f16_t, false>(in, P, out, B, K, M, N, mfma, s);
}

// per-image sums of gout in^T into `partial` (B*M*K floats), storage type T
template <typename T>
static hipError_t launch_gradw_as(const void* gout, const void* in, float* partial, int B, int K, int M, int N, hipStream_t s) {
    const bool mfma = sizeof(T) == 2 && N % 16 == 0 && (size_t)N * 2 * 32 < (1ull << 31);
    const int ktiles = (K + 31) / 32, mtiles = mfma ? (M + 31) / 32 : (M + 7) / 8;
    const long blocks = (long)B * mtiles * ktiles;
    if (blocks > 0x7fffffffl) return hipErrorInvalidValue;
    const bool wide = blocks * 4 < 2048;     // eight waves per tile while four would leave a compute unit under eight
    if constexpr (sizeof(T) == 2) {
        if (mfma && wide)
            hipLaunchKernelGGL((proxy_gradw_mfma_kernel<T, 8>), dim3((unsigned)blocks), dim3(512), 0, s, (const T*)gout, (const T*)in,
                               partial, K, M, N, mtiles, ktiles);
        else if (mfma)
            hipLaunchKernelGGL((proxy_gradw_mfma_kernel<T, 4>), dim3((unsigned)blocks), dim3(256), 0, s, (const T*)gout, (const T*)in,
                               partial, K, M, N, mtiles, ktiles);
        if (mfma) return hipGetLastError();
    }
    hipLaunchKernelGGL(proxy_gradw_fma_kernel<T>, dim3((unsigned)blocks), dim3(256), 0, s, (const T*)gout, (const T*)in,
                       partial, K, M, N, mtiles, ktiles);
    return hipGetLastError();
}

// Gradients of the projection (chain rule on the sum above): gin = P^T gout per pixel (storage type, may be NULL) and
// gP = sum over images and pixels of gout in^T (fp32 [M, K], may be NULL; `partial` = B*M*K floats of the caller's).
hipError_t launch_proxy_project_bwd(const void* gout, const void* in, const void* P, void* gin, float* gP, float* partial,
                                    int B, int K, int M, int N, int dtype, hipStream_t s) {
    if (gin) {
        // the forward kernels with the matrix read transposed: K output channels, contraction over the M channels of gout
        const bool mfma = proxy_mfma_applicable(B, M, K, N, dtype);
        const hipError_t e = dtype == 0 ? launch_project_as<float, true>(gout, P, gin, B, M, K, N, false, s)
                           : dtype == 1 ? launch_project_as<bf16_t, true>(gout, P, gin, B, M, K, N, mfma, s)
                                        : launch_project_as<f16_t, true>(gout, P, gin, B, M, K, N, mfma, s);
        if (e != hipSuccess) return e;
    }
    if (gP) {
        if (!partial) return hipErrorInvalidValue;
        hipError_t e = dtype == 0 ? launch_gradw_as<float>(gout, in, partial, B, K, M, N, s)
                     : dtype == 1 ? launch_gradw_as<bf16_t>(gout, in, partial, B, K, M, N, s)
                                  : launch_gradw_as<f16_t>(gout, in, partial, B, K, M, N, s);
        if (e != hipSuccess) return e;
        const int MK = M * K;
        hipLaunchKernelGGL(proxy_gradw_sum_kernel, dim3((unsigned)((MK + 255) / 256)), dim3(256), 0, s, partial, gP, B, MK);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// ---- the same call for callers that cannot allocate (HIP graph capture, serving loops): the per-image sums go to a
// static device array instead of a workspace of the caller's.  Each GPU the library runs on holds its own copy of the
// array at its own address; the array's name is only a host-side handle, so the address is looked up once per device
// and that pointer is what the kernels get.
static __device__ __align__(256) float scratch[PROXY_SCRATCH_FLOATS];

static hipError_t scratch_address(float** out) {
    constexpr int MAX_DEVICES = 64;
    static float* per_device[MAX_DEVICES] = {};
    static std::mutex mu;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> guard(mu);
    if (!per_device[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));      // with device `dev` current: this device's copy
        if (e != hipSuccess) return e;
        per_device[dev] = (float*)p;
    }
    *out = per_device[dev];
    return hipSuccess;
}

// Every element [b][m][k] of the workspace is overwritten by the first kernel before the second reads it, so the array
// needs no clearing between calls; calls that overlap on one GPU (two streams) would race on it.
hipError_t launch_proxy_project_bwd_static(const void* gout, const void* in, const void* P, void* gin, float* gP,
                                           int B, int K, int M, int N, int dtype, hipStream_t s) {
    float* partial = nullptr;
    if (gP) {
        if ((size_t)B * M * K > PROXY_SCRATCH_FLOATS) return hipErrorInvalidValue;     // checked by the caller
        const hipError_t e = scratch_address(&partial);
        if (e != hipSuccess) return e;
    }
    return launch_proxy_project_bwd(gout, in, P, gin, gP, partial, B, K, M, N, dtype, s);
}

}  // namespace gspn
