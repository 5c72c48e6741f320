// GSPN-local (Sec. 3.2) with the stretch as a work item of its own (Sec. 4.1: the grid is indexed by
// (chunk, n, c), each block scanning its own stretch): for calls with so few (image, channel) planes that
// one workgroup per plane leaves most of the chip idle.  A stretch of kchunk lines is an independent scan
// (zero state before its first line), so a call with H/kchunk + W/kchunk stretches per plane and pair of
// directions has that many times more work items than planes, each with kchunk scan steps instead of H or W.
//
// Two launches per call, in stream order (a pixel's vertical and horizontal stretches belong to different work
// items, so their contributions meet in y):
//   1. vertical stretches: one workgroup per (plane, band of kchunk image rows), wave 0 runs the top->bottom
//      scan of the band, wave 1 the bottom->top one; both put u*h into an fp32 LDS tile of their own, and
//      the workgroup writes the sum of the two tiles to y (whole rows);
//   2. horizontal stretches: one workgroup per (plane, band of kchunk image columns), wave 0 left->right,
//      wave 1 right->left; the sum of the two tiles is added onto the y of launch 1 (read-modify-write by
//      the workgroup that owns the band: no atomics, fixed order).  In bf16 storage y is therefore rounded twice.
// A workgroup per plane with all stretches as waves of one launch (both tiles of a 128x128 plane fit in LDS) was
// measured slower: what bounds these calls is the rate at which ONE compute unit pulls lines into its L1, so the
// work has to be spread over as many compute units as there are stretches.
// h_save and the reverse sweep of the two-pass backward (e per direction, gx merged; template flags SAVE,
// BWD) run on the same kernels.
#include "gspn_tile_common.hpp"

namespace gspn {

namespace {

struct ChunkArgs {
    FwdParams p;
    int ns;      // stretches along the scan axis of this launch
};

// tensors of one (plane, direction) behind buffer resources
struct PlaneRefs {
    rsrc_t xb, lb, ub, w0b, w1b, w2b, yb, hb;
};
template <typename T, bool SAVE>
__device__ __forceinline__ PlaneRefs plane_refs(const FwdParams& p, int b, int c, int d) {
    const int HW = p.H * p.W;
    const int g = c / p.cpg;
    const size_t planes = (size_t)p.B * p.C;
    const size_t slot_c = p.shared ? 0 : (size_t)d * planes * HW;
    const size_t slot_w = p.shared ? 0 : (size_t)d * p.B * p.G * 3 * HW;
    const size_t plane0 = ((size_t)b * p.C + c) * HW;
    const size_t plane_bytes = (size_t)HW * sizeof(T);
    const char* wbase = (const char*)p.w + (slot_w + ((size_t)b * p.G + g) * 3 * HW) * sizeof(T);
    PlaneRefs r;
    r.xb = make_rsrc((const char*)p.x + plane0 * sizeof(T));
    r.lb = make_rsrc((const char*)p.lam + (slot_c + plane0) * sizeof(T));
    r.ub = make_rsrc((const char*)p.u + (slot_c + plane0) * sizeof(T));
    r.w0b = make_rsrc(wbase); r.w1b = make_rsrc(wbase + plane_bytes); r.w2b = make_rsrc(wbase + 2 * plane_bytes);
    r.yb = make_rsrc((char*)p.y + plane0 * sizeof(T));
    r.hb = make_rsrc(SAVE ? (char*)p.hs + ((size_t)d * planes * HW + plane0) * sizeof(T) : (char*)p.y);
    return r;
}

// y (+)= A + B for `nseg` segments of SEG = 16 B / sizeof(T) elements; segment s of the band starts at byte
// seg_off(s) of the plane and at float tile_off(s) of both tiles
template <typename T, bool RMW, typename SegOff, typename TileOff>
__device__ __forceinline__ void merge_tiles(rsrc_t yb, const float* A, const float* B, int nseg, int tid, int nthreads,
                                            SegOff seg_off, TileOff tile_off) {
    constexpr int SEG = 16 / (int)sizeof(T);
    for (int s = tid; s < nseg; s += nthreads) {
        const uint32_t go = (uint32_t)seg_off(s);
        uint32_t yr[4];
        if constexpr (RMW) ld_buf<16>(yb, go, 0, yr);
        const int to = tile_off(s);
        float v[SEG];
#pragma unroll
        for (int e = 0; e < SEG; ++e) v[e] = A[to + e] + B[to + e];
        if constexpr (RMW) {
#pragma unroll
            for (int e = 0; e < SEG; ++e) v[e] += elem<T>(yr, e);
        }
        uint32_t o[4];
        pack<T, SEG>(v, o);
        const u32x4 ov = {o[0], o[1], o[2], o[3]};
        st_b128(yb, go, ov);
    }
}

// The same with the y words of a thread's first NPRE segments requested up front (`pre`), so that their latency
// passes behind the scan: y += A + B.  Covers segments tid, tid + nthreads, ... below NPRE*nthreads.
template <typename T, int NPRE, typename SegOff>
__device__ __forceinline__ void request_y(rsrc_t yb, int nseg, int tid, int nthreads, SegOff seg_off, uint32_t (&pre)[NPRE][4]) {
#pragma unroll
    for (int i = 0; i < NPRE; ++i) {
        const int s = tid + i * nthreads;
        // clamped to segment 0: redundant but in bounds (a band of fewer segments than threads -- 64 rows of one
        // segment -- leaves threads without any segment of their own)
        ld_buf<16>(yb, (uint32_t)seg_off(s < nseg ? s : 0), 0, pre[i]);
    }
}
template <typename T, int NPRE, typename SegOff, typename TileOff>
__device__ __forceinline__ void merge_tiles_onto(rsrc_t yb, const float* A, const float* B, int nseg, int tid, int nthreads,
                                                 SegOff seg_off, TileOff tile_off, const uint32_t (&pre)[NPRE][4]) {
    constexpr int SEG = 16 / (int)sizeof(T);
#pragma unroll
    for (int i = 0; i < NPRE; ++i) {
        const int s = tid + i * nthreads;
        if (s < nseg) {
            const int to = tile_off(s);
            float v[SEG];
#pragma unroll
            for (int e = 0; e < SEG; ++e) v[e] = A[to + e] + B[to + e] + elem<T>(pre[i], e);
            uint32_t o[4];
            pack<T, SEG>(v, o);
            const u32x4 ov = {o[0], o[1], o[2], o[3]};
            st_b128(yb, (uint32_t)seg_off(s), ov);
        }
    }
}

// ---------------------------------------------------------------------------
// vertical stretch: one wave, the rows [row0, row0 + kchunk) of plane (b, c)
// ---------------------------------------------------------------------------
// REV: the wave walks the rows upwards.  u*h of image row r, positions lane*V.., goes to tile_at(r)[0..V).
template <typename T, int V, bool SAVE, bool BWD, bool REV, typename TileAt>
__device__ __forceinline__ void vertical_band(const FwdParams& p, int b, int c, int row0, int lane, TileAt tile_at) {
    constexpr int NB = V * (int)sizeof(T);
    constexpr int NR = NB / 4;
    constexpr int PF = NB >= 16 ? 4 : 8;                      // lines in flight
    struct Line { uint32_t x[NR], l[NR], u[NR], w0[NR], w1[NR], w2[NR]; };
    // forward: the wave that walks downwards runs the top->bottom scan; reverse sweep: it runs against the
    // bottom->top scan, on that scan's parameters
    constexpr int d = (REV != BWD) ? 1 : 0;
    const PlaneRefs t = plane_refs<T, SAVE>(p, b, c, d);
    const int k = p.kchunk;
    const int row_bytes = p.W * (int)sizeof(T);
    const uint32_t voff = (uint32_t)(lane * NB);
    const bool first = lane == 0, last = lane == 63;

    float h[V], wp0[V], wp1[V], wp2[V];
#pragma unroll
    for (int v = 0; v < V; ++v) { h[v] = 0.f; wp0[v] = 0.f; wp1[v] = 0.f; wp2[v] = 0.f; }

    auto row_of = [&](int s) { return REV ? row0 + k - 1 - s : row0 + s; };
    Line slot[PF];
    auto issue = [&](Line& s, int step) {
        const int so = row_of(step < k ? step : k - 1) * row_bytes;     // clamped: redundant but in bounds
        ld_buf<NB>(t.xb, voff, so, s.x);
        ld_buf<NB>(t.lb, voff, so, s.l);
        ld_buf<NB>(t.ub, voff, so, s.u);
        ld_buf<NB>(t.w0b, voff, so, s.w0);
        ld_buf<NB>(t.w1b, voff, so, s.w1);
        ld_buf<NB>(t.w2b, voff, so, s.w2);
    };
#pragma unroll
    for (int q = 0; q < PF; ++q) issue(slot[q], q);
    for (int s0 = 0; s0 < k; s0 += PF) {
#pragma unroll
        for (int q = 0; q < PF; ++q) {
            const int s = s0 + q;
            if (s < k) {
                const Line& cur = slot[q];
                float av[V], c0[V], c1[V], c2[V];
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    av[v] = elem<T>(cur.l, v) * elem<T>(cur.x, v);
                    c0[v] = elem<T>(cur.w0, v); c1[v] = elem<T>(cur.w1, v); c2[v] = elem<T>(cur.w2, v);
                }
                if constexpr (BWD) {
                    // e of this line from e of the line swept before and that line's taps (0 before the first)
                    line_update_transposed<V>(h, av, wp0, wp1, wp2, first, last);
#pragma unroll
                    for (int v = 0; v < V; ++v) {
                        wp0[v] = (first && v == 0) ? 0.f : c0[v];
                        wp1[v] = c1[v];
                        wp2[v] = (last && v == V - 1) ? 0.f : c2[v];
                    }
                } else {
                    // the first line of a stretch has no predecessor: its weights are never used
                    const bool start = s == 0;
#pragma unroll
                    for (int v = 0; v < V; ++v) {
                        c0[v] = start ? 0.f : c0[v]; c1[v] = start ? 0.f : c1[v]; c2[v] = start ? 0.f : c2[v];
                    }
                    line_update<V>(h, av, c0, c1, c2, first, last);
                }
                const int r = row_of(s);
                float* trow = tile_at(r);
#pragma unroll
                for (int v = 0; v < V; ++v) trow[v] = elem<T>(cur.u, v) * h[v];
                if constexpr (SAVE) {
                    uint32_t o[NR];
                    pack<T, V>(h, o);
                    st_buf<NB, CP_STREAM>(t.hb, voff, r * row_bytes, o);
                }
                issue(slot[q], s + PF);
            }
        }
    }
}

// launch 1 of the two-launch form: vertical stretches
template <typename T, int V, bool SAVE, bool BWD>
__global__ void __launch_bounds__(128) chunk_vertical_kernel(ChunkArgs a) {
    static_assert(!BWD || SAVE, "the reverse sweep saves its state");
    extern __shared__ __align__(16) float lds[];
    const FwdParams& p = a.p;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));   // uniform: the tensors' resources stay scalar
    const int W = p.W, k = p.kchunk;
    const int st = (int)(blockIdx.x % (unsigned)a.ns);
    const int plane = (int)(blockIdx.x / (unsigned)a.ns);
    const int b = plane / p.C, c = plane - b * p.C;
    const int row0 = st * k;
    float* mine = lds + (size_t)wave * k * W;
    auto tile_at = [&](int r) { return mine + (size_t)(r - row0) * W + lane * V; };
    if (wave == 0) vertical_band<T, V, SAVE, BWD, false>(p, b, c, row0, lane, tile_at);
    else vertical_band<T, V, SAVE, BWD, true>(p, b, c, row0, lane, tile_at);
    __syncthreads();
    // the band's rows are contiguous in memory: y = tile of wave 0 + tile of wave 1
    constexpr int SEG = 16 / (int)sizeof(T);
    const rsrc_t yb = make_rsrc((char*)p.y + ((size_t)b * p.C + c) * p.H * W * sizeof(T));
    const int band0 = row0 * W * (int)sizeof(T);
    merge_tiles<T, false>(yb, lds, lds + (size_t)k * W, k * W / SEG, (int)threadIdx.x, 128,
                          [&](int s) { return band0 + s * 16; }, [&](int s) { return s * SEG; });
}

// ---------------------------------------------------------------------------
// horizontal stretch: one wave, the columns [col0, col0 + kchunk) of plane (b, c)
// ---------------------------------------------------------------------------
// tile row of image row i: the R rows of a lane sit 64 tile rows apart, so that the 64 lanes of a wave write 64
// consecutive tile rows (odd pitch: no bank conflict)
template <int R> __device__ __forceinline__ int tile_row(int i) { return (i % R) * 64 + i / R; }

// one wave's scan over the band: REV = it walks the columns leftwards (compile-time, so that every register array is
// indexed by constants)
// u*h of image row R*lane + r, column col0 + j, goes to mine[(r*64 + lane)*pitch + j]
template <typename T, int R, bool SAVE, bool BWD, bool REV>
__device__ __forceinline__ void horizontal_band(const FwdParams& p, float* mine, int pitch, int b, int c, int col0, int lane) {
    constexpr int CS = 16 / (int)sizeof(T);                  // columns per request
    constexpr int PF = R >= 4 ? 2 : (R == 2 ? 3 : 4);        // requests in flight per row and tensor
    struct Sub { uint32_t x[R][4], l[R][4], u[R][4], w0[R][4], w1[R][4], w2[R][4]; };
    // forward: the wave that walks rightwards runs the left->right scan; reverse sweep: it runs against the
    // right->left scan, on that scan's parameters
    constexpr int d = (REV != BWD) ? 3 : 2;
    const PlaneRefs t = plane_refs<T, SAVE>(p, b, c, d);
    const int W = p.W, k = p.kchunk;
    const int nsub = k / CS;
    const bool first = lane == 0, last = lane == 63;
    uint32_t voff[R];
#pragma unroll
    for (int r = 0; r < R; ++r) voff[r] = (uint32_t)((((R * lane + r) * W) + col0) * (int)sizeof(T));

    float h[R], wp0[R], wp1[R], wp2[R];
#pragma unroll
    for (int r = 0; r < R; ++r) { h[r] = 0.f; wp0[r] = 0.f; wp1[r] = 0.f; wp2[r] = 0.f; }

    auto sub_of = [&](int q) { return REV ? nsub - 1 - q : q; };
    Sub slot[PF];
    auto issue = [&](Sub& s, int q) {
        const int so = sub_of(q < nsub ? q : nsub - 1) * 16;              // clamped: redundant but in bounds
#pragma unroll
        for (int r = 0; r < R; ++r) {
            ld_buf<16>(t.xb, voff[r], so, s.x[r]);
            ld_buf<16>(t.lb, voff[r], so, s.l[r]);
            ld_buf<16>(t.ub, voff[r], so, s.u[r]);
            ld_buf<16>(t.w0b, voff[r], so, s.w0[r]);
            ld_buf<16>(t.w1b, voff[r], so, s.w1[r]);
            ld_buf<16>(t.w2b, voff[r], so, s.w2[r]);
        }
    };
#pragma unroll
    for (int q = 0; q < PF; ++q) issue(slot[q], q);
    for (int q0 = 0; q0 < nsub; q0 += PF) {
#pragma unroll
        for (int qq = 0; qq < PF; ++qq) {
            const int q = q0 + qq;
            if (q < nsub) {
                const Sub& cur = slot[qq];
                const int sub = sub_of(q);
                float hq[R][CS];
#pragma unroll
                for (int kk = 0; kk < CS; ++kk) {
                    const int e = REV ? CS - 1 - kk : kk;
                    float av[R], c0[R], c1[R], c2[R];
#pragma unroll
                    for (int r = 0; r < R; ++r) {
                        av[r] = elem<T>(cur.l[r], e) * elem<T>(cur.x[r], e);
                        c0[r] = elem<T>(cur.w0[r], e); c1[r] = elem<T>(cur.w1[r], e); c2[r] = elem<T>(cur.w2[r], e);
                    }
                    if constexpr (BWD) {
                        // e of this column from e of the column swept before and that column's taps (0 before the first)
                        line_update_transposed<R>(h, av, wp0, wp1, wp2, first, last);
#pragma unroll
                        for (int r = 0; r < R; ++r) {
                            wp0[r] = (first && r == 0) ? 0.f : c0[r];
                            wp1[r] = c1[r];
                            wp2[r] = (last && r == R - 1) ? 0.f : c2[r];
                        }
                    } else {
                        // the first column of a stretch has no predecessor: its weights are never used
                        const bool start = q == 0 && kk == 0;
#pragma unroll
                        for (int r = 0; r < R; ++r) {
                            c0[r] = start ? 0.f : c0[r]; c1[r] = start ? 0.f : c1[r]; c2[r] = start ? 0.f : c2[r];
                        }
                        line_update<R>(h, av, c0, c1, c2, first, last);
                    }
                    const int col = sub * CS + e;
#pragma unroll
                    for (int r = 0; r < R; ++r) {
                        mine[(size_t)(r * 64 + lane) * pitch + col] = elem<T>(cur.u[r], e) * h[r];
                        if constexpr (SAVE) hq[r][e] = h[r];
                    }
                }
                if constexpr (SAVE) {
#pragma unroll
                    for (int r = 0; r < R; ++r) {
                        uint32_t o[4];
                        pack<T, CS>(hq[r], o);
                        const u32x4 ov = {o[0], o[1], o[2], o[3]};
                        st_b128<CP_STREAM>(t.hb, voff[r] + (uint32_t)(sub * 16), ov);
                    }
                }
                issue(slot[qq], q + PF);
            }
        }
    }
}

// launch 2 of the two-launch form: horizontal stretches
template <typename T, int R, bool SAVE, bool BWD>
__global__ void __launch_bounds__(128) chunk_horizontal_kernel(ChunkArgs a) {
    static_assert(!BWD || SAVE, "the reverse sweep saves its state");
    extern __shared__ __align__(16) float lds[];
    constexpr int CS = 16 / (int)sizeof(T);
    const FwdParams& p = a.p;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int H = p.H, W = p.W, k = p.kchunk;
    const int st = (int)(blockIdx.x % (unsigned)a.ns);
    const int plane = (int)(blockIdx.x / (unsigned)a.ns);
    const int b = plane / p.C, c = plane - b * p.C;
    const int col0 = st * k;
    const int nsub = k / CS;
    const int pitch = k + 1;
    float* mine = lds + (size_t)wave * H * pitch;
    // y of the band (H rows of kchunk columns) += tile of wave 0 + tile of wave 1; the band's y is requested before the
    // scan where a thread's share fits NPRE requests
    constexpr int NPRE = R >= 4 ? 4 : 8;
    const rsrc_t yb = make_rsrc((char*)p.y + ((size_t)b * p.C + c) * H * W * sizeof(T));
    const int row_bytes = W * (int)sizeof(T);
    const int band0 = col0 * (int)sizeof(T);
    const int nseg = H * nsub;
    auto seg_off = [&](int s) { const int i = s / nsub; return i * row_bytes + band0 + (s - i * nsub) * 16; };
    auto tile_off = [&](int s) { const int i = s / nsub; return tile_row<R>(i) * pitch + (s - i * nsub) * CS; };
    const bool ahead = nseg <= NPRE * 128;
    uint32_t pre[NPRE][4];
    if (ahead) request_y<T, NPRE>(yb, nseg, (int)threadIdx.x, 128, seg_off, pre);
    if (wave == 0) horizontal_band<T, R, SAVE, BWD, false>(p, mine, pitch, b, c, col0, lane);
    else horizontal_band<T, R, SAVE, BWD, true>(p, mine, pitch, b, c, col0, lane);
    __syncthreads();
    if (ahead) merge_tiles_onto<T, NPRE>(yb, lds, lds + (size_t)H * pitch, nseg, (int)threadIdx.x, 128, seg_off, tile_off, pre);
    else merge_tiles<T, true>(yb, lds, lds + (size_t)H * pitch, nseg, (int)threadIdx.x, 128, seg_off, tile_off);
}

bool chunk_shape_ok(const FwdParams& p, int dtype) {
    const int es = dtype == 0 ? 4 : 2, seg = 16 / es;
    if (p.kchunk <= 0 || p.logits || p.xt || p.mask != 15u) return false;
    if (p.H != 64 && p.H != 128 && p.H != 256) return false;
    if (p.W != 64 && p.W != 128 && p.W != 256) return false;
    if (dtype != 0 && p.W == 64) return false;                           // one bf16 position per lane: no packed pair
    const int k = p.kchunk;
    if (k >= p.H && k >= p.W) return false;                              // a single stretch either way: nothing to gain
    if (k > p.H || k > p.W || p.H % k || p.W % k || k % seg) return false;
    if ((size_t)2 * k * p.W * 4 > 160 * 1024 || (size_t)2 * p.H * (k + 1) * 4 > 160 * 1024) return false;
    const size_t items = (size_t)p.B * p.C * ((p.H > p.W ? p.H : p.W) / k);
    return items <= 0x7fffffffull;
}

template <typename T, int V, bool SAVE, bool BWD>
hipError_t launch_vertical(const ChunkArgs& a, hipStream_t s) {
    const FwdParams& p = a.p;
    const int lds = 2 * p.kchunk * p.W * 4;
    auto kern = chunk_vertical_kernel<T, V, SAVE, BWD>;
    hipError_t e = allow_dynamic_lds((const void*)kern, 160 * 1024);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)((size_t)p.B * p.C * a.ns)), dim3(128), lds, s, a);
    return hipGetLastError();
}
template <typename T, int R, bool SAVE, bool BWD>
hipError_t launch_horizontal(const ChunkArgs& a, hipStream_t s) {
    const FwdParams& p = a.p;
    const int lds = 2 * p.H * (p.kchunk + 1) * 4;
    auto kern = chunk_horizontal_kernel<T, R, SAVE, BWD>;
    hipError_t e = allow_dynamic_lds((const void*)kern, 160 * 1024);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)((size_t)p.B * p.C * a.ns)), dim3(128), lds, s, a);
    return hipGetLastError();
}

template <typename T, bool SAVE, bool BWD>
hipError_t launch_chunk(const FwdParams& p, hipStream_t s) {
    ChunkArgs v{p, p.H / p.kchunk}, hz{p, p.W / p.kchunk};
    hipError_t e;
    switch (p.W / 64) {
        case 1: if constexpr (sizeof(T) == 4) { e = launch_vertical<T, 1, SAVE, BWD>(v, s); break; } return hipErrorInvalidValue;
        case 2: e = launch_vertical<T, 2, SAVE, BWD>(v, s); break;
        case 4: e = launch_vertical<T, 4, SAVE, BWD>(v, s); break;
        default: return hipErrorInvalidValue;
    }
    if (e != hipSuccess) return e;
    switch (p.H / 64) {
        case 1: return launch_horizontal<T, 1, SAVE, BWD>(hz, s);
        case 2: return launch_horizontal<T, 2, SAVE, BWD>(hz, s);
        case 4: return launch_horizontal<T, 4, SAVE, BWD>(hz, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

// Worth it when one workgroup per plane (or pair of planes) cannot fill the chip's 256 CUs and the stretches do not
// overfill it: up to two workgroups per CU and launch (measured on 128x128 maps with kchunk 32, one image: 32 / 64 / 128
// channels 25 / 31 / 59 us against 71 / 71 / 75 us on the per-plane kernel in fp32, 256 channels 142 against 81 us).
bool fwd_chunk_applicable(const FwdParams& p, int dtype) {
    if (!chunk_shape_ok(p, dtype)) return false;
    const size_t planes = (size_t)p.B * p.C;
    const size_t stretches = (size_t)((p.H > p.W ? p.H : p.W) / p.kchunk);
    return planes <= 256 && planes * stretches <= 512;
}
hipError_t launch_fwd_chunk(const FwdParams& p, int dtype, hipStream_t s) {
    if (!fwd_chunk_applicable(p, dtype)) return hipErrorInvalidValue;
    if (dtype == 0) return p.hs ? launch_chunk<float, true, false>(p, s) : launch_chunk<float, false, false>(p, s);
    if (dtype == 2) return p.hs ? launch_chunk<f16_t, true, false>(p, s) : launch_chunk<f16_t, false, false>(p, s);
    return p.hs ? launch_chunk<bf16_t, true, false>(p, s) : launch_chunk<bf16_t, false, false>(p, s);
}
bool reverse_sweep_chunk_applicable(const FwdParams& p, int dtype) {
    return p.hs != nullptr && fwd_chunk_applicable(p, dtype);
}
hipError_t launch_reverse_sweep_chunk(const FwdParams& p, int dtype, hipStream_t s) {
    if (!reverse_sweep_chunk_applicable(p, dtype)) return hipErrorInvalidValue;
    if (dtype == 2) return launch_chunk<f16_t, true, true>(p, s);
    return dtype == 0 ? launch_chunk<float, true, true>(p, s) : launch_chunk<bf16_t, true, true>(p, s);
}

}  // namespace gspn
