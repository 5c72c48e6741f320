/* gspn.h -- C ABI of libgspn: the GSPN line-scan propagation on AMD MI355X (gfx950).
 *
 * The operation (GSPN-2 paper, Sec. 3.2 Eq. 1-2; shared-weight form of Sec. 4.2):
 *
 *     h_i = T_i h_{i-1} + lambda_i (.) x_i ,     y_i = u_i (.) h_i
 *
 * swept line by line over an [H, W] feature map.  T_i is tridiagonal: position j
 * of line i reads positions j-1, j, j+1 of line i-1 with the three weights
 * w[0..2] stored for (i, j); a neighbour outside the line contributes 0
 * whatever weight is stored for it; the state before the first line is 0 (first
 * block row of Eq. 3), so the weights stored for the first line of a scan are
 * never read.  The three weights are shared by the C/G channels of one weight
 * group (Sec. 4.2 "compact channel propagation"; G == C is the per-channel form
 * of Eq. 1, G == 1 the single shared matrix).  Up to four scan directions run in
 * one call (Sec. 3.2: top->bottom, bottom->top, left->right, right->left) and
 * their outputs are merged by a plain sum.
 *
 * Direction ids / mask bits:  0 top->bottom (1), 1 bottom->top (2),
 * 2 left->right (4), 3 right->left (8).  For directions 0/1 a "line" is an image
 * row and weight plane k addresses column j+k-1 of the previous row; for
 * directions 2/3 a line is an image column and plane k addresses row j+k-1 of
 * the previous column.  Planes are in image coordinates: they are not mirrored
 * for the reversed directions.
 *
 * Layouts (all contiguous, row-major, element type given by `dtype`):
 *     x, y, gy, gx            [B][C][H][W]
 *     w, gw                   [4][B][G][3][H][W]      slot d = direction d
 *     lam, u, h_save, glam, gu [4][B][C][H][W]        slot d = direction d
 * Channel c belongs to group c / (C/G).  Slots of directions not in `dir_mask`
 * are neither read nor written.  With GSPN_FLAG_SHARED_PARAMS the inputs w, lam, u
 * have a single slot that every direction reads (outputs keep four slots).
 *
 * Pointers are DEVICE pointers (hipMalloc'ed or equivalent), 16-byte aligned,
 * owned by the caller; inputs and outputs must not alias.  The library keeps no
 * pointer after a call returns, allocates nothing and frees nothing.
 * Element types (`dtype`): GSPN_F32 (fp32), GSPN_BF16 (bfloat16) and GSPN_F16 (IEEE binary16), in every entry point.
 * fp16 values are converted by the hardware: to nearest even, subnormals kept, a result beyond 65504 becomes infinity
 * (with row-stochastic weights the states of a scan are running sums of lam * x, so that is a matter of the caller's
 * scaling).
 *
 * Arithmetic: inputs are widened to fp32, the carried state and all sums are
 * fp32, each stored value is rounded once to nearest-even -- except the merged
 * bf16 / fp16 y / gx where the running sum over the directions is kept in storage
 * precision (feature maps too large to stage on chip, merged in place in global
 * memory, and 128x128 maps on the "pair" kernels, whose on-chip tile is in storage precision):
 * at most one extra rounding per direction.
 *
 * Calls only enqueue work on `stream` (a hipStream_t passed as void*; NULL = the
 * default stream) and return without synchronising.  Outputs are overwritten in
 * full; no pre-zeroing is needed.  Concurrent calls on different streams are
 * safe as long as their output buffers differ.
 *
 * Errors: the return value is a gspn_status.  Argument errors are detected on
 * the host before anything is launched and leave every output untouched.  A
 * failed launch returns GSPN_ERR_HIP.  Nothing is printed and nothing aborts.
 */
#ifndef GSPN_H
#define GSPN_H

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    GSPN_OK = 0,
    GSPN_ERR_NULL = 1,        /* a required pointer is NULL                              */
    GSPN_ERR_SHAPE = 2,       /* a dimension or kchunk < 1, C % G != 0, dir_mask == 0 or > 15 */
    GSPN_ERR_DTYPE = 3,       /* dtype is not one the entry point takes                   */
    GSPN_ERR_ALIGN = 4,       /* a pointer is not 16-byte aligned                        */
    GSPN_ERR_UNSUPPORTED = 5, /* a line longer than GSPN_MAX_LINE (GSPN_MAX_LINE_LOGITS), unknown flag bits */
    GSPN_ERR_HIP = 6          /* the HIP runtime refused the launch                      */
} gspn_status;

enum { GSPN_F32 = 0, GSPN_BF16 = 1, GSPN_F16 = 2 };
enum { GSPN_DIR_TB = 1, GSPN_DIR_BT = 2, GSPN_DIR_LR = 4, GSPN_DIR_RL = 8, GSPN_DIR_ALL = 15 };
enum { GSPN_FLAG_SHARED_PARAMS = 1 };
enum { GSPN_MAX_LINE = 16384 };  /* largest H or W */

/* Forward scan (Eq. 1, Eq. 2, sum over the directions in dir_mask).
 *   x      in   [B,C,H,W]
 *   w      in   [4][B,G,3,H,W] normalised tridiagonal weights
 *   lam,u  in   [4][B,C,H,W]
 *   y      out  [B,C,H,W]
 *   h_save out  [4][B,C,H,W] hidden states per direction for the backward call, or NULL
 */
int gspn_scan_fwd(const void* x, const void* w, const void* lam, const void* u,
                  void* y, void* h_save,
                  int B, int C, int H, int W, int G,
                  unsigned dir_mask, int dtype, unsigned flags, void* stream);

/* Backward scan: gradients of a scalar loss L given gy = dL/dy.  The paper gives
 * timings but no algorithm for it (Sec. 5.1); this is the chain rule on Eq. 1-2.
 * With e_i = dL/dh_i, per direction, swept against the scan order:
 *     e_i   = u_i*gy_i + T_{i+1}^T e_{i+1}            (0 past the last line)
 *     gu_i  = gy_i*h_i ,  glam_i = x_i*e_i ,  gx_i += lam_i*e_i  (summed over directions)
 *     gw_i[k][j] = sum over the group's channels of e_i[j]*h_{i-1}[j+k-1]
 * gw is the gradient w.r.t. the normalised weights as free variables; it is 0 on
 * the first line of a scan and for out-of-line neighbours.
 *   gy, x in  [B,C,H,W];  w, lam, u as in the forward call
 *   h_save in [4][B,C,H,W] as written by gspn_scan_fwd (required)
 *   gx out [B,C,H,W];  gw out [4][B,G,3,H,W];  glam, gu out [4][B,C,H,W]
 * The outputs must not alias each other or an input: on large maps glam holds e
 * between the two passes of the call.
 */
int gspn_scan_bwd(const void* gy, const void* x, const void* w, const void* lam, const void* u,
                  const void* h_save,
                  void* gx, void* gw, void* glam, void* gu,
                  int B, int C, int H, int W, int G,
                  unsigned dir_mask, int dtype, unsigned flags, void* stream);

/* GSPN-local (Sec. 3.2): the same two calls with propagation confined to stretches of `kchunk` lines
 * along the scan axis.  The scan axis of every direction (rows for top<->bottom, columns for
 * left<->right) is cut at image lines 0, kchunk, 2*kchunk, ... -- the same cut for a direction and its
 * reverse, the last stretch shorter when kchunk does not divide the axis -- and each stretch is a scan
 * of its own: the state before its first line in scan order is 0, so that line's weights are never
 * read and its gw is 0.  kchunk >= max(H, W) is the global scan; kchunk == 1 leaves no propagation
 * (y = sum over directions of u*lam*x).  kchunk < 1 is GSPN_ERR_SHAPE.  Everything else (layouts,
 * ownership, stream semantics, errors) is as for gspn_scan_fwd / gspn_scan_bwd, and h_save written by
 * the local forward call is what the local backward call with the same kchunk expects.
 * Every kernel family has local instantiations, so a local call runs on the same family as the global
 * call of its shape (gspn_fwd_local_plan / gspn_bwd_local_plan name it) -- except calls with few planes
 * (B*C <= 256 and B*C*max(H, W)/kchunk <= 512) on maps of 64, 128 or 256 rows and columns whose kchunk divides both sides (and is a
 * multiple of 16 bytes of storage), all four directions, no logits: there the stretches are the work items
 * (Sec. 4.1: the chunk index is part of the grid; plan "chunk"), one workgroup per (plane, stretch) in two
 * launches (vertical stretches, then horizontal ones adding onto y: in bf16 storage y is rounded twice),
 * and the reverse sweep of the backward call runs the same way. */
int gspn_scan_fwd_local(const void* x, const void* w, const void* lam, const void* u,
                        void* y, void* h_save,
                        int B, int C, int H, int W, int G, int kchunk,
                        unsigned dir_mask, int dtype, unsigned flags, void* stream);
int gspn_scan_bwd_local(const void* gy, const void* x, const void* w, const void* lam, const void* u,
                        const void* h_save,
                        void* gx, void* gw, void* glam, void* gu,
                        int B, int C, int H, int W, int G, int kchunk,
                        unsigned dir_mask, int dtype, unsigned flags, void* stream);

/* Weights given as raw logits: the normalisation of Sec. 3.2 ("learned and normalized to be row-stochastic")
 * done inside the call instead of by a pass of its own over w beforehand.  z has the layout of w,
 * [4][B,G,3,H,W]; the weights used are the softmax of the three logits stored for a position, taken over the
 * taps whose neighbour exists: at the two ends of a line the tap that points outside gets weight 0 and takes no
 * part in the normalisation, whatever its logit holds (it is never read), so every row of T_i sums to 1.  The
 * logits of a line without predecessor (first line of the scan, of a stretch) are never read either.  The
 * softmax is computed in fp32 from the stored logits and is not rounded to the storage type.
 * The backward call returns gz, the gradient w.r.t. the logits, where gspn_scan_bwd returns gw:
 *     gz_k = w_k * (gw_k - sum_j w_j gw_j)      per position, with gw as defined above;
 * it is 0 for taps that point outside the line and on lines without predecessor.
 * kchunk as in the GSPN-local calls; pass GSPN_MAX_LINE for the global scan.  H, W <= GSPN_MAX_LINE_LOGITS,
 * else GSPN_ERR_UNSUPPORTED.  A learned per-direction (per-channel) merge weight needs no entry point of its
 * own: y = sum_d m_d u_d h_d is this call with u_d scaled by m_d. */
enum { GSPN_MAX_LINE_LOGITS = 4096 };
int gspn_scan_fwd_logits(const void* x, const void* z, const void* lam, const void* u,
                         void* y, void* h_save,
                         int B, int C, int H, int W, int G, int kchunk,
                         unsigned dir_mask, int dtype, unsigned flags, void* stream);
int gspn_scan_bwd_logits(const void* gy, const void* x, const void* z, const void* lam, const void* u,
                         const void* h_save,
                         void* gx, void* gz, void* glam, void* gu,
                         int B, int C, int H, int W, int G, int kchunk,
                         unsigned dir_mask, int dtype, unsigned flags, void* stream);

/* Forward scan with the horizontal directions stored transposed (Sec. 4.3 reaches coalesced access by laying the
 * data out along the orthogonal axis; this is that layout offered to a caller who can produce it, e.g. by
 * computing the parameters of the two horizontal directions from a transposed feature map).  Slots 0 and 1 of
 * w, lam, u are as in gspn_scan_fwd; slots 2 and 3 hold the tensors of the left->right / right->left directions
 * transposed, [B,G,3,W,H] and [B,C,W,H], and xt is x transposed, [B,C,W,H].  Weight plane k of a horizontal
 * direction still addresses row j+k-1 of the previous column.  y is [B,C,H,W] as always: the transposition back
 * happens on chip.  Inference only (no h_save).  Every scan then reads whole contiguous lines: on maps the tile
 * kernel takes (H, W even, at most 128) the horizontal directions run at the speed of the vertical ones.
 * With GSPN_FLAG_SHARED_PARAMS the single slot is read untransposed by directions 0/1 and transposed by 2/3,
 * which is only meaningful for square maps with symmetric parameters: not recommended. */
int gspn_scan_fwd_transposed(const void* x, const void* xt, const void* w, const void* lam, const void* u, void* y,
                             int B, int C, int H, int W, int G,
                             unsigned dir_mask, int dtype, unsigned flags, void* stream);
const char* gspn_fwd_transposed_plan(int B, int C, int H, int W, int G, unsigned dir_mask, int dtype, unsigned flags);

/* COMPARATOR, not a product path: gspn_scan_fwd computed the way the first GSPN implementation ran it (Sec. 3.3;
 * the step-by-step optimisation figure and Table 1 of Sec. 5.1): one small kernel launch per line and per
 * direction, the hidden state of the previous line handed from launch to launch through global memory.  It is
 * here so that the fused kernels can be timed against the structure they replace on the same hardware; no other
 * entry point ever dispatches to it.  Arguments as for gspn_scan_fwd, plus a workspace of the caller's of at
 * least gspn_unfused_workspace_bytes(B, C, H, W) bytes (two fp32 lines per (image, channel); a smaller one is
 * GSPN_ERR_SHAPE).  The call enqueues (number of directions) x (lines per scan) launches on `stream`.  bf16 y is
 * accumulated in storage precision direction by direction. */
int gspn_scan_fwd_unfused(const void* x, const void* w, const void* lam, const void* u, void* y, void* h_save,
                          void* workspace, unsigned long long workspace_bytes,
                          int B, int C, int H, int W, int G,
                          unsigned dir_mask, int dtype, unsigned flags, void* stream);
unsigned long long gspn_unfused_workspace_bytes(int B, int C, int H, int W);

/* Compressive proxy projection (Sec. 4.2, "Compressive Proxy Dimension"): the 1x1 convolution over the channel
 * axis that takes x from C channels to C_proxy before the scan, and the learned 1x1 projection back to C after it:
 *     out[b][m][h][w] = sum_k P[m][k] * in[b][k][h][w]
 *   in  [B,K,H,W]   P [M,K] row-major   out [B,M,H,W]   (down: K = C, M = C_proxy; up: K = C_proxy, M = C)
 * The scan in the proxy space is an ordinary gspn_scan_fwd on [B,C_proxy,H,W].  16-bit storage (bf16, fp16) with K and H*W
 * multiples of 8 runs on the matrix cores (fp32 accumulation, one rounding per output); other shapes and fp32
 * storage run a plain FMA kernel.  Pointers, stream and errors as for the scan calls. */
int gspn_proxy_project(const void* in, const void* P, void* out, int B, int K, int M, int H, int W, int dtype,
                       void* stream);
/* Gradients of gspn_proxy_project for a scalar loss L, given gout = dL/dout (chain rule on the sum above):
 *     gin[b][k][h][w] = sum_m P[m][k] * gout[b][m][h][w]                  the projection with P transposed
 *     gP[m][k]        = sum over b, h, w of gout[b][m][h][w] * in[b][k][h][w]
 *   gout in [B,M,H,W]; in [B,K,H,W] and P [M,K] as in the forward call
 *   gin     out [B,K,H,W] in the storage type, or NULL (not computed)
 *   gP      out [M,K] in fp32 whatever the storage type, or NULL (not computed; at least one of gin, gP is required)
 *   partial workspace of the caller's, B*M*K floats, required with gP (NULL otherwise): it receives the per-image
 *           sums, which a second small kernel adds in image order -- no atomics, the result is bitwise repeatable.
 * The library still allocates nothing.  16-bit storage runs on the matrix cores when M (for gin) and H*W (both; for gP
 * a multiple of 16) allow, as in the forward call; other shapes and fp32 storage run plain FMA kernels. */
int gspn_proxy_project_bwd(const void* gout, const void* in, const void* P, void* gin, float* gP, float* partial,
                           int B, int K, int M, int H, int W, int dtype, void* stream);
/* gspn_proxy_project_bwd for callers that cannot allocate device memory and have no workspace to pass: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The same kernels and the
 * same results, bit for bit; the per-image sums go to a static device array of the library's
 * (GSPN_PROXY_STATIC_MAX_FLOATS floats = 4 MiB, held on every GPU the library runs on until the process
 * ends) instead of `partial`.  With gP, B*M*K beyond that size is GSPN_ERR_UNSUPPORTED (nothing is launched).
 * The call allocates and frees nothing.  Every call on a GPU uses that GPU's one array, so two calls that
 * overlap on one GPU (different streams, no ordering between them) race on it; calls on one stream, or
 * ordered by events, are safe.  The array needs no clearing: each call overwrites what it reads.  Other
 * arguments, errors and stream semantics as for gspn_proxy_project_bwd. */
#define GSPN_PROXY_STATIC_MAX_FLOATS (1 << 20)
int gspn_proxy_project_bwd_static(const void* gout, const void* in, const void* P, void* gin, float* gP,
                                  int B, int K, int M, int H, int W, int dtype, void* stream);
/* "mfma" or "fma": which kernel gspn_proxy_project runs for these arguments ("invalid" for bad ones). */
const char* gspn_proxy_plan(int B, int K, int M, int H, int W, int dtype);

/* Name of the kernel family the forward / backward call would dispatch to for
 * these arguments: "plane" (small maps, whole planes through LDS), "pair" (128x128 maps in 16-bit storage
 * with an even number of channels per weight group, all four directions, the global scan or GSPN-local, normalised
 * weights or logits: two channels of a group per workgroup, the merged output accumulated on chip in storage precision, i.e. rounded
 * after each of the four additions), "tile" (maps whose merged output fits in LDS), "stream"
 * (larger maps with rows and columns in multiples of 64: up to 512 rows and lines of 256, 512 or 1024 positions in
 * one launch; also up to 1024 rows and lines of 256 to 2048 positions -- and, for the global scan with normalised
 * weights, up to 2048 rows in multiples of 128 -- in two launches: the vertical pair, then the horizontal pair; the
 * merged output is accumulated in place in y), "twopass" (backward
 * on the maps the forward plane, tile or stream kernels take: the reverse sweep per
 * channel on those kernels, then the sum over each group's channels; in 16-bit
 * storage e passes through storage precision between the two), "generic" (any shape);
 * static string, never NULL.  Host only.
 *
 * Environment variables for tests (results are the same whichever kernel runs, up to the rounding of
 * the storage type).  They are read once per process, by the first call that dispatches; a process
 * that changes them afterwards calls gspn_reload_env():
 *   GSPN_FORCE_GENERIC=1   always the generic kernels
 *   GSPN_FWD_NO_PLANE=1, GSPN_BWD_NO_PLANE=1   skip the "plane" kernels
 *   GSPN_BWD_NO_TWOPASS=1   skip the "twopass" backward (the "tile" / "generic" kernels take its maps)
 *   GSPN_FWD_NO_PAIR=1   skip the "pair" kernels (forward and the reverse sweep of the two-pass backward)
 *   GSPN_STREAM_NO_STAGED=1   the general "stream" kernel (the one fp32 maps take) on the 16-bit maps
 *                             that have a kernel of their own
 *   GSPN_STREAM_TWO_CHANNELS=1  two channels of a weight group per workgroup on those maps also in calls with at most 256
 *                               planes (which normally keep one channel per workgroup: a compute unit holds one workgroup)
 *   GSPN_STREAM_ONE_CHANNEL=1   the "stream" kernel with one channel per workgroup on 256- and 512-row bf16 maps (two channels of a
 *                               weight group share a workgroup and the weights there otherwise)
 *   GSPN_FWD_NO_CHUNK=1   skip the "chunk" kernels of GSPN-local (forward and the reverse sweep of the two-pass backward) */
const char* gspn_fwd_plan(int B, int C, int H, int W, int G, unsigned dir_mask, int dtype, unsigned flags, int has_h_save);
const char* gspn_bwd_plan(int B, int C, int H, int W, int G, unsigned dir_mask, int dtype, unsigned flags);
/* the same for the GSPN-local calls */
const char* gspn_fwd_local_plan(int B, int C, int H, int W, int G, int kchunk, unsigned dir_mask, int dtype,
                                unsigned flags, int has_h_save);
const char* gspn_bwd_local_plan(int B, int C, int H, int W, int G, int kchunk, unsigned dir_mask, int dtype,
                                unsigned flags);
/* ... and for the calls that take logits */
const char* gspn_fwd_logits_plan(int B, int C, int H, int W, int G, int kchunk, unsigned dir_mask, int dtype,
                                 unsigned flags, int has_h_save);
const char* gspn_bwd_logits_plan(int B, int C, int H, int W, int G, int kchunk, unsigned dir_mask, int dtype,
                                 unsigned flags);

/* Static, human-readable text for a gspn_status value. */
const char* gspn_status_string(int status);

/* Library version: major*10000 + minor*100 + patch. */
int gspn_version(void);

/* Reads the GSPN_* environment variables listed above again (host only, thread-safe; calls already
 * enqueued are not affected). */
void gspn_reload_env(void);

#ifdef __cplusplus
}
#endif
#endif /* GSPN_H */
