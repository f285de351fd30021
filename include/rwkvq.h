/*
 * rwkvq - weight-only-quantized linear layers of an RWKV model on one MI355X (gfx950).
 *
 * Every weight matrix W [N, K] (N output channels, K input channels) is stored either
 *   - scalar-quantized (SQ): b-bit codes with one fp16 scale s and one fp16 zero point z per
 *     group of consecutive input channels.  RWKVQuant Sec. 2.2, Eq. "SQ" defines the forward map
 *     Q(w) = clamp(round(w/s) + z, 0, 2^b - 1); this library evaluates its inverse
 *     Deq(q) = (q - z) * s  (one binary32 subtraction, then one binary32 multiplication), or
 *   - vector-quantized (VQ): W viewed as (N*K/d, d) row-major vectors (d consecutive input
 *     channels of one output row), each replaced by a k-bit index into a (2^k, d) fp16 codebook;
 *     Deq returns the indexed codebook row.  Sec. 2.2, Eq. "VQ".
 * Which of the two a matrix uses is the per-matrix flag phi_m of Sec. 3.1 (Eq. "optimization
 * goal" and Eq. "multi-scale proxy"): 1 = SQ, 0 = VQ.  The library computes the linear maps
 * y = x * Deq(W)^T that App. A.1 writes as r_t = W_r(...), k_t = W_k(...), and so on.
 *
 * GENERAL RULES
 *   - Every pointer argument is a DEVICE pointer owned by the caller unless a comment says
 *     "host".  Device pointers must be 16-byte aligned.  The library never allocates or frees
 *     device memory and keeps no reference to a buffer after the enqueued work has finished.
 *   - Every call validates its arguments on the host before anything is launched and returns an
 *     rwkvq_status; on any error nothing has been enqueued.  Nothing throws or aborts.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the default stream);
 *     no call synchronises.
 *   - Inputs must be finite.  Supported formats: SQ with bits = 3, group = 128; VQ with
 *     vdim = 2, kbits = 6 or 8, block_rows = block_cols = 256.  N must be a multiple of 16 (SQ)
 *     or of block_rows (VQ); K must be a multiple of 256.
 *
 * CANONICAL LAYOUT (interchange format)
 *   A row of packed fields is an array of uint32 words read as one little-endian bit string:
 *   bit p of the row is bit (p & 31) of word (p >> 5); field i of width b is bits [b*i, b*i+b).
 *     SQ codes      uint32 [N][K*bits/32]        code of column k = field k of row n
 *     SQ scales     fp16   [N][K/group]
 *     SQ zeros      fp16   [N][K/group]
 *     VQ indices    uint32 [N][(K/vdim)*kbits/32] index of columns (2j, 2j+1) = field j of row n
 *     VQ codebooks  fp16   [N/block_rows][K/block_cols][2^kbits][vdim]
 *
 * NATIVE LAYOUT (what the fast kernels stream; produced once by rwkvq_*_prepack)
 *   Same number of bytes as the canonical buffers, reordered into tiles of 16 rows x 256 columns
 *   so that one wavefront reads a tile with contiguous 16-byte loads and every lane's words hold
 *   the fields of its own matrix-core operand.  Within a tile, lane = 16*kg + r (r = row in the
 *   tile, kg = 0..3) owns, for unit u = 0,1 and step t = 0..3, the eight columns
 *   256*T + 128*u + 32*t + 8*kg + (0..7); its 32 fields per unit are numbered c = 8*t + j and
 *   paired as P = c/2 (low element c even, high element c odd).
 *     SQ codes: 384 words per tile: words [4*lane + i] (i = 0..3) then [256 + 2*lane + (i-4)]
 *       (i = 4,5) are the lane's words L[0..5]; unit u uses L[3u .. 3u+2].  Pair P < 15 sits in
 *       word P/5 at bits 1 + 3*(P%5) (+16 for the odd element); pair 15 is spread over bit 0
 *       (even element) and bit 16 (odd element) of the three words, code bit b in word b.
 *     SQ scale/zero: fp16 [N/16][K/256][16 rows][2 units][scale, zero] in one buffer.
 *     VQ kbits = 6: same word positions; pair P < 15 is one index at bits 2 + 6*(P%5) of word
 *       P/5; index 15 is spread over bits 0,1 of the three words, index bits 2w, 2w+1 in word w.
 *     VQ kbits = 8: 512 words per tile: lane words L[i] = [4*lane + i] (i < 4), [256 + 4*lane
 *       + (i-4)] (i >= 4); unit u uses L[4u .. 4u+3]; index P is byte P%4 of word P/4.
 *     VQ codebooks are used as they are (canonical).
 */
#ifndef RWKVQ_H
#define RWKVQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    RWKVQ_OK = 0,
    RWKVQ_ERR_NULL = 1,        /* a required pointer is NULL */
    RWKVQ_ERR_SHAPE = 2,       /* M, N or K is non-positive or not a multiple of the tile/group/block size */
    RWKVQ_ERR_UNSUPPORTED = 3, /* a format or dtype this build has no kernel for */
    RWKVQ_ERR_ALIGN = 4,       /* a device pointer is not 16-byte aligned */
    RWKVQ_ERR_DEVICE = 5       /* the HIP runtime reported an error at launch */
} rwkvq_status;

typedef enum { RWKVQ_F16 = 0, RWKVQ_BF16 = 1, RWKVQ_F32 = 2 } rwkvq_dtype;
typedef enum { RWKVQ_VQ = 0, RWKVQ_SQ = 1 } rwkvq_kind;            /* = phi_m of Sec. 3.1 */
typedef enum { RWKVQ_CANONICAL = 0, RWKVQ_NATIVE = 1 } rwkvq_layout;

/* One quantized matrix (a host struct holding device pointers). */
typedef struct rwkvq_matrix {
    int32_t kind;        /* rwkvq_kind */
    int32_t layout;      /* rwkvq_layout of `codes` (and of `scales` for SQ) */
    int32_t N, K;
    int32_t bits, group;                            /* SQ: 3, 128 (ignored for VQ) */
    int32_t vdim, kbits, block_rows, block_cols;    /* VQ: 2, 6|8, 256, 256 (ignored for SQ) */
    const void* codes;     /* SQ codes or VQ indices */
    const void* scales;    /* SQ canonical: scales; SQ native: the scale/zero buffer; VQ: NULL */
    const void* zeros;     /* SQ canonical: zeros; otherwise NULL */
    const void* codebooks; /* VQ: codebooks; SQ: NULL */
} rwkvq_matrix;

int rwkvq_version(void);
const char* rwkvq_status_string(int status);

/* Process-wide settings that replace a choice the library otherwise makes from the sizes of a call
 * (for tests, which run both sides of each choice, and for tuning on another machine).  Thread-safe;
 * a call made after rwkvq_set_option returns sees the new value.
 *   RWKVQ_OPT_SMALL_BATCH_PATH    how native-layout matrices run at 16 < M <= 128 (see rwkvq_sq_gemm):
 *                                 RWKVQ_SMALL_BATCH_AUTO (default: the estimate below), _STREAM, _MATRIX_CORES
 *   RWKVQ_OPT_PREFILL_TILE_ROWS   rows of x per matrix-core workgroup: 0 (default: chosen per launch), 128, 256
 *   the constants of the small-batch estimate, measured on the RWKV-6-7B shapes on one MI355X
 *   (0 restores the default):
 *   RWKVQ_OPT_STREAM_WIDE_GBPS    packed-weight GB/s of a streaming pass over 17..32 batch rows (2800)
 *   RWKVQ_OPT_STREAM_NARROW_GBPS  ... over <= 16 batch rows (4100)
 *   RWKVQ_OPT_STREAM_WIDE_MIN_US  least duration of such a pass in microseconds (24)
 *   RWKVQ_OPT_STREAM_NARROW_MIN_US  (12)
 *   RWKVQ_OPT_MFMA_KSTEP_NS       one 64-column step of a 128-row matrix-core workgroup in nanoseconds (1500)
 *   RWKVQ_OPT_STREAM_TWO_PASS_MIN_WGS  batch 2..32 on the streaming kernels: a workgroup covers 256 rows of W
 *                                 (two stretches that share each staged activation tile) when the launch
 *                                 still has at least this many workgroups that way, and 128 rows otherwise
 *                                 (2048; 1 = always 256 rows, 1000000 = never)
 *   RWKVQ_OPT_STREAM_SPLIT_MAX_WORK    batch 2..32 on the streaming kernels: a launch takes the small-launch form (one
 *                                 workgroup per 32 rows of W, its wavefronts split the columns, every workgroup
 *                                 reads all of x) when (rows of all its matrices / 32) x (16 + M) is at most this
 *                                 (65536: one RWKV-6-7B layer at any M <= 16, two layers up to M = 8; 1 = never;
 *                                 at M = 17..32 a third of the value is the limit unless it is 1000000 or more)
 *   RWKVQ_OPT_SPLIT_GRID_2D       batch 1, launches of at most eight matrices with few rows (the stages of a block): 1 = a
 *                                 workgroup takes its matrix and row tile from a two-dimensional grid, 2 = from the
 *                                 table of first-workgroup indices that larger launches use (1; same output bits)
 * Errors: RWKVQ_ERR_UNSUPPORTED (unknown option, value out of range), RWKVQ_ERR_NULL. */
enum { RWKVQ_OPT_SMALL_BATCH_PATH = 0, RWKVQ_OPT_PREFILL_TILE_ROWS = 1, RWKVQ_OPT_STREAM_WIDE_GBPS = 2,
       RWKVQ_OPT_STREAM_NARROW_GBPS = 3, RWKVQ_OPT_STREAM_WIDE_MIN_US = 4, RWKVQ_OPT_STREAM_NARROW_MIN_US = 5,
       RWKVQ_OPT_MFMA_KSTEP_NS = 6, RWKVQ_OPT_STREAM_TWO_PASS_MIN_WGS = 7, RWKVQ_OPT_STREAM_SPLIT_MAX_WORK = 8,
       RWKVQ_OPT_SPLIT_GRID_2D = 9 };
enum { RWKVQ_SMALL_BATCH_AUTO = 0, RWKVQ_SMALL_BATCH_STREAM = 1, RWKVQ_SMALL_BATCH_MATRIX_CORES = 2 };
int rwkvq_set_option(int option, int value);
int rwkvq_get_option(int option, int* value /* host */);

/* One-time reordering canonical -> native (see the layout section above).  Output buffers have
 * the same sizes as the inputs: codes_native K*bits/8*N bytes, sz_native 4*N*K/group bytes;
 * indices_native (K/vdim)*kbits/8*N bytes.  Outputs must not overlap inputs. */
int rwkvq_sq_prepack(const void* codes, const void* scales, const void* zeros, int N, int K,
                     int bits, int group, void* codes_native, void* sz_native, void* stream);
int rwkvq_vq_prepack(const void* indices, int N, int K, int vdim, int kbits, void* indices_native,
                     void* stream);

/* Deq(W) written out as a dense row-major [N][K] array (Sec. 2.2; "Deq" of Sec. 3.2).
 * w_dtype = RWKVQ_F32 gives the binary32 value defined at the top of this file, bit for bit;
 * RWKVQ_F16 / RWKVQ_BF16 give that value rounded to nearest even, which is exactly what the
 * matrix-core path feeds its multipliers for activations of that type.  For layout =
 * RWKVQ_NATIVE, `scales` is the scale/zero buffer and `zeros` must be NULL. */
int rwkvq_sq_dequant(const void* codes, const void* scales, const void* zeros, int layout, int N,
                     int K, int bits, int group, void* w_out, int w_dtype, void* stream);
int rwkvq_vq_dequant(const void* indices, const void* codebooks, int layout, int N, int K, int vdim,
                     int kbits, int block_rows, int block_cols, void* w_out, int w_dtype,
                     void* stream);

/* y[M][N] = x[M][K] * Deq(W)^T for one matrix (the W. products of App. A.1).
 * x is row-major fp16 or bf16 (any finite values: the streaming kernels multiply fp16 operands and
 * bring bf16 activations into fp16's range group by group with exact power-of-two scales - a
 * group being the columns that share an accumulator, at most 256 consecutive ones of a row of x - so
 * an activation enters its sum exactly unless it is more than 2^29 times smaller than the largest
 * of its group, which is below the resolution of the binary32 sum); y is row-major fp16, bf16 or
 * fp32; products are accumulated in binary32 and y is rounded to nearest even.  The path is chosen from M and the layout:
 *   canonical layout: a plain reference kernel (any M);
 *   native layout, M <= 16: streaming dequant-GEMV kernels bound by HBM bandwidth;
 *   native layout, M  > 16: tiles dequantized into LDS and multiplied on the matrix cores in
 *                           the type of x, weights rounded to that type;
 *   native layout, 16 < M <= 128: the matrix cores (M padded to 128 rows), or ceil(M / 32) passes
 *                           of the streaming kernels over blocks of 32 rows of x (weights exact),
 *                           whichever is estimated cheaper for the matrices of the call: a call
 *                           of few matrices gives the matrix-core kernel few tiles.  A matrix
 *                           whose N is not a multiple of 256 has no matrix-core tiles: streaming
 *                           passes up to M = 128, beyond that the plain reference kernel.
 * x and y must not overlap. */
int rwkvq_sq_gemm(const void* codes, const void* scales, const void* zeros, int layout,
                  const void* x, void* y, int M, int N, int K, int bits, int group, int x_dtype,
                  int y_dtype, void* stream);
int rwkvq_vq_gemm(const void* indices, const void* codebooks, int layout, const void* x, void* y,
                  int M, int N, int K, int vdim, int kbits, int block_rows, int block_cols,
                  int x_dtype, int y_dtype, void* stream);

/* The hybrid of Sec. 3.1: ys[i] = xs[i] * Deq(mats[i])^T for i < n_mats, each matrix SQ or VQ
 * as its `kind` says, all enqueued on one stream as grouped launches (matrices share a launch;
 * there is no ordering between matrices of one call, so no ys[i] may alias an xs[j]).
 * `mats`, `xs` and `ys` are HOST arrays (of descriptors / device pointers) read before return.
 * All matrices share M and the dtypes.  xs[i] is [M][mats[i].K], ys[i] is [M][mats[i].N].
 * Reproducibility: a call gives the same bits every time.  At M = 1 the kernel is chosen by the
 * number of rows in the call (small calls split each row's columns over several wavefronts), so
 * the same matrix dispatched alone and inside a large call may differ in the order of its
 * binary32 sums (a few units in the last place); for 2 <= M <= 16 and for M > 128 the order is
 * fixed; for 16 < M <= 128 the path (see rwkvq_sq_gemm) is chosen from the sizes of the call's
 * matrices, not from their values.
 * No scratch memory; safe to record into a HIP graph. */
int rwkvq_linear_dispatch(const rwkvq_matrix* mats, const void* const* xs, void* const* ys,
                          int n_mats, int M, int x_dtype, int y_dtype, void* stream);

/* Which kernels rwkvq_linear_dispatch would run for each matrix of such a call (no launch, no device
 * access; the weight pointers of the descriptors must be non-NULL and aligned but are not read).
 * paths[i], HOST, one of:
 *   RWKVQ_PATH_REFERENCE     plain reference kernel (canonical layout; shapes no other path takes);
 *   RWKVQ_PATH_STREAM        streaming kernels, M <= 16: weights exact;
 *   RWKVQ_PATH_STREAM_PASSES ceil(M / 32) passes of the streaming kernels, 16 < M <= 128: weights exact;
 *   RWKVQ_PATH_MATRIX_CORES  matrix-core kernels: weights rounded once to the type of x.
 * The path depends on M and on the sizes and layouts of the call's matrices only (see rwkvq_sq_gemm),
 * so a caller can learn beforehand how the weights of a call will be fed.  Errors: RWKVQ_ERR_NULL,
 * RWKVQ_ERR_SHAPE, and those of the descriptors. */
enum { RWKVQ_PATH_REFERENCE = 0, RWKVQ_PATH_STREAM = 1, RWKVQ_PATH_STREAM_PASSES = 2, RWKVQ_PATH_MATRIX_CORES = 3 };
int rwkvq_linear_dispatch_plan(const rwkvq_matrix* mats, int n_mats, int M, int32_t* paths);

/* ---- the SQ / VQ decision (Sec. 3.1, "Coarse-grained Proxy" and "Fine-grained Proxy") ----------
 *
 * For each of n_mats dense weight matrices ws[i] (DEVICE pointers in a HOST array; matrix i is
 * Ns[i] x Ks[i], row-major, fp16 or bf16 bit patterns or binary32 values, all of one type, finite;
 * Ns and Ks are HOST arrays) compute
 *   P_c = H(uniform) - H(G')                       Eq. "coarse_proxy", natural logarithm
 *   P_f = sum_{k=2}^{terms} v_k |M_k|              Eq. "fine_proxy", K = terms in [2, 8]
 *   phi = 1 (RWKVQ_SQ) if P_c < tau_c and P_f < tau_f, else 0 (RWKVQ_VQ)    Eq. "multi_scale_proxy"
 * where G' are the normalised intervals between neighbours of the sorted, flattened weights
 * (Eqs. "interval", "interval_norm"), 0 ln 0 := 0 for the zero intervals between equal weights, and
 * a constant matrix gives P_c = P_f = 0.  All arithmetic after the pass over the weights is
 * binary64 in a fixed order.  Sixteen-bit matrices are reduced to the set of bit patterns that
 * occur (one pass over the matrix, many matrices per launch); binary32 matrices are sorted (four
 * passes of a radix sort over order-preserving keys), one matrix after another.
 *
 * proxies: DEVICE pointer to 2 n_mats doubles (P_c, P_f per matrix); phi: DEVICE pointer to n_mats
 * int32.  workspace: DEVICE pointer to rwkvq_proxy_workspace_size(Ns, Ks, n_mats, w_dtype) bytes of
 * scratch owned by the caller (contents irrelevant on entry, undefined on exit): 8 KiB per matrix
 * for 16-bit weights (= rwkvq_proxy_workspace_bytes(n_mats)); for binary32 about 8.3 bytes per weight
 * of the largest matrix (two key buffers, digit counts and partial sums; 0 is returned for arguments
 * rwkvq_proxy would reject).  workspace, proxies and every ws[i] 16-byte aligned, phi 4-byte aligned.
 * The host arrays are read before return; the call is asynchronous on `stream`; calls that share a
 * workspace must be ordered by the stream.
 * Errors: RWKVQ_ERR_NULL, RWKVQ_ERR_ALIGN, RWKVQ_ERR_SHAPE (n_mats < 1, N or K < 1, a matrix of
 * fewer than two weights or more than 2^32 - 1), RWKVQ_ERR_UNSUPPORTED (w_dtype, terms outside
 * [2, 8]), RWKVQ_ERR_DEVICE. */
size_t rwkvq_proxy_workspace_bytes(int n_mats);
size_t rwkvq_proxy_workspace_size(const int* Ns, const int* Ks, int n_mats, int w_dtype);
int rwkvq_proxy(const void* const* ws, const int* Ns, const int* Ks, int n_mats, int w_dtype, int terms,
                double tau_c, double tau_f, void* workspace, double* proxies, int32_t* phi,
                void* stream);

/* rwkvq_proxy for callers that cannot allocate device memory or hand over a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and
 * errors as rwkvq_proxy without `workspace`, for fp16 / bf16 matrices (binary32: RWKVQ_ERR_UNSUPPORTED): the bitmaps live in a device array inside the library
 * (8 KiB per matrix, RWKVQ_PROXY_STATIC_MAX_MATS matrices = 2 MiB, held on every GPU the library
 * runs on until the process ends), whose address is looked up on the first call on each device.  The
 * call allocates nothing, on the host or on the device.  n_mats > RWKVQ_PROXY_STATIC_MAX_MATS returns
 * RWKVQ_ERR_SHAPE.  Every call on a GPU uses that GPU's one array (cleared by a kernel at the start of
 * each call): calls on one GPU must be ordered, by one stream or by events; calls that overlap race. */
#define RWKVQ_PROXY_STATIC_MAX_MATS 256
int rwkvq_proxy_static(const void* const* ws, const int* Ns, const int* Ks, int n_mats, int w_dtype, int terms,
                       double tau_c, double tau_f, double* proxies, int32_t* phi, void* stream);

/* ---- encoders (Sec. 2.2, Eq. "SQ" and Eq. "VQ"): dense weights -> canonical-layout codes -----------
 *
 * w: DEVICE pointer, row-major [N][K], fp16 / bf16 bit patterns or binary32 (w_dtype), finite.
 * Every floating-point step is one binary32 operation rounded to nearest even, so the integer
 * results are reproducible by any implementation of the same steps.
 *
 * rwkvq_sq_encode, per row and group of `group` = 128 columns, bits = 3:
 *     s = (max - min) / (2^bits - 1)  stored as fp16;   z = -min / s  (with the stored s), stored
 *     as fp16;   q = clamp(rne(w / s + z), 0, 2^bits - 1)  with the stored s and z (ties to even).
 *   A constant group, or one whose fp16 scale would be zero, takes s = 1, z = -min.  A group's
 *   scale and zero point must fit fp16.  Outputs in the canonical layout: codes [N][3K/32],
 *   scales [N][K/128], zeros [N][K/128].
 *
 * rwkvq_vq_assign (vdim = 2, kbits = 6 or 8, 256 x 256 blocks): index of the codebook entry
 *   nearest to (w[n][2j], w[n][2j+1]) in squared Euclidean distance
 *   fl(fl((v0 - c0)^2) + fl((v1 - c1)^2)); equal distances resolve to the lowest index.
 *   codebooks as for rwkvq_vq_gemm; indices out in the canonical layout [N][(K/2) kbits / 32].
 *
 * All pointers 16-byte aligned; asynchronous on `stream`; no scratch memory.
 * Errors: RWKVQ_ERR_NULL, RWKVQ_ERR_UNSUPPORTED (format parameters, dtype), RWKVQ_ERR_SHAPE (K not a
 * multiple of the group / N, K not multiples of the block), RWKVQ_ERR_ALIGN, RWKVQ_ERR_DEVICE. */
int rwkvq_sq_encode(const void* w, int w_dtype, int N, int K, int bits, int group, void* codes,
                    void* scales, void* zeros, void* stream);
int rwkvq_vq_assign(const void* w, int w_dtype, const void* codebooks, int N, int K, int vdim, int kbits,
                    int block_rows, int block_cols, void* indices, void* stream);

/* ---- element-wise multiplication weights (Sec. 3.2, "Codebook Optimization for Element-wise
 *      Multiplication") and the token-shift mix of Eq. "time mixing r/k/v", "channel mixing r/k" ----
 *
 * rwkvq_clip_mean: the representative activation X of a calibration batch.  x: DEVICE pointer,
 *   row-major [n_samples][n] (fp16 / bf16 bit patterns or binary32, finite); per position the
 *   samples are limited to the range between their percentile-th and (100 - percentile)-th
 *   percentile (linear interpolation between order statistics, rank (B - 1) q / 100, binary64) and
 *   averaged (binary64 sum in sample order, divided by B, rounded to binary32).  xbar: DEVICE
 *   pointer to n floats.  percentile in [0, 50] (0 = plain mean); n_samples <= 65536.
 *
 * rwkvq_mu_codebook: X^2-weighted Lloyd iterations (weighted KMeans under the loss of Eq.
 *   "quantization loss of mul") for n_tensors weight tensors at once.  Tensor i: mus[i] = n_elems[i]
 *   weights (mu_dtype; row-major flattening, cut into vectors of 2 consecutive elements),
 *   xbars[i] = n_elems[i] floats (element weight = xbar^2 in binary32), codebooks[i] = 2^kbits x 2
 *   fp16 entries: the initial codebook on entry (the caller draws it), the final one on return;
 *   indices[i] = n_elems[i] / 2 bytes out, the entry of each vector under the final codebook.
 *   Per iteration: assignment argmin_e fl(fl(w0 fl(t0^2)) + fl(w1 fl(t1^2))), t = mu - c_e, binary32,
 *   lowest index on ties; update c_ej = sum w mu / sum w over the assigned vectors (binary64),
 *   rounded once to fp16; a coordinate whose weight sum is zero keeps its value.  `iters` updates,
 *   then one more assignment.  kbits = 6 or 8; n_elems[i] even, >= 2.  The arrays of pointers and
 *   n_elems are HOST arrays of DEVICE pointers, read before return.
 *
 * rwkvq_token_shift_mix: outs[p][t][j] = mu_p[j] x[t][j] + (1 - mu_p[j]) x[t-1][j] for n_proj <= 8
 *   projections in one pass, mu_p[j] = codebooks[p][indices[p][j / 2]][j % 2]; row 0 takes x[-1]
 *   from x_prev[d].  Binary32 with one rounding per operation, fl(fl(m x_t) + fl(fl(1 - m) x_prev)),
 *   then rounded once to x_dtype (fp16 or bf16).  x: [M][d], outs[p]: [M][d], d a multiple of 8.
 *
 * All device pointers 16-byte aligned (xbar of rwkvq_clip_mean: 4); asynchronous on `stream`; no
 * scratch memory.  Errors: RWKVQ_ERR_NULL, RWKVQ_ERR_UNSUPPORTED (dtype, kbits, percentile, n_proj,
 * iters outside [0, 1000]), RWKVQ_ERR_SHAPE, RWKVQ_ERR_ALIGN, RWKVQ_ERR_DEVICE. */
int rwkvq_clip_mean(const void* x, int x_dtype, int n_samples, int n, double percentile, float* xbar,
                    void* stream);
int rwkvq_mu_codebook(const void* const* mus, const float* const* xbars, const int* n_elems, int n_tensors,
                      int mu_dtype, int kbits, int iters, void* const* codebooks, uint8_t* const* indices,
                      void* stream);
int rwkvq_token_shift_mix(const void* x, const void* x_prev, int x_dtype, int M, int d,
                          const uint8_t* const* indices, const void* const* codebooks, int kbits, int n_proj,
                          void* const* outs, void* stream);

/* rwkvq_linear_dispatch_mixed: batch 1 with the token-shift mix fused into the GEMV.  For matrix i
 *   y_i = Deq(W_i) . round_x( mu_i (.) x_i + (1 - mu_i) (.) x_prev_i ),  mu_i[j] =
 *   codebook_i[indices_i[j / 2]][j % 2]:  the mix is evaluated element by element as
 *   rwkvq_token_shift_mix defines it (binary32, one rounding per operation, then rounded to x_dtype)
 *   while the activations are loaded, so the result equals that of rwkvq_token_shift_mix followed by
 *   rwkvq_linear_dispatch on the same matrices, bit for bit, without the pass over memory and the
 *   launch in between.  mats: native layout only; ys[i]: [N_i] values of y_dtype.
 *   Errors as rwkvq_linear_dispatch; RWKVQ_ERR_UNSUPPORTED also for canonical-layout matrices,
 *   K > 20480 and kbits other than 6 or 8. */
typedef struct rwkvq_mix_input {
    const void* x;           /* DEVICE: [K] activations of the current token (x_dtype) */
    const void* x_prev;      /* DEVICE: [K] activations of the previous token */
    const uint8_t* indices;  /* DEVICE: [K / 2] indices of the mix weight's 2-vectors */
    const void* codebook;    /* DEVICE: 2^kbits x 2 fp16 entries */
    int32_t kbits;           /* 6 or 8 */
    int32_t reserved;
} rwkvq_mix_input;
int rwkvq_linear_dispatch_mixed(const rwkvq_matrix* mats, const rwkvq_mix_input* mixes, void* const* ys,
                                int n_mats, int x_dtype, int y_dtype, void* stream);

/* ---- element-wise operators of the RWKV block between the projections (App. A.1) ----
 *
 * rwkvq_wkv: Eq. "time mixing wkv" and the gate of Eq. "time mixing o" for a chunk of M tokens:
 *   out[t][c] = sigma(r[t][c]) * wkv_t[c], the vector that W_o multiplies, with
 *   wkv_t = (sum_{i<t} exp(-(t-1-i) w + k_i) v_i + exp(u + k_t) v_t) / (the same sums without v).
 *   The sums over earlier tokens are carried in `state`, 3 x d floats (a[d], b[d], p[d]): they equal
 *   a exp(p) and b exp(p); the call reads the state of the tokens before the chunk and leaves that
 *   after it.  A new sequence starts from a = b = 0, p = -1e38 (then wkv_1 = v_1).  r, k, v, out:
 *   DEVICE [M][d] of x_dtype (fp16 or bf16; out may not alias them); w (decay, positive forgets),
 *   u (bonus of the current token): DEVICE [d] floats.  Binary32 arithmetic, every exp() argument
 *   <= 0.  Sigma is the logistic function.  Chunks of fewer than 128 tokens run token by token, so
 *   that splitting such a chunk into several calls gives the same bits; longer chunks are cut into
 *   64 pieces that run side by side and are merged (the recurrence is linear in the carried sums),
 *   which agrees with the token-by-token result to rounding, not bit for bit.
 * rwkvq_relu2: out[i] = max(x[i], 0)^2 (Eq. "channel mixing o", the vector that W'_v multiplies).
 * rwkvq_sigmoid_gate: out[i] = sigma(r[i]) * y[i] (the gates of Eq. "time mixing o" and "channel
 *   mixing o").  n values of x_dtype each; out may alias an input.
 * r, k, v, x, y, out 16-byte aligned, w, u, state 4; asynchronous on `stream`; no scratch memory.
 * Errors: RWKVQ_ERR_NULL, RWKVQ_ERR_UNSUPPORTED (dtype), RWKVQ_ERR_SHAPE, RWKVQ_ERR_ALIGN,
 * RWKVQ_ERR_DEVICE. */
int rwkvq_wkv(const void* r, const void* k, const void* v, int x_dtype, int M, int d, const float* w,
              const float* u, float* state, void* out, void* stream);
int rwkvq_relu2(const void* x, int x_dtype, long long n, void* out, void* stream);

/* rwkvq_rkv_wkv: one token of time mixing in one launch: the three projections r, k, v (rkv[0..2], native
 *   layout, equal N = d, K <= 20480, any mix of SQ / VQ) of xs[0..2] ([K_i] of x_dtype each), stored in
 *   ys[0..2] ([d] of y_dtype, fp16 or bf16), and the step of rwkvq_wkv on them: `state` (3 x d floats)
 *   advanced in place, out[c] = sigma(r[c]) * wkv[c] ([d] of y_dtype).  The recurrence is per channel and
 *   channel c needs output row c of the three matrices: the workgroup that computes a row tile of all
 *   three steps its 16 channels.  The columns of a row are split over four wavefronts: the same bits as
 *   rwkvq_linear_dispatch on the three matrices (one call, M = 1) followed by rwkvq_wkv with M = 1
 *   when that call splits them the same way (d >= 2736), otherwise equal up to the order of the
 *   binary32 sums.  rkv, xs, ys: HOST arrays of three entries, read before
 *   return.  Errors: RWKVQ_ERR_NULL, RWKVQ_ERR_UNSUPPORTED (dtypes, canonical layout, K too long),
 *   RWKVQ_ERR_SHAPE (different N, or a descriptor's), RWKVQ_ERR_ALIGN, RWKVQ_ERR_DEVICE. */
int rwkvq_rkv_wkv(const rwkvq_matrix* rkv, const void* const* xs, void* const* ys, const float* w, const float* u,
                  float* state, void* out, int x_dtype, int y_dtype, void* stream);
int rwkvq_sigmoid_gate(const void* r, const void* y, int x_dtype, long long n, void* out, void* stream);

/* rwkvq_linear_dispatch_post: batch-1 projections with the element-wise operator that follows them
 *   in the block (App. A.1) applied before the output is stored, and optionally the token-shift mix
 *   in front (as rwkvq_linear_dispatch_mixed).  For matrix i, with y = Deq(W_i) . x_i rounded to
 *   y_dtype:  RWKVQ_POST_NONE stores y;  RWKVQ_POST_RELU2 stores max(y, 0)^2 (the input of W'_v,
 *   Eq. "channel mixing o");  RWKVQ_POST_SIGMOID_GATE stores sigma(gate[n]) * y[n] (Eq. "time mixing
 *   o", "channel mixing o"), gate: DEVICE [N_i] values of y_dtype written by an EARLIER call or
 *   launch (not by another matrix of this call).  The operator works in binary32 on the rounded y and
 *   its result is rounded to y_dtype: bit for bit what rwkvq_linear_dispatch (or _mixed) followed by
 *   rwkvq_relu2 / rwkvq_sigmoid_gate stores, without the launch and the pass in between.
 *   mixes == NULL: xs[i] is the input of matrix i ([K_i] of x_dtype).  mixes != NULL: mixes[i]
 *   describes it (x, x_prev and the quantized mix weight), xs is not read and may be NULL.
 *   n_mix > 0: besides z = op(y) in ys[i], the call stores, for p < n_mix,
 *   mix[p].out[n] = mu_p[n] z[n] + (1 - mu_p[n]) x_prev[n], mu_p[n] = codebook_p[indices_p[n / 2]][n % 2]:
 *   the token-shift mixes of Eq. "time mixing r/k/v" / "channel mixing r/k" that the NEXT stage's
 *   projections read, taken where the vector is produced (the mix is element-wise) instead of by every
 *   workgroup of the stage that consumes it; arithmetic and bits as rwkvq_token_shift_mix on the stored
 *   z.  Needs mixes == NULL (plain inputs) and a 16-bit y_dtype, else RWKVQ_ERR_UNSUPPORTED; x_prev and
 *   the mix outputs must not alias ys[i].
 *   mats: native layout, K <= 20480; posts, mats, xs, ys, mixes: HOST arrays, read before return.
 *   Errors as rwkvq_linear_dispatch_mixed; RWKVQ_ERR_UNSUPPORTED also for an unknown op,
 *   RWKVQ_ERR_NULL for a missing gate. */
enum { RWKVQ_POST_NONE = 0, RWKVQ_POST_RELU2 = 1, RWKVQ_POST_SIGMOID_GATE = 2 };
typedef struct rwkvq_post_mix {  /* one token-shift mix of the stage that follows */
    const uint8_t* indices;  /* DEVICE: [N / 2] indices of the mix weight's 2-vectors */
    const void* codebook;    /* DEVICE: 2^kbits x 2 fp16 entries */
    void* out;               /* DEVICE: [N] values of y_dtype */
    int32_t kbits;           /* 6 or 8 */
    int32_t reserved;
} rwkvq_post_mix;
typedef struct rwkvq_post_op {
    int32_t op;         /* RWKVQ_POST_* */
    int32_t n_mix;      /* 0..4: the stored output z (after `op`) also leaves as n_mix token-shift mixes */
    const void* gate;   /* DEVICE, RWKVQ_POST_SIGMOID_GATE only */
    const void* x_prev; /* DEVICE, n_mix > 0: [N] values of y_dtype, the previous token's z */
    rwkvq_post_mix mix[4];
} rwkvq_post_op;
int rwkvq_linear_dispatch_post(const rwkvq_matrix* mats, const void* const* xs, const rwkvq_mix_input* mixes,
                               const rwkvq_post_op* posts, void* const* ys, int n_mats, int x_dtype, int y_dtype,
                               void* stream);

#ifdef __cplusplus
}
#endif
#endif /* RWKVQ_H */
