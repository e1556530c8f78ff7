/* grass.h -- C ABI of the GraSS / FactGraSS per-sample gradient compression
 * library for AMD MI355X (gfx950).
 *
 * Conventions shared by every entry point
 *   - Pointers are DEVICE pointers unless the parameter name starts with
 *     `host_`.  Matrices are row-major; `ld*` is the distance between rows in
 *     ELEMENTS.  The caller owns every buffer; the library allocates nothing.
 *   - Scratch memory is a caller-supplied workspace `ws` of at least the size
 *     the matching `*_workspace_bytes` query returns for the same dimension
 *     arguments (a query may return 0, then `ws` may be NULL).  Workspace
 *     contents are undefined on return.  `ws` must be 256-byte aligned.
 *   - Every call enqueues its kernels on `stream` (a hipStream_t passed as an
 *     opaque pointer; NULL is the default stream) and returns without
 *     synchronising.  Outputs are overwritten, never accumulated into, and
 *     are valid once the stream has been synchronised.
 *   - Errors are reported through the return value only.  All argument checks
 *     run on the host before anything is launched, so a call that returns
 *     GRASS_EINVAL, GRASS_EWORKSPACE or GRASS_EUNSUPPORTED has done nothing.
 *     n == 0 is a successful no-op.  Index arrays (`idx*`) are trusted to be
 *     ascending, distinct and in range; `grass_check_indices` verifies that.
 *   - Randomness: every index, bucket and sign is a pure function of
 *     (seed, stream_id, counter) through the splitmix64 generator
 *         sm(seed, c)            = finalise(seed + (c + 1) * 0x9E3779B97F4A7C15)
 *         H(seed, stream_id, c)  = sm(sm(seed, stream_id), c)
 *     evaluated in registers; no table is kept between calls (the unmasked
 *     SJLT of long rows fills a transient table of 2 bytes per position in its
 *     workspace, see grass_sjlt).
 *     Suggested stream ids: 0 mask and 1 SJLT for general vectors; for linear
 *     layer l, 16+4l input mask, 17+4l output-gradient mask, 18+4l SJLT.
 *   - Determinism: integer outputs (indices, tables) are bit-reproducible.
 *     Floating-point outputs use a fixed cross-block reduction order; inside
 *     a block, additions into LDS buckets happen in hardware-arbitrated order,
 *     so results can differ between runs in the last bits.
 *   - Threads: the library keeps no mutable process-wide settings.  Entry
 *     points may be called from several host threads at once as long as calls
 *     that share a workspace or an output buffer are ordered by the caller
 *     (same stream, or events).
 */
#ifndef GRASS_H
#define GRASS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    GRASS_OK = 0,
    GRASS_EINVAL = 1,       /* a size or pointer argument is invalid            */
    GRASS_EWORKSPACE = 2,   /* workspace missing, misaligned or too small        */
    GRASS_EHIP = 3,         /* the HIP runtime reported an error at launch       */
    GRASS_EUNSUPPORTED = 4, /* valid request outside what the kernels cover      */
    GRASS_ETOOLARGE = 5     /* needs more scratch memory than the library's fixed
                               buffer holds (grass_sjlt_noalloc)                 */
} grass_status;

typedef void* grass_stream;

/* Optional launch-shape overrides for experiments, handed to the calls that
 * take a `host_tuning` argument (a HOST pointer, read during the call only;
 * NULL = the library's heuristics).  A field that is 0 or not one of the listed
 * values leaves that choice to the heuristic.  The workspace query and the call
 * must be given the same values.  There is no process-wide setting.
 *   sjlt_rows_per_block  1, 2, 4 or 8 rows (samples) per workgroup
 *   sjlt_column_chunks   chunks of SJLT input positions per row group
 *   sjlt_threads         256, 512 or 1024 threads per workgroup
 *   sjlt_accumulator     2 = fp32 LDS buckets updated by compare-and-swap,
 *                        3 = fp64 LDS buckets updated by the fp64 atomic add
 *   factgrass_tokens_per_block  tokens per workgroup (rounded up to 32)      */
typedef struct {
    int sjlt_rows_per_block;
    int sjlt_column_chunks;
    int sjlt_threads;
    int sjlt_accumulator;
    int factgrass_tokens_per_block;
} grass_tuning;

/* Largest SJLT output dimension k the LDS-resident accumulators cover. */
#define GRASS_MAX_K 32768u
/* Largest masked factor width (k_in', k_out') of factgrass_linear. */
#define GRASS_MAX_FACTOR 128u

const char* grass_strerror(int status);
int grass_version(void);

/* ---------------------------------------------------------------- Random Mask
 * Sec. 3.2 "Random Mask": keep a uniformly random subset of k' of the p
 * coordinates.  Coordinate j draws key_j = H(seed, stream_id, j); the k'
 * smallest (key_j, j) pairs are kept and written to idx[0..k') in ascending
 * order of j (k' == p yields 0..p-1).  p < 2^31.
 * One-time set-up per (seed, stream_id, p, k').                              */
grass_status grass_mask_indices_workspace_bytes(uint64_t p, uint32_t kprime, size_t* host_bytes);
grass_status grass_mask_indices(uint64_t seed, uint64_t stream_id, uint64_t p, uint32_t kprime,
                                int32_t* idx, void* ws, size_t ws_bytes, grass_stream stream);

/* Debug helper: *host_ok = 1 iff idx[0..kprime) is strictly ascending and
 * within [0, p).  Synchronises the stream; concurrent calls are serialised
 * inside the library (they share one result word per device).               */
grass_status grass_check_indices(const int32_t* idx, uint32_t kprime, uint64_t p, int* host_ok,
                                 grass_stream stream);

/* Sec. 3.2: Mask_k'(g) = M g, the sub-vector g[idx] of every row (Random Mask
 * or Selective Mask indices, supplied by the caller).
 * g: n x p fp32 (ldg >= p); out: n x kprime fp32 (ldo >= kprime).            */
grass_status grass_mask(const float* g, uint64_t n, uint64_t p, uint64_t ldg,
                        const int32_t* idx, uint32_t kprime,
                        float* out, uint64_t ldo, grass_stream stream);

/* ----------------------------------------------------------------------- SJLT
 * Sec. 3.1 "Sparse Johnson-Lindenstrauss Transform": out = P g with s
 * non-zeros of magnitude 1/sqrt(s) per column of P.  s must divide k; with
 * m = k/s, the r-th non-zero (r in [0,s)) of input position j is
 *     h = H(seed, stream_id, j*s + r);  row = r*m + floor((h >> 32) * m / 2^32);
 *     sign = +1 if (h & 1) == 0 else -1.
 *
 * grass_sjlt_tables writes these for j in [0,d): bucket[j*s + r], sign[j*s + r]
 * (tests and inspection only; the hot path recomputes them in registers).    */
grass_status grass_sjlt_tables(uint64_t seed, uint64_t stream_id, uint64_t d, uint32_t k, uint32_t s,
                               uint32_t* bucket, int8_t* sign, grass_stream stream);

/* grass_sjlt: idx == NULL  -> SJLT_k of every row of g (n x p), input dim p.
 *             idx != NULL  -> GraSS = SJLT_k o Mask_k' (Sec. 3.3.1), fused: the
 *                             masked vector g[:, idx] (k' entries) is never
 *                             written; the hash key is the position inside it.
 * g: n x p fp32, ldg >= p.  kprime is ignored when idx == NULL.
 * out: n x k fp32, ldo >= k.  k <= GRASS_MAX_K.
 * Fastest when g and ldg are 16-byte aligned (ldg % 4 == 0); any alignment
 * of at least 4 bytes works.
 * Workspace: partial sums of the column chunks, and for long unmasked inputs
 * with s == 1 room for a per-call table of 16-bit (bucket, sign) entries.  A
 * workspace that is too small for the partial sums is GRASS_EWORKSPACE; one
 * that holds them but not the table is accepted and the call hashes every
 * position instead (same result bit for bit, a few per cent slower).         */
grass_status grass_sjlt_workspace_bytes(uint64_t n, uint64_t p, uint32_t kprime_or_0,
                                        uint32_t k, uint32_t s, const grass_tuning* host_tuning,
                                        size_t* host_bytes);
grass_status grass_sjlt(const float* g, uint64_t n, uint64_t p, uint64_t ldg,
                        const int32_t* idx, uint32_t kprime,
                        uint32_t k, uint32_t s, uint64_t seed, uint64_t stream_id,
                        float* out, uint64_t ldo,
                        void* ws, size_t ws_bytes, const grass_tuning* host_tuning, grass_stream stream);
/* The same operation on gradients stored as bf16 (n x p 16-bit words, ldg in
 * elements, 2-byte aligned): every value is used exactly (a bf16 is the upper
 * half of an fp32), accumulation and output are as in grass_sjlt.  Workspace:
 * grass_sjlt_workspace_bytes.  Fastest when rows are 16-byte aligned
 * (ldg % 8 == 0) or the batch has enough rows to be grouped by alignment.     */
grass_status grass_sjlt_bf16(const void* g, uint64_t n, uint64_t p, uint64_t ldg,
                             const int32_t* idx, uint32_t kprime,
                             uint32_t k, uint32_t s, uint64_t seed, uint64_t stream_id,
                             float* out, uint64_t ldo,
                             void* ws, size_t ws_bytes, const grass_tuning* host_tuning, grass_stream stream);

/* Introspection for benchmarks and profiles: writes into host_text (a HOST
 * buffer of host_text_bytes, 160 are enough) which kernel instantiation and
 * launch shape grass_sjlt / grass_sjlt_bf16 would use for these arguments, e.g.
 *   "sjlt_kernel<float,4,1,4,true,3,1> grid=1024x1 block=1024 lds=131072 chunks=1 reduce=0 table=0"
 * (template arguments: input type, rows per workgroup, positions per load,
 * loads in flight, fused mask, accumulator, hash mode -- the name a profiler
 * lists, without spaces).  g may be NULL (its alignment then counts as
 * unknown); with_workspace says whether the call would be given the workspace
 * the query reports.  Launches nothing.                                       */
grass_status grass_sjlt_describe(const void* g, int input_is_bf16, uint64_t n, uint64_t p, uint64_t ldg,
                                 uint32_t kprime_or_0, uint32_t k, uint32_t s, int with_workspace,
                                 const grass_tuning* host_tuning, char* host_text, size_t host_text_bytes);

/* grass_sjlt for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same operation, arguments and results as grass_sjlt (fp32
 * input, heuristic launch shape) without `ws`: the partial sums of the column
 * chunks (and the transient table, when it fits behind them) live in a buffer
 * of GRASS_NOALLOC_SCRATCH_BYTES that is part of the library's device code, one
 * copy per GPU for the life of the process.  The call allocates and frees
 * nothing; its first call on a device looks up the buffer's address.
 * A problem whose partial sums (column chunks x n x k x 4 bytes) exceed the
 * buffer is refused with GRASS_ETOOLARGE before anything is launched: use
 * grass_sjlt with a workspace for those.  Large batches of the fused mask path
 * need no scratch memory at all and are never refused.
 * All calls on one GPU share the buffer: calls that may overlap in time (on
 * different streams, or from different threads) race on it and must be ordered
 * by the caller.  Nothing in the buffer needs to start at zero.               */
#define GRASS_NOALLOC_SCRATCH_BYTES (32u << 20)
grass_status grass_sjlt_noalloc(const float* g, uint64_t n, uint64_t p, uint64_t ldg,
                                const int32_t* idx, uint32_t kprime,
                                uint32_t k, uint32_t s, uint64_t seed, uint64_t stream_id,
                                float* out, uint64_t ldo, grass_stream stream);

/* ------------------------------------------------------------------ FactGraSS
 * Sec. 3.3.2 "Factorized GraSS" for one linear layer, using Eq. (2)/(3):
 *   1. mask every token's layer input x_t (d_in) to idx_in (k_in' entries) and
 *      its pre-activation gradient g_t (d_out) to idx_out (k_out' entries);
 *   2. v[a*k_out' + b] = sum_t x_t[idx_in[a]] * g_t[idx_out[b]]  (fp32 accumulate
 *      of exact bf16 products; the d_out x d_in gradient is never formed);
 *   3. out_i = SJLT_k(v) with input dimension k_in'*k_out' (hash as above).
 * x: (n, T, d_in) bf16, gout: (n, T, d_out) bf16, both contiguous.
 * out: n x k fp32 with row distance ldo (lets the caller place layer l at a
 * column offset of a concatenated row).  k_in', k_out' <= GRASS_MAX_FACTOR.  */
grass_status factgrass_linear_workspace_bytes(uint64_t n, uint64_t T, uint32_t kin_p, uint32_t kout_p,
                                              uint32_t k, uint32_t s, const grass_tuning* host_tuning,
                                              size_t* host_bytes);
grass_status factgrass_linear(const void* x, const void* gout,
                              uint64_t n, uint64_t T, uint32_t d_in, uint32_t d_out,
                              const int32_t* idx_in, uint32_t kin_p,
                              const int32_t* idx_out, uint32_t kout_p,
                              uint32_t k, uint32_t s, uint64_t seed, uint64_t stream_id,
                              float* out, uint64_t ldo,
                              void* ws, size_t ws_bytes, const grass_tuning* host_tuning, grass_stream stream);

/* The same for many linear layers of one model pass in a single launch (the
 * per-layer gradients are compressed independently, Sec. 3.3.2; concatenating
 * the blocks gives k = sum_l k_l).  All layers share n, T, the mask widths, k
 * and s; each brings its own shapes, indices, SJLT stream id and output block.
 * host_layers is a HOST array; every pointer inside it is a device pointer.
 * The table is copied into the workspace on `stream` before the kernels run.   */
typedef struct {
    const void* x;            /* (n, T, d_in)  bf16 */
    const void* gout;         /* (n, T, d_out) bf16 */
    const int32_t* idx_in;    /* kin_p ascending indices into [0, d_in)  */
    const int32_t* idx_out;   /* kout_p ascending indices into [0, d_out) */
    uint32_t d_in, d_out;
    uint64_t stream_id;       /* SJLT stream of this layer */
    float* out;               /* n x k block of this layer, row distance ldo */
} factgrass_layer;
grass_status factgrass_layers_workspace_bytes(uint32_t n_layers, uint64_t n, uint64_t T, uint32_t kin_p,
                                              uint32_t kout_p, uint32_t k, uint32_t s,
                                              const grass_tuning* host_tuning, size_t* host_bytes);
grass_status factgrass_layers(const factgrass_layer* host_layers, uint32_t n_layers,
                              uint64_t n, uint64_t T, uint32_t kin_p, uint32_t kout_p,
                              uint32_t k, uint32_t s, uint64_t seed, uint64_t ldo,
                              void* ws, size_t ws_bytes, const grass_tuning* host_tuning, grass_stream stream);

/* ---------------------------------------------------------- LoGra baseline
 * Sec. 3.3.2 "Recap on LoGra", Eq. (3): the factorised dense projection
 * Gauss_{k_in (x) k_out} FactGraSS is compared with,
 *     out_i[a*k_out + b] = sum_t (P_in x_t)[a] * (P_out g_t)[b].
 * x: (n, T, d_in) bf16, gout: (n, T, d_out) bf16, P_in: k_in x d_in bf16,
 * P_out: k_out x d_out bf16 (all contiguous; e.g. grass_gauss_matrix followed by
 * grass_to_bf16).  out: n x (k_in*k_out) fp32, ldo >= k_in*k_out.  bf16 products
 * are exact in fp32; both contractions accumulate in fp32.
 * k_in, k_out <= 64; d_in, d_out multiples of 8 and at most 2^24 (GRASS_EUNSUPPORTED otherwise). */
grass_status logra_linear_workspace_bytes(uint64_t n, uint64_t T, uint32_t k_in, uint32_t k_out,
                                          size_t* host_bytes);
grass_status logra_linear(const void* x, const void* gout,
                          uint64_t n, uint64_t T, uint32_t d_in, uint32_t d_out,
                          const void* P_in, uint32_t k_in, const void* P_out, uint32_t k_out,
                          float* out, uint64_t ldo,
                          void* ws, size_t ws_bytes, grass_stream stream);

/* ---------------------------------------------------------------------- score
 * Sec. 2.1, attribute stage: scores[m, i] = <test_m, train_i> for all pairs of
 * compressed gradients (no preconditioner).
 * train: N x K fp32 (ld_train >= K), test: M x K fp32, scores: M x N fp32.
 * compute_mode 0: fp32 MFMA.  1: inputs rounded to bf16 (nearest-even), bf16
 * MFMA with fp32 accumulation.
 * Workspace (optional, from grass_score_workspace_bytes): with it, mode 1
 * rounds both operands once into the workspace and runs the direct-to-LDS bf16
 * kernel (about twice as fast as rounding on the fly), and products whose M x N
 * output has few tiles but a long K are split over K ranges with fixed-order
 * partial sums.  ws == NULL selects the paths that need no scratch memory; a
 * non-NULL workspace that is too small or not 256-byte aligned is
 * GRASS_EWORKSPACE.                                                           */
grass_status grass_score_workspace_bytes(uint64_t N, uint64_t M, uint64_t K, int compute_mode,
                                         size_t* host_bytes);
grass_status grass_score(const float* train, const float* test, int compute_mode,
                         uint64_t N, uint64_t M, uint64_t K,
                         uint64_t ld_train, uint64_t ld_test,
                         float* scores, uint64_t ld_scores,
                         void* ws, size_t ws_bytes, grass_stream stream);

/* The same scores for callers that keep compressed gradients in bf16 (Sec. 2.1;
 * halves the bytes of the attribute stage): train N x K and test M x K are bf16
 * bit patterns, products are exact in fp32, accumulation is fp32.  Requires
 * K, ld_train and ld_test to be multiples of 8 and 16-byte aligned bases
 * (GRASS_EUNSUPPORTED otherwise).  grass_to_bf16 converts an fp32 matrix
 * (rows x cols) to bf16 with round-to-nearest-even.                           */
grass_status grass_to_bf16(const float* src, uint64_t rows, uint64_t cols, uint64_t ld_src,
                           void* dst, uint64_t ld_dst, grass_stream stream);
grass_status grass_score_bf16(const void* train, const void* test,
                              uint64_t N, uint64_t M, uint64_t K,
                              uint64_t ld_train, uint64_t ld_test,
                              float* scores, uint64_t ld_scores, grass_stream stream);

/* ---------------------------------------------- dense Gaussian baseline (Sec. 2.2)
 * g_hat = P g with P (k x p), P_ab ~ N(0, 1/k), generated from the counter
 * hash by Box-Muller: entry (a, b) uses H(seed, stream_id, a*p + b).
 * grass_gauss_matrix writes columns [p0, p0+pc) of P as a k x pc fp32 matrix
 * (ldP >= pc); grass_gauss_project computes out = g P^T (n x k fp32) in
 * p-chunks of at most p_chunk columns, regenerating P chunk by chunk in the
 * workspace.  compute_mode 0: fp32 MFMA.  1: both the chunk of P and the chunk
 * of g are rounded to bf16 (nearest-even), bf16 MFMA, fp32 accumulation.      */
grass_status grass_gauss_matrix(uint64_t seed, uint64_t stream_id, uint64_t p, uint32_t k,
                                uint64_t p0, uint64_t pc, float* P, uint64_t ldP, grass_stream stream);
grass_status grass_gauss_project_workspace_bytes(uint64_t n, uint64_t p, uint32_t k, uint64_t p_chunk,
                                                 size_t* host_bytes);
grass_status grass_gauss_project(const float* g, uint64_t n, uint64_t p, uint64_t ldg,
                                 uint32_t k, uint64_t seed, uint64_t stream_id,
                                 uint64_t p_chunk, int compute_mode,
                                 float* out, uint64_t ldo,
                                 void* ws, size_t ws_bytes, grass_stream stream);

/* ------------------------------------------- projected FIM and iFVP (cache stage)
 * Sec. 2.1, cache stage steps 2 and 3, applied to compressed gradients (the
 * "projected FIM" of Sec. 2.2; per layer block for the block-diagonal FIM of
 * Sec. 3.3.2), with the damping term of App. B.
 *
 * grass_fim: F = (1/N) sum_i g_i g_i^T for the rows of G (N x k fp32 device,
 * ldg >= k).  F is k x k fp32 (ldf >= k), written in full and exactly
 * symmetric.  fp32 MFMA, accumulated over interleaved ranges of the rows of G
 * in a fixed order (bit-reproducible).  Fastest when G is 16-byte aligned and k
 * and ldg are multiples of 4: G is then read in place, otherwise transposed
 * chunks go through the workspace.  Workspace from
 * grass_fim_workspace_bytes(N, k), 256-byte aligned.
 *
 * grass_fim_inverse: W = (F + lambda I)^{-1}, k x k fp32 (ldw >= k), lambda >= 0
 * absolute.  Only the lower triangle of F is read.  The factorisation runs in
 * fp64 (blocked Cholesky, triangular inverse, W = L^{-T} L^{-1}) and is rounded
 * to fp32 once at the end.  info (device int32, may be NULL) receives 0, or the
 * 1-based index of the first non-positive pivot (F + lambda I not positive
 * definite in fp64; W is then meaningless).  k <= 32768.  Workspace
 * 2 * kp^2 * 8 bytes with kp = k rounded up to 64.
 *
 * grass_ifvp: out (N x k fp32, ldo >= k), row i = W g_i for the rows g_i of G
 * (N x k).  W must be symmetric (as grass_fim_inverse writes it).  fp32 MFMA.
 * Scores with the preconditioner are then grass_score(out_train, test) =
 * <g_test, (F + lambda I)^{-1} g_i>.
 * Errors: GRASS_EINVAL for null pointers, k = 0, N = 0 in grass_fim, short
 * leading dimensions, negative or NaN lambda; GRASS_EWORKSPACE; GRASS_EHIP.   */
grass_status grass_fim_workspace_bytes(uint64_t N, uint32_t k, size_t* host_bytes);
grass_status grass_fim(const float* G, uint64_t N, uint32_t k, uint64_t ldg, float* F, uint64_t ldf,
                       void* ws, size_t ws_bytes, grass_stream stream);
grass_status grass_fim_inverse_workspace_bytes(uint32_t k, size_t* host_bytes);
grass_status grass_fim_inverse(const float* F, uint32_t k, uint64_t ldf, double lambda,
                               float* W, uint64_t ldw, int32_t* info,
                               void* ws, size_t ws_bytes, grass_stream stream);
grass_status grass_ifvp(const float* G, uint64_t N, uint32_t k, uint64_t ldg,
                        const float* W, uint64_t ldw, float* out, uint64_t ldo, grass_stream stream);

/* ------------------------------------------------------------- Selective Mask
 * Sec. 3.2 "Selective Mask", Eq. (1), with the practical notes of App. B.4:
 * logits S in R^p are trained to maximise
 *   mean over test rows t of corr_i( <g_i, gt_t>, <sigma*g_i, sigma*gt_t> )  -  lambda * sum_j sigma_j,
 * sigma = sigmoid(S / temperature), corr the Pearson correlation over the n train
 * rows.  The paper fixes no optimiser: grass_selective_mask_grad gives the value
 * and gradient any first-order method needs, grass_selective_mask_train runs
 * plain gradient ascent with them.
 *
 * grass_selective_mask_grad: objective value and gradient with respect to S.
 *   G  (n x p fp32, ldg)  train gradients;  Gt (m x p fp32, ldgt) test gradients
 *      (fastest when G is 16-byte aligned and ldg is a multiple of 4: both large
 *      products then take G in place from HBM; any 4-byte alignment works);
 *   A  (m x n fp32, lda)  exact scores A[t][i] = <gt_t, g_i>, i.e.
 *                         grass_score(train = G, test = Gt), computed once;
 *   S  (p fp32) logits;  grad (p fp32) receives d objective / d S;
 *   objective (device double, may be NULL) receives the objective value.
 *   n >= 2, m >= 1.  A test row whose exact or masked scores are constant over i
 *   has no correlation: it contributes 0 to the value and to the gradient.
 *   Two fp32 MFMA GEMMs of 2*m*n*p flops each; reductions in fp64, fixed order.
 *
 * grass_selective_mask_indices: index extraction.  k == 0: every j with
 *   sigma(S_j) >= 1/2 (S_j >= 0), ascending; their number goes to *count (device
 *   uint32, required) and idx must hold p entries.  k > 0 ("ensuring exact k"):
 *   the k largest logits, ties towards the smaller index, ascending; count (may
 *   be NULL) receives k.  S must not contain NaN.  p < 2^31.
 * All pointers device; workspaces from the *_workspace_bytes queries.           */
grass_status grass_selective_mask_grad_workspace_bytes(uint64_t n, uint64_t m, uint64_t p, size_t* host_bytes);
grass_status grass_selective_mask_grad(const float* G, uint64_t n, uint64_t ldg,
                                       const float* Gt, uint64_t m, uint64_t ldgt, uint64_t p,
                                       const float* A, uint64_t lda, const float* S,
                                       double lambda, double temperature,
                                       float* grad, double* objective,
                                       void* ws, size_t ws_bytes, grass_stream stream);
/* grass_selective_mask_train: solves Eq. (1) by first-order ascent (the paper
 * names no optimiser; this is plain gradient ascent over all rows handed in),
 *     S <- S + lr * d objective / d S   at temperature host_temperatures[i],
 * for i = 0 .. steps-1, with the decreasing inverse-temperature schedule of
 * App. B.4 ("Ensuring Exact k") supplied by the caller as a HOST array of
 * `steps` positive numbers (a constant array trains without annealing).  S (p
 * fp32, device) is updated in place; objectives (device double[steps], may be
 * NULL) receives the objective before each step.  All steps are enqueued back to
 * back; the host array is read during the call only.  Start from logits that are
 * not all equal: constant logits give correlation 1 and a zero data gradient.
 * Follow with grass_selective_mask_indices to extract the mask.  G, Gt, A as in
 * grass_selective_mask_grad.
 *
 * grass_score_correlation: *mean_corr (device double) = mean over the m rows of
 * the Pearson correlation (1/n moments, fp64, fixed order) between row t of X
 * and row t of Y, two m x n fp32 score matrices; a row that is constant in X or
 * Y contributes 0.  With X = grass_score(G, Gt) and Y the scores of the masked
 * gradients (grass_mask on both, then grass_score) this is the first term of
 * Eq. (1) for a binary mask.  n >= 2.                                          */
grass_status grass_selective_mask_train_workspace_bytes(uint64_t n, uint64_t m, uint64_t p, size_t* host_bytes);
grass_status grass_selective_mask_train(const float* G, uint64_t n, uint64_t ldg,
                                        const float* Gt, uint64_t m, uint64_t ldgt, uint64_t p,
                                        const float* A, uint64_t lda, float* S,
                                        double lambda, double lr, const double* host_temperatures, uint32_t steps,
                                        double* objectives, void* ws, size_t ws_bytes, grass_stream stream);
grass_status grass_score_correlation_workspace_bytes(uint64_t m, size_t* host_bytes);
grass_status grass_score_correlation(const float* X, uint64_t ldx, const float* Y, uint64_t ldy,
                                     uint64_t m, uint64_t n, double* mean_corr,
                                     void* ws, size_t ws_bytes, grass_stream stream);
/* Factorised form for one linear layer (App. B.4 "Linear Layer", one token per
 * sample as in the paper's formula): per-sample gradients are z_in (x) z_out,
 * the mask is sigma(S_in) (x) sigma(S_out), the penalty lambda * (|sigma(S_in)|_1
 * + |sigma(S_out)|_1).  Z_in n x d_in, Z_out n x d_out (train), Zt_in m x d_in,
 * Zt_out m x d_out (test), A[t][i] = <zt_in_t, z_in_i> * <zt_out_t, z_out_i>
 * (two grass_score calls and a product).  grad_in (d_in) and grad_out (d_out)
 * receive d objective / d S_in and d S_out.  The layer gradient is never formed. */
grass_status grass_selective_mask_grad_factorized_workspace_bytes(uint64_t n, uint64_t m, uint64_t d_in,
                                                                  uint64_t d_out, size_t* host_bytes);
grass_status grass_selective_mask_grad_factorized(const float* Z_in, const float* Z_out, uint64_t n,
                                                  uint64_t ld_zin, uint64_t ld_zout,
                                                  const float* Zt_in, const float* Zt_out, uint64_t m,
                                                  uint64_t ld_ztin, uint64_t ld_ztout,
                                                  uint64_t d_in, uint64_t d_out,
                                                  const float* A, uint64_t lda,
                                                  const float* S_in, const float* S_out,
                                                  double lambda, double temperature,
                                                  float* grad_in, float* grad_out, double* objective,
                                                  void* ws, size_t ws_bytes, grass_stream stream);
/* Samples that are sequences of tokens (the case FactGraSS compresses): the
 * layer gradient of a sample is sum_t z_in_t (x) z_out_t (Eq. (2)), so an inner
 * product of two layer gradients is the sum over all token pairs of
 * <z_in_t, z_in_t'> * <z_out_t, z_out_t'>, with or without the mask weights.
 * Rows of Z_in / Z_out are tokens: train sample i owns rows i*T .. i*T+T-1 of
 * the (n*T)-row matrices, test sample t rows t*Tt .. t*Tt+Tt-1 of the
 * (m*Tt)-row matrices.  T = Tt = 1 is grass_selective_mask_grad_factorized.
 *
 * grass_graddot_factorized: A (m x n fp32, lda) receives the exact scores
 *   A[t][i] = <layer gradient of test sample t, layer gradient of train sample i>.
 * grass_selective_mask_grad_factorized_seq: objective and both gradients for
 *   such samples; A as produced by grass_graddot_factorized.
 * Both use the workspace of the _seq query; n*T and m*Tt below 2^31.          */
grass_status grass_graddot_factorized_workspace_bytes(uint64_t n, uint64_t T, uint64_t m, uint64_t Tt,
                                                      uint64_t d_in, uint64_t d_out, size_t* host_bytes);
grass_status grass_graddot_factorized(const float* Z_in, const float* Z_out, uint64_t n, uint64_t T,
                                      uint64_t ld_zin, uint64_t ld_zout,
                                      const float* Zt_in, const float* Zt_out, uint64_t m, uint64_t Tt,
                                      uint64_t ld_ztin, uint64_t ld_ztout,
                                      uint64_t d_in, uint64_t d_out, float* A, uint64_t lda,
                                      void* ws, size_t ws_bytes, grass_stream stream);
grass_status grass_selective_mask_grad_factorized_seq_workspace_bytes(uint64_t n, uint64_t T, uint64_t m, uint64_t Tt,
                                                                      uint64_t d_in, uint64_t d_out,
                                                                      size_t* host_bytes);
grass_status grass_selective_mask_grad_factorized_seq(const float* Z_in, const float* Z_out, uint64_t n, uint64_t T,
                                                      uint64_t ld_zin, uint64_t ld_zout,
                                                      const float* Zt_in, const float* Zt_out, uint64_t m, uint64_t Tt,
                                                      uint64_t ld_ztin, uint64_t ld_ztout,
                                                      uint64_t d_in, uint64_t d_out,
                                                      const float* A, uint64_t lda,
                                                      const float* S_in, const float* S_out,
                                                      double lambda, double temperature,
                                                      float* grad_in, float* grad_out, double* objective,
                                                      void* ws, size_t ws_bytes, grass_stream stream);
/* grass_selective_mask_train_factorized: the same first-order ascent as
 * grass_selective_mask_train on the factorised problem: both logit vectors take
 *     S_in <- S_in + lr * dL/dS_in,   S_out <- S_out + lr * dL/dS_out
 * per entry of the host temperature schedule, both derivatives evaluated at the
 * logits before the step.  S_in (d_in) and S_out (d_out) are updated in place;
 * objectives (device double[steps], may be NULL) receives the objective before
 * each step.  Other arguments as in grass_selective_mask_grad_factorized.     */
grass_status grass_selective_mask_train_factorized_workspace_bytes(uint64_t n, uint64_t m, uint64_t d_in,
                                                                   uint64_t d_out, size_t* host_bytes);
grass_status grass_selective_mask_train_factorized(const float* Z_in, const float* Z_out, uint64_t n,
                                                   uint64_t ld_zin, uint64_t ld_zout,
                                                   const float* Zt_in, const float* Zt_out, uint64_t m,
                                                   uint64_t ld_ztin, uint64_t ld_ztout,
                                                   uint64_t d_in, uint64_t d_out,
                                                   const float* A, uint64_t lda,
                                                   float* S_in, float* S_out,
                                                   double lambda, double lr,
                                                   const double* host_temperatures, uint32_t steps,
                                                   double* objectives,
                                                   void* ws, size_t ws_bytes, grass_stream stream);
/* grass_selective_mask_train_factorized_seq: that training loop for samples that
 * are sequences of tokens (the layer gradient of a sample is the sum over its
 * tokens of the Kronecker products, Eq. (2)); rows of Z_* are tokens as in
 * grass_selective_mask_grad_factorized_seq, T = Tt = 1 is the call above.      */
grass_status grass_selective_mask_train_factorized_seq_workspace_bytes(uint64_t n, uint64_t T, uint64_t m, uint64_t Tt,
                                                                       uint64_t d_in, uint64_t d_out,
                                                                       size_t* host_bytes);
grass_status grass_selective_mask_train_factorized_seq(const float* Z_in, const float* Z_out, uint64_t n, uint64_t T,
                                                       uint64_t ld_zin, uint64_t ld_zout,
                                                       const float* Zt_in, const float* Zt_out, uint64_t m, uint64_t Tt,
                                                       uint64_t ld_ztin, uint64_t ld_ztout,
                                                       uint64_t d_in, uint64_t d_out,
                                                       const float* A, uint64_t lda,
                                                       float* S_in, float* S_out,
                                                       double lambda, double lr,
                                                       const double* host_temperatures, uint32_t steps,
                                                       double* objectives,
                                                       void* ws, size_t ws_bytes, grass_stream stream);
grass_status grass_selective_mask_indices_workspace_bytes(uint64_t p, size_t* host_bytes);
grass_status grass_selective_mask_indices(const float* S, uint64_t p, uint32_t k, int32_t* idx,
                                          uint32_t* count, void* ws, size_t ws_bytes, grass_stream stream);

/* ------------------------------------------- factorised baselines of Table 2
 * Sec. 3.3.2 ("Bottlenecks of integrating GraSS with LoGra"): the dense factor
 * projections of LoGra can be replaced by other compressors, giving
 * Mask_{k_in x k_out}, SJLT_{k_in x k_out} and GraSS_{k_in x k_out}.
 *
 * factmask_linear: Mask_{k_in x k_out}, i.e. stages 1 and 2 of factgrass_linear
 * without the sparse projection: out_i[a*k_out' + b] = sum_t x_t[idx_in[a]] *
 * g_t[idx_out[b]]; out is n x (k_in'*k_out') fp32, ldo >= k_in'*k_out'.  Arguments
 * as in factgrass_linear.
 *
 * grass_projection_matrix: the compressor as an explicit dense matrix P (k x p
 * fp32, ldP >= p, fully overwritten): idx == NULL -> the SJLT matrix of
 * grass_sjlt (s non-zeros +-1/sqrt(s) per column); idx != NULL -> the GraSS
 * matrix SJLT_k * Mask_k' (non-zeros only in the kept columns).  Handing two such
 * matrices (converted with grass_to_bf16; exact for s = 1, 4, 16) to
 * logra_linear gives SJLT_{k_in x k_out} or GraSS_{k_in x k_out}: at factor sizes
 * k_in, k_out <= 64 the dense matrix-core product is the fast way to apply a
 * sparse projection on this chip.  Also a debugging aid (P g == grass_sjlt(g)). */
grass_status factmask_linear_workspace_bytes(uint64_t n, uint64_t T, uint32_t kin_p, uint32_t kout_p,
                                             size_t* host_bytes);
grass_status factmask_linear(const void* x, const void* gout,
                             uint64_t n, uint64_t T, uint32_t d_in, uint32_t d_out,
                             const int32_t* idx_in, uint32_t kin_p,
                             const int32_t* idx_out, uint32_t kout_p,
                             float* out, uint64_t ldo,
                             void* ws, size_t ws_bytes, grass_stream stream);
grass_status grass_projection_matrix(uint64_t seed, uint64_t stream_id, uint64_t p,
                                     const int32_t* idx, uint32_t kprime,
                                     uint32_t k, uint32_t s, float* P, uint64_t ldP, grass_stream stream);

/* --------------------------------------------------------- measurement aid
 * Not part of the method; for whoever measures this library against the memory
 * system it runs on.  grass_probe_line_reads launches `blocks` workgroups of 256
 * threads; every thread reads one float from each of 16 pseudo-randomly chosen
 * 128-byte lines of src (src_floats floats, 128-byte aligned, expected to hold
 * zeros and to be far larger than the caches): the mask gather of Sec. 3.1
 * reduced to its memory traffic.
 *   mode 0  non-temporal reads only
 *   mode 1  and each value written to dst with coalesced non-temporal stores
 *           (dst_floats >= blocks * 256 * 16): 4 bytes written per line read,
 *           the ratio of grass_mask at the headline sizes
 *   mode 2  reads without the non-temporal hint
 *   mode 3  for comparison, a plain stream: every thread reads 16 x 16 bytes,
 *           workgroup after workgroup through src (blocks * 64 KB per launch)
 * Lines read per launch: blocks * 256 * 16 (mode 3: blocks * 512, every byte of
 * them).  dst needs one float in modes 0, 2, 3.                                 */
grass_status grass_probe_line_reads(const float* src, uint64_t src_floats, float* dst, uint64_t dst_floats,
                                    int mode, uint64_t salt, uint32_t blocks, grass_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* GRASS_H */
