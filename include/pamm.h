/*
 * libpamm: Point-Approximate Matrix Multiplication (PAMM) on one AMD MI355X (gfx950).
 *
 * The two calls follow the paper's statement of the method (Sec. 3.2): approximate
 * O = A^T B for A in R^{b x n}, B in R^{b x m} in two stages,
 *
 *   pamm_compress   first stage (compression of A): choose k generator rows C, and for every row A_i
 *                   the generator f(i) whose line gives the smallest projection residual
 *                   together with the coefficient alpha_i = <A_i,C_f(i)>/||C_f(i)||^2
 *                   (Eq. 1, Lemma 1; Alg. 1, procedure Compress, at eps = infinity);
 *   pamm_grad       second stage (the approximate product): Btilde_j = sum_{i: f(i)=j} alpha_i B_i,
 *                   O~ = C^T Btilde  (Alg. 1, procedure ApproxMM).
 *
 * In training, A is the saved input X of the fused Q|K|V projection, B is dY = [dQ|dK|dV]
 * and O~ is the approximate weight gradient (Alg. 2 and Alg. 3).
 *
 * Conventions that hold for every entry point
 *   - Matrices are row-major and contiguous.  X, C and dY share one element type
 *     (pamm_dtype); f is int32 and 0-based; alpha is fp32; dW is fp32, n x m
 *     (the orientation of O = A^T B), and is overwritten, not accumulated into.
 *   - Unless a parameter is marked "host", pointers are DEVICE pointers on the
 *     current HIP device, owned by the caller, 16-byte aligned.  The library never
 *     frees or retains them past the call's enqueued work.
 *   - Row lengths must keep every row 16-byte aligned: n and m multiples of 8 for
 *     PAMM_BF16, multiples of 4 for PAMM_F32 (otherwise PAMM_ERR_UNSUPPORTED).
 *   - b, n, m < 2^31; k <= min(b, 16384) (larger k: PAMM_ERR_UNSUPPORTED).
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL = default
 *     stream).  The calls do not synchronise the stream: outputs are valid once the
 *     stream has reached the end of the enqueued work.  Scratch memory comes from the
 *     caller through (ws, ws_bytes), sized by the *_workspace queries; the compute
 *     calls allocate nothing, take no lock and never block.  (Sampled indices travel in
 *     kernel argument blocks, 512 per launch, so a captured launch replays with the
 *     indices it was captured with.)
 *   - Errors are return codes.  All argument checks happen on the host before
 *     anything is enqueued; on a non-OK return nothing was enqueued and no output
 *     was touched, except PAMM_ERR_DEVICE (a HIP call failed part-way).
 *   - Calls that share a workspace must be ordered on one stream.
 */
#ifndef PAMM_H
#define PAMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PAMM_OK = 0,
    PAMM_ERR_INVALID_ARG = 1,   /* null pointer, size out of range, misaligned pointer */
    PAMM_ERR_UNSUPPORTED = 2,   /* unknown dtype, row length that breaks 16-byte row alignment */
    PAMM_ERR_WORKSPACE = 3,     /* ws is NULL or ws_bytes is below the matching *_workspace() */
    PAMM_ERR_DEVICE = 4         /* a HIP runtime call failed */
} pamm_status;

typedef enum { PAMM_F32 = 0, PAMM_BF16 = 1 } pamm_dtype;   /* element type of X, C and dY */

/* Orientation of the weight gradient written by pamm_grad_out. */
typedef enum {
    PAMM_DW_N_BY_M = 0,   /* n x m: O = A^T B as the paper writes it (Sec. 3.2); what pamm_grad writes */
    PAMM_DW_M_BY_N = 1    /* m x n: its transpose, for a weight stored as outputs x inputs */
} pamm_layout;

/* Human-readable name of a status code (static storage, never NULL). */
const char *pamm_status_string(pamm_status s);

/*
 * Bytes of device scratch pamm_compress / pamm_compress_idx need for these sizes
 * (0 if the sizes or dtype are invalid).  Host-only, pure.
 */
size_t pamm_compress_workspace(int64_t b, int64_t n, int64_t k, pamm_dtype dt);

/* Bytes of device scratch pamm_grad needs (0 if the sizes or dtype are invalid).  Host-only, pure. */
size_t pamm_grad_workspace(int64_t b, int64_t n, int64_t k, int64_t m, pamm_dtype dt);

/*
 * Alg. 1, Compress, sampling step: k distinct row numbers, every k-subset equally likely.
 * The paper fixes only the distribution; this library fixes the stream as: splitmix64
 * seeded with `seed`; draw t = 0..k-1 takes r = t + u where u is uniform on [0, b-t)
 * by rejection on the 64-bit output (reject x < 2^64 mod (b-t), u = x mod (b-t));
 * Fisher-Yates exchange of positions t and r of the identity arrangement of [0,b);
 * idx[t] is the value then at position t.  Generator j is draw j (draw order).
 * idx_host: HOST pointer to k int32, written by the call.  Pure host function.
 */
pamm_status pamm_sample_indices(int64_t b, int64_t k, uint64_t seed, int32_t *idx_host);

/*
 * Alg. 1, procedure Compress, with eps = infinity (no row dropped, beta = 1).
 *   X      in   b x n, dtype dt
 *   seed   in   selects the generators through pamm_sample_indices(b, k, seed)
 *   C      out  k x n, dtype dt: C_j = X[idx_j], bit copies                     (Alg. 1, generator rows)
 *   f      out  b int32: f(i) = lowest j maximising <X_i,C_j>^2/||C_j||^2       (Lemma 1: argmax |csim|)
 *   alpha  out  b fp32:  alpha_i = <X_i,C_f(i)>/||C_f(i)||^2                    (Eq. 1)
 * A generator with zero norm scores 0 and yields alpha 0; a zero row gets f = 0, alpha = 0.
 * Scores are accumulated in fp32; rows whose two best scores are within 2^-12 relative of
 * each other are re-decided in fp64, so f agrees with an fp64 evaluation except for
 * ties below fp64 resolution.
 */
pamm_status pamm_compress(const void *X, int64_t b, int64_t n, int64_t k, uint64_t seed, pamm_dtype dt,
                          void *C, int32_t *f, float *alpha,
                          void *ws, size_t ws_bytes, void *stream);

/*
 * The same with caller-chosen generators (Sec. 3.2 allows any set of representative rows;
 * also the hook tests use to bypass the sampler).
 *   idx_dev  in  DEVICE pointer to k int32 row numbers in [0,b); duplicates are allowed
 *                (the lowest j of identical generators wins).  Values outside [0,b) are
 *                clamped into range by the kernel rather than faulting.
 */
pamm_status pamm_compress_idx(const void *X, int64_t b, int64_t n, int64_t k, const int32_t *idx_dev,
                              pamm_dtype dt, void *C, int32_t *f, float *alpha,
                              void *ws, size_t ws_bytes, void *stream);

/*
 * Alg. 1, procedure Compress, with a finite tolerance eps >= 0: the neighbourhood condition of Eq. 2,
 *   ||X_i - alpha_i C_f(i)||_2 <= eps ||X_i||_2,
 * is applied to the representative of every row; a row that fails it is dropped, i.e. its alpha is set to 0 (its
 * f stays: Alg. 1 only zeroes alpha).  Eq. 2 (relative to ||X_i||) is taken where Alg. 1 prints the absolute e > eps.
 * eps = 0 keeps only rows lying exactly on a generator's line: uniform column-row sampling (Sec. 4.1).
 * eps >= 1 (or +infinity) can drop nothing and is the same as pamm_compress.  Negative or NaN: PAMM_ERR_INVALID_ARG.
 *   eta    out  DEVICE pointer to one int32 (4-byte aligned): the number of rows dropped.  The normalisation factor
 *               of Sec. 3.2 is beta = b / (b - eta); pamm_grad_eps applies it.
 * All other arguments as pamm_compress / pamm_compress_idx.  The test is taken in fp32 (||X_i||^2 comes from the
 * same pass over X, on the matrix cores) except for rows within 2^-11 ||X_i||^2 of the limit, which are decided in
 * fp64 like the near-ties of f.
 */
pamm_status pamm_compress_eps(const void *X, int64_t b, int64_t n, int64_t k, uint64_t seed, float eps, pamm_dtype dt,
                              void *C, int32_t *f, float *alpha, int32_t *eta,
                              void *ws, size_t ws_bytes, void *stream);
pamm_status pamm_compress_idx_eps(const void *X, int64_t b, int64_t n, int64_t k, const int32_t *idx_dev, float eps,
                                  pamm_dtype dt, void *C, int32_t *f, float *alpha, int32_t *eta,
                                  void *ws, size_t ws_bytes, void *stream);

/*
 * Alg. 1, procedure ApproxMM: dW = C^T Btilde with Btilde_j = sum_{i: f(i)=j} alpha_i dY_i.
 *   C      in   k x n, dtype dt          f      in  b int32 in [0,k)        alpha  in  b fp32
 *   dY     in   b x m, dtype dt
 *   dW     out  n x m fp32, overwritten
 * Rows are grouped by f with a stable counting sort (rows of one generator stay in increasing
 * order) and summed in fp32 in that order, so the result is bit-reproducible from call to call.  Rows with alpha_i = 0 add nothing and are
 * left out: their rows of dY are never read.  For PAMM_BF16 the contracted rows are
 * rounded to bf16 once before the C^T Btilde product (fp32 accumulation); for PAMM_F32 the
 * product is carried out in fp32 throughout.  Entries of f outside [0,k) are clamped into
 * range by the kernels rather than faulting.
 */
pamm_status pamm_grad(const void *C, const int32_t *f, const float *alpha, const void *dY,
                      int64_t b, int64_t n, int64_t k, int64_t m, pamm_dtype dt,
                      float *dW, void *ws, size_t ws_bytes, void *stream);

/*
 * ApproxMM with the normalisation factor of Sec. 3.2: dW = beta C^T Btilde, beta = b / (b - eta) (0 if eta = b), so
 * that the dropped rows do not bias the estimate.
 *   eta    in   DEVICE pointer to one int32, as written by pamm_compress_eps on the same stream or earlier
 * All other arguments as pamm_grad.
 */
pamm_status pamm_grad_eps(const void *C, const int32_t *f, const float *alpha, const int32_t *eta, const void *dY,
                          int64_t b, int64_t n, int64_t k, int64_t m, pamm_dtype dt,
                          float *dW, void *ws, size_t ws_bytes, void *stream);

/*
 * ApproxMM (Alg. 1) with a choice of element type and orientation for the weight gradient that the backward pass
 * of the linear layer (Alg. 3) hands on, for callers that store the weight as outputs x inputs or keep its gradient
 * in bf16.
 *   eta     in   as pamm_grad_eps, or NULL for beta = 1 (then the call computes what pamm_grad computes)
 *   out_dt       PAMM_F32, or PAMM_BF16: every element is the fp32 result rounded once, to nearest even
 *   layout       PAMM_DW_N_BY_M (n x m) or PAMM_DW_M_BY_N (m x n); the values are the same, element for element
 *   dW      out  n*m elements of out_dt in that orientation, overwritten
 * PAMM_BF16 output needs an even row length of dW (PAMM_ERR_UNSUPPORTED otherwise; always true for PAMM_BF16
 * inputs).  All other arguments, the workspace and the summation order as pamm_grad.
 */
pamm_status pamm_grad_out(const void *C, const int32_t *f, const float *alpha, const int32_t *eta, const void *dY,
                          int64_t b, int64_t n, int64_t k, int64_t m, pamm_dtype dt,
                          pamm_dtype out_dt, pamm_layout layout, void *dW,
                          void *ws, size_t ws_bytes, void *stream);

/*
 * pamm_grad for callers that cannot allocate device memory, not even a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Computes exactly what pamm_grad computes (same kernels,
 * same summation order, bit-identical dW), with the scratch memory taken from a device array of
 * PAMM_STATIC_SCRATCH_BYTES that is part of the library's image: every GPU the library runs on holds its copy until
 * the process ends.  The call allocates nothing and frees nothing.
 *   - Sizes whose pamm_grad_workspace() exceeds PAMM_STATIC_SCRATCH_BYTES are refused with PAMM_ERR_WORKSPACE before
 *     anything is enqueued (the 1B-shaped layer, b = 65536, n = 2048, m = 6144, k = 128, bf16, needs about 13 MiB).
 *   - All calls on one GPU share that GPU's array, which keeps the last call's contents; no part of it has to be
 *     cleared between calls.  Calls that overlap on one GPU (different streams, or different threads without
 *     ordering) race on it: order them on one stream.
 *   - The array's device address is looked up on the first call on each device; make that first call outside
 *     stream capture.
 * Arguments as pamm_grad, without (ws, ws_bytes).
 */
#define PAMM_STATIC_SCRATCH_BYTES (16u << 20)
pamm_status pamm_grad_static(const void *C, const int32_t *f, const float *alpha, const void *dY,
                             int64_t b, int64_t n, int64_t k, int64_t m, pamm_dtype dt,
                             float *dW, void *stream);

/*
 * Test/benchmark hook: only the contraction stage of ApproxMM.
 *   Btilde out  k x m fp32: Btilde_j = sum_{i: f(i)=j} alpha_i dY_i          (Sec. 3.2, second displayed sum)
 * Same workspace as pamm_grad.
 */
pamm_status pamm_contract(const int32_t *f, const float *alpha, const void *dY,
                          int64_t b, int64_t k, int64_t m, pamm_dtype dt,
                          float *Btilde, void *ws, size_t ws_bytes, void *stream);

/*
 * The random-projection baseline of the ablation (Sec. 4.6, the comparison with a low-rank sketch of the activation):
 * instead of (C, f, alpha) the layer keeps S = X P, with P an n x r random matrix with E[P P^T] = I, and estimates
 * the weight gradient as P (S^T dY).  On the same harness as the calls above, for comparisons at equal memory
 * (the sketch holds b r numbers, PAMM's compression k n + 2 b).  The random numbers are the caller's: P is passed
 * through its transpose Pt (r x n, row-major, element type dt), row j being the j-th direction of the sketch.
 *
 *   pamm_sketch        S (b x r, element type dt) = X Pt^T, fp32 accumulation, rounded once to dt.  No workspace.
 *   pamm_sketch_grad   dW (n x m fp32) = Pt^T G, G = S^T dY (r x m): G is accumulated in fp32 over chunks of tokens on
 *                      the matrix cores while dY streams once, rounded once to dt, and multiplied by the kernels of
 *                      pamm_grad's last step.
 * r is a multiple of 8 (of 4 for PAMM_F32), r <= min(b, 128); other sizes as above.
 */
size_t pamm_sketch_grad_workspace(int64_t b, int64_t n, int64_t r, int64_t m, pamm_dtype dt);
pamm_status pamm_sketch(const void *X, const void *Pt, int64_t b, int64_t n, int64_t r, pamm_dtype dt,
                        void *S, void *stream);
pamm_status pamm_sketch_grad(const void *Pt, const void *S, const void *dY,
                             int64_t b, int64_t n, int64_t r, int64_t m, pamm_dtype dt,
                             float *dW, void *ws, size_t ws_bytes, void *stream);

/*
 * Per-kernel timing for benchmarks (the paper reports its own cost per operation in App. F, Tables 6-7).
 * Between pamm_profile_begin() and pamm_profile_end() every kernel the library launches is bracketed by
 * a pair of HIP events on its launch stream (events are created per launch: not for use on a hot path).
 * pamm_profile_end waits for those events and returns, per kernel id in [0, PAMM_NUM_KERNELS), the summed
 * elapsed milliseconds and the number of launches; both arrays are HOST pointers of PAMM_NUM_KERNELS
 * entries.  pamm_kernel_name gives the name of a kernel id ("" if out of range).  Process-wide state.
 */
#define PAMM_NUM_KERNELS 10
pamm_status pamm_profile_begin(void);
pamm_status pamm_profile_end(double *ms_total, int64_t *launches);
const char *pamm_kernel_name(int id);

/*
 * Test hooks (host-only, process-wide, not thread-safe; no product call needs them).
 *
 * pamm_debug_set_plan overrides the launch heuristics of the calls above so that tests can run the kernel variants
 * and grid decompositions the heuristics do not pick at small shapes; a field that is 0 or out of its range leaves
 * the heuristic in charge, NULL clears every override.  The overrides also enter the *_workspace queries, so query
 * the workspace after setting them.
 *   score_tg       32-generator fragments per wave of the score kernel: 1, 2, 4 or 8 (at most what k allows)
 *   score_nw       waves per workgroup of the score kernel: 2, 4 or 8
 *   piece_rows     positions of the sorted list per chunk of the contraction: a multiple of 16 in [16, 4096]
 *   contract_w     512-column groups per wave of the contraction: 1, 2 or 3
 *   sort_one_rows  largest b grouped by the single-workgroup counting sort: 1..16384
 *   small_tiles    the big-tile kernel that C^T Btilde takes at large shapes with at least 512 generators:
 *                  1: not used; 2: used with 256 x 256 tiles (one workgroup per compute unit) instead of 256 x 128 (two)
 *
 * pamm_debug_bounded writes `count` consecutive draws of the sampler's bounded step (uniform on [0, range) by
 * rejection, as specified at pamm_sample_indices) from one generator seeded with `seed` into out_host, so that a
 * test can drive the rejection branch with ranges near 2^63, which the sampler itself (range < 2^31) takes with
 * probability below 2^-33.  range = 0 or out_host = NULL: PAMM_ERR_INVALID_ARG.
 */
typedef struct {
    int score_tg, score_nw, piece_rows, contract_w, sort_one_rows, small_tiles;
} pamm_debug_plan;
pamm_status pamm_debug_set_plan(const pamm_debug_plan *plan_host);
pamm_status pamm_debug_bounded(uint64_t seed, uint64_t range, int64_t count, uint64_t *out_host);

#ifdef __cplusplus
}
#endif
#endif /* PAMM_H */
