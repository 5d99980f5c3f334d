/*
 * llla.h -- C ABI of the MI355X (gfx950) Local Linear Attention library.
 *
 * Local Linear Attention (arxiv 2510.01450, Section 2.3): for every query q_i, fit
 * f(x) = b + W (x - q_i) to the visible key/value pairs (k_j, v_j) by weighted ridge least squares
 * (objective Eq. (lla_obj)) and return the intercept b as the output o_i.  In the paper's symbols
 * (Eq. (query_specific), Eq. (lla)):
 *
 *     w_ij   = exp(scale * <q_i, k_j> - m_i),   m_i = max over visible j of scale * <q_i, k_j>
 *     z_ij   = k_j - q_i
 *     omega_i = sum_j w_ij,  mu_i = sum_j w_ij z_ij,  Sigma_i = sum_j w_ij z_ij z_ij^T + lambda I
 *     rho_i  = Sigma_i^{-1} mu_i,   delta_i = omega_i - mu_i . rho_i
 *     o_i    = sum_j w_ij (1 - z_ij . rho_i) / delta_i * v_j
 *
 * Conventions of this library where the paper leaves a choice:
 *   - the kernel is the dot-product exponential of the matrix form and Algorithm 1 (Section 3.2),
 *     scale = 1/h;  the paper's default bandwidth corresponds to scale = 1/sqrt(d);
 *   - lambda is added to moments of the row-max-normalised weights above (largest weight of a row
 *     is exactly 1), which is what Algorithm 1 computes after its last key block; outputs are
 *     therefore invariant to adding a constant to all logits of a row;
 *   - "+ lambda I" exactly as in Eq. (query_specific); the intercept is not penalised;
 *   - causal means j <= i, inclusive (the tril mask of Section 3.2);
 *   - the per-query system is solved exactly (on-chip factorisation), not by a fixed number of
 *     conjugate-gradient iterations (Appendix C is the paper's approximate alternative).
 *
 * Memory and execution contract (all entry points):
 *   - every data pointer is a DEVICE pointer owned by the caller; the library never allocates or
 *     frees device memory, never synchronises the device, keeps no state between calls (it is
 *     thread-safe), and enqueues all work on `stream` (a hipStream_t passed as void*; NULL = the
 *     default stream);
 *   - tensors are [batch, head, seq, d] with the innermost (d) stride equal to 1; the other strides
 *     are given in elements in an llla_strides;
 *   - inputs are never modified, outputs are fully overwritten, results are deterministic;
 *   - arguments are validated on the host before anything is enqueued; on error nothing has been
 *     launched and the outputs are untouched (LLLA_ERR_LAUNCH excepted);
 *   - `workspace` is scratch of at least the size the matching *_workspace_bytes() call returns
 *     (256-byte aligned); it holds Theta(B*H*n*d) data only -- no per-query d x d matrix and no
 *     n x n matrix is ever written to device memory.  Calls that share a workspace must be
 *     ordered on one stream.
 *
 * Value range of the matrix-core kernels.  LLLA_PATH_AUTO serves bf16 inputs with d = 64 or 128 on
 * the matrix cores (llla_forward, llla_forward_ex, llla_forward_cg, llla_backward, and llla_decode
 * with a cache capacity of at least 256 rows; llla_forward and llla_forward_ex also d = 16 and 32 from 32 rows on).  Those kernels hand the keys (and, in decode, queries and
 * values) to the MFMA units as f16: every |x| must be at most 65504 (larger ones become
 * infinite and the rows whose 64-key blocks hold them NaN; no status is returned, the data being device memory), and
 * magnitudes below 6.1e-5 lose bits to the f16 subnormal range.  bf16 values of ordinary size
 * (8 significant bits, |x| in [6.1e-5, 65504]) convert exactly.  LLLA_PATH_VALU computes in fp32
 * throughout and has no such limit (what it can carry is bounded by the conditioning of the rows' systems in fp32).
 */
#ifndef LLLA_H
#define LLLA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LLLA_OK = 0,
    LLLA_ERR_NULL = 1,        /* a required pointer is NULL */
    LLLA_ERR_SHAPE = 2,       /* B, H, n, L or d <= 0, or a stride too small for the shape */
    LLLA_ERR_DTYPE = 3,       /* unknown llla_dtype */
    LLLA_ERR_PARAM = 4,       /* lambda <= 0 or not finite, scale not finite */
    LLLA_ERR_ALIGN = 5,       /* base pointer or stride not 16-byte compatible */
    LLLA_ERR_WORKSPACE = 6,   /* workspace NULL/unaligned or smaller than *_workspace_bytes() */
    LLLA_ERR_UNSUPPORTED = 7, /* d not in {16, 32, 64, 128}, or a path forced that does not serve the call */
    LLLA_ERR_LAUNCH = 8       /* the HIP runtime refused a launch */
} llla_status;

typedef enum { LLLA_F32 = 0, LLLA_BF16 = 1 } llla_dtype;

/* Element strides of a [batch, head, seq, d] tensor; the d stride is 1 by contract.
 * Each must be a multiple of 4 (f32) or 8 (bf16) elements so that rows stay 16-byte aligned. */
typedef struct {
    int64_t batch;
    int64_t head;
    int64_t seq;
} llla_strides;

/* Which kernels a forward call uses.  AUTO picks the MFMA path when it exists for (dtype, d) and
 * the portable vector-ALU path otherwise; the other two force one (for tests and measurement). */
typedef enum { LLLA_PATH_AUTO = 0, LLLA_PATH_VALU = 1, LLLA_PATH_MFMA = 2 } llla_path;

/*
 * llla_forward -- Section 3.2 (matrix form and Algorithm 1): O = LLA(Q, K, V; lambda, h) for all
 * n query rows of every (batch, head).
 *   Q, K, V : device, [B, H, n, d] in dtype `in`, strides sq / sk / sv
 *   O       : device, [B, H, n, d] in dtype `out`, strides so
 *   causal  : 1 = row i sees keys 0..i (the paper's tril mask); 0 = every row sees all n keys
 *   lambda  : ridge, > 0 (Sigma_i has rank <= i without it, Appendix C)
 *   scale   : 1/h
 *   Returns LLLA_OK or the first failed check.
 */
size_t llla_forward_workspace_bytes(int B, int H, int n, int d, llla_dtype in);

llla_status llla_forward(const void *Q, const void *K, const void *V, void *O,
                         llla_strides sq, llla_strides sk, llla_strides sv, llla_strides so,
                         int B, int H, int n, int d, llla_dtype in, llla_dtype out,
                         int causal, float lambda, float scale,
                         void *workspace, size_t workspace_bytes, void *stream);

/* Same as llla_forward with the kernel family chosen by the caller.  LLLA_PATH_MFMA: bf16 inputs with d = 64 or 128,
 * fp32 inputs with d = 64, and -- for either dtype -- d = 16 and 32, which run the d = 64 kernels on zero-padded
 * copies held in the workspace (exact: with features d..63 zero the system of Eq. (query_specific) splits into the
 * original one and lambda * y = 0); other calls return LLLA_ERR_UNSUPPORTED.  LLLA_PATH_AUTO takes the matrix-core
 * kernels wherever they exist, except where the vector kernels measured faster: d = 16 with fp32 inputs, d = 32 with
 * fp32 inputs and fewer than 1024 rows, and bf16 inputs with d = 16 / 32 and fewer than 32 rows.  bf16 inputs on the matrix cores are subject to the f16 value
 * range stated at the top of this file. */
llla_status llla_forward_path(const void *Q, const void *K, const void *V, void *O,
                              llla_strides sq, llla_strides sk, llla_strides sv, llla_strides so,
                              int B, int H, int n, int d, llla_dtype in, llla_dtype out,
                              int causal, float lambda, float scale, llla_path path,
                              void *workspace, size_t workspace_bytes, void *stream);

/*
 * llla_forward_ex -- llla_forward_path with the two quantities the paper attaches to the forward pass:
 *   lambda_rows : device float [B, H, n] contiguous, or NULL.  Appendix C makes the ridge a learnable,
 *                 position-dependent quantity: row i then uses lambda_rows[b, h, i] in Eq. (query_specific)
 *                 and `lambda` is ignored.  Every entry must be finite and > 0;
 *                 being device memory they are not checked.
 *   rho, delta  : device float [B, H, n, d] and [B, H, n] contiguous, or NULL each.  rho_i = Sigma_i^{-1} mu_i
 *                 and delta_i = omega_i - mu_i . rho_i of Eq. (lla), the per-row statistics FlashLLA keeps
 *                 for its backward pass (end of Section 3.2), relative to the same max-normalised weights
 *                 as everything else here; written in fp32.
 * Everything else as llla_forward_path.
 */
llla_status llla_forward_ex(const void *Q, const void *K, const void *V, void *O,
                            llla_strides sq, llla_strides sk, llla_strides sv, llla_strides so,
                            int B, int H, int n, int d, llla_dtype in, llla_dtype out,
                            int causal, float lambda, const float *lambda_rows, float scale,
                            float *rho, float *delta, llla_path path,
                            void *workspace, size_t workspace_bytes, void *stream);

/*
 * llla_forward_cg -- the paper's approximate forward (Section 3.1 "matrix-free inversion via conjugate gradients",
 * solver of Appendix C): rho_i is the iterate after at most `max_steps` conjugate-gradient steps on
 * Sigma_i rho = mu_i, started at 0, with Sigma_i applied matrix-free; delta_i and the output follow from Eq. (lla)
 * with that rho_i.  A row whose residual norm ||mu_i - Sigma_i rho|| is at or below `eps` when a step starts takes
 * no further steps (the paper's active mask); eps = 0 runs max_steps steps unless the residual becomes exactly 0.
 * max_steps = 0 gives softmax attention (rho = 0).  Causal; bf16 inputs only (LLLA_ERR_UNSUPPORTED otherwise); d = 16
 * and 32 run at d = 64 on zero-padded copies, whose padded entries stay zero in every iterate.  0 <= max_steps <= 4096, eps >= 0.
 *   rho, delta : optional outputs as in llla_forward_ex;  steps: optional device int32 [B, H, n], steps taken per row.
 * Workspace: llla_forward_cg_workspace_bytes (larger than the exact forward's: the CG vectors of every row).
 */
size_t llla_forward_cg_workspace_bytes(int B, int H, int n, int d, llla_dtype in);

llla_status llla_forward_cg(const void *Q, const void *K, const void *V, void *O,
                            llla_strides sq, llla_strides sk, llla_strides sv, llla_strides so,
                            int B, int H, int n, int d, llla_dtype in, llla_dtype out,
                            float lambda, float scale, int max_steps, float eps,
                            float *rho, float *delta, int32_t *steps,
                            void *workspace, size_t workspace_bytes, void *stream);

/*
 * llla_backward -- Appendix D (backward derivation): the gradients of L = sum_i dO_i . o_i, o = the causal
 * llla_forward_ex output, with respect to Q, K, V and the ridge of every row.  As in Appendix D the work per row is
 * one more linear solve with the row's matrix (the paper's u_i) plus matrix products of the size of the forward's;
 * the value gradient is S^T dO with S the output weights of Eq. (lla).  The forward here applies the ridge to
 * max-normalised weights, so the output depends on the row maximum m_i; that dependence is differentiated too
 * (it equals lambda_i dL/dlambda_i and flows into the logit of the key that attains the maximum; with several keys
 * at the maximum, the first).  Nothing is kept from the forward call: the row statistics are recomputed.
 *   Q, K, V, dO : device, [B, H, n, d] in dtype `in`, strides sq / sk / sv / sdo
 *   dQ, dK, dV  : device float [B, H, n, d] contiguous, 16-byte aligned, fully overwritten
 *   dlambda     : device float [B, H, n] contiguous or NULL; dL/dlambda_i of every row (sum them for a scalar ridge)
 *   lambda, lambda_rows, scale : as in llla_forward_ex
 *   path        : LLLA_PATH_AUTO / VALU / MFMA as in llla_forward_path.  The vector path serves every supported d and
 *                 both dtypes in fp32 arithmetic.  The matrix-core path (bf16, d = 64 or 128) recomputes the row
 *                 moments and does both solves of a row with the forward's matrix-core kernel; the O(d)-per-pair
 *                 sweeps around it run in fp32 on the vector ALU.  bf16 inputs with d = 16 or 32 run it at d = 64 on
 *                 zero-padded copies, as the forward does (the gradient of a padded feature is zero and is dropped);
 *                 LLLA_PATH_AUTO takes that route for d = 32 from 64 rows on, and for d = 16 from 512 rows on.
 * Causal only.  Workspace: llla_backward_workspace_bytes (Theta(B H n d); enough for either path).
 */
size_t llla_backward_workspace_bytes(int B, int H, int n, int d, llla_dtype in);

llla_status llla_backward(const void *Q, const void *K, const void *V, const void *dO,
                          llla_strides sq, llla_strides sk, llla_strides sv, llla_strides sdo,
                          float *dQ, float *dK, float *dV, float *dlambda,
                          int B, int H, int n, int d, llla_dtype in,
                          float lambda, const float *lambda_rows, float scale, llla_path path,
                          void *workspace, size_t workspace_bytes, void *stream);

/*
 * llla_decode -- the inference step the paper mentions (Sections 1 and 2.3: LLA keeps a Theta(n d)
 * KV cache): one new query per (batch, head) against the cached keys and values, the new token's
 * own (k, v) already appended, i.e. the last row of a causal forward over seqlens[b] positions.
 *   q       : device, [B, H, d] contiguous, dtype `in`
 *   Kc, Vc  : device, [B, H, L_max, d] caches in dtype `in`, strides sk / sv
 *   o       : device, [B, H, d] contiguous, dtype `out`
 *   seqlens : device int32 [B], valid length of each sequence (1..L_max), or NULL = all L_max;
 *             cache rows at and beyond a sequence's length are never read
 */
size_t llla_decode_workspace_bytes(int B, int H, int L_max, int d, llla_dtype in);

llla_status llla_decode(const void *q, const void *Kc, const void *Vc, void *o,
                        llla_strides sk, llla_strides sv, const int32_t *seqlens,
                        int B, int H, int L_max, int d, llla_dtype in, llla_dtype out,
                        float lambda, float scale,
                        void *workspace, size_t workspace_bytes, void *stream);

/* Same as llla_decode with the kernel family chosen by the caller.  The matrix-core kernels serve bf16 caches with
 * d = 64 or 128, L_max >= 256 and B * H <= 65535 (queries, keys and values must lie in the f16 range, |x| <= 65504);
 * LLLA_PATH_MFMA on any other call returns LLLA_ERR_UNSUPPORTED, LLLA_PATH_AUTO takes the vector kernels there. */
llla_status llla_decode_path(const void *q, const void *Kc, const void *Vc, void *o,
                             llla_strides sk, llla_strides sv, const int32_t *seqlens,
                             int B, int H, int L_max, int d, llla_dtype in, llla_dtype out,
                             float lambda, float scale, llla_path path,
                             void *workspace, size_t workspace_bytes, void *stream);

/*
 * llla_decode_static -- llla_decode for callers that cannot allocate device memory and therefore have no workspace
 * to pass: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * kernels and bit-identical results; the partial-moment records that llla_decode keeps in `workspace` live in a
 * device array of LLLA_STATIC_SCRATCH_BYTES inside the library instead (one copy per GPU, held from the moment the
 * library is loaded on that GPU until the process ends).  The call allocates and frees nothing and does not
 * synchronise.  A call whose llla_decode_workspace_bytes() exceeds LLLA_STATIC_SCRATCH_BYTES returns
 * LLLA_ERR_WORKSPACE (the decode configuration of 32 x 16 heads x 32768 keys at d = 64 needs 56 MB and fits);
 * LLLA_ERR_LAUNCH if the runtime cannot report the array's address.  Every call on a GPU uses that GPU's one array:
 * calls on the same stream are ordered and safe, calls that overlap on one GPU (different streams, different
 * threads) race on it -- unlike every other entry point, this one is not re-entrant per device.
 */
#define LLLA_STATIC_SCRATCH_BYTES ((size_t)64 << 20)

llla_status llla_decode_static(const void *q, const void *Kc, const void *Vc, void *o,
                               llla_strides sk, llla_strides sv, const int32_t *seqlens,
                               int B, int H, int L_max, int d, llla_dtype in, llla_dtype out,
                               float lambda, float scale, void *stream);

/* Static, NUL-terminated description of a status code. */
const char *llla_status_string(llla_status status);

/* Library version, "major.minor.patch". */
const char *llla_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LLLA_H */
