/*
 * libsvdp — decode step of a ReGLU FFN gated by a low-rank SVD sparsity
 * predictor, for AMD MI355X (gfx950).  C ABI; every pointer named "device" is
 * a device pointer owned by the caller, the library never frees or keeps it.
 *
 * Notation follows the paper: d = hidden size, D = intermediate size,
 * r = predictor rank, x in R^d a decode token, W_gate, W_up in R^{D x d},
 * W_down in R^{d x D} (Sec. 3).  The predictor A B x + b of Sec. 4.1, eq. (2)
 * is passed in row-vector form: P = B^T (d x r), Q = A (D x r), so that the
 * scores are s = (x P) Q^T + b.
 *
 * Common rules for every call that takes a stream:
 *  - asynchronous on `stream` (a hipStream_t passed as void*, NULL = default
 *    stream); the call never synchronises (svdp_whiten_factors, an offline step,
 *    is the one exception and says so), never allocates device memory and
 *    never copies device data to the host, so it can be captured in a HIP graph;
 *  - arguments are validated on the host first; on any error nothing is
 *    enqueued and a status other than SVDP_OK is returned;
 *  - `ws` is a device scratch buffer of at least svdp_workspace_bytes() bytes,
 *    256-byte aligned, owned by the caller; its contents are undefined between
 *    calls; two calls that may overlap in time need distinct workspaces;
 *  - the library keeps no mutable state between calls: everything a call does
 *    follows from its arguments, so calls on different streams and from
 *    different host threads are independent (given distinct workspaces);
 *  - B is the number of tokens decoded together, 1 <= B <= SVDP_MAX_BATCH; all
 *    tokens of a batch share ONE mask (the union of their masks) and one index
 *    list, and every token is computed exactly over that list;
 *  - results are deterministic: floating-point sums are formed in a fixed
 *    order that depends only on the shapes and on the index list (no
 *    floating-point atomics, as in the paper's App. C down projection).
 *
 * Shape limits (else SVDP_ERR_UNSUPPORTED): D % 64 == 0, and with
 * e = 4 (fp32) or 8 (bf16) elements per 16 bytes: d % e == 0, r % e == 0,
 * r <= 2048, d <= 16384; the tokens of a batch must also fit the 160 KB of
 * local memory of a compute unit next to a kernel's scratch (B * d storage
 * elements; svdp_workspace_bytes returns 0 for a shape and batch that do not).
 * Every matrix pointer must be 16-byte aligned.
 */
#ifndef SVDP_H
#define SVDP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SVDP_MAX_BATCH 8

typedef enum {
    SVDP_OK = 0,
    SVDP_ERR_INVALID_ARG = 1,  /* null pointer, bad size, misaligned pointer   */
    SVDP_ERR_UNSUPPORTED = 2,  /* shape or dtype outside the limits above       */
    SVDP_ERR_WORKSPACE = 3,    /* ws is NULL, misaligned or too small           */
    SVDP_ERR_HIP = 4           /* the HIP runtime refused a launch              */
} svdp_status;

typedef enum {
    SVDP_F32 = 0,  /* IEEE binary32 */
    SVDP_BF16 = 1  /* bfloat16 bit patterns (upper 16 bits of a binary32) */
} svdp_dtype;

/* Flags of svdp_layer.flags */
enum {
    /* dReLU variant (paper Sec. 5.1, eq. 6): ReLU is applied to the up branch too. */
    SVDP_FLAG_DRELU = 1u,
    /* Sequential pipeline (paper Sec. 4.2, "Gate/up execution order"): the gate
     * product of a predicted-active neuron re-validates the prediction; when it is
     * <= 0 for every token of the batch, neither its W_up row nor its W_down row
     * is read.  The output is unchanged (such a neuron contributes exactly zero);
     * what changes is the bytes read: d*w per listed neuron for the gate, 2*d*w more
     * only for those that survive.  Pays when the predictor over-predicts (low rank,
     * cautious bias); costs one more dependent fetch per row otherwise.  A dedicated
     * row kernel runs (vector units).                                                */
    SVDP_FLAG_REVALIDATE = 2u,
    /* Which arithmetic units the batch-sensitive kernels use.  The paper's App. C gives a
     * row-at-a-time kernel (Alg. 3) and a gather-then-dense-contraction form (Alg. 4); its
     * Sec. 6 notes that batching lowers the sparsity the first can exploit.
     *  neither flag (default): per kernel and batch capacity, whichever was measured faster on
     *      MI355X: matrix cores for the scores from 3 tokens and for the rows from 5 tokens,
     *      vector units below.
     *  SVDP_FLAG_ENGINE_VECTOR: fp32 vector arithmetic everywhere (any dtype, batch, flags).
     *  SVDP_FLAG_ENGINE_MATRIX: matrix cores wherever a kernel for them exists:
     *      - rows (gate, up, down over the list): taken 16 at a time as MFMA tiles straight
     *        from their place in the weight matrices (no gathered copy), bf16 x bf16 -> fp32
     *        for gate and up, fp32 outer products for the down projection; needs bf16 storage,
     *        d a multiple of 512 and no SVDP_FLAG_REVALIDATE;
     *      - scores (t Q^T + b): bf16 MFMAs with t split into three bf16 terms (exact to fp32);
     *        needs bf16 storage, r a multiple of 32, r <= 512.
     *      Layers that do not qualify use the vector kernels.
     * Both engines give the same mask and list (up to scores within rounding of zero) and a y
     * that agrees to fp32 rounding (sums are cut differently).  Setting both is an error.     */
    SVDP_FLAG_ENGINE_VECTOR = 4u,
    SVDP_FLAG_ENGINE_MATRIX = 8u
};

/* One FFN layer with its predictor.  All pointers are device pointers.
 * Storage precision policy (paper App. C, "Precision"): weights, predictor
 * factors and tokens are stored in `wdtype`; all arithmetic, the rank-r
 * intermediate t = x P, the scores and y are fp32.                              */
typedef struct svdp_layer {
    int32_t d, D, r;
    int32_t wdtype;        /* svdp_dtype of P, Q, W_gate, W_up, W_downT and of x          */
    const void *P;         /* [d][r] row-major                                            */
    const void *Q;         /* [D][r] row-major                                            */
    const float *b;        /* [D] fp32 bias (= minus the calibrated threshold, Alg. 2)    */
    const void *W_gate;    /* [D][d] row-major: row i = neuron i                          */
    const void *W_up;      /* [D][d] row-major                                            */
    const void *W_downT;   /* [D][d] row-major: row i = column i of W_down (the paper's
                              column-major W_down, App. C "Memory")                       */
    uint32_t flags;        /* SVDP_FLAG_*                                                 */
} svdp_layer;

/* Bytes of device scratch any call below needs for this layer and up to
 * max_batch tokens.  Host-only, pure.  Returns 0 if the layer is unsupported.   */
size_t svdp_workspace_bytes(const svdp_layer *layer, int32_t max_batch);

/* Predictor scores (Sec. 4.1, eq. 2, before the step function; first line of
 * Alg. 3):  s[t][i] = sum_k (sum_j x[t][j] P[j][k]) Q[i][k] + b[i].
 * x: device [B][d] in layer->wdtype.  s: device [B][D] fp32, fully written.     */
svdp_status svdp_predict(const svdp_layer *layer, const void *x, int32_t B,
                         float *s, void *ws, size_t ws_bytes, void *stream);

/* Mask and index list (step function H of eq. 2; Alg. 4's nonzero):
 * neuron i is active iff s[t][i] > 0 (strictly; NaN is inactive) for at least
 * one token t < B.
 * s: device [B][D] fp32.  mask: device [D/64] 64-bit words, bit j of word k is
 * neuron 64k+j, fully written.  idx: device [D] int32, receives the active neurons
 * in ascending order in idx[0..nnz), the rest is left untouched.  nnz: device
 * [1] int32.  ws, ws_bytes: accepted for uniformity with the other calls; this
 * call needs no scratch, NULL and 0 are fine.                                   */
svdp_status svdp_compact(const float *s, int32_t B, int32_t D, uint64_t *mask,
                         int32_t *idx, int32_t *nnz, void *ws, size_t ws_bytes, void *stream);

/* Sparse ReGLU FFN over an index list (Sec. 3; Alg. 3's three kernels / Alg. 4):
 *   y[t][:] = sum_{n < nnz} ReLU(W_gate[i_n]·x[t]) * (W_up[i_n]·x[t]) * W_downT[i_n][:],
 * i_n = idx[n].  Only the listed rows of the three matrices are read.
 * idx: device int32, entries in [0, D), ascending not required but duplicates
 * are summed twice; an entry outside [0, D) is skipped on the device (it
 * contributes nothing and no row is read out of bounds).  nnz: device [1] int32,
 * clamped on the device to 0 <= *nnz <= D (never read on the host).  y: device [B][d] fp32, fully written (zeros
 * when *nnz == 0).                                                              */
svdp_status svdp_sparse_ffn(const svdp_layer *layer, const void *x, int32_t B,
                            const int32_t *idx, const int32_t *nnz, float *y,
                            void *ws, size_t ws_bytes, void *stream);

/* Dense ReGLU FFN (Sec. 3, eq. 1) over all D neurons: the same-GPU baseline
 * the sparse step is compared with.  y: device [B][d] fp32.                     */
svdp_status svdp_dense_ffn(const svdp_layer *layer, const void *x, int32_t B,
                           float *y, void *ws, size_t ws_bytes, void *stream);

/* The whole decode step of Alg. 3 for one batch: scores, union mask, index
 * list, sparse FFN.  Equivalent to svdp_predict + svdp_compact +
 * svdp_sparse_ffn without materialising the scores.
 * mask_out [D/64], idx_out [D], nnz_out [1]: device, each nullable; when given
 * they receive what svdp_compact would have produced.  y: device [B][d] fp32.   */
svdp_status svdp_ffn_step(const svdp_layer *layer, const void *x, int32_t B, float *y,
                          uint64_t *mask_out, int32_t *idx_out, int32_t *nnz_out,
                          void *ws, size_t ws_bytes, void *stream);

/* svdp_ffn_step for callers that cannot hand over or allocate scratch memory (code under HIP
 * graph capture that owns no buffer, tight serving loops, harnesses that forbid allocation):
 * the same step, with the scratch taken from an array of SVDP_STATIC_SCRATCH_BYTES that the
 * library's image holds on every GPU it runs on until the process ends.  Allocates nothing.
 * Layers and batches whose svdp_workspace_bytes() exceeds the array are refused with
 * SVDP_ERR_WORKSPACE (the 7B- and Mistral-shaped bf16 layers fit with one token).
 * All calls on one GPU share that GPU's array: two calls that may overlap in time on the same
 * GPU (different streams, different threads) race; serialise them or use svdp_ffn_step.
 * Nothing in the array needs to start at zero, and nothing is kept in it between calls.
 * Results are bit for bit those of svdp_ffn_step.                                              */
#define SVDP_STATIC_SCRATCH_BYTES (8u << 20)
svdp_status svdp_ffn_step_static(const svdp_layer *layer, const void *x, int32_t B, float *y,
                                 uint64_t *mask_out, int32_t *idx_out, int32_t *nnz_out, void *stream);

/* The sparse FFN of svdp_ffn_step from given mask words, without the predictor (Alg. 3 after its
 * first line): the row kernel scans the mask words, takes its share of the ascending list and
 * computes gate and up over the active rows; the down projection follows and y [B][d] is fully
 * written, bit for bit what svdp_ffn_step gives for the same mask.  With y == NULL everything but
 * the final sum of the partial results is enqueued (the row kernel; for batches on the matrix
 * cores the gate/up kernel and the down-projection kernel) and the partial results stay in the
 * workspace: that form exists so that the dominant kernels can be timed by themselves.
 * mask: device [D/64] words as written by svdp_compact or svdp_ffn_step.                        */
svdp_status svdp_active_rows(const svdp_layer *layer, const void *x, int32_t B, const uint64_t *mask,
                             float *y, void *ws, size_t ws_bytes, void *stream);

/* Glue between stacked layers used by the stacked benchmark (not from the
 * paper): v = x + y; x_next = v / sqrt(mean(v^2) + eps) + shift, rounded to
 * `dtype`.  x: device [d] in `dtype`; y: device [d] fp32; shift: device [d]
 * fp32; x_next: device [d] in `dtype` (may alias x).  d must be a multiple of 8
 * (bf16) or 4 (fp32), all four pointers 16-byte aligned.                       */
svdp_status svdp_stack_glue(const void *x, const float *y, const float *shift,
                            int32_t d, int32_t dtype, float eps, void *x_next,
                            void *stream);

/* ---- offline build: greedy bias calibration (Alg. 2; App. A "Greedy threshold selection") ----
 *
 * svdp_calib_bias runs Alg. 2 from its sort onward on given statistics of a calibration set:
 *   w [D][T] fp32  damage weights  |ReLU(W_gate[i,:] x_t) (W_up[i,:] x_t)|^2 ||W_down[:, i]||^2
 *   s [D][T] fp32  proxy scores    (A B x_t)_i  = the predictor's scores without bias
 * (row i = neuron i, column t = sample t; both device, read only; no NaN).
 * Per neuron the samples are sorted by score (equal scores keep sample order), the pointer starts at
 * the first positive weight (at T if there is none) with tau = the score there, and the greedy loop
 * advances the neuron whose next `eta` samples cost least (fp32 sum, left to right; smallest index
 * among equal costs; pointer update k <- min(k + eta, T)) until at least `need` of the D*T
 * (neuron, sample) pairs satisfy s <= tau, or no step is left.  For a sparsity level sp of Alg. 2,
 * need = the smallest integer >= sp*D*T.
 * Outputs (device): b [D] fp32 = -tau; k [D] int32 (nullable) the final pointers (counts, 1..T);
 * steps [1] int32 (nullable) the number of greedy steps taken; kendall [D] fp32 (nullable) App. A's
 * check 1 - K_d / (M (M-1)) of the eta-step sums' order, M = T / eta.
 * The result equals the sequential priority-queue loop exactly (integers and bit patterns).
 * Limits: 1 <= T <= 4096, eta >= 1, D >= 1; otherwise SVDP_ERR_UNSUPPORTED / SVDP_ERR_INVALID_ARG.
 * ws: device, 256-byte aligned, >= svdp_calib_workspace_bytes(D, T, eta) (0 for invalid sizes).
 * Asynchronous on `stream`, no allocation, no host read-back.                                     */
size_t svdp_calib_workspace_bytes(int32_t D, int32_t T, int32_t eta);

/* The integer `need` of svdp_calib_bias for a sparsity level sp of Alg. 2 ("while the sparsity is below
 * s"): the smallest integer n with n >= sp * D * T, the product taken in double precision from left to
 * right, clamped to [0, D * T].  Host-only, pure.  Returns -1 for D < 1, T < 1 or sp not a number.     */
int64_t svdp_calib_need(double sparsity, int32_t D, int32_t T);

/* The statistics svdp_calib_bias consumes, for T calibration tokens X [T][d] (device, in the
 * layer's storage type): w [D][T] and s [D][T] as defined above, with A B x evaluated the way
 * the runtime predictor does, (x P) Q^T in fp32 (the layer's bias b is not used).  Dense
 * contractions on the matrix cores.  bf16 storage only (SVDP_ERR_UNSUPPORTED otherwise).
 * ws: device, 256-byte aligned, >= svdp_calib_stats_workspace_bytes(layer, T).                     */
size_t svdp_calib_stats_workspace_bytes(const svdp_layer *layer, int32_t T);
svdp_status svdp_calib_stats(const svdp_layer *layer, const void *X, int32_t T, float *w, float *s,
                             void *ws, size_t ws_bytes, void *stream);
svdp_status svdp_calib_bias(const float *w, const float *s, int32_t D, int32_t T, int32_t eta, int64_t need,
                            float *b, int32_t *k, int32_t *steps, float *kendall,
                            void *ws, size_t ws_bytes, void *stream);

/* ---- offline build: predictor factors with data whitening (Sec. 4.1, Alg. 1) ----
 *
 * From the gate matrix W_gate [D][d] and T calibration tokens X [T][d] (both device, in `wdtype`):
 * with S any factor of the tokens' second moments, S S^T = X^T X, and U Sigma V^T the SVD of W_gate S,
 * the rank-r pair A = U_r Sigma_r, B = V_r^T S^-1 minimises ||(W_gate - A B) X^T||_F over rank-r products.
 * Outputs in the library's letters, fp32, device: Q = A [D][r], P = B^T [d][r], so that the predictor's
 * scores are (x P) Q^T; the caller rounds them to the layer's storage type.  sigma [r] (host, nullable):
 * the r leading singular values of W_gate S, descending.  sweeps [2] (host, nullable): sweeps[0] = 0,
 * sweeps[1] = block-Jacobi sweeps the eigen-decomposition took.
 * S is the lower Cholesky factor of X^T X, as Alg. 1 prints it (blocked factorisation, 64-wide blocks);
 * V and Sigma^2 come from the symmetric eigen-decomposition of (W_gate S)^T (W_gate S) by block Jacobi
 * sweeps, and S^-1 is applied to the r chosen vectors by block back-substitution.  All arithmetic is
 * fp64, the contractions on the matrix cores.
 * Needs d a multiple of 64, T >= d and X^T X positive definite to working precision (every pivot of
 * the factorisation above 1e-13 of the largest diagonal element), r <= d; otherwise
 * SVDP_ERR_UNSUPPORTED.
 * Unlike the decode calls this one is an offline step: it SYNCHRONISES `stream` several times (it reads
 * the factorisation's verdict, convergence figures and eigenvalues on the host) and cannot be captured in a graph.  It allocates
 * nothing on the device.  ws: device, 256-byte aligned, >= svdp_whiten_workspace_bytes(d, D, T, r)
 * (0 for sizes it does not take).                                                                      */
size_t svdp_whiten_workspace_bytes(int32_t d, int32_t D, int32_t T, int32_t r);
svdp_status svdp_whiten_factors(const void *W_gate, const void *X, int32_t d, int32_t D, int32_t T, int32_t r,
                                int32_t wdtype, float *P, float *Q, float *sigma, int32_t *sweeps,
                                void *ws, size_t ws_bytes, void *stream);

/* svdp_ffn_step with svdp_stack_glue in front of it, in the same launches: the step's token is
 * x = RMSNorm(x_prev + y_prev) + shift rounded to `wdtype` (bit for bit what svdp_stack_glue writes),
 * formed inside the step's first kernel, which saves the glue's own launch between stacked layers.
 * x_prev [B][d] in `wdtype`, y_prev [B][d] fp32, shift [d] fp32 (shared by the tokens): device, read;
 * x_out [B][d] in `wdtype`: device, receives x (must not alias x_prev or y_prev; the row kernel reads it).
 * The other arguments as in svdp_ffn_step; y may alias y_prev.                                     */
svdp_status svdp_ffn_step_glued(const svdp_layer *layer, const void *x_prev, const float *y_prev,
                                const float *shift, float eps, void *x_out, int32_t B, float *y,
                                uint64_t *mask_out, int32_t *idx_out, int32_t *nnz_out,
                                void *ws, size_t ws_bytes, void *stream);

/* Static string for a status code.  Never NULL. */
const char *svdp_status_string(svdp_status st);

/* Library version, "major.minor". */
const char *svdp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SVDP_H */
