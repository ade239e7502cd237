/*
 * probsparse.h -- C ABI of the MI355X (gfx950) prob-sparse self-attention forward.
 *
 * The operation is Sec. 3.2 of arXiv 2106.09236 ("Efficient Conformer with
 * Prob-Sparse Attention Mechanism for End-to-End Speech Recognition"): per
 * (batch, head)
 *   a1. score every query against its sampled keys and form the sampled
 *       sparsity measure  M_i = max_t s_it - mean_t s_it,  s = q.k/sqrt(d)   (Eq. 11)
 *   a2. keep the u queries with the largest M (I_sparse; ties to the lower index)
 *   a3. softmax attention over all valid keys for the kept queries        (Eq. 7, 8, 12)
 *   a4. every other valid query row receives the mean of the valid value rows
 *       (Sec. 3.1: uniform scores give the plain average of the values);
 *       rows at or beyond the item's length receive zeros.
 * u = ceil(c * ln(len_b)) clamped to [1, len_b] for batch item b.
 *
 * Conventions for every entry point
 *   - All tensor arguments are DEVICE pointers, 16-byte aligned, row-major and
 *     contiguous with the last dimension fastest.  `shape` is a HOST pointer.
 *   - The library allocates nothing, frees nothing and never synchronises (the only state it
 *     keeps is per device: which kernels have had their dynamic-LDS limit raised, and the
 *     address of the static scratch of probsparse_attn_fwd_static): all
 *     work is enqueued on `stream` (a hipStream_t; NULL = the default stream).
 *     The caller owns every buffer and must keep it alive until the stream has
 *     drained.  `out` and `workspace` must not alias any input.
 *   - Return value: 0 (PSA_OK) or a negative psa_status_t.  All argument checks
 *     run before the first launch, so a failed call has enqueued nothing
 *     (except PSA_ERR_HIP, which reports a launch error from the runtime).
 *   - Device-side preconditions, not checked on the host: 0 <= lengths[b] <= L_K
 *     (values outside are clamped), and 0 <= sample_idx < lengths[b].  A sample
 *     index outside [0, lengths[b]) is never dereferenced: it is dropped from
 *     the max and the mean.  A query left with no usable sample has M = 0.
 */
#ifndef PROBSPARSE_H
#define PROBSPARSE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum psa_dtype {
    PSA_F32  = 0,   /* Q, K, V, out are IEEE binary32                                   */
    PSA_BF16 = 1    /* Q, K, V, out are bfloat16; all accumulation is binary32 or wider */
} psa_dtype_t;

typedef enum psa_status {
    PSA_OK            =  0,
    PSA_ERR_NULL      = -1,   /* a required pointer is NULL                              */
    PSA_ERR_SHAPE     = -2,   /* non-positive dim, D != 64, L_Q != L_K, U < 1, too large */
    PSA_ERR_DTYPE     = -3,   /* dtype is not a psa_dtype_t                              */
    PSA_ERR_ARG       = -4,   /* factor not finite and positive; bad mask, rule, fill, u_stride */
    PSA_ERR_WORKSPACE = -5,   /* workspace_bytes < probsparse_attn_workspace_bytes()     */
    PSA_ERR_HIP       = -6,   /* the HIP runtime refused a launch or a copy              */
    PSA_ERR_ALIGN     = -7    /* a device pointer is not 16-byte aligned                 */
} psa_status_t;

/* Problem shape.  Self-attention only (Sec. 3.1: Q, K, V are projections of the
 * same L frames), so L_Q must equal L_K.  D is the per-head dimension and must
 * be 64 (256 model dims over 4 heads, Sec. 4.2).  U is the number of sampled
 * keys per query, i.e. the last dimension of sample_idx. */
typedef struct psa_shape {
    int32_t B, H, L_Q, L_K, D, U;
    int32_t dtype;            /* psa_dtype_t */
} psa_shape_t;

/* How many queries of an item with len_b valid frames are kept in step a2.
 *   PSA_U_LOG    u_b = clamp(ceil(factor * ln len_b), 1, len_b): the rule of the
 *                Informer work the paper builds on (Sec. 1, Sec. 3.2), factor = c
 *   PSA_U_RATIO  u_b = clamp(ceil(factor * len_b), 1, len_b): the paper's own
 *                L_sparse = r_sparse * L (Sec. 3.2; r_sparse = 0.5 in Sec. 4.2) */
typedef enum psa_u_rule {
    PSA_U_LOG   = 0,
    PSA_U_RATIO = 1
} psa_u_rule_t;

/* What a valid query outside I_sparse receives in step a4.
 *   PSA_FILL_MEAN   the mean of the item's valid value rows (Sec. 3.1)
 *   PSA_FILL_VALUE  its own value row v_i (Eq. 12, lower branch, as printed) */
typedef enum psa_fill {
    PSA_FILL_MEAN  = 0,
    PSA_FILL_VALUE = 1
} psa_fill_t;

typedef struct psa_options {
    int32_t u_rule;           /* psa_u_rule_t */
    int32_t fill;             /* psa_fill_t */
    double  factor;           /* c (PSA_U_LOG) or r_sparse (PSA_U_RATIO); finite, > 0 */
} psa_options_t;

/* Pipeline stages, for probsparse_attn_fwd_stages().
 *   MEASURE  a1, plus float64 column sums of the valid V rows (for a4)
 *   SELECT   a2 as a kernel of its own; only launched for heads whose K does not
 *            fit the measure kernel's LDS (more than 512 frames in float32, 1024
 *            in bfloat16); shorter heads select inside ATTEND and the bit is a no-op
 *   ATTEND   a2 (short heads), a3 and a4: writes every row of `out` */
enum {
    PSA_STAGE_MEASURE = 1,
    PSA_STAGE_SELECT  = 2,
    PSA_STAGE_ATTEND  = 4,
    PSA_STAGE_ALL     = 7
};

/* Bytes of device scratch the forward needs for `shape` and `c`; 0 if the
 * arguments are invalid.  Pure host arithmetic, no HIP call. */
size_t probsparse_attn_workspace_bytes(const psa_shape_t* shape, double c);

/* The whole forward, steps a1..a4 (Sec. 3.2, Eq. 11 and Eq. 12).
 *   Q, K, V     [B, H, L, D]     dtype per shape->dtype
 *   lengths     [B] int32        valid frames per batch item; NULL = all L valid
 *   sample_idx  [B, H, L_Q, U]   int32, the sampled keys of each query
 *   c           sampling/selection factor, u_b = clamp(ceil(c ln len_b), 1, len_b)
 *   out         [B, H, L_Q, D]   same dtype as the inputs; every element is written
 *   workspace   device scratch of at least probsparse_attn_workspace_bytes() bytes,
 *               256-byte aligned; contents on entry are ignored
 */
int probsparse_attn_fwd(const void* Q, const void* K, const void* V,
                        const int32_t* lengths, const int32_t* sample_idx,
                        double c, void* out, const psa_shape_t* shape,
                        void* workspace, size_t workspace_bytes, void* stream);

/* For callers that cannot allocate device memory or pass a workspace: code running under
 * HIP-graph capture, tight serving loops, harnesses that forbid hipMalloc.  The same forward
 * as probsparse_attn_fwd (same kernels, same results) with the scratch in a fixed array of
 * probsparse_static_workspace_bytes() = 16 MiB inside the library's device image, one per
 * GPU, held until the process ends.  The call allocates and frees nothing.
 *   - A shape whose probsparse_attn_workspace_bytes() exceeds the array is rejected with
 *     PSA_ERR_WORKSPACE before anything is enqueued (host arithmetic: testable without a GPU).
 *   - The array's device address is looked up on the first call on each device, or by
 *     probsparse_init(); call that first if the first call on a device is captured into a graph.
 *   - All such calls on one GPU share the one array, which keeps the last call's contents
 *     (the kernels reset the counters they need, as they do for any workspace): two calls
 *     that overlap in time on one GPU (different streams, or two graphs replayed
 *     concurrently) race on it and give wrong results.  Calls on one stream are safe. */
size_t probsparse_static_workspace_bytes(void);
int probsparse_attn_fwd_static(const void* Q, const void* K, const void* V,
                               const int32_t* lengths, const int32_t* sample_idx,
                               double c, void* out, const psa_shape_t* shape, void* stream);

/* Same call, with taps for parity checks.  Any tap may be NULL.
 *   M_out    [B, H, L_Q] float32   the measure of Eq. 11 (0 on padded queries)
 *   sel_out  [B, H, u_max] int32   I_sparse, free of duplicates, in no particular order,
 *                                  -1 padded; u_max = probsparse_u_max(shape, c)
 *   u_out    [B] int32             u_b
 */
int probsparse_attn_fwd_debug(const void* Q, const void* K, const void* V,
                              const int32_t* lengths, const int32_t* sample_idx,
                              double c, void* out, const psa_shape_t* shape,
                              void* workspace, size_t workspace_bytes, void* stream,
                              float* M_out, int32_t* sel_out, int32_t* u_out);

/* Run only the stages in `stage_mask` (PSA_STAGE_* OR-ed), in pipeline order.
 * Intermediates live in `workspace`, so a stage may be run alone after a full
 * call with the same arguments (this is how single kernels are timed). */
int probsparse_attn_fwd_stages(const void* Q, const void* K, const void* V,
                               const int32_t* lengths, const int32_t* sample_idx,
                               double c, void* out, const psa_shape_t* shape,
                               void* workspace, size_t workspace_bytes, void* stream,
                               int stage_mask);

/* Largest u_b any batch item can have: clamp(ceil(c ln L_K), 1, L_K); 0 on bad args. */
int32_t probsparse_u_max(const psa_shape_t* shape, double c);

/* The forward with the paper's own choices selectable (Sec. 3.2: L_sparse =
 * r_sparse * L; Eq. 12: v_i for the queries outside I_sparse).  Arguments as
 * for probsparse_attn_fwd_debug, `opt` (HOST pointer) in place of c; the taps
 * may be NULL.  With {PSA_U_LOG, PSA_FILL_MEAN, c} it is probsparse_attn_fwd_debug.
 * sel_out has probsparse_u_max_opt() columns.  Errors: PSA_ERR_ARG for an
 * unknown rule or fill or a factor that is not finite and positive. */
size_t  probsparse_attn_workspace_bytes_opt(const psa_shape_t* shape, const psa_options_t* opt);
int32_t probsparse_u_max_opt(const psa_shape_t* shape, const psa_options_t* opt);
int probsparse_attn_fwd_opt(const void* Q, const void* K, const void* V,
                            const int32_t* lengths, const int32_t* sample_idx,
                            const psa_options_t* opt, void* out, const psa_shape_t* shape,
                            void* workspace, size_t workspace_bytes, void* stream,
                            float* M_out, int32_t* sel_out, int32_t* u_out);

/* Steps a3 and a4 for index sets the caller already has (Sec. 4.4: the layers
 * that follow a prob-sparse layer reuse its I_sparse and skip the measure and
 * the selection; also serves the random-selection ablation of Sec. 4.2).
 *   sel       [B, H, u_stride] int32 DEVICE: the kept queries of each head in
 *             its first u[b] entries, in any order.  An entry outside
 *             [0, lengths[b]) is ignored; a repeated entry is computed twice
 *             to the same result.  The layout of probsparse_attn_fwd_debug's
 *             sel_out with u_stride = probsparse_u_max().
 *   u         [B] int32 DEVICE: entries of each sel row in use; clamped to
 *             [0, min(u_stride, lengths[b])]
 *   u_stride  1 .. L_Q
 *   fill      psa_fill_t
 * shape->U is ignored.  Everything else as for probsparse_attn_fwd. */
size_t probsparse_attn_with_indices_workspace_bytes(const psa_shape_t* shape, int32_t u_stride);
int probsparse_attn_fwd_with_indices(const void* Q, const void* K, const void* V,
                                     const int32_t* lengths, const int32_t* sel, const int32_t* u,
                                     int32_t u_stride, int32_t fill, void* out, const psa_shape_t* shape,
                                     void* workspace, size_t workspace_bytes, void* stream);

/* Gradients of steps a3 and a4 for a fixed index set (Eq. 7, Eq. 8, Eq. 12; Sec. 4.2 retrains a
 * prob-sparse model starting from a trained dense one, which needs them).  I_sparse is a hard
 * choice: no gradient flows through the measure or the selection.  With G = dOut the gradient
 * of a loss with respect to `out`, p_ij the softmax weights of the kept queries:
 *   kept query i:      dQ_i = (1/sqrt(D)) sum_j g_ij k_j,  g_ij = p_ij (G_i.v_j - sum_j' p_ij' G_i.v_j')
 *                      dK_j += (1/sqrt(D)) g_ij q_i,        dV_j += p_ij G_i
 *   other valid i:     dQ_i = 0;  PSA_FILL_MEAN: dV_j += G_i / len_b for every valid j;
 *                      PSA_FILL_VALUE: dV_i += G_i
 *   rows >= len_b:     dQ = dK = dV = 0
 *   sel, u, u_stride, fill   as for probsparse_attn_fwd_with_indices (the sel_out / u_out of a
 *             forward call with u_stride = probsparse_u_max()); the entries in use of a row
 *             must be distinct (an entry outside [0, len_b) is ignored)
 *   dOut      [B, H, L_Q, D] DEVICE, the tensors' dtype
 *   dQ, dK, dV  [B, H, L, D] DEVICE, the tensors' dtype; every element is written
 * The softmax weights are recomputed from Q and K (the forward keeps no statistics); all
 * arithmetic is float64 for both tensor types (the difference G_i.v_j - sum_j' p_ij' G_i.v_j'
 * cancels almost completely for sharply peaked rows).  shape->U is ignored. */
size_t probsparse_attn_bwd_workspace_bytes(const psa_shape_t* shape, int32_t u_stride);
int probsparse_attn_bwd(const void* Q, const void* K, const void* V, const int32_t* lengths,
                        const int32_t* sel, const int32_t* u, int32_t u_stride, int32_t fill,
                        const void* dOut, void* dQ, void* dK, void* dV, const psa_shape_t* shape,
                        void* workspace, size_t workspace_bytes, void* stream);

/* The multi-head module around the path (Sec. 3.1: Q = X W_q, K = X W_k, V = X W_v;
 * Sec. 2.2, Eq. 5: the MHSA module of a Conformer block; Sec. 4.2: heads of 64
 * dimensions), d_model = H * 64:
 *   Q[b,h,l,e] = sum_k X[b,l,k] Wq[h*64+e, k] + bq[h*64+e]      (likewise K, V)
 *   A = prob-sparse attention of (Q, K, V) per head             (probsparse_attn_fwd_opt)
 *   Y[b,l,j]   = sum_{h,e} A[b,h,l,e] Wo[j, h*64+e] + bo[j]
 * Every matrix is stored [d_out, d_in] row-major in the tensors' dtype, i.e. row
 * n holds column n of the paper's W; a bias pointer may be NULL.  The projected
 * tensors are written head-major [B, H, L, 64] directly, and the output matrix
 * reads the attention result in that layout, so no transpose ever touches memory.
 * Q, K, V and A are rounded once to the tensors' dtype where they are stored.
 * Arithmetic of the projections: products accumulate in float32.  bfloat16
 * operands are multiplied exactly; float32 operands are multiplied as sums of
 * three bfloat16 parts each (six partial products, error 2^-25 of |a||w| per
 * product), which gives the accuracy of a float32 contraction.
 * Frames at or beyond lengths[b] are projected like any other (the attention
 * ignores them; their rows of A are zero, so their rows of Y equal bo). */
typedef struct psa_mhsa_weights {
    const void *Wq, *Wk, *Wv, *Wo;      /* [H*64, H*64] DEVICE, 16-byte aligned */
    const void *bq, *bk, *bv, *bo;      /* [H*64] DEVICE or NULL               */
} psa_mhsa_weights_t;

/* The two projections alone (X, Y: [B, L, H*64]; Q, K, V, A: [B, H, L, 64]).  shape->U is ignored. */
int probsparse_qkv_project(const void* X, const psa_mhsa_weights_t* weights, void* Q, void* K, void* V,
                           const psa_shape_t* shape, void* stream);
int probsparse_out_project(const void* A, const psa_mhsa_weights_t* weights, void* Y,
                           const psa_shape_t* shape, void* stream);

/* The whole module.  The workspace holds Q, K, V, A and the attention's own
 * scratch; sample_idx, lengths and opt as for probsparse_attn_fwd_opt. */
size_t probsparse_mhsa_workspace_bytes(const psa_shape_t* shape, const psa_options_t* opt);
int probsparse_mhsa_fwd(const void* X, const psa_mhsa_weights_t* weights,
                        const int32_t* lengths, const int32_t* sample_idx, const psa_options_t* opt,
                        void* Y, const psa_shape_t* shape, void* workspace, size_t workspace_bytes, void* stream);

/* Diagnostic: the exact sparsity measure of Eq. 10 for every query,
 *   M[b,h,i] = ln sum_j exp(q_i.k_j / sqrt(D)) - (1/len_b) sum_j q_i.k_j / sqrt(D)
 * over the len_b valid keys of the item (Eq. 9 is this minus ln len_b).  It is
 * what the sampled measure of step a1 approximates (Sec. 3.2), at the cost of a
 * dense pass over all keys; the forward never calls it.
 *   M_out  [B, H, L_Q] float32 DEVICE, 4-byte aligned; 0 for padded queries
 * shape->U is ignored; no workspace. */
int probsparse_exact_measure(const void* Q, const void* K, const int32_t* lengths, float* M_out,
                             const psa_shape_t* shape, void* stream);

/* Baseline for comparison: dense softmax(Q K^T / sqrt(D)) V over the valid keys
 * of each item (Eq. 6); padded query rows are zero.  shape->U is ignored. */
size_t dense_attn_workspace_bytes(const psa_shape_t* shape);
int dense_attn_fwd(const void* Q, const void* K, const void* V, const int32_t* lengths,
                   void* out, const psa_shape_t* shape,
                   void* workspace, size_t workspace_bytes, void* stream);

/* Host only, no GPU needed: which kernels a call with this shape would launch, as
 * one line of `key=value` words in `buf` (NUL-terminated), e.g. which measure kernel
 * (`measure=lds|lds_half|stream|none`), how I_sparse is found (`select=lists|kernel|
 * segments|given_inline|given_prep`), which attend kernel (`attend=key_split|rows|
 * rows_half_keys`) and how partial results are merged.  For tests and for reading
 * profiles; the words are not a stable interface.  `opt` gives the selection rule
 * (steps a1..a4); with u_stride > 0 the plan is that of
 * probsparse_attn_fwd_with_indices and `opt` may be NULL.  Errors: PSA_ERR_NULL,
 * PSA_ERR_SHAPE / PSA_ERR_DTYPE, PSA_ERR_ARG (bad rule or stride, or `buf` too small). */
int probsparse_describe_plan(const psa_shape_t* shape, const psa_options_t* opt, int32_t u_stride,
                             char* buf, size_t buf_bytes);

/* Optional one-time set-up for the current device: raises the dynamic-LDS limit of
 * the kernels that use more than the default 64 KB.  Every entry point does this by
 * itself on first use, so the call is only needed by callers whose first call on a
 * device happens under HIP-graph capture and who want no attribute call inside it.
 * Thread-safe and idempotent.  Returns PSA_OK or PSA_ERR_HIP. */
int probsparse_init(void);

/* Static, NUL-terminated description of a status code. */
const char* probsparse_strerror(int code);

/* Library version, major * 10000 + minor * 100 + patch. */
int probsparse_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PROBSPARSE_H */
