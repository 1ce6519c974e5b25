/*
 * sla.h -- C ABI of the MI355X (gfx950) Sparse Linear Attention forward.
 *
 * The operator (paper eq. (1), App. A, Alg. 1):
 *     O = A_sparse(Q,K,V) + Proj(A_lin(Q,K,V))
 * evaluated at block granularity, the way the SLA module the paper adopts works:
 *   1. Q and K are mean-pooled over blocks of bq / bk tokens; the pooled logits
 *      s_ij = qbar_i . kbar_j (Alg. 1 step 2 on block means) rank the key blocks of every
 *      query block; the top k_crit are "critical", the bottom k_neg "negligible", the rest
 *      "marginal" (Alg. 1 step 3, TopKMask, at block level).
 *   2. Sparse branch (Alg. 1 steps 4-5): softmax(Q K^T * sm_scale) V restricted to the
 *      tokens of the critical blocks (masked-out keys are excluded from the softmax).
 *   3. Linear branch (Alg. 1 steps 6-9) with the feature map phi (sla_phi_t below):
 *      h_j = phi(K_j)^T V_j, z_j = sum_t phi(K_j,t) per key block, summed over the marginal
 *      blocks of a query block: O_lin = phi(Q) H_i / (phi(Q) . Z_i); 0 if there is none.
 *   4. Combine (Alg. 1 step 10): O = O_sparse + O_lin W_proj.
 * Negligible blocks contribute to neither branch.
 *
 * Conventions common to every entry point
 *   - All tensor pointers are DEVICE pointers unless the comment says "host".  Tensors are
 *     dense, row-major, last index fastest: Q, K, V, O are [B, H, N, D] with D = 64.
 *   - bf16 tensors are raw 16-bit patterns; fp8 tensors are OCP E4M3 ("e4m3fn", max 448,
 *     App. B.1) codes with one fp32 scale per (b, h, token block): value = code * scale.
 *     Scale blocks are the pooling blocks: bq tokens for Q, bk tokens for K and V.
 *   - The caller owns all memory, including the workspace.  The library never allocates,
 *     frees or synchronises; every kernel is enqueued on `stream` (a hipStream_t passed as
 *     void*; NULL = the default stream).  Inputs are read-only; outputs and workspace must
 *     not alias inputs or each other.  Pointers must be 16-byte aligned (256 for workspace).
 *   - Every function returns a status; parameter errors are detected on the host before any
 *     launch.  No C++ exception crosses the boundary.  sla_last_error() returns a
 *     thread-local description of the most recent failure on the calling thread.
 *   - Calls on distinct streams with distinct workspaces may run concurrently.
 *
 * Block labels (int8): 2 = critical, 1 = marginal, 0 = negligible.  One total order per
 * row decides them: pooled logit descending, then key-block index ascending; critical =
 * first k_crit entries, negligible = last k_neg entries.
 */
#ifndef SLA_H_
#define SLA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SLA_OK = 0,
    SLA_ERR_INVALID_ARG = -1,   /* null pointer, bad shape, fraction out of range, misaligned pointer */
    SLA_ERR_UNSUPPORTED = -2,   /* valid request this build does not implement (D != 64, bk != 64, ...) */
    SLA_ERR_WORKSPACE = -3,     /* workspace too small or misaligned */
    SLA_ERR_HIP = -4            /* a HIP launch failed */
} sla_status_t;

typedef enum { SLA_BF16 = 0, SLA_FP8_E4M3 = 1 } sla_dtype_t;
/* feature map phi of the linear branch (Alg. 1 step 6): softmax over the D channels of the row (the benchmark
 * configurations), or ELU(x)+1 elementwise as the algorithm prints it (x+1 for x > 0, exp(x) otherwise) */
typedef enum { SLA_PHI_SOFTMAX = 0, SLA_PHI_ELU1 = 1 } sla_phi_t;

/* memory layout of Q, K, V, O (and dO): [B,H,N,D], or [B,N,H,D] as a fused qkv projection leaves its heads
 * (a row of D elements is contiguous either way; block scales, labels and W_proj are not affected) */
typedef enum { SLA_LAYOUT_BHND = 0, SLA_LAYOUT_BNHD = 1 } sla_layout_t;

typedef struct {
    int32_t B, H, N, D;          /* batch, heads, tokens per (b,h), head dim (must be 64) */
    int32_t bq, bk;              /* query block (64 or 128) and key block (64) sizes */
    double  crit_frac, neg_frac; /* fractions of key blocks per query block, in [0,1], sum <= 1 */
    int32_t k_crit, k_neg;       /* explicit block counts; -1 = derive from the fractions:
                                    k_crit = crit_frac > 0 ? max(1, floor(crit_frac*Nkb + 0.5)) : 0,
                                    k_neg  = min(Nkb - k_crit, floor(neg_frac*Nkb + 0.5)) */
    int32_t dtype;               /* sla_dtype_t of Q, K, V */
    int32_t phi;                 /* sla_phi_t */
    int32_t proj_per_head;       /* 0: W_proj is [D, D]; 1: [H, D, D] */
    float   sm_scale;            /* softmax scale of the sparse branch; 0 = 1/sqrt(D) (section 3.3) */
    int32_t layout;              /* sla_layout_t of Q, K, V, O, dO */
} sla_params_t;

/* Derived sizes: Nqb = ceil(N/bq), Nkb = ceil(N/bk). */

/* Host only.  Resolves the block counts the other calls will use (see k_crit / k_neg above). */
sla_status_t sla_resolve_counts(const sla_params_t *p, int32_t *k_crit, int32_t *k_neg);

/* Host only.  Bytes of workspace sla_forward (and every staged call) needs for these params. */
sla_status_t sla_workspace_bytes(const sla_params_t *p, size_t *bytes);

/*
 * Whole forward, eq. (1): steps 1-4 above.
 *   Q, K, V   in   [B,H,N,D] bf16 or E4M3
 *   sQ,sK,sV  in   fp32 [B,H,Nqb], [B,H,Nkb], [B,H,Nkb]; required for E4M3, NULL for bf16
 *   W_proj    in   bf16 [D_in, D_out] or [H, D_in, D_out] (right-multiplied, no bias)
 *   O         out  bf16 [B,H,N,D]
 *   labels    out  optional int8 [B,H,Nqb,Nkb]; NULL to skip
 */
sla_status_t sla_forward(const sla_params_t *p,
                         const void *Q, const void *K, const void *V,
                         const float *sQ, const float *sK, const float *sV,
                         const void *W_proj, void *O, int8_t *labels,
                         void *workspace, size_t workspace_bytes, void *stream);

/*
 * sla_forward for callers that cannot allocate device memory or pass a workspace (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): the same kernels and the same results as sla_forward, with
 * the workspace taken from a device array of SLA_STATIC_WORKSPACE_BYTES bytes that is part of the library (one copy
 * per GPU, held until the process ends).  Arguments as sla_forward without the workspace.  The call allocates
 * nothing and issues only kernel launches; on the first call on a device it looks up that device's copy of the array
 * (hipGetSymbolAddress) with the device current.  Shapes whose sla_workspace_bytes exceeds the array are rejected
 * with SLA_ERR_WORKSPACE before any launch.  Every call on a GPU uses that GPU's one array: calls that overlap on the
 * same GPU (different streams or threads) race; the array keeps the previous call's contents, and nothing in it has
 * to start at zero (every part is written before it is read).  sla_wproj_grad cannot follow this call (it needs the
 * caller's workspace).
 */
#define SLA_STATIC_WORKSPACE_BYTES (96u * 1024u * 1024u)
sla_status_t sla_forward_static(const sla_params_t *p,
                                const void *Q, const void *K, const void *V,
                                const float *sQ, const float *sK, const float *sV,
                                const void *W_proj, void *O, int8_t *labels, void *stream);

/*
 * The forward with the block labels given instead of computed: steps 2-4 on the labels of an earlier call
 * (e.g. the masks of one layer reused by the next, whose Q and K differ little).  Arguments as sla_forward, except
 *   labels   in   int8 [B,H,Nqb,Nkb], 2 critical / 1 marginal / 0 negligible.  A row may hold any number of marginal
 *                 blocks; of its critical blocks the first k_crit (ascending index) are attended, so rows taken from
 *                 sla_forward with the same params are reproduced exactly.
 * Leaves the workspace in the state sla_forward leaves it in (sla_wproj_grad may follow).
 */
sla_status_t sla_forward_with_labels(const sla_params_t *p,
                                     const void *Q, const void *K, const void *V,
                                     const float *sQ, const float *sK, const float *sV,
                                     const void *W_proj, const int8_t *labels, void *O,
                                     void *workspace, size_t workspace_bytes, void *stream);

/*
 * Gradient with respect to W_proj, the only parameter the method trains (section 3.3; Alg. 1 step 10:
 * O = O_sparse + O_lin W_O):
 *     dW[w][d_in][d_out] = sum over the (b,h) that use matrix w and over their tokens t of
 *                          O_lin[b,h,t][d_in] * dO[b,h,t][d_out]
 * with O_lin the normalised output of the linear branch before the projection.  No gradient flows through the
 * block masks or into Q, K, V.  O_lin is recomputed from Q and the aggregated states that a preceding
 * sla_forward with the same params and the same Q, K, V left in `workspace`: pass that workspace,
 * untouched since that call.
 *   Q, sQ   in   as in sla_forward
 *   dO      in   bf16 [B,H,N,D], the gradient of the loss with respect to O
 *   dW      out  fp32 [D_in, D_out] or [H, D_in, D_out] (written, not accumulated into)
 * The sum is formed in a fixed order (no atomics): the same inputs give the same bits.
 * With B, H or N zero, dW is set to zero with hipMemsetAsync: do not capture that case into a HIP graph.
 */
sla_status_t sla_wproj_grad(const sla_params_t *p, const void *Q, const float *sQ, const void *dO, float *dW,
                            void *workspace, size_t workspace_bytes, void *stream);

/*
 * Scaled FP8 quantiser (App. B.2: scale = max|x| / 448, clamp, cast to E4M3) applied per block of `blk`
 * consecutive tokens of every (b, h), which is the form sla_forward takes E4M3 Q, K and V in (blk = bq for Q,
 * bk for K and V):
 *     scale = max(amax, 1e-8) / 448 (fp32),   code = E4M3(clamp(x / scale, -448, 448)), round to nearest even
 *   X       in   bf16 [B,H,N,64], or [B,N,H,64] with layout = SLA_LAYOUT_BNHD
 *   blk     64 or 128
 *   codes   out  uint8, same layout as X
 *   scales  out  fp32 [B,H,ceil(N/blk)]
 * The result is defined bit for bit (fp32 division, one rounding).
 */
sla_status_t sla_quantise_e4m3(const void *X, int32_t B, int32_t H, int32_t N, int32_t blk, int32_t layout, void *codes,
                               float *scales, void *stream);

/*
 * Forward of the FP8 fake-quantised linear layer (Alg. 2; App. B.2-B.4), e.g. the qkv projection in front of the
 * attention: activations quantised per token, weights per output channel, both to E4M3 with
 * scale = max(amax, 1e-8) / 448, then  y = x_fp8 W_fp8^T + b  on the FP8 matrix unit (exact products, fp32
 * accumulation), scales and bias applied in fp32.
 *   x     in   bf16 [N, d_in]          d_in a multiple of 128
 *   W     in   bf16 [d_out, d_in]      d_out a multiple of 8
 *   bias  in   bf16 [d_out] or NULL
 *   y     out  bf16 [N, d_out]
 *   workspace  sla_fp8_linear_workspace_bytes(N, d_in, d_out) bytes, 256-byte aligned (the code matrices and scales)
 */
sla_status_t sla_fp8_linear_workspace_bytes(int32_t N, int32_t d_in, int32_t d_out, size_t *bytes);
sla_status_t sla_fp8_linear(const void *x, const void *W, const void *bias, int32_t N, int32_t d_in, int32_t d_out, void *y,
                            void *workspace, size_t workspace_bytes, void *stream);

/*
 * sla_fp8_linear as the qkv projection in front of the attention, with the per-block E4M3 quantiser in the epilogue of
 * the GEMM (Alg. 2; App. B.2-B.4): the layer's output y [B*N, 3*H*64] (channels ordered [q|k|v][head][64]) is never
 * written; instead each (head, token block) of it is quantised as sla_quantise_e4m3 would (blk = bq for Q, 64 for K and
 * V) and the call leaves Q, K and V in the form sla_forward takes with dtype = SLA_FP8_E4M3 and layout = SLA_LAYOUT_BNHD.
 * Bit for bit the result of sla_fp8_linear followed by sla_quantise_e4m3 on the three slices of y.
 *   x           in   bf16 [B*N, d_in]           d_in a multiple of 128
 *   W           in   bf16 [3*H*64, d_in]
 *   bias        in   bf16 [3*H*64] or NULL
 *   Q8, K8, V8  out  uint8 E4M3 codes [B,N,H,64]
 *   sQ          out  fp32 [B,H,ceil(N/bq)];   sK, sV  out  fp32 [B,H,ceil(N/64)]
 *   workspace   sla_fp8_linear_workspace_bytes(B*N, d_in, 3*H*64) bytes, 256-byte aligned
 * With B > 1, N must be a multiple of the GEMM's token tile (256, or 128 for small problems): a token block may not
 * straddle a tile; otherwise SLA_ERR_UNSUPPORTED.
 */
sla_status_t sla_fp8_linear_qkv(const void *x, const void *W, const void *bias, int32_t B, int32_t N, int32_t H, int32_t d_in,
                                int32_t bq, void *Q8, void *K8, void *V8, float *sQ, float *sK, float *sV,
                                void *workspace, size_t workspace_bytes, void *stream);

/*
 * Measurement variant of sla_forward: identical kernels and results, but every kernel is
 * bracketed by HIP events on `stream`; the call then WAITS for the stream and writes the
 * duration of each kernel in milliseconds to stage_ms[SLA_NUM_STAGES] (host memory).
 * It creates and destroys its events, so unlike every other entry point it touches the HIP
 * runtime beyond launches and synchronises.  sla_stage_name(i) names stage i.  Rows of at most
 * 256 key blocks take the fused classifier, reported as "scores"; "pool_q" and "select" are
 * then empty (their figure is the cost of an event pair).
 */
#define SLA_NUM_STAGES 6
sla_status_t sla_forward_profiled(const sla_params_t *p,
                                  const void *Q, const void *K, const void *V,
                                  const float *sQ, const float *sK, const float *sV,
                                  const void *W_proj, void *O, int8_t *labels,
                                  void *workspace, size_t workspace_bytes, void *stream,
                                  float *stage_ms);
const char *sla_stage_name(int stage);

/*
 * Step 1 alone: block mean-pool, pooled logits, classifier (Alg. 1 steps 2-3 at block level).
 *   labels    out  int8 [B,H,Nqb,Nkb]                                   (required)
 *   crit_idx  out  optional int32 [B,H,Nqb,k_crit], ascending key-block indices
 *   Pc        out  optional fp32 [B,H,Nqb,Nkb], softmax_j(s_ij * sm_scale) (compressed block scores)
 *   qbar,kbar out  optional fp64 [B,H,Nqb,D], [B,H,Nkb,D] block means
 *   scores    out  optional fp64 [B,H,Nqb,Nkb] pooled logits (unscaled)
 * Means are exact block sums (ascending token order, fp64) times 1/count; a logit is the
 * 64-step fp64 fused-multiply-add chain over the channel index, so labels are reproducible
 * bit for bit.
 */
sla_status_t sla_pool_classify(const sla_params_t *p, const void *Q, const void *K,
                               const float *sQ, const float *sK,
                               int8_t *labels, int32_t *crit_idx, float *Pc,
                               double *qbar, double *kbar, double *scores,
                               void *workspace, size_t workspace_bytes, void *stream);

/*
 * Step 3a alone: per-key-block linear states (Alg. 1 steps 6-8 restricted to one block).
 *   hT  out  bf16 [B,H,Nkb,65,D]: rows e = 0..63 hold h_j transposed, hT[e][d] = sum_t phi(K_t)[d] V_t[e];
 *            row 64 holds z_j[d] = sum_t phi(K_t)[d].  Tokens past N contribute nothing.
 */
sla_status_t sla_linear_states(const sla_params_t *p, const void *K, const void *V,
                               const float *sK, const float *sV, void *hT, void *stream);

/*
 * Step 3b alone: sum of the states over the marginal blocks of each query block.
 *   labels in   int8 [B,H,Nqb,Nkb]
 *   hT     in   bf16 [B,H,Nkb,65,D] (from sla_linear_states)
 *   Hq     out  bf16 [B,H,Nqb,65,D], same row layout as hT
 */
sla_status_t sla_marginal_aggregate(const sla_params_t *p, const int8_t *labels, const void *hT,
                                    void *Hq, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Steps 2, 3c and 4: block-sparse attention over the critical blocks of `labels`, linear
 * output from Hq, projection and sum.
 *   labels in   int8 [B,H,Nqb,Nkb]; every row must hold exactly k_crit entries equal to 2
 *   Hq     in   bf16 [B,H,Nqb,65,D], or NULL: then O = O_sparse only (W_proj may be NULL too)
 *   O      out  bf16 [B,H,N,D]
 */
sla_status_t sla_sparse_combine(const sla_params_t *p,
                                const void *Q, const void *K, const void *V,
                                const float *sQ, const float *sK, const float *sV,
                                const void *W_proj, const int8_t *labels, const void *Hq, void *O,
                                void *workspace, size_t workspace_bytes, void *stream);

/*
 * sla_sparse_combine with the result left in fp32: O32 [B,H,N,D] (same layout switch) receives the values the bf16
 * store of sla_sparse_combine rounds (round to nearest even), from the same kernel and the same arithmetic.  For tests
 * and diagnosis: it separates the error of the kernel's arithmetic from the rounding of the output format, which on
 * heavy-tailed rows (|O| far above the tensor's RMS) is by itself larger than the tolerance stated relative to the RMS.
 */
sla_status_t sla_sparse_combine_f32(const sla_params_t *p,
                                    const void *Q, const void *K, const void *V,
                                    const float *sQ, const float *sK, const float *sV,
                                    const void *W_proj, const int8_t *labels, const void *Hq, float *O32,
                                    void *workspace, size_t workspace_bytes, void *stream);

const char *sla_strerror(sla_status_t status);
const char *sla_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* SLA_H_ */
