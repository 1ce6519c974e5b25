// Host-side launch functions of the SLA kernels (internal to the library).
// Each returns the hipError_t of its launch; none allocates or synchronises.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "sla_common.hpp"

namespace sla {

// block mean-pool: X [BH,N,64] (bf16 or e4m3 + scales [BH,nblk]) -> mean fp64 [BH,nblk,64]
// rm (here and below): where the rows of a (b,h) live in the Q / K / V / O tensors (head-major or token-major)
hipError_t launch_pool(const void *X, const float *scales, bool fp8, RowMap rm, int BH, int N, int blk,
                       double *mean, hipStream_t st);

// pooled logits: S[bh][i][j] = fma-chain_d(qbar[bh][i][d], kbar[bh][j][d]); row pitch `pitch`
hipError_t launch_scores(const double *qbar, const double *kbar, int BH, int Nqb, int Nkb,
                         int pitch, double *S, hipStream_t st);

// three-way classifier on every score row.  mbits receives the marginal mask of every row, one bit
// per key block (bit j%64 of word j/64, lab_pitch/64 words per row, lab_pitch a multiple of 64, pad
// bits 0); lab_dense ([.,Nkb]), crit_idx ([.,k_c]), Pc ([.,Nkb]), S_dense ([.,Nkb]) are optional.
hipError_t launch_select(const double *S, int pitch, long rows, int Nkb, int k_c, int k_n,
                         uint64_t *mbits, int lab_pitch, int8_t *lab_dense, int32_t *crit_idx,
                         float *Pc, double *S_dense, float sm_scale, hipStream_t st);

// The same two steps for long rows when neither the logits nor the block-score softmax are wanted: the logits are
// stored as 32-bit keys (upper half of the order-preserving key of the fp64 logit; keys [rows, pitch], pitch in
// keys) and the selection runs on those, evaluating the exact logit again only for the members of a group of equal
// 32-bit keys that a threshold cuts through.  Same labels, mask and critical lists as launch_scores + launch_select.
hipError_t launch_score_keys(const double *qbar, const double *kbar, int BH, int Nqb, int Nkb, int pitch, uint32_t *keys,
                             hipStream_t st);
hipError_t launch_select_keys(const uint32_t *keys, int pitch, const double *qbar, const double *kbar, long rows, int Nqb, int Nkb,
                              int k_c, int k_n, uint64_t *mbits, int lab_pitch, int8_t *lab_dense, int32_t *crit_idx, hipStream_t st);

// short rows (Nkb <= 256): block mean of Q + pooled logits + classifier in one launch; kbar holds the
// block means of K.  Outputs as launch_select; qbar_out (optional) receives the block means of Q.
hipError_t launch_classify_fused(const void *Q, const float *sQ, bool fp8, RowMap rm, const double *kbar, int BH, int N, int bq, int Nkb,
                                 int k_c, int k_n, uint64_t *mbits, int lab_pitch, int8_t *lab_dense, int32_t *crit_idx,
                                 float *Pc, double *S_dense, double *qbar_out, float sm_scale, hipStream_t st);

// dense labels -> marginal masks + critical index lists (unfilled slots = -1)
hipError_t launch_labels_prepare(const int8_t *lab_dense, long rows, int Nkb, int k_c,
                                 uint64_t *mbits, int lab_pitch, int32_t *crit_idx, hipStream_t st);

// phi (here and below): feature map of the linear branch, 0 = softmax over the channels, 1 = ELU(x)+1.
// per-key-block states: hT [BH,Nkb,65,64] bf16; optionally also Vp [BH,Nkb,64,64] fp16, the transposed,
// key-permuted V tiles the attention kernel reads (bf16 V divided by a power of two per block, E4M3 codes
// unscaled) with lvs [BH,Nkb] fp32, the base-2 logarithm of what one unit of Vp stands for (that power of two,
// or the E4M3 block scale), and kbar [BH,Nkb,64] fp64, the block means of K (same arithmetic as launch_pool);
// NULL skips Vp + lvs, or kbar.  With W != NULL the launch also does the work of launch_transpose_w(W, nW, WT)
// in nW extra workgroups.
hipError_t launch_states(const void *K, const void *V, const float *sK, const float *sV, bool fp8, RowMap rm,
                         int BH, int N, void *hT, void *Vp, float *lvs, double *kbar, int phi, const void *W, int nW, void *WT, hipStream_t st);

// Hq[bh][i][:] = sum over the key blocks j whose bit is set in row (bh,i) of mbits of hT[bh][j][:]   (bf16 MFMA, fp32 accumulate)
hipError_t launch_aggregate(const uint64_t *mbits, int lab_pitch, const void *hT, int BH, int Nqb,
                            int Nkb, void *Hq, hipStream_t st);

// W [nW,64,64] bf16 -> WT[nW][e_out][e_in]
hipError_t launch_transpose_w(const void *W, int nW, void *WT, hipStream_t st);

// block-sparse attention over critical blocks + linear output + projection + sum (Vp, lvs: from launch_states).
// O32 != NULL: the result is written there as fp32 (the values before the bf16 rounding) and O is not touched.
hipError_t launch_attend(const void *Q, const void *K, const void *Vp, const float *lvs,
                         const float *sQ, const float *sK, bool fp8, RowMap rm,
                         const int32_t *crit_idx, int k_c, const void *Hq, const void *WT,
                         int proj_per_head, int phi, int B, int H, int N, int bq, float sm_scale,
                         void *O, float *O32, hipStream_t st);

// dW[w] = sum over the (b,h) that use projection matrix w and their tokens of O_lin^T dO, O_lin recomputed from Q and
// the aggregated states Hq; part is scratch of wproj_grad_groups(BH, N) * BH * 64 * 64 floats
int wproj_grad_groups(int BH, int N);
hipError_t launch_wproj_grad(const void *Q, const float *sQ, bool fp8, RowMap rm, const void *dO, const void *Hq, int B, int H, int N, int bq,
                             int proj_per_head, int phi, float *part, float *dW, hipStream_t st);

// X bf16 [BH,N,64] -> codes e4m3 [BH,N,64] + fp32 scales [BH, ceil(N/blk)], blk = 64 or 128 (App. B.2 per token block)
hipError_t launch_quantise_e4m3(const void *X, RowMap rm, int BH, int N, int blk, void *codes, float *scales, hipStream_t st);

// X bf16 [rows, cols] (cols a multiple of 8) -> E4M3 codes [rows, cols] + one fp32 scale per row (App. B.2 / B.3)
hipError_t launch_quantise_rows(const void *X, long rows, int cols, void *codes, float *scales, hipStream_t st);
// Y bf16 [M,O] = (A8 [M,K] x W8 [O,K]^T) * sa[i] * sw[o] + bias[o]; E4M3 codes, K a multiple of 128, O of 8; bias may be NULL
hipError_t launch_fp8_gemm(const void *A8, const float *sa, const void *W8, const float *sw, const void *bias, int M, int O, int K,
                           void *Y, hipStream_t st);

// The same GEMM as the qkv projection in front of the attention: A8 [B*N, K], W8 [3*H*64, K] (output channels ordered
// [q|k|v][head][64]); instead of y it writes the per-block scaled E4M3 form of Q, K and V: codes[w] [B,N,H,64] and
// scales[w] [B,H,ceil(N/blk)] for w = 0 (Q, blk = bq), 1 (K, blk = 64), 2 (V, blk = 64).  A token block must not
// straddle a token tile of fp8_gemm_qkv_token_tile(B*N, H) tokens: B == 1, or N a multiple of that tile.
int fp8_gemm_qkv_token_tile(int M, int H);
hipError_t launch_fp8_gemm_qkv(const void *A8, const float *sa, const void *W8, const float *sw, const void *bias, int B, int N, int H, int K,
                               int bq, void *const codes[3], float *const scales[3], hipStream_t st);

}  // namespace sla
