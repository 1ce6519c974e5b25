// C ABI of the SLA forward: parameter validation, workspace carving and kernel sequencing.
// Host code only; every device operation is a kernel launch on the caller's stream.
#include "../../include/sla.h"
#include "sla_common.hpp"
#include "sla_kernels.hpp"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>

// Workspace of sla_forward_static: device memory that belongs to the library, one copy per GPU, held from the moment
// the code object is loaded until the process ends.  In host code the name is only a handle for hipGetSymbolAddress.
static __device__ __align__(256) unsigned char g_static_workspace[SLA_STATIC_WORKSPACE_BYTES];

namespace {

thread_local char g_err[512] = "";

sla_status_t fail(sla_status_t st, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return st;
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
bool aligned(const void *p, size_t a) { return ((uintptr_t)p % a) == 0; }

struct Plan {
    int BH, Nqb, Nkb, k_c, k_n, lab_pitch, s_pitch, nW;
    sla::RowMap rm;      // where the rows of a (b,h) live in Q, K, V, O, dO
    float sm_scale;
    bool fp8, empty;
    size_t off_qbar, off_kbar, off_scores, off_lab, off_crit, off_hT, off_Hq, off_WT, off_Vp, off_lvs, off_dWpart, total;
};

// Validates the parameter block and derives every size used downstream.
sla_status_t make_plan(const sla_params_t *p, Plan &pl)
{
    if (!p) return fail(SLA_ERR_INVALID_ARG, "params is NULL");
    if (p->B < 0 || p->H < 0 || p->N < 0) return fail(SLA_ERR_INVALID_ARG, "B, H, N must be >= 0 (got %d, %d, %d)", p->B, p->H, p->N);
    if (p->D != 64) return fail(SLA_ERR_UNSUPPORTED, "head dim D = %d; only 64 is implemented", p->D);
    if (p->bk != 64) return fail(SLA_ERR_UNSUPPORTED, "key block bk = %d; only 64 is implemented", p->bk);
    if (p->bq != 64 && p->bq != 128) return fail(SLA_ERR_UNSUPPORTED, "query block bq = %d; only 64 and 128 are implemented", p->bq);
    if (p->dtype != SLA_BF16 && p->dtype != SLA_FP8_E4M3) return fail(SLA_ERR_INVALID_ARG, "unknown dtype %d", p->dtype);
    if (p->phi != SLA_PHI_SOFTMAX && p->phi != SLA_PHI_ELU1) return fail(SLA_ERR_INVALID_ARG, "unknown feature map %d", p->phi);
    if (p->proj_per_head != 0 && p->proj_per_head != 1) return fail(SLA_ERR_INVALID_ARG, "proj_per_head must be 0 or 1");
    if (p->layout != SLA_LAYOUT_BHND && p->layout != SLA_LAYOUT_BNHD) return fail(SLA_ERR_INVALID_ARG, "unknown layout %d", p->layout);
    if (!(p->sm_scale >= 0.f) || !std::isfinite(p->sm_scale)) return fail(SLA_ERR_INVALID_ARG, "sm_scale must be finite and >= 0");
    memset(&pl, 0, sizeof pl);
    pl.empty = p->B == 0 || p->H == 0 || p->N == 0;
    if ((long)p->B * p->H > 65535) return fail(SLA_ERR_UNSUPPORTED, "B*H = %ld exceeds 65535", (long)p->B * p->H);
    pl.BH = p->B * p->H;
    pl.Nqb = (p->N + p->bq - 1) / p->bq;
    pl.Nkb = (p->N + p->bk - 1) / p->bk;
    if (pl.Nkb > 4096) return fail(SLA_ERR_UNSUPPORTED, "N = %d gives %d key blocks; at most 4096 are supported", p->N, pl.Nkb);
    if ((long)pl.BH * pl.Nqb > 0x7FFFFFF0L) return fail(SLA_ERR_UNSUPPORTED, "too many query blocks");
    pl.sm_scale = p->sm_scale > 0.f ? p->sm_scale : 0.125f;   // 1/sqrt(64)
    pl.fp8 = p->dtype == SLA_FP8_E4M3;
    pl.nW = p->proj_per_head ? p->H : 1;
    pl.rm = sla::make_rowmap(p->layout == SLA_LAYOUT_BNHD, p->H > 0 ? p->H : 1, p->N);

    if (p->k_crit >= 0 || p->k_neg >= 0) {
        if (p->k_crit < 0 || p->k_neg < 0) return fail(SLA_ERR_INVALID_ARG, "k_crit and k_neg must both be given or both be -1");
        if (p->k_crit + p->k_neg > pl.Nkb && !pl.empty)
            return fail(SLA_ERR_INVALID_ARG, "k_crit + k_neg = %d exceeds the %d key blocks", p->k_crit + p->k_neg, pl.Nkb);
        pl.k_c = p->k_crit;
        pl.k_n = p->k_neg;
    } else {
        const double fc = p->crit_frac, fn = p->neg_frac;
        if (!(fc >= 0.0 && fc <= 1.0) || !(fn >= 0.0 && fn <= 1.0)) return fail(SLA_ERR_INVALID_ARG, "fractions must lie in [0,1]");
        if (fc + fn > 1.0 + 1e-12) return fail(SLA_ERR_INVALID_ARG, "crit_frac + neg_frac = %g exceeds 1", fc + fn);
        int kc = 0;
        if (fc > 0.0) { kc = (int)std::floor(fc * pl.Nkb + 0.5); kc = kc < 1 ? 1 : kc; kc = kc > pl.Nkb ? pl.Nkb : kc; }
        int kn = (int)std::floor(fn * pl.Nkb + 0.5);
        kn = kn > pl.Nkb - kc ? pl.Nkb - kc : kn;
        pl.k_c = kc;
        pl.k_n = kn < 0 ? 0 : kn;
    }

    pl.lab_pitch = (int)align_up((size_t)pl.Nkb, 64);
    pl.s_pitch = (int)align_up((size_t)pl.Nkb, 8);
    size_t off = 0;
    auto carve = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    const size_t BH = (size_t)pl.BH;
    pl.off_qbar = carve(BH * pl.Nqb * 64 * sizeof(double));
    pl.off_kbar = carve(BH * pl.Nkb * 64 * sizeof(double));
    pl.off_scores = carve(BH * pl.Nqb * pl.s_pitch * sizeof(double));
    pl.off_lab = carve(BH * pl.Nqb * (size_t)(pl.lab_pitch / 8));   // marginal masks, one bit per (query block, key block)
    pl.off_crit = carve(BH * pl.Nqb * (size_t)(pl.k_c > 0 ? pl.k_c : 1) * sizeof(int32_t));
    pl.off_hT = carve(BH * pl.Nkb * sla::kStateElems * 2);
    pl.off_Hq = carve(BH * pl.Nqb * sla::kStateElems * 2);
    pl.off_WT = carve((size_t)pl.nW * 64 * 64 * 2);
    pl.off_Vp = carve(BH * pl.Nkb * 64 * 64 * 2);
    pl.off_lvs = carve(BH * pl.Nkb * sizeof(float));
    pl.off_dWpart = carve(pl.empty ? 0 : BH * (size_t)sla::wproj_grad_groups(pl.BH, p->N) * 64 * 64 * sizeof(float));
    pl.total = off;
    return SLA_OK;
}

sla_status_t check_ws(const Plan &pl, const void *ws, size_t bytes)
{
    if (!ws) return fail(SLA_ERR_WORKSPACE, "workspace is NULL (%zu bytes needed)", pl.total);
    if (!aligned(ws, 256)) return fail(SLA_ERR_WORKSPACE, "workspace must be 256-byte aligned");
    if (bytes < pl.total) return fail(SLA_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", bytes, pl.total);
    return SLA_OK;
}

#define SLA_REQ_PTR(ptr)                                                                              \
    do {                                                                                              \
        if (!(ptr)) return fail(SLA_ERR_INVALID_ARG, #ptr " is NULL");                                \
        if (!aligned((ptr), 16)) return fail(SLA_ERR_INVALID_ARG, #ptr " must be 16-byte aligned");   \
    } while (0)
#define SLA_OPT_PTR(ptr)                                                                              \
    do {                                                                                              \
        if ((ptr) && !aligned((ptr), 16)) return fail(SLA_ERR_INVALID_ARG, #ptr " must be 16-byte aligned"); \
    } while (0)
#define SLA_HIP(call)                                                                                 \
    do {                                                                                              \
        hipError_t e_ = (call);                                                                       \
        if (e_ != hipSuccess) return fail(SLA_ERR_HIP, "%s failed: %s", #call, hipGetErrorString(e_)); \
    } while (0)

template <class T> T *at(void *ws, size_t off) { return (T *)((char *)ws + off); }

// Pooling, pooled logits and classifier.  Leaves the marginal bit masks and the critical lists in the workspace.
sla_status_t run_classify(const sla_params_t *p, const Plan &pl, const void *Q, const void *K, const float *sQ,
                          const float *sK, int8_t *labels, int32_t *crit_out, float *Pc, double *qbar_out,
                          double *kbar_out, double *scores_out, void *ws, hipStream_t st, hipEvent_t *ev = nullptr, bool pooled = false)
{
    auto mark = [&](int i) { return ev ? hipEventRecord(ev[i], st) : hipSuccess; };
    double *qbar = qbar_out ? qbar_out : at<double>(ws, pl.off_qbar);
    double *kbar = kbar_out ? kbar_out : at<double>(ws, pl.off_kbar);
    int32_t *crit = crit_out ? crit_out : at<int32_t>(ws, pl.off_crit);
    const bool fused = pl.Nkb <= 256;   // short rows: Q means, logits and classification in one launch
    if (!pooled) {                      // sla_forward gets the K means from the states pass (and pools Q itself if needed)
        if (!fused) SLA_HIP(sla::launch_pool(Q, sQ, pl.fp8, pl.rm, pl.BH, p->N, p->bq, qbar, st));
        SLA_HIP(sla::launch_pool(K, sK, pl.fp8, pl.rm, pl.BH, p->N, p->bk, kbar, st));
    }
    SLA_HIP(mark(2));
    if (fused) {
        SLA_HIP(sla::launch_classify_fused(Q, sQ, pl.fp8, pl.rm, kbar, pl.BH, p->N, p->bq, pl.Nkb, pl.k_c, pl.k_n, at<uint64_t>(ws, pl.off_lab),
                                           pl.lab_pitch, labels, pl.k_c > 0 ? crit : nullptr, Pc, scores_out,
                                           qbar_out ? qbar_out : nullptr, pl.sm_scale, st));
        SLA_HIP(mark(3));
        return SLA_OK;
    }
    if (!Pc && !scores_out) {           // only the order matters: 32-bit keys instead of fp64 logits
        uint32_t *keys = at<uint32_t>(ws, pl.off_scores);
        SLA_HIP(sla::launch_score_keys(qbar, kbar, pl.BH, pl.Nqb, pl.Nkb, pl.s_pitch, keys, st));
        SLA_HIP(mark(3));
        SLA_HIP(sla::launch_select_keys(keys, pl.s_pitch, qbar, kbar, (long)pl.BH * pl.Nqb, pl.Nqb, pl.Nkb, pl.k_c, pl.k_n,
                                        at<uint64_t>(ws, pl.off_lab), pl.lab_pitch, labels, pl.k_c > 0 ? crit : nullptr, st));
        return SLA_OK;
    }
    SLA_HIP(sla::launch_scores(qbar, kbar, pl.BH, pl.Nqb, pl.Nkb, pl.s_pitch, at<double>(ws, pl.off_scores), st));
    SLA_HIP(mark(3));
    SLA_HIP(sla::launch_select(at<double>(ws, pl.off_scores), pl.s_pitch, (long)pl.BH * pl.Nqb, pl.Nkb, pl.k_c, pl.k_n,
                               at<uint64_t>(ws, pl.off_lab), pl.lab_pitch, labels, pl.k_c > 0 ? crit : nullptr, Pc,
                               scores_out, pl.sm_scale, st));
    return SLA_OK;
}

}  // namespace

extern "C" {

const char *sla_strerror(sla_status_t s)
{
    switch (s) {
    case SLA_OK: return "ok";
    case SLA_ERR_INVALID_ARG: return "invalid argument";
    case SLA_ERR_UNSUPPORTED: return "unsupported configuration";
    case SLA_ERR_WORKSPACE: return "workspace too small or misaligned";
    case SLA_ERR_HIP: return "HIP launch failed";
    }
    return "unknown status";
}

const char *sla_last_error(void) { return g_err; }

sla_status_t sla_resolve_counts(const sla_params_t *p, int32_t *k_crit, int32_t *k_neg)
{
    Plan pl;
    sla_status_t s = make_plan(p, pl);
    if (s != SLA_OK) return s;
    if (!k_crit || !k_neg) return fail(SLA_ERR_INVALID_ARG, "output pointer is NULL");
    *k_crit = pl.k_c;
    *k_neg = pl.k_n;
    return SLA_OK;
}

sla_status_t sla_workspace_bytes(const sla_params_t *p, size_t *bytes)
{
    Plan pl;
    sla_status_t s = make_plan(p, pl);
    if (s != SLA_OK) return s;
    if (!bytes) return fail(SLA_ERR_INVALID_ARG, "bytes is NULL");
    *bytes = pl.total;
    return SLA_OK;
}

sla_status_t sla_pool_classify(const sla_params_t *p, const void *Q, const void *K, const float *sQ, const float *sK,
                               int8_t *labels, int32_t *crit_idx, float *Pc, double *qbar, double *kbar, double *scores,
                               void *workspace, size_t workspace_bytes, void *stream)
{
    Plan pl;
    sla_status_t s = make_plan(p, pl);
    if (s != SLA_OK) return s;
    if (pl.empty) return SLA_OK;
    SLA_REQ_PTR(Q); SLA_REQ_PTR(K);
    if (!labels) return fail(SLA_ERR_INVALID_ARG, "labels is NULL");
    if (pl.fp8) { SLA_REQ_PTR(sQ); SLA_REQ_PTR(sK); }
    SLA_OPT_PTR(qbar); SLA_OPT_PTR(kbar); SLA_OPT_PTR(scores);
    if ((s = check_ws(pl, workspace, workspace_bytes)) != SLA_OK) return s;
    return run_classify(p, pl, Q, K, sQ, sK, labels, crit_idx, Pc, qbar, kbar, scores, workspace, (hipStream_t)stream);
}

sla_status_t sla_linear_states(const sla_params_t *p, const void *K, const void *V, const float *sK, const float *sV,
                               void *hT, void *stream)
{
    Plan pl;
    sla_status_t s = make_plan(p, pl);
    if (s != SLA_OK) return s;
    if (pl.empty) return SLA_OK;
    SLA_REQ_PTR(K); SLA_REQ_PTR(V); SLA_REQ_PTR(hT);
    if (pl.fp8) { SLA_REQ_PTR(sK); SLA_REQ_PTR(sV); }
    SLA_HIP(sla::launch_states(K, V, sK, sV, pl.fp8, pl.rm, pl.BH, p->N, hT, nullptr, nullptr, nullptr, p->phi, nullptr, 0, nullptr, (hipStream_t)stream));
    return SLA_OK;
}

sla_status_t sla_marginal_aggregate(const sla_params_t *p, const int8_t *labels, const void *hT, void *Hq,
                                    void *workspace, size_t workspace_bytes, void *stream)
{
    Plan pl;
    sla_status_t s = make_plan(p, pl);
    if (s != SLA_OK) return s;
    if (pl.empty) return SLA_OK;
    if (!labels) return fail(SLA_ERR_INVALID_ARG, "labels is NULL");
    SLA_REQ_PTR(hT); SLA_REQ_PTR(Hq);
    if ((s = check_ws(pl, workspace, workspace_bytes)) != SLA_OK) return s;
    hipStream_t st = (hipStream_t)stream;
    SLA_HIP(sla::launch_labels_prepare(labels, (long)pl.BH * pl.Nqb, pl.Nkb, pl.k_c > 0 ? pl.k_c : 1,
                                       at<uint64_t>(workspace, pl.off_lab), pl.lab_pitch, at<int32_t>(workspace, pl.off_crit), st));
    SLA_HIP(sla::launch_aggregate(at<uint64_t>(workspace, pl.off_lab), pl.lab_pitch, hT, pl.BH, pl.Nqb, pl.Nkb, Hq, st));
    return SLA_OK;
}

static sla_status_t sparse_combine_impl(const sla_params_t *p, const void *Q, const void *K, const void *V, const float *sQ,
                                        const float *sK, const float *sV, const void *W_proj, const int8_t *labels, const void *Hq,
                                        void *O, float *O32, void *workspace, size_t workspace_bytes, void *stream)
{
    Plan pl;
    sla_status_t s = make_plan(p, pl);
    if (s != SLA_OK) return s;
    if (pl.empty) return SLA_OK;
    SLA_REQ_PTR(Q); SLA_REQ_PTR(K); SLA_REQ_PTR(V);
    if (O32) SLA_REQ_PTR(O32); else SLA_REQ_PTR(O);
    if (!labels) return fail(SLA_ERR_INVALID_ARG, "labels is NULL");
    if (pl.fp8) { SLA_REQ_PTR(sQ); SLA_REQ_PTR(sK); SLA_REQ_PTR(sV); }
    SLA_OPT_PTR(Hq);
    if (Hq) SLA_REQ_PTR(W_proj);
    if ((s = check_ws(pl, workspace, workspace_bytes)) != SLA_OK) return s;
    hipStream_t st = (hipStream_t)stream;
    SLA_HIP(sla::launch_labels_prepare(labels, (long)pl.BH * pl.Nqb, pl.Nkb, pl.k_c > 0 ? pl.k_c : 1,
                                       at<uint64_t>(workspace, pl.off_lab), pl.lab_pitch, at<int32_t>(workspace, pl.off_crit), st));
    if (Hq) SLA_HIP(sla::launch_transpose_w(W_proj, pl.nW, at<void>(workspace, pl.off_WT), st));
    // the attention kernel reads V as transposed tiles; the states pass produces them (its states go to the workspace)
    SLA_HIP(sla::launch_states(K, V, sK, sV, pl.fp8, pl.rm, pl.BH, p->N, at<void>(workspace, pl.off_hT), at<void>(workspace, pl.off_Vp), at<float>(workspace, pl.off_lvs), nullptr, p->phi, nullptr, 0, nullptr, st));
    SLA_HIP(sla::launch_attend(Q, K, at<void>(workspace, pl.off_Vp), at<float>(workspace, pl.off_lvs), sQ, sK, pl.fp8, pl.rm, at<int32_t>(workspace, pl.off_crit), pl.k_c, Hq,
                               at<void>(workspace, pl.off_WT), p->proj_per_head, p->phi, p->B, p->H, p->N, p->bq, pl.sm_scale, O, O32, st));
    return SLA_OK;
}

sla_status_t sla_sparse_combine(const sla_params_t *p, const void *Q, const void *K, const void *V, const float *sQ,
                                const float *sK, const float *sV, const void *W_proj, const int8_t *labels, const void *Hq,
                                void *O, void *workspace, size_t workspace_bytes, void *stream)
{
    return sparse_combine_impl(p, Q, K, V, sQ, sK, sV, W_proj, labels, Hq, O, nullptr, workspace, workspace_bytes, stream);
}

sla_status_t sla_sparse_combine_f32(const sla_params_t *p, const void *Q, const void *K, const void *V, const float *sQ,
                                    const float *sK, const float *sV, const void *W_proj, const int8_t *labels, const void *Hq,
                                    float *O32, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!O32) return fail(SLA_ERR_INVALID_ARG, "O32 is NULL");
    return sparse_combine_impl(p, Q, K, V, sQ, sK, sV, W_proj, labels, Hq, nullptr, O32, workspace, workspace_bytes, stream);
}

sla_status_t sla_forward_with_labels(const sla_params_t *p, const void *Q, const void *K, const void *V, const float *sQ,
                                     const float *sK, const float *sV, const void *W_proj, const int8_t *labels, void *O,
                                     void *workspace, size_t workspace_bytes, void *stream)
{
    Plan pl;
    sla_status_t s = make_plan(p, pl);
    if (s != SLA_OK) return s;
    if (pl.empty) return SLA_OK;
    SLA_REQ_PTR(Q); SLA_REQ_PTR(K); SLA_REQ_PTR(V); SLA_REQ_PTR(W_proj); SLA_REQ_PTR(O);
    if (!labels) return fail(SLA_ERR_INVALID_ARG, "labels is NULL");
    if (pl.fp8) { SLA_REQ_PTR(sQ); SLA_REQ_PTR(sK); SLA_REQ_PTR(sV); }
    if ((s = check_ws(pl, workspace, workspace_bytes)) != SLA_OK) return s;
    hipStream_t st = (hipStream_t)stream;
    // the forward without its classifier: the given labels become the bit masks and critical lists of the workspace
    SLA_HIP(sla::launch_labels_prepare(labels, (long)pl.BH * pl.Nqb, pl.Nkb, pl.k_c > 0 ? pl.k_c : 1,
                                       at<uint64_t>(workspace, pl.off_lab), pl.lab_pitch, at<int32_t>(workspace, pl.off_crit), st));
    SLA_HIP(sla::launch_states(K, V, sK, sV, pl.fp8, pl.rm, pl.BH, p->N, at<void>(workspace, pl.off_hT), at<void>(workspace, pl.off_Vp),
                               at<float>(workspace, pl.off_lvs), nullptr, p->phi, W_proj, pl.nW, at<void>(workspace, pl.off_WT), st));
    SLA_HIP(sla::launch_aggregate(at<uint64_t>(workspace, pl.off_lab), pl.lab_pitch, at<void>(workspace, pl.off_hT), pl.BH, pl.Nqb, pl.Nkb,
                                  at<void>(workspace, pl.off_Hq), st));
    SLA_HIP(sla::launch_attend(Q, K, at<void>(workspace, pl.off_Vp), at<float>(workspace, pl.off_lvs), sQ, sK, pl.fp8, pl.rm, at<int32_t>(workspace, pl.off_crit), pl.k_c,
                               at<void>(workspace, pl.off_Hq), at<void>(workspace, pl.off_WT), p->proj_per_head, p->phi, p->B, p->H,
                               p->N, p->bq, pl.sm_scale, O, nullptr, st));
    return SLA_OK;
}

static sla_status_t forward_impl(const sla_params_t *p, const void *Q, const void *K, const void *V, const float *sQ,
                                 const float *sK, const float *sV, const void *W_proj, void *O, int8_t *labels,
                                 void *workspace, size_t workspace_bytes, void *stream, hipEvent_t *ev, bool *launched)
{
    Plan pl;
    sla_status_t s = make_plan(p, pl);
    if (s != SLA_OK) return s;
    if (pl.empty) return SLA_OK;
    SLA_REQ_PTR(Q); SLA_REQ_PTR(K); SLA_REQ_PTR(V); SLA_REQ_PTR(W_proj); SLA_REQ_PTR(O);
    if (pl.fp8) { SLA_REQ_PTR(sQ); SLA_REQ_PTR(sK); SLA_REQ_PTR(sV); }
    if ((s = check_ws(pl, workspace, workspace_bytes)) != SLA_OK) return s;
    hipStream_t st = (hipStream_t)stream;
    auto mark = [&](int i) { return ev ? hipEventRecord(ev[i], st) : hipSuccess; };
    if (launched) *launched = true;
    SLA_HIP(mark(0));
    if (pl.Nkb > 256) SLA_HIP(sla::launch_pool(Q, sQ, pl.fp8, pl.rm, pl.BH, p->N, p->bq, at<double>(workspace, pl.off_qbar), st));
    SLA_HIP(mark(1));     // states + V^T tiles + block means of K: the one pass over K and V besides the attention kernel;
                          // a few extra workgroups of the same launch lay out W_proj for the attention epilogue
    SLA_HIP(sla::launch_states(K, V, sK, sV, pl.fp8, pl.rm, pl.BH, p->N, at<void>(workspace, pl.off_hT), at<void>(workspace, pl.off_Vp),
                               at<float>(workspace, pl.off_lvs), at<double>(workspace, pl.off_kbar), p->phi, W_proj, pl.nW, at<void>(workspace, pl.off_WT), st));
    if ((s = run_classify(p, pl, Q, K, sQ, sK, labels, nullptr, nullptr, nullptr, nullptr, nullptr, workspace, st, ev, true)) != SLA_OK) return s;
    SLA_HIP(mark(4));
    SLA_HIP(sla::launch_aggregate(at<uint64_t>(workspace, pl.off_lab), pl.lab_pitch, at<void>(workspace, pl.off_hT), pl.BH, pl.Nqb,
                                  pl.Nkb, at<void>(workspace, pl.off_Hq), st));
    SLA_HIP(mark(5));
    SLA_HIP(sla::launch_attend(Q, K, at<void>(workspace, pl.off_Vp), at<float>(workspace, pl.off_lvs), sQ, sK, pl.fp8, pl.rm, at<int32_t>(workspace, pl.off_crit), pl.k_c,
                               at<void>(workspace, pl.off_Hq), at<void>(workspace, pl.off_WT), p->proj_per_head, p->phi, p->B, p->H,
                               p->N, p->bq, pl.sm_scale, O, nullptr, st));
    SLA_HIP(mark(6));
    return SLA_OK;
}

sla_status_t sla_forward(const sla_params_t *p, const void *Q, const void *K, const void *V, const float *sQ,
                         const float *sK, const float *sV, const void *W_proj, void *O, int8_t *labels,
                         void *workspace, size_t workspace_bytes, void *stream)
{
    return forward_impl(p, Q, K, V, sQ, sK, sV, W_proj, O, labels, workspace, workspace_bytes, stream, nullptr, nullptr);
}

sla_status_t sla_forward_static(const sla_params_t *p, const void *Q, const void *K, const void *V, const float *sQ,
                                const float *sK, const float *sV, const void *W_proj, void *O, int8_t *labels, void *stream)
{
    Plan pl;
    sla_status_t s = make_plan(p, pl);
    if (s != SLA_OK) return s;
    if (pl.total > (size_t)SLA_STATIC_WORKSPACE_BYTES)
        return fail(SLA_ERR_WORKSPACE, "this shape needs %zu bytes of workspace; sla_forward_static holds %zu (use sla_forward with a caller workspace)",
                    pl.total, (size_t)SLA_STATIC_WORKSPACE_BYTES);
    // address of the current device's copy of the array, looked up once per device
    constexpr int kMaxDevices = 64;
    static void *ptrs[kMaxDevices] = {};
    static std::mutex mtx;
    int dev = -1;
    SLA_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(SLA_ERR_UNSUPPORTED, "device ordinal %d out of range", dev);
    void *ws = nullptr;
    {
        std::lock_guard<std::mutex> lock(mtx);
        if (!ptrs[dev]) {
            void *ptr = nullptr;
            SLA_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_static_workspace)));
            if (!ptr) return fail(SLA_ERR_HIP, "hipGetSymbolAddress returned a null address");
            ptrs[dev] = ptr;
        }
        ws = ptrs[dev];
    }
    return forward_impl(p, Q, K, V, sQ, sK, sV, W_proj, O, labels, ws, (size_t)SLA_STATIC_WORKSPACE_BYTES, stream, nullptr, nullptr);
}

sla_status_t sla_wproj_grad(const sla_params_t *p, const void *Q, const float *sQ, const void *dO, float *dW,
                            void *workspace, size_t workspace_bytes, void *stream)
{
    Plan pl;
    sla_status_t s = make_plan(p, pl);
    if (s != SLA_OK) return s;
    SLA_REQ_PTR(dW);
    hipStream_t st = (hipStream_t)stream;
    if (pl.empty) {                      // no tokens: the gradient is zero
        SLA_HIP(hipMemsetAsync(dW, 0, (size_t)pl.nW * 64 * 64 * sizeof(float), st));
        return SLA_OK;
    }
    SLA_REQ_PTR(Q); SLA_REQ_PTR(dO);
    if (pl.fp8) SLA_REQ_PTR(sQ);
    if ((s = check_ws(pl, workspace, workspace_bytes)) != SLA_OK) return s;
    SLA_HIP(sla::launch_wproj_grad(Q, sQ, pl.fp8, pl.rm, dO, at<void>(workspace, pl.off_Hq), p->B, p->H, p->N, p->bq, p->proj_per_head, p->phi,
                                   at<float>(workspace, pl.off_dWpart), dW, st));
    return SLA_OK;
}

sla_status_t sla_quantise_e4m3(const void *X, int32_t B, int32_t H, int32_t N, int32_t blk, int32_t layout, void *codes,
                               float *scales, void *stream)
{
    if (layout != SLA_LAYOUT_BHND && layout != SLA_LAYOUT_BNHD) return fail(SLA_ERR_INVALID_ARG, "unknown layout %d", layout);
    if (B < 0 || H < 0 || N < 0) return fail(SLA_ERR_INVALID_ARG, "negative size (B=%d H=%d N=%d)", B, H, N);
    if (blk != 64 && blk != 128) return fail(SLA_ERR_UNSUPPORTED, "block of %d tokens; only 64 and 128 are implemented", blk);
    if ((long)B * H > 0x7FFFFFF0L / 4) return fail(SLA_ERR_UNSUPPORTED, "B*H = %ld is too large", (long)B * H);
    if (B == 0 || H == 0 || N == 0) return SLA_OK;
    SLA_REQ_PTR(X); SLA_REQ_PTR(codes);
    if (!scales) return fail(SLA_ERR_INVALID_ARG, "scales is NULL");
    SLA_HIP(sla::launch_quantise_e4m3(X, sla::make_rowmap(layout == SLA_LAYOUT_BNHD, H, N), B * H, N, blk, codes, scales, (hipStream_t)stream));
    return SLA_OK;
}

namespace {
struct LinPlan { size_t off_cx, off_sx, off_cw, off_sw, total; };
static sla_status_t make_lin_plan(int32_t N, int32_t d_in, int32_t d_out, LinPlan &lp)
{
    if (N < 0 || d_in <= 0 || d_out <= 0) return fail(SLA_ERR_INVALID_ARG, "bad sizes (N=%d d_in=%d d_out=%d)", N, d_in, d_out);
    if (d_in % 128 != 0) return fail(SLA_ERR_UNSUPPORTED, "d_in = %d; only multiples of 128 are implemented", d_in);
    if (d_out % 8 != 0) return fail(SLA_ERR_UNSUPPORTED, "d_out = %d; only multiples of 8 are implemented", d_out);
    if ((double)N * d_in >= 4.0e9 || (double)d_out * d_in >= 4.0e9) return fail(SLA_ERR_UNSUPPORTED, "operand of 4 GB or more");
    size_t off = 0;
    auto carve = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    lp.off_cx = carve((size_t)N * d_in);
    lp.off_sx = carve((size_t)N * sizeof(float));
    lp.off_cw = carve((size_t)d_out * d_in);
    lp.off_sw = carve((size_t)d_out * sizeof(float));
    lp.total = off;
    return SLA_OK;
}
}  // namespace

sla_status_t sla_fp8_linear_workspace_bytes(int32_t N, int32_t d_in, int32_t d_out, size_t *bytes)
{
    LinPlan lp;
    sla_status_t s = make_lin_plan(N, d_in, d_out, lp);
    if (s != SLA_OK) return s;
    if (!bytes) return fail(SLA_ERR_INVALID_ARG, "bytes is NULL");
    *bytes = lp.total;
    return SLA_OK;
}

sla_status_t sla_fp8_linear(const void *x, const void *W, const void *bias, int32_t N, int32_t d_in, int32_t d_out, void *y,
                            void *workspace, size_t workspace_bytes, void *stream)
{
    LinPlan lp;
    sla_status_t s = make_lin_plan(N, d_in, d_out, lp);
    if (s != SLA_OK) return s;
    if (N == 0) return SLA_OK;
    SLA_REQ_PTR(x); SLA_REQ_PTR(W); SLA_REQ_PTR(y);
    SLA_OPT_PTR(bias);
    if (!workspace) return fail(SLA_ERR_WORKSPACE, "workspace is NULL (%zu bytes needed)", lp.total);
    if (!aligned(workspace, 256)) return fail(SLA_ERR_WORKSPACE, "workspace must be 256-byte aligned");
    if (workspace_bytes < lp.total) return fail(SLA_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, lp.total);
    hipStream_t st = (hipStream_t)stream;
    SLA_HIP(sla::launch_quantise_rows(x, N, d_in, at<void>(workspace, lp.off_cx), at<float>(workspace, lp.off_sx), st));
    SLA_HIP(sla::launch_quantise_rows(W, d_out, d_in, at<void>(workspace, lp.off_cw), at<float>(workspace, lp.off_sw), st));
    SLA_HIP(sla::launch_fp8_gemm(at<void>(workspace, lp.off_cx), at<float>(workspace, lp.off_sx), at<void>(workspace, lp.off_cw),
                                 at<float>(workspace, lp.off_sw), bias, N, d_out, d_in, y, st));
    return SLA_OK;
}

sla_status_t sla_fp8_linear_qkv(const void *x, const void *W, const void *bias, int32_t B, int32_t N, int32_t H, int32_t d_in,
                                int32_t bq, void *Q8, void *K8, void *V8, float *sQ, float *sK, float *sV,
                                void *workspace, size_t workspace_bytes, void *stream)
{
    if (B < 0 || N < 0 || H <= 0) return fail(SLA_ERR_INVALID_ARG, "bad sizes (B=%d N=%d H=%d)", B, N, H);
    if (bq != 64 && bq != 128) return fail(SLA_ERR_UNSUPPORTED, "query block bq = %d; only 64 and 128 are implemented", bq);
    if ((double)B * N >= 2.0e9) return fail(SLA_ERR_UNSUPPORTED, "too many tokens");
    const int32_t tokens = B * N, d_out = 3 * H * 64;
    LinPlan lp;
    sla_status_t s = make_lin_plan(tokens, d_in, d_out, lp);
    if (s != SLA_OK) return s;
    if (tokens == 0) return SLA_OK;
    const int tile = sla::fp8_gemm_qkv_token_tile(tokens, H);
    if (B > 1 && N % tile != 0)
        return fail(SLA_ERR_UNSUPPORTED, "with B > 1, N must be a multiple of %d (a token block may not straddle a token tile); N = %d", tile, N);
    SLA_REQ_PTR(x); SLA_REQ_PTR(W); SLA_REQ_PTR(Q8); SLA_REQ_PTR(K8); SLA_REQ_PTR(V8);
    SLA_OPT_PTR(bias);
    if (!sQ || !sK || !sV) return fail(SLA_ERR_INVALID_ARG, "a scale output is NULL");
    if (!workspace) return fail(SLA_ERR_WORKSPACE, "workspace is NULL (%zu bytes needed)", lp.total);
    if (!aligned(workspace, 256)) return fail(SLA_ERR_WORKSPACE, "workspace must be 256-byte aligned");
    if (workspace_bytes < lp.total) return fail(SLA_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, lp.total);
    hipStream_t st = (hipStream_t)stream;
    SLA_HIP(sla::launch_quantise_rows(x, tokens, d_in, at<void>(workspace, lp.off_cx), at<float>(workspace, lp.off_sx), st));
    SLA_HIP(sla::launch_quantise_rows(W, d_out, d_in, at<void>(workspace, lp.off_cw), at<float>(workspace, lp.off_sw), st));
    void *const codes[3] = {Q8, K8, V8};
    float *const scales[3] = {sQ, sK, sV};
    SLA_HIP(sla::launch_fp8_gemm_qkv(at<void>(workspace, lp.off_cx), at<float>(workspace, lp.off_sx), at<void>(workspace, lp.off_cw),
                                     at<float>(workspace, lp.off_sw), bias, B, N, H, d_in, bq, codes, scales, st));
    return SLA_OK;
}

const char *sla_stage_name(int stage)
{
    static const char *names[SLA_NUM_STAGES] = {"pool_q", "states", "scores", "select", "aggregate", "attend"};
    return stage >= 0 && stage < SLA_NUM_STAGES ? names[stage] : "?";
}

sla_status_t sla_forward_profiled(const sla_params_t *p, const void *Q, const void *K, const void *V, const float *sQ,
                                  const float *sK, const float *sV, const void *W_proj, void *O, int8_t *labels,
                                  void *workspace, size_t workspace_bytes, void *stream, float *stage_ms)
{
    if (!stage_ms) return fail(SLA_ERR_INVALID_ARG, "stage_ms is NULL");
    hipEvent_t ev[SLA_NUM_STAGES + 1];
    int made = 0;
    sla_status_t s = SLA_OK;
    for (; made <= SLA_NUM_STAGES; ++made)
        if (hipEventCreate(&ev[made]) != hipSuccess) { s = fail(SLA_ERR_HIP, "hipEventCreate failed"); break; }
    bool launched = false;
    if (s == SLA_OK) s = forward_impl(p, Q, K, V, sQ, sK, sV, W_proj, O, labels, workspace, workspace_bytes, stream, ev, &launched);
    for (int i = 0; i < SLA_NUM_STAGES; ++i) stage_ms[i] = 0.f;
    if (s == SLA_OK && launched) {
        if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) s = fail(SLA_ERR_HIP, "hipStreamSynchronize failed");
        for (int i = 0; s == SLA_OK && i < SLA_NUM_STAGES; ++i)
            if (hipEventElapsedTime(&stage_ms[i], ev[i], ev[i + 1]) != hipSuccess) s = fail(SLA_ERR_HIP, "hipEventElapsedTime failed");
    }
    for (int i = 0; i < made; ++i) (void)hipEventDestroy(ev[i]);
    return s;
}

}  // extern "C"
