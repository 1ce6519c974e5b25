/*
 * sla_oracle.c -- plain, slow, fp64 CPU oracle of the Sparse Linear Attention (SLA) forward.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the independent definition that the GPU library
 * is checked against; it shares no code, header, table or helper with the HIP path and the
 * product never calls it.  Only the tests, the smoke check and the benchmark's
 * "cpu_baseline" leg load it.
 *
 * What is computed (per batch item b and head h, independently), citing the paper:
 *   - eq. (1) / App. A:      O = A_sparse(Q,K,V) + Proj(A_lin(Q,K,V))
 *   - Alg. 1 steps 2-5:      scores, top-k mask, masked softmax, sparse output
 *   - Alg. 1 steps 6-9:      feature map phi, key-value summary, normaliser, linear output
 *   - Alg. 1 step 10:        O = O_sparse + O_lin W_O
 * at the block granularity of the SLA module the paper adopts (its SLA citation): the
 * top-k mask of Alg. 1 step 3 is taken over key blocks per query block on mean-pooled
 * Q/K, giving three classes (critical / marginal / negligible); the sparse branch
 * (steps 4-5) runs over the tokens of critical blocks, the linear branch (steps 7-9) over
 * the tokens of marginal blocks, negligible blocks are skipped.  phi is the softmax over
 * the head dimension (the benchmark configurations fix this) or, selectable, the ELU(x)+1 of
 * Alg. 1 step 6.
 *
 * Readings where the paper is silent (all listed in the design notes):
 *   - masked entries are excluded from the softmax (-inf), not multiplied by 0;
 *   - one total order per score row: score descending, then key-block index ascending;
 *     critical = first k_c of that order, negligible = last k_n, marginal = the rest;
 *   - classification uses the pooled logits (softmax is monotone, same sets);
 *   - pooled mean = (sum over the block's valid tokens, ascending token order) * (1/count);
 *   - pooled logit = 64-step fused-multiply-add chain over the channel index, ascending,
 *     starting from 0.0 (this fixes the rounding so a GPU can reproduce it bit for bit);
 *   - O_lin = 0 for a query block without marginal blocks; projection after normalisation;
 *   - W_O is row-major [D_in, D_out], right-multiplied, no bias (4096 parameters).
 *
 * Parity pins (tests/test_oracle_*.py): all-critical == brute-force dense softmax
 * attention; all-marginal == token-level linear attention of Alg. 1 steps 6-10; V == 1
 * closed form; constant-key closed form; convexity; rank definition by brute force;
 * known-order scores; permutation invariance; E4M3 code table against the format
 * definition.  Unpinned by the paper (fixed by the readings above): rounding rule of
 * fraction*blocks, tie order, phi temperature, per-block fp8 scale granularity.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t B, H, N, D;        /* D must be 64 */
    int32_t bq, bk;            /* query / key block sizes */
    int32_t k_crit, k_neg;     /* number of critical / negligible key blocks per query block */
    int32_t dtype;             /* 0: bf16 bit patterns (uint16); 1: E4M3 codes (uint8) + fp32 block scales */
    int32_t proj_per_head;     /* 0: W [D,D]; 1: W [H,D,D] */
    double  sm_scale;          /* 1/sqrt(D) normally */
    int32_t phi;               /* feature map of the linear branch: 0 softmax over the channels, 1 ELU(x)+1 (Alg. 1 step 6) */
} sla_oracle_params;

#define DH 64

static int nblocks(int n, int b) { return (n + b - 1) / b; }

/* ---- number formats ------------------------------------------------------------------ */

static double bf16_to_double(uint16_t bits)
{
    uint32_t u = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* E4M3 (App. B.1): 1 sign, 4 exponent (bias 7), 3 mantissa bits; no infinities; the
 * all-ones exponent+mantissa pattern is NaN; largest finite value 448. */
static double e4m3_to_double(uint8_t c)
{
    int s = c >> 7, e = (c >> 3) & 15, m = c & 7;
    double v;
    if (e == 15 && m == 7) return NAN;
    if (e == 0) v = ldexp((double)m, -9);
    else        v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return s ? -v : v;
}

/* Decode one head's [N,64] tensor to double.  fp8: value = code * scale[block] (exact in fp64). */
static void decode_head(const sla_oracle_params *p, const void *X, const float *scales, int blk,
                        int bh, double *out)
{
    const int N = p->N;
    if (p->dtype == 0) {
        const uint16_t *x = (const uint16_t *)X + (size_t)bh * N * DH;
        for (size_t i = 0; i < (size_t)N * DH; ++i) out[i] = bf16_to_double(x[i]);
    } else {
        const uint8_t *x = (const uint8_t *)X + (size_t)bh * N * DH;
        const float *sc = scales + (size_t)bh * nblocks(N, blk);
        for (int t = 0; t < N; ++t) {
            double s = (double)sc[t / blk];
            for (int d = 0; d < DH; ++d) out[(size_t)t * DH + d] = e4m3_to_double(x[(size_t)t * DH + d]) * s;
        }
    }
}

/* ---- step 1: block mean-pool --------------------------------------------------------- */
static void pool(const double *x, int N, int blk, double *mean /* [nblk][64] */)
{
    int nb = nblocks(N, blk);
    for (int j = 0; j < nb; ++j) {
        int t0 = j * blk, t1 = t0 + blk < N ? t0 + blk : N;
        double inv = 1.0 / (double)(t1 - t0);
        for (int d = 0; d < DH; ++d) {
            double s = 0.0;
            for (int t = t0; t < t1; ++t) s += x[(size_t)t * DH + d];
            mean[(size_t)j * DH + d] = s * inv;
        }
    }
}

/* ---- step 2: pooled logits (Alg. 1 step 2 on block means, without the 1/sqrt(d)) ------ */
static double pooled_logit(const double *q, const double *k)
{
    double s = 0.0;
    for (int d = 0; d < DH; ++d) s = fma(q[d], k[d], s);
    return s;
}

/* compressed block-score softmax P_c[i,:] = softmax_j(s_ij * sm_scale) */
static void row_softmax(const double *s, int n, double scale, double *pc)
{
    double m = -INFINITY, sum = 0.0;
    for (int j = 0; j < n; ++j) if (s[j] * scale > m) m = s[j] * scale;
    for (int j = 0; j < n; ++j) { pc[j] = exp(s[j] * scale - m); sum += pc[j]; }
    for (int j = 0; j < n; ++j) pc[j] /= sum;
}

/* ---- steps 3-4: counts and classification (Alg. 1 step 3 at block level) -------------- */
void sla_oracle_counts(double crit_frac, double neg_frac, int32_t Nkb, int32_t *k_crit, int32_t *k_neg)
{
    int kc = 0, kn;
    if (crit_frac > 0.0) { kc = (int)floor(crit_frac * Nkb + 0.5); if (kc < 1) kc = 1; if (kc > Nkb) kc = Nkb; }
    kn = (int)floor(neg_frac * Nkb + 0.5);
    if (kn > Nkb - kc) kn = Nkb - kc;
    if (kn < 0) kn = 0;
    *k_crit = kc; *k_neg = kn;
}

typedef struct { double s; int j; } scored;

static int by_score_desc_index_asc(const void *a, const void *b)
{
    const scored *x = (const scored *)a, *y = (const scored *)b;
    if (x->s > y->s) return -1;
    if (x->s < y->s) return 1;
    return (x->j > y->j) - (x->j < y->j);
}

/* labels: 2 critical, 1 marginal, 0 negligible */
static void classify_row(const double *s, int Nkb, int k_c, int k_n, int8_t *lab)
{
    scored *o = (scored *)malloc(sizeof(scored) * (size_t)Nkb);
    for (int j = 0; j < Nkb; ++j) { o[j].s = s[j]; o[j].j = j; }
    qsort(o, (size_t)Nkb, sizeof(scored), by_score_desc_index_asc);
    for (int r = 0; r < Nkb; ++r)
        lab[o[r].j] = r < k_c ? 2 : (r >= Nkb - k_n ? 0 : 1);
    free(o);
}

/* ---- feature map (Alg. 1 step 6): softmax over the 64 channels (the benchmark configurations),
 * or ELU(x)+1 elementwise as the algorithm prints it: x+1 for x > 0, exp(x) otherwise ------------ */
static void phi_softmax(const double *x, double *out)
{
    double m = x[0], sum = 0.0;
    for (int d = 1; d < DH; ++d) if (x[d] > m) m = x[d];
    for (int d = 0; d < DH; ++d) { out[d] = exp(x[d] - m); sum += out[d]; }
    for (int d = 0; d < DH; ++d) out[d] /= sum;
}
static void phi_map(int kind, const double *x, double *out)
{
    if (kind == 0) { phi_softmax(x, out); return; }
    for (int d = 0; d < DH; ++d) out[d] = x[d] > 0.0 ? x[d] + 1.0 : exp(x[d]);
}

/* ---- step 5: sparse branch for one query row (Alg. 1 steps 2, 4, 5 over critical tokens) */
static void sparse_row(const double *q, const double *K, const double *V, int N, int bk,
                       const int8_t *lab, int Nkb, double scale, double *out)
{
    double m = -INFINITY, l = 0.0;
    int any = 0;
    for (int e = 0; e < DH; ++e) out[e] = 0.0;
    for (int j = 0; j < Nkb; ++j) {
        if (lab[j] != 2) continue;
        int t1 = (j + 1) * bk < N ? (j + 1) * bk : N;
        for (int t = j * bk; t < t1; ++t) {
            double s = 0.0;
            for (int d = 0; d < DH; ++d) s += q[d] * K[(size_t)t * DH + d];
            s *= scale;
            if (s > m) m = s;
            any = 1;
        }
    }
    if (!any) return;
    for (int j = 0; j < Nkb; ++j) {
        if (lab[j] != 2) continue;
        int t1 = (j + 1) * bk < N ? (j + 1) * bk : N;
        for (int t = j * bk; t < t1; ++t) {
            double s = 0.0;
            for (int d = 0; d < DH; ++d) s += q[d] * K[(size_t)t * DH + d];
            double w = exp(s * scale - m);
            l += w;
            for (int e = 0; e < DH; ++e) out[e] += w * V[(size_t)t * DH + e];
        }
    }
    for (int e = 0; e < DH; ++e) out[e] /= l;
}

/* ---- step 6a: per-key-block linear states (Alg. 1 steps 7-8 restricted to one block) --- */
static void block_state(int phi, const double *K, const double *V, int t0, int t1, double *h /*[64][64]*/, double *z /*[64]*/)
{
    double f[DH];
    memset(h, 0, sizeof(double) * DH * DH);
    memset(z, 0, sizeof(double) * DH);
    for (int t = t0; t < t1; ++t) {
        phi_map(phi, K + (size_t)t * DH, f);
        for (int d = 0; d < DH; ++d) {
            z[d] += f[d];
            for (int e = 0; e < DH; ++e) h[d * DH + e] += f[d] * V[(size_t)t * DH + e];
        }
    }
}

/* ---- exported entry points ------------------------------------------------------------- */

/* Steps 1-4 for every (b,h).  Outputs (any may be NULL except labels):
 *   labels [B,H,Nqb,Nkb] int8; scores [B,H,Nqb,Nkb] double (pooled logits, unscaled);
 *   Pc same shape (softmax of scaled logits); qbar [B,H,Nqb,64]; kbar [B,H,Nkb,64]. */
int sla_oracle_classify(const sla_oracle_params *p, const void *Q, const void *K,
                        const float *sQ, const float *sK,
                        int8_t *labels, double *scores, double *Pc, double *qbar_out, double *kbar_out)
{
    if (!p || p->D != DH || !labels) return -1;
    const int N = p->N, Nqb = nblocks(N, p->bq), Nkb = nblocks(N, p->bk), BH = p->B * p->H;
    if (p->k_crit < 0 || p->k_neg < 0 || p->k_crit + p->k_neg > Nkb) return -1;
    #pragma omp parallel for schedule(dynamic, 1)
    for (int bh = 0; bh < BH; ++bh) {
        double *x = (double *)malloc(sizeof(double) * (size_t)N * DH);
        double *qb = (double *)malloc(sizeof(double) * (size_t)Nqb * DH);
        double *kb = (double *)malloc(sizeof(double) * (size_t)Nkb * DH);
        double *srow = (double *)malloc(sizeof(double) * (size_t)Nkb);
        decode_head(p, Q, sQ, p->bq, bh, x); pool(x, N, p->bq, qb);
        decode_head(p, K, sK, p->bk, bh, x); pool(x, N, p->bk, kb);
        if (qbar_out) memcpy(qbar_out + (size_t)bh * Nqb * DH, qb, sizeof(double) * (size_t)Nqb * DH);
        if (kbar_out) memcpy(kbar_out + (size_t)bh * Nkb * DH, kb, sizeof(double) * (size_t)Nkb * DH);
        for (int i = 0; i < Nqb; ++i) {
            size_t row = ((size_t)bh * Nqb + i) * Nkb;
            for (int j = 0; j < Nkb; ++j) srow[j] = pooled_logit(qb + (size_t)i * DH, kb + (size_t)j * DH);
            if (scores) memcpy(scores + row, srow, sizeof(double) * (size_t)Nkb);
            if (Pc) row_softmax(srow, Nkb, p->sm_scale, Pc + row);
            classify_row(srow, Nkb, p->k_crit, p->k_neg, labels + row);
        }
        free(x); free(qb); free(kb); free(srow);
    }
    return 0;
}

/* Step 6a for one (b,h): h [Nkb,64,64] (h[j][d][e]), z [Nkb,64]. */
int sla_oracle_states_head(const sla_oracle_params *p, const void *K, const void *V,
                           const float *sK, const float *sV, int32_t bh, double *h, double *z)
{
    if (!p || p->D != DH) return -1;
    const int N = p->N, Nkb = nblocks(N, p->bk);
    double *Kd = (double *)malloc(sizeof(double) * (size_t)N * DH);
    double *Vd = (double *)malloc(sizeof(double) * (size_t)N * DH);
    decode_head(p, K, sK, p->bk, bh, Kd);
    decode_head(p, V, sV, p->bk, bh, Vd);
    #pragma omp parallel for schedule(dynamic, 4)
    for (int j = 0; j < Nkb; ++j) {
        int t1 = (j + 1) * p->bk < N ? (j + 1) * p->bk : N;
        block_state(p->phi, Kd, Vd, j * p->bk, t1, h + (size_t)j * DH * DH, z + (size_t)j * DH);
    }
    free(Kd); free(Vd);
    return 0;
}

/* Steps 5-7 for a list of query blocks, given the labels.
 *   sel_bh[n], sel_i[n]: (b*H+h, query-block index) pairs, grouped arbitrarily.
 *   O, O_sparse, O_lin: [n_sel, bq, 64] double (rows past the sequence end are left 0);
 *   O_sparse / O_lin may be NULL.  O_lin is the normalised linear output before Proj. */
int sla_oracle_attend(const sla_oracle_params *p, const void *Q, const void *K, const void *V,
                      const float *sQ, const float *sK, const float *sV, const uint16_t *W,
                      const int8_t *labels, int32_t n_sel, const int32_t *sel_bh, const int32_t *sel_i,
                      double *O, double *O_sparse, double *O_lin)
{
    if (!p || p->D != DH || !labels || !O) return -1;
    const int N = p->N, bq = p->bq, bk = p->bk, Nqb = nblocks(N, bq), Nkb = nblocks(N, bk), BH = p->B * p->H;
    for (int bh = 0; bh < BH; ++bh) {
        int used = 0;
        for (int s = 0; s < n_sel; ++s) if (sel_bh[s] == bh) { used = 1; break; }
        if (!used) continue;
        double *Qd = (double *)malloc(sizeof(double) * (size_t)N * DH);
        double *Kd = (double *)malloc(sizeof(double) * (size_t)N * DH);
        double *Vd = (double *)malloc(sizeof(double) * (size_t)N * DH);
        double *h = (double *)malloc(sizeof(double) * (size_t)Nkb * DH * DH);
        double *z = (double *)malloc(sizeof(double) * (size_t)Nkb * DH);
        double Wd[DH * DH];
        decode_head(p, Q, sQ, bq, bh, Qd);
        decode_head(p, K, sK, bk, bh, Kd);
        decode_head(p, V, sV, bk, bh, Vd);
        const uint16_t *Wh = W + (p->proj_per_head ? (size_t)(bh % p->H) * DH * DH : 0);
        for (int i = 0; i < DH * DH; ++i) Wd[i] = bf16_to_double(Wh[i]);
        #pragma omp parallel for schedule(dynamic, 4)
        for (int j = 0; j < Nkb; ++j) {
            int t1 = (j + 1) * bk < N ? (j + 1) * bk : N;
            block_state(p->phi, Kd, Vd, j * bk, t1, h + (size_t)j * DH * DH, z + (size_t)j * DH);
        }
        #pragma omp parallel for schedule(dynamic, 1)
        for (int s = 0; s < n_sel; ++s) {
            if (sel_bh[s] != bh) continue;
            const int i = sel_i[s];
            const int8_t *lab = labels + ((size_t)bh * Nqb + i) * Nkb;
            double *Hi = (double *)calloc((size_t)DH * DH, sizeof(double));
            double Zi[DH], f[DH], osp[DH], olin[DH];
            int n_marg = 0;
            memset(Zi, 0, sizeof Zi);
            /* step 6b: sum the states of the marginal blocks */
            for (int j = 0; j < Nkb; ++j) {
                if (lab[j] != 1) continue;
                ++n_marg;
                for (int x = 0; x < DH * DH; ++x) Hi[x] += h[(size_t)j * DH * DH + x];
                for (int d = 0; d < DH; ++d) Zi[d] += z[(size_t)j * DH + d];
            }
            int t1 = (i + 1) * bq < N ? (i + 1) * bq : N;
            for (int t = i * bq; t < t1; ++t) {
                size_t orow = ((size_t)s * bq + (t - i * bq)) * DH;
                const double *q = Qd + (size_t)t * DH;
                sparse_row(q, Kd, Vd, N, bk, lab, Nkb, p->sm_scale, osp);
                /* step 6c: O_lin = phi(q) H / (phi(q) . Z)  (Alg. 1 step 9) */
                for (int e = 0; e < DH; ++e) olin[e] = 0.0;
                if (n_marg > 0) {
                    double den = 0.0;
                    phi_map(p->phi, q, f);
                    for (int d = 0; d < DH; ++d) {
                        den += f[d] * Zi[d];
                        for (int e = 0; e < DH; ++e) olin[e] += f[d] * Hi[d * DH + e];
                    }
                    for (int e = 0; e < DH; ++e) olin[e] /= den;
                }
                /* step 7: O = O_sparse + O_lin W  (Alg. 1 step 10, eq. 1) */
                for (int eo = 0; eo < DH; ++eo) {
                    double acc = 0.0;
                    for (int e = 0; e < DH; ++e) acc += olin[e] * Wd[e * DH + eo];
                    O[orow + eo] = osp[eo] + acc;
                }
                if (O_sparse) memcpy(O_sparse + orow, osp, sizeof osp);
                if (O_lin) memcpy(O_lin + orow, olin, sizeof olin);
            }
            free(Hi);
        }
        free(Qd); free(Kd); free(Vd); free(h); free(z);
    }
    return 0;
}

/* number of worker threads the OpenMP loops above will use */
#ifdef _OPENMP
#include <omp.h>
int sla_oracle_threads(void) { return omp_get_max_threads(); }
#else
int sla_oracle_threads(void) { return 1; }
#endif

/* single-value decoders, exported so the format tests can pin them against the definitions */
double sla_oracle_decode_e4m3(uint8_t code) { return e4m3_to_double(code); }
double sla_oracle_decode_bf16(uint16_t bits) { return bf16_to_double(bits); }
