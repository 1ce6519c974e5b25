// Gradient of the projection of the linear branch (Alg. 1 step 10 of the paper: O = O_sparse + O_lin W_O,
// with W_O the only parameter the method trains, section 3.3):
//     dW[d_in][d_out] = sum_t O_lin[t][d_in] * dO[t][d_out],   O_lin[t] = phi(Q_t) H_i / (phi(Q_t) . Z_i)
// summed over the tokens of a head (and, by the reduction kernel below, over every (b, h) that shares the matrix).
// O_lin is recomputed from Q and the aggregated states Hq the forward left in the workspace, with the arithmetic of
// the forward epilogue (phi(Q) rounded to bf16, fp32 accumulation, 1/(phi.Z) applied in fp32, O_lin rounded to bf16
// as the operand of the second product).
//
// One wavefront takes 32 query rows at a time and keeps D = dW^T (64 x 64 fp32) in 64 accumulator registers:
//     O_lin[q][e]      = phi(Q) (A operand, registers; lane = query row)  x  Hq (B operand: LDS rows of hT[e][.])
//     D[d_out][e]     += dO^T (A operand: LDS, transposed on its way in)  x  O_lin (B operand = the accumulators of
//                        the first product re-packed in place; their row order is a permutation of the 32 query
//                        rows, which the dO^T fragments are read with)
// The four waves of a workgroup walk a contiguous range of a head's rows, add their accumulators through LDS and
// write one partial per workgroup; a second kernel adds the partials in a fixed order (no atomics: the result does
// not depend on scheduling).  The pass is bound by HBM: Q, dO and Hq are each read once (about twice for Hq, whose
// 8 KB tile is fetched by every wave that needs it).
#include "sla_common.hpp"
#include "sla_kernels.hpp"

namespace sla {

namespace {
constexpr int kGRow = 72;      // bf16 per LDS row of the state tile: 64 + 8 pad (144 B)
constexpr int kTRow = 40;      // bf16 per LDS row of the transposed dO tile: 32 tokens + 8 pad (80 B)
constexpr int kHsBytes = 64 * kGRow * 2, kZsBytes = 128, kTsBytes = 64 * kTRow * 2, kDsBytes = 128;
constexpr int kWaveLds = kHsBytes + kZsBytes + kTsBytes + kDsBytes;      // 14592 bytes per wave
constexpr float kLog2eB = 1.4426950408889634f;
}  // namespace

template <bool FP8>
__global__ __launch_bounds__(256) void wproj_grad_kernel(const void *__restrict__ Qp, const float *__restrict__ sQ,
                                                         const uint16_t *__restrict__ dO, const uint16_t *__restrict__ Hq,
                                                         RowMap rm, int N, int bq, int Nqb, int units, int upw, int groups, int phi,
                                                         float *__restrict__ part)
{
    static_assert(3 * 16384 <= 4 * kWaveLds, "three parked accumulators must fit the workgroup's LDS");
    __shared__ __attribute__((aligned(16))) uint8_t lds[4 * kWaveLds];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, g = lane >> 5;
    const long bh = blockIdx.x / groups;
    const int grp = blockIdx.x % groups;
    uint8_t *my = lds + wave * kWaveLds;
    uint16_t *Hs = (uint16_t *)my;                                   // hT tile of the query block: [e][d]
    uint16_t *Zs = (uint16_t *)(my + kHsBytes);                      // its Z row
    uint16_t *Ts = (uint16_t *)(my + kHsBytes + kZsBytes);           // dO^T of the 32 rows: [d_out][token]
    float *Ds = (float *)(my + kHsBytes + kZsBytes + kTsBytes);      // 1/(phi.Z) per row
    const size_t head = rm.head(bh);

    f32x16 acc[2][2];                                                // [ot][et]: D[32 ot + ..][32 et + l32]
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int x = 0; x < 16; ++x) acc[a][b][x] = 0.f;

    // Raw global data of one 32-row unit, held in registers while the previous unit is processed (plain dwords:
    // arrays of vectors are not reliably kept in registers).
    struct Unit {
        uint32_t h[32];      // state tile: 8 pieces of 16 bytes
        uint32_t z[4];       // Z row: 16 bytes in each of the first eight lanes
        uint32_t d[16];      // dO: 8 tokens x 4 channels
        uint32_t q[FP8 ? 8 : 16];
        float qscale;
    };
    auto load_unit = [&](int u, Unit &r) {
        const int t0 = 32 * u, i = t0 / bq, q = t0 + l32;
        const uint16_t *Hi = Hq + ((size_t)bh * Nqb + i) * kStateElems;
#pragma unroll
        for (int x = 0; x < 8; ++x) {
            const int c = lane + 64 * x, row = c >> 3, col = (c & 7) * 8;
            const uint4 v = *(const uint4 *)(Hi + row * kD + col);
            r.h[4 * x] = v.x; r.h[4 * x + 1] = v.y; r.h[4 * x + 2] = v.z; r.h[4 * x + 3] = v.w;
        }
        {
            const uint4 v = *(const uint4 *)(Hi + 64 * kD + (lane & 7) * 8);      // every lane reads it; eight store it
            r.z[0] = v.x; r.z[1] = v.y; r.z[2] = v.z; r.z[3] = v.w;
        }
        const int eq = lane & 15, tg = lane >> 4;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int t = t0 + 8 * tg + k;
            const uint2 v = *(const uint2 *)(dO + head + (size_t)min(t, N - 1) * rm.ts + 4 * eq);
            r.d[2 * k] = t < N ? v.x : 0u;                                        // rows past the end of the sequence are zero
            r.d[2 * k + 1] = t < N ? v.y : 0u;
        }
        const int qc = min(q, N - 1);                                             // such rows are switched off through 1/(phi.Z) = 0
        if constexpr (FP8) {
            const uint8_t *qr = (const uint8_t *)Qp + head + (size_t)qc * rm.ts + 32 * g;
            const uint4 w0 = *(const uint4 *)qr, w1 = *(const uint4 *)(qr + 16);
            r.q[0] = w0.x; r.q[1] = w0.y; r.q[2] = w0.z; r.q[3] = w0.w; r.q[4] = w1.x; r.q[5] = w1.y; r.q[6] = w1.z; r.q[7] = w1.w;
            r.qscale = sQ[bh * Nqb + i];
        } else {
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const uint4 w = *(const uint4 *)((const uint16_t *)Qp + head + (size_t)qc * rm.ts + 16 * s + 8 * g);
                r.q[4 * s] = w.x; r.q[4 * s + 1] = w.y; r.q[4 * s + 2] = w.z; r.q[4 * s + 3] = w.w;
            }
            r.qscale = 1.0f;
        }
    };

    const int u1 = min((grp + 1) * upw, units);
    Unit cur;
    if (grp * upw + wave < u1) load_unit(grp * upw + wave, cur);
    for (int u = grp * upw + wave; u < u1; u += 4) {
        const int t0 = 32 * u;
        const bool qok = t0 + l32 < N;
        wave_lds_sync();                                             // the previous rows' LDS reads are done

        // ---- state tile and Z row -> LDS; dO rows -> dO^T in LDS (8 tokens x 4 channels per lane, transposed in registers)
#pragma unroll
        for (int x = 0; x < 8; ++x) {
            const int c = lane + 64 * x, row = c >> 3, col = (c & 7) * 8;
            *(uint4 *)(Hs + row * kGRow + col) = make_uint4(cur.h[4 * x], cur.h[4 * x + 1], cur.h[4 * x + 2], cur.h[4 * x + 3]);
        }
        if (lane < 8) *(uint4 *)(Zs + lane * 8) = make_uint4(cur.z[0], cur.z[1], cur.z[2], cur.z[3]);
        {
            const int eq = lane & 15, tg = lane >> 4;
            const uint32_t *w = cur.d;
            uint4 c0, c1, c2, c3;                                    // channel 4 eq + c over the 8 tokens
            c0.x = __builtin_amdgcn_perm(w[2], w[0], 0x05040100);   c1.x = __builtin_amdgcn_perm(w[2], w[0], 0x07060302);
            c2.x = __builtin_amdgcn_perm(w[3], w[1], 0x05040100);   c3.x = __builtin_amdgcn_perm(w[3], w[1], 0x07060302);
            c0.y = __builtin_amdgcn_perm(w[6], w[4], 0x05040100);   c1.y = __builtin_amdgcn_perm(w[6], w[4], 0x07060302);
            c2.y = __builtin_amdgcn_perm(w[7], w[5], 0x05040100);   c3.y = __builtin_amdgcn_perm(w[7], w[5], 0x07060302);
            c0.z = __builtin_amdgcn_perm(w[10], w[8], 0x05040100);  c1.z = __builtin_amdgcn_perm(w[10], w[8], 0x07060302);
            c2.z = __builtin_amdgcn_perm(w[11], w[9], 0x05040100);  c3.z = __builtin_amdgcn_perm(w[11], w[9], 0x07060302);
            c0.w = __builtin_amdgcn_perm(w[14], w[12], 0x05040100); c1.w = __builtin_amdgcn_perm(w[14], w[12], 0x07060302);
            c2.w = __builtin_amdgcn_perm(w[15], w[13], 0x05040100); c3.w = __builtin_amdgcn_perm(w[15], w[13], 0x07060302);
            uint16_t *dst = Ts + (4 * eq) * kTRow + 8 * tg;
            *(uint4 *)(dst) = c0;
            *(uint4 *)(dst + kTRow) = c1;
            *(uint4 *)(dst + 2 * kTRow) = c2;
            *(uint4 *)(dst + 3 * kTRow) = c3;
        }

        // ---- phi(Q): softmax over the 64 channels of the row (this lane holds 32, lane^32 the rest).
        // x[8s + c] is channel dcol(s) + c, the channel slot c of K-step s carries in the product below.
        float x[32];
        if constexpr (FP8) {
#pragma unroll
            for (int w = 0; w < 8; ++w) {
                const f32x2 lo = __builtin_amdgcn_cvt_pk_f32_fp8(cur.q[w], false), hi = __builtin_amdgcn_cvt_pk_f32_fp8(cur.q[w], true);
                x[4 * w + 0] = lo[0] * cur.qscale; x[4 * w + 1] = lo[1] * cur.qscale; x[4 * w + 2] = hi[0] * cur.qscale; x[4 * w + 3] = hi[1] * cur.qscale;
            }
        } else {
#pragma unroll
            for (int w = 0; w < 16; ++w) { x[2 * w] = bf16_lo(cur.q[w]); x[2 * w + 1] = bf16_hi(cur.q[w]); }
        }
        if (u + 4 < u1) load_unit(u + 4, cur);                       // the next unit's loads fly while this one is processed
        float inv = 1.0f;
        if (phi == 0) {
            float mx = x[0];
#pragma unroll
            for (int d = 1; d < 32; ++d) mx = fmaxf(mx, x[d]);
            mx = pair_max(mx);
            float sum = 0.f;
#pragma unroll
            for (int d = 0; d < 32; ++d) { x[d] = fast_exp2((x[d] - mx) * kLog2eB); sum += x[d]; }
            sum += xchg32(sum);
            inv = 1.0f / sum;
        } else {                                                     // ELU(x)+1, elementwise
#pragma unroll
            for (int d = 0; d < 32; ++d) x[d] = x[d] > 0.f ? x[d] + 1.0f : fast_exp2(x[d] * kLog2eB);
        }
        wave_lds_sync();                                             // the tiles staged above are visible
        bf16x8 fq[4];
        float den = 0.f;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int dcol = FP8 ? 32 * g + 8 * s : 16 * s + 8 * g;
            uint4 o;
            o.x = pack_bf16(x[8 * s + 0] * inv, x[8 * s + 1] * inv); o.y = pack_bf16(x[8 * s + 2] * inv, x[8 * s + 3] * inv);
            o.z = pack_bf16(x[8 * s + 4] * inv, x[8 * s + 5] * inv); o.w = pack_bf16(x[8 * s + 6] * inv, x[8 * s + 7] * inv);
            fq[s] = __builtin_bit_cast(bf16x8, o);
            const uint4 z = *(const uint4 *)(Zs + dcol);
            den += bf16_lo(o.x) * bf16_lo(z.x) + bf16_hi(o.x) * bf16_hi(z.x) + bf16_lo(o.y) * bf16_lo(z.y) + bf16_hi(o.y) * bf16_hi(z.y)
                 + bf16_lo(o.z) * bf16_lo(z.z) + bf16_hi(o.z) * bf16_hi(z.z) + bf16_lo(o.w) * bf16_lo(z.w) + bf16_hi(o.w) * bf16_hi(z.w);
        }
        den += xchg32(den);
        // no marginal block: H = Z = 0 and O_lin = 0; a row past the end of the sequence contributes nothing either
        if (g == 0) Ds[l32] = (qok && den > 0.f) ? 1.0f / den : 0.f;
        wave_lds_sync();

        // ---- O_lin[q][e] = sum_d phi(Q)[q][d] h[d][e]: lane = column e, registers = rows q = 8a + 4g + b
        f32x16 ol[2];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int dcol = FP8 ? 32 * g + 8 * s : 16 * s + 8 * g;
#pragma unroll
            for (int et = 0; et < 2; ++et) {
                const bf16x8 hf = *(const bf16x8 *)(Hs + (32 * et + l32) * kGRow + dcol);
                if (s == 0) {
                    f32x16 zero;
#pragma unroll
                    for (int y = 0; y < 16; ++y) zero[y] = 0.f;
                    ol[et] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fq[s], hf, zero, 0, 0, 0);
                } else {
                    ol[et] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fq[s], hf, ol[et], 0, 0, 0);
                }
            }
        }
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const float4 d4 = *(const float4 *)(Ds + 8 * a + 4 * g);
#pragma unroll
            for (int et = 0; et < 2; ++et) {
                ol[et][4 * a + 0] *= d4.x; ol[et][4 * a + 1] *= d4.y; ol[et][4 * a + 2] *= d4.z; ol[et][4 * a + 3] *= d4.w;
            }
        }

        // ---- D[d_out][e] += sum_q dO[q][d_out] O_lin[q][e].  K-slot 8g + j of step uu of the re-packed accumulators is
        // query row 16 uu + 8 (j >> 2) + 4 g + (j & 3); the dO^T fragment is assembled in the same order from two
        // 8-byte pieces (rows 16 uu + 4 g .. + 3 and 16 uu + 8 + 4 g .. + 3).
#pragma unroll
        for (int uu = 0; uu < 2; ++uu) {
            const bf16x8 pf0 = pack8(ol[0], 8 * uu), pf1 = pack8(ol[1], 8 * uu);
#pragma unroll
            for (int ot = 0; ot < 2; ++ot) {
                const uint16_t *row = Ts + (32 * ot + l32) * kTRow + 16 * uu + 4 * g;
                const uint2 lo = *(const uint2 *)row, hi = *(const uint2 *)(row + 8);
                const bf16x8 af = __builtin_bit_cast(bf16x8, make_uint4(lo.x, lo.y, hi.x, hi.y));
                acc[ot][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, pf0, acc[ot][0], 0, 0, 0);
                acc[ot][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, pf1, acc[ot][1], 0, 0, 0);
            }
        }
    }

    // ---- add the four waves' accumulators (waves 1..3 park theirs in LDS, in register order) and write the
    // workgroup's partial as dW[d_in][d_out]: register 4a + b of acc[ot][et] is d_out = 32 ot + 8 a + 4 g + b, d_in = 32 et + l32
    __syncthreads();                                                 // every wave is done with its LDS slice
    if (wave > 0) {
        float4 *dst = (float4 *)(lds + (wave - 1) * 16384);
#pragma unroll
        for (int ot = 0; ot < 2; ++ot)
#pragma unroll
            for (int et = 0; et < 2; ++et)
#pragma unroll
                for (int a = 0; a < 4; ++a)
                    dst[((ot * 2 + et) * 4 + a) * 64 + lane] = make_float4(acc[ot][et][4 * a], acc[ot][et][4 * a + 1], acc[ot][et][4 * a + 2], acc[ot][et][4 * a + 3]);
    }
    __syncthreads();
    if (wave == 0) {
        float *out = part + (size_t)blockIdx.x * kD * kD;
#pragma unroll
        for (int ot = 0; ot < 2; ++ot)
#pragma unroll
            for (int et = 0; et < 2; ++et)
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    float4 v = make_float4(acc[ot][et][4 * a], acc[ot][et][4 * a + 1], acc[ot][et][4 * a + 2], acc[ot][et][4 * a + 3]);
#pragma unroll
                    for (int w = 0; w < 3; ++w) {
                        const float4 o = ((const float4 *)(lds + w * 16384))[((ot * 2 + et) * 4 + a) * 64 + lane];
                        v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w;
                    }
                    *(float4 *)(out + (32 * et + l32) * kD + 32 * ot + 8 * a + 4 * g) = v;
                }
    }
}

// dW[w][x] = sum of the partials of every (b, h) that uses matrix w, in ascending (b, h, group) order
__global__ __launch_bounds__(256) void wproj_grad_reduce_kernel(const float *__restrict__ part, int B, int H, int groups,
                                                                int per_head, float *__restrict__ dW)
{
    const int w = blockIdx.y, x = blockIdx.x * 256 + threadIdx.x;   // x < 4096 by construction of the grid
    float s = 0.f;
    for (int b = 0; b < B; ++b)
        for (int h = per_head ? w : 0; h < (per_head ? w + 1 : H); ++h) {
            const float *p = part + ((size_t)(b * H + h) * groups) * kD * kD + x;
#pragma unroll 8
            for (int gidx = 0; gidx < groups; ++gidx) s += p[(size_t)gidx * kD * kD];      // loads batch, adds stay in order
        }
    dW[(size_t)w * kD * kD + x] = s;
}

int wproj_grad_groups(int BH, int N)
{
    const int units = (N + 31) / 32;
    int g = (2048 + 4 * BH - 1) / (4 * BH);          // about 2048 waves in all
    const int gmax = (units + 3) / 4;
    g = g > gmax ? gmax : g;
    return g < 1 ? 1 : g;
}

hipError_t launch_wproj_grad(const void *Q, const float *sQ, bool fp8, RowMap rm, const void *dO, const void *Hq, int B, int H, int N, int bq,
                             int proj_per_head, int phi, float *part, float *dW, hipStream_t st)
{
    const int BH = B * H, Nqb = (N + bq - 1) / bq, units = (N + 31) / 32;
    const int groups = wproj_grad_groups(BH, N), upw = (units + groups - 1) / groups;
    const unsigned grid = (unsigned)BH * groups;
    if (fp8) wproj_grad_kernel<true><<<grid, 256, 0, st>>>(Q, sQ, (const uint16_t *)dO, (const uint16_t *)Hq, rm, N, bq, Nqb, units, upw, groups, phi, part);
    else     wproj_grad_kernel<false><<<grid, 256, 0, st>>>(Q, sQ, (const uint16_t *)dO, (const uint16_t *)Hq, rm, N, bq, Nqb, units, upw, groups, phi, part);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    wproj_grad_reduce_kernel<<<dim3(kD * kD / 256, proj_per_head ? H : 1), 256, 0, st>>>(part, B, H, groups, proj_per_head, dW);
    return hipGetLastError();
}

}  // namespace sla
