// Per-key-block linear-attention states (Alg. 1 steps 6-8 of the paper restricted to one
// key block; phi = softmax over the head dimension, or the ELU(x)+1 the algorithm prints):
//     h_j = phi(K_j)^T V_j   (64 x 64),   z_j = sum_t phi(K_j,t)   (64)
// written as bf16 hT[j][e][d] = h_j[d][e] (rows 0..63) and hT[j][64][d] = z_j[d].
//
// One wavefront owns a contiguous run of key blocks.  Per block it stages K (row-major) and V
// (transposed) in its own LDS slice, every lane normalises one token row (no cross-lane work
// for the softmax), the 64x64x64 product runs on v_mfma_f32_32x32x16_bf16, and the state leaves
// in the layout the aggregation GEMM and the attention epilogue read.  The same pass also leaves
// V^T of the block (fp16, key-permuted) for the attention kernel, which can then fetch both of
// its tiles as plain 16-byte rows, and (optionally) the fp64 block mean of K for the classifier,
// so K is read from HBM once per layer by this kernel instead of twice.
// The fp16 copy of V is exact: bf16 values are first divided by the power of two 2^e of the block's largest
// magnitude (so that any bf16 tensor fits the range of fp16; entries more than 2^24 below the block's maximum
// are the only ones to lose bits), E4M3 codes are taken as they are; the attention kernel gets e, or the base-2
// logarithm of the E4M3 block scale, in `lvs` and folds it into the exponent of its softmax weights.
// The loads of the next block are in flight (in registers) while the current one is processed, and the
// state and V^T tiles leave through LDS so that every store instruction writes 1 KB of whole rows:
// the kernel is bound by HBM (16 KB in, 16.6 KB out per block for bf16 inputs).  A few workgroups past
// the states grid lay out the projection matrices for the attention epilogue (one launch fewer).
#include "sla_common.hpp"
#include "sla_kernels.hpp"

namespace sla {

constexpr int kLdsRow = 72;            // bf16 elements per LDS row (64 + 8 pad: 144 B stride)
constexpr int kWavesPerWG = 2;

// Raw global data of one key block, as loaded: K as 16-byte row chunks, V as 8-byte (bf16) or
// 4-byte (e4m3) pieces of four channels arranged for the register transpose.
template <bool FP8>
struct BlockRegs {
    uint32_t k[FP8 ? 16 : 32];    // plain dwords: arrays of vectors are not reliably kept in registers
    uint32_t v[FP8 ? 16 : 32];
};

// Rows past the end of the sequence (ragged last block of a head) repeat the last valid row: their
// phi is multiplied by zero below, and finite stand-in values keep every product finite.
template <bool FP8>
__device__ __forceinline__ void load_block(BlockRegs<FP8> &r, const void *K, const void *V, size_t tok0, int ts, int valid, int lane)
{
    const int last = valid - 1;
    if (!FP8) {
        const uint16_t *Kg = (const uint16_t *)K + tok0, *Vg = (const uint16_t *)V + tok0;
        // K: chunk c = lane + 64 x is 8 channels (16 B) of row c/8
#pragma unroll
        for (int x = 0; x < 8; ++x) {
            const int c = lane + 64 * x, t = min(c >> 3, last), col = (c & 7) * 8;
            const uint4 w = *(const uint4 *)(Kg + (size_t)t * ts + col);
            r.k[4 * x] = w.x; r.k[4 * x + 1] = w.y; r.k[4 * x + 2] = w.z; r.k[4 * x + 3] = w.w;
        }
        // V: unit u = lane + 64 x is 4 channels (quad u%16) x 8 consecutive tokens (group u/16)
#pragma unroll
        for (int x = 0; x < 2; ++x) {
            const int u = lane + 64 * x, eq = u & 15, tg = u >> 4;
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int t = min(tg * 8 + k, last);
                const uint2 w = *(const uint2 *)(Vg + (size_t)t * ts + 4 * eq);
                r.v[16 * x + 2 * k] = w.x;
                r.v[16 * x + 2 * k + 1] = w.y;
            }
        }
    } else {
        const uint8_t *Kg = (const uint8_t *)K + tok0, *Vg = (const uint8_t *)V + tok0;
        // K: chunk c = lane + 64 x is 16 channels (16 B of e4m3) of row c/4
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const int c = lane + 64 * x, t = min(c >> 2, last), col = (c & 3) * 16;
            const uint4 w = *(const uint4 *)(Kg + (size_t)t * ts + col);
            r.k[4 * x] = w.x; r.k[4 * x + 1] = w.y; r.k[4 * x + 2] = w.z; r.k[4 * x + 3] = w.w;
        }
        // V: unit u = lane + 64 x is 4 channels (quad u%16) x 8 consecutive tokens (group u/16)
#pragma unroll
        for (int x = 0; x < 2; ++x) {
            const int u = lane + 64 * x, eq = u & 15, tg = u >> 4;
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int t = min(tg * 8 + k, last);
                r.v[8 * x + k] = *(const uint32_t *)(Vg + (size_t)t * ts + 4 * eq);
            }
        }
    }
}

__device__ __forceinline__ uint4 e4m3x8_to_bf16x8(uint32_t lo, uint32_t hi)
{
    const f32x2 a0 = __builtin_amdgcn_cvt_pk_f32_fp8(lo, false), a1 = __builtin_amdgcn_cvt_pk_f32_fp8(lo, true);
    const f32x2 a2 = __builtin_amdgcn_cvt_pk_f32_fp8(hi, false), a3 = __builtin_amdgcn_cvt_pk_f32_fp8(hi, true);
    uint4 o;
    o.x = pack_bf16(a0[0], a0[1]); o.y = pack_bf16(a1[0], a1[1]);
    o.z = pack_bf16(a2[0], a2[1]); o.w = pack_bf16(a3[0], a3[1]);
    return o;
}

// Exponent field (1..254) of the largest magnitude among the bf16 values of V a wave holds for one key block.
__device__ __forceinline__ int block_max_exponent(const uint32_t (&v)[32])
{
    uint32_t mx = 0;
#pragma unroll
    for (int x = 0; x < 32; ++x) mx = max(mx, max(v[x] & 0x7FFFu, (v[x] >> 16) & 0x7FFFu));
    for (int o = 32; o > 0; o >>= 1) mx = max(mx, (uint32_t)__shfl_xor((int)mx, o, 64));
    const int e = (int)(mx >> 7);
    return e < 1 ? 1 : (e > 254 ? 254 : e);
}

// four bf16 (two dwords) times 2^sh -> four fp16 (two dwords), round to nearest even where bits are lost
__device__ __forceinline__ uint2 bf16x4_to_f16x4(uint2 w, int sh)
{
    typedef __attribute__((ext_vector_type(2))) _Float16 h2;
    h2 a, b;
    a[0] = (_Float16)ldexpf(bf16_lo(w.x), sh); a[1] = (_Float16)ldexpf(bf16_hi(w.x), sh);
    b[0] = (_Float16)ldexpf(bf16_lo(w.y), sh); b[1] = (_Float16)ldexpf(bf16_hi(w.y), sh);
    return make_uint2(__builtin_bit_cast(uint32_t, a), __builtin_bit_cast(uint32_t, b));
}

// Registers -> LDS: K rows as bf16 (e4m3 codes widened exactly, the block scale is applied later
// in fp32), V transposed to [channel][token] bf16 (e4m3 widened exactly, unscaled).
template <bool FP8>
__device__ __forceinline__ void stage_block(const BlockRegs<FP8> &r, uint16_t *Ks, uint16_t *Vt, int lane)
{
    if (!FP8) {
#pragma unroll
        for (int x = 0; x < 8; ++x) {
            const int c = lane + 64 * x, t = c >> 3, col = (c & 7) * 8;
            *(uint4 *)(Ks + t * kLdsRow + col) = make_uint4(r.k[4 * x], r.k[4 * x + 1], r.k[4 * x + 2], r.k[4 * x + 3]);
        }
#pragma unroll
        for (int x = 0; x < 2; ++x) {
            const int u = lane + 64 * x, eq = u & 15, tg = u >> 4;
            const uint32_t *w = r.v + 16 * x;      // w[2k], w[2k+1]: channels 4eq..4eq+3 of token 8 tg + k
            uint4 c0, c1, c2, c3;                  // channel 4eq + c over the 8 tokens
            c0.x = __builtin_amdgcn_perm(w[2], w[0], 0x05040100);   c1.x = __builtin_amdgcn_perm(w[2], w[0], 0x07060302);
            c2.x = __builtin_amdgcn_perm(w[3], w[1], 0x05040100);   c3.x = __builtin_amdgcn_perm(w[3], w[1], 0x07060302);
            c0.y = __builtin_amdgcn_perm(w[6], w[4], 0x05040100);   c1.y = __builtin_amdgcn_perm(w[6], w[4], 0x07060302);
            c2.y = __builtin_amdgcn_perm(w[7], w[5], 0x05040100);   c3.y = __builtin_amdgcn_perm(w[7], w[5], 0x07060302);
            c0.z = __builtin_amdgcn_perm(w[10], w[8], 0x05040100);  c1.z = __builtin_amdgcn_perm(w[10], w[8], 0x07060302);
            c2.z = __builtin_amdgcn_perm(w[11], w[9], 0x05040100);  c3.z = __builtin_amdgcn_perm(w[11], w[9], 0x07060302);
            c0.w = __builtin_amdgcn_perm(w[14], w[12], 0x05040100); c1.w = __builtin_amdgcn_perm(w[14], w[12], 0x07060302);
            c2.w = __builtin_amdgcn_perm(w[15], w[13], 0x05040100); c3.w = __builtin_amdgcn_perm(w[15], w[13], 0x07060302);
            uint16_t *dst = Vt + (4 * eq) * kLdsRow + tg * 8;
            *(uint4 *)(dst) = c0;
            *(uint4 *)(dst + kLdsRow) = c1;
            *(uint4 *)(dst + 2 * kLdsRow) = c2;
            *(uint4 *)(dst + 3 * kLdsRow) = c3;
        }
    } else {
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const int c = lane + 64 * x, t = c >> 2, col = (c & 3) * 16;
            *(uint4 *)(Ks + t * kLdsRow + col) = e4m3x8_to_bf16x8(r.k[4 * x], r.k[4 * x + 1]);
            *(uint4 *)(Ks + t * kLdsRow + col + 8) = e4m3x8_to_bf16x8(r.k[4 * x + 2], r.k[4 * x + 3]);
        }
#pragma unroll
        for (int x = 0; x < 2; ++x) {
            const int u = lane + 64 * x, eq = u & 15, tg = u >> 4;
            const uint32_t *w = r.v + 8 * x;
#pragma unroll
            for (int ch = 0; ch < 4; ++ch) {
                float f[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const f32x2 p = (ch & 2) ? __builtin_amdgcn_cvt_pk_f32_fp8(w[k], true) : __builtin_amdgcn_cvt_pk_f32_fp8(w[k], false);
                    f[k] = p[ch & 1];
                }
                uint4 o;
                o.x = pack_bf16(f[0], f[1]); o.y = pack_bf16(f[2], f[3]);
                o.z = pack_bf16(f[4], f[5]); o.w = pack_bf16(f[6], f[7]);
                *(uint4 *)(Vt + (4 * eq + ch) * kLdsRow + tg * 8) = o;
            }
        }
    }
}

template <bool FP8>
__global__ __launch_bounds__(64 * kWavesPerWG) __attribute__((amdgpu_waves_per_eu(2, 2))) void states_kernel(const void *__restrict__ K, const void *__restrict__ V,
                                                                  const float *__restrict__ sK, const float *__restrict__ sV,
                                                                  RowMap rm, int N, int Nkb, long nblocks, int per_wave,
                                                                  uint16_t *__restrict__ hT, uint16_t *__restrict__ Vp, float *__restrict__ lvs,
                                                                  double *__restrict__ kbar, int phi, unsigned state_wgs,
                                                                  const uint16_t *__restrict__ W, uint16_t *__restrict__ WT)
{
    asm volatile("" ::"s"(K), "s"(V), "s"(sK), "s"(sV), "s"(rm.bs), "s"(rm.hs), "s"(rm.ts), "s"(rm.H), "s"(N), "s"(Nkb), "s"(nblocks), "s"(per_wave), "s"(hT), "s"(Vp), "s"(lvs), "s"(kbar), "s"(phi), "s"(state_wgs), "s"(W), "s"(WT));      // all kernel arguments in one batch of scalar loads, here
    if (blockIdx.x >= state_wgs) {     // workgroups past the states grid each lay out one projection matrix for the attention kernel
        const size_t m = (size_t)(blockIdx.x - state_wgs) * kD * kD;
        transpose_w_tile(W + m, WT + m, 64 * kWavesPerWG);
        return;
    }
    __shared__ __attribute__((aligned(16))) uint16_t lds[kWavesPerWG][2][64 * kLdsRow];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const long first = ((long)blockIdx.x * kWavesPerWG + wave) * per_wave;
    const long last = min(first + per_wave, nblocks);          // this wave owns blocks [first, last)
    if (first >= last) return;                                  // whole wave exits together; no workgroup barrier below
    uint16_t *Ks = lds[wave][0];                     // K rows, later phi^T [d][t]
    uint16_t *Vt = lds[wave][1];                     // V^T [e][t]
    const int l32 = lane & 31, g = lane >> 5;

    auto block_geometry = [&](long blk, size_t &tok0, int &valid) {
        const long bh = blk / Nkb;
        const int t0 = (int)(blk - bh * Nkb) * kBK;
        valid = min(kBK, N - t0);
        tok0 = rm.head(bh) + (size_t)t0 * rm.ts;
    };

    BlockRegs<FP8> regs;
    {
        size_t tok0; int valid;
        block_geometry(first, tok0, valid);
        load_block<FP8>(regs, K, V, tok0, rm.ts, valid, lane);
    }
    for (long blk = first; blk < last; ++blk) {
        size_t tok0; int valid;
        block_geometry(blk, tok0, valid);
        wave_lds_sync();                             // the previous block's LDS reads are done
        stage_block<FP8>(regs, Ks, Vt, lane);
        int vexp = 127;                              // bf16: exponent field of the block's largest |V| (127 = 2^0)
        if constexpr (!FP8) { if (Vp != nullptr) vexp = block_max_exponent(regs.v); }
        if (blk + 1 < last) {                        // next block's loads fly while this one is processed
            size_t tn; int vn;
            block_geometry(blk + 1, tn, vn);
            load_block<FP8>(regs, K, V, tn, rm.ts, vn, lane);
        }
        wave_lds_sync();

        // ---- block mean of K for the classifier: lane d adds the tokens of channel d serially in fp64
        // (ascending token order) and multiplies by 1/count -- the same arithmetic as the pooling kernel
        if (kbar != nullptr) {
            const double s = FP8 ? (double)sK[blk] : 1.0;
            double acc = 0.0;
#pragma unroll 8
            for (int t = 0; t < valid; ++t) {
                const double v = (double)bf16_bits_to_f32(Ks[t * kLdsRow + lane]);
                acc += FP8 ? v * s : v;
            }
            kbar[blk * kD + lane] = acc * (1.0 / (double)valid);
        }

        // ---- phi: lane t owns token row t
        float x[64];
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const uint4 w = *(const uint4 *)(Ks + lane * kLdsRow + c * 8);
            x[c * 8 + 0] = bf16_lo(w.x); x[c * 8 + 1] = bf16_hi(w.x);
            x[c * 8 + 2] = bf16_lo(w.y); x[c * 8 + 3] = bf16_hi(w.y);
            x[c * 8 + 4] = bf16_lo(w.z); x[c * 8 + 5] = bf16_hi(w.z);
            x[c * 8 + 6] = bf16_lo(w.w); x[c * 8 + 7] = bf16_hi(w.w);
        }
        // phi = 0: softmax over the 64 channels; phi = 1: ELU(x)+1 elementwise (x+1 above 0, exp(x) below).
        // s is 1 for bf16 inputs and the K block scale for e4m3.
        const float cexp = (FP8 ? sK[blk] : 1.0f) * 1.4426950408889634f;
        float inv;
        if (phi == 0) {
            float mx = x[0];
#pragma unroll
            for (int d = 1; d < 64; ++d) mx = fmaxf(mx, x[d]);
            // exp(s*(x - mx)) = exp2(x*c - mx*c), c = s*log2(e)
            const float mc = mx * cexp;
            float sum = 0.f;
#pragma unroll
            for (int d = 0; d < 64; ++d) { x[d] = fast_exp2(fmaf(x[d], cexp, -mc)); sum += x[d]; }
            inv = lane < valid ? 1.0f / sum : 0.0f;             // rows past the sequence end contribute nothing
        } else {
            const float sc = FP8 ? sK[blk] : 1.0f;
#pragma unroll
            for (int d = 0; d < 64; ++d) x[d] = x[d] > 0.f ? fmaf(x[d], sc, 1.0f) : fast_exp2(x[d] * cexp);
            inv = lane < valid ? 1.0f : 0.0f;
        }
        wave_lds_sync();                                        // all rows are in registers: Ks may be overwritten
#pragma unroll
        for (int d = 0; d < 64; ++d) Ks[d * kLdsRow + lane] = (uint16_t)(pack_bf16(x[d] * inv, 0.f) & 0xFFFFu);
        wave_lds_sync();

        // ---- V^T tile for the attention kernel: Vp[e][.] with the 2nd and 3rd group of 4 tokens of every
        // 16 swapped (slot 16s + 8g + 4a + b holds token 16s + 8a + 4g + b), which is the key order the
        // accumulator-as-operand trick of that kernel needs.  fp16: bf16 V divided by 2^(vexp - 127), e4m3 codes as they are.
        if (Vp != nullptr) {
            uint16_t *vt = Vp + (size_t)blk * kD * kBK;
            const int c = lane & 7, src = 16 * (c >> 1) + 4 * (c & 1);   // 16-byte piece c of a row: tokens src..src+3, src+8..src+11
#pragma unroll
            for (int x = 0; x < 8; ++x) {                                // a wave-wide store covers 8 whole rows (1 KB)
                const int e = 8 * x + (lane >> 3);
                const uint2 lo = bf16x4_to_f16x4(*(const uint2 *)(Vt + e * kLdsRow + src), 127 - vexp);
                const uint2 hi = bf16x4_to_f16x4(*(const uint2 *)(Vt + e * kLdsRow + src + 8), 127 - vexp);
                *(uint4 *)(vt + e * kBK + 8 * c) = make_uint4(lo.x, lo.y, hi.x, hi.y);
            }
            if (lane == 0) lvs[blk] = FP8 ? __log2f(fmaxf(sV[blk], 1e-30f)) : (float)(vexp - 127);
        }

        // ---- z: lane d sums phi^T row d (the bf16 values the product below consumes)
        float z = 0.f;
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const uint4 w = *(const uint4 *)(Ks + lane * kLdsRow + c * 8);
            z += bf16_lo(w.x) + bf16_hi(w.x) + bf16_lo(w.y) + bf16_hi(w.y) + bf16_lo(w.z) + bf16_hi(w.z) + bf16_lo(w.w) + bf16_hi(w.w);
        }

        // ---- h[d][e] = sum_t phi^T[d][t] * V^T[e][t]
        f32x16 zero16;
#pragma unroll
        for (int i = 0; i < 16; ++i) zero16[i] = 0.f;
        f32x16 acc[2][2];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            bf16x8 af[2], bfr[2];
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                af[a] = *(const bf16x8 *)(Ks + (32 * a + l32) * kLdsRow + 16 * s + 8 * g);
                bfr[a] = *(const bf16x8 *)(Vt + (32 * a + l32) * kLdsRow + 16 * s + 8 * g);
            }
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a], bfr[b], s == 0 ? zero16 : acc[a][b], 0, 0, 0);
        }

        // ---- write hT[e][d]: accumulator (a,b) register 4q+r holds d = 32a + 8q + 4g + r, e = 32b + l32.
        // The tile goes through LDS (phi^T is consumed) so that it leaves as whole rows, 1 KB per wave-wide store.
        uint16_t *out = hT + (size_t)blk * kStateElems;
        const float vs = FP8 ? sV[blk] : 1.0f;
        wave_lds_sync();                                        // the operand reads of phi^T are done
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    uint2 o;
                    o.x = pack_bf16(acc[a][b][4 * q + 0] * vs, acc[a][b][4 * q + 1] * vs);
                    o.y = pack_bf16(acc[a][b][4 * q + 2] * vs, acc[a][b][4 * q + 3] * vs);
                    *(uint2 *)(Ks + (32 * b + l32) * kLdsRow + 32 * a + 8 * q + 4 * g) = o;
                }
        wave_lds_sync();
#pragma unroll
        for (int x = 0; x < 8; ++x) {
            const int e = 8 * x + (lane >> 3), c = lane & 7;
            *(uint4 *)(out + e * kD + 8 * c) = *(const uint4 *)(Ks + e * kLdsRow + 8 * c);
        }
        out[64 * kD + lane] = (uint16_t)(pack_bf16(z, 0.f) & 0xFFFFu);
    }
}

hipError_t launch_states(const void *K, const void *V, const float *sK, const float *sV, bool fp8, RowMap rm,
                         int BH, int N, void *hT, void *Vp, float *lvs, double *kbar, int phi, const void *W, int nW, void *WT, hipStream_t st)
{
    const int Nkb = (N + kBK - 1) / kBK;
    const long nblocks = (long)BH * Nkb;
    // enough waves to fill the chip (256 CUs x 8 resident waves), each with a contiguous run of blocks
    const long target_waves = 256L * 8;
    const int per_wave = (int)((nblocks + target_waves - 1) / target_waves);
    const long waves = (nblocks + per_wave - 1) / per_wave;
    const unsigned grid = (unsigned)((waves + kWavesPerWG - 1) / kWavesPerWG);
    const unsigned extra = W != nullptr ? (unsigned)nW : 0u;
    if (fp8) states_kernel<true><<<grid + extra, 64 * kWavesPerWG, 0, st>>>(K, V, sK, sV, rm, N, Nkb, nblocks, per_wave, (uint16_t *)hT, (uint16_t *)Vp, lvs, kbar, phi, grid, (const uint16_t *)W, (uint16_t *)WT);
    else     states_kernel<false><<<grid + extra, 64 * kWavesPerWG, 0, st>>>(K, V, sK, sV, rm, N, Nkb, nblocks, per_wave, (uint16_t *)hT, (uint16_t *)Vp, lvs, kbar, phi, grid, (const uint16_t *)W, (uint16_t *)WT);
    return hipGetLastError();
}

}  // namespace sla
