// Forward of the FP8 fake-quantised linear layer (Alg. 2 of the paper, with the scaled quantiser of App. B.2/B.3):
//     x_fp8 = E4M3(clamp(x / s_x, +-448)) * s_x   per token,          s_x = max(amax(x_i), 1e-8) / 448
//     W_fp8 = E4M3(clamp(W / s_W, +-448)) * s_W   per output channel, s_W likewise
//     y = x_fp8 W_fp8^T + b
// Two kernels.  quantise_rows_kernel turns a bf16 matrix into E4M3 codes plus one fp32 scale per row (one wavefront
// per row, two passes over the row: absolute maximum, then divide / clamp / convert; bit for bit the arithmetic of
// the block quantiser).  fp8_gemm_kernel multiplies the code matrices on v_mfma_f32_32x32x64_f8f6f4 (products of
// two E4M3 numbers are exact in the fp32 accumulator) and applies s_x[i] s_W[o] and the bias in its epilogue.
//
// GEMM tiling: workgroup tile 128 or 256 tokens x 128 output channels, 4 waves as 2 x 2, K step 128 bytes (two
// MFMA K steps).  Both operands are K-contiguous in memory, so their tiles go to LDS as 16-byte chunks of 128-byte
// rows (chunk index XOR-ed with row bits against bank conflicts) and an MFMA operand is two 16-byte reads.  The
// kernel forms the transposed tile D[o][i] (W rows as the A operand), so that a lane's four consecutive accumulator
// registers are four consecutive output channels of one token and leave through LDS as 16-byte stores.  Global
// loads run two K steps ahead of their use in registers, LDS is double buffered with an LDS-only barrier.
// Problems with many tiles take fp8_gemm_big_kernel instead (256 x 256 tiles, described at the kernel).
#include "sla_common.hpp"
#include "sla_kernels.hpp"

#include <type_traits>

namespace sla {

__global__ __launch_bounds__(256) void quantise_rows_kernel(const uint16_t *__restrict__ X, long rows, int cols,
                                                            uint8_t *__restrict__ codes, float *__restrict__ scales)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const long row = (long)blockIdx.x * 4 + wave;
    if (row >= rows) return;                         // the whole wave leaves; nothing below synchronises across waves
    const uint16_t *x = X + row * cols;
    float amax = 0.f;
    for (int c = lane * 8; c < cols; c += 512) {     // cols is a multiple of 8: whole 16-byte pieces
        const uint4 v = *(const uint4 *)(x + c);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int q = 0; q < 4; ++q) amax = fmaxf(amax, fmaxf(fabsf(bf16_lo(w[q])), fabsf(bf16_hi(w[q]))));
    }
    amax = wave_max(amax);
    const float scale = fmaxf(amax, 1e-8f) / 448.0f;
    if (lane == 0) scales[row] = scale;
    uint8_t *out = codes + row * cols;
    for (int c = lane * 8; c < cols; c += 512) {
        const uint4 v = *(const uint4 *)(x + c);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
        float y[8];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            y[2 * q] = fminf(fmaxf(bf16_lo(w[q]) / scale, -448.0f), 448.0f);
            y[2 * q + 1] = fminf(fmaxf(bf16_hi(w[q]) / scale, -448.0f), 448.0f);
        }
        int lo = 0, hi = 0;
        lo = __builtin_amdgcn_cvt_pk_fp8_f32(y[0], y[1], lo, false);
        lo = __builtin_amdgcn_cvt_pk_fp8_f32(y[2], y[3], lo, true);
        hi = __builtin_amdgcn_cvt_pk_fp8_f32(y[4], y[5], hi, false);
        hi = __builtin_amdgcn_cvt_pk_fp8_f32(y[6], y[7], hi, true);
        *(uint2 *)(out + c) = make_uint2((uint32_t)lo, (uint32_t)hi);
    }
}

namespace {
constexpr int kLinK = 128;                           // bytes (= E4M3 elements) of K per step
constexpr int kLinOutRow = 128 + 8;                  // bf16 per row of the output staging tile
__device__ __forceinline__ int lin_swz(int row) { return (row >> 1) & 7; }
}  // namespace

// Y[i][o] = (sum_k A8[i][k] W8[o][k]) * sa[i] * sw[o] + bias[o];  A8 [M,K], W8 [O,K] E4M3 codes, K a multiple of 128.
// TB: 32-token sub-tiles per wave.  TB = 2: tile 128 tokens x 128 channels, LDS double buffered (one barrier per K
// step).  TB = 4: tile 256 tokens x 128 channels for large token counts -- a wave's 64 x 128 tile needs six operand
// reads per eight MFMAs instead of four per four, which takes the LDS read rate off the critical path; one LDS buffer
// (two barriers per K step) so that two workgroups still share a CU.
//
// QKV: the layer is the qkv projection in front of the attention (O = 3 H 64 output channels ordered [q|k|v][head][64])
// and the epilogue, instead of storing y, quantises it per (head, token block) with the scaled E4M3 quantiser of
// App. B.2 -- the form sla_forward takes E4M3 inputs in -- and stores codes [B,N,H,64] and scales [B,H,blocks] of Q, K
// and V directly: the bf16 tile staged in LDS is the y the unfused layer would have written, a wavefront takes one
// (token block, head) of it at a time (absolute maximum by a wave reduction, then divide / clamp / convert: the
// arithmetic of quantise_e4m3_kernel), so the result is bit for bit that of sla_fp8_linear followed by
// sla_quantise_e4m3, without y's round trip through HBM.  Token blocks never straddle a tile (the host checks).
// x / d for many x and one d, with the bits of the IEEE division: y = RN(1 / d) once (a true division), then
// q = RN(x y), r = x - d q (exact in one fma), RN(q + r y) is the correctly rounded quotient (Markstein's division
// step; it needs y correctly rounded and fails only for a significand of d of all ones, which takes the division).
// Quotients here are at most 448 in magnitude and anything below 2^-10 becomes the code 0, so the exponent range
// plays no part.  Three instructions per element instead of the ten of the division's expansion.
struct BlockDivisor {
    float d, y;
    bool plain;
    __device__ __forceinline__ explicit BlockDivisor(float d_) : d(d_), y(1.0f / d_), plain((__float_as_uint(d_) & 0x7FFFFFu) == 0x7FFFFFu) {}
    __device__ __forceinline__ float operator()(float x) const
    {
        if (plain) return x / d;
        const float q = x * y;
        return fmaf(fmaf(-q, d, x), y, q);
    }
};

struct QkvOut {
    uint8_t *codes[3];          // Q, K, V codes, [B,N,H,64]
    float *scales[3];           // [B,H,ceil(N/blk)], blk = bq for Q, 64 for K and V
    int N, H, bq;
};

template <int TB, bool QKV>
__global__ __launch_bounds__(256) void fp8_gemm_kernel(const uint8_t *__restrict__ A8, const float *__restrict__ sa,
                                                       const uint8_t *__restrict__ W8, const float *__restrict__ sw,
                                                       const uint16_t *__restrict__ bias, int M, int O, int K, int n_it,
                                                       long total, uint16_t *__restrict__ Y, QkvOut qkv)
{
    asm volatile("" ::"s"(A8), "s"(sa), "s"(W8), "s"(sw), "s"(bias), "s"(M), "s"(O), "s"(K), "s"(n_it), "s"(total), "s"(Y), "s"(qkv.codes[0]), "s"(qkv.codes[1]), "s"(qkv.codes[2]),
                 "s"(qkv.scales[0]), "s"(qkv.scales[1]), "s"(qkv.scales[2]), "s"(qkv.N), "s"(qkv.H), "s"(qkv.bq));      // all kernel arguments in one batch of scalar loads, here
    constexpr int kTok = 64 * TB;                                                // tokens per workgroup tile
    constexpr int kBufs = TB == 2 ? 2 : 1;
    constexpr int kBufBytes = (kTok + 128) * kLinK;                              // token tile, then channel tile
    constexpr int kStageBytes = kTok * kLinOutRow * 2;
    constexpr int kSmem = kBufs * kBufBytes > kStageBytes ? kBufs * kBufBytes : kStageBytes;
    constexpr int kAx = 2 * TB;                                                  // 16-byte chunks of the token tile per thread
    __shared__ __attribute__((aligned(16))) uint8_t smem[kSmem];
    // channel tile fastest: the workgroups that share a token tile run side by side on one XCD, so the activations come
    // from HBM once; the weight matrix (a few MB) stays in every XCD's L2
    const long item = xcd_remap(blockIdx.x, total);
    if (item >= total) return;
    const int n_ot = (int)(total / n_it);
    const int ot = (int)(item % n_ot), it = (int)(item / n_ot);
    const int i0 = it * kTok, o0 = ot * 128;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, g = lane >> 5;
    const int wo = (wave >> 1) * 64, wi = (wave & 1) * (32 * TB);                // wave's first channel / token within the tile

    // loader: 16-byte chunk id = tid + 256 x of a tile of 128-byte rows: row id / 8, chunk id % 8 (rows past the end of
    // the matrix repeat its last row: their results are never stored)
    uint32_t ga[kAx], gw[4];                       // byte offsets into A8 / W8 (the host checks that both stay below 4 GB)
    int la[kAx], lw[4];
#pragma unroll
    for (int x = 0; x < kAx; ++x) {
        const int id = tid + 256 * x, row = id >> 3, ch = id & 7;
        ga[x] = (uint32_t)min(i0 + row, M - 1) * (uint32_t)K + ch * 16;
        la[x] = row * kLinK + ((ch ^ lin_swz(row)) << 4);
    }
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        const int id = tid + 256 * x, row = id >> 3, ch = id & 7;
        gw[x] = (uint32_t)min(o0 + row, O - 1) * (uint32_t)K + ch * 16;
        lw[x] = kTok * kLinK + row * kLinK + ((ch ^ lin_swz(row)) << 4);
    }
    uint32_t ra[kBufs][4 * kAx], rw[kBufs][16];                                  // register sets (plain dwords)
    auto load_tile = [&](int ks, uint32_t (&a)[4 * kAx], uint32_t (&w)[16]) {
#pragma unroll
        for (int x = 0; x < kAx; ++x) {
            const uint4 v = *(const uint4 *)(A8 + ga[x] + (uint32_t)ks * kLinK);
            a[4 * x] = v.x; a[4 * x + 1] = v.y; a[4 * x + 2] = v.z; a[4 * x + 3] = v.w;
        }
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const uint4 v = *(const uint4 *)(W8 + gw[x] + (uint32_t)ks * kLinK);
            w[4 * x] = v.x; w[4 * x + 1] = v.y; w[4 * x + 2] = v.z; w[4 * x + 3] = v.w;
        }
    };
    auto store_tile = [&](uint8_t *buf, const uint32_t (&a)[4 * kAx], const uint32_t (&w)[16]) {
#pragma unroll
        for (int x = 0; x < kAx; ++x) *(uint4 *)(buf + la[x]) = make_uint4(a[4 * x], a[4 * x + 1], a[4 * x + 2], a[4 * x + 3]);
#pragma unroll
        for (int x = 0; x < 4; ++x) *(uint4 *)(buf + lw[x]) = make_uint4(w[4 * x], w[4 * x + 1], w[4 * x + 2], w[4 * x + 3]);
    };
    // operand of one MFMA: 32 bytes of K (bytes 64 s + 32 g ..) of row `row` of the tile at `tile`
    auto frag = [&](const uint8_t *tile, int row, int s) {
        const int c0 = 4 * s + 2 * g;
        const uint4 u0 = *(const uint4 *)(tile + row * kLinK + ((c0 ^ lin_swz(row)) << 4));
        const uint4 u1 = *(const uint4 *)(tile + row * kLinK + (((c0 + 1) ^ lin_swz(row)) << 4));
        i32x8 f;
        f[0] = u0.x; f[1] = u0.y; f[2] = u0.z; f[3] = u0.w; f[4] = u1.x; f[5] = u1.y; f[6] = u1.z; f[7] = u1.w;
        return f;
    };

    f32x16 acc[2][TB];                                                          // [channel sub-tile][token sub-tile]
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < TB; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.f;
    auto mma_step = [&](const uint8_t *buf) {
        const uint8_t *At = buf, *Wt = buf + kTok * kLinK;
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            i32x8 wf[2], af[TB];
#pragma unroll
            for (int a = 0; a < 2; ++a) wf[a] = frag(Wt, wo + 32 * a + l32, s);
#pragma unroll
            for (int b = 0; b < TB; ++b) af[b] = frag(At, wi + 32 * b + l32, s);
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < TB; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(wf[a], af[b], acc[a][b], 0, 0, 0, 0, 0, 0);
        }
    };

    const int ksteps = K / kLinK;
    if constexpr (kBufs == 2) {
        load_tile(0, ra[0], rw[0]);
        load_tile(min(1, ksteps - 1), ra[1], rw[1]);
        store_tile(smem, ra[0], rw[0]);
        lds_barrier();
        for (int ks0 = 0; ks0 < ksteps; ks0 += 2) {
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int ks = ks0 + u;
                if (ks < ksteps) {                                              // uniform over the workgroup
                    load_tile(min(ks + 2, ksteps - 1), ra[u], rw[u]);           // set u went to LDS one step ago; past the end: a repeat nobody uses
                    mma_step(smem + (ks & 1) * kBufBytes);
                    store_tile(smem + ((ks + 1) & 1) * kBufBytes, ra[(u + 1) & 1], rw[(u + 1) & 1]);
                    lds_barrier();
                }
            }
        }
    } else {
        load_tile(0, ra[0], rw[0]);
        for (int ks = 0; ks < ksteps; ++ks) {
            store_tile(smem, ra[0], rw[0]);
            lds_barrier();                                                      // tile ks is in LDS
            load_tile(min(ks + 1, ksteps - 1), ra[0], rw[0]);                   // the next one flies during the products
            mma_step(smem);
            lds_barrier();                                                      // every wave has read tile ks
        }
    }

    // accumulator (a,b) register 4q+r of lane (l32, g): channel o0 + wo + 32a + 8q + 4g + r, token i0 + wi + 32b + l32.
    // Scales and bias applied in fp32, staged as [token][channel], stored as 16-byte pieces.
    uint16_t *stage = (uint16_t *)smem;
#pragma unroll
    for (int b = 0; b < TB; ++b) {
        const int i = i0 + wi + 32 * b + l32;
        const float si = sa[min(i, M - 1)];
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int o = o0 + wo + 32 * a + 8 * q + 4 * g;
                float v[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int oc = min(o + r, O - 1);
                    v[r] = acc[a][b][4 * q + r] * (si * sw[oc]) + (bias ? bf16_bits_to_f32(bias[oc]) : 0.f);
                }
                uint2 p;
                p.x = pack_bf16(v[0], v[1]);
                p.y = pack_bf16(v[2], v[3]);
                *(uint2 *)(stage + (wi + 32 * b + l32) * kLinOutRow + wo + 32 * a + 8 * q + 4 * g) = p;
            }
    }
    __syncthreads();
    if constexpr (!QKV) {
#pragma unroll
        for (int t = 0; t < kTok / 16; ++t) {
            const int idx = tid + 256 * t, r = idx >> 4, seg = idx & 15;
            if (i0 + r < M && o0 + 8 * seg < O)                                  // O is a multiple of 8: a segment is in or out as a whole
                *(uint4 *)(Y + (size_t)(i0 + r) * O + o0 + 8 * seg) = *(const uint4 *)(stage + r * kLinOutRow + 8 * seg);
        }
    } else {
        // units of the tile: (64-channel half = one head of q, k or v) x (token block of that tensor); one wave per unit
        const int N = qkv.N, H = qkv.H, rr = lane >> 3, cc = lane & 7;
        for (int hf = 0; hf < 2; ++hf) {
            const int ch0 = o0 + 64 * hf;
            if (ch0 >= O) break;
            const int which = ch0 / (H * 64), h = (ch0 - which * H * 64) >> 6;
            const int blk = which == 0 ? qkv.bq : kBK, nblk_seq = (N + blk - 1) / blk;
            for (int tb = wave; tb * blk < kTok; tb += 4) {
                const int t0 = i0 + tb * blk;
                if (t0 >= M) break;                                              // uniform over the wave
                const int b = t0 / N, tin = t0 - b * N, valid = min(blk, N - tin);
                const uint16_t *src = stage + (tb * blk) * kLinOutRow + 64 * hf + 8 * cc;
                float amax = 0.f;
                for (int r = rr; r < valid; r += 8) {
                    const uint4 v = *(const uint4 *)(src + r * kLinOutRow);
                    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                    for (int q = 0; q < 4; ++q) amax = fmaxf(amax, fmaxf(fabsf(bf16_lo(w[q])), fabsf(bf16_hi(w[q]))));
                }
                amax = wave_max(amax);
                const float scale = fmaxf(amax, 1e-8f) / 448.0f;
                const BlockDivisor by_scale(scale);
                if (lane == 0) qkv.scales[which][((size_t)b * H + h) * nblk_seq + tin / blk] = scale;
                uint8_t *dst = qkv.codes[which] + (((size_t)b * N + tin) * H + h) * 64 + 8 * cc;
                for (int r = rr; r < valid; r += 8) {
                    const uint4 v = *(const uint4 *)(src + r * kLinOutRow);
                    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
                    float y[8];
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        y[2 * q] = fminf(fmaxf(by_scale(bf16_lo(w[q])), -448.0f), 448.0f);
                        y[2 * q + 1] = fminf(fmaxf(by_scale(bf16_hi(w[q])), -448.0f), 448.0f);
                    }
                    int lo = 0, hi = 0;
                    lo = __builtin_amdgcn_cvt_pk_fp8_f32(y[0], y[1], lo, false);
                    lo = __builtin_amdgcn_cvt_pk_fp8_f32(y[2], y[3], lo, true);
                    hi = __builtin_amdgcn_cvt_pk_fp8_f32(y[4], y[5], hi, false);
                    hi = __builtin_amdgcn_cvt_pk_fp8_f32(y[6], y[7], hi, true);
                    *(uint2 *)(dst + (size_t)r * H * 64) = make_uint2((uint32_t)lo, (uint32_t)hi);
                }
            }
        }
    }
}

hipError_t launch_quantise_rows(const void *X, long rows, int cols, void *codes, float *scales, hipStream_t st)
{
    quantise_rows_kernel<<<(unsigned)((rows + 3) / 4), 256, 0, st>>>((const uint16_t *)X, rows, cols, (uint8_t *)codes, scales);
    return hipGetLastError();
}

// The same product on 256 tokens x 256 channels per workgroup, for problems with enough of those tiles: four waves as
// 2 x 2, a wave's tile is 128 channels x 128 tokens = 4 x 4 MFMA tiles (256 accumulator registers, one wave per SIMD).
// Eight operand fragments feed sixteen MFMAs, so the LDS read rate (the limit of the smaller tiles: twelve fragment
// reads per sixteen MFMAs on each of four waves is three quarters of the LDS bandwidth) drops to half of it.  Tiles go
// from global memory straight into LDS (global_load_lds_dwordx4: 1 KB per wave instruction, the chunk swizzle applied on
// the global side), two stages of 64 KB, the copies two K steps ahead of the products, one barrier per step (the
// schedule is written out at the loop).  The copies are inline assembly, invisible to the compiler's wait counting; the wait is explicit.
// Epilogue: scales and bias in fp32, each wave stages its [token][channel] tile in its own quarter of LDS (16-byte
// chunks XOR-ed with the token row against bank conflicts) and stores 16 bytes per lane, 256 contiguous bytes per row.
#ifdef SLA_PROBE_TIME   /* timing probe only: cycle counter of one wave at the phase boundaries of its tile */
__device__ unsigned long long sla_gemm_probe_times[16];
#define SLA_GT(pt) do { if (gprobe) { const unsigned long long t_ = __builtin_readcyclecounter(), r_ = __builtin_amdgcn_s_memrealtime(); if ((threadIdx.x & 63) == 0) { sla_gemm_probe_times[pt] = t_; sla_gemm_probe_times[8 + pt] = r_; } } } while (0)
#else
#define SLA_GT(pt)
#endif
template <bool QKV>
__global__ __launch_bounds__(256, 1) void fp8_gemm_big_kernel(const uint8_t *__restrict__ A8, const float *__restrict__ sa,
                                                              const uint8_t *__restrict__ W8, const float *__restrict__ sw,
                                                              const uint16_t *__restrict__ bias, int M, int O, int K, int n_it,
                                                              long total, uint16_t *__restrict__ Y, QkvOut qkv)
{
    asm volatile("" ::"s"(A8), "s"(sa), "s"(W8), "s"(sw), "s"(bias), "s"(M), "s"(O), "s"(K), "s"(n_it), "s"(total), "s"(Y), "s"(qkv.codes[0]), "s"(qkv.codes[1]), "s"(qkv.codes[2]),
                 "s"(qkv.scales[0]), "s"(qkv.scales[1]), "s"(qkv.scales[2]), "s"(qkv.N), "s"(qkv.H), "s"(qkv.bq));      // all kernel arguments in one batch of scalar loads, here
    constexpr int kStage = 2 * 256 * kLinK;                                      // bytes of one stage: A tile + W tile
    __shared__ __attribute__((aligned(1024))) uint8_t smem[2 * kStage + 2048];   // behind the stages: the tile's 256 channel scales and biases
    const long item = xcd_remap(blockIdx.x, total);
    if (item >= total) return;
#ifdef SLA_PROBE_TIME
    const bool gprobe = __builtin_amdgcn_readfirstlane((int)(item == total / 2 + 5 && threadIdx.x < 64)) != 0;
#endif
    SLA_GT(0);
    const int n_ot = (int)(total / n_it);
    const int ot = (int)(item % n_ot), it = (int)(item / n_ot);                  // channel tile fastest (see above)
    const int i0 = it * 256, o0 = ot * 256;
    {   // thread t brings channel o0 + t's scale and bias; published by the first barrier, read in the epilogue
        const int oc = min(o0 + (int)threadIdx.x, O - 1);
        float *cs = (float *)(smem + 2 * kStage);
        cs[threadIdx.x] = sw[oc];
        cs[256 + threadIdx.x] = bias ? bf16_bits_to_f32(bias[oc]) : 0.f;
    }
    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);                  // uniform: LDS destinations of the copies sit in scalar registers
    const int wo = (wave >> 1) * 128, wi = (wave & 1) * 128;                     // wave's first channel / token within the tile

    // copies: wave w brings rows 64 w .. 64 w + 63 of both tiles, 8 rows (1 KB) per instruction; lane l lands at
    // row 8 x + l / 8, chunk position l % 8, and fetches the chunk that belongs there (rows past the end of a matrix
    // repeat its last row: their results are never stored)
    uint32_t va[8], vw[8];
#pragma unroll
    for (int x = 0; x < 8; ++x) {
        const int row = 64 * wave + 8 * x + (lane >> 3), ch = (lane & 7) ^ lin_swz(row);
        va[x] = (uint32_t)min(i0 + row, M - 1) * (uint32_t)K + ch * 16;
        vw[x] = (uint32_t)min(o0 + row, O - 1) * (uint32_t)K + ch * 16;
    }
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void *)smem;
    auto issue = [&](int ks, int stage) {
        const uint32_t dst = lds_base + stage * kStage + wave * 8192;
#pragma unroll
        for (int x = 0; x < 8; ++x) {
            copy_1k_to_lds(A8 + (size_t)ks * kLinK, va[x], dst + x * 1024);
            copy_1k_to_lds(W8 + (size_t)ks * kLinK, vw[x], dst + 256 * kLinK + x * 1024);
        }
    };
    auto frag = [&](const uint8_t *tile, int row, int s) {
        const int c0 = 4 * s + 2 * g;
        const uint4 u0 = *(const uint4 *)(tile + row * kLinK + ((c0 ^ lin_swz(row)) << 4));
        const uint4 u1 = *(const uint4 *)(tile + row * kLinK + (((c0 + 1) ^ lin_swz(row)) << 4));
        i32x8 f;
        f[0] = u0.x; f[1] = u0.y; f[2] = u0.z; f[3] = u0.w; f[4] = u1.x; f[5] = u1.y; f[6] = u1.z; f[7] = u1.w;
        return f;
    };

    f32x16 acc[4][4];                                                           // [channel sub-tile][token sub-tile]
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.f;

    // Schedule of one K step ks (stage st = ks & 1; a step is two 64-byte slices s0, s1, sixteen MFMAs each):
    //     MFMAs of (ks, s0), the reads of the fragments of (ks, s1) slipped in after the first eight
    //     wait: copies of step ks+1 landed (issued a whole step ago), own reads returned; barrier
    //     MFMAs of (ks, s1); slipped in: the reads of the fragments of (ks+1, s0) after the first eight, one copy of
    //     step ks+2 (into stage st, which every wave has finished reading) after each of the sixteen
    // so the wave keeps the matrix unit's queue filled except at the barrier: every LDS read has at least eight MFMAs
    // (five hundred cycles) to arrive in, the copies run two steps ahead on two stages, one barrier per step.
    const int ksteps = K / kLinK;
    // Workgroups that share an operand tile run at the same time and would ask the same L2 channels for the same lines
    // at the same moment; each starts its K loop at a different step instead (measured: 9 % faster).  The sum over K is
    // then taken in a rotated order: same products, fp32 rounding in a different order than the smaller tiles take.
    const int rot = (int)(item % ksteps);
#define KS_(k) (((k) + rot) % ksteps)
    i32x8 wf0[4], af0[4], wf1[4], af1[4];
    auto read_one = [&](i32x8 (&wf)[4], i32x8 (&af)[4], int stage, int sl, int idx) {     // fragment idx of 8: 0..3 W, 4..7 A
        const uint8_t *At = smem + stage * kStage, *Wt = At + 256 * kLinK;
        if (idx < 4) wf[idx] = frag(Wt, wo + 32 * idx + l32, sl);
        else af[idx - 4] = frag(At, wi + 32 * (idx - 4) + l32, sl);
    };
    auto copy_one = [&](const uint8_t *An, const uint8_t *Wn, uint32_t dst0, int idx) {   // copy idx of 16 of a step: even A, odd W
        const uint32_t dst = dst0 + (idx >> 1) * 1024;
        if (idx & 1) copy_1k_to_lds(Wn, vw[idx >> 1], dst + 256 * kLinK);
        else copy_1k_to_lds(An, va[idx >> 1], dst);
    };
#define SLA_SB() __builtin_amdgcn_sched_barrier(0)
    issue(KS_(0), 0);
    if (ksteps > 1) issue(KS_(1), 1);
    if (ksteps > 1) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");           // the sixteen copies of step 0 (those of step 1 may fly on)
    else            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    SLA_GT(1);
#ifdef SLA_PROBE_TIME
    unsigned long long wait_copy_ = 0, wait_bar_ = 0;
#endif
#pragma unroll
    for (int f = 0; f < 8; ++f) read_one(wf0, af0, 0, 0, f);
    // k2: the K slice that step ks+2 works on (kept by increment: a division per copy would cost more than the MFMA
    // the copy hides behind)
    int k2 = KS_(2 % ksteps);
    for (int ks = 0; ks < ksteps; ++ks) {
        const bool more1 = ks + 1 < ksteps, more2 = ks + 2 < ksteps;
        const int st = ks & 1;
        const uint8_t *An = A8 + (size_t)k2 * kLinK, *Wn = W8 + (size_t)k2 * kLinK;
        const uint32_t dst0 = lds_base + st * kStage + wave * 8192;
        // F0 was requested at least eight MFMAs ago: say here that it has arrived, so that the wait the compiler puts in
        // front of its first use does not cover the reads that follow
        __builtin_amdgcn_s_waitcnt(0xC07F);        // lgkmcnt(0) only
        SLA_SB();
#pragma unroll
        for (int m = 0; m < 16; ++m) {
            acc[m >> 2][m & 3] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(wf0[m >> 2], af0[m & 3], acc[m >> 2][m & 3], 0, 0, 0, 0, 0, 0);
            if (m < 8) read_one(wf1, af1, st, 1, m);
            SLA_SB();
        }
#ifdef SLA_PROBE_TIME
        unsigned long long w0_ = 0, w1_ = 0;
        if (gprobe) w0_ = __builtin_readcyclecounter();
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        if (gprobe) w1_ = __builtin_readcyclecounter();
#else
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#endif
        __builtin_amdgcn_s_waitcnt(0xC07F);        // lgkmcnt(0), as a builtin: the compiler then knows F1 has arrived
        __builtin_amdgcn_s_barrier();
#ifdef SLA_PROBE_TIME
        if (gprobe) { const unsigned long long w2_ = __builtin_readcyclecounter(); wait_copy_ += w1_ - w0_; wait_bar_ += w2_ - w1_; }
#endif
        SLA_SB();
#pragma unroll
        for (int m = 0; m < 16; ++m) {
            acc[m >> 2][m & 3] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(wf1[m >> 2], af1[m & 3], acc[m >> 2][m & 3], 0, 0, 0, 0, 0, 0);
            if (m < 8 && more1) read_one(wf0, af0, st ^ 1, 0, m);
            if (more2) copy_one(An, Wn, dst0, m);
            SLA_SB();
        }
        k2 = k2 + 1 == ksteps ? 0 : k2 + 1;
    }
#undef SLA_SB
    SLA_GT(2);
#ifdef SLA_PROBE_TIME
    if (gprobe && (threadIdx.x & 63) == 0) { sla_gemm_probe_times[6] = wait_copy_; sla_gemm_probe_times[7] = wait_bar_; }
#endif
    __builtin_amdgcn_s_waitcnt(0xC07F);
    __builtin_amdgcn_s_barrier();                                                // every wave is past its last fragment reads
    SLA_GT(3);

    // accumulator (a,b) register 4q+r of lane (l32, g): channel o0 + wo + 32a + 8q + 4g + r, token i0 + wi + 32b + l32.
    // The wave's tile as [128 tokens][128 channels] bf16 in its own 32 KB: the 8-byte piece of channels 4 c2 .. 4 c2 + 3
    // (c2 = 8a + 2q + g) of token row t goes to 16-byte chunk (c2 / 2) ^ (t % 16), half c2 % 2.
    uint8_t *stage = smem + wave * 32768;
    // y = (acc * s_token) * s_channel + bias, two roundings before the bf16 store.  Everything the loop below needs is
    // requested first and awaited once (left alone, the compiler puts each LDS read in front of its first use and waits
    // for it there, thirty-two round trips one after the other).
    float si[4];
    const float *cs = (const float *)(smem + 2 * kStage);
#pragma unroll
    for (int b = 0; b < 4; ++b) si[b] = sa[min(i0 + wi + 32 * b + l32, M - 1)];
    float4 sw4[2][4], bi4[2][4];                                                 // one channel sub-tile in use, the next one on its way
    auto fetch = [&](int a, int buf) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int c = wo + 32 * a + 8 * q + 4 * g;
            sw4[buf][q] = *(const float4 *)(cs + c);
            bi4[buf][q] = *(const float4 *)(cs + 256 + c);
        }
    };
    auto landed = [&](int buf) {
#pragma unroll
        for (int q = 0; q < 4; ++q)
            asm volatile("" : "+v"(sw4[buf][q].x), "+v"(sw4[buf][q].y), "+v"(sw4[buf][q].z), "+v"(sw4[buf][q].w),
                              "+v"(bi4[buf][q].x), "+v"(bi4[buf][q].y), "+v"(bi4[buf][q].z), "+v"(bi4[buf][q].w));
    };
    fetch(0, 0);
    asm volatile("" : "+v"(si[0]), "+v"(si[1]), "+v"(si[2]), "+v"(si[3]));
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const int buf = a & 1;
        __builtin_amdgcn_sched_barrier(0);
        if (a + 1 < 4) fetch(a + 1, buf ^ 1);
        __builtin_amdgcn_sched_barrier(0);
        landed(buf);
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int t = 32 * b + l32;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float v0 = fmaf(acc[a][b][4 * q + 0] * si[b], sw4[buf][q].x, bi4[buf][q].x);
                const float v1 = fmaf(acc[a][b][4 * q + 1] * si[b], sw4[buf][q].y, bi4[buf][q].y);
                const float v2 = fmaf(acc[a][b][4 * q + 2] * si[b], sw4[buf][q].z, bi4[buf][q].z);
                const float v3 = fmaf(acc[a][b][4 * q + 3] * si[b], sw4[buf][q].w, bi4[buf][q].w);
                const int c2 = 8 * a + 2 * q + g;
                *(uint2 *)(stage + t * 256 + (((c2 >> 1) ^ (t & 15)) << 4) + ((c2 & 1) << 3)) = make_uint2(pack_bf16(v0, v1), pack_bf16(v2, v3));
            }
        }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");                          // the wave reads back what it wrote itself
    SLA_GT(4);
    if constexpr (!QKV) {
#pragma unroll
        for (int x0 = 0; x0 < 32; x0 += 16) {                                    // sixteen rows' pieces read, then sixteen stores
            uint4 piece[16];
#pragma unroll
            for (int x = 0; x < 16; ++x) {
                const int t = 4 * (x0 + x) + (lane >> 4), c = lane & 15;         // 16 lanes per token row: 256 contiguous bytes
                piece[x] = *(const uint4 *)(stage + t * 256 + ((c ^ (t & 15)) << 4));
            }
#pragma unroll
            for (int x = 0; x < 16; ++x) {
                const int t = 4 * (x0 + x) + (lane >> 4), c = lane & 15;
                const int i = i0 + wi + t, o = o0 + wo + 8 * c;
                if (i < M && o < O) *(uint4 *)(Y + (size_t)i * O + o) = piece[x];    // O is a multiple of 8: a piece is in or out as a whole
            }
        }
    } else {
        // the wave's tile is two heads (of q, k or v) x 128 tokens = whole token blocks of those heads: it quantises
        // them by itself, one (head, token block) at a time, with the arithmetic of quantise_e4m3_kernel
        const int N = qkv.N, H = qkv.H, rr = lane >> 3, cc = lane & 7;
        for (int hf = 0; hf < 2; ++hf) {
            const int ch0 = o0 + wo + 64 * hf;
            if (ch0 >= O) break;
            const int which = ch0 / (H * 64), h = (ch0 - which * H * 64) >> 6;
            const int blk = which == 0 ? qkv.bq : kBK, nblk_seq = (N + blk - 1) / blk;
            for (int tb = 0; tb * blk < 128; ++tb) {
                const int t0 = i0 + wi + tb * blk;
                if (t0 >= M) break;                                              // uniform over the wave
                const int b = t0 / N, tin = t0 - b * N, valid = min(blk, N - tin);
                float amax = 0.f;
                for (int r = rr; r < valid; r += 8) {
                    const int t = tb * blk + r;
                    const uint4 v = *(const uint4 *)(stage + t * 256 + (((8 * hf + cc) ^ (t & 15)) << 4));
                    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                    for (int q = 0; q < 4; ++q) amax = fmaxf(amax, fmaxf(fabsf(bf16_lo(w[q])), fabsf(bf16_hi(w[q]))));
                }
                amax = wave_max(amax);
                const float scale = fmaxf(amax, 1e-8f) / 448.0f;
                const BlockDivisor by_scale(scale);
                if (lane == 0) qkv.scales[which][((size_t)b * H + h) * nblk_seq + tin / blk] = scale;
                uint8_t *dst = qkv.codes[which] + (((size_t)b * N + tin) * H + h) * 64 + 8 * cc;
                for (int r = rr; r < valid; r += 8) {
                    const int t = tb * blk + r;
                    const uint4 v = *(const uint4 *)(stage + t * 256 + (((8 * hf + cc) ^ (t & 15)) << 4));
                    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
                    float y[8];
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        y[2 * q] = fminf(fmaxf(by_scale(bf16_lo(w[q])), -448.0f), 448.0f);
                        y[2 * q + 1] = fminf(fmaxf(by_scale(bf16_hi(w[q])), -448.0f), 448.0f);
                    }
                    int lo = 0, hi = 0;
                    lo = __builtin_amdgcn_cvt_pk_fp8_f32(y[0], y[1], lo, false);
                    lo = __builtin_amdgcn_cvt_pk_fp8_f32(y[2], y[3], lo, true);
                    hi = __builtin_amdgcn_cvt_pk_fp8_f32(y[4], y[5], hi, false);
                    hi = __builtin_amdgcn_cvt_pk_fp8_f32(y[6], y[7], hi, true);
                    *(uint2 *)(dst + (size_t)r * H * 64) = make_uint2((uint32_t)lo, (uint32_t)hi);
                }
            }
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    SLA_GT(5);
}
#ifdef SLA_PROBE_TIME
extern "C" int sla_probe_read_gemm(unsigned long long *dst) { return (int)hipMemcpyFromSymbol(dst, HIP_SYMBOL(sla_gemm_probe_times), sizeof(unsigned long long) * 16); }
#endif
#undef KS_

static bool lin_big_tiles(int M, int O) { return (long)((M + 255) / 256) * ((O + 255) / 256) >= 512; }   // two rounds of the chip

static bool lin_wide_tiles(int M, int n_ot) { return (long)((M + 255) / 256) * n_ot >= 512; }   // enough 256-token tiles to fill the chip twice over

hipError_t launch_fp8_gemm(const void *A8, const float *sa, const void *W8, const float *sw, const void *bias, int M, int O, int K,
                           void *Y, hipStream_t st)
{
    if (lin_big_tiles(M, O)) {
        const int n_it = (M + 255) / 256;
        const long total = (long)n_it * ((O + 255) / 256);
        fp8_gemm_big_kernel<false><<<(unsigned)xcd_grid(total), 256, 0, st>>>((const uint8_t *)A8, sa, (const uint8_t *)W8, sw, (const uint16_t *)bias, M, O, K,
                                                                              n_it, total, (uint16_t *)Y, QkvOut{});
        return hipGetLastError();
    }
    const int n_ot = (O + 127) / 128;
    const QkvOut none = {};
    if (lin_wide_tiles(M, n_ot)) {
        const int n_it = (M + 255) / 256;
        const long total = (long)n_it * n_ot;
        fp8_gemm_kernel<4, false><<<(unsigned)xcd_grid(total), 256, 0, st>>>((const uint8_t *)A8, sa, (const uint8_t *)W8, sw, (const uint16_t *)bias, M, O, K,
                                                                              n_it, total, (uint16_t *)Y, none);
    } else {
        const int n_it = (M + 127) / 128;
        const long total = (long)n_it * n_ot;
        fp8_gemm_kernel<2, false><<<(unsigned)xcd_grid(total), 256, 0, st>>>((const uint8_t *)A8, sa, (const uint8_t *)W8, sw, (const uint16_t *)bias, M, O, K,
                                                                              n_it, total, (uint16_t *)Y, none);
    }
    return hipGetLastError();
}

int fp8_gemm_qkv_token_tile(int M, int H) { return (lin_big_tiles(M, 3 * H * 64) || lin_wide_tiles(M, (3 * H * 64 + 127) / 128)) ? 256 : 128; }

hipError_t launch_fp8_gemm_qkv(const void *A8, const float *sa, const void *W8, const float *sw, const void *bias, int B, int N, int H, int K,
                               int bq, void *const codes[3], float *const scales[3], hipStream_t st)
{
    const int M = B * N, O = 3 * H * 64, n_ot = (O + 127) / 128;
    QkvOut q;
    for (int w = 0; w < 3; ++w) { q.codes[w] = (uint8_t *)codes[w]; q.scales[w] = scales[w]; }
    q.N = N; q.H = H; q.bq = bq;
    if (lin_big_tiles(M, O)) {
        const int n_it = (M + 255) / 256;
        const long total = (long)n_it * ((O + 255) / 256);
        fp8_gemm_big_kernel<true><<<(unsigned)xcd_grid(total), 256, 0, st>>>((const uint8_t *)A8, sa, (const uint8_t *)W8, sw, (const uint16_t *)bias, M, O, K,
                                                                             n_it, total, nullptr, q);
        return hipGetLastError();
    }
    if (lin_wide_tiles(M, n_ot)) {
        const int n_it = (M + 255) / 256;
        const long total = (long)n_it * n_ot;
        fp8_gemm_kernel<4, true><<<(unsigned)xcd_grid(total), 256, 0, st>>>((const uint8_t *)A8, sa, (const uint8_t *)W8, sw, (const uint16_t *)bias, M, O, K,
                                                                             n_it, total, nullptr, q);
    } else {
        const int n_it = (M + 127) / 128;
        const long total = (long)n_it * n_ot;
        fp8_gemm_kernel<2, true><<<(unsigned)xcd_grid(total), 256, 0, st>>>((const uint8_t *)A8, sa, (const uint8_t *)W8, sw, (const uint16_t *)bias, M, O, K,
                                                                             n_it, total, nullptr, q);
    }
    return hipGetLastError();
}

}  // namespace sla
