// Scaled FP8 quantiser of App. B.2 of the paper, applied per block of `blk` consecutive tokens of every (b, h) --
// the granularity the E4M3 configuration of the SLA forward consumes for Q, K and V:
//     scale = max(amax, 1e-8) / 448  (fp32),   code = E4M3(clamp(x / scale, -448, 448)),  round-to-nearest-even
// One wavefront per block: the block's rows are read once as 16-byte pieces and stay in registers, the absolute
// maximum is reduced across the wave, and every lane converts its own pieces (v_cvt_pk_fp8_f32 rounds to nearest
// even; the operands are clamped first, so its overflow behaviour never matters) and stores 8 bytes per piece, 512
// contiguous bytes per wave-wide store.  HBM bound: 2 bytes in and 1 byte out per element.
#include "sla_common.hpp"
#include "sla_kernels.hpp"

namespace sla {

template <int BLK>
__global__ __launch_bounds__(256) void quantise_e4m3_kernel(const uint16_t *__restrict__ X, RowMap rm, int N, int nblk, long blocks,
                                                            uint8_t *__restrict__ codes, float *__restrict__ scales)
{
    asm volatile("" ::"s"(X), "s"(rm.bs), "s"(rm.hs), "s"(rm.ts), "s"(rm.H), "s"(N), "s"(nblk), "s"(blocks), "s"(codes), "s"(scales));      // all kernel arguments in one batch of scalar loads, here
    constexpr int kPieces = BLK / 8;                 // 16-byte pieces per lane: rows r = lane/8 + 8 k, channels 8 (lane%8) ..
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const long blk = (long)blockIdx.x * 4 + wave;
    if (blk >= blocks) return;                       // the whole wave leaves; nothing below synchronises across waves
    const long bh = blk / nblk;
    const int t0 = (int)(blk - bh * nblk) * BLK, valid = min(BLK, N - t0);
    const uint16_t *x = X + rm.head(bh) + (size_t)t0 * rm.ts + (lane & 7) * 8;
    uint32_t w[kPieces][4];
    float amax = 0.f;
#pragma unroll
    for (int k = 0; k < kPieces; ++k) {
        const int r = (lane >> 3) + 8 * k;
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (r < valid) v = *(const uint4 *)(x + (size_t)r * rm.ts);
        w[k][0] = v.x; w[k][1] = v.y; w[k][2] = v.z; w[k][3] = v.w;
#pragma unroll
        for (int c = 0; c < 4; ++c) amax = fmaxf(amax, fmaxf(fabsf(bf16_lo(w[k][c])), fabsf(bf16_hi(w[k][c]))));
    }
    amax = wave_max(amax);
    const float scale = fmaxf(amax, 1e-8f) / 448.0f;
    if (lane == 0) scales[blk] = scale;
    uint8_t *out = codes + rm.head(bh) + (size_t)t0 * rm.ts + (lane & 7) * 8;
#pragma unroll
    for (int k = 0; k < kPieces; ++k) {
        const int r = (lane >> 3) + 8 * k;
        if (r >= valid) continue;
        float y[8];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            y[2 * c] = fminf(fmaxf(bf16_lo(w[k][c]) / scale, -448.0f), 448.0f);
            y[2 * c + 1] = fminf(fmaxf(bf16_hi(w[k][c]) / scale, -448.0f), 448.0f);
        }
        int lo = 0, hi = 0;
        lo = __builtin_amdgcn_cvt_pk_fp8_f32(y[0], y[1], lo, false);
        lo = __builtin_amdgcn_cvt_pk_fp8_f32(y[2], y[3], lo, true);
        hi = __builtin_amdgcn_cvt_pk_fp8_f32(y[4], y[5], hi, false);
        hi = __builtin_amdgcn_cvt_pk_fp8_f32(y[6], y[7], hi, true);
        *(uint2 *)(out + (size_t)r * rm.ts) = make_uint2((uint32_t)lo, (uint32_t)hi);
    }
}

hipError_t launch_quantise_e4m3(const void *X, RowMap rm, int BH, int N, int blk, void *codes, float *scales, hipStream_t st)
{
    const int nblk = (N + blk - 1) / blk;
    const long blocks = (long)BH * nblk;
    const unsigned grid = (unsigned)((blocks + 3) / 4);
    if (blk == 64) quantise_e4m3_kernel<64><<<grid, 256, 0, st>>>((const uint16_t *)X, rm, N, nblk, blocks, (uint8_t *)codes, scales);
    else           quantise_e4m3_kernel<128><<<grid, 256, 0, st>>>((const uint16_t *)X, rm, N, nblk, blocks, (uint8_t *)codes, scales);
    return hipGetLastError();
}

}  // namespace sla
