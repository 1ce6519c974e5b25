// Sum of the key-block states over the marginal blocks of every query block:
//     Hq[i][:] = sum_{j : label(i,j) == marginal} hT[j][:]          (4160 values per block)
// evaluated per head as the product  M[Nqb x Nkb] * Hf[Nkb x 4160]  with M the 0/1 marginal
// mask, on v_mfma_f32_32x32x16_bf16 with fp32 accumulation.  A gather would move
// Nqb*k_m*8.3 KB per head; the product re-uses every state tile across 128 query blocks.
//
// Workgroup tile 128 (query blocks) x 128 (state columns), K step 32 key blocks, 4 waves in
// a 2x2 arrangement of 64x64 wave tiles.  The mask operand is built on the fly from the
// int8 labels; the state operand is transposed in registers while it is staged so both MFMA
// operands are read from LDS as 16-byte rows.
#include "sla_common.hpp"
#include "sla_kernels.hpp"

namespace sla {

constexpr int kAggRow = 40;   // bf16 per LDS row: 32 K-values + 8 pad (80 B stride)

__global__ __launch_bounds__(256) void aggregate_kernel(const int8_t *__restrict__ lab, int lab_pitch,
                                                        const uint16_t *__restrict__ hT, int Nqb, int Nkb,
                                                        uint16_t *__restrict__ Hq)
{
    __shared__ __attribute__((aligned(16))) uint16_t As[128 * kAggRow];
    __shared__ __attribute__((aligned(16))) uint16_t Bs[128 * kAggRow];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1, l32 = lane & 31, g = lane >> 5;
    const int n0 = blockIdx.x * 128, i0 = blockIdx.y * 128;
    const long bh = blockIdx.z;
    const int8_t *labh = lab + bh * (long)Nqb * lab_pitch;
    const uint16_t *Hf = hT + bh * (long)Nkb * kStateElems;

    // A loader: thread -> (row i = tid/2, 16 labels at k = 16*(tid&1))
    const int ai = tid >> 1, ak = (tid & 1) * 16;
    const bool a_ok = i0 + ai < Nqb;
    // B loader: thread -> (column pair 2p, 2p+1; 8 consecutive key blocks 8*kg..)
    const int bp = tid & 63, bkg = tid >> 6;
    const bool b_ok = n0 + 2 * bp < kStateElems;      // kStateElems is even: the pair is in or out together

    f32x16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

    uint4 areg = make_uint4(0, 0, 0, 0);
    uint32_t breg[8];
    auto load_tile = [&](int k0) {
        areg = make_uint4(0, 0, 0, 0);
        if (a_ok && k0 + ak < lab_pitch) areg = *(const uint4 *)(labh + (long)(i0 + ai) * lab_pitch + k0 + ak);
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int j = k0 + bkg * 8 + r;
            breg[r] = (b_ok && j < Nkb) ? *(const uint32_t *)(Hf + (long)j * kStateElems + n0 + 2 * bp) : 0u;
        }
    };
    auto store_tile = [&]() {
        // 16 labels -> 16 bf16 mask values (1.0 where the label is "marginal")
        uint32_t w[4] = {areg.x, areg.y, areg.z, areg.w};
        uint32_t o[8];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t b0 = (w[q] & 0xFFu) == 1u, b1 = ((w[q] >> 8) & 0xFFu) == 1u;
            const uint32_t b2 = ((w[q] >> 16) & 0xFFu) == 1u, b3 = (w[q] >> 24) == 1u;
            o[2 * q] = (b0 ? 0x3F80u : 0u) | (b1 ? 0x3F800000u : 0u);
            o[2 * q + 1] = (b2 ? 0x3F80u : 0u) | (b3 ? 0x3F800000u : 0u);
        }
        *(uint4 *)(As + ai * kAggRow + ak) = make_uint4(o[0], o[1], o[2], o[3]);
        *(uint4 *)(As + ai * kAggRow + ak + 8) = make_uint4(o[4], o[5], o[6], o[7]);
        uint4 lo, hi;
        lo.x = __builtin_amdgcn_perm(breg[1], breg[0], 0x05040100); hi.x = __builtin_amdgcn_perm(breg[1], breg[0], 0x07060302);
        lo.y = __builtin_amdgcn_perm(breg[3], breg[2], 0x05040100); hi.y = __builtin_amdgcn_perm(breg[3], breg[2], 0x07060302);
        lo.z = __builtin_amdgcn_perm(breg[5], breg[4], 0x05040100); hi.z = __builtin_amdgcn_perm(breg[5], breg[4], 0x07060302);
        lo.w = __builtin_amdgcn_perm(breg[7], breg[6], 0x05040100); hi.w = __builtin_amdgcn_perm(breg[7], breg[6], 0x07060302);
        *(uint4 *)(Bs + (2 * bp) * kAggRow + bkg * 8) = lo;
        *(uint4 *)(Bs + (2 * bp + 1) * kAggRow + bkg * 8) = hi;
    };

    const int ksteps = (Nkb + 31) / 32;
    load_tile(0);
    for (int ks = 0; ks < ksteps; ++ks) {
        __syncthreads();               // previous tile fully consumed
        store_tile();
        __syncthreads();
        if (ks + 1 < ksteps) load_tile((ks + 1) * 32);
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            bf16x8 af[2], bfr[2];
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                af[a] = *(const bf16x8 *)(As + (64 * wm + 32 * a + l32) * kAggRow + 16 * s + 8 * g);
                bfr[a] = *(const bf16x8 *)(Bs + (64 * wn + 32 * a + l32) * kAggRow + 16 * s + 8 * g);
            }
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a], bfr[b], acc[a][b], 0, 0, 0);
        }
    }

    // accumulator (a,b) register 4q+r: row i = i0 + 64wm + 32a + 8q + 4g + r, column n = n0 + 64wn + 32b + l32
    uint16_t *out = Hq + bh * (long)Nqb * kStateElems;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int n = n0 + 64 * wn + 32 * b + l32;
            if (n >= kStateElems) continue;
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int i = i0 + 64 * wm + 32 * a + 8 * q + 4 * g + r;
                    if (i < Nqb) out[(long)i * kStateElems + n] = (uint16_t)(pack_bf16(acc[a][b][4 * q + r], 0.f) & 0xFFFFu);
                }
        }
}

hipError_t launch_aggregate(const int8_t *lab_pad, int lab_pitch, const void *hT, int BH, int Nqb,
                            int Nkb, void *Hq, hipStream_t st)
{
    dim3 grid((kStateElems + 127) / 128, (Nqb + 127) / 128, BH);
    aggregate_kernel<<<grid, 256, 0, st>>>(lab_pad, lab_pitch, (const uint16_t *)hT, Nqb, Nkb, (uint16_t *)Hq);
    return hipGetLastError();
}

}  // namespace sla
