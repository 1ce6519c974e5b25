// Sum of the key-block states over the marginal blocks of every query block:
//     Hq[i][:] = sum_{j : label(i,j) == marginal} hT[j][:]          (4160 values per block)
// evaluated per head as the product  M[Nqb x Nkb] * Hf[Nkb x 4160]  with M the 0/1 marginal
// mask, on v_mfma_f32_32x32x16_bf16 with fp32 accumulation.  A gather would move
// Nqb*k_m*8.3 KB per head; the product re-uses every state tile across all query blocks of a
// workgroup tile.
//
// The kernel computes the transposed tile  D^T[n][i] = sum_j Hf[j][n] M[i][j]:  the state slab is
// the MFMA A operand and goes through LDS (transposed in registers on its way in, so the operand
// is read as 16-byte rows); the mask is the B operand and never touches LDS: a lane's eight mask
// values of one MFMA are eight consecutive bits of the row's marginal bit mask, expanded in
// registers to bf16 2.0 / 0.0 (a bf16 power of two has a single bit set; the accumulators are
// halved at the end, which is exact).  A lane's four consecutive accumulator registers are four
// consecutive state columns of one query block and leave through LDS as 16-byte stores.
//
// Workgroup: 4 waves, tile 128 state columns x BM query blocks.  Long heads: BM = 256, every wave
// takes all 128 columns (TA = 4 sub-tiles of 32) and 64 query blocks (TB = 2), so the state slab,
// which dominates the L2 traffic, is read once per 256 query blocks and one expanded mask operand
// feeds four MFMAs.  Short heads: BM = 64, waves as 2 x 2 with TA = 2, TB = 1; frame-sized heads (at most 32
// query blocks): BM = 32, four waves side by side along the columns, TA = TB = 1.  K step 64
// key blocks; global loads run AHEAD (three, or one for very short heads) K steps ahead of their use in
// register sets, LDS is double buffered: one barrier per K step.
#include "sla_common.hpp"
#include "sla_kernels.hpp"

namespace sla {

namespace {
constexpr int kAggK = 64;             // key blocks per K step (one 64-bit mask word)
constexpr int kAggRow = kAggK + 8;    // bf16 per state-operand row in LDS: 144 B, consecutive rows start 9 16-byte slots apart
constexpr int kAggOutRow = 128 + 8;   // bf16 per row of the output staging tile (272 B)
constexpr int kAggBuf = 128 * kAggRow;
}  // namespace

// AHEAD: K steps between a global load and its use (register sets); 1 for heads of one or two K steps, where
// deeper sets would only cost registers and with them resident workgroups
// NBUF: LDS operand buffers, 2 in general, 1 for heads of a single K step (more workgroups per CU)
template <int TA, int TB, int AHEAD, int NBUF>
__global__ __launch_bounds__(256, (TA == 2 && AHEAD == 3) ? 4 : 1) void aggregate_kernel(const uint2 *__restrict__ mbits, int nkw,
                                                        const uint16_t *__restrict__ hT, int Nqb, int Nkb, int n_it,
                                                        long total, uint16_t *__restrict__ Hq)
{
    asm volatile("" ::"s"(mbits), "s"(nkw), "s"(hT), "s"(Nqb), "s"(Nkb), "s"(n_it), "s"(total), "s"(Hq));      // all kernel arguments in one batch of scalar loads, here
    constexpr int kWN = 4 / TA;                   // waves along the columns (TA 32-column sub-tiles each)
    constexpr int kWI = 4 / kWN;                  // waves along the query blocks (TB 32-block sub-tiles each)
    constexpr int BM = 32 * TB * kWI;             // query blocks per workgroup tile
    constexpr int kStage = BM * kAggOutRow > NBUF * kAggBuf ? BM * kAggOutRow : NBUF * kAggBuf;
    __shared__ __attribute__((aligned(16))) uint16_t smem[kStage];

    const long item = xcd_remap(blockIdx.x, total);      // (head, column tile, query tile), query tile fastest:
    if (item >= total) return;                           // neighbours on one XCD share a state slab in its L2
    // (32-bit divisions: the grid fits 32 bits, and a 64-bit division is some sixty instructions)
    const unsigned rest = (unsigned)item / (unsigned)n_it;
    const int it = (int)((unsigned)item - rest * (unsigned)n_it);
    constexpr int kNT = (kStateElems + 127) / 128;
    const long bh = rest / kNT;
    const int nt = (int)(rest - (unsigned)bh * kNT);
    const int n0 = nt * 128, i0 = it * BM;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, g = lane >> 5;
    const int wn = (wave / kWI) * (32 * TA), wi = (wave % kWI) * (32 * TB);   // wave's first column / query block within the tile
    const uint16_t *Hf = hT + bh * (long)Nkb * kStateElems;

    // state loader: thread -> 4 columns (4 n4 ..) x 8 key blocks (8 jg ..).  Lane bits 0-1 and 4-6 select the
    // column group, bits 2-3 and 7 the key-block group: a load instruction covers whole 128-byte lines and the
    // sixteen lanes of one LDS write pass land on sixteen different 16-byte slots.
    // The loads of the main loop are unconditional (indices are clamped instead: key blocks past the end repeat
    // the last one and meet mask bits that are zero, columns and query blocks past the end give results nobody
    // stores), so the compiler can count the loads in flight and wait for exactly the set it needs.
    const int n4 = (tid & 3) | ((tid >> 2) & 0x1C), jg = ((tid >> 2) & 3) | ((tid >> 5) & 4);
    // byte offsets inside the head's slab fit 32 bits (a slab is Nkb x 8320 bytes): the loads take the slab's base from
    // scalar registers and a 32-bit offset per lane, formed with full-rate instructions (64-bit address arithmetic
    // per load was a quarter-rate multiply and more, a third of the loop's vector time)
    const uint8_t *Hf8 = (const uint8_t *)Hf;
    const uint32_t colb = 2u * (uint32_t)(n0 + 4 * n4 < kStateElems ? n0 + 4 * n4 : 0);   // kStateElems % 4 == 0: a group is in or out as a whole
    auto state_piece = [&](int j) { return *(const uint2 *)(Hf8 + (__umul24((uint32_t)j, 2u * kStateElems) + colb)); };
    // mask rows of this lane: query block i0 + wi + 32 b + l32, one 64-bit word per K step
    const uint2 *mrow[TB];
#pragma unroll
    for (int b = 0; b < TB; ++b) {
        const int i = i0 + wi + 32 * b + l32;
        mrow[b] = mbits + (bh * (long)Nqb + (i < Nqb ? i : 0)) * nkw;
    }
    const int ksteps = (Nkb + kAggK - 1) / kAggK;            // == nkw

    uint2 hreg[AHEAD][8];
    uint2 mreg[AHEAD][TB];
    auto load_tile = [&](int ks, uint2 (&h)[8], uint2 (&m)[TB]) {          // main loop: ks < ksteps
#pragma unroll
        for (int b = 0; b < TB; ++b) m[b] = mrow[b][ks];
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int j = min(ks * kAggK + jg * 8 + r, Nkb - 1);
            h[r] = state_piece(j);
        }
    };
    // first and last steps: the same tile, but key blocks past the end are skipped instead of repeated (short
    // heads have K steps that are mostly padding)
    auto load_tile_edge = [&](int ks, uint2 (&h)[8], uint2 (&m)[TB]) {
#pragma unroll
        for (int b = 0; b < TB; ++b) m[b] = mrow[b][ks];
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int j = ks * kAggK + jg * 8 + r;
            h[r] = j < Nkb ? state_piece(j) : make_uint2(0u, 0u);
        }
    };
    auto store_tile = [&](uint16_t *As, const uint2 (&h)[8]) {
        // column c of the 8x4 piece -> one 16-byte row segment (8 key blocks of one column)
        uint4 c0, c1, c2, c3;
        c0.x = __builtin_amdgcn_perm(h[1].x, h[0].x, 0x05040100); c1.x = __builtin_amdgcn_perm(h[1].x, h[0].x, 0x07060302);
        c2.x = __builtin_amdgcn_perm(h[1].y, h[0].y, 0x05040100); c3.x = __builtin_amdgcn_perm(h[1].y, h[0].y, 0x07060302);
        c0.y = __builtin_amdgcn_perm(h[3].x, h[2].x, 0x05040100); c1.y = __builtin_amdgcn_perm(h[3].x, h[2].x, 0x07060302);
        c2.y = __builtin_amdgcn_perm(h[3].y, h[2].y, 0x05040100); c3.y = __builtin_amdgcn_perm(h[3].y, h[2].y, 0x07060302);
        c0.z = __builtin_amdgcn_perm(h[5].x, h[4].x, 0x05040100); c1.z = __builtin_amdgcn_perm(h[5].x, h[4].x, 0x07060302);
        c2.z = __builtin_amdgcn_perm(h[5].y, h[4].y, 0x05040100); c3.z = __builtin_amdgcn_perm(h[5].y, h[4].y, 0x07060302);
        c0.w = __builtin_amdgcn_perm(h[7].x, h[6].x, 0x05040100); c1.w = __builtin_amdgcn_perm(h[7].x, h[6].x, 0x07060302);
        c2.w = __builtin_amdgcn_perm(h[7].y, h[6].y, 0x05040100); c3.w = __builtin_amdgcn_perm(h[7].y, h[6].y, 0x07060302);
        uint16_t *a = As + (4 * n4) * kAggRow + jg * 8;
        *(uint4 *)(a) = c0;
        *(uint4 *)(a + kAggRow) = c1;
        *(uint4 *)(a + 2 * kAggRow) = c2;
        *(uint4 *)(a + 3 * kAggRow) = c3;
    };
    // eight mask bits (key blocks 16 s + 8 g .. + 7 of the K step) -> the B operand of one MFMA: bf16 2.0 where set.
    // x | x << 15 puts a second copy of the byte 15 bits up, so that one shift brings bit 2d to bit 14 and bit 2d+1 to
    // bit 30 of the same dword: the two bf16 exponent bits of 2.0.  (The empty asm keeps the compiler from turning
    // the four shifts of that word into four multiplications of x by wide constants: v_mul_lo_u32 runs at a quarter
    // of the rate of a shift, and three of them per operand were a third of the loop's vector time.)
    auto mask_frag = [&](const uint2 &w, int s) {
        const uint32_t x = ((s < 2 ? w.x : w.y) >> (16 * (s & 1) + 8 * g)) & 0xFFu;
        uint32_t m = x | (x << 15);
        asm("" : "+v"(m));
        union { uint32_t u[4]; bf16x8 v; } f;
        f.u[0] = (m << 14) & 0x40004000u;
        f.u[1] = (m << 12) & 0x40004000u;
        f.u[2] = (m << 10) & 0x40004000u;
        f.u[3] = (m << 8) & 0x40004000u;
        return f.v;
    };

    f32x16 acc[TA][TB];
#pragma unroll
    for (int a = 0; a < TA; ++a)
#pragma unroll
        for (int b = 0; b < TB; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.f;

    // one K step: the operand tile of step ks is in LDS buffer ks & 1, its mask words in mw
    auto mma_step = [&](int ks, const uint2 (&mw)[TB]) {
        const uint16_t *As = smem + (ks & (NBUF - 1)) * kAggBuf;
#pragma unroll
        for (int s = 0; s < kAggK / 16; ++s) {
            bf16x8 af[TA];
#pragma unroll
            for (int a = 0; a < TA; ++a) af[a] = *(const bf16x8 *)(As + (wn + 32 * a + l32) * kAggRow + 16 * s + 8 * g);
#pragma unroll
            for (int b = 0; b < TB; ++b) {
                const bf16x8 mf = mask_frag(mw[b], s);
#pragma unroll
                for (int a = 0; a < TA; ++a)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a], mf, acc[a][b], 0, 0, 0);
            }
        }
    };

#pragma unroll
    for (int u = 0; u < AHEAD; ++u)
        if (u < ksteps) load_tile_edge(u, hreg[u], mreg[u]);
    store_tile(smem, hreg[0]);
    lds_barrier();

    // main part: groups of AHEAD steps whose look-ahead loads are all real, as straight-line code (register
    // set u holds step ks0 + u); the compiler waits for one set at a time and leaves the later ones in flight
    int ks0 = 0;
    for (; ks0 + 2 * AHEAD <= ksteps; ks0 += AHEAD) {
#pragma unroll
        for (int u = 0; u < AHEAD; ++u) {
            const int ks = ks0 + u;
            uint2 mw[TB];
#pragma unroll
            for (int b = 0; b < TB; ++b) mw[b] = mreg[u][b];
            load_tile(ks + AHEAD, hreg[u], mreg[u]);      // set u: its states went to LDS one step ago, its mask words are copied
            mma_step(ks, mw);
            store_tile(smem + ((ks + 1) & (NBUF - 1)) * kAggBuf, hreg[(u + 1) % AHEAD]);
            lds_barrier();                                     // not __syncthreads(): the loads of later steps stay in flight
        }
    }
    // the remaining steps (fewer than 2 AHEAD), with the loads that are still due issued under a condition
    for (; ks0 < ksteps; ks0 += AHEAD) {
#pragma unroll
        for (int u = 0; u < AHEAD; ++u) {
            const int ks = ks0 + u;
            if (ks < ksteps) {                                 // uniform over the workgroup
                uint2 mw[TB];
#pragma unroll
                for (int b = 0; b < TB; ++b) mw[b] = mreg[u][b];
                if (ks + AHEAD < ksteps) load_tile_edge(ks + AHEAD, hreg[u], mreg[u]);
                mma_step(ks, mw);
                if (ks + 1 < ksteps) store_tile(smem + ((ks + 1) & (NBUF - 1)) * kAggBuf, hreg[(u + 1) % AHEAD]);
                lds_barrier();
            }
        }
    }

    // accumulator (a,b) register 4q+r of lane (l32, g): column n0 + wn + 32a + 8q + 4g + r, query block i0 + wi + 32b + l32.
    // Staged as [query block][column] so that a query block's 128 columns leave as 16-byte stores; the factor 0.5
    // undoes the mask value 2.0.
#pragma unroll
    for (int a = 0; a < TA; ++a)
#pragma unroll
        for (int b = 0; b < TB; ++b)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                uint2 o;
                o.x = pack_bf16(0.5f * acc[a][b][4 * q], 0.5f * acc[a][b][4 * q + 1]);
                o.y = pack_bf16(0.5f * acc[a][b][4 * q + 2], 0.5f * acc[a][b][4 * q + 3]);
                *(uint2 *)(smem + (wi + 32 * b + l32) * kAggOutRow + wn + 32 * a + 8 * q + 4 * g) = o;
            }
    __syncthreads();
    uint16_t *out = Hq + bh * (long)Nqb * kStateElems;
#pragma unroll
    for (int t = 0; t < BM * 16 / 256; ++t) {
        const int idx = tid + 256 * t, r = idx >> 4, seg = idx & 15;
        if (i0 + r < Nqb && n0 + 8 * seg < kStateElems)       // kStateElems % 8 == 0: the segment is in or out as a whole
            *(uint4 *)(out + (long)(i0 + r) * kStateElems + n0 + 8 * seg) = *(const uint4 *)(smem + r * kAggOutRow + 8 * seg);
    }
}

hipError_t launch_aggregate(const uint64_t *mbits, int lab_pitch, const void *hT, int BH, int Nqb,
                            int Nkb, void *Hq, hipStream_t st)
{
    constexpr int kNT = (kStateElems + 127) / 128;
    const int nkw = lab_pitch / 64;
    if (Nqb <= 32 && Nkb <= kAggK) {   // frame-sized heads (one K step): 32-query-block tiles, 32 x 32 per wave, one LDS buffer
        const long total = (long)BH * kNT;
        aggregate_kernel<1, 1, 1, 1><<<(unsigned)xcd_grid(total), 256, 0, st>>>((const uint2 *)mbits, nkw, (const uint16_t *)hT, Nqb, Nkb,
                                                                              1, total, (uint16_t *)Hq);
    } else if (Nqb <= 192) {    // short heads: 64-query-block tiles waste less of the matrix unit and give more workgroups
        const int n_it = (Nqb + 63) / 64;
        const long total = (long)BH * kNT * n_it;
        if (Nkb <= 128)
            aggregate_kernel<2, 1, 1, 2><<<(unsigned)xcd_grid(total), 256, 0, st>>>((const uint2 *)mbits, nkw, (const uint16_t *)hT, Nqb, Nkb,
                                                                               n_it, total, (uint16_t *)Hq);
        else
            aggregate_kernel<2, 1, 3, 2><<<(unsigned)xcd_grid(total), 256, 0, st>>>((const uint2 *)mbits, nkw, (const uint16_t *)hT, Nqb, Nkb,
                                                                               n_it, total, (uint16_t *)Hq);
    } else {
        const int n_it = (Nqb + 255) / 256;
        const long total = (long)BH * kNT * n_it;
        aggregate_kernel<4, 2, 3, 2><<<(unsigned)xcd_grid(total), 256, 0, st>>>((const uint2 *)mbits, nkw, (const uint16_t *)hT, Nqb, Nkb,
                                                                        n_it, total, (uint16_t *)Hq);
    }
    return hipGetLastError();
}

}  // namespace sla
