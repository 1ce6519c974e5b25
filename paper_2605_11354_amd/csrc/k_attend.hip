// Block-sparse flash attention over the critical key blocks of each query block, fused with
// the linear-branch output, the projection and the sum (Alg. 1 steps 4-5, 9, 10; eq. (1)):
//     O_i = softmax_{t' in critical blocks}(Q_i K_t'^T * scale) V_t'
//           + [ phi(Q_i) H_i / (phi(Q_i) . Z_i) ] W_proj
//
// Work decomposition.  One workgroup per (b, h, query block); each wavefront owns 32 query
// rows and keeps everything transposed so that a lane owns ONE query row:
//     S^T[t'][q]  = K_tile (A operand, LDS rows)  x  Q^T (B operand, registers)
//     O^T[e][q]  += V^T_tile (A operand, LDS)     x  P^T (B operand = the S^T accumulators,
//                                                   re-used in place: no LDS round trip)
// With v_mfma_f32_32x32x16_bf16 a lane holds column q = lane%32 of the 32x32 result, rows
// 8a + 4g + b (g = lane/32; register 4a+b), so the online-softmax row statistics are 31
// in-lane operations plus one exchange with lane^32.  The B operand of the second product
// takes accumulator registers 8u..8u+7, i.e. keys 16s + 8a' + 4g + b; the V^T rows are read
// with exactly that key permutation: the states kernel leaves V^T of every key block in that
// order (bf16), so a V^T fragment is one 16-byte LDS read like a K fragment.
// Template parameters: NW query groups of 32 rows (2 for 64-row, 4 for 128-row query blocks); KS = 2 splits the
// critical list of a 64-row block between two wave pairs (alternate tiles) whose (maximum, sum, O) are merged
// through LDS before the epilogue, so that short lists still give a workgroup four waves of work.
//
// Memory pipeline.  K and V^T tiles go from global memory straight into LDS
// (global_load_lds_dwordx4, no staging registers) into a ring of three stages (two for lists of at most two
// tiles, see STG below); the tile of
// iteration c+2 is requested while tile c is consumed, and a single workgroup barrier per
// iteration both publishes tile c and frees the stage of tile c-1.  Rows are stored unpadded
// with the 16-byte chunk index XOR-ed by row bits (applied on the global side of the copy),
// which keeps the fragment reads free of bank conflicts.  Every wave issues the same number of
// copies per tile (rows past a ragged end are clamped, absent list entries copy block 0), so
// s_waitcnt vmcnt(n) with a compile-time n identifies "tile c has landed".  The key mask of a
// ragged last block enters as the initial accumulator of S^T (0 / -inf), costing nothing per tile.
//
// E4M3 inputs.  S^T is one v_mfma_f32_32x32x64_f8f6f4 per 32 keys (the whole head dimension
// is the K dimension of the instruction; products of two E4M3 numbers are exact in the fp32
// accumulator), with the per-block scales folded into the exp2 constant.  P is NOT cast to
// E4M3: three mantissa bits on the softmax weights put the output error at several percent
// of its RMS, above the 6e-2 bar, so P stays bf16, V^T arrives widened to bf16 (exactly) from
// the states kernel, and the second product runs on the bf16 MFMA.  The V block scale is folded into the
// exponent of the weights, so no operand of that product is rounded twice.
//
// Epilogue (per wave, all MFMA): O_lin^T = Hq^T-tile x phi(Q)^T, scaled by 1/(phi(Q).Z),
// then O^T += W^T x O_lin^T accumulated onto the normalised sparse output, stored as bf16.
#include "sla_common.hpp"
#include "sla_kernels.hpp"

namespace sla {

constexpr float kLog2e = 1.4426950408889634f;
// Slack allowed before a row raises its running maximum.  0 = exact running maximum: the dominant weight of a
// row is then exactly 1.0 and survives the bf16 rounding of P untouched; a slack of 8 (rescaling the
// accumulators far less often) was measured 6 % faster but doubled the output error of peaked rows.
constexpr float kLazyMax = 0.0f;

typedef __attribute__((address_space(3))) void *lds_void_p;
typedef __attribute__((address_space(1))) const void *glb_void_p;

// XOR swizzle of 16-byte chunks: 8 chunks per 128-byte row / 4 chunks per 64-byte row
__device__ __forceinline__ int swz8(int row) { return (row >> 1) & 7; }
__device__ __forceinline__ int swz4(int row) { return (row >> 2) & 3; }

// Waits until at most N of this wave's tile copies are outstanding, then joins the workgroup.
// The copies below are issued from inline assembly so that the compiler's own wait-count
// insertion does not see them: it would otherwise drain ALL outstanding copies (vmcnt(0))
// before every LDS read and serialise the prefetch ring.  The waits are therefore explicit.
template <int N> __device__ __forceinline__ void wait_copies_and_barrier()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_waitcnt lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}

// One 1 KB copy global -> LDS: lane l moves the 16 bytes at base + voff(l) to LDS byte lds_addr + 16 l.
// base and lds_addr are wave-uniform (SGPRs); M0 carries the LDS address for this instruction only.  The s_nop is
// the wait state the ISA asks for between a scalar write of M0 and an instruction that moves data into LDS through
// it (the compiler's hazard recogniser does not look inside inline assembly).
__device__ __forceinline__ void copy_1k_to_lds(const uint8_t *base, uint32_t voff, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(base), "s"(lds_addr) : "memory");
}

template <int NW, bool FP8>
struct Tile {
    static constexpr int KBYTES = FP8 ? 64 * 64 : 64 * 128;     // K tile (e4m3 / bf16)
    static constexpr int VBYTES = 64 * 128;                     // V^T tile (always bf16)
    static constexpr int STAGE = KBYTES + VBYTES;
    static constexpr int KINS = KBYTES / 1024 / NW;             // 1 KB copy instructions per wave
    static constexpr int VINS = VBYTES / 1024 / NW;
    static constexpr int LOADS = KINS + VINS;                   // per wave per tile
};

// Per-lane byte offsets (inside a tile) of the 16-byte chunk each lane copies, one per copy
// instruction of this wave: LDS position (row, slot) <- global chunk slot ^ swizzle(row).
template <int NW, bool FP8>
struct CopyOffsets {
    using T = Tile<NW, FP8>;
    int k[T::KINS], v[T::VINS];
    int krow[T::KINS];            // K row of this lane per instruction (for clamping at a ragged end)
    // krowb: bytes between consecutive K rows in global memory (64 or 128 when the heads are contiguous)
    __device__ __forceinline__ void init(int wave, int lane, int krowb)
    {
#pragma unroll
        for (int x = 0; x < T::KINS; ++x) {
            const int ins = wave * T::KINS + x;
            if (FP8) { const int r = ins * 16 + (lane >> 2); krow[x] = r; k[x] = r * krowb + (((lane & 3) ^ swz4(r)) << 4); }
            else     { const int r = ins * 8 + (lane >> 3);  krow[x] = r; k[x] = r * krowb + (((lane & 7) ^ swz8(r)) << 4); }
        }
#pragma unroll
        for (int x = 0; x < T::VINS; ++x) {
            const int ins = wave * T::VINS + x, r = ins * 8 + (lane >> 3);
            v[x] = r * 128 + (((lane & 7) ^ swz8(r)) << 4);
        }
    }
};

// Requests one K tile and one V^T tile into the LDS stage at byte address stage (wave-uniform).
// kt / vt: first byte of the tiles in global memory (wave-uniform); valid: number of real rows of
// the K tile (rows past it are clamped to the last, they are masked later; V^T tiles are complete).
template <int NW, bool FP8>
__device__ __forceinline__ void issue_tile(uint32_t stage, const uint8_t *kt, const uint8_t *vt, int valid, int KROW,
                                           const CopyOffsets<NW, FP8> &co, int wave)
{
    using T = Tile<NW, FP8>;
    if (valid == kBK) {
#pragma unroll
        for (int x = 0; x < T::KINS; ++x) copy_1k_to_lds(kt, co.k[x], stage + (wave * T::KINS + x) * 1024);
    } else {
#pragma unroll
        for (int x = 0; x < T::KINS; ++x)
            copy_1k_to_lds(kt, co.k[x] - (co.krow[x] - min(co.krow[x], valid - 1)) * KROW, stage + (wave * T::KINS + x) * 1024);
    }
#pragma unroll
    for (int x = 0; x < T::VINS; ++x) copy_1k_to_lds(vt, co.v[x], stage + T::KBYTES + (wave * T::VINS + x) * 1024);
}

// NW: 32-row query groups per workgroup (query block = 32 NW rows).  KS: key split -- with KS = 2
// two waves share a query group and each takes one 32-key half of every tile (used for 64-row
// query blocks so that a workgroup still has four waves); their partial (max, sum, O) are merged
// through LDS after the loop and the KS = 0 wave of each pair runs the epilogue.
// STG: stages of the tile ring.  3 in general (copies run two tiles ahead).  2 for lists of at most two critical
// blocks (bf16, no key split): both tiles are requested at the start, the epilogue operands share the stage the
// first tile leaves free, and the smaller LDS footprint lets four workgroups instead of three share a CU, which is
// what a loop this short needs.
template <int NW, int KS, bool FP8, int STG>
__global__ __launch_bounds__(64 * NW * KS, (NW == 2 && KS == 1) ? 2 : 3) void attend_kernel(
    const void *__restrict__ Qp, const void *__restrict__ Kp, const uint16_t *__restrict__ Vp,
    const float *__restrict__ sQ, const float *__restrict__ sK, const float *__restrict__ sV, RowMap rm,
    const int32_t *__restrict__ crit_idx, int k_c, const uint16_t *__restrict__ Hq, const uint16_t *__restrict__ WT,
    int proj_per_head, int phi, int H, int N, int Nqb, int Nkb, long total, float c_exp, uint16_t *__restrict__ O)
{
    constexpr int NWAVES = NW * KS;
    using T = Tile<NWAVES, FP8>;
    constexpr int BQ = 32 * NW;
    constexpr int ES = FP8 ? 1 : 2;                     // bytes per input element
    constexpr int NH = 2 / KS;                          // 32-key halves of a tile this wave processes
    constexpr int NS = 4 / KS;                          // 16-key steps of the second product this wave processes
    static_assert(STG == 3 || (STG == 2 && KS == 1 && !FP8), "the two-stage ring is for unsplit bf16 lists of at most two tiles");
    constexpr int kZBytes = STG == 2 ? 256 : 0;         // two-stage ring: the Z row gets its own slot behind the ring
    __shared__ __attribute__((aligned(1024))) uint8_t lds[STG * T::STAGE + kZBytes];
    const long work = xcd_remap(blockIdx.x, total);
    if (work >= total) return;                        // the whole workgroup leaves together
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, g = lane >> 5;
    const int wq = wave % NW, kh = wave / NW;         // query group and key half (kh = 0 when KS = 1)
    const long bh = work / Nqb;
    const int i = (int)(work - bh * Nqb);
    const int q = i * BQ + 32 * wq + l32;             // this lane's query row
    const bool qok = q < N;
    const size_t head = rm.head(bh);                  // element offset of this (b,h); rows are rm.ts elements apart
    const int krowb = rm.ts * ES;                     // bytes between consecutive K rows
    const uint8_t *Kh = (const uint8_t *)Kp + head * ES;
    const uint8_t *Vh = (const uint8_t *)(Vp + (size_t)bh * Nkb * kBK * kD);

    // Q as the B operand of S^T: bf16 -> 4 K-steps of 8 channels (16s + 8g ..), e4m3 -> 32 channels (32g ..)
    bf16x8 qf[4];
    i32x8 q8;
    if (FP8) {
        uint4 w0 = make_uint4(0, 0, 0, 0), w1 = w0;
        if (qok) {
            const uint8_t *qr = (const uint8_t *)Qp + head + (size_t)q * rm.ts + 32 * g;
            w0 = *(const uint4 *)qr;
            w1 = *(const uint4 *)(qr + 16);
        }
        q8[0] = w0.x; q8[1] = w0.y; q8[2] = w0.z; q8[3] = w0.w; q8[4] = w1.x; q8[5] = w1.y; q8[6] = w1.z; q8[7] = w1.w;
    } else {
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            uint4 w = make_uint4(0, 0, 0, 0);
            if (qok) w = *(const uint4 *)((const uint16_t *)Qp + head + (size_t)q * rm.ts + 16 * s + 8 * g);
            qf[s] = __builtin_bit_cast(bf16x8, w);
        }
    }
    const float qscale = FP8 ? sQ[work] : 1.0f;       // scale blocks of Q are the query blocks

    // per-lane LDS byte offsets of the fragments (swizzled 16-byte chunks):
    //   koff[s]: K row 32 kh + l32 (+32 for the second half when KS = 1), channel chunk of step s
    //   voff[ss]: V^T row l32 (+32 for channels 32..63), key chunk 2 s + g of this wave's step s = NS kh + ss
    int koff[4], voff[NS];
#pragma unroll
    for (int s = 0; s < 4; ++s)
        koff[s] = (FP8 ? l32 * 64 + ((((2 * g + (s & 1)) ^ swz4(l32))) << 4) : l32 * 128 + (((2 * s + g) ^ swz8(l32)) << 4))
                  + kh * 32 * (FP8 ? 64 : 128);
#pragma unroll
    for (int ss = 0; ss < NS; ++ss) voff[ss] = T::KBYTES + l32 * 128 + (((2 * (NS * kh + ss) + g) ^ swz8(l32)) << 4);

    f32x16 zero16;
#pragma unroll
    for (int x = 0; x < 16; ++x) zero16[x] = 0.f;
    f32x16 oacc[2] = {zero16, zero16};
    float m_run = -INFINITY, l_run = 0.f;             // running maximum in the log2 domain, running sum
    const bf16x8 ones = __builtin_bit_cast(bf16x8, make_uint4(0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u));

    const int32_t *ci = crit_idx + work * (long)k_c;
    auto tile_index = [&](int c) {                     // -1: no such tile (list exhausted or entry absent)
        int j = c < k_c ? ci[c] : -1;
        return (j < 0 || j >= Nkb) ? -1 : j;
    };
    CopyOffsets<NWAVES, FP8> co;
    co.init(wave, lane, krowb);
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);                       // same value, provably uniform
    const uint32_t lds_base = (uint32_t)(uintptr_t)(lds_void_p)lds;                // LDS byte address of the ring
    auto request = [&](int c, int j) {
        const int jj = j < 0 ? 0 : j;                  // absent entries still copy (block 0) so the copy count is uniform
        issue_tile<NWAVES, FP8>(lds_base + (c % STG) * T::STAGE, Kh + (size_t)jj * kBK * krowb, Vh + (size_t)jj * kBK * kD * 2,
                                min(kBK, N - jj * kBK), krowb, co, wave_u);
    };
    // The operands of the linear/projection epilogue (the 64x64 tile of Hq^T, the Z row, W^T) travel the
    // same way into the two ring stages that are idle during the last tile, so their latency hides
    // behind that tile's arithmetic.  c_next: index of the first idle stage.
    const uint8_t *Hi8 = Hq ? (const uint8_t *)(Hq + (size_t)work * kStateElems) : nullptr;
    const uint8_t *Wh8 = (const uint8_t *)(WT + (proj_per_head ? (size_t)(bh % H) * kD * kD : 0));
    auto request_epilogue = [&](int c_next) {
        const uint32_t sa = lds_base + (c_next % STG) * T::STAGE;
        const uint32_t sb = STG == 2 ? sa + 8192 : lds_base + ((c_next + 1) % STG) * T::STAGE;
        const uint32_t sz = STG == 2 ? lds_base + STG * T::STAGE : sa + 8192;
#pragma unroll
        for (int x = 0; x < T::VINS; ++x) copy_1k_to_lds(Hi8, co.v[x], sa + (wave_u * T::VINS + x) * 1024);
#pragma unroll
        for (int x = 0; x < T::VINS; ++x) copy_1k_to_lds(Wh8, co.v[x], sb + (wave_u * T::VINS + x) * 1024);
        if (tid < 8) copy_1k_to_lds(Hi8 + 64 * kD * 2, tid * 16, sz);             // Z: 128 bytes, 8 lanes of wave 0
    };
    if (Hq != nullptr && k_c == 0) request_epilogue(0);

    // Key mask of a ragged last block: it enters as the initial accumulator of S^T (0 for real keys,
    // -inf for keys past the end), built on the fly only for such a tile; every other tile starts from 0.
    auto key_mask = [&](int valid, f32x16 (&m)[NH]) {
#pragma unroll
        for (int hh = 0; hh < NH; ++hh)
#pragma unroll
            for (int x = 0; x < 16; ++x)
                m[hh][x] = (32 * (kh + hh) + 8 * (x >> 2) + 4 * g + (x & 3)) < valid ? 0.f : -INFINITY;
    };
    // S^T = K Q^T (+ init) of this wave's key halves of the tile staged at st
    auto compute_S = [&](const uint8_t *st, const f32x16 (&init)[NH], f32x16 (&s2)[NH]) {
        if (FP8) {
#pragma unroll
            for (int hh = 0; hh < NH; ++hh) {
                const uint4 w0 = *(const uint4 *)(st + koff[0] + hh * 32 * 64), w1 = *(const uint4 *)(st + koff[1] + hh * 32 * 64);
                i32x8 k8;
                k8[0] = w0.x; k8[1] = w0.y; k8[2] = w0.z; k8[3] = w0.w; k8[4] = w1.x; k8[5] = w1.y; k8[6] = w1.z; k8[7] = w1.w;
                s2[hh] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(k8, q8, init[hh], 0, 0, 0, 0, 0, 0);
            }
        } else {
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int hh = 0; hh < NH; ++hh) {
                    const bf16x8 kf = *(const bf16x8 *)(st + koff[s] + hh * 32 * 128);
                    s2[hh] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s], s == 0 ? init[hh] : s2[hh], 0, 0, 0);
                }
        }
    };
    int j0 = tile_index(0), j1 = tile_index(1);
    if (k_c > 0) request(0, j0);
    if (k_c > 1) request(1, j1);
    // Let the Q fragments (ordinary loads the compiler tracks) land here, once: left to the compiler, its
    // vmcnt(0) for them would sit in front of their first use inside the loop and drain the ring every trip.
    __builtin_amdgcn_s_waitcnt(0 | (7 << 4) | (15 << 8));

    for (int c = 0; c < k_c; ++c) {
        const int j = j0;
        // copies of tiles 0..c+1 have been requested; tile c has landed once only those of tile c+1 remain
        if (c + 1 < k_c) wait_copies_and_barrier<T::LOADS>();   // tile c visible to all waves; stage of tile c-1 free
        else wait_copies_and_barrier<0>();
        j0 = j1;
        j1 = tile_index(c + 2);
        if (c + 2 < k_c) request(c + 2, j1);
        if (Hq != nullptr && c + 1 == k_c) request_epilogue(c + 1);
        if (j < 0) continue;
        const uint8_t *st = lds + (c % STG) * T::STAGE;
        const int valid = min(kBK, N - j * kBK);
        // exp2 constant of this tile: softmax scale * log2(e) (* Q and K block scales for e4m3)
        const float cj = FP8 ? fmaxf(c_exp * qscale * sK[bh * Nkb + j], 1e-30f) : c_exp;
        // E4M3: the V block scale rides on the weights, P' = P * sV_j (an offset in the exponent); the
        // row sum of P' is divided by sV_j again, so numerator and denominator stay consistent.
        const float svj = FP8 ? fmaxf(sV[bh * Nkb + j], 1e-30f) : 1.0f;
        const float lsv = FP8 ? __log2f(svj) : 0.0f;

        // ---- S^T = K Q^T
        f32x16 sacc[NH];
        if (valid == kBK) {
            f32x16 init[NH];
#pragma unroll
            for (int hh = 0; hh < NH; ++hh) init[hh] = zero16;
            compute_S(st, init, sacc);
        } else {
            f32x16 init[NH];
            key_mask(valid, init);
            compute_S(st, init, sacc);
        }

        // ---- online softmax, one query row per lane (shared with lane^32)
        float mx = sacc[0][0];
#pragma unroll
        for (int hh = 0; hh < NH; ++hh)
#pragma unroll
            for (int x = 0; x < 16; ++x) mx = fmaxf(mx, sacc[hh][x]);
        mx = pair_max(mx);
        // the accumulators are rescaled only in iterations where some row of the wave raised its maximum;
        // a half tile may hold no real key (ragged end): its maximum is -inf and leaves the state alone
        mx *= cj;
        if (__ballot(mx > m_run + kLazyMax)) {
            const float m_new = mx > m_run + kLazyMax ? fmaxf(m_run, mx) : m_run;
            const float alpha = m_new == m_run ? 1.0f : fast_exp2(m_run - m_new);
            m_run = m_new;
            l_run *= alpha;
#pragma unroll
            for (int e = 0; e < 2; ++e)
#pragma unroll
                for (int x = 0; x < 16; ++x) oacc[e][x] *= alpha;
        }
        const float moff = lsv - (m_run == -INFINITY ? 0.f : m_run);
#pragma unroll
        for (int hh = 0; hh < NH; ++hh)
#pragma unroll
            for (int x = 0; x < 16; ++x) sacc[hh][x] = fast_exp2(fmaf(sacc[hh][x], cj, moff));

        // ---- O^T += V^T P^T, and the row sums as ones^T P^T on the same bf16-rounded P, so that
        // numerator and denominator of the softmax see identical weights
        f32x16 lsum;
#pragma unroll
        for (int ss = 0; ss < NS; ++ss) {
            const bf16x8 pf = pack8(sacc[ss >> 1], 8 * (ss & 1));
            lsum = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ones, pf, ss == 0 ? zero16 : lsum, 0, 0, 0);
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const bf16x8 vf = *(const bf16x8 *)(st + voff[ss] + e * 32 * 128);
                oacc[e] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, oacc[e], 0, 0, 0);
            }
        }
        l_run += FP8 ? lsum[0] / svj : lsum[0];        // every row of ones^T P^T is the sum over this wave's keys
    }

    // ring stages after the loop: A, B hold the epilogue operands, L (the last tile's stage) is free
    const int c_next = k_c;
    uint8_t *stA = lds + (c_next % STG) * T::STAGE, *stB = STG == 2 ? stA + 8192 : lds + ((c_next + 1) % STG) * T::STAGE;
    uint8_t *stL = lds + ((c_next + 2) % STG) * T::STAGE;            // used by the key-split merge only (STG == 3)
    const uint8_t *zrow = STG == 2 ? lds + STG * T::STAGE : stA + 8192;
    wait_copies_and_barrier<0>();                      // epilogue operands landed; every wave is past its last tile

    if (KS == 2) {
        // ---- merge the two key halves: the kh = 1 wave parks (O, max, sum) in LDS, its partner folds them in.
        // Four 4 KB slots for the two 32-channel halves of the two parked waves: three in stage L and one
        // behind W^T in stage B (an e4m3 stage is only 12 KB); max/sum go behind the Z row in stage A.
        auto slot = [&](int r) { return r < 3 ? stL + r * 4096 : (T::STAGE >= 16384 ? stL + 12288 : stB + 8192); };
        float *ml = (float *)(stA + 8448) + wq * 128;
        if (kh == 1) {
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                uint8_t *dst = slot(2 * wq + e);
#pragma unroll
                for (int x4 = 0; x4 < 4; ++x4)
                    *(float4 *)(dst + x4 * 1024 + lane * 16) = make_float4(oacc[e][4 * x4], oacc[e][4 * x4 + 1], oacc[e][4 * x4 + 2], oacc[e][4 * x4 + 3]);
            }
            ml[lane] = m_run;
            ml[64 + lane] = l_run;
        }
        wait_copies_and_barrier<0>();
        if (kh == 0) {
            const float m1 = ml[lane], l1 = ml[64 + lane];
            const float m = fmaxf(m_run, m1);
            const float a0 = m_run == m ? 1.0f : fast_exp2(m_run - m), a1 = m1 == m ? 1.0f : fast_exp2(m1 - m);   // -inf - -inf avoided
            l_run = l_run * a0 + l1 * a1;
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const uint8_t *src = slot(2 * wq + e);
#pragma unroll
                for (int x4 = 0; x4 < 4; ++x4) {
                    const float4 o1 = *(const float4 *)(src + x4 * 1024 + lane * 16);
                    oacc[e][4 * x4 + 0] = oacc[e][4 * x4 + 0] * a0 + o1.x * a1;
                    oacc[e][4 * x4 + 1] = oacc[e][4 * x4 + 1] * a0 + o1.y * a1;
                    oacc[e][4 * x4 + 2] = oacc[e][4 * x4 + 2] * a0 + o1.z * a1;
                    oacc[e][4 * x4 + 3] = oacc[e][4 * x4 + 3] * a0 + o1.w * a1;
                }
            }
        }
    }

    // ---- normalise the sparse output
    const float inv_l = l_run > 0.f ? 1.0f / l_run : 0.f;
#pragma unroll
    for (int e = 0; e < 2; ++e)
#pragma unroll
        for (int x = 0; x < 16; ++x) oacc[e][x] *= inv_l;

    if (Hq != nullptr && kh == 0) {
        // ---- phi(Q): softmax over the 64 channels of the row (this lane holds 32, lane^32 the rest).
        // x[8s + c] is channel dcol(s) + c, the channel slot c of K-step s carries in the product below.
        float x[32];
        if (FP8) {
#pragma unroll
            for (int w = 0; w < 8; ++w) {
                const f32x2 lo = __builtin_amdgcn_cvt_pk_f32_fp8(q8[w], false), hi = __builtin_amdgcn_cvt_pk_f32_fp8(q8[w], true);
                x[4 * w + 0] = lo[0] * qscale; x[4 * w + 1] = lo[1] * qscale; x[4 * w + 2] = hi[0] * qscale; x[4 * w + 3] = hi[1] * qscale;
            }
        } else {
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const uint4 w = __builtin_bit_cast(uint4, qf[s]);
                x[8 * s + 0] = bf16_lo(w.x); x[8 * s + 1] = bf16_hi(w.x);
                x[8 * s + 2] = bf16_lo(w.y); x[8 * s + 3] = bf16_hi(w.y);
                x[8 * s + 4] = bf16_lo(w.z); x[8 * s + 5] = bf16_hi(w.z);
                x[8 * s + 6] = bf16_lo(w.w); x[8 * s + 7] = bf16_hi(w.w);
            }
        }
        float inv = 1.0f;
        if (phi == 0) {
            float mx = x[0];
#pragma unroll
            for (int d = 1; d < 32; ++d) mx = fmaxf(mx, x[d]);
            mx = pair_max(mx);
            float sum = 0.f;
#pragma unroll
            for (int d = 0; d < 32; ++d) { x[d] = fast_exp2((x[d] - mx) * kLog2e); sum += x[d]; }
            sum += xchg32(sum);
            inv = 1.0f / sum;
        } else {                                               // ELU(x)+1, elementwise
#pragma unroll
            for (int d = 0; d < 32; ++d) x[d] = x[d] > 0.f ? x[d] + 1.0f : fast_exp2(x[d] * kLog2e);
        }
        bf16x8 fq[4];
        float den = 0.f;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int dcol = FP8 ? 32 * g + 8 * s : 16 * s + 8 * g;
            uint4 o;
            o.x = pack_bf16(x[8 * s + 0] * inv, x[8 * s + 1] * inv); o.y = pack_bf16(x[8 * s + 2] * inv, x[8 * s + 3] * inv);
            o.z = pack_bf16(x[8 * s + 4] * inv, x[8 * s + 5] * inv); o.w = pack_bf16(x[8 * s + 6] * inv, x[8 * s + 7] * inv);
            fq[s] = __builtin_bit_cast(bf16x8, o);
            const uint4 z = *(const uint4 *)(zrow + dcol * 2);
            den += bf16_lo(o.x) * bf16_lo(z.x) + bf16_hi(o.x) * bf16_hi(z.x) + bf16_lo(o.y) * bf16_lo(z.y) + bf16_hi(o.y) * bf16_hi(z.y)
                 + bf16_lo(o.z) * bf16_lo(z.z) + bf16_hi(o.z) * bf16_hi(z.z) + bf16_lo(o.w) * bf16_lo(z.w) + bf16_hi(o.w) * bf16_hi(z.w);
        }
        den += xchg32(den);
        const float inv_den = den > 0.f ? 1.0f / den : 0.f;     // no marginal block: H = Z = 0 and O_lin = 0

        // ---- O_lin^T = Hq^T phi(Q)^T   (Hq^T tile staged with the tile swizzle)
        f32x16 lacc[2];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int hchunk = FP8 ? 4 * g + s : 2 * s + g;      // 16-byte chunk holding channels dcol(s)..dcol(s)+7
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const bf16x8 hf = *(const bf16x8 *)(stA + (32 * e + l32) * 128 + ((hchunk ^ swz8(l32)) << 4));
                lacc[e] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(hf, fq[s], s == 0 ? zero16 : lacc[e], 0, 0, 0);
            }
        }
#pragma unroll
        for (int e = 0; e < 2; ++e)
#pragma unroll
            for (int y = 0; y < 16; ++y) lacc[e][y] *= inv_den;

        // ---- O^T += W^T O_lin^T   (W^T staged transposed and key-permuted like a V^T tile)
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const bf16x8 pf = pack8(lacc[s >> 1], 8 * (s & 1));
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const bf16x8 wf = *(const bf16x8 *)(stB + (32 * e + l32) * 128 + (((2 * s + g) ^ swz8(l32)) << 4));
                oacc[e] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, pf, oacc[e], 0, 0, 0);
            }
        }
    }

    // ---- store.  Register 4a+b of oacc[e] is channel 32e + 8a + 4g + b of row q: the wave's 32x64 tile
    // is transposed through a private 4 KB LDS slice (8-byte pieces, XOR-swizzled by row) so that it
    // leaves as full 128-byte rows, 16 bytes per lane.
    wait_copies_and_barrier<0>();                      // all waves are done reading the ring
    if (kh == 0) {
        uint8_t *ot = lds + wq * 4096;
        const int f = ((l32 >> 1) & 7) << 1;
#pragma unroll
        for (int e = 0; e < 2; ++e)
#pragma unroll
            for (int aa = 0; aa < 4; ++aa) {
                uint2 o;
                o.x = pack_bf16(oacc[e][4 * aa + 0], oacc[e][4 * aa + 1]);
                o.y = pack_bf16(oacc[e][4 * aa + 2], oacc[e][4 * aa + 3]);
                const int piece = 8 * e + 2 * aa + g;
                *(uint2 *)(ot + l32 * 128 + ((piece ^ f) << 3)) = o;
            }
        wave_lds_sync();
        const int q0w = i * BQ + 32 * wq;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int r = 8 * k + (lane >> 3), ch = lane & 7;      // row of the tile, 16-byte chunk of the row
            const int fr = ((r >> 1) & 7) << 1;
            const uint4 v = *(const uint4 *)(ot + r * 128 + (((2 * ch) ^ fr) << 3));
            if (q0w + r < N) *(uint4 *)(O + head + (size_t)(q0w + r) * rm.ts + ch * 8) = v;
        }
    }
}

// W [nW][e_in][e_out] -> WT [nW][e_out][slot] as its own launch (the whole forward folds this into the states pass)
__global__ __launch_bounds__(256) void transpose_w_kernel(const uint16_t *__restrict__ W, uint16_t *__restrict__ WT)
{
    transpose_w_tile(W + (size_t)blockIdx.x * kD * kD, WT + (size_t)blockIdx.x * kD * kD, 256);
}

hipError_t launch_transpose_w(const void *W, int nW, void *WT, hipStream_t st)
{
    transpose_w_kernel<<<nW, 256, 0, st>>>((const uint16_t *)W, (uint16_t *)WT);
    return hipGetLastError();
}

template <int NW, int KS, bool FP8, int STG>
static hipError_t launch_attend_t(const void *Q, const void *K, const void *Vp, const float *sQ, const float *sK, const float *sV, RowMap rm,
                                  const int32_t *crit_idx, int k_c, const void *Hq, const void *WT, int proj_per_head, int phi,
                                  int H, int N, int Nqb, int Nkb, long total, float c_exp, void *O, hipStream_t st)
{
    attend_kernel<NW, KS, FP8, STG><<<(unsigned)xcd_grid(total), 64 * NW * KS, 0, st>>>(Q, K, (const uint16_t *)Vp, sQ, sK, sV, rm, crit_idx, k_c, (const uint16_t *)Hq,
                                                                          (const uint16_t *)WT, proj_per_head, phi, H, N, Nqb, Nkb,
                                                                          total, c_exp, (uint16_t *)O);
    return hipGetLastError();
}

hipError_t launch_attend(const void *Q, const void *K, const void *Vp,
                         const float *sQ, const float *sK, const float *sV, bool fp8, RowMap rm,
                         const int32_t *crit_idx, int k_c, const void *Hq, const void *WT,
                         int proj_per_head, int phi, int B, int H, int N, int bq, float sm_scale,
                         void *O, hipStream_t st)
{
    const int Nqb = (N + bq - 1) / bq, Nkb = (N + kBK - 1) / kBK;
    const long total = (long)B * H * Nqb;
    const float c_exp = sm_scale * kLog2e;
#define SLA_ATT(NW, KS, F8, STG) return launch_attend_t<NW, KS, F8, STG>(Q, K, Vp, sQ, sK, sV, rm, crit_idx, k_c, Hq, WT, proj_per_head, phi, H, N, Nqb, Nkb, total, c_exp, O, st)
    if (bq == 128) { if (fp8) SLA_ATT(4, 1, true, 3); else SLA_ATT(4, 1, false, 3); }
    // 64-row query blocks: two query groups x two key halves, so a workgroup still has four waves;
    // with very few critical blocks per row the merge of the halves costs more than it hides
    if (k_c >= 4) { if (fp8) SLA_ATT(2, 2, true, 3); else SLA_ATT(2, 2, false, 3); }
    if (fp8) SLA_ATT(2, 1, true, 3);
    if (k_c <= 2) SLA_ATT(2, 1, false, 2);
    SLA_ATT(2, 1, false, 3);
#undef SLA_ATT
}

}  // namespace sla
