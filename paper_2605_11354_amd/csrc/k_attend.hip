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
// With the 32x32x16 MFMA a lane holds column q = lane%32 of the 32x32 result, rows
// 8a + 4g + b (g = lane/32; register 4a+b).  The B operand of the second product takes
// accumulator registers 8u..8u+7, i.e. keys 16s + 8a' + 4g + b; the V^T rows are read with
// exactly that key permutation: the states kernel leaves V^T of every key block in that order,
// so a V^T fragment is one 16-byte LDS read like a K fragment.
// Template parameters: NW query groups of 32 rows (2 for 64-row, 4 for 128-row query blocks), one wave each.  (An earlier
// form split every tile of a 64-row block between two wave pairs that merged their partial results through LDS; with
// the software pipeline below two waves per workgroup are faster at every list length, 13 to 16 % on lists of 9 and 34.)
//
// Arithmetic of the weights.  P is rounded to fp16 (11 significant bits) and V^T arrives as fp16 from the states
// kernel (bf16 or E4M3 values are exact in fp16 once divided by the power of two the states kernel picks per key
// block; its base-2 logarithm comes in `lvs` and is added to the exponent of the weights, so the product is
// unchanged).  The second product runs on the fp16 MFMA at the rate of the bf16 one with an eighth of the rounding
// error on the weights.  That margin pays for a running maximum that is only raised when a lane sees an exponent
// above kRaise: the accumulators are rescaled a few times per row instead of once per tile, and the softmax of a
// 32-key unit needs nothing from other lanes before its exponentials.
//
// Software pipeline.  The work of a wave is a stream of units (32 keys x 32 queries).  In step u the matrix unit
// runs O += V P of unit u-1 and S of unit u+1 while the vector unit runs the softmax of unit u; the three have no
// dependency on each other, so MFMA and VALU instructions alternate in one basic block (scheduling barriers and
// value pins below hold the order).  Everything with control flow (raising the maximum, the first unit of a row, a
// ragged key block, a key block whose V scale is far below the first one's) sits between the steps or in the
// "careful" variant of a step.  In the middle of a list, where none of the special cases can occur (one bit per list
// entry says so), iterations run three at a time in a form without guards.
//
// Memory pipeline.  K and V^T tiles go from global memory straight into LDS (global_load_lds_dwordx4, no staging
// registers) into two rings of three slots each.  K runs ahead of V^T by the pipeline's skew, so the copies of an
// iteration are needed two iterations later; one workgroup barrier per tile publishes what has landed and frees
// the slots that were consumed.  Rows are stored unpadded with the 16-byte chunk index XOR-ed by row bits (applied
// on the global side of the copy), which keeps the fragment reads free of bank conflicts.  The copies are inline
// assembly, invisible to the compiler's wait-count insertion, and are awaited by explicit s_waitcnt vmcnt(n).
//
// E4M3 inputs.  S^T is one v_mfma_f32_32x32x64_f8f6f4 per 32 keys (the whole head dimension is the K dimension of
// the instruction; products of two E4M3 numbers are exact in the fp32 accumulator), with the per-block scales
// folded into the exp2 constant.  P is NOT cast to E4M3: three mantissa bits on the softmax weights put the output
// error at several percent of its RMS, above the 6e-2 bar; the second product is the fp16 one described above, with
// the V block scale in the exponent of the weights.
//
// Epilogue (per wave, all MFMA): O_lin^T = Hq^T-tile x phi(Q)^T, scaled by 1/(phi(Q).Z),
// then O^T += W^T x O_lin^T accumulated onto the normalised sparse output, stored as bf16.
#include "sla_common.hpp"
#include "sla_kernels.hpp"

#include <type_traits>

namespace sla {

constexpr float kLog2e = 1.4426950408889634f;
// A lane raises the running maximum of its row when a weight of the current unit would exceed 2^kRaise times
// the largest weight seen when the maximum was last set; fp16 holds 2^kRaise with room to spare (max 65504).
constexpr float kRaise = 12.0f;
// A key block whose V scale differs from that of the row's first block by more than 2^kTinyV either way takes the
// careful step: its weights (or the factor that divides the scale out of the row sums again) would leave the range
// of fp16, so its row sums are formed in fp32.
constexpr float kTinyV = 8.0f;

typedef __attribute__((address_space(3))) void *lds_void_p;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;

// XOR swizzle of 16-byte chunks: 8 chunks per 128-byte row / 4 chunks per 64-byte row
__device__ __forceinline__ int swz8(int row) { return (row >> 1) & 7; }
__device__ __forceinline__ int swz4(int row) { return (row >> 2) & 3; }

// Waits until at most N of this wave's tile copies are outstanding and its LDS reads have returned, then joins
// the workgroup.  The copies below are issued from inline assembly so that the compiler's own wait-count
// insertion does not see them: it would otherwise drain ALL outstanding copies (vmcnt(0)) before every LDS read
// and serialise the prefetch ring.  The waits are therefore explicit.
template <int N> __device__ __forceinline__ void wait_copies_and_barrier()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
#ifdef SLA_PROBE_NOBARRIER   /* timing probe only (results are wrong): how much of the time is waves waiting for each other */
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_waitcnt lgkmcnt(0)" ::"n"(N) : "memory");
#else
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_waitcnt lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
#endif
}

// N such copies from the same base to consecutive kilobytes of LDS (per-lane offsets voff[0..N-1]) in one statement
template <int N> __device__ __forceinline__ void copy_nk_to_lds(const uint8_t *base, const int (&voff)[N], uint32_t lds_addr)
{
    static_assert(N == 1 || N == 2 || N == 4, "1, 2 or 4 copies");
    uint32_t saved_m0;
    if constexpr (N == 1) {
        copy_1k_to_lds(base, voff[0], lds_addr);
    } else if constexpr (N == 2) {
        asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %4\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %3\n\t"
                     "s_add_u32 m0, m0, 0x400\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3\n\ts_mov_b32 m0, %0"
                     : "=&s"(saved_m0) : "v"(voff[0]), "v"(voff[1]), "s"(base), "s"(lds_addr) : "memory", "scc");
    } else {
        asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %6\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %5\n\t"
                     "s_add_u32 m0, m0, 0x400\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %5\n\t"
                     "s_add_u32 m0, m0, 0x400\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %3, %5\n\t"
                     "s_add_u32 m0, m0, 0x400\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %4, %5\n\ts_mov_b32 m0, %0"
                     : "=&s"(saved_m0) : "v"(voff[0]), "v"(voff[1]), "v"(voff[2]), "v"(voff[3]), "s"(base), "s"(lds_addr) : "memory", "scc");
    }
}

__device__ __forceinline__ uint32_t pack_f16(float lo, float hi)
{
    f16x2 r;
    r[0] = (_Float16)lo;
    r[1] = (_Float16)hi;
    return __builtin_bit_cast(uint32_t, r);
}
__device__ __forceinline__ f16x8 pack8_f16(const f32x16 &a, int base)
{
    uint4 o;
    o.x = pack_f16(a[base + 0], a[base + 1]); o.y = pack_f16(a[base + 2], a[base + 3]);
    o.z = pack_f16(a[base + 4], a[base + 5]); o.w = pack_f16(a[base + 6], a[base + 7]);
    return __builtin_bit_cast(f16x8, o);
}
__device__ __forceinline__ float max3(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }
// largest of the 16 values a lane holds of one unit of S^T
__device__ __forceinline__ float max16(const f32x16 &s)
{
    const float a = max3(s[0], s[1], s[2]), b = max3(s[3], s[4], s[5]), c = max3(s[6], s[7], s[8]);
    const float d = max3(s[9], s[10], s[11]), e = max3(s[12], s[13], s[14]);
    return max3(max3(a, b, c), max3(d, e, s[15]), a);
}

template <int NWAVES, bool FP8, int NSLOTS = 3>
struct Tile {
    static constexpr int KBYTES = FP8 ? 64 * 64 : 64 * 128;     // K tile (e4m3 / bf16)
    static constexpr int VBYTES = 64 * 128;                     // V^T tile (always fp16)
    static constexpr int KINS = KBYTES / 1024 / NWAVES;         // 1 KB copy instructions per wave
    static constexpr int VINS = VBYTES / 1024 / NWAVES;
    static constexpr int LOADS = KINS + VINS;                   // per wave per tile
    static constexpr int SLOTS = NSLOTS;                        // slots of the K ring and of the V^T ring
    static constexpr int VRING = SLOTS * KBYTES;                // the V^T ring follows the K ring
    // behind the rings: a 256-byte slot for the Z row, and, for E4M3 inputs (whose K ring is too small for both
    // epilogue operands), 8 KB for W^T
    static constexpr int ZOFF = SLOTS * (KBYTES + VBYTES);
    static constexpr int WOFF = ZOFF + 256;
    static constexpr int LDS = WOFF + (FP8 ? 8192 : 0);
};

// Per-lane byte offsets (inside a tile) of the 16-byte chunk each lane copies, one per copy
// instruction of this wave: LDS position (row, slot) <- global chunk slot ^ swizzle(row).
template <int NWAVES, bool FP8>
struct CopyOffsets {
    using T = Tile<NWAVES, FP8>;
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

template <bool B> using flag = std::integral_constant<bool, B>;

#ifdef SLA_PROBE_TIME   /* timing probe only: cycle counter of one wave at five points of every tile */
__device__ unsigned long long sla_wg_times[2 * 32768];      // 100 MHz clock at the start and the end of every workgroup (the first 32768)
__device__ unsigned long long sla_probe_times[64 * 8];
#define SLA_TP(row, pt) do { if (probe_on) { const unsigned long long t_ = __builtin_readcyclecounter(); if (lane == 0) tprobe[(row) * 8 + (pt)] = t_; } } while (0)
#define SLA_T(c, pt) do { if ((c) < 61) SLA_TP(c, pt); } while (0)      /* rows 61..63: epilogue, prologue, wave life */
#else
#define SLA_TP(row, pt)
#define SLA_T(c, pt)
#endif

// NW: 32-row query groups per workgroup (query block = 32 NW rows), one wave per group.
// SL: ring slots (three: the pipeline described above).
template <int NW, bool FP8, int SL>
__global__ __launch_bounds__(64 * NW, 2) void attend_kernel(
    const void *__restrict__ Qp, const void *__restrict__ Kp, const uint16_t *__restrict__ Vp, const float *__restrict__ lvs,
    const float *__restrict__ sQ, const float *__restrict__ sK, RowMap rm,
    const int32_t *__restrict__ crit_idx, int k_c, const uint16_t *__restrict__ Hq, const uint16_t *__restrict__ WT,
    int proj_per_head, int phi, int H, int N, int Nqb, int Nkb, long total, float c_exp, uint16_t *__restrict__ O, float *__restrict__ O32)
{
    constexpr int NWAVES = NW;
    using T = Tile<NWAVES, FP8, SL>;
    static_assert(SL == 3, "the pipeline below needs three ring slots");
    constexpr int BQ = 32 * NW;
    constexpr int ES = FP8 ? 1 : 2;                     // bytes per input element
    constexpr int KROWB = FP8 ? 64 : 128;               // bytes of a K row in LDS
    __shared__ __attribute__((aligned(1024))) uint8_t lds[T::LDS];
    // All kernel arguments are fetched here, in one batch of scalar loads: left to the compiler each would be loaded in
    // front of its first use, a dozen scalar-cache round trips one after the other along the prologue and the epilogue.
    asm volatile("" ::"s"(Qp), "s"(Kp), "s"(Vp), "s"(lvs), "s"(sQ), "s"(sK), "s"(rm.bs), "s"(rm.hs), "s"(rm.ts), "s"(rm.H), "s"(crit_idx),
                 "s"(k_c), "s"(Hq), "s"(WT), "s"(proj_per_head), "s"(phi), "s"(H), "s"(N), "s"(Nqb), "s"(Nkb), "s"(total), "s"(c_exp), "s"(O), "s"(O32));
    const long work = xcd_remap(blockIdx.x, total);
    if (work >= total) return;                        // the whole workgroup leaves together
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, g = lane >> 5;
#ifdef SLA_PROBE_TIME
    __shared__ unsigned long long tprobe[64 * 8];
#ifdef SLA_PROBE_PAD
    __shared__ uint8_t lds_pad[SLA_PROBE_PAD];
    if (Nqb < 0) lds_pad[tid] = 1;                    // keeps the array
#endif
    const bool probe_on = __builtin_amdgcn_readfirstlane((int)(work == total / 2 + 3 && wave == 1)) != 0;
    const unsigned long long tp_c0 = __builtin_readcyclecounter(), tp_r0 = __builtin_amdgcn_s_memrealtime();
    if (tid == 0 && work < 32768) sla_wg_times[2 * work] = tp_r0;
#endif
    const int wq = wave;                              // query group of this wave
    const long bh = (long)((unsigned)work / (unsigned)Nqb);      // (the grid fits 32 bits)
    const int i = (int)(work - bh * Nqb);
    const int q = i * BQ + 32 * wq + l32;             // this lane's query row
    const bool qok = q < N;
    const size_t head = rm.head(bh);                  // element offset of this (b,h); rows are rm.ts elements apart
    const int krowb = rm.ts * ES;                     // bytes between consecutive K rows
    const uint8_t *Kh = (const uint8_t *)Kp + head * ES;
    const uint8_t *Vh = (const uint8_t *)(Vp + (size_t)bh * Nkb * kBK * kD);
    const float *lvh = lvs + bh * Nkb;

    SLA_TP(62, 0);
    // The critical list of the row is asked for first of all: the tile copies, the scale gather and with them the whole
    // prologue wait for it (loads return in order: behind the Q rows it would arrive after them).
    const int32_t *ci = crit_idx + work * (long)k_c;
    const int j0_first = lane < k_c ? ci[lane] : -1;
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

    // per-lane LDS byte offsets of the fragments inside a tile (swizzled 16-byte chunks):
    //   koff[s]: K row l32 of a 32-key half, channel chunk of step s
    //   voff[st]: V^T row l32 (+32 for channels 32..63), key chunk 2 st + g of 16-key step st of the tile
    int koff[4], voff[4];
#pragma unroll
    for (int s = 0; s < 4; ++s)
        koff[s] = FP8 ? l32 * 64 + ((((2 * g + (s & 1)) ^ swz4(l32))) << 4) : l32 * 128 + (((2 * s + g) ^ swz8(l32)) << 4);
#pragma unroll
    for (int st = 0; st < 4; ++st) voff[st] = l32 * 128 + (((2 * st + g) ^ swz8(l32)) << 4);

    f32x16 zero16;
#pragma unroll
    for (int x = 0; x < 16; ++x) zero16[x] = 0.f;
    f32x16 oacc[2] = {zero16, zero16};
    // Running state of the lane's row.  m_run: reference exponent (log2 domain) of the weights; l_part: this lane's
    // share of the row sum, accumulated from the fp16 weights the second product consumes (divided by the V scale
    // ratio again); l_full: row sums formed in fp32 by the careful steps (already complete over the lane pair).
    float m_run = -INFINITY, l_part = 0.f, l_alt = 0.f, l_full = 0.f;      // (l_alt: second partial sum of the fast steps)

    // Ragged block: only the last key block of the sequence can be short.
    const int tail_rows = N & (kBK - 1), ragged_j = tail_rows ? Nkb - 1 : -1;
    // The list lives in registers, one entry per lane, as a window of 64 entries starting at wbase (a multiple of 32):
    // block index, log2 of its V scale and (e4m3) its exp2 constant.  The loop takes what it needs with v_readlane,
    // so no scalar load (and none of their waits) sits between the steps; the window moves every 32 tiles.
    int wbase = 0, d_j = 0;
    float d_lv = 0.f, d_cj = 0.f, lv_ref = 0.f;
    // One bit per window entry: set if its tile needs the guarded form of an iteration (past the end of the list,
    // the ragged last block, a V scale far from the first tile's).
    unsigned long long d_bad = ~0ull;
    // k: number of leading valid entries of the list (a list taken from given labels may end in -1 entries)
    int k = 0;
    {
        const int j0 = j0_first;                        // the first window doubles as the first chunk of the count
        unsigned long long ok = __ballot(j0 >= 0 && j0 < Nkb);
        d_j = (j0 >= 0 && j0 < Nkb) ? j0 : 0;
        if (ok != ~0ull) k = __builtin_ctzll(~ok);
        else {
            k = 64;
            for (int base = 64; base < k_c; base += 64) {
                const int idx = base + lane;
                const int j = idx < k_c ? ci[idx] : -1;
                ok = __ballot(j >= 0 && j < Nkb);
                if (ok == ~0ull) { k += 64; continue; }
                k += __builtin_ctzll(~ok);
                break;
            }
        }
        k = __builtin_amdgcn_readfirstlane(k);
    }
    // the scales of the window's blocks: a gather that depends on the indices (the first tile copies are requested
    // between the two, see the prologue)
    auto load_window_scales = [&](bool first) __attribute__((always_inline)) {
        float lv = lvh[d_j];
        // exp2 constant of the tile: softmax scale * log2(e) (* Q and K block scales for e4m3)
        d_cj = FP8 ? fmaxf(c_exp * qscale * sK[bh * Nkb + d_j], 1e-30f) : c_exp;
        asm volatile("" : "+v"(lv), "+v"(d_cj));       // the loads complete here, not at some later first use
        // log2 of the V scale of the first tile: the reference of the weights
        if (first) lv_ref = __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(lv)));
        d_lv = lv - lv_ref;
        d_bad = __ballot(wbase + lane >= k || d_j == ragged_j || !(fabsf(d_lv) <= kTinyV));
    };
    auto load_window = [&](int wb) __attribute__((always_inline)) {
        const int idx = wb + lane;
        d_j = idx < k ? ci[idx] : 0;
        asm volatile("" : "+v"(d_j));
        wbase = wb;
        load_window_scales(false);
    };
    auto entry_j = [&](int c) { return __builtin_amdgcn_readlane(d_j, c - wbase); };

    SLA_TP(62, 1);
    CopyOffsets<NWAVES, FP8> co;
    co.init(wave, lane, krowb);
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);                       // same value, provably uniform
    const uint32_t lds_base = (uint32_t)(uintptr_t)(lds_void_p)lds;                // LDS byte address of the K ring
    const uint32_t ktile_bytes = (uint32_t)kBK * (uint32_t)krowb;                  // bytes from one K block to the next
    const uint32_t kdst0 = lds_base + wave_u * T::KINS * 1024, vdst0 = lds_base + T::VRING + wave_u * T::VINS * 1024;
    // slot: byte offset of the ring slot (a multiple of the tile size below 3 tiles)
    auto request_K = [&](int c, uint32_t slot, bool full = false) __attribute__((always_inline)) {       // K tile of list entry c into the slot at byte offset `slot` of the K ring (full: known not to be the ragged block)
#ifdef SLA_PROBE_NOCOPY
        return;
#endif
        const uint32_t j = (uint32_t)entry_j(c);
        const uint8_t *kt = Kh + (uint64_t)j * ktile_bytes;
        if (full || (int)j != ragged_j) {
            copy_nk_to_lds<T::KINS>(kt, co.k, kdst0 + slot);
        } else {                                       // rows past the end are clamped to the last one; they are masked later
#pragma unroll
            for (int x = 0; x < T::KINS; ++x)
                copy_1k_to_lds(kt, co.k[x] - (co.krow[x] - min(co.krow[x], tail_rows - 1)) * krowb, kdst0 + slot + x * 1024);
        }
    };
    auto request_V = [&](int c, uint32_t slot) __attribute__((always_inline)) {       // V^T tile of list entry c into the slot at byte offset `slot` of the V^T ring
#ifdef SLA_PROBE_NOCOPY
        return;
#endif
        const uint8_t *vt = Vh + (uint64_t)(uint32_t)entry_j(c) * (uint32_t)(kBK * kD * 2);
        copy_nk_to_lds<T::VINS>(vt, co.v, vdst0 + slot);
    };
    // The operands of the linear/projection epilogue (the 64x64 tile of Hq^T, the Z row, W^T) travel the same way
    // into the K ring, which is idle during the last tile, so their latency hides behind that tile's arithmetic.
    const uint8_t *Hi8 = Hq ? (const uint8_t *)(Hq + (size_t)work * kStateElems) : nullptr;
    const uint8_t *Wh8 = (const uint8_t *)(WT + (proj_per_head ? (size_t)((unsigned)bh % (unsigned)H) * kD * kD : 0));
    constexpr int kHqOff = 0, kWtOff = FP8 ? T::WOFF : 8192;
    auto request_epilogue = [&]() __attribute__((always_inline)) {
        if (Hq == nullptr) return;
#pragma unroll
        for (int x = 0; x < T::VINS; ++x) copy_1k_to_lds(Hi8, co.v[x], lds_base + kHqOff + (wave_u * T::VINS + x) * 1024);
#pragma unroll
        for (int x = 0; x < T::VINS; ++x) copy_1k_to_lds(Wh8, co.v[x], lds_base + kWtOff + (wave_u * T::VINS + x) * 1024);
        if (tid < 8) copy_1k_to_lds(Hi8 + 64 * kD * 2, tid * 16, lds_base + T::ZOFF);   // Z: 128 bytes, 8 lanes of wave 0
    };

    // ---- per-tile constants (wave-uniform)
    struct TileInfo { int valid; float cj, lsv, invr; bool tiny; };
    auto tile_info = [&](int c) __attribute__((always_inline)) {
        TileInfo t;
        t.valid = entry_j(c) == ragged_j ? tail_rows : kBK;
        t.cj = FP8 ? __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(d_cj), c - wbase)) : c_exp;
        t.lsv = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(d_lv), c - wbase));   // the V scale of the tile rides on the weights: P' = P * 2^lsv
        t.tiny = fabsf(t.lsv) > kTinyV;
        t.invr = fast_exp2(-t.lsv);                    // and is divided out of the row sums again
        return t;
    };

    // ---- pieces of a step.  Unit u of a wave is the 32-key half `half` of tile c: u = 2 c + half
    // S^T of a unit: K rows 32 half .. 32 half + 31 of the tile in K slot c % 3
    // kbase / vbase: byte offset of a slot of the K ring / of the V^T ring (wave-uniform); the per-lane part koff / voff
    // is added once per slot, the half of the tile is an immediate offset of the read (K) or picks the register (V^T)
    auto k_frag_addr = [&](int kbase, int half, int s) {
        return lds + half * 32 * KROWB + (kbase + koff[s]);
    };
    auto v_frag_addr = [&](int vbase, int half, int ss, int e) {
        return lds + e * 32 * 128 + (vbase + voff[2 * half + ss]);
    };
    // key mask of a ragged block as the initial accumulator: 0 for real keys, -inf for keys past the end
    auto s_init = [&](int valid, int half) {
        f32x16 m;
#pragma unroll
        for (int x = 0; x < 16; ++x) m[x] = (32 * half + 8 * (x >> 2) + 4 * g + (x & 3)) < valid ? 0.f : -INFINITY;
        return m;
    };
    struct KFrag { i32x4 w[FP8 ? 2 : 4]; };
    struct VFrag { f16x8 f[2][2]; };                   // [16-key step][channel half]
    auto load_kfrag = [&](int kbase, int half) __attribute__((always_inline)) {
        KFrag f;
#ifdef SLA_PROBE_NOLDS
        for (int s = 0; s < (FP8 ? 2 : 4); ++s) f.w[s] = i32x4{kbase, half, s, 1};
        return f;
#endif
#pragma unroll
        for (int s = 0; s < (FP8 ? 2 : 4); ++s) f.w[s] = *(const i32x4 *)k_frag_addr(kbase, half, s);
        return f;
    };
    auto load_vfrag = [&](int vbase, int half) __attribute__((always_inline)) {
        VFrag f;
#ifdef SLA_PROBE_NOLDS
        for (int ss = 0; ss < 2; ++ss) for (int e = 0; e < 2; ++e) f.f[ss][e] = __builtin_bit_cast(f16x8, i32x4{vbase, half, ss, e});
        return f;
#endif
#pragma unroll
        for (int ss = 0; ss < 2; ++ss)
#pragma unroll
            for (int e = 0; e < 2; ++e) f.f[ss][e] = *(const f16x8 *)v_frag_addr(vbase, half, ss, e);
        return f;
    };
    auto compute_S = [&](const KFrag &kf, const f32x16 &init) __attribute__((always_inline)) {
        f32x16 s;
        if (FP8) {
            i32x8 k8;
            k8[0] = kf.w[0][0]; k8[1] = kf.w[0][1]; k8[2] = kf.w[0][2]; k8[3] = kf.w[0][3];
            k8[4] = kf.w[1][0]; k8[5] = kf.w[1][1]; k8[6] = kf.w[1][2]; k8[7] = kf.w[1][3];
            s = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(k8, q8, init, 0, 0, 0, 0, 0, 0);
        } else {
            s = init;
#pragma unroll
            for (int st = 0; st < 4; ++st)
                s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kf.w[st]), qf[st], s, 0, 0, 0);
        }
        return s;
    };
    // O^T += V^T P^T of one unit, and the lane's share of its row sums from the same fp16 weights
    struct Weights { f16x8 p[2]; float invr; };        // invr = 0: the row sums of this unit were formed elsewhere
    auto accumulate = [&](const VFrag &vf, const Weights &w) __attribute__((always_inline)) {
        const f16x2 iv = {(_Float16)w.invr, (_Float16)w.invr};
#pragma unroll
        for (int ss = 0; ss < 2; ++ss) {
#pragma unroll
            for (int e = 0; e < 2; ++e) oacc[e] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf.f[ss][e], w.p[ss], oacc[e], 0, 0, 0);
            const uint4 pw = __builtin_bit_cast(uint4, w.p[ss]);
            l_part = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, pw.x), iv, l_part, false);
            l_part = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, pw.y), iv, l_part, false);
            l_part = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, pw.z), iv, l_part, false);
            l_part = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, pw.w), iv, l_part, false);
        }
    };
    auto rescale = [&](float alpha) __attribute__((always_inline)) {
        l_part *= alpha;
        l_alt *= alpha;
        l_full *= alpha;
#pragma unroll
        for (int e = 0; e < 2; ++e)
#pragma unroll
            for (int x = 0; x < 16; ++x) oacc[e][x] *= alpha;
    };
    // Careful form (first unit of a row, ragged or tiny-scale tiles): exact maximum of the unit, row sums in fp32
    // from weights that do not carry the V scale.
    auto softmax_careful = [&](f32x16 &s, const TileInfo &t, Weights &w) __attribute__((always_inline)) {
        const float top = pair_max(max16(s)) * t.cj + t.lsv;        // -inf if the lane's row sees no real key in this unit
        if (__ballot(top > m_run)) {
            const float m_new = fmaxf(m_run, top);
            rescale(m_new == m_run ? 1.0f : fast_exp2(m_run - m_new));
            m_run = m_new;
        }
        const float mfin = m_run == -INFINITY ? 0.f : m_run;
        const float r = fast_exp2(t.lsv);
        float sum = 0.f;
#pragma unroll
        for (int x = 0; x < 16; ++x) {
            const float pu = fast_exp2(fmaf(s[x], t.cj, -mfin));   // weight without the V scale: what the row sum adds up
            sum += pu;
            s[x] = pu * r;                                          // weight with it: what multiplies the scaled V^T
        }
        l_full += sum + xchg32(sum);
        w.p[0] = pack8_f16(s, 0);
        w.p[1] = pack8_f16(s, 8);
        w.invr = 0.f;
    };

    // ---- prologue: the first copies, Q, and S^T of unit 0
    if (k == 0) request_epilogue();
    if (k > 0) request_K(0, 0);
    if (k > 1) request_K(1, T::KBYTES);
    if (k > 2) request_K(2, 2 * T::KBYTES);
    if (k > 0) request_V(0, 0);
    if (k > 1) request_V(1, T::VBYTES);
    SLA_TP(62, 2);
    load_window_scales(true);
    // Let the Q fragments (ordinary loads the compiler tracks) and the first tiles land here, once: left to the
    // compiler, its vmcnt(0) for Q would sit in front of their first use inside the loop and drain the ring every trip.
    SLA_TP(62, 3);
    __builtin_amdgcn_s_waitcnt(0 | (7 << 4) | (15 << 8));      // vmcnt(0), as a builtin so that the compiler's bookkeeping sees it
    wait_copies_and_barrier<0>();
    SLA_TP(62, 4);

    // Units of this wave: u = 2 c + hh is the 32-key half hh of tile c.  Step u accumulates unit u-1
    // (V^T fragments vf_use), forms S^T of unit u+1 (K fragments kf_use) and runs the softmax of unit u; meanwhile the
    // fragments of step u+1 are read from LDS (vf_pre, kf_pre), so that a slot is done with one step before its
    // arithmetic and the LDS latency is off the critical path.
    auto unit_tile = [&](int u) { return u >> 1; };
    auto unit_half = [&](int u) { return u & 1; };
    f32x16 s_cur = zero16;
    Weights w_prev;
    w_prev.p[0] = w_prev.p[1] = __builtin_bit_cast(f16x8, make_uint4(0, 0, 0, 0));
    w_prev.invr = 0.f;
    KFrag kf_use, kf_pre;
    VFrag vf_use, vf_pre;
    TileInfo t_cur, t_nxt;
    const int U = 2 * k;                               // units of this wave
    if (k > 0) {
        t_cur = tile_info(0);
        s_cur = compute_S(load_kfrag(0, unit_half(0)), t_cur.valid == kBK ? zero16 : s_init(t_cur.valid, unit_half(0)));
        if (U > 1) kf_use = load_kfrag(unit_tile(1) * T::KBYTES, unit_half(1));     // for S^T of unit 1, formed in step 0
    }

    SLA_TP(62, 5);
#define SLA_SB() __builtin_amdgcn_sched_barrier(0)
#define SLA_PIN(...) asm volatile("" : __VA_ARGS__)
    // Whether some lane's largest exponent in the unit whose S^T is s would exceed kRaise against the lane's running
    // maximum (stale by that much, or still -inf): such a unit takes the careful step, which raises the maximum exactly.
    auto overflows = [&](const f32x16 &s, const TileInfo &t) __attribute__((always_inline)) {
        return __ballot(!(fmaf(max16(s), t.cj, t.lsv - m_run) <= kRaise)) != 0;
    };
    bool over_cur = true;                              // the first unit is careful anyway

    // One step of the pipeline (see above), careful form: exact softmax, no particular instruction order.
    // t: tile of unit u; tn, half_n: tile and half of unit u+1 (key mask of a ragged block); has_pv / has_s: unit u-1 /
    // u+1 exists; (cv, hv) / (ck, hk): ring slot (byte offset) and half whose V^T / K fragments step u+1 will use.
    auto careful_step = [&](bool has_pv, bool has_s, const TileInfo &t, const TileInfo &tn, int half_n, int cv, int hv, int ck, int hk)
                            __attribute__((always_inline)) {
        f32x16 s_nxt = zero16;
        Weights w;
        vf_pre = load_vfrag(cv, hv);                   // always in bounds (a slot of the ring); unused if there is no such step
        kf_pre = load_kfrag(ck, hk);
        if (has_pv) accumulate(vf_use, w_prev);
        if (has_s) s_nxt = compute_S(kf_use, tn.valid == kBK ? zero16 : s_init(tn.valid, half_n));
        softmax_careful(s_cur, t, w);
        over_cur = has_s ? overflows(s_nxt, tn) : true;
        s_cur = s_nxt; w_prev = w; vf_use = vf_pre; kf_use = kf_pre;
    };
    // Fast form (a unit in the middle of the list, full tiles, no exponent above kRaise), written out in issue order:
    // one MFMA, then a share of the vector work (staggered: exponentials of one pair of weights, the pack of the pair
    // before, the multiply-adds of the pair after) (the matrix unit needs 32 cycles per MFMA, the share of vector work
    // about as long).  The order is held by data dependencies the compiler cannot see through: every share ends in
    // an empty asm statement that "rewrites" the results of the share and the exponent offset the next one starts
    // from, so nothing can move from one share into another (the instruction selector would otherwise bunch the MFMAs
    // that open a new accumulator at the end of the block, and the exponentials behind them), and in a scheduling
    // barrier for the later passes.  The running maximum stays where it is.  The step ends with the overflow check of
    // the next unit, while the last MFMA runs.
    auto fast_step = [&](const TileInfo &t, const TileInfo &tn, int cv, int hv, int ck, int hk) __attribute__((always_inline)) {
        f32x16 s_nxt = zero16;
        Weights w;
        vf_pre = load_vfrag(cv, hv);
        kf_pre = load_kfrag(ck, hk);
        const f16x2 iv = {(_Float16)w_prev.invr, (_Float16)w_prev.invr};
        uint32_t pw[8];
        float moff = t.lsv - m_run;
        auto pv = [&](int ss, int e) { oacc[e] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf_use.f[ss][e], w_prev.p[ss], oacc[e], 0, 0, 0); };
        auto sm = [&](int st) {
            if (FP8) {
                i32x8 k8;
                k8[0] = kf_use.w[0][0]; k8[1] = kf_use.w[0][1]; k8[2] = kf_use.w[0][2]; k8[3] = kf_use.w[0][3];
                k8[4] = kf_use.w[1][0]; k8[5] = kf_use.w[1][1]; k8[6] = kf_use.w[1][2]; k8[7] = kf_use.w[1][3];
                s_nxt = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(k8, q8, zero16, 0, 0, 0, 0, 0, 0);
            } else {
                s_nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kf_use.w[st]), qf[st], s_nxt, 0, 0, 0);
            }
        };
        auto fm = [&](int x0, int x1) {
#pragma unroll
            for (int x = x0; x <= x1; ++x) s_cur[x] = fmaf(s_cur[x], t.cj, moff);
        };
        auto ex = [&](int x0, int x1) {
#pragma unroll
            for (int x = x0; x <= x1; ++x) s_cur[x] = fast_exp2(s_cur[x]);
        };
        auto cv2 = [&](int pr) { pw[pr] = pack_f16(s_cur[2 * pr], s_cur[2 * pr + 1]); };
        auto dots = [&](int ss) {
            const uint4 q4 = __builtin_bit_cast(uint4, w_prev.p[ss]);
            l_part = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, q4.x), iv, l_part, false);
            l_alt = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, q4.y), iv, l_alt, false);
            l_part = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, q4.z), iv, l_part, false);
            l_alt = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, q4.w), iv, l_alt, false);
        };
        SLA_SB();
        if (!FP8) {
            // S^T of the next unit first: its last MFMA then has four more behind it before the step ends with the
            // overflow check on its result (and the next step starts with its exponentials)
            // the vector work of a share is staggered: the exponentials of pair i, the pack of pair i-1 (whose
            // exponentials have left the quarter-rate pipe by now) and the multiply-adds of pair i+1
            fm(0, 1);
            sm(0);    ex(0, 1);   fm(2, 3);
            SLA_PIN("+v"(s_nxt), "+v"(moff)); SLA_SB();
            sm(1);    ex(2, 3);   cv2(0); fm(4, 5);
            SLA_PIN("+v"(s_nxt), "+v"(moff), "+v"(pw[0])); SLA_SB();
            sm(2);    ex(4, 5);   cv2(1); fm(6, 7);
            SLA_PIN("+v"(s_nxt), "+v"(moff), "+v"(pw[1])); SLA_SB();
            sm(3);    ex(6, 7);   cv2(2); fm(8, 9);
            SLA_PIN("+v"(s_nxt), "+v"(moff), "+v"(pw[2])); SLA_SB();
            pv(0, 0); ex(8, 9);   cv2(3); fm(10, 11);
            SLA_PIN("+v"(oacc[0]), "+v"(moff), "+v"(pw[3])); SLA_SB();
            pv(0, 1); ex(10, 11); cv2(4); fm(12, 13);
            SLA_PIN("+v"(oacc[1]), "+v"(moff), "+v"(pw[4])); SLA_SB();
            pv(1, 0); ex(12, 13); cv2(5); fm(14, 15); dots(0);
            SLA_PIN("+v"(oacc[0]), "+v"(pw[5]), "+v"(l_part), "+v"(l_alt)); SLA_SB();
            pv(1, 1); ex(14, 15); cv2(6); dots(1);
            SLA_PIN("+v"(oacc[1]), "+v"(pw[6]), "+v"(l_part), "+v"(l_alt)); SLA_SB();
            cv2(7);
        } else {
            fm(0, 4);                                                            // the e4m3 MFMA takes twice as long: a larger first share
            sm(0);    ex(0, 4);   fm(5, 7);
            SLA_PIN("+v"(s_nxt), "+v"(moff)); SLA_SB();
            pv(0, 0); ex(5, 7);   cv2(0); cv2(1); fm(8, 10);
            SLA_PIN("+v"(oacc[0]), "+v"(moff), "+v"(pw[0]), "+v"(pw[1])); SLA_SB();
            pv(0, 1); ex(8, 10);  cv2(2); cv2(3); fm(11, 13);
            SLA_PIN("+v"(oacc[1]), "+v"(moff), "+v"(pw[2]), "+v"(pw[3])); SLA_SB();
            pv(1, 0); ex(11, 13); cv2(4); fm(14, 15); dots(0);
            SLA_PIN("+v"(oacc[0]), "+v"(pw[4]), "+v"(l_part), "+v"(l_alt)); SLA_SB();
            pv(1, 1); ex(14, 15); cv2(5); cv2(6); dots(1);
            SLA_PIN("+v"(oacc[1]), "+v"(pw[5]), "+v"(pw[6]), "+v"(l_part), "+v"(l_alt)); SLA_SB();
            cv2(7);
        }
        w.p[0] = __builtin_bit_cast(f16x8, make_uint4(pw[0], pw[1], pw[2], pw[3]));
        w.p[1] = __builtin_bit_cast(f16x8, make_uint4(pw[4], pw[5], pw[6], pw[7]));
        w.invr = t.invr;
        over_cur = overflows(s_nxt, tn);
        // the fragments requested at the top of this step have long arrived: say so here, so that the wait the
        // compiler places in front of their first use in the next step does not also cover that step's own reads
        __builtin_amdgcn_s_waitcnt(0xC07F);        // lgkmcnt(0) only
        s_cur = s_nxt; w_prev = w; vf_use = vf_pre; kf_use = kf_pre;
    };
#undef SLA_PIN

    // Raises the running maximum of the rows to the exact maximum over the unit whose S^T is s_cur, in front of a fast
    // step: the accumulators, the row sums and the weights of the previous unit (not yet multiplied into the
    // accumulators) are rescaled; the fast step that follows then sees no exponent above zero.
    auto raise_reference = [&](const TileInfo &t) __attribute__((always_inline)) {
        const float top = pair_max(max16(s_cur)) * t.cj + t.lsv;
        const float m_new = fmaxf(m_run, top);
        const float alpha = m_new == m_run ? 1.0f : fast_exp2(m_run - m_new);
        rescale(alpha);
        const _Float16 ah = (_Float16)alpha;
#pragma unroll
        for (int ss = 0; ss < 2; ++ss)
#pragma unroll
            for (int x = 0; x < 8; ++x) w_prev.p[ss][x] *= ah;
        m_run = m_new;
    };

    // Ring bookkeeping.  During iteration c the LDS reads touch V^T tile c and K tile c + KAHEAD - 2 (the fragments of
    // the following step); both must have landed at its barrier, and that barrier frees the slots of the tiles before
    // them, into which the copies of V^T tile c + 2 and K tile c + KAHEAD go: needed two iterations later.
    constexpr int KAHEAD = 3;
    // Ring slots of iteration c, with P = c mod SLOTS: the V^T tile whose fragments are read sits in slot P, the K tile
    // whose fragments are read (tile c+1) in slot P+1, the K tile requested (c+3) goes where tile c was, the V^T tile
    // requested (c+2) into slot P+2.  The loop is unrolled over P so that the slots are constants: the fragment reads
    // take them as immediate offsets and no slot arithmetic is left in the loop.
    auto iteration = [&](int c, auto phase) __attribute__((always_inline)) {
        constexpr int P = decltype(phase)::value, S = T::SLOTS;
        constexpr uint32_t kreq = ((P + KAHEAD) % S) * T::KBYTES, vreq = ((P + 2) % S) * T::VBYTES;
        constexpr int kslot = ((P + KAHEAD - 2) % S) * T::KBYTES, vslot = T::VRING + P * T::VBYTES;
        SLA_T(c, 0);
        // copies that may stay in flight here: those requested one iteration ago
        if (c == 0) wait_copies_and_barrier<0>();      // (nothing is in flight; joins the waves after the prologue's LDS reads)
        else if (c + KAHEAD - 1 < k) wait_copies_and_barrier<T::LOADS>();
        else if (c + 1 < k) wait_copies_and_barrier<T::VINS>();
        else wait_copies_and_barrier<0>();
        SLA_T(c, 1);
        if (c + KAHEAD - wbase >= 64) load_window(wbase + 32);     // (never for lists of at most 64 blocks)
        if (c + KAHEAD < k) request_K(c + KAHEAD, kreq);
        if (c + 2 < k) request_V(c + 2, vreq);
        if (c + 1 == k) request_epilogue();
        const bool more = c + 1 < k;
        if (more) t_nxt = tile_info(c + 1);
        const bool ragged_n = more && t_nxt.valid != kBK;
        SLA_T(c, 2);
        // first half of tile c: accumulates the second half of tile c-1, forms S^T of the second half of tile c;
        // reads the fragments of the next step: V^T tile c first half, K tile c+1 first half
        if (over_cur || c == 0 || t_cur.tiny || t_cur.valid != kBK) careful_step(c > 0, true, t_cur, t_cur, 1, vslot, 0, kslot, 0);
        else fast_step(t_cur, t_cur, vslot, 0, kslot, 0);
        SLA_T(c, 3);
        // second half of tile c: accumulates its first half, forms S^T of the first half of tile c+1;
        // reads V^T tile c second half and K tile c+1 second half for the first step of the next iteration
        if (over_cur || !more || t_cur.tiny || ragged_n) careful_step(true, more, t_cur, t_nxt, 0, vslot, 1, kslot, 1);
        else fast_step(t_cur, t_nxt, vslot, 1, kslot, 1);
        SLA_T(c, 4);
        t_cur = t_nxt;
    };
    // The lean form of an iteration, for the middle of a list: tile c is not the first, tiles c .. c + KAHEAD exist, are
    // full and none has a far-off V scale, and the window holds them (lean_ok checks this for three iterations at a
    // time).  Nothing is conditional but the raise of the running maximum; both steps are fast steps.
    auto lean_iteration = [&](int c, auto phase) __attribute__((always_inline)) {
        constexpr int P = decltype(phase)::value, S = T::SLOTS;
        constexpr uint32_t kreq = ((P + KAHEAD) % S) * T::KBYTES, vreq = ((P + 2) % S) * T::VBYTES;
        constexpr int kslot = ((P + KAHEAD - 2) % S) * T::KBYTES, vslot = T::VRING + P * T::VBYTES;
        SLA_T(c, 0);
        wait_copies_and_barrier<T::LOADS>();
        SLA_T(c, 1);
        request_K(c + KAHEAD, kreq, true);
        request_V(c + 2, vreq);
        t_nxt.valid = kBK; t_nxt.tiny = false;
        t_nxt.cj = FP8 ? __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(d_cj), c + 1 - wbase)) : c_exp;
        t_nxt.lsv = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(d_lv), c + 1 - wbase));
        t_nxt.invr = fast_exp2(-t_nxt.lsv);
        SLA_T(c, 2);
        if (over_cur) raise_reference(t_cur);
        fast_step(t_cur, t_cur, vslot, 0, kslot, 0);
        SLA_T(c, 3);
        if (over_cur) raise_reference(t_cur);
        fast_step(t_cur, t_nxt, vslot, 1, kslot, 1);
        SLA_T(c, 4);
        t_cur = t_nxt;
    };
    // three lean iterations from tile c on are possible: bits c .. c + 2 + KAHEAD of d_bad are clear and inside the window
    auto lean_ok = [&](int c) {
        return c + 2 + KAHEAD - wbase < 64 && ((uint32_t)(d_bad >> (c - wbase)) & ((1u << (KAHEAD + 3)) - 1)) == 0;
    };
    for (int c = 0; c < k;) {
        iteration(c, std::integral_constant<int, 0>{});
        if (c + 1 < k) iteration(c + 1, std::integral_constant<int, 1>{});
        if (T::SLOTS == 3 && c + 2 < k) iteration(c + 2, std::integral_constant<int, 2 % T::SLOTS>{});
        c += T::SLOTS;
        if constexpr (T::SLOTS == 3) {
            while (lean_ok(c)) {
                lean_iteration(c, std::integral_constant<int, 0>{});
                lean_iteration(c + 1, std::integral_constant<int, 1>{});
                lean_iteration(c + 2, std::integral_constant<int, 2>{});
                c += 3;
            }
        }
    }
#undef SLA_SB

    wait_copies_and_barrier<0>();                      // epilogue operands landed; every wave is past its last tile
    SLA_TP(61, 0);
    if (k > 0) accumulate(vf_use, w_prev);             // the last unit's weights
    l_part += l_alt;
    float l_run = l_part + xchg32(l_part) + l_full;

    uint8_t *stA = lds + kHqOff, *stB = lds + kWtOff;
    const uint8_t *zrow = lds + T::ZOFF;
    // ---- normalise the sparse output: the weights carried the V scale relative to the first tile's
    const float inv_l = l_run > 0.f ? fast_exp2(lv_ref) / l_run : 0.f;
#pragma unroll
    for (int e = 0; e < 2; ++e)
#pragma unroll
        for (int x = 0; x < 16; ++x) oacc[e][x] *= inv_l;

    SLA_TP(61, 1);
    if (Hq != nullptr) {
        // The sixteen operand fragments of the two products below are read from LDS here, in one go, so that their latency
        // passes behind the arithmetic of phi(Q) (read where they are used, each would be awaited on its own).
        bf16x8 hfr[4][2], wfr[4][2];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int hchunk = FP8 ? 4 * g + s : 2 * s + g;      // 16-byte chunk holding channels dcol(s)..dcol(s)+7
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                hfr[s][e] = *(const bf16x8 *)(stA + (32 * e + l32) * 128 + ((hchunk ^ swz8(l32)) << 4));
                wfr[s][e] = *(const bf16x8 *)(stB + (32 * e + l32) * 128 + (((2 * s + g) ^ swz8(l32)) << 4));
            }
        }
        __builtin_amdgcn_sched_barrier(0);
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
            const float nmx = -mx * kLog2e;
            float sum = 0.f;
#pragma unroll
            for (int d = 0; d < 32; ++d) { x[d] = fast_exp2(fmaf(x[d], kLog2e, nmx)); sum += x[d]; }
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
            den = dot2_bf16(o.w, z.w, dot2_bf16(o.z, z.z, dot2_bf16(o.y, z.y, dot2_bf16(o.x, z.x, den))));
        }
        den += xchg32(den);
        const float inv_den = den > 0.f ? 1.0f / den : 0.f;     // no marginal block: H = Z = 0 and O_lin = 0

        SLA_TP(61, 2);
        // ---- O_lin^T = Hq^T phi(Q)^T   (Hq^T tile staged with the tile swizzle)
        f32x16 lacc[2];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
#pragma unroll
            for (int e = 0; e < 2; ++e) lacc[e] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(hfr[s][e], fq[s], s == 0 ? zero16 : lacc[e], 0, 0, 0);
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
            for (int e = 0; e < 2; ++e) oacc[e] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wfr[s][e], pf, oacc[e], 0, 0, 0);
        }
    }

    // ---- store.  Register 4a+b of oacc[e] is channel 32e + 8a + 4g + b of row q: the wave's 32x64 tile
    // is transposed through a private 4 KB LDS slice (8-byte pieces, XOR-swizzled by row) so that it
    // leaves as full 128-byte rows, 16 bytes per lane.
    SLA_TP(61, 3);
    wait_copies_and_barrier<0>();                      // all waves are done reading the epilogue operands
    SLA_TP(61, 4);
    if (O32 != nullptr) {
        // diagnostic output: the fp32 values the bf16 store below would round, straight from the accumulators
        if (qok) {
#pragma unroll
            for (int e = 0; e < 2; ++e)
#pragma unroll
                for (int aa = 0; aa < 4; ++aa)
                    *(float4 *)(O32 + head + (size_t)q * rm.ts + 32 * e + 8 * aa + 4 * g) =
                        make_float4(oacc[e][4 * aa + 0], oacc[e][4 * aa + 1], oacc[e][4 * aa + 2], oacc[e][4 * aa + 3]);
        }
    } else {
        uint8_t *ot = lds + T::VRING + wq * 4096;
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
        for (int kk = 0; kk < 4; ++kk) {
            const int r = 8 * kk + (lane >> 3), ch = lane & 7;      // row of the tile, 16-byte chunk of the row
            const int fr = ((r >> 1) & 7) << 1;
            const uint4 v = *(const uint4 *)(ot + r * 128 + (((2 * ch) ^ fr) << 3));
            if (q0w + r < N) *(uint4 *)(O + head + (size_t)(q0w + r) * rm.ts + ch * 8) = v;
        }
    }
    SLA_TP(61, 5);
#ifdef SLA_PROBE_TIME
    if (tid == 0 && work < 32768) sla_wg_times[2 * work + 1] = __builtin_amdgcn_s_memrealtime();
    if (probe_on) {
        const unsigned long long tp_c1 = __builtin_readcyclecounter(), tp_r1 = __builtin_amdgcn_s_memrealtime();
        if (lane == 0) { tprobe[63 * 8 + 6] = tp_c1 - tp_c0; tprobe[63 * 8 + 7] = tp_r1 - tp_r0; }   // wave life: shader clock, 100 MHz clock
        for (int x = lane; x < 64 * 8; x += 64) sla_probe_times[x] = tprobe[x];
    }
#endif
}

// The same computation for SHORT critical lists (frame attention: one or two blocks per row; up to kShortList), where
// a workgroup's life is memory latency (list -> tiles, operands of the linear branch) and little arithmetic: no software
// pipeline and no rings, so that the kernel fits 128 registers and 17 KB of LDS and eight workgroups of two waves (four
// of four) share a CU and hide each other's round trips.  Order of work: the linear branch first (its operands, the Hq^T
// tile, W^T and Z, are asked for together with Q and the list; its result waits in sixteen registers as bf16), then one
// tile at a time through a single K slot and a single V^T slot: S^T, exact running maximum, fp16 weights carrying the
// block's V exponent, O^T += V^T P^T (the arithmetic of the careful step above); at the end O = O_sparse / l + O_lin W.
constexpr int kShortList = 2;
// (Two tile buffers, the copies of tile c+1 in flight while tile c is worked on, were measured on lists of nine: a
// workgroup then lives 20 us instead of 31, but only four fit a CU instead of eight, and the launch takes the same time.)
template <int NW, bool FP8>
__global__ __launch_bounds__(64 * NW, 4) void attend_short_kernel(
    const void *__restrict__ Qp, const void *__restrict__ Kp, const uint16_t *__restrict__ Vp, const float *__restrict__ lvs,
    const float *__restrict__ sQ, const float *__restrict__ sK, RowMap rm,
    const int32_t *__restrict__ crit_idx, int k_c, const uint16_t *__restrict__ Hq, const uint16_t *__restrict__ WT,
    int proj_per_head, int phi, int H, int N, int Nqb, int Nkb, long total, float c_exp, uint16_t *__restrict__ O, float *__restrict__ O32)
{
    using T = Tile<NW, FP8, 2>;                       // (for the copy-instruction counts and tile sizes only)
    constexpr int BQ = 32 * NW;
    constexpr int ES = FP8 ? 1 : 2;
    constexpr int KROWB = FP8 ? 64 : 128;
    constexpr int kA = 0, kB = 8192, kZ = 16384;      // LDS: slot A (K tile / Hq^T), slot B (V^T tile / W^T), the Z row
    __shared__ __attribute__((aligned(1024))) uint8_t lds[kZ + 256];
    asm volatile("" ::"s"(Qp), "s"(Kp), "s"(Vp), "s"(lvs), "s"(sQ), "s"(sK), "s"(rm.bs), "s"(rm.hs), "s"(rm.ts), "s"(rm.H), "s"(crit_idx),
                 "s"(k_c), "s"(Hq), "s"(WT), "s"(proj_per_head), "s"(phi), "s"(H), "s"(N), "s"(Nqb), "s"(Nkb), "s"(total), "s"(c_exp), "s"(O), "s"(O32));
    const long work = xcd_remap(blockIdx.x, total);
    if (work >= total) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, g = lane >> 5;
#ifdef SLA_PROBE_TIME
    if (tid == 0 && work < 32768) sla_wg_times[2 * work] = __builtin_amdgcn_s_memrealtime();
#endif
    const long bh = (long)((unsigned)work / (unsigned)Nqb);
    const int i = (int)(work - bh * Nqb);
    const int q = i * BQ + 32 * wave + l32;
    const bool qok = q < N;
    const size_t head = rm.head(bh);
    const int krowb = rm.ts * ES;
    const uint8_t *Kh = (const uint8_t *)Kp + head * ES;
    const uint8_t *Vh = (const uint8_t *)(Vp + (size_t)bh * Nkb * kBK * kD);

    // the list (at most kShortList entries, one per lane), then Q
    const int j0 = lane < k_c ? crit_idx[work * (long)k_c + lane] : -1;
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
    const float qscale = FP8 ? sQ[work] : 1.0f;

    CopyOffsets<NW, FP8> co;
    co.init(wave, lane, krowb);
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const uint32_t lds_base = (uint32_t)(uintptr_t)(lds_void_p)lds;
    const uint32_t ktile_bytes = (uint32_t)kBK * (uint32_t)krowb;
    const int tail_rows = N & (kBK - 1), ragged_j = tail_rows ? Nkb - 1 : -1;

    // ---- the linear branch: operands on their way while the list and Q arrive
    if (Hq != nullptr) {
        const uint8_t *Hi8 = (const uint8_t *)(Hq + (size_t)work * kStateElems);
        const uint8_t *Wh8 = (const uint8_t *)(WT + (proj_per_head ? (size_t)((unsigned)bh % (unsigned)H) * kD * kD : 0));
#pragma unroll
        for (int x = 0; x < T::VINS; ++x) copy_1k_to_lds(Hi8, co.v[x], lds_base + kA + (wave_u * T::VINS + x) * 1024);
#pragma unroll
        for (int x = 0; x < T::VINS; ++x) copy_1k_to_lds(Wh8, co.v[x], lds_base + kB + (wave_u * T::VINS + x) * 1024);
        if (tid < 8) copy_1k_to_lds(Hi8 + 64 * kD * 2, tid * 16, lds_base + kZ);
    }
    // number of leading valid entries, their V exponents and exp2 constants (a gather that depends on the list)
    const bool jok = j0 >= 0 && j0 < Nkb;
    const unsigned long long okm = __ballot(jok);
    int k = okm == ~0ull ? 64 : __builtin_ctzll(~okm);
    k = __builtin_amdgcn_readfirstlane(min(k, k_c));
    const int d_j = jok ? j0 : 0;
    float d_lv = lvs[bh * Nkb + d_j];
    float d_cj = FP8 ? fmaxf(c_exp * qscale * sK[bh * Nkb + d_j], 1e-30f) : c_exp;
    asm volatile("" : "+v"(d_lv), "+v"(d_cj));
    const float lv_ref = __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(d_lv)));
    d_lv -= lv_ref;
    __builtin_amdgcn_s_waitcnt(0 | (7 << 4) | (15 << 8));      // vmcnt(0): Q, the list and the operands have landed
    wait_copies_and_barrier<0>();

    f32x16 zero16;
#pragma unroll
    for (int x = 0; x < 16; ++x) zero16[x] = 0.f;
    uint32_t lin[16];                                  // O_lin W of this lane's row, bf16 pairs (channel 32e + 8a + 4g + b: lin[8e + 2a + b/2])
#pragma unroll
    for (int x = 0; x < 16; ++x) lin[x] = 0u;
    if (Hq != nullptr) {
        const uint8_t *stA = lds + kA, *stB = lds + kB, *zrow = lds + kZ;
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
            const float nmx = -mx * kLog2e;
            float sum = 0.f;
#pragma unroll
            for (int d = 0; d < 32; ++d) { x[d] = fast_exp2(fmaf(x[d], kLog2e, nmx)); sum += x[d]; }
            sum += xchg32(sum);
            inv = 1.0f / sum;
        } else {
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
            den = dot2_bf16(o.w, z.w, dot2_bf16(o.z, z.z, dot2_bf16(o.y, z.y, dot2_bf16(o.x, z.x, den))));
        }
        den += xchg32(den);
        const float inv_den = den > 0.f ? 1.0f / den : 0.f;
        f32x16 lacc[2];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int hchunk = FP8 ? 4 * g + s : 2 * s + g;
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
        f32x16 pl[2];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const bf16x8 pf = pack8(lacc[s >> 1], 8 * (s & 1));
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const bf16x8 wf = *(const bf16x8 *)(stB + (32 * e + l32) * 128 + (((2 * s + g) ^ swz8(l32)) << 4));
                pl[e] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, pf, s == 0 ? zero16 : pl[e], 0, 0, 0);
            }
        }
#pragma unroll
        for (int e = 0; e < 2; ++e)
#pragma unroll
            for (int y = 0; y < 8; ++y) lin[8 * e + y] = pack_bf16(pl[e][2 * y], pl[e][2 * y + 1]);
    }
    wait_copies_and_barrier<0>();                      // every wave is done with the operands: the slots take tiles now
    auto request_tile = [&](int c) __attribute__((always_inline)) {
        const uint32_t j = (uint32_t)__builtin_amdgcn_readlane(d_j, c);
        const uint8_t *kt = Kh + (uint64_t)j * ktile_bytes;
        const uint32_t kdst = lds_base + kA + wave_u * T::KINS * 1024, vdst = lds_base + kB + wave_u * T::VINS * 1024;
        if ((int)j != ragged_j) copy_nk_to_lds<T::KINS>(kt, co.k, kdst);
        else {
#pragma unroll
            for (int x = 0; x < T::KINS; ++x)
                copy_1k_to_lds(kt, co.k[x] - (co.krow[x] - min(co.krow[x], tail_rows - 1)) * krowb, kdst + x * 1024);
        }
        copy_nk_to_lds<T::VINS>(Vh + (uint64_t)j * (uint32_t)(kBK * kD * 2), co.v, vdst);
    };

    // ---- the tiles, one at a time
    int koff[4], voff[4];
#pragma unroll
    for (int s = 0; s < 4; ++s)
        koff[s] = FP8 ? l32 * 64 + ((((2 * g + (s & 1)) ^ swz4(l32))) << 4) : l32 * 128 + (((2 * s + g) ^ swz8(l32)) << 4);
#pragma unroll
    for (int st = 0; st < 4; ++st) voff[st] = l32 * 128 + (((2 * st + g) ^ swz8(l32)) << 4);
    f32x16 oacc[2] = {zero16, zero16};
    float m_run = -INFINITY, l_sum = 0.f;
    for (int c = 0; c < k; ++c) {
        const uint8_t *ldsb = lds;
        const uint32_t j = (uint32_t)__builtin_amdgcn_readlane(d_j, c);
        request_tile(c);
        const int valid = (int)j == ragged_j ? tail_rows : kBK;
        const float cj = FP8 ? __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(d_cj), c)) : c_exp;
        const float lsv = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(d_lv), c));
        const float rsv = fast_exp2(lsv);
        wait_copies_and_barrier<0>();                  // tile c has landed
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            f32x16 sacc;
#pragma unroll
            for (int x = 0; x < 16; ++x) sacc[x] = (32 * half + 8 * (x >> 2) + 4 * g + (x & 3)) < valid ? 0.f : -INFINITY;
            if (FP8) {
                const i32x4 w0 = *(const i32x4 *)(ldsb + kA + half * 32 * KROWB + koff[0]), w1 = *(const i32x4 *)(ldsb + kA + half * 32 * KROWB + koff[1]);
                i32x8 k8;
                k8[0] = w0[0]; k8[1] = w0[1]; k8[2] = w0[2]; k8[3] = w0[3]; k8[4] = w1[0]; k8[5] = w1[1]; k8[6] = w1[2]; k8[7] = w1[3];
                sacc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(k8, q8, sacc, 0, 0, 0, 0, 0, 0);
            } else {
#pragma unroll
                for (int st = 0; st < 4; ++st) {
                    const bf16x8 kf = *(const bf16x8 *)(ldsb + kA + half * 32 * KROWB + koff[st]);
                    sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[st], sacc, 0, 0, 0);
                }
            }
            const float top = pair_max(max16(sacc)) * cj + lsv;        // -inf if the row sees no real key in this unit
            if (__ballot(top > m_run)) {
                const float m_new = fmaxf(m_run, top);
                const float alpha = m_new == m_run ? 1.0f : fast_exp2(m_run - m_new);
                l_sum *= alpha;
#pragma unroll
                for (int e = 0; e < 2; ++e)
#pragma unroll
                    for (int x = 0; x < 16; ++x) oacc[e][x] *= alpha;
                m_run = m_new;
            }
            const float mfin = m_run == -INFINITY ? 0.f : m_run;
            float sum = 0.f;
#pragma unroll
            for (int x = 0; x < 16; ++x) {
                const float pu = fast_exp2(fmaf(sacc[x], cj, -mfin));
                sum += pu;
                sacc[x] = pu * rsv;
            }
            l_sum += sum;
            const f16x8 p0 = pack8_f16(sacc, 0), p1 = pack8_f16(sacc, 8);
#pragma unroll
            for (int ss = 0; ss < 2; ++ss)
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    const f16x8 vf = *(const f16x8 *)(ldsb + kB + e * 32 * 128 + voff[2 * half + ss]);
                    oacc[e] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf, ss == 0 ? p0 : p1, oacc[e], 0, 0, 0);
                }
        }
        wait_copies_and_barrier<0>();                  // all waves are done with the tile before the next one is asked for
    }

    // ---- O = O_sparse / l + O_lin W
    const float l_run = l_sum + xchg32(l_sum);
    const float inv_l = l_run > 0.f ? fast_exp2(lv_ref) / l_run : 0.f;
#pragma unroll
    for (int e = 0; e < 2; ++e)
#pragma unroll
        for (int y = 0; y < 8; ++y) {
            oacc[e][2 * y] = fmaf(oacc[e][2 * y], inv_l, bf16_lo(lin[8 * e + y]));
            oacc[e][2 * y + 1] = fmaf(oacc[e][2 * y + 1], inv_l, bf16_hi(lin[8 * e + y]));
        }
    if (O32 != nullptr) {
        if (qok) {
#pragma unroll
            for (int e = 0; e < 2; ++e)
#pragma unroll
                for (int aa = 0; aa < 4; ++aa)
                    *(float4 *)(O32 + head + (size_t)q * rm.ts + 32 * e + 8 * aa + 4 * g) =
                        make_float4(oacc[e][4 * aa + 0], oacc[e][4 * aa + 1], oacc[e][4 * aa + 2], oacc[e][4 * aa + 3]);
        }
    } else {
        uint8_t *ot = lds + wave * 4096;               // (NW x 4 KB: inside the two slots)
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
        const int q0w = i * BQ + 32 * wave;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const int r = 8 * kk + (lane >> 3), ch = lane & 7;
            const int fr = ((r >> 1) & 7) << 1;
            const uint4 v = *(const uint4 *)(ot + r * 128 + (((2 * ch) ^ fr) << 3));
            if (q0w + r < N) *(uint4 *)(O + head + (size_t)(q0w + r) * rm.ts + ch * 8) = v;
        }
    }
#ifdef SLA_PROBE_TIME
    if (tid == 0 && work < 32768) sla_wg_times[2 * work + 1] = __builtin_amdgcn_s_memrealtime();
#endif
}

// W [nW][e_in][e_out] -> WT [nW][e_out][slot] as its own launch (the whole forward folds this into the states pass)
__global__ __launch_bounds__(256) void transpose_w_kernel(const uint16_t *__restrict__ W, uint16_t *__restrict__ WT)
{
    transpose_w_tile(W + (size_t)blockIdx.x * kD * kD, WT + (size_t)blockIdx.x * kD * kD, 256);
}

#ifdef SLA_PROBE_TIME
extern "C" int sla_probe_read_wg(unsigned long long *dst, int n) { return (int)hipMemcpyFromSymbol(dst, HIP_SYMBOL(sla_wg_times), sizeof(unsigned long long) * 2 * n); }
extern "C" int sla_probe_read(unsigned long long *dst) { return (int)hipMemcpyFromSymbol(dst, HIP_SYMBOL(sla_probe_times), sizeof(unsigned long long) * 64 * 8); }
#endif

hipError_t launch_transpose_w(const void *W, int nW, void *WT, hipStream_t st)
{
    transpose_w_kernel<<<nW, 256, 0, st>>>((const uint16_t *)W, (uint16_t *)WT);
    return hipGetLastError();
}

template <int NW, bool FP8, int SL = 3>
static hipError_t launch_attend_t(const void *Q, const void *K, const void *Vp, const float *lvs, const float *sQ, const float *sK, RowMap rm,
                                  const int32_t *crit_idx, int k_c, const void *Hq, const void *WT, int proj_per_head, int phi,
                                  int H, int N, int Nqb, int Nkb, long total, float c_exp, void *O, float *O32, hipStream_t st)
{
    attend_kernel<NW, FP8, SL><<<(unsigned)xcd_grid(total), 64 * NW, 0, st>>>(Q, K, (const uint16_t *)Vp, lvs, sQ, sK, rm, crit_idx, k_c, (const uint16_t *)Hq,
                                                                     (const uint16_t *)WT, proj_per_head, phi, H, N, Nqb, Nkb,
                                                                     total, c_exp, (uint16_t *)O, O32);
    return hipGetLastError();
}

hipError_t launch_attend(const void *Q, const void *K, const void *Vp, const float *lvs,
                         const float *sQ, const float *sK, bool fp8, RowMap rm,
                         const int32_t *crit_idx, int k_c, const void *Hq, const void *WT,
                         int proj_per_head, int phi, int B, int H, int N, int bq, float sm_scale,
                         void *O, float *O32, hipStream_t st)
{
    const int Nqb = (N + bq - 1) / bq, Nkb = (N + kBK - 1) / kBK;
    const long total = (long)B * H * Nqb;
    const float c_exp = sm_scale * kLog2e;
#define SLA_ATT(NW, F8, SL) return launch_attend_t<NW, F8, SL>(Q, K, Vp, lvs, sQ, sK, rm, crit_idx, k_c, Hq, WT, proj_per_head, phi, H, N, Nqb, Nkb, total, c_exp, O, O32, st)
    if (bq == 128) { if (fp8) SLA_ATT(4, true, 3); else SLA_ATT(4, false, 3); }
    // lists of at most two blocks (frame attention): the kernel without a pipeline, eight workgroups per CU
    if (k_c <= kShortList) {
        if (fp8) attend_short_kernel<2, true><<<(unsigned)xcd_grid(total), 128, 0, st>>>(Q, K, (const uint16_t *)Vp, lvs, sQ, sK, rm, crit_idx, k_c, (const uint16_t *)Hq,
                                                                                       (const uint16_t *)WT, proj_per_head, phi, H, N, Nqb, Nkb, total, c_exp, (uint16_t *)O, O32);
        else attend_short_kernel<2, false><<<(unsigned)xcd_grid(total), 128, 0, st>>>(Q, K, (const uint16_t *)Vp, lvs, sQ, sK, rm, crit_idx, k_c, (const uint16_t *)Hq,
                                                                                      (const uint16_t *)WT, proj_per_head, phi, H, N, Nqb, Nkb, total, c_exp, (uint16_t *)O, O32);
        return hipGetLastError();
    }
    if (fp8) SLA_ATT(2, true, 3);
    SLA_ATT(2, false, 3);
#undef SLA_ATT
}

}  // namespace sla
