// Block mean-pool, pooled logits and the three-way block classifier
// (Alg. 1 steps 2-3 of the paper, evaluated on block means).
//
// Reproducibility contract (labels must equal a CPU evaluation bit for bit):
//   * a block mean is the fp64 sum over the block's tokens in ascending token order times
//     the fp64 value 1/count -- one thread owns a (block, channel) sum and adds serially;
//   * a pooled logit is the 64-step fp64 fma chain over the channel index from 0.0;
//   * the classifier works on the total order (logit descending, index ascending).
#include "sla_common.hpp"
#include "sla_kernels.hpp"

namespace sla {

// ------------------------------------------------------------------------------------- pool
// 64 / CPT threads per token block, each owning CPT consecutive channels (CPT x 2 bytes of bf16 / CPT bytes of e4m3
// per token), serial over the tokens of the block.  Bound: HBM (one streaming read of X).  A thread keeps 32 rows in
// flight; CPT is chosen at the launch so that there are enough waves to hide the rest of the latency (eight channels
// per thread are one wave per 512 token rows: fewer than one wave per SIMD on the benchmark shapes).
template <int BYTES> struct PoolWord;
template <> struct PoolWord<16> { typedef uint4 type; };
template <> struct PoolWord<8> { typedef uint2 type; };
template <> struct PoolWord<4> { typedef uint32_t type; };
template <> struct PoolWord<2> { typedef uint16_t type; };

__device__ __forceinline__ uint32_t pool_dword(const uint4 &w, int i) { return i == 0 ? w.x : i == 1 ? w.y : i == 2 ? w.z : w.w; }
__device__ __forceinline__ uint32_t pool_dword(const uint2 &w, int i) { return i == 0 ? w.x : w.y; }
__device__ __forceinline__ uint32_t pool_dword(uint32_t w, int) { return w; }
__device__ __forceinline__ uint32_t pool_dword(uint16_t w, int) { return w; }

template <bool FP8, int CPT>
__global__ __launch_bounds__(256) void pool_kernel(const void *__restrict__ X, const float *__restrict__ scales,
                                                   RowMap rm, int N, int blk, int nblk, long units, double *__restrict__ mean)
{
    constexpr int TPB = kD / CPT, ES = FP8 ? 1 : 2;       // threads per token block, bytes per element
    typedef typename PoolWord<CPT * ES>::type Word;
    asm volatile("" ::"s"(X), "s"(scales), "s"(rm.bs), "s"(rm.hs), "s"(rm.ts), "s"(rm.H), "s"(N), "s"(blk), "s"(nblk), "s"(units), "s"(mean));      // all kernel arguments in one batch of scalar loads, here
    const long u = (long)blockIdx.x * 256 + threadIdx.x;
    if (u >= units) return;
    const int c = (int)(u % TPB);
    const long blkid = u / TPB;
    const long bh = blkid / nblk;
    const int j = (int)(blkid - bh * nblk);
    const int t0 = j * blk;
    const int cnt = min(N - t0, blk);
    double acc[CPT];
#pragma unroll
    for (int k = 0; k < CPT; ++k) acc[k] = 0.0;
    const double s = FP8 ? (double)scales[blkid] : 1.0;
    auto add_row = [&](Word w) {
        if (FP8) {
#pragma unroll
            for (int k = 0; k < CPT; k += 2) {
                const f32x2 a = (k & 2) ? __builtin_amdgcn_cvt_pk_f32_fp8(pool_dword(w, k >> 2), true)
                                        : __builtin_amdgcn_cvt_pk_f32_fp8(pool_dword(w, k >> 2), false);
                acc[k] += (double)a[0] * s;
                acc[k + 1] += (double)a[1] * s;
            }
        } else {
#pragma unroll
            for (int k = 0; k < CPT; k += 2) {
                acc[k] += (double)bf16_lo(pool_dword(w, k >> 1));
                acc[k + 1] += (double)bf16_hi(pool_dword(w, k >> 1));
            }
        }
    };
    const uint8_t *x = (const uint8_t *)X + (rm.head(bh) + (size_t)t0 * rm.ts + c * CPT) * ES;
    const size_t rowb = (size_t)rm.ts * ES;
    // sixteen rows are requested before the first is consumed, and the next sixteen before that
    Word wa[16], wb[16];
    auto fetch = [&](Word (&w)[16], int t) {
#pragma unroll
        for (int k = 0; k < 16; ++k) w[k] = *(const Word *)(x + (size_t)(t + k) * rowb);
    };
    auto consume = [&](const Word (&w)[16]) {
#pragma unroll
        for (int k = 0; k < 16; ++k) add_row(w[k]);
    };
    int t = 0;
    if (cnt >= 16) fetch(wa, 0);
    for (; t + 32 <= cnt; t += 32) {
        fetch(wb, t + 16);
        consume(wa);
        if (t + 48 <= cnt) fetch(wa, t + 32);
        consume(wb);
    }
    if (t + 16 <= cnt) { consume(wa); t += 16; }
    for (; t < cnt; ++t) add_row(*(const Word *)(x + (size_t)t * rowb));
    const double inv = 1.0 / (double)cnt;
    double *o = mean + blkid * kD + c * CPT;
#pragma unroll
    for (int k = 0; k < CPT; ++k) o[k] = acc[k] * inv;
}

template <bool FP8, int CPT>
static hipError_t launch_pool_t(const void *X, const float *scales, RowMap rm, int BH, int N, int blk, double *mean, hipStream_t st)
{
    const int nblk = (N + blk - 1) / blk;
    const long units = (long)BH * nblk * (kD / CPT);
    pool_kernel<FP8, CPT><<<(unsigned)((units + 255) / 256), 256, 0, st>>>(X, scales, rm, N, blk, nblk, units, mean);
    return hipGetLastError();
}

hipError_t launch_pool(const void *X, const float *scales, bool fp8, RowMap rm, int BH, int N, int blk,
                       double *mean, hipStream_t st)
{
    // the widest loads that still give about four waves per SIMD (4096 waves of 64 threads)
    const long blocks = (long)BH * ((N + blk - 1) / blk);
    if (fp8) {
        if (blocks * 8 >= 4096L * 64) return launch_pool_t<true, 8>(X, scales, rm, BH, N, blk, mean, st);
        return launch_pool_t<true, 4>(X, scales, rm, BH, N, blk, mean, st);
    }
    if (blocks * 8 >= 4096L * 64) return launch_pool_t<false, 8>(X, scales, rm, BH, N, blk, mean, st);
    if (blocks * 16 >= 4096L * 64) return launch_pool_t<false, 4>(X, scales, rm, BH, N, blk, mean, st);
    return launch_pool_t<false, 2>(X, scales, rm, BH, N, blk, mean, st);
}

// ----------------------------------------------------------------------------------- scores
// fp64 register-tiled product: workgroup tile 64(i) x 64(j), thread tile 4 x 4, the channel
// loop runs in ascending order so every (i,j) accumulator is the canonical fma chain.
// Bound: fp64 vector FMA (2*Nqb*Nkb*64 flops per head).
__device__ __forceinline__ uint64_t desc_key(double s);

// KEYS: instead of the logits, store the upper halves of their order-preserving keys (uint32 [rows, pitch], pitch in
// keys): all the long-row classifier needs unless a threshold cuts through a group of equal upper halves.
template <bool KEYS>
__global__ __launch_bounds__(256, 5) void scores_kernel(const double *__restrict__ qbar, const double *__restrict__ kbar,
                                                        int Nqb, int Nkb, int pitch, double *__restrict__ S)
{
    // Channels in four quarters of sixteen through one LDS buffer of 17 KB, and at most 102 registers: five workgroups
    // per CU, so that the 1056 tiles of a 16-head launch of 344 x 687 blocks are resident at once.  (Halves of 32
    // channels, 34 KB and four workgroups per CU, measured the same on that launch.)
    constexpr int QC = 16;
    __shared__ double qs[QC][66];
    __shared__ double ks[QC][66];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int j0 = blockIdx.x * 64, i0 = blockIdx.y * 64;
    const long bh = blockIdx.z;
    const double *qh = qbar + bh * (long)Nqb * kD;
    const double *kh = kbar + bh * (long)Nkb * kD;
    double acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = 0.0;

    // element r of a thread in a quarter: channel (tid & 15) of row (tid >> 4) + 16 r (row indices clamped, so the
    // loads are unconditional); the next quarter is requested before the present one is consumed
    const int sd = tid & 15, srow = tid >> 4;
    const double *qsrc[4], *ksrc[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        qsrc[r] = qh + (long)min(i0 + srow + 16 * r, Nqb - 1) * kD + sd;
        ksrc[r] = kh + (long)min(j0 + srow + 16 * r, Nkb - 1) * kD + sd;
    }
    double qr[4], kr[4];
    auto fetch = [&](int c) {
#pragma unroll
        for (int r = 0; r < 4; ++r) { qr[r] = qsrc[r][c * QC]; kr[r] = ksrc[r][c * QC]; }
    };
    fetch(0);
#pragma unroll
    for (int c = 0; c < kD / QC; ++c) {
        if (c) lds_barrier();              // the quarter before is consumed
#pragma unroll
        for (int r = 0; r < 4; ++r) {      // rows past the end repeat the last one; their results are not stored
            qs[sd][srow + 16 * r] = qr[r];
            ks[sd][srow + 16 * r] = kr[r];
        }
        if (c + 1 < kD / QC) fetch(c + 1);
        lds_barrier();
#pragma unroll 4
        for (int d = 0; d < QC; ++d) {
            double qv[4], kv[4];
#pragma unroll
            for (int a = 0; a < 4; ++a) { qv[a] = qs[d][ty * 4 + a]; kv[a] = ks[d][tx * 4 + a]; }
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b) acc[a][b] = fma(qv[a], kv[b], acc[a][b]);
        }
    }
    // a thread's four logits of a row are 32 contiguous bytes; the row pitch is a multiple of 8 entries, so the
    // group is inside the row's allocation as a whole (entries in [Nkb, pitch) are padding nobody reads)
    const int gj = j0 + tx * 4;
    if constexpr (KEYS) {
        uint32_t *Kh = (uint32_t *)S + bh * (long)Nqb * pitch;
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const int gi = i0 + ty * 4 + a;
            if (gi < Nqb && gj < pitch)
                *(uint4 *)(Kh + (long)gi * pitch + gj) = make_uint4((uint32_t)(desc_key(acc[a][0]) >> 32), (uint32_t)(desc_key(acc[a][1]) >> 32),
                                                                     (uint32_t)(desc_key(acc[a][2]) >> 32), (uint32_t)(desc_key(acc[a][3]) >> 32));
        }
    } else {
        double *Sh = S + bh * (long)Nqb * pitch;
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const int gi = i0 + ty * 4 + a;
            if (gi < Nqb && gj < pitch) {
                double2 *dst = (double2 *)(Sh + (long)gi * pitch + gj);
                dst[0] = double2{acc[a][0], acc[a][1]};
                dst[1] = double2{acc[a][2], acc[a][3]};
            }
        }
    }
}

// The same product with an 8 x 8 register tile per thread (workgroup tile 128 x 128, 256 threads), for heads with
// enough tiles to fill the chip.  With 4 x 4 tiles a channel step reads 64 bytes of LDS per lane for 16 fma and LDS is
// the busy unit; 8 x 8 reads 128 bytes for 64 fma, so the fp64 pipe is.  Channels arrive sixteen at a time: the next
// chunk is in flight in registers while the present one is consumed, and goes to the other LDS buffer (one barrier
// per chunk).  Each accumulator still sees its channels in ascending order: the same fma chain, the same bits.
template <bool KEYS>
__global__ __launch_bounds__(256, 2) void scores_big_kernel(const double *__restrict__ qbar, const double *__restrict__ kbar,
                                                            int Nqb, int Nkb, int pitch, double *__restrict__ S)
{
    constexpr int TILE = 128, CH = 16, PER = TILE * CH / 256, LP = TILE + 2;
    __shared__ __align__(16) double qs[2][CH][LP];
    __shared__ __align__(16) double ks[2][CH][LP];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int j0 = blockIdx.x * TILE, i0 = blockIdx.y * TILE;
    const long bh = blockIdx.z;
    const double *qh = qbar + bh * (long)Nqb * kD;
    const double *kh = kbar + bh * (long)Nkb * kD;
    double acc[8][8];
#pragma unroll
    for (int a = 0; a < 8; ++a)
#pragma unroll
        for (int b = 0; b < 8; ++b) acc[a][b] = 0.0;
    // element r of a thread: channel (tid & 15) of row (tid >> 4) + 16 r of the chunk; rows past the end repeat the
    // last one (their results are not stored), so the loads are unconditional
    const int sd = tid & 15, srow = tid >> 4;
    const double *qsrc[PER], *ksrc[PER];
#pragma unroll
    for (int r = 0; r < PER; ++r) {
        qsrc[r] = qh + (long)min(i0 + srow + 16 * r, Nqb - 1) * kD + sd;
        ksrc[r] = kh + (long)min(j0 + srow + 16 * r, Nkb - 1) * kD + sd;
    }
    double qr[PER], kr[PER];
    auto fetch = [&](int c) {
#pragma unroll
        for (int r = 0; r < PER; ++r) { qr[r] = qsrc[r][c * CH]; kr[r] = ksrc[r][c * CH]; }
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int r = 0; r < PER; ++r) { qs[buf][sd][srow + 16 * r] = qr[r]; ks[buf][sd][srow + 16 * r] = kr[r]; }
    };
    fetch(0);
    stage(0);
    lds_barrier();
#pragma unroll
    for (int c = 0; c < kD / CH; ++c) {
        if (c + 1 < kD / CH) fetch(c + 1);
#pragma unroll 2
        for (int d = 0; d < CH; ++d) {
            double qv[8], kv[8];
#pragma unroll
            for (int a = 0; a < 8; ++a) { qv[a] = qs[c & 1][d][ty * 8 + a]; kv[a] = ks[c & 1][d][tx * 8 + a]; }
#pragma unroll
            for (int a = 0; a < 8; ++a)
#pragma unroll
                for (int b = 0; b < 8; ++b) acc[a][b] = fma(qv[a], kv[b], acc[a][b]);
        }
        if (c + 1 < kD / CH) {
            stage((c + 1) & 1);            // every wave is past the chunk before this one (the barrier of the last trip)
            lds_barrier();
        }
    }
    // a thread's eight results of a row are contiguous; the row pitch is a multiple of 8 entries
    const int gj = j0 + tx * 8;
    if constexpr (KEYS) {
        uint32_t *Kh = (uint32_t *)S + bh * (long)Nqb * pitch;
#pragma unroll
        for (int a = 0; a < 8; ++a) {
            const int gi = i0 + ty * 8 + a;
            if (gi < Nqb && gj < pitch) {
                uint4 *dst = (uint4 *)(Kh + (long)gi * pitch + gj);
                dst[0] = make_uint4((uint32_t)(desc_key(acc[a][0]) >> 32), (uint32_t)(desc_key(acc[a][1]) >> 32),
                                    (uint32_t)(desc_key(acc[a][2]) >> 32), (uint32_t)(desc_key(acc[a][3]) >> 32));
                dst[1] = make_uint4((uint32_t)(desc_key(acc[a][4]) >> 32), (uint32_t)(desc_key(acc[a][5]) >> 32),
                                    (uint32_t)(desc_key(acc[a][6]) >> 32), (uint32_t)(desc_key(acc[a][7]) >> 32));
            }
        }
    } else {
        double *Sh = S + bh * (long)Nqb * pitch;
#pragma unroll
        for (int a = 0; a < 8; ++a) {
            const int gi = i0 + ty * 8 + a;
            if (gi < Nqb && gj < pitch) {
                double2 *dst = (double2 *)(Sh + (long)gi * pitch + gj);
#pragma unroll
                for (int b = 0; b < 4; ++b) dst[b] = double2{acc[a][2 * b], acc[a][2 * b + 1]};
            }
        }
    }
}

// launches with at least one 128 x 128 tile for each of the chip's 512 workgroup slots (two per compute unit) use the
// big-tile kernel; smaller ones fill the chip better with 64 x 64 tiles
constexpr long kBigScoreTiles = 512;

hipError_t launch_scores(const double *qbar, const double *kbar, int BH, int Nqb, int Nkb,
                         int pitch, double *S, hipStream_t st)
{
    const dim3 big((Nkb + 127) / 128, (Nqb + 127) / 128, BH);
    if ((long)big.x * big.y * big.z >= kBigScoreTiles) {
        scores_big_kernel<false><<<big, 256, 0, st>>>(qbar, kbar, Nqb, Nkb, pitch, S);
        return hipGetLastError();
    }
    dim3 grid((Nkb + 63) / 64, (Nqb + 63) / 64, BH);
    scores_kernel<false><<<grid, 256, 0, st>>>(qbar, kbar, Nqb, Nkb, pitch, S);
    return hipGetLastError();
}

// ----------------------------------------------------------------------------------- select
// One wavefront per score row; lane l holds the keys of blocks j = m*64 + l.  A key is the
// bit pattern of the logit mapped so that unsigned ascending order == logit descending
// order; k-th smallest keys are found with an 8-bit-digit radix select on an LDS histogram
// (keys are first shifted to the row's [min,max] range so two or three passes suffice), and
// exact ties are resolved by ascending block index.

// Cross-lane steps as DPP moves (row shifts, then the two row broadcasts that carry a row's last lane into
// the following rows) instead of LDS permutes: a wave-wide scan or reduction is six short VALU steps.
//   kShr1/2/4/8: lane l reads lane l-n of its row of 16;  kBc15: rows 1 and 3 read lane 15 of the row before;
//   kBc31: rows 2 and 3 read lane 31.  A lane without a source receives `old`.
constexpr int kShr1 = 0x111, kShr2 = 0x112, kShr4 = 0x114, kShr8 = 0x118, kBc15 = 0x142, kBc31 = 0x143;
template <int CTRL, int ROWS>
__device__ __forceinline__ uint32_t dpp_get(uint32_t old, uint32_t src)
{
    return (uint32_t)__builtin_amdgcn_update_dpp((int)old, (int)src, CTRL, ROWS, 0xf, false);
}
// inclusive prefix sum over the 64 lanes
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v)
{
    v += dpp_get<kShr1, 0xf>(0u, v);
    v += dpp_get<kShr2, 0xf>(0u, v);
    v += dpp_get<kShr4, 0xf>(0u, v);
    v += dpp_get<kShr8, 0xf>(0u, v);
    v += dpp_get<kBc15, 0xa>(0u, v);
    v += dpp_get<kBc31, 0xc>(0u, v);
    return v;
}
template <bool MAX, int CTRL, int ROWS>
__device__ __forceinline__ uint64_t dpp_minmax_step(uint64_t v)
{
    const uint32_t lo = dpp_get<CTRL, ROWS>((uint32_t)v, (uint32_t)v), hi = dpp_get<CTRL, ROWS>((uint32_t)(v >> 32), (uint32_t)(v >> 32));
    const uint64_t w = ((uint64_t)hi << 32) | lo;      // a lane without a source sees its own value
    return MAX ? (w > v ? w : v) : (w < v ? w : v);
}
template <bool MAX>
__device__ __forceinline__ uint64_t wave_minmax_u64(uint64_t v)
{
    v = dpp_minmax_step<MAX, kShr1, 0xf>(v);
    v = dpp_minmax_step<MAX, kShr2, 0xf>(v);
    v = dpp_minmax_step<MAX, kShr4, 0xf>(v);
    v = dpp_minmax_step<MAX, kShr8, 0xf>(v);
    v = dpp_minmax_step<MAX, kBc15, 0xa>(v);
    v = dpp_minmax_step<MAX, kBc31, 0xc>(v);           // lane 63 now holds the result over all lanes
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, 63), hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), 63);
    return ((uint64_t)hi << 32) | lo;
}
__device__ __forceinline__ uint64_t wave_min_u64(uint64_t v) { return wave_minmax_u64<false>(v); }
__device__ __forceinline__ uint64_t wave_max_u64(uint64_t v) { return wave_minmax_u64<true>(v); }
// value of lane src (uniform) in every lane
__device__ __forceinline__ uint32_t bcast_u32(uint32_t v, int src)
{
    return (uint32_t)__builtin_amdgcn_readlane((int)v, __builtin_amdgcn_readfirstlane(src));
}
__device__ __forceinline__ uint64_t bcast_u64(uint64_t v, int src)
{
    return ((uint64_t)bcast_u32((uint32_t)(v >> 32), src) << 32) | bcast_u32((uint32_t)v, src);
}

// logit -> key with (key ascending) == (logit descending); -0.0 is folded onto +0.0
__device__ __forceinline__ uint64_t desc_key(double s)
{
    uint64_t u = (uint64_t)__double_as_longlong(s == 0.0 ? 0.0 : s);
    u = (u >> 63) ? ~u : (u | 0x8000000000000000ull);   // ascending with the value
    return ~u;
}
__device__ __forceinline__ double key_to_logit(uint64_t key)
{
    uint64_t u = ~key;
    u = (u >> 63) ? (u & 0x7FFFFFFFFFFFFFFFull) : ~u;
    return __longlong_as_double((long long)u);
}

#ifdef SLA_PROBE_TIME   /* timing probe only: cycle counter of one row's wave at the phase boundaries of the selection */
__device__ unsigned long long sla_select_probe_times[32];
__device__ int sla_select_probe_on;                      // set by the probed wave for the helpers it calls
#define SLA_ST(on, pt) do { if (on) { const unsigned long long t_ = __builtin_readcyclecounter(); if ((threadIdx.x & 63) == 0) sla_select_probe_times[pt] = t_; } } while (0)
extern "C" int sla_probe_read_select(unsigned long long *dst) { return (int)hipMemcpyFromSymbol(dst, HIP_SYMBOL(sla_select_probe_times), sizeof(unsigned long long) * 32); }
#else
#define SLA_ST(on, pt)
#endif

// (T, r, n): the k smallest (value, index) pairs among the candidates are the candidates with value < T plus the r
// lowest-index ones of the n candidates with value == T, or, if r == n == 1, the candidates with value <= T (T is then
// an upper bound of the one key at the threshold, below the next key, rather than that key itself).
struct Cut { uint32_t T; int r, n; };

// The row's keys live in LDS (kv[j] = key of block j) and every pass over them is a rolled loop.  (Held in registers
// with the loops unrolled the kernel was 18 000 instructions of straight-line code and, with 34 keys per lane, spilled.)
// The kernel is bound by instruction issue -- about three waves per SIMD, each instruction of a wave taking the SIMD
// some six cycles -- so the passes are written for few instructions per key: sixteen bytes per LDS read where the
// order of the keys does not matter, no predicated atomics (a key that does not count adds to a spare word of its
// lane instead, which costs one select where masking the lane out costs four scalar instructions).

// The keys a radix descent looks at.  AllKeys: every entry of kv[0, 256 nit), four consecutive ones per lane and trip.
struct AllKeys {
    const uint32_t *kv;
    int nit;
    template <class F>
    __device__ __forceinline__ void for_each(F f) const
    {
        const uint4 *q = (const uint4 *)kv + (threadIdx.x & 63);
#pragma unroll 2
        for (int it = 0; it < nit; ++it) {
            const uint4 v = q[it * 64];
            f(v.x); f(v.y); f(v.z); f(v.w);
        }
    }
};
// MemberKeys: entry 64 m + lane for the set bits m of the lane's mask.
struct MemberKeys {
    const uint32_t *kv;
    int nslots;
    uint64_t mem;
    template <class F>
    __device__ __forceinline__ void for_each(F f) const
    {
        const int lane = threadIdx.x & 63;
        for (int m = 0; m < nslots; ++m)
            if ((mem >> m) & 1) f(kv[m * 64 + lane]);
    }
};

// Radix descent, eight bits at a time from the top, for up to two ranks at once (want[t] = rank t wanted) over the
// keys of `keys`; while both ranks follow the same prefix one histogram serves both.  hist: two histograms of 256
// counters and, from spare_at on, a spare word per lane, private to the wave.  Requires 1 <= k[t] <= number of keys.
template <class Keys>
__device__ __forceinline__ void radix_cuts(const Keys keys, const int (&k)[2], const bool (&want)[2],
                                           uint32_t *hist, Cut (&cut)[2], bool probe = false, uint32_t spare_at = 512u)
{
    const int lane = threadIdx.x & 63;
    int pass_ = 0;
    (void)pass_; (void)probe;
    uint32_t prefix[2] = {0u, 0u};
    int kk[2] = {k[0], k[1]};
    bool act[2] = {want[0], want[1]};
    const uint32_t spare = spare_at + lane;           // (a caller that asks for one rank only needs one histogram: spare_at = 256)
    for (int shift = 24; shift >= 0 && (act[0] || act[1]); shift -= 8) {
        const bool both = act[0] && act[1], two = both && prefix[0] != prefix[1];
        wave_lds_sync();
        *(uint4 *)(hist + lane * 4) = make_uint4(0u, 0u, 0u, 0u);
        if (two) *(uint4 *)(hist + 256 + lane * 4) = make_uint4(0u, 0u, 0u, 0u);
        wave_lds_sync();
        const uint32_t pf0 = prefix[act[0] ? 0 : 1], pf1 = prefix[1];   // the first histogram counts for the first active rank
        SLA_ST(probe && pass_ < 4, 4 + 3 * pass_);
        if (shift == 24) {                                   // no prefix yet: every key counts (both ranks, one histogram)
            keys.for_each([&](uint32_t v) { atomicAdd(&hist[v >> 24], 1u); });
        } else if (!two) {
            keys.for_each([&](uint32_t v) {
                const uint32_t d = (v >> shift) & 255u;
                atomicAdd(&hist[(v >> (shift + 8)) == pf0 ? d : spare], 1u);
            });
        } else {
            keys.for_each([&](uint32_t v) {
                const uint32_t p = v >> (shift + 8), d = (v >> shift) & 255u;
                atomicAdd(&hist[p == pf0 ? d : spare], 1u);
                atomicAdd(&hist[p == pf1 ? 256u + d : spare], 1u);
            });
        }
        wave_lds_sync();
        SLA_ST(probe && pass_ < 4, 5 + 3 * pass_);
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            if (!act[t]) continue;
            const uint32_t *h = hist + ((t == 1 && two) ? 256 : 0);
            const uint4 c4 = *(const uint4 *)(h + lane * 4);
            const uint32_t c[4] = {c4.x, c4.y, c4.z, c4.w};
            const uint32_t mine = c[0] + c[1] + c[2] + c[3];
            const uint32_t incl = wave_incl_scan(mine), excl = incl - mine;
            const bool here = excl < (uint32_t)kk[t] && (uint32_t)kk[t] <= incl;
            const int src = __ffsll((long long)__ballot(here)) - 1;          // exactly one lane
            uint32_t before = excl, digit = 0, cnt = 0;
            if (here) {
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    if (cnt == 0) {
                        if (before + c[b] >= (uint32_t)kk[t]) { digit = lane * 4 + b; cnt = c[b]; }
                        else before += c[b];
                    }
                }
            }
            digit = bcast_u32(digit, src);
            before = bcast_u32(before, src);
            cnt = bcast_u32(cnt, src);
            prefix[t] = (prefix[t] << 8) | digit;
            kk[t] -= (int)before;
            if (shift == 0) { cut[t] = Cut{prefix[t], kk[t], (int)cnt}; act[t] = false; }
            else if (cnt == 1) {
                // one key carries this prefix: the largest value with the prefix cuts the keys where that key does
                cut[t] = Cut{(prefix[t] << shift) | ((1u << shift) - 1u), 1, 1};
                act[t] = false;
            }
        }
        SLA_ST(probe && pass_ < 4, 6 + 3 * pass_);
        ++pass_;
    }
}

// RegKeys: KPL values per lane, in registers (short rows).
template <int KPL>
struct RegKeys {
    const uint32_t (&w)[KPL];
    template <class F>
    __device__ __forceinline__ void for_each(F f) const
    {
#pragma unroll
        for (int m = 0; m < KPL; ++m) f(w[m]);
    }
};

// Finds (T, r): the k smallest (key, index) pairs of the row are exactly the keys < T plus the
// r lowest-index keys == T.  Requires 1 <= k <= Nkb.  Uniform across the wave.  hist: 256 counters private
// to this wave (LDS operations of one wave execute in order, so no workgroup barrier is involved).
template <int KPL>
__device__ __forceinline__ void radix_select(const uint64_t (&key)[KPL], int Nkb, int k, uint32_t *hist, uint64_t &T, int &r)
{
    const int lane = threadIdx.x & 63;
    uint64_t prefix = 0;
    int kk = k, shift = 56, nb = 0;
    for (;;) {
        wave_lds_sync();
#pragma unroll
        for (int b = 0; b < 4; ++b) hist[lane * 4 + b] = 0;
        wave_lds_sync();
#pragma unroll
        for (int m = 0; m < KPL; ++m) {
            const bool cand = (m * 64 + lane < Nkb) && (shift == 56 || (key[m] >> (shift + 8)) == prefix);
            if (cand) atomicAdd(&hist[(uint32_t)(key[m] >> shift) & 255u], 1u);
        }
        wave_lds_sync();
        uint32_t c[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) c[b] = hist[lane * 4 + b];
        const uint32_t mine = c[0] + c[1] + c[2] + c[3];
        const uint32_t incl = wave_incl_scan(mine);
        const uint32_t excl = incl - mine;
        const bool here = excl < (uint32_t)kk && (uint32_t)kk <= incl;
        const uint64_t bal = __ballot(here);
        const int src = __ffsll((long long)bal) - 1;          // exactly one lane
        uint32_t before = excl, digit = 0, cnt = 0;
        if (here) {
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                if (cnt == 0) {
                    if (before + c[b] >= (uint32_t)kk) { digit = lane * 4 + b; cnt = c[b]; }
                    else before += c[b];
                }
            }
        }
        digit = bcast_u32(digit, src);
        before = bcast_u32(before, src);
        nb = (int)bcast_u32(cnt, src);
        prefix = (prefix << 8) | digit;
        kk -= (int)before;
        if (nb == 1 || shift == 0) break;
        shift -= 8;
    }
    if (shift == 0) { T = prefix; r = kk; return; }
    // a single key carries this prefix: fetch it
    uint64_t found = 0;
    bool have = false;
#pragma unroll
    for (int m = 0; m < KPL; ++m)
        if ((m * 64 + lane < Nkb) && (key[m] >> shift) == prefix) { found = key[m]; have = true; }
    const int src = __ffsll((long long)__ballot(have)) - 1;
    T = bcast_u64(found, src);
    r = 1;
}

// Classifies one score row held by one wave (key[m] of lane l belongs to block j = 64 m + l; slots with
// j >= Nkb hold ~0) and writes labels / critical list / compressed softmax for that row.
template <int KPL>
__device__ __forceinline__ void classify_row_wave(uint64_t (&key)[KPL], long row, int Nkb, int k_c, int k_n, uint32_t *hist,
                                  uint64_t *__restrict__ mbits, int lab_pitch, int8_t *__restrict__ lab_dense,
                                  int32_t *__restrict__ crit_idx, float *__restrict__ Pc, float sm_scale)
{
    const int lane = threadIdx.x & 63;
    uint64_t kmin = ~0ull, kmax = 0;
#pragma unroll
    for (int m = 0; m < KPL; ++m)
        if (m * 64 + lane < Nkb) {
            kmin = key[m] < kmin ? key[m] : kmin;
            kmax = key[m] > kmax ? key[m] : kmax;
        }
    kmin = wave_min_u64(kmin);
    kmax = wave_max_u64(kmax);

    if (Pc) {   // compressed block-score softmax (fp32 output), max logit == smallest key
        const double smax = key_to_logit(kmin);
        float e[KPL], sum = 0.f;
#pragma unroll
        for (int m = 0; m < KPL; ++m) {
            e[m] = 0.f;
            if (m * 64 + lane < Nkb) { e[m] = __expf((float)((key_to_logit(key[m]) - smax) * (double)sm_scale)); sum += e[m]; }
        }
        sum = wave_sum(sum);
        const float inv = 1.f / sum;
#pragma unroll
        for (int m = 0; m < KPL; ++m)
            if (m * 64 + lane < Nkb) Pc[row * Nkb + m * 64 + lane] = e[m] * inv;
    }

    // Both ranks are first looked for among 32-bit values w = floor((s_max - s) 2^32 / (s_max - s_min)), which spread a
    // row like its logits (the keys' own leading digits are sign and exponent: nearly every key of a row in one bin).
    // w is a non-increasing function of the logit, so where the group at a threshold is taken whole (nearly always one
    // key) the cut of w is the cut of the exact order.  Otherwise the exact keys are ranked as before.
    const int k_keep = Nkb - k_n;          // first k_keep of the order are not negligible
    const bool want[2] = {k_c > 0 && k_c < Nkb, k_keep > 0 && k_keep < Nkb};
    uint32_t w[KPL];
    {
        const double s_max = key_to_logit(kmin), s_min = key_to_logit(kmax);
        const double span = s_max - s_min, scale = span > 0.0 ? 4294967040.0 / span : 0.0;   // 2^32 - 2^8: below the padding value
#pragma unroll
        for (int m = 0; m < KPL; ++m) w[m] = (m * 64 + lane < Nkb) ? (uint32_t)((s_max - key_to_logit(key[m])) * scale) : ~0u;
    }
    // (one rank per descent: a single histogram, so that four workgroups of the fused kernel still fit a CU's LDS)
    Cut cut[2] = {Cut{0u, 0, 0}, Cut{0u, 0, 0}}, c1[2];
    const bool one[2] = {true, false};
    if (want[0]) { const int k1[2] = {k_c, 0}; radix_cuts(RegKeys<KPL>{w}, k1, one, hist, c1, false, 256u); cut[0] = c1[0]; }
    if (want[1]) { const int k1[2] = {k_keep, 0}; radix_cuts(RegKeys<KPL>{w}, k1, one, hist, c1, false, 256u); cut[1] = c1[0]; }
    const bool whole = (!want[0] || cut[0].r == cut[0].n) && (!want[1] || cut[1].r == cut[1].n);

    uint64_t Tc = 0, Tn = 0;
    int rc = 0, rn = 0;
    if (!whole) {
        // shift keys into the row's range so the leading radix digits discriminate
        const uint64_t range = kmax - kmin;
        const int sh = range ? __clzll((long long)range) : 0;
#pragma unroll
        for (int m = 0; m < KPL; ++m) key[m] = (key[m] - kmin) << sh;   // invalid slots are never read
        if (want[0]) radix_select<KPL>(key, Nkb, k_c, hist, Tc, rc);
        if (want[1]) radix_select<KPL>(key, Nkb, k_keep, hist, Tn, rn);
    }

    int tie_c = 0, tie_n = 0, ncrit = 0;
    const uint64_t lt = (1ull << lane) - 1;
#pragma unroll
    for (int m = 0; m < KPL; ++m) {
        const int j = m * 64 + lane;
        const bool valid = j < Nkb;
        bool selc, seln;
        if (k_c <= 0) selc = false;
        else if (k_c >= Nkb) selc = valid;
        else if (whole) selc = valid && w[m] <= cut[0].T;
        else {
            const bool eq = valid && key[m] == Tc;
            const uint64_t b = __ballot(eq);
            selc = valid && (key[m] < Tc || (eq && tie_c + (int)__popcll(b & lt) < rc));
            tie_c += __popcll(b);
        }
        if (k_keep <= 0) seln = false;
        else if (k_keep >= Nkb) seln = valid;
        else if (whole) seln = valid && w[m] <= cut[1].T;
        else {
            const bool eq = valid && key[m] == Tn;
            const uint64_t b = __ballot(eq);
            seln = valid && (key[m] < Tn || (eq && tie_n + (int)__popcll(b & lt) < rn));
            tie_n += __popcll(b);
        }
        const int8_t lab = selc ? 2 : (seln ? 1 : 0);
        const uint64_t mb = __ballot(lab == 1);                 // marginal mask of this chunk, bit = lane
        if (lane == 0 && m * 64 < lab_pitch) mbits[row * (lab_pitch >> 6) + m] = mb;
        if (lab_dense && valid) lab_dense[row * Nkb + j] = lab;
        if (crit_idx) {
            const uint64_t b = __ballot(selc);
            const int pos = ncrit + (int)__popcll(b & lt);
            if (selc && pos < k_c) crit_idx[row * k_c + pos] = j;
            ncrit += __popcll(b);
        }
    }
}

template <int KPL>
__global__ __launch_bounds__(64) void select_kernel(const double *__restrict__ S, int pitch, int Nkb, int k_c, int k_n,
                                                    uint64_t *__restrict__ mbits, int lab_pitch,
                                                    int8_t *__restrict__ lab_dense, int32_t *__restrict__ crit_idx,
                                                    float *__restrict__ Pc, double *__restrict__ S_dense, float sm_scale)
{
    __shared__ __align__(16) uint32_t hist[256 + 64];     // a histogram and a spare word per lane
    const long row = blockIdx.x;
    const int lane = threadIdx.x;
    const double *s = S + row * pitch;
    uint64_t key[KPL];
#pragma unroll
    for (int m = 0; m < KPL; ++m) {
        const int j = m * 64 + lane;
        key[m] = ~0ull;
        if (j < Nkb) {
            const double v = s[j];
            if (S_dense) S_dense[row * Nkb + j] = v;
            key[m] = desc_key(v);
        }
    }
    classify_row_wave<KPL>(key, row, Nkb, k_c, k_n, hist, mbits, lab_pitch, lab_dense, crit_idx, Pc, sm_scale);
}

// Fused classifier for short rows (Nkb <= 64 KPL <= 256): block mean of Q, pooled logits and
// classification in one launch.  A workgroup of four waves takes four consecutive query blocks of one
// (b, h).  Lane d of wave w first forms channel d of the block mean of query block w (serial fp64 sum
// over the tokens in ascending order, times 1/count; the rows come in as whole 16-byte pieces through the wave's slice of LDS).  Chunk of 64 key blocks by chunk, the K means are staged in LDS
// (the next chunk already on its way in registers) and lane l of wave w runs the 64-step fma chain of
// (query block w, key block l), reading its K mean two channels per LDS access and channel d of the
// Q mean out of lane d; the logits never leave registers.
template <int KPL, bool FP8>
__global__ __launch_bounds__(256) void classify_fused_kernel(const void *__restrict__ Q, const float *__restrict__ sQ, RowMap rm,
                                                             const double *__restrict__ kbar, int N, int bq, int Nqb, int Nkb,
                                                             int k_c, int k_n, uint64_t *__restrict__ mbits, int lab_pitch,
                                                             int8_t *__restrict__ lab_dense, int32_t *__restrict__ crit_idx,
                                                             float *__restrict__ Pc, double *__restrict__ S_dense,
                                                             double *__restrict__ qbar_out, float sm_scale)
{
    constexpr int kPitch = 66;             // doubles per row of the K-mean buffer: 16-byte aligned rows, and the
                                           // sixteen lanes of one 16-byte access pass cover all 64 banks once
    __shared__ __align__(16) double ks[64 * kPitch];
    __shared__ __align__(16) uint32_t hist[4][256 + 64];   // per wave: a histogram and a spare word per lane
    // every kernel argument is fetched here, in one batch of scalar loads (left to the compiler: a dozen round trips to the
    // scalar cache, each in front of the first use of an argument)
    asm volatile("" ::"s"(Q), "s"(sQ), "s"(rm.bs), "s"(rm.hs), "s"(rm.ts), "s"(rm.H), "s"(kbar), "s"(N), "s"(bq), "s"(Nqb), "s"(Nkb), "s"(k_c), "s"(k_n),
                 "s"(mbits), "s"(lab_pitch), "s"(lab_dense), "s"(crit_idx), "s"(Pc), "s"(S_dense), "s"(qbar_out), "s"(sm_scale));
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const long bh = blockIdx.y;
    const int i = blockIdx.x * 4 + wave;
    const bool rowok = i < Nqb;
    const long row = bh * Nqb + i;
    const double *kh = kbar + bh * (long)Nkb * kD;

    double2 nx[8];                         // the chunk of K means on its way to LDS (two channels per lane and load)
    auto load_chunk = [&](int m) {
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int idx = tid + 256 * r, j = m * 64 + (idx >> 5);
            nx[r] = j < Nkb ? *(const double2 *)(kh + (long)j * kD + (idx & 31) * 2) : double2{0.0, 0.0};
        }
    };
    load_chunk(0);

    double mean = 0.0;
    if (rowok && KPL == 1) {
        // Rows of at most 64 key blocks (frame attention): the block arrives 64 tokens at a time as whole rows (16-byte
        // pieces, a wave instruction moves 1 KB of consecutive memory) into the wave's slice of the K-mean buffer, which
        // is idle until the first chunk of K means is stored below; lane d then adds channel d of the tokens in
        // ascending order (the order of the sum is part of the contract).  Rows past a ragged end repeat the last one
        // and are not added.  (Measured: 18 % faster there; with more chunks of K means LDS is the busy unit and the
        // direct loads below are faster.)
        const int t0 = i * bq, cnt = min(bq, N - t0);
        uint8_t *stg = (uint8_t *)ks + wave * 8192;
        double acc = 0.0;
        const double sc = FP8 ? (double)sQ[row] : 1.0;
        for (int h0 = 0; h0 < cnt; h0 += 64) {
            const int nrow = min(64, cnt - h0);
            if (FP8) {
                const uint8_t *x = (const uint8_t *)Q + rm.head(bh) + (size_t)(t0 + h0) * rm.ts + (lane & 3) * 16;
                uint4 v[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) v[k] = *(const uint4 *)(x + (size_t)min((lane >> 2) + 16 * k, nrow - 1) * rm.ts);
#pragma unroll
                for (int k = 0; k < 4; ++k) *(uint4 *)(stg + ((lane >> 2) + 16 * k) * 64 + (lane & 3) * 16) = v[k];
            } else {
                const uint16_t *x = (const uint16_t *)Q + rm.head(bh) + (size_t)(t0 + h0) * rm.ts + (lane & 7) * 8;
                uint4 v[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) v[k] = *(const uint4 *)(x + (size_t)min((lane >> 3) + 8 * k, nrow - 1) * rm.ts);
#pragma unroll
                for (int k = 0; k < 8; ++k) *(uint4 *)(stg + ((lane >> 3) + 8 * k) * 128 + (lane & 7) * 16) = v[k];
            }
            wave_lds_sync();
            if (FP8) {
#pragma unroll 16
                for (int t = 0; t < nrow; ++t) acc += (double)__builtin_amdgcn_cvt_f32_fp8((int)stg[t * 64 + lane], 0) * sc;
            } else {
#pragma unroll 16
                for (int t = 0; t < nrow; ++t) acc += (double)bf16_bits_to_f32(*(const uint16_t *)(stg + t * 128 + 2 * lane));
            }
            wave_lds_sync();               // the next 64 tokens overwrite the slice
        }
        mean = acc * (1.0 / (double)cnt);
        if (qbar_out) qbar_out[row * kD + lane] = mean;
    } else if (rowok) {                    // 2-byte (1-byte) loads straight from global memory: LDS is the busy unit here
        const int t0 = i * bq, cnt = min(bq, N - t0);
        double acc = 0.0;
        if (FP8) {
            const uint8_t *x = (const uint8_t *)Q + rm.head(bh) + (size_t)t0 * rm.ts + lane;
            const double sc = (double)sQ[row];
#pragma unroll 16
            for (int t = 0; t < cnt; ++t) acc += (double)__builtin_amdgcn_cvt_f32_fp8((int)x[(size_t)t * rm.ts], 0) * sc;
        } else {
            const uint16_t *x = (const uint16_t *)Q + rm.head(bh) + (size_t)t0 * rm.ts + lane;
#pragma unroll 16
            for (int t = 0; t < cnt; ++t) acc += (double)bf16_bits_to_f32(x[(size_t)t * rm.ts]);
        }
        mean = acc * (1.0 / (double)cnt);
        if (qbar_out) qbar_out[row * kD + lane] = mean;
    }
    const int mlo = __double2loint(mean), mhi = __double2hiint(mean);

    uint64_t key[KPL];
#pragma unroll
    for (int m = 0; m < KPL; ++m) {
        __syncthreads();                   // previous chunk consumed
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int idx = tid + 256 * r;
            *(double2 *)(ks + (idx >> 5) * kPitch + (idx & 31) * 2) = nx[r];
        }
        __syncthreads();
        if (m + 1 < KPL) load_chunk(m + 1);
        double s = 0.0;
#pragma unroll
        for (int d = 0; d < kD; d += 2) {
            const double2 kv = *(const double2 *)(ks + lane * kPitch + d);
            const double q0 = __hiloint2double(__builtin_amdgcn_readlane(mhi, d), __builtin_amdgcn_readlane(mlo, d));
            const double q1 = __hiloint2double(__builtin_amdgcn_readlane(mhi, d + 1), __builtin_amdgcn_readlane(mlo, d + 1));
            s = fma(q0, kv.x, s);
            s = fma(q1, kv.y, s);
        }
        const int j = m * 64 + lane;
        key[m] = ~0ull;
        if (rowok && j < Nkb) {
            if (S_dense) S_dense[row * Nkb + j] = s;
            key[m] = desc_key(s);
        }
    }
    if (rowok)
        classify_row_wave<KPL>(key, row, Nkb, k_c, k_n, hist[wave], mbits, lab_pitch, lab_dense, crit_idx, Pc, sm_scale);
}

// ---- workgroup-per-row variant for long rows (Nkb > 256) ------------------------------------
// NT threads (128 or 256), thread t owns the KPT consecutive blocks j = t*KPT .. t*KPT+KPT-1, so index order
// is (thread, slot) order and every ordered step (tie ranks, index-list compaction) is one
// workgroup-wide exclusive scan of per-thread counts.

struct SelShared {
    uint32_t mb[128];      // marginal mask of the row, one bit per key block
    uint32_t hist[256];
    uint32_t wsum[4];
    uint32_t bc[4];
    uint64_t red[8];
};

// exclusive prefix over the NT threads of per-thread value v; *total receives the sum
template <int NT>
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, SelShared &sh, uint32_t *total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t incl = wave_incl_scan(v);
    __syncthreads();                                   // wsum may still be read by a previous scan
    if (lane == 63) sh.wsum[wave] = incl;
    __syncthreads();
    uint32_t base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < NT / 64; ++w) { const uint32_t x = sh.wsum[w]; if (w < wave) base += x; tot += x; }
    if (total) *total = tot;
    return base + incl - v;
}

template <int KPT, int NT>
__device__ __forceinline__ void block_radix_select(const uint64_t (&key)[KPT], int j0, int Nkb, int k, SelShared &sh, uint64_t &T, int &r)
{
    constexpr int BPT = 256 / NT;                 // histogram bins per thread
    const int tid = threadIdx.x;
    uint64_t prefix = 0;
    int kk = k, shift = 56, nb = 0;
    for (;;) {
        __syncthreads();
#pragma unroll
        for (int b = 0; b < BPT; ++b) sh.hist[tid * BPT + b] = 0;
        __syncthreads();
#pragma unroll
        for (int m = 0; m < KPT; ++m) {
            const bool cand = (j0 + m < Nkb) && (shift == 56 || (key[m] >> (shift + 8)) == prefix);
            if (cand) atomicAdd(&sh.hist[(uint32_t)(key[m] >> shift) & 255u], 1u);
        }
        __syncthreads();
        uint32_t c[BPT], mine = 0;
#pragma unroll
        for (int b = 0; b < BPT; ++b) { c[b] = sh.hist[tid * BPT + b]; mine += c[b]; }
        uint32_t before = block_excl_scan<NT>(mine, sh, nullptr);
        if (before < (uint32_t)kk && (uint32_t)kk <= before + mine) {       // exactly one thread
#pragma unroll
            for (int b = 0; b < BPT; ++b) {
                if (before + c[b] >= (uint32_t)kk) { sh.bc[0] = tid * BPT + b; sh.bc[1] = before; sh.bc[2] = c[b]; break; }
                before += c[b];
            }
        }
        __syncthreads();
        prefix = (prefix << 8) | sh.bc[0];
        kk -= (int)sh.bc[1];
        nb = (int)sh.bc[2];
        if (nb == 1 || shift == 0) break;
        shift -= 8;
    }
    if (shift == 0) { T = prefix; r = kk; return; }
    __syncthreads();
#pragma unroll
    for (int m = 0; m < KPT; ++m)
        if ((j0 + m < Nkb) && (key[m] >> shift) == prefix) sh.red[0] = key[m];   // exactly one thread
    __syncthreads();
    T = sh.red[0];
    r = 1;
}

template <int KPT, int NT>
__global__ __launch_bounds__(NT) void select_block_kernel(const double *__restrict__ S, int pitch, int Nkb, int k_c, int k_n,
                                                           uint64_t *__restrict__ mbits, int lab_pitch,
                                                           int8_t *__restrict__ lab_dense, int32_t *__restrict__ crit_idx,
                                                           float *__restrict__ Pc, double *__restrict__ S_dense, float sm_scale)
{
    __shared__ SelShared sh;
    const long row = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int j0 = tid * KPT;
    const double *s = S + row * pitch;
    if (tid < 128) sh.mb[tid] = 0;          // ordered before its use by the barriers of the selection below (NT >= 128)
    uint64_t key[KPT];
    uint64_t kmin = ~0ull, kmax = 0;
#pragma unroll
    for (int m = 0; m < KPT; ++m) {
        const int j = j0 + m;
        key[m] = ~0ull;
        if (j < Nkb) {
            const double v = s[j];
            if (S_dense) S_dense[row * Nkb + j] = v;
            key[m] = desc_key(v);
            kmin = key[m] < kmin ? key[m] : kmin;
            kmax = key[m] > kmax ? key[m] : kmax;
        }
    }
    kmin = wave_min_u64(kmin);
    kmax = wave_max_u64(kmax);
    if (lane == 0) { sh.red[wave] = kmin; sh.red[4 + wave] = kmax; }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < NT / 64; ++w) {
        kmin = sh.red[w] < kmin ? sh.red[w] : kmin;
        kmax = sh.red[4 + w] > kmax ? sh.red[4 + w] : kmax;
    }
    __syncthreads();

    if (Pc) {
        const double smax = key_to_logit(kmin);
        float e[KPT], sum = 0.f;
#pragma unroll
        for (int m = 0; m < KPT; ++m) {
            e[m] = 0.f;
            if (j0 + m < Nkb) { e[m] = __expf((float)((key_to_logit(key[m]) - smax) * (double)sm_scale)); sum += e[m]; }
        }
        sum = wave_sum(sum);
        float *fs = (float *)sh.wsum;
        if (lane == 0) fs[wave] = sum;
        __syncthreads();
        float tot = 0.f;
#pragma unroll
        for (int w = 0; w < NT / 64; ++w) tot += fs[w];
        const float inv = 1.f / tot;
        __syncthreads();
#pragma unroll
        for (int m = 0; m < KPT; ++m)
            if (j0 + m < Nkb) Pc[row * Nkb + j0 + m] = e[m] * inv;
    }

    const uint64_t range = kmax - kmin;
    const int shn = range ? __clzll((long long)range) : 0;
#pragma unroll
    for (int m = 0; m < KPT; ++m) key[m] = (key[m] - kmin) << shn;

    const int k_keep = Nkb - k_n;
    uint64_t Tc = 0, Tn = 0;
    int rc = 0, rn = 0;
    const bool do_c = k_c > 0 && k_c < Nkb, do_n = k_keep > 0 && k_keep < Nkb;
    if (do_c) block_radix_select<KPT, NT>(key, j0, Nkb, k_c, sh, Tc, rc);
    if (do_n) block_radix_select<KPT, NT>(key, j0, Nkb, k_keep, sh, Tn, rn);

    // ranks among exact ties of each threshold, in index order
    uint32_t eqc = 0, eqn = 0;
#pragma unroll
    for (int m = 0; m < KPT; ++m) {
        const bool valid = j0 + m < Nkb;
        eqc += (do_c && valid && key[m] == Tc) ? 1u : 0u;
        eqn += (do_n && valid && key[m] == Tn) ? 1u : 0u;
    }
    uint32_t tie_c = do_c ? block_excl_scan<NT>(eqc, sh, nullptr) : 0u;
    uint32_t tie_n = do_n ? block_excl_scan<NT>(eqn, sh, nullptr) : 0u;

    int8_t lab[KPT];
    uint32_t ncrit = 0;
#pragma unroll
    for (int m = 0; m < KPT; ++m) {
        const bool valid = j0 + m < Nkb;
        bool selc, seln;
        if (!do_c) selc = k_c > 0 && valid;            // k_c >= Nkb: everything critical; k_c == 0: nothing
        else {
            const bool eq = valid && key[m] == Tc;
            selc = valid && (key[m] < Tc || (eq && (int)tie_c < rc));
            tie_c += eq ? 1u : 0u;
        }
        if (!do_n) seln = k_keep > 0 && valid;
        else {
            const bool eq = valid && key[m] == Tn;
            seln = valid && (key[m] < Tn || (eq && (int)tie_n < rn));
            tie_n += eq ? 1u : 0u;
        }
        lab[m] = selc ? 2 : (seln ? 1 : 0);
        ncrit += selc ? 1u : 0u;
    }
    uint32_t mine = 0;                                          // marginal bits of this thread's KPT blocks
#pragma unroll
    for (int m = 0; m < KPT; ++m) {
        const int j = j0 + m;
        mine |= (lab[m] == 1 ? 1u : 0u) << m;
        if (lab_dense && j < Nkb) lab_dense[row * Nkb + j] = lab[m];
    }
    {   // assemble the row's marginal mask in LDS (cleared at kernel entry) and write it as whole dwords
        const int w = j0 >> 5, off = j0 & 31;
        if (mine) {
            atomicOr(&sh.mb[w], mine << off);
            if (off + KPT > 32 && (mine >> (32 - off))) atomicOr(&sh.mb[w + 1], mine >> (32 - off));
        }
        __syncthreads();
        if (tid < (lab_pitch >> 5)) ((uint32_t *)mbits)[row * (lab_pitch >> 5) + tid] = sh.mb[tid];
    }
    if (crit_idx) {
        uint32_t pos = block_excl_scan<NT>(ncrit, sh, nullptr);
#pragma unroll
        for (int m = 0; m < KPT; ++m)
            if (lab[m] == 2) { if ((int)pos < k_c) crit_idx[row * k_c + pos] = j0 + m; ++pos; }
    }
}

template <int KPT, int NT>
static hipError_t launch_select_block_t(const double *S, int pitch, long rows, int Nkb, int k_c, int k_n, uint64_t *mbits,
                                        int lab_pitch, int8_t *lab_dense, int32_t *crit_idx, float *Pc, double *S_dense,
                                        float sm_scale, hipStream_t st)
{
    select_block_kernel<KPT, NT><<<(unsigned)rows, NT, 0, st>>>(S, pitch, Nkb, k_c, k_n, mbits, lab_pitch, lab_dense,
                                                                crit_idx, Pc, S_dense, sm_scale);
    return hipGetLastError();
}

template <int KPL>
static hipError_t launch_select_t(const double *S, int pitch, long rows, int Nkb, int k_c, int k_n, uint64_t *mbits,
                                  int lab_pitch, int8_t *lab_dense, int32_t *crit_idx, float *Pc, double *S_dense,
                                  float sm_scale, hipStream_t st)
{
    select_kernel<KPL><<<(unsigned)rows, 64, 0, st>>>(S, pitch, Nkb, k_c, k_n, mbits, lab_pitch, lab_dense, crit_idx,
                                                      Pc, S_dense, sm_scale);
    return hipGetLastError();
}

hipError_t launch_select(const double *S, int pitch, long rows, int Nkb, int k_c, int k_n,
                         uint64_t *mbits, int lab_pitch, int8_t *lab_dense, int32_t *crit_idx,
                         float *Pc, double *S_dense, float sm_scale, hipStream_t st)
{
#define SLA_SEL(K) return launch_select_t<K>(S, pitch, rows, Nkb, k_c, k_n, mbits, lab_pitch, lab_dense, crit_idx, Pc, S_dense, sm_scale, st)
    if (lab_pitch <= 64) SLA_SEL(1);
    if (lab_pitch <= 128) SLA_SEL(2);
    if (lab_pitch <= 256) SLA_SEL(4);
    // one wave per row up to 24 keys per lane: no workgroup barriers and 16 to 32 rows in flight per CU.  Beyond
    // that (36 keys per lane: 153 VGPRs, measured 20 % slower on 2147 key blocks) a workgroup takes the row.
    if (lab_pitch <= 512) SLA_SEL(8);
    if (lab_pitch <= 768) SLA_SEL(12);
    if (lab_pitch <= 1024) SLA_SEL(16);
    if (lab_pitch <= 1536) SLA_SEL(24);
#undef SLA_SEL
#define SLA_SELB(K) return launch_select_block_t<K, 256>(S, pitch, rows, Nkb, k_c, k_n, mbits, lab_pitch, lab_dense, crit_idx, Pc, S_dense, sm_scale, st)
    if (lab_pitch <= 2048) SLA_SELB(8);
    if (lab_pitch <= 2560) SLA_SELB(10);
    if (lab_pitch <= 3072) SLA_SELB(12);
    if (lab_pitch <= 4096) SLA_SELB(16);
#undef SLA_SELB
    return hipErrorInvalidValue;
}

template <int KPL>
static hipError_t launch_classify_fused_t(const void *Q, const float *sQ, bool fp8, RowMap rm, const double *kbar, int BH, int N, int bq,
                                          int Nqb, int Nkb, int k_c, int k_n, uint64_t *mbits, int lab_pitch, int8_t *lab_dense,
                                          int32_t *crit_idx, float *Pc, double *S_dense, double *qbar_out, float sm_scale,
                                          hipStream_t st)
{
    dim3 grid((Nqb + 3) / 4, BH);
    if (fp8) classify_fused_kernel<KPL, true><<<grid, 256, 0, st>>>(Q, sQ, rm, kbar, N, bq, Nqb, Nkb, k_c, k_n, mbits, lab_pitch, lab_dense, crit_idx, Pc, S_dense, qbar_out, sm_scale);
    else     classify_fused_kernel<KPL, false><<<grid, 256, 0, st>>>(Q, sQ, rm, kbar, N, bq, Nqb, Nkb, k_c, k_n, mbits, lab_pitch, lab_dense, crit_idx, Pc, S_dense, qbar_out, sm_scale);
    return hipGetLastError();
}

hipError_t launch_classify_fused(const void *Q, const float *sQ, bool fp8, RowMap rm, const double *kbar, int BH, int N, int bq, int Nkb,
                                 int k_c, int k_n, uint64_t *mbits, int lab_pitch, int8_t *lab_dense, int32_t *crit_idx,
                                 float *Pc, double *S_dense, double *qbar_out, float sm_scale, hipStream_t st)
{
    const int Nqb = (N + bq - 1) / bq;
#define SLA_CF(K) return launch_classify_fused_t<K>(Q, sQ, fp8, rm, kbar, BH, N, bq, Nqb, Nkb, k_c, k_n, mbits, lab_pitch, lab_dense, crit_idx, Pc, S_dense, qbar_out, sm_scale, st)
    if (Nkb <= 64) SLA_CF(1);
    if (Nkb <= 128) SLA_CF(2);
    if (Nkb <= 192) SLA_CF(3);
    if (Nkb <= 256) SLA_CF(4);
#undef SLA_CF
    return hipErrorInvalidValue;
}

// ---- long rows without the fp64 round trip (Nkb > 256, no logits or block-score softmax asked for) ------------
// The classifier needs the ORDER of a row's logits, not their values, and the order is almost always decided by
// the leading bits.  So the logits go to memory as 32-bit keys -- the upper half of the order-preserving 64-bit
// key of the fp64 logit: sign, exponent and 20 bits of mantissa -- and the selection runs on those (on a linear
// spread of the values they stand for, see select_keys_kernel): one 32-bit word per key.  Where a threshold falls
// inside a group the 32-bit values do not separate and the group is not taken as a whole, the members' logits are
// evaluated again (the same 64-step fma chain, so the same bits) and their exact keys decide, then the block
// index: the labels are those of the full fp64 order, bit for bit.

hipError_t launch_score_keys(const double *qbar, const double *kbar, int BH, int Nqb, int Nkb, int pitch, uint32_t *keys,
                             hipStream_t st)
{
    const dim3 big((Nkb + 127) / 128, (Nqb + 127) / 128, BH);
    if ((long)big.x * big.y * big.z >= kBigScoreTiles) {
        scores_big_kernel<true><<<big, 256, 0, st>>>(qbar, kbar, Nqb, Nkb, pitch, (double *)keys);
        return hipGetLastError();
    }
    dim3 grid((Nkb + 63) / 64, (Nqb + 63) / 64, BH);
    scores_kernel<true><<<grid, 256, 0, st>>>(qbar, kbar, Nqb, Nkb, pitch, (double *)keys);
    return hipGetLastError();
}

// wave-wide minimum / maximum of a 32-bit value (DPP steps as above), uniform result
template <bool MAX>
__device__ __forceinline__ uint32_t wave_minmax_u32(uint32_t v)
{
    auto step = [](uint32_t a, uint32_t b) { return MAX ? (a > b ? a : b) : (a < b ? a : b); };
    v = step(v, dpp_get<kShr1, 0xf>(v, v));
    v = step(v, dpp_get<kShr2, 0xf>(v, v));
    v = step(v, dpp_get<kShr4, 0xf>(v, v));
    v = step(v, dpp_get<kShr8, 0xf>(v, v));
    v = step(v, dpp_get<kBc15, 0xa>(v, v));
    v = step(v, dpp_get<kBc31, 0xc>(v, v));
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

// Per-lane bit mask (bit m = slot m) of the k first slots in the order (exact 64-bit key ascending, index ascending),
// given the cut of the row's 32-bit ranks (which are a non-decreasing function of the keys).  Works in place: the members
// of the group at the threshold carry first the upper, then, if those tie too, the lower halves of their exact keys in
// kv while they are ranked, and get their rank value back at the end.
__device__ __forceinline__ uint64_t take_first(uint32_t *kv, int nslots, const Cut &cut, int Nkb, const double *__restrict__ q,
                                               const double *__restrict__ kh, uint32_t *hist)
{
    const int lane = threadIdx.x & 63;
    uint64_t bits = 0;
    if (cut.r == cut.n) {                                   // the group at the threshold is taken as a whole (nearly always: n == 1)
#pragma unroll 4
        for (int m = 0; m < nslots; ++m) bits |= (uint64_t)(kv[m * 64 + lane] <= cut.T) << m;
        return bits;
    }
    // r of the n slots with rank value T: their exact keys decide.
    const uint32_t T = cut.T;
    uint64_t mem = 0;                                       // bit m: slot m belongs to the group
    for (int m = 0; m < nslots; ++m) {
        const uint32_t v = kv[m * 64 + lane];
        if (v == T && m * 64 + lane < Nkb) mem |= 1ull << m;
        else if (v < T) bits |= 1ull << m;
    }
    // The half `lower` of the exact keys of the slots in `who` -> kv.  One row with a group to resolve is on the
    // kernel's critical path (the other rows are long done), so the 64-step chain is fed from LDS (the Q mean, staged
    // once per call in the histogram's place) and from registers loaded eight channels at a time (more would cost the
    // whole kernel occupancy): eight memory round trips per member, each of four 16-byte loads.
    auto exact_halves = [&](uint64_t who, bool lower) {
        double *qs = (double *)hist;
        wave_lds_sync();
        qs[lane] = q[lane];
        wave_lds_sync();
        for (int m = 0; m < nslots; ++m) {
            if (!((who >> m) & 1)) continue;
            const int j = m * 64 + lane;
            const double *kr = kh + (long)j * kD;
            double s = 0.0;
#pragma unroll 1
            for (int c = 0; c < kD; c += 8) {
                double kk[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) kk[e] = kr[c + e];
#pragma unroll
                for (int e = 0; e < 8; ++e) s = fma(qs[c + e], kk[e], s);
            }
            const uint64_t key = desc_key(s);
            kv[j] = lower ? (uint32_t)key : (uint32_t)(key >> 32);
        }
        wave_lds_sync();
    };
    const uint64_t lt = (1ull << lane) - 1;
    if (cut.n <= 64) {
        // A small group (nearly always two or three blocks): the members' exact keys go to LDS in index order, lane t
        // counts the members in front of member t, and the first r are taken.  (The radix descents below are for large
        // groups: runs of equal blocks.)
        double *qs = (double *)hist;                        // words 0..127: the Q mean; 128..255: keys; 256..319: taken or not
        uint64_t *xk = (uint64_t *)(hist + 128);
        uint32_t *taken = hist + 256;
        wave_lds_sync();
        qs[lane] = q[lane];
        wave_lds_sync();
        int n = 0;
        for (int m = 0; m < nslots; ++m) {
            const bool in = (mem >> m) & 1;
            const uint64_t b = __ballot(in);
            if (!b) continue;
            if (in) {
                const double *kr = kh + (long)(m * 64 + lane) * kD;
                double s = 0.0;
#pragma unroll 1
                for (int c = 0; c < kD; c += 8) {
                    double kk[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) kk[e] = kr[c + e];
#pragma unroll
                    for (int e = 0; e < 8; ++e) s = fma(qs[c + e], kk[e], s);
                }
                xk[n + (int)__popcll(b & lt)] = desc_key(s);
            }
            n += __popcll(b);
        }
        wave_lds_sync();
        const uint64_t mine = lane < n ? xk[lane] : 0;
        int ahead = 0;
        for (int u = 0; u < n; ++u) {
            const uint64_t other = xk[u];
            ahead += (other < mine || (other == mine && u < lane)) ? 1 : 0;
        }
        taken[lane] = (lane < n && ahead < cut.r) ? 1u : 0u;
        wave_lds_sync();
        n = 0;
        for (int m = 0; m < nslots; ++m) {
            const bool in = (mem >> m) & 1;
            const uint64_t b = __ballot(in);
            if (!b) continue;
            if (in && taken[n + (int)__popcll(b & lt)]) bits |= 1ull << m;
            n += __popcll(b);
        }
        wave_lds_sync();
        return bits;
    }
    const bool w2[2] = {true, false};
    uint64_t who = mem;                                     // the slots still tied
    int need = cut.r;                                       // how many of them to take
    for (int level = 0; level < 2 && need > 0; ++level) {
        exact_halves(who, level == 1);
        const int k2[2] = {need, 0};
        Cut c2[2];
        radix_cuts(MemberKeys{kv, nslots, who}, k2, w2, hist, c2);
        const uint32_t T2 = c2[0].T;
        const bool whole = c2[0].r == c2[0].n;
        uint64_t tied = 0;
        int tie = 0;
        for (int m = 0; m < nslots; ++m) {
            const bool in = (who >> m) & 1;
            const uint32_t x = kv[m * 64 + lane];
            const bool eq = in && x == T2 && !whole;
            bool sel = in && (whole ? x <= T2 : x < T2);
            if (level == 1) {                               // equal keys: by index
                const uint64_t b = __ballot(eq);
                sel = sel || (eq && tie + (int)__popcll(b & lt) < c2[0].r);
                tie += __popcll(b);
            } else if (eq) tied |= 1ull << m;
            bits |= (uint64_t)sel << m;
        }
        who = tied;
        need = whole ? 0 : c2[0].r;
    }
    for (int m = 0; m < nslots; ++m)
        if ((mem >> m) & 1) kv[m * 64 + lane] = T;
    return bits;
}

// One wavefront per row; lane l owns the 32-bit keys of blocks j = 64 m + l (KPL: slots per lane the LDS buffer holds).
template <int KPL>
__global__ __launch_bounds__(64) void select_keys_kernel(const uint32_t *__restrict__ keys, int pitch, const double *__restrict__ qbar,
                                                         const double *__restrict__ kbar, int Nqb, int Nkb, int k_c, int k_n,
                                                         uint64_t *__restrict__ mbits, int lab_pitch,
                                                         int8_t *__restrict__ lab_dense, int32_t *__restrict__ crit_idx)
{
    __shared__ __align__(16) uint32_t kv[256 * ((KPL + 3) / 4)];
    __shared__ __align__(16) uint32_t hist[512 + 64];        // two histograms and a spare word per lane; later the critical list
    const long row = blockIdx.x;
    const int lane = threadIdx.x;
    const int nslots = (Nkb + 63) >> 6;
    const uint32_t *kr = keys + row * pitch;
#ifdef SLA_PROBE_TIME
    const bool sprobe = row == (long)(gridDim.x / 2 + 5);
    if (sprobe && lane < 32) sla_select_probe_times[lane] = 0;
#endif
    SLA_ST(sprobe, 0);
    // Lane l of trip `it` owns the four keys from j = 4 (64 it + l) on, in the row and in kv alike.  Trips whose 256 keys
    // all exist run unchecked; the last one or two read no further than the row's allocation (pitch: a multiple of
    // eight keys; what lies past Nkb is padding) and leave keys past the end out of the minimum and maximum.
    const int nit = (nslots + 3) >> 2, nfull = Nkb >> 8;
    const uint4 *kr4 = (const uint4 *)kr;
    uint4 *kv4 = (uint4 *)kv;
    uint32_t kmin = ~0u, kmax = 0u;
#pragma unroll 4
    for (int it = 0; it < nfull; ++it) {
        const uint4 v = kr4[it * 64 + lane];
        kv4[it * 64 + lane] = v;
        kmin = min(min(kmin, v.x), min(min(v.y, v.z), v.w));
        kmax = max(max(kmax, v.x), max(max(v.y, v.z), v.w));
    }
    for (int it = nfull; it < nit; ++it) {
        const int q = it * 64 + lane, j = 4 * q;
        const uint4 v = kr4[min(q, (pitch >> 2) - 1)];
        kv4[q] = v;
        if (j + 0 < Nkb) { kmin = min(kmin, v.x); kmax = max(kmax, v.x); }
        if (j + 1 < Nkb) { kmin = min(kmin, v.y); kmax = max(kmax, v.y); }
        if (j + 2 < Nkb) { kmin = min(kmin, v.z); kmax = max(kmax, v.z); }
        if (j + 3 < Nkb) { kmin = min(kmin, v.w); kmax = max(kmax, v.w); }
    }
    kmin = wave_minmax_u32<false>(kmin);
    kmax = wave_minmax_u32<true>(kmax);
    SLA_ST(sprobe, 1);
    // The selection ranks 32-bit values w = floor((s_max - s) * 2^32 / (s_max - s_min)) of the row, s being the logit
    // with the lower half of its fp64 pattern cleared (what a 32-bit key holds): a non-decreasing function of the key,
    // so cutting the row at a rank of w is cutting it at that rank of the keys wherever w separates them, and where it
    // does not (equal w at the threshold) the exact keys are consulted as for equal keys.  The keys themselves are a
    // poor radix: sign and exponent lead, and the first digit of a row puts three quarters of its keys into one bin
    // (atomics of forty lanes on one counter), the second digit most of those again.  w spreads a row like its logits.
    // Entries past the end get the largest value: they sort after every block of the row (equal values go by index).
    auto key_value = [](uint32_t key) {                       // the fp64 whose upper half the key encodes, lower half zero
        const uint32_t hi = key ^ ((uint32_t)~((int32_t)key >> 31) >> 1);
        return __longlong_as_double((long long)((uint64_t)hi << 32));
    };
    const double s_max = key_value(kmin), s_min = key_value(kmax);
    const double span = s_max - s_min, scale = span > 0.0 ? 4294967040.0 / span : 0.0;      // 2^32 - 2^8: below the padding value
    auto spread = [&](uint32_t key) { return (uint32_t)((s_max - key_value(key)) * scale); };
#pragma unroll 2
    for (int it = 0; it < nfull; ++it) {
        uint4 v = kv4[it * 64 + lane];
        v.x = spread(v.x); v.y = spread(v.y); v.z = spread(v.z); v.w = spread(v.w);
        kv4[it * 64 + lane] = v;
    }
    for (int it = nfull; it < nit; ++it) {
        const int q = it * 64 + lane, j = 4 * q;
        uint4 v = kv4[q];
        v.x = j + 0 < Nkb ? spread(v.x) : ~0u; v.y = j + 1 < Nkb ? spread(v.y) : ~0u;
        v.z = j + 2 < Nkb ? spread(v.z) : ~0u; v.w = j + 3 < Nkb ? spread(v.w) : ~0u;
        kv4[q] = v;
    }
    wave_lds_sync();                       // from here on the keys are read by other lanes than the ones that wrote them
    SLA_ST(sprobe, 2);

    const int k_keep = Nkb - k_n;          // the first k_keep of the order are not negligible
    const int k2[2] = {k_c, k_keep};
    const bool want[2] = {k_c > 0 && k_c < Nkb, k_keep > 0 && k_keep < Nkb};
    Cut cut[2] = {Cut{0u, 0, 0}, Cut{0u, 0, 0}};
#ifdef SLA_PROBE_TIME
    radix_cuts(AllKeys{kv, nit}, k2, want, hist, cut, sprobe);
#else
    radix_cuts(AllKeys{kv, nit}, k2, want, hist, cut);
#endif
    SLA_ST(sprobe, 16);

    // whole: the groups at both thresholds are taken whole (nearly always: single keys) and two compares label a slot;
    // otherwise per-lane bit masks say which slots are among the first k_c / k_keep of the exact order
    const bool whole = (!want[0] || cut[0].r == cut[0].n) && (!want[1] || cut[1].r == cut[1].n);
    uint64_t cm = 0, nm = 0;
    if (!whole) {
        const long bh = row / Nqb;
        const double *q = qbar + row * kD, *kh = kbar + bh * (long)Nkb * kD;
        if (want[0]) cm = take_first(kv, nslots, cut[0], Nkb, q, kh, hist);
        if (want[1]) nm = take_first(kv, nslots, cut[1], Nkb, q, kh, hist);
    }
    const uint32_t Tc = cut[0].T, Tn = cut[1].T;
    uint32_t mb_lo = 0, mb_hi = 0;         // lane m keeps the marginal mask of chunk m: one 8-byte store per lane at the end
    int ncrit = 0;
    // The critical list is collected in LDS (the histogram is done with) and leaves as whole rows at the end (stores
    // entry by entry each waited for the one before); a list longer than the buffer goes to memory entry by entry.
    const bool list_in_lds = k_c <= 512;
    wave_lds_sync();
    // bc, bn: the lanes of chunk m among the first k_c / k_keep of the order (as wave masks)
    auto emit = [&](int m, uint64_t bc, uint64_t bn) {
        const uint64_t mb = bn & ~bc;                           // marginal: kept, not critical
        if (lane == m) { mb_lo = (uint32_t)mb; mb_hi = (uint32_t)(mb >> 32); }
        const int j = m * 64 + lane;
        const bool selc = (bc >> lane) & 1;
        if (lab_dense && j < Nkb) lab_dense[row * Nkb + j] = selc ? 2 : (int8_t)((bn >> lane) & 1);
        if (crit_idx && bc) {                                   // (a chunk without critical block: nothing to list)
            const int pos = ncrit + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(bc >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bc, 0u));
            if (list_in_lds) hist[selc && pos < k_c ? pos : 512 + lane] = (uint32_t)j;     // other lanes write to a spare row
            else if (selc && pos < k_c) crit_idx[row * k_c + pos] = j;
            ncrit += __popcll(bc);
        }
    };
    if (whole && want[0] && want[1] && !lab_dense && crit_idx && list_in_lds) {
        // the forward's case, without a branch in the loop: every lane writes its block index, the ones that are not
        // critical to the spare row.  Four slots per trip, written out (the compiler does not unroll a loop of unknown
        // length around wave-wide votes), so that the four LDS reads are in flight together.
        auto step = [&](int m, uint32_t v) {
            const bool selc = v <= Tc;
            const uint64_t bc = __ballot(selc), mb = __ballot(v <= Tn) & ~bc;
            if (lane == m) { mb_lo = (uint32_t)mb; mb_hi = (uint32_t)(mb >> 32); }
            const int pos = ncrit + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(bc >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bc, 0u));
            hist[selc && pos < k_c ? pos : 512 + lane] = (uint32_t)(m * 64 + lane);
            ncrit += __popcll(bc);
        };
        int m = 0;
        for (; m + 4 <= nslots; m += 4) {
            const uint32_t v0 = kv[m * 64 + lane], v1 = kv[m * 64 + 64 + lane], v2 = kv[m * 64 + 128 + lane], v3 = kv[m * 64 + 192 + lane];
            step(m, v0); step(m + 1, v1); step(m + 2, v2); step(m + 3, v3);
        }
        for (; m < nslots; ++m) step(m, kv[m * 64 + lane]);
    } else if (whole) {
        const uint64_t all_c = k_c > 0 ? ~0ull : 0ull, all_n = k_keep > 0 ? ~0ull : 0ull;
        for (int m = 0; m < nslots; ++m) {
            const uint32_t v = kv[m * 64 + lane];
            const uint64_t valid = __ballot(m * 64 + lane < Nkb);
            emit(m, want[0] ? __ballot(v <= Tc) : (all_c & valid), want[1] ? __ballot(v <= Tn) : (all_n & valid));
        }
    } else {
        uint64_t vm = 0;
        for (int m = 0; m < nslots; ++m) vm |= (uint64_t)(m * 64 + lane < Nkb) << m;
        if (!want[0]) cm = k_c > 0 ? vm : 0ull;
        if (!want[1]) nm = k_keep > 0 ? vm : 0ull;
        for (int m = 0; m < nslots; ++m) emit(m, __ballot((cm >> m) & 1), __ballot((nm >> m) & 1));
    }
    SLA_ST(sprobe, 17);
    if (crit_idx && list_in_lds) {
        wave_lds_sync();
        const int n = min(ncrit, k_c);
        for (int t = lane; t < n; t += 64) crit_idx[row * k_c + t] = (int32_t)hist[t];
    }
    if (lane < (lab_pitch >> 6)) mbits[row * (lab_pitch >> 6) + lane] = ((uint64_t)mb_hi << 32) | mb_lo;
    SLA_ST(sprobe, 18);
}

template <int KPL>
static hipError_t launch_select_keys_t(const uint32_t *keys, int pitch, const double *qbar, const double *kbar, long rows, int Nqb,
                                       int Nkb, int k_c, int k_n, uint64_t *mbits, int lab_pitch, int8_t *lab_dense,
                                       int32_t *crit_idx, hipStream_t st)
{
    select_keys_kernel<KPL><<<(unsigned)rows, 64, 0, st>>>(keys, pitch, qbar, kbar, Nqb, Nkb, k_c, k_n, mbits, lab_pitch, lab_dense, crit_idx);
    return hipGetLastError();
}

hipError_t launch_select_keys(const uint32_t *keys, int pitch, const double *qbar, const double *kbar, long rows, int Nqb, int Nkb,
                              int k_c, int k_n, uint64_t *mbits, int lab_pitch, int8_t *lab_dense, int32_t *crit_idx, hipStream_t st)
{
#define SLA_SK(K) if (lab_pitch <= 64 * K) return launch_select_keys_t<K>(keys, pitch, qbar, kbar, rows, Nqb, Nkb, k_c, k_n, mbits, lab_pitch, lab_dense, crit_idx, st)
    SLA_SK(8); SLA_SK(16); SLA_SK(34); SLA_SK(64);
#undef SLA_SK
    return hipErrorInvalidValue;
}

// --------------------------------------------------------------------------- labels_prepare
// dense labels -> marginal bit mask + ascending critical index list per row (one wavefront per row;
// slots beyond the number of critical blocks found are set to -1, surplus ones are dropped).
__global__ __launch_bounds__(64) void labels_prepare_kernel(const int8_t *__restrict__ lab_dense, int Nkb, int k_c,
                                                            uint64_t *__restrict__ mbits, int lab_pitch,
                                                            int32_t *__restrict__ crit_idx)
{
    const long row = blockIdx.x;
    const int lane = threadIdx.x;
    const uint64_t lt = (1ull << lane) - 1;
    int n = 0;
    for (int j0 = 0; j0 < lab_pitch; j0 += 64) {
        const int j = j0 + lane;
        const int8_t v = j < Nkb ? lab_dense[row * Nkb + j] : (int8_t)0;
        const uint64_t mb = __ballot(v == 1);
        if (lane == 0) mbits[row * (lab_pitch >> 6) + (j0 >> 6)] = mb;
        const uint64_t b = __ballot(v == 2);
        const int pos = n + __popcll(b & lt);
        if (v == 2 && pos < k_c) crit_idx[row * k_c + pos] = j;
        n += __popcll(b);
    }
    for (int pos = n + lane; pos < k_c; pos += 64) crit_idx[row * k_c + pos] = -1;
}

hipError_t launch_labels_prepare(const int8_t *lab_dense, long rows, int Nkb, int k_c,
                                 uint64_t *mbits, int lab_pitch, int32_t *crit_idx, hipStream_t st)
{
    labels_prepare_kernel<<<(unsigned)rows, 64, 0, st>>>(lab_dense, Nkb, k_c, mbits, lab_pitch, crit_idx);
    return hipGetLastError();
}

}  // namespace sla
