// Shared device-side helpers of the gfx950 SLA kernels (types, bf16/fp8 conversions,
// wave-level primitives).  Wavefront size is 64 throughout.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sla {

constexpr int kD = 64;          // head dimension
constexpr int kBK = 64;         // key block size
constexpr int kStateRows = 65;  // rows of a block state: 64 rows of h^T plus one row of z
constexpr int kStateElems = kStateRows * kD;   // 4160

// Where the rows of one (b, h) live inside a Q / K / V / O tensor: element offset of (bh, token t, channel 0) is
// head(bh) + t * ts.  Head-major [B,H,N,64]: bs = H N 64, hs = N 64, ts = 64; token-major [B,N,H,64] (what a fused
// qkv projection leaves): bs = N H 64, hs = 64, ts = 64 H.  A row is 64 contiguous elements either way.
struct RowMap {
    long bs, hs;
    int ts, H;
    // (b, h) of bh = b H + h by 32-bit division (B H fits 31 bits; a 64-bit division is some sixty instructions)
    __host__ __device__ size_t head(long bh) const
    {
        const unsigned b = (unsigned)bh / (unsigned)H, h = (unsigned)bh - b * (unsigned)H;
        return (size_t)b * bs + (size_t)h * hs;
    }
};
inline RowMap make_rowmap(int token_major, int H, int N)
{
    RowMap m;
    m.H = H;
    if (token_major) { m.bs = (long)N * H * 64; m.hs = 64; m.ts = 64 * H; }
    else             { m.bs = (long)H * N * 64; m.hs = (long)N * 64; m.ts = 64; }
    return m;
}

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(8))) int i32x8;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(2))) int i32x2;

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// two bf16 packed in a dword -> two floats
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// acc + a.lo b.lo + a.hi b.hi for two dwords of packed bf16 (v_dot2c_f32_bf16)
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float acc)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), acc, false);
}

// round-to-nearest-even pack of two floats into one dword of bf16 (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    bf16x2 r;
    r[0] = (__bf16)lo;
    r[1] = (__bf16)hi;
    return __builtin_bit_cast(uint32_t, r);
}

__device__ __forceinline__ float bf16_round(float x) { return (float)(__bf16)x; }

// exp2 on the hardware transcendental unit (v_exp_f32); exp2(-inf) = 0
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// value held by the lane 32 positions away (lanes l and l^32 exchange)
__device__ __forceinline__ float xchg32(float v) { return __shfl_xor(v, 32, 64); }

__device__ __forceinline__ float wave_max(float v)
{
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v)
{
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// max of v over the lane pair (l, l^32): after the swap one register holds lanes 0..31 twice, the
// other lanes 32..63 twice
__device__ __forceinline__ float pair_max(float v)
{
    const uint32_t u = __float_as_uint(v);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

__device__ __forceinline__ bf16x8 pack8(const f32x16 &a, int base)
{
    uint4 o;
    o.x = pack_bf16(a[base + 0], a[base + 1]); o.y = pack_bf16(a[base + 2], a[base + 3]);
    o.z = pack_bf16(a[base + 4], a[base + 5]); o.w = pack_bf16(a[base + 6], a[base + 7]);
    return __builtin_bit_cast(bf16x8, o);
}

// Orders LDS traffic between the lanes of one wavefront (LDS operations of a wave execute in
// program order; this only stops the compiler from moving accesses across the point).
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Workgroup barrier that orders LDS traffic only: the wave waits for its own LDS operations and then
// for the other waves, but not for global loads still in flight to registers, which __syncthreads()
// would drain (its fence covers global memory) and with them any prefetch distance beyond one step.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// 1 KB copies global -> LDS: lane l moves the 16 bytes at base + voff(l) to LDS byte lds_addr + 16 l.
// base and lds_addr are wave-uniform (SGPRs); M0 carries the LDS address for the copy and is put back afterwards
// (the compiler reserves M0 for its own use and does not accept it as a clobber, so the statement leaves it as it
// found it).  The s_nop is the wait state the ISA asks for between a scalar write of M0 and an instruction that
// moves data into LDS through it (the compiler's hazard recogniser does not look inside inline assembly).
__device__ __forceinline__ void copy_1k_to_lds(const uint8_t *base, uint32_t voff, uint32_t lds_addr)
{
    uint32_t saved_m0;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2\n\ts_mov_b32 m0, %0"
                 : "=&s"(saved_m0) : "v"(voff), "s"(base), "s"(lds_addr) : "memory");
}
// One projection matrix W [e_in][e_out] -> WT [e_out][slot], slot 16s + 8g + 4a + b holding e_in = 16s + 8a + 4g + b
// (transposed, and with the same permutation of the contraction index as the V^T tiles, so the projection
// product of the attention kernel reads it with the fragment addressing of its main loop).  One workgroup of
// nthreads threads per matrix.
__device__ __forceinline__ void transpose_w_tile(const uint16_t *__restrict__ w, uint16_t *__restrict__ o, int nthreads)
{
    for (int idx = threadIdx.x; idx < kD * kD; idx += nthreads) {
        const int eo = idx >> 6, slot = idx & 63;
        const int ei = (slot & 0x33) | ((slot & 4) << 1) | ((slot & 8) >> 1);      // swap bits 2 and 3
        o[idx] = w[ei * kD + eo];
    }
}

// blockIdx -> work item so that each of the 8 XCDs (workgroups are dealt round-robin to them)
// walks a contiguous range of items and therefore keeps one head's K/V in its own L2.
__device__ __forceinline__ long xcd_remap(long bid, long total)
{
    const long chunk = (total + 7) / 8;
    return (bid & 7) * chunk + (bid >> 3);
}
inline long xcd_grid(long total) { return ((total + 7) / 8) * 8; }

}  // namespace sla
