// Shared device/host helpers of the gfx950 kernels: storage types, the fragment-packed matrix
// layout, wavefront reductions.  Everything here is for 64-wide wavefronts.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ccs {

typedef uint16_t bf16_t;  // bf16 bit pattern
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;

// 16-byte streaming accesses (data touched once: weights, cached K/V, clone traffic)
__device__ __forceinline__ uint4 ld_stream(const uint4 *p)
{
    u32x4_t v = __builtin_nontemporal_load((const u32x4_t *)p);
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void st_stream(uint4 *p, const uint4 &v)
{
    u32x4_t t = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(t, (u32x4_t *)p);
}

__device__ __forceinline__ float bf2f(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// fp32 -> bf16, round to nearest even; NaN stays NaN.  gfx950 converts in hardware
// (v_cvt_pk_bf16_f32, two values per instruction).
typedef __bf16 bf16x2_native_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ bf16_t f2bf(float f)
{
    return __builtin_bit_cast(bf16_t, (__bf16)f);
}
__device__ __forceinline__ uint32_t pack2bf(float lo, float hi)
{
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_native_t));
}
// 2^x on the transcendental unit (v_exp_f32); for softmax weights: x <= 0 or -inf
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float bf_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// ---- fragment-packed layout --------------------------------------------------------------
// A bf16 matrix [R, K] (R padded to 16, K a multiple of 32) that feeds the matrix cores is
// stored as 1 KiB fragments of 16 rows x 32 columns, fragment (rb, kb) at ((rb * K/32) + kb);
// inside a fragment lane l = (r % 16) + 16 * ((k % 32) / 8) owns 8 consecutive k (16 bytes).
// This is exactly the operand register layout of v_mfma_f32_16x16x32_bf16 (both operands), so
// a wavefront fetches one operand with one fully coalesced 1 KiB load and LDS copies of packed
// data are bank-conflict free.
__host__ __device__ __forceinline__ size_t packed_index(int r, int k, int kfrags)
{
    return ((((size_t)(r >> 4) * kfrags + (k >> 5)) * 64) + (r & 15) + 16 * ((k & 31) >> 3)) * 8 + (k & 7);
}

// Weights use the same fragments in a grouped order: the 16-row blocks are taken in groups of
// kWGroup (128 rows; the block count is padded to a multiple, padding fragments are zero) and
// fragment (nb, kb) sits at ((nb / kWGroup) * K/32 + kb) * kWGroup + nb % kWGroup.  The fragments
// of one group for one k-step are then one contiguous 8 KiB piece and consecutive k-steps follow
// each other, which is what a weight-streaming wavefront reads.
constexpr int kWGroup = 8;
__host__ __device__ __forceinline__ size_t weight_fragment(int nb, int kb, int kfrags)
{
    return ((size_t)(nb / kWGroup) * kfrags + kb) * kWGroup + (nb % kWGroup);
}
__host__ __device__ __forceinline__ size_t packed_weight_bytes(int N, int K)
{
    const size_t nblk = ((size_t)(N + 15) / 16 + kWGroup - 1) / kWGroup * kWGroup;
    return nblk * 16 * (size_t)K * 2;
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// Rotary angle of pair i at position pos from the per-module table of inverse frequencies
// (theta_i = base^(-2i/d) split into an fp32 head and tail, computed once in fp64): the product
// pos * theta_i is formed with an exact fp32 residual, the head goes through the accurate
// sincosf and the residual is applied to first order, so the angle error stays ~1e-7 rad at any
// position instead of growing with pos * 2^-24.
__device__ __forceinline__ void rope_cs(const float2 *__restrict__ tab, int i, int pos, float &c, float &s)
{
    const float2 f = tab[i];
    const float p = (float)pos;
    const float a = p * f.x;
    const float dl = fmaf(p, f.y, fmaf(p, f.x, -a));
    float s0, c0;
    sincosf(a, &s0, &c0);
    s = fmaf(dl, c0, s0);
    c = fmaf(-dl, s0, c0);
}

// Cached length of sequence i in a decode step, forced into [0, cap - 1]: the host validates its
// copy of the lengths, this keeps a device copy that disagrees from pushing accesses out of the cache.
__device__ __forceinline__ int cached_len(const int32_t *__restrict__ lens, int i, int cap)
{
    return min(max(lens[i], 0), cap - 1);
}

template <typename T> struct io;
template <> struct io<float> {
    static __device__ __forceinline__ float ld(const float *p) { return *p; }
    static __device__ __forceinline__ void st(float *p, float v) { *p = v; }
};
template <> struct io<bf16_t> {
    static __device__ __forceinline__ float ld(const bf16_t *p) { return bf2f(*p); }
    static __device__ __forceinline__ void st(bf16_t *p, float v) { *p = f2bf(v); }
};

}  // namespace ccs
