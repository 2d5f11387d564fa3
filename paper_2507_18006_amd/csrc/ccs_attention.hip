// KV-cache attention of the decoder layer (paper, Section 2.1: prefill processes the whole
// prompt, decode one token against the growing KV cache and is memory-bound).
//
//  * attn_generic: any head_dim <= 256, fp32 or bf16, prefill or decode; one wavefront per
//    (query row, head).  Used by the fp32 path and as the first bf16 prefill kernel.
//  * attn_decode:  bf16, head_dim 128.  One wavefront per (sequence, kv head, 256-key chunk)
//    streams K then V of its chunk with fully coalesced 1 KiB loads (16 lanes per key row,
//    4 keys per load) and serves all query heads of the GQA group from the same registers;
//    chunk results (max, sum, weighted values) are merged in chunk order by attn_combine.
//    The chunking depends only on the sequence's own length, so a sequence's output bits do
//    not depend on the batch it is in.
#include "ccs_common.h"
#include "ccs_kernels.h"

namespace ccs {

// =============================================================================================
template <typename T>
__global__ __launch_bounds__(256) void attn_generic_kernel(
    const T *__restrict__ qkv, T *__restrict__ out, int rows, int nq, int nkv, int d, int decode,
    int seq_pad, const int32_t *__restrict__ lens, const T *__restrict__ kc, const T *__restrict__ vc,
    int cap, int max_keys)
{
    extern __shared__ float smem[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float *sc = smem + (size_t)wave * max_keys;
    float *qs = smem + (size_t)4 * max_keys + wave * 256;
    const long unit = (long)blockIdx.x * 4 + wave;
    const int width = (nq + 2 * nkv) * d;
    bool active = unit < (long)rows * nq;
    int row = 0, h = 0, n_keys = 0;
    const T *kbase = nullptr, *vbase = nullptr;
    size_t kstride = 0;
    if (active) {
        row = (int)(unit / nq);
        h = (int)(unit % nq);
        const int kvh = h / (nq / nkv);
        if (decode) {
            n_keys = lens[row] + 1;
            kbase = kc + ((size_t)row * nkv + kvh) * cap * d;
            vbase = vc + ((size_t)row * nkv + kvh) * cap * d;
            kstride = d;
        } else {
            const int seq = row / seq_pad, pos = row % seq_pad;
            if (pos >= lens[seq]) active = false;
            n_keys = pos + 1;
            kbase = qkv + (size_t)seq * seq_pad * width + (size_t)(nq + kvh) * d;
            vbase = qkv + (size_t)seq * seq_pad * width + (size_t)(nq + nkv + kvh) * d;
            kstride = width;
        }
    }
    if (active) {
        const T *q = qkv + (size_t)row * width + (size_t)h * d;
        for (int c = lane; c < d; c += 64) qs[c] = io<T>::ld(q + c);
    }
    __syncthreads();
    float mx = -INFINITY;
    const float scale = 1.0f / sqrtf((float)d);
    if (active) {
        for (int j = lane; j < n_keys; j += 64) {
            const T *kr = kbase + (size_t)j * kstride;
            float a = 0.f;
            for (int c = 0; c < d; ++c) a = fmaf(qs[c], io<T>::ld(kr + c), a);
            a *= scale;
            sc[j] = a;
            mx = fmaxf(mx, a);
        }
        mx = wave_max(mx);
    }
    float den = 0.f;
    if (active) {
        for (int j = lane; j < n_keys; j += 64) {
            float p = expf(sc[j] - mx);
            sc[j] = p;
            den += p;
        }
        den = wave_sum(den);
    }
    __syncthreads();
    if (active) {
        const float inv = 1.0f / den;
        for (int c = lane; c < d; c += 64) {
            float a = 0.f;
            for (int j = 0; j < n_keys; ++j) a = fmaf(sc[j], io<T>::ld(vbase + (size_t)j * kstride + c), a);
            a *= inv;
            if constexpr (sizeof(T) == 4)
                io<T>::st(out + (size_t)row * nq * d + (size_t)h * d + c, a);
            else
                io<T>::st(out + packed_index(row, h * d + c, (nq * d) >> 5), a);
        }
    }
}

hipError_t launch_attn_generic(int dtype, const void *qkv, void *out, int rows, int nq, int nkv,
                               int d, int decode, int seq_pad, const int32_t *lens_dev,
                               const void *k_cache, const void *v_cache, int cap, hipStream_t st)
{
    if (rows <= 0) return hipSuccess;
    const int max_keys = decode ? cap : seq_pad;
    const size_t smem = ((size_t)4 * max_keys + 4 * 256) * sizeof(float);
    if (smem > 160 * 1024) return hipErrorInvalidValue;
    const long units = (long)rows * nq;
    dim3 grid((unsigned)((units + 3) / 4)), block(256);
    if (dtype == DT_BF16) {
        auto kern = attn_generic_kernel<bf16_t>;
        if (smem > 64 * 1024) {
            hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL(kern, grid, block, smem, st, (const bf16_t *)qkv, (bf16_t *)out, rows, nq, nkv, d,
                           decode, seq_pad, lens_dev, (const bf16_t *)k_cache, (const bf16_t *)v_cache, cap, max_keys);
    } else {
        auto kern = attn_generic_kernel<float>;
        if (smem > 64 * 1024) {
            hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL(kern, grid, block, smem, st, (const float *)qkv, (float *)out, rows, nq, nkv, d,
                           decode, seq_pad, lens_dev, (const float *)k_cache, (const float *)v_cache, cap, max_keys);
    }
    return hipGetLastError();
}

// =============================================================================================
// Decode attention, bf16, head_dim 128
// =============================================================================================
constexpr int kDecChunk = 256;   // keys per split; a property of the kernel, not of the batch
constexpr int kDecPart = 132;    // floats per partial: [0] max (log2 domain), [1] sum, [4..131] values

static inline int dec_chunks(int cap) { return (cap + kDecChunk - 1) / kDecChunk; }

size_t attn_decode_partial_bytes(int n_seqs, int nq, int cap)
{
    return (size_t)n_seqs * nq * dec_chunks(cap) * kDecPart * sizeof(float);
}

__device__ __forceinline__ float row16_sum(float v)
{
    v += __shfl_xor(v, 1, 64);
    v += __shfl_xor(v, 2, 64);
    v += __shfl_xor(v, 4, 64);
    v += __shfl_xor(v, 8, 64);
    return v;
}

template <int G, int IT>
__global__ __launch_bounds__(256) void attn_decode_kernel(
    const bf16_t *__restrict__ qkv, float *__restrict__ part, int n_seqs, int nq, int nkv,
    const int32_t *__restrict__ lens, const uint4 *__restrict__ kc, const uint4 *__restrict__ vc, int cap,
    int nchunks)
{
    const int lane = threadIdx.x & 63;
    const long unit = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (unit >= (long)n_seqs * nkv * nchunks) return;
    const int chunk = (int)(unit % nchunks);
    const int kvh = (int)((unit / nchunks) % nkv);
    const int b = (int)(unit / ((long)nchunks * nkv));
    const int n_keys = lens[b] + 1;
    const int j0 = chunk * kDecChunk;
    if (j0 >= n_keys) return;
    const int j1 = min(n_keys, j0 + kDecChunk);
    const int width = (nq + 2 * nkv) * 128;
    const int dpart = lane & 15, krow = lane >> 4;
    // softmax in the log2 domain: s' = (q.k) * log2(e)/sqrt(128)
    const float qscale = 1.4426950408889634f * 0.08838834764831845f;

    float q[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const uint4 v = *(const uint4 *)(qkv + (size_t)b * width + (size_t)(kvh * G + g) * 128 + dpart * 8);
        q[g][0] = bf_lo(v.x) * qscale; q[g][1] = bf_hi(v.x) * qscale;
        q[g][2] = bf_lo(v.y) * qscale; q[g][3] = bf_hi(v.y) * qscale;
        q[g][4] = bf_lo(v.z) * qscale; q[g][5] = bf_hi(v.z) * qscale;
        q[g][6] = bf_lo(v.w) * qscale; q[g][7] = bf_hi(v.w) * qscale;
    }
    const uint4 *kb = kc + ((size_t)b * nkv + kvh) * cap * 16 + lane;
    const uint4 *vb = vc + ((size_t)b * nkv + kvh) * cap * 16 + lane;

    float m[G], l[G], acc[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        m[g] = -INFINITY;
        l[g] = 0.f;
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[g][c] = 0.f;
    }

    for (int jb = j0; jb < j1; jb += 4 * IT) {
        uint4 kk[IT], vv[IT];
#pragma unroll
        for (int it = 0; it < IT; ++it) {
            const int j = jb + it * 4 + krow;
            kk[it] = (j < j1) ? ld_stream(kb + (size_t)(jb + it * 4) * 16) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int it = 0; it < IT; ++it) {
            const int j = jb + it * 4 + krow;
            vv[it] = (j < j1) ? ld_stream(vb + (size_t)(jb + it * 4) * 16) : make_uint4(0, 0, 0, 0);
        }
        float s[IT][G];
#pragma unroll
        for (int it = 0; it < IT; ++it) {
            const float k0 = bf_lo(kk[it].x), k1 = bf_hi(kk[it].x), k2 = bf_lo(kk[it].y), k3 = bf_hi(kk[it].y);
            const float k4 = bf_lo(kk[it].z), k5 = bf_hi(kk[it].z), k6 = bf_lo(kk[it].w), k7 = bf_hi(kk[it].w);
            const bool valid = (jb + it * 4 + krow) < j1;
#pragma unroll
            for (int g = 0; g < G; ++g) {
                float a = q[g][0] * k0;
                a = fmaf(q[g][1], k1, a); a = fmaf(q[g][2], k2, a); a = fmaf(q[g][3], k3, a);
                a = fmaf(q[g][4], k4, a); a = fmaf(q[g][5], k5, a); a = fmaf(q[g][6], k6, a);
                a = fmaf(q[g][7], k7, a);
                a = row16_sum(a);
                s[it][g] = valid ? a : -INFINITY;
            }
        }
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float mb = s[0][g];
#pragma unroll
            for (int it = 1; it < IT; ++it) mb = fmaxf(mb, s[it][g]);
            mb = fmaxf(mb, __shfl_xor(mb, 16, 64));
            mb = fmaxf(mb, __shfl_xor(mb, 32, 64));
            const float mn = fmaxf(m[g], mb);  // finite: this sub-block holds at least one valid key
            const float alpha = exp2f(m[g] - mn);
            m[g] = mn;
            l[g] *= alpha;
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[g][c] *= alpha;
#pragma unroll
            for (int it = 0; it < IT; ++it) s[it][g] = exp2f(s[it][g] - mn);
        }
#pragma unroll
        for (int it = 0; it < IT; ++it) {
            const float v0 = bf_lo(vv[it].x), v1 = bf_hi(vv[it].x), v2 = bf_lo(vv[it].y), v3 = bf_hi(vv[it].y);
            const float v4 = bf_lo(vv[it].z), v5 = bf_hi(vv[it].z), v6 = bf_lo(vv[it].w), v7 = bf_hi(vv[it].w);
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const float p = s[it][g];
                l[g] += p;
                acc[g][0] = fmaf(p, v0, acc[g][0]); acc[g][1] = fmaf(p, v1, acc[g][1]);
                acc[g][2] = fmaf(p, v2, acc[g][2]); acc[g][3] = fmaf(p, v3, acc[g][3]);
                acc[g][4] = fmaf(p, v4, acc[g][4]); acc[g][5] = fmaf(p, v5, acc[g][5]);
                acc[g][6] = fmaf(p, v6, acc[g][6]); acc[g][7] = fmaf(p, v7, acc[g][7]);
            }
        }
    }
    // merge the four key rows of the wavefront (fixed butterfly), then lanes 0..15 hold the chunk result
#pragma unroll
    for (int g = 0; g < G; ++g) {
        l[g] += __shfl_xor(l[g], 16, 64);
        l[g] += __shfl_xor(l[g], 32, 64);
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            acc[g][c] += __shfl_xor(acc[g][c], 16, 64);
            acc[g][c] += __shfl_xor(acc[g][c], 32, 64);
        }
        if (krow == 0) {
            float *p = part + (((size_t)b * nq + kvh * G + g) * nchunks + chunk) * kDecPart;
            if (dpart == 0) { p[0] = m[g]; p[1] = l[g]; }
            *(float4 *)(p + 4 + dpart * 8) = make_float4(acc[g][0], acc[g][1], acc[g][2], acc[g][3]);
            *(float4 *)(p + 8 + dpart * 8) = make_float4(acc[g][4], acc[g][5], acc[g][6], acc[g][7]);
        }
    }
}

// Merge the chunk partials of one (sequence, head) in chunk order; thread c owns value c.
__global__ __launch_bounds__(128) void attn_combine_kernel(const float *__restrict__ part,
                                                           bf16_t *__restrict__ out, int nq,
                                                           const int32_t *__restrict__ lens, int nchunks)
{
    const int b = blockIdx.x / nq, h = blockIdx.x % nq, c = threadIdx.x;
    const int n = (lens[b] + 1 + kDecChunk - 1) / kDecChunk;
    const float *p = part + ((size_t)b * nq + h) * nchunks * kDecPart;
    float M = -INFINITY;
    for (int i = 0; i < n; ++i) M = fmaxf(M, p[(size_t)i * kDecPart]);
    float L = 0.f, a = 0.f;
    for (int i = 0; i < n; ++i) {
        const float w = exp2f(p[(size_t)i * kDecPart] - M);
        L = fmaf(p[(size_t)i * kDecPart + 1], w, L);
        a = fmaf(p[(size_t)i * kDecPart + 4 + c], w, a);
    }
    out[packed_index(b, h * 128 + c, (nq * 128) >> 5)] = f2bf(a / L);
}

hipError_t launch_attn_decode_main(const void *qkv, float *partials, int n_seqs, int nq, int nkv,
                                   const int32_t *lens_dev, const void *k_cache,
                                   const void *v_cache, int cap, hipStream_t st)
{
    if (n_seqs <= 0) return hipSuccess;
    const int nchunks = dec_chunks(cap), G = nq / nkv;
    const long units = (long)n_seqs * nkv * nchunks;
    dim3 grid((unsigned)((units + 3) / 4)), block(256);
#define CCS_DEC(GV, ITV)                                                                                   \
    hipLaunchKernelGGL((attn_decode_kernel<GV, ITV>), grid, block, 0, st, (const bf16_t *)qkv, partials,   \
                       n_seqs, nq, nkv, lens_dev, (const uint4 *)k_cache, (const uint4 *)v_cache, cap, nchunks)
    switch (G) {
        case 1: CCS_DEC(1, 16); break;
        case 2: CCS_DEC(2, 8); break;
        case 4: CCS_DEC(4, 4); break;
        case 8: CCS_DEC(8, 4); break;
        default: return hipErrorInvalidValue;
    }
#undef CCS_DEC
    return hipGetLastError();
}

hipError_t launch_attn_decode_combine(const float *partials, void *out_packed, int n_seqs, int nq,
                                      const int32_t *lens_dev, int cap, hipStream_t st)
{
    if (n_seqs <= 0) return hipSuccess;
    const int nchunks = dec_chunks(cap);
    hipLaunchKernelGGL(attn_combine_kernel, dim3(n_seqs * nq), dim3(128), 0, st, partials, (bf16_t *)out_packed,
                       nq, lens_dev, nchunks);
    return hipGetLastError();
}

}  // namespace ccs
