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
// Prefill attention, bf16, head_dim 128, on the matrix cores
// =============================================================================================
// One workgroup = one (sequence, query head, 128 query rows); 4 wavefronts of 32 query rows.
// Keys/values stream in blocks of 32 keys: 8 packed K fragments + 8 transposed V fragments
// (16 KiB) per block, fetched with direct-to-LDS loads into a 4-stage ring shared by the 4
// wavefronts (two workgroups fit a CU, so one wavefront's softmax overlaps another's MFMAs).
// All products use v_mfma_f32_16x16x32_bf16:
//   scores transposed, S^T[key][q] = K Q^T: A = K fragment (16 keys x 32 d), B = Q^T fragment;
//   an accumulator lane then owns ONE query (lane % 16) and 4 keys per 16-key tile, so the
//   softmax statistics of a row live in one lane (plus a 4-lane butterfly) and the rescale
//   factor of the output accumulators is a per-lane scalar;
//   output transposed, O^T[d][q] += V^T P^T: A = V^T fragment (16 d x 32 keys), B = P^T built in
//   registers from the two score tiles (slots 0..3 first tile, 4..7 second tile - the order V^T
//   was packed in), so probabilities never go through LDS.
// A wavefront's last block is its diagonal block (keys q0..q0+31), the only one that needs the
// causal mask; softmax runs in the log2 domain with running maximum and sum (online softmax).
constexpr int kPfStages = 4;
constexpr int kPfStageU4 = 1024;  // uint4 per stage (16 KiB)

__device__ __forceinline__ void pf_dma_one(const uint4 *src, uint4 *lds_dst)
{
    __builtin_amdgcn_global_load_lds(src, lds_dst, 16, 0, 0);
}

__device__ __forceinline__ f32x4_t pf_mfma(const u32x4_t &a, const u32x4_t &b, f32x4_t c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c,
                                                   0, 0, 0);
}

__global__ __launch_bounds__(256, 2) void attn_prefill_mfma_kernel(
    const bf16_t *__restrict__ qkv, const uint4 *__restrict__ Kp, const uint4 *__restrict__ VTp,
    bf16_t *__restrict__ out, int nq, int nkv, int seq_pad, int S32, const int32_t *__restrict__ lens)
{
    extern __shared__ uint4 lds[];
    const int b = blockIdx.z, h = blockIdx.y, qb = gridDim.x - 1 - blockIdx.x;  // long blocks first
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, c16 = lane & 15;
    const int q_start = qb * 128;
    const int ofrags = (nq * 128) >> 5;
    const size_t row0 = (size_t)b * seq_pad;
    if (q_start >= lens[b]) {
        // nothing but padding in this block: defined (zero) output, no work
        for (int idx = tid; idx < 128 * 32; idx += 256) {
            const int t = q_start + (idx >> 5);
            if (t < seq_pad) *(uint2 *)(out + packed_index((int)(row0 + t), h * 128 + (idx & 31) * 4, ofrags)) = make_uint2(0, 0);
        }
        return;
    }
    const int q0w = q_start + wave * 32;                                // first query row of this wavefront
    const int last_q = min(q_start + 127, seq_pad - 1);
    const int nkb = (last_q >> 5) + 1;                                   // key blocks the workgroup walks
    const int my_blocks = (q0w < seq_pad) ? (q0w >> 5) + 1 : 0;          // key blocks this wavefront multiplies
    const int kvh = h / (nq / nkv);
    const uint4 *kbase = Kp + ((size_t)b * nkv + kvh) * S32 * 16 + lane;   // 16 uint4 per key
    const uint4 *vbase = VTp + ((size_t)b * nkv + kvh) * S32 * 16 + lane;
    const int width = (nq + 2 * nkv) * 128;

    // this wavefront's 4 fragments of a key block: 0,1 -> K fragments 4*(wave&1).., 2,3 -> V fragments
    const uint4 *dsrc = (wave < 2 ? kbase : vbase) + (wave & 1) * 4 * 64;
    uint4 *ddst = lds + wave * 4 * 64;
#define PF_DMA(kb, stage)                                                                        \
    do {                                                                                         \
        const uint4 *s__ = dsrc + (size_t)(kb) * 512;                                            \
        uint4 *d__ = ddst + (stage) * kPfStageU4;                                                \
        pf_dma_one(s__, d__); pf_dma_one(s__ + 64, d__ + 64);                                    \
        pf_dma_one(s__ + 128, d__ + 128); pf_dma_one(s__ + 192, d__ + 192);                      \
    } while (0)

    // Q^T fragments (B operand): lane -> query c16 of tile qt, d = dblk*32 + g*8 .. +8
    u32x4_t qf[2][4];
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
        const int t = min(q0w + qt * 16 + c16, seq_pad - 1);
        const bf16_t *qrow = qkv + (row0 + t) * width + (size_t)h * 128 + g * 8;
#pragma unroll
        for (int dblk = 0; dblk < 4; ++dblk) {
            const uint4 v = *(const uint4 *)(qrow + dblk * 32);
            qf[qt][dblk] = u32x4_t{v.x, v.y, v.z, v.w};
        }
    }

    f32x4_t o[2][8];
    float m_run[2], l_run[2];
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
        m_run[qt] = -INFINITY;
        l_run[qt] = 0.f;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) o[qt][dt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    }

    const uint32_t lds_lane = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint4 *)lds + lane * 16;
    const float sc = 1.4426950408889634f * 0.08838834764831845f;  // log2(e) / sqrt(128)

#pragma unroll
    for (int s = 0; s < kPfStages - 1; ++s) PF_DMA(min(s, nkb - 1), s);

#define PF_READ(dst, base, OFF) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(base), "i"(OFF) : "memory")
    for (int kb = 0; kb < nkb; ++kb) {
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((kPfStages - 2) * 4) : "memory");
        __syncthreads();   // block kb is in LDS for everybody; everybody is done with block kb - 1
        PF_DMA(min(kb + kPfStages - 1, nkb - 1), (kb + kPfStages - 1) % kPfStages);
        if (kb >= my_blocks) continue;
        const uint32_t sb = lds_lane + (uint32_t)(kb % kPfStages) * (kPfStageU4 * 16);

        u32x4_t kf[8], vf[8];
        PF_READ(kf[0], sb, 0); PF_READ(kf[1], sb, 1024); PF_READ(kf[2], sb, 2048); PF_READ(kf[3], sb, 3072);
        PF_READ(kf[4], sb, 4096); PF_READ(kf[5], sb, 5120); PF_READ(kf[6], sb, 6144); PF_READ(kf[7], sb, 7168);
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : "+v"(kf[0]), "+v"(kf[1]), "+v"(kf[2]), "+v"(kf[3]), "+v"(kf[4]), "+v"(kf[5]), "+v"(kf[6]), "+v"(kf[7])::"memory");
        PF_READ(vf[0], sb, 8192); PF_READ(vf[1], sb, 9216); PF_READ(vf[2], sb, 10240); PF_READ(vf[3], sb, 11264);
        PF_READ(vf[4], sb, 12288); PF_READ(vf[5], sb, 13312); PF_READ(vf[6], sb, 14336); PF_READ(vf[7], sb, 15360);

        // S^T[key tile kt2][query tile qt] over d = 4 x 32
        f32x4_t st[2][2];
#pragma unroll
        for (int kt2 = 0; kt2 < 2; ++kt2)
#pragma unroll
            for (int qt = 0; qt < 2; ++qt) {
                f32x4_t a = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int dblk = 0; dblk < 4; ++dblk) a = pf_mfma(kf[kt2 * 4 + dblk], qf[qt][dblk], a);
                st[kt2][qt] = a;
            }

        const bool diag = (kb == my_blocks - 1);
        u32x4_t pfrag[2];
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) {
            float v[2][4];
            const int qrow = q0w + qt * 16 + c16;
            float mx = -INFINITY;
#pragma unroll
            for (int kt2 = 0; kt2 < 2; ++kt2)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    float x = st[kt2][qt][r] * sc;
                    if (diag && (kb * 32 + kt2 * 16 + g * 4 + r) > qrow) x = -INFINITY;
                    v[kt2][r] = x;
                    mx = fmaxf(mx, x);
                }
            mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float mn = fmaxf(m_run[qt], mx);   // finite: key q0w of the diagonal block is visible to every row
            const float alpha = exp2f(m_run[qt] - mn);
            m_run[qt] = mn;
            float ls = 0.f;
#pragma unroll
            for (int kt2 = 0; kt2 < 2; ++kt2)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    v[kt2][r] = exp2f(v[kt2][r] - mn);
                    ls += v[kt2][r];
                }
            l_run[qt] = l_run[qt] * alpha + ls;
#pragma unroll
            for (int dt = 0; dt < 8; ++dt)
#pragma unroll
                for (int r = 0; r < 4; ++r) o[qt][dt][r] *= alpha;
            pfrag[qt] = u32x4_t{pack2bf(v[0][0], v[0][1]), pack2bf(v[0][2], v[0][3]), pack2bf(v[1][0], v[1][1]),
                                pack2bf(v[1][2], v[1][3])};
        }
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : "+v"(vf[0]), "+v"(vf[1]), "+v"(vf[2]), "+v"(vf[3]), "+v"(vf[4]), "+v"(vf[5]), "+v"(vf[6]), "+v"(vf[7])::"memory");
#pragma unroll
        for (int dt = 0; dt < 8; ++dt)
#pragma unroll
            for (int qt = 0; qt < 2; ++qt) o[qt][dt] = pf_mfma(vf[dt], pfrag[qt], o[qt][dt]);
    }
#undef PF_READ
#undef PF_DMA
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // no load may land in LDS after the workgroup is gone

    // O^T accumulators: lane -> query c16 of tile qt, d = dt*16 + g*4 + r
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
        float l = l_run[qt];
        l += __shfl_xor(l, 16, 64);
        l += __shfl_xor(l, 32, 64);
        const float inv = 1.0f / l;
        const int t = q0w + qt * 16 + c16;
        if (t >= seq_pad) continue;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
            const f32x4_t a = o[qt][dt];
            *(uint2 *)(out + packed_index((int)(row0 + t), h * 128 + dt * 16 + g * 4, ofrags)) =
                make_uint2(pack2bf(a[0] * inv, a[1] * inv), pack2bf(a[2] * inv, a[3] * inv));
        }
    }
}

hipError_t launch_attn_prefill_mfma(const void *qkv, const void *kp, const void *vtp, void *out_packed,
                                    int n_seqs, int seq_pad, int nq, int nkv, const int32_t *lens_dev,
                                    hipStream_t st)
{
    if (n_seqs <= 0) return hipSuccess;
    const int S32 = (seq_pad + 31) / 32 * 32;
    const size_t smem = (size_t)kPfStages * kPfStageU4 * 16;
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute((const void *)attn_prefill_mfma_kernel,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    dim3 grid((seq_pad + 127) / 128, nq, n_seqs);
    hipLaunchKernelGGL(attn_prefill_mfma_kernel, grid, dim3(256), smem, st, (const bf16_t *)qkv, (const uint4 *)kp,
                       (const uint4 *)vtp, (bf16_t *)out_packed, nq, nkv, seq_pad, S32, lens_dev);
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

// Grouped-query variant (G = 2, 4, 8 query heads per kv head).  With G heads the all-VALU kernel
// above spends G x (8 FMA + a 16-lane reduction) per key on the scores alone and falls far below
// the HBM rate; here the scores go to the matrix cores in the transposed form of the prefill
// kernel - S^T[key][head] = K Q^T with the cached K rows as the A operand (16 keys x 32 d read
// straight from the row-major cache) and the group's query heads as the B columns - so a lane
// owns one head and 4 keys per 16-key tile and the softmax statistics stay per lane.  The
// probabilities and rescale factors cross to the value layout (16 lanes per key row, fully
// coalesced V loads as above) through a 1 KiB wavefront-private LDS tile; P V stays on the VALU,
// where it is G x 8 FMAs per 16 bytes of V.  Same chunking and partial format as above.
template <int G>
__global__ __launch_bounds__(256) void attn_decode_gqa_kernel(
    const bf16_t *__restrict__ qkv, float *__restrict__ part, int n_seqs, int nq, int nkv,
    const int32_t *__restrict__ lens, const uint4 *__restrict__ kc, const uint4 *__restrict__ vc, int cap,
    int nchunks)
{
    __shared__ float pt[4][32][8];   // per wavefront: probabilities [key in block][head]
    __shared__ float al[4][8];       // per wavefront: rescale factor per head
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const long unit = (long)blockIdx.x * 4 + wv;
    if (unit >= (long)n_seqs * nkv * nchunks) return;
    const int chunk = (int)(unit % nchunks);
    const int kvh = (int)((unit / nchunks) % nkv);
    const int b = (int)(unit / ((long)nchunks * nkv));
    const int n_keys = lens[b] + 1;
    const int j0 = chunk * kDecChunk;
    if (j0 >= n_keys) return;
    const int j1 = min(n_keys, j0 + kDecChunk);
    const int width = (nq + 2 * nkv) * 128;
    const int c16 = lane & 15, g4 = lane >> 4;
    const float sc = 1.4426950408889634f * 0.08838834764831845f;  // log2(e) / sqrt(128)

    // Q^T fragments: lane -> head column c16 (zero beyond the group), d = dblk*32 + g4*8 .. +8
    u32x4_t qf[4];
#pragma unroll
    for (int dblk = 0; dblk < 4; ++dblk) {
        uint4 v = make_uint4(0, 0, 0, 0);
        if (c16 < G) v = *(const uint4 *)(qkv + (size_t)b * width + (size_t)(kvh * G + c16) * 128 + dblk * 32 + g4 * 8);
        qf[dblk] = u32x4_t{v.x, v.y, v.z, v.w};
    }
    const uint4 *kb = kc + ((size_t)b * nkv + kvh) * cap * 16;   // 16 uint4 per cached row
    const uint4 *vb = vc + ((size_t)b * nkv + kvh) * cap * 16 + lane;

    float m_run = -INFINITY, l_run = 0.f;   // of head c16 (score layout)
    float acc[G][8];                         // value layout: d = c16*8 .. +8, key row g4
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[g][c] = 0.f;

    for (int jb = j0; jb < j1; jb += 32) {
        uint4 kf[2][4], vv[8];
#pragma unroll
        for (int kt2 = 0; kt2 < 2; ++kt2) {
            const int key = min(jb + kt2 * 16 + c16, j1 - 1);   // rows past the end are masked below
#pragma unroll
            for (int dblk = 0; dblk < 4; ++dblk) kf[kt2][dblk] = ld_stream(kb + (size_t)key * 16 + dblk * 4 + g4);
        }
#pragma unroll
        for (int it = 0; it < 8; ++it)
            vv[it] = (jb + it * 4 + g4 < j1) ? ld_stream(vb + (size_t)(jb + it * 4) * 16) : make_uint4(0, 0, 0, 0);

        float x[2][4];
        float mx = -INFINITY;
#pragma unroll
        for (int kt2 = 0; kt2 < 2; ++kt2) {
            f32x4_t st = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int dblk = 0; dblk < 4; ++dblk)
                st = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kf[kt2][dblk]),
                                                             __builtin_bit_cast(bf16x8_t, qf[dblk]), st, 0, 0, 0);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float v = (jb + kt2 * 16 + g4 * 4 + r < j1) ? st[r] * sc : -INFINITY;
                x[kt2][r] = v;
                mx = fmaxf(mx, v);
            }
        }
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float mn = fmaxf(m_run, mx);   // finite: key jb of this block is valid
        const float alpha = exp2f(m_run - mn);
        m_run = mn;
        float ls = 0.f;
#pragma unroll
        for (int kt2 = 0; kt2 < 2; ++kt2)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float pv = exp2f(x[kt2][r] - mn);
                ls += pv;
                if (c16 < 8) pt[wv][kt2 * 16 + g4 * 4 + r][c16] = pv;
            }
        l_run = l_run * alpha + ls;
        if (g4 == 0 && c16 < 8) al[wv][c16] = alpha;
        __builtin_amdgcn_wave_barrier();   // same wavefront: LDS operations execute in program order

        float a_g[G];
#pragma unroll
        for (int g = 0; g < G; ++g) a_g[g] = al[wv][g];
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[g][c] *= a_g[g];
#pragma unroll
        for (int it = 0; it < 8; ++it) {
            const float v0 = bf_lo(vv[it].x), v1 = bf_hi(vv[it].x), v2 = bf_lo(vv[it].y), v3 = bf_hi(vv[it].y);
            const float v4 = bf_lo(vv[it].z), v5 = bf_hi(vv[it].z), v6 = bf_lo(vv[it].w), v7 = bf_hi(vv[it].w);
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const float pv = pt[wv][it * 4 + g4][g];
                acc[g][0] = fmaf(pv, v0, acc[g][0]); acc[g][1] = fmaf(pv, v1, acc[g][1]);
                acc[g][2] = fmaf(pv, v2, acc[g][2]); acc[g][3] = fmaf(pv, v3, acc[g][3]);
                acc[g][4] = fmaf(pv, v4, acc[g][4]); acc[g][5] = fmaf(pv, v5, acc[g][5]);
                acc[g][6] = fmaf(pv, v6, acc[g][6]); acc[g][7] = fmaf(pv, v7, acc[g][7]);
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
    // the four key groups of a head hold partial sums of its probabilities; the four key rows of
    // the value layout hold partial value sums: merge both with the fixed butterfly
    l_run += __shfl_xor(l_run, 16, 64);
    l_run += __shfl_xor(l_run, 32, 64);
    if (g4 == 0 && c16 < G) {
        float *p = part + (((size_t)b * nq + kvh * G + c16) * nchunks + chunk) * kDecPart;
        p[0] = m_run;
        p[1] = l_run;
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            acc[g][c] += __shfl_xor(acc[g][c], 16, 64);
            acc[g][c] += __shfl_xor(acc[g][c], 32, 64);
        }
        if (g4 == 0) {
            float *p = part + (((size_t)b * nq + kvh * G + g) * nchunks + chunk) * kDecPart;
            *(float4 *)(p + 4 + c16 * 8) = make_float4(acc[g][0], acc[g][1], acc[g][2], acc[g][3]);
            *(float4 *)(p + 8 + c16 * 8) = make_float4(acc[g][4], acc[g][5], acc[g][6], acc[g][7]);
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
#define CCS_GQA(GV)                                                                                        \
    hipLaunchKernelGGL((attn_decode_gqa_kernel<GV>), grid, block, 0, st, (const bf16_t *)qkv, partials, n_seqs, \
                       nq, nkv, lens_dev, (const uint4 *)k_cache, (const uint4 *)v_cache, cap, nchunks)
    switch (G) {
        case 1: CCS_DEC(1, 16); break;
        case 2: CCS_GQA(2); break;
        case 4: CCS_GQA(4); break;
        case 8: CCS_GQA(8); break;
        default: return hipErrorInvalidValue;
    }
#undef CCS_DEC
#undef CCS_GQA
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
