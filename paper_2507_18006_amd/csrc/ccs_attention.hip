// KV-cache attention of the decoder layer (paper, Section 2.1: prefill processes the whole
// prompt, decode one token against the growing KV cache and is memory-bound).
//
//  * attn_generic: any head_dim <= 256, fp32 or bf16, prefill or decode; one wavefront per
//    (query row, head), all-VALU.  The fp32 path.
//  * attn_prefill_mfma: bf16, head_dim 128, both products on the matrix cores, K / V^T blocks
//    of 32 keys through a direct-to-LDS ring.
//  * attn_decode_mfma: bf16, head_dim 128.  One wavefront per (sequence, kv head, 128-key
//    chunk) serves all query heads of the GQA group, so K and V are read once: scores on the
//    matrix cores with K rows straight from the cache, V through LDS and the transposing LDS
//    read; chunk results (max, sum, weighted values) are merged in chunk order by attn_combine.
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
            n_keys = cached_len(lens, row, cap) + 1;
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
        hipLaunchKernelGGL(kern, grid, block, smem, st, (const bf16_t *)qkv, (bf16_t *)out, rows, nq, nkv, d,
                           decode, seq_pad, lens_dev, (const bf16_t *)k_cache, (const bf16_t *)v_cache, cap, max_keys);
    } else {
        auto kern = attn_generic_kernel<float>;
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
    bf16_t *__restrict__ out, int nq, int nkv, int S32, int nqb, const int32_t *__restrict__ offs)
{
    extern __shared__ uint4 lds[];
    // Workgroups go to the 8 XCDs round-robin by index and every XCD has its own L2.  The (sequence,
    // kv head) groups are dealt to the XCDs in turn and all workgroups of a group - its query
    // blocks and the query heads that share the kv head - run on that XCD, so the group's keys and
    // values are fetched into one L2 (when the number of groups is no multiple of 8 the list is
    // walked in plain order).
    const int G = nq / nkv, per_group = G * nqb, groups = (int)gridDim.x / per_group;
    int grp, within;
    if ((groups & 7) == 0) {
        const int i = blockIdx.x >> 3;
        grp = (blockIdx.x & 7) + 8 * (i / per_group);
        within = i % per_group;
    } else {
        grp = blockIdx.x / per_group;
        within = blockIdx.x % per_group;
    }
    const int b = grp / nkv, h = (grp % nkv) * G + within / nqb, qb = nqb - 1 - within % nqb;  // long blocks first
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, c16 = lane & 15;
    const int q_start = qb * 128;
    const int ofrags = (nq * 128) >> 5;
    const size_t row0 = (size_t)offs[b];                                 // rows are dense: sequence b starts at offs[b]
    const int len = offs[b + 1] - offs[b];
    if (q_start >= len) return;                                          // no query of this sequence here
    const int q0w = q_start + wave * 32;                                // first query row of this wavefront
    const int last_q = min(q_start + 127, len - 1);
    const int nkb = (last_q >> 5) + 1;                                   // key blocks the workgroup walks
    const int my_blocks = (q0w < len) ? (q0w >> 5) + 1 : 0;              // key blocks this wavefront multiplies
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
        const int t = min(q0w + qt * 16 + c16, len - 1);
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
            const float alpha = fast_exp2(m_run[qt] - mn);
            m_run[qt] = mn;
            float ls = 0.f;
#pragma unroll
            for (int kt2 = 0; kt2 < 2; ++kt2)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    v[kt2][r] = fast_exp2(v[kt2][r] - mn);
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
        if (t >= len) continue;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
            const f32x4_t a = o[qt][dt];
            *(uint2 *)(out + packed_index((int)(row0 + t), h * 128 + dt * 16 + g * 4, ofrags)) =
                make_uint2(pack2bf(a[0] * inv, a[1] * inv), pack2bf(a[2] * inv, a[3] * inv));
        }
    }
}

hipError_t launch_attn_prefill_mfma(const void *qkv, const void *kp, const void *vtp, void *out_packed,
                                    int n_seqs, int seq_pad, int nq, int nkv, const int32_t *offs, hipStream_t st)
{
    if (n_seqs <= 0) return hipSuccess;
    const int S32 = (seq_pad + 31) / 32 * 32;
    const size_t smem = (size_t)kPfStages * kPfStageU4 * 16;
    const int nqb = (seq_pad + 127) / 128;   // 128-row query blocks per sequence
    dim3 grid((unsigned)nqb * nq * n_seqs);
    hipLaunchKernelGGL(attn_prefill_mfma_kernel, grid, dim3(256), smem, st, (const bf16_t *)qkv, (const uint4 *)kp,
                       (const uint4 *)vtp, (bf16_t *)out_packed, nq, nkv, S32, nqb, offs);
    return hipGetLastError();
}

// =============================================================================================
// Decode attention, bf16, head_dim 128
// =============================================================================================
// keys per split: a property of the kernel, never of the batch (128 measured best for the 7B
// multi-head and the ragged 70B grouped-query decode configurations; 256 within 2 %)
constexpr int kDecChunkMin = 128;
constexpr int kDecPart = 132;    // floats per partial: [0] max (log2 domain), [1] sum, [4..131] values
static inline int dec_chunk_keys(int, int) { return kDecChunkMin; }
static inline int dec_chunks(int cap, int chunk_keys) { return (cap + chunk_keys - 1) / chunk_keys; }

size_t attn_decode_partial_bytes(int n_seqs, int nq, int cap)
{
    return (size_t)n_seqs * nq * dec_chunks(cap, kDecChunkMin) * kDecPart * sizeof(float);
}

// ---------------------------------------------------------------------------------------------
// Decode attention with both products on the matrix cores (any group size G <= 8).
// One wavefront = one (sequence, kv head, chunk of chunk_keys keys); it serves the G query heads of
// the group at once, so K and V are read exactly once.  Scores are computed transposed, as in the
// prefill kernel: S^T[key][head] = K Q^T with 16 cached K rows x 32 d read straight from the
// row-major cache as the A operand and the group's query heads as the B columns (columns >= G
// are zero), so an accumulator lane owns ONE head and 4 keys per 16-key tile and the softmax
// statistics (log2 domain, running maximum and sum) stay per lane.  Each chunk writes a partial
// (max, sum, 128 unnormalised values) per head; attn_combine_kernel merges them in chunk order.
// The value product needs V^T as an operand - for a fixed d, 8 consecutive KEYS per lane - while
// the cache holds rows of d: the 32 x 128 block of V goes global -> LDS with direct-to-LDS loads
// (row-major, 16-byte pieces XOR-swizzled by the row so that the reads below touch every bank
// twice, the minimum) and comes back transposed with ds_read_b64_tr_b16: inside each group of 16
// lanes lane i supplies the address of 4 values (row i/4, columns 4(i%4)..) and lane j receives
// column j of those 4 rows.  With rows 4g..4g+3 (then 16+4g..) for lane group g this is exactly
// the A operand of O^T[d][head] += V^T P^T whose 8 contraction slots of group g are the keys
// 4g..4g+3, 16+4g..16+4g+3 - the keys whose scores the same lanes already hold, so P^T is built
// in registers, the rescale factor is a per-lane scalar and nothing but V crosses LDS.
// A wavefront owns one (sequence, kv head, chunk) and a private double buffer (2 x 8 KiB): the
// loads of block i + 1 (K to registers, V to LDS) are in flight while block i is multiplied.
// No load is outstanding when the loop ends (each block waits for its successor's loads).
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ void dm_issue_v(const uint4 *__restrict__ vrow, int jb, int j1, int lane, uint4 *stage)
{
    // instruction t fills LDS rows 4t..4t+3 of the stage: lane -> row 4t + lane/16, piece lane%16,
    // which holds global piece (lane%16) ^ (2 * (row % 8))
    const int r4 = lane >> 4, pc = lane & 15;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        const int R = 4 * t + r4;
        const int c = pc ^ (((4 * (t & 1)) + r4) << 1);
        const int row = min(jb + R, j1 - 1);   // rows past the end repeat the last key (weight 0)
        __builtin_amdgcn_global_load_lds(vrow + (size_t)row * 16 + c, stage + t * 64, 16, 0, 0);
    }
}

// K rows go to registers with hand-issued loads and hand-placed waits: left to the compiler, the
// wait for them lands behind the loads of the next block (it waits for everything outstanding).
// The compiler does not know that these registers are still being written after the asm statement:
// between a load and its dm_wait_all the register set must not be live across a control-flow join
// that could make the compiler copy it (a chunk loop around the block loop did: the copies read
// registers whose loads had not landed).  Keep the two register sets in ONE flat block loop.
__device__ __forceinline__ void dm_load_k(const uint4 *__restrict__ krow, int jb, int j1, int c16, int g4,
                                          u32x4_t (&kf)[2][4])
{
#pragma unroll
    for (int kt2 = 0; kt2 < 2; ++kt2) {
        const int key = min(jb + kt2 * 16 + c16, j1 - 1);   // rows past the end are masked by the caller
        const uint4 *p = krow + (size_t)key * 16 + g4;
        asm volatile("global_load_dwordx4 %0, %1, off nt" : "=v"(kf[kt2][0]) : "v"(p) : "memory");
        asm volatile("global_load_dwordx4 %0, %1, off offset:64 nt" : "=v"(kf[kt2][1]) : "v"(p) : "memory");
        asm volatile("global_load_dwordx4 %0, %1, off offset:128 nt" : "=v"(kf[kt2][2]) : "v"(p) : "memory");
        asm volatile("global_load_dwordx4 %0, %1, off offset:192 nt" : "=v"(kf[kt2][3]) : "v"(p) : "memory");
    }
}

// everything this wavefront has in flight (K registers named here, V in LDS) has landed
__device__ __forceinline__ void dm_wait_all(u32x4_t (&kf)[2][4])
{
    asm volatile("s_waitcnt vmcnt(0)"
                 : "+v"(kf[0][0]), "+v"(kf[0][1]), "+v"(kf[0][2]), "+v"(kf[0][3]), "+v"(kf[1][0]), "+v"(kf[1][1]),
                   "+v"(kf[1][2]), "+v"(kf[1][3])::"memory");
}

#define DM_TR(dst, addr, OFF) asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "i"(OFF) : "memory")

template <int STAGE>
__device__ __forceinline__ void dm_block(const u32x4_t (&kf)[2][4], const u32x4_t (&qf)[4], const uint32_t (&vaddr)[8],
                                         int jb, int j1, int g4, float sc, float &m_run, float &l_run,
                                         f32x4_t (&o)[8])
{
    u32x2_t va[8][2];
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) {
        DM_TR(va[dt][0], vaddr[dt], STAGE * 8192);
        DM_TR(va[dt][1], vaddr[dt], STAGE * 8192 + 4096);
    }
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
    const float alpha = fast_exp2(m_run - mn);
    m_run = mn;
    float ls = 0.f;
#pragma unroll
    for (int kt2 = 0; kt2 < 2; ++kt2)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            x[kt2][r] = fast_exp2(x[kt2][r] - mn);
            ls += x[kt2][r];
        }
    l_run = l_run * alpha + ls;
#pragma unroll
    for (int dt = 0; dt < 8; ++dt)
#pragma unroll
        for (int r = 0; r < 4; ++r) o[dt][r] *= alpha;
    const u32x4_t pfrag = u32x4_t{pack2bf(x[0][0], x[0][1]), pack2bf(x[0][2], x[0][3]), pack2bf(x[1][0], x[1][1]),
                                  pack2bf(x[1][2], x[1][3])};
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(va[0][0]), "+v"(va[0][1]), "+v"(va[1][0]), "+v"(va[1][1]), "+v"(va[2][0]), "+v"(va[2][1]),
                   "+v"(va[3][0]), "+v"(va[3][1]), "+v"(va[4][0]), "+v"(va[4][1]), "+v"(va[5][0]), "+v"(va[5][1]),
                   "+v"(va[6][0]), "+v"(va[6][1]), "+v"(va[7][0]), "+v"(va[7][1])::"memory");
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) {
        const u32x4_t a = u32x4_t{va[dt][0].x, va[dt][0].y, va[dt][1].x, va[dt][1].y};
        o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                        __builtin_bit_cast(bf16x8_t, pfrag), o[dt], 0, 0, 0);
    }
}

template <int G>
__global__ __launch_bounds__(256, 2) void attn_decode_mfma_kernel(
    const bf16_t *__restrict__ qkv, float *__restrict__ part, int n_seqs, int nq, int nkv,
    const int32_t *__restrict__ lens, const uint4 *__restrict__ kc, const uint4 *__restrict__ vc, int cap,
    int nchunks, int chunk_keys)
{
    extern __shared__ uint4 lds[];   // 4 wavefronts x 2 stages x 8 KiB
    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // Units are the NON-EMPTY (sequence, kv head, chunk) triples in that order (chunk fastest, so the
    // wavefronts of a workgroup read neighbouring pieces of one K / V stream): a sequence of n keys
    // has ceil(n / chunk_keys) chunks per kv head, found with a prefix sum over the batch's
    // lengths.  The grid is sized for full caches; wavefronts past the last unit leave at once.
    const long unit = (long)blockIdx.x * 4 + wv;
    int b = -1, chunk = 0, kvh = 0;
    long base = 0;
    for (int s0 = 0; s0 < n_seqs; s0 += 64) {
        const int i = s0 + lane;
        const int nch = i < n_seqs ? (cached_len(lens, i, cap) + chunk_keys) / chunk_keys : 0;
        int pre = nch;   // inclusive prefix sum over the 64 lanes
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int t = __shfl_up(pre, o, 64);
            if (lane >= o) pre += t;
        }
        const long tot = (long)__shfl(pre, 63, 64) * nkv;
        if (unit < base + tot) {
            const long lo = base + (long)(pre - nch) * nkv, hi = base + (long)pre * nkv;
            const unsigned long long hit = __ballot(unit >= lo && unit < hi);
            const int src = __ffsll((long long)hit) - 1;
            const int nch_b = __shfl(nch, src, 64);
            const int r = (int)(unit - base - (long)__shfl(pre - nch, src, 64) * nkv);
            b = s0 + src;
            kvh = r / nch_b;
            chunk = r % nch_b;
            break;
        }
        base += tot;
    }
    if (b < 0) return;
    b = __builtin_amdgcn_readfirstlane(b);
    chunk = __builtin_amdgcn_readfirstlane(chunk);
    kvh = __builtin_amdgcn_readfirstlane(kvh);
    const int n_keys = cached_len(lens, b, cap) + 1;
    const int j0 = chunk * chunk_keys;          // < n_keys by construction
    const int j1 = min(n_keys, j0 + chunk_keys);
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
    const uint4 *krow = kc + ((size_t)b * nkv + kvh) * cap * 16;   // 16 uint4 per cached row
    const uint4 *vrow = vc + ((size_t)b * nkv + kvh) * cap * 16;
    uint4 *stage0 = lds + wv * 1024, *stage1 = stage0 + 512;

    // transposing-read addresses inside a stage: rows 4*g4 + c16/4 (+16 by immediate), 8 bytes at
    // column 16*dt + 4*(c16%4) of the swizzled row
    uint32_t vaddr[8];
    {
        const int R = g4 * 4 + (c16 >> 2);
        const uint32_t base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint4 *)stage0 + R * 256 +
                              ((c16 >> 1) & 1) * 16 + (c16 & 1) * 8;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) vaddr[dt] = base + ((dt ^ (R & 7)) << 5);
    }

    float m_run = -INFINITY, l_run = 0.f;   // of head c16
    f32x4_t o[8];                            // O^T: head c16, d = dt*16 + g4*4 + r
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) o[dt] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    u32x4_t ka[2][4], kb2[2][4];
    dm_load_k(krow, j0, j1, c16, g4, ka);
    dm_issue_v(vrow, j0, j1, lane, stage0);
    dm_wait_all(ka);
    for (int jb = j0;; jb += 64) {
        const bool more1 = jb + 32 < j1;
        if (more1) {
            dm_load_k(krow, jb + 32, j1, c16, g4, kb2);
            dm_issue_v(vrow, jb + 32, j1, lane, stage1);
        }
        dm_block<0>(ka, qf, vaddr, jb, j1, g4, sc, m_run, l_run, o);
        if (!more1) break;
        dm_wait_all(kb2);
        const bool more2 = jb + 64 < j1;
        if (more2) {
            dm_load_k(krow, jb + 64, j1, c16, g4, ka);
            dm_issue_v(vrow, jb + 64, j1, lane, stage0);
        }
        dm_block<1>(kb2, qf, vaddr, jb + 32, j1, g4, sc, m_run, l_run, o);
        if (!more2) break;
        dm_wait_all(ka);
    }

    l_run += __shfl_xor(l_run, 16, 64);
    l_run += __shfl_xor(l_run, 32, 64);
    if (c16 < G) {
        float *p = part + (((size_t)b * nq + kvh * G + c16) * nchunks + chunk) * kDecPart;
        if (g4 == 0) {
            p[0] = m_run;
            p[1] = l_run;
        }
#pragma unroll
        for (int dt = 0; dt < 8; ++dt)
            *(float4 *)(p + 4 + dt * 16 + g4 * 4) = make_float4(o[dt][0], o[dt][1], o[dt][2], o[dt][3]);
    }
}

// ---------------------------------------------------------------------------------------------
// The same with ONE workgroup per (sequence, kv head) and no second kernel, for modules with many
// kv heads (multi-head attention: 16 kv heads or more, so that the (sequence, kv head) pairs alone
// fill the GPU and are all about equally long per sequence).  Wavefront w of the workgroup takes
// the 128-key chunks w, w + 4, w + 8, ... of the cache one after the other, carrying its running
// maximum, sum and values across them (the online softmax does not care where a chunk ends); the
// four wavefronts' results are then merged through LDS in wavefront order and the normalised
// output goes out fragment-packed.  No partial sums in memory, no combine launch; the chunking and
// the merge order depend only on the sequence's own length.
// ---------------------------------------------------------------------------------------------
template <int G>
__global__ __launch_bounds__(256, 2) void attn_decode_whole_kernel(
    const bf16_t *__restrict__ qkv, bf16_t *__restrict__ out, int n_seqs, int nq, int nkv,
    const int32_t *__restrict__ lens, const uint4 *__restrict__ kc, const uint4 *__restrict__ vc, int cap,
    int chunk_keys)
{
    extern __shared__ uint4 lds[];   // 4 wavefronts x 2 stages x 8 KiB; reused for the merge
    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int b = blockIdx.x / nkv, kvh = blockIdx.x % nkv;
    const int n_keys = cached_len(lens, b, cap) + 1;
    const int nch = (n_keys + chunk_keys - 1) / chunk_keys;
    const int width = (nq + 2 * nkv) * 128;
    const int c16 = lane & 15, g4 = lane >> 4;
    const float sc = 1.4426950408889634f * 0.08838834764831845f;  // log2(e) / sqrt(128)

    u32x4_t qf[4];
#pragma unroll
    for (int dblk = 0; dblk < 4; ++dblk) {
        uint4 v = make_uint4(0, 0, 0, 0);
        if (c16 < G) v = *(const uint4 *)(qkv + (size_t)b * width + (size_t)(kvh * G + c16) * 128 + dblk * 32 + g4 * 8);
        qf[dblk] = u32x4_t{v.x, v.y, v.z, v.w};
    }
    const uint4 *krow = kc + ((size_t)b * nkv + kvh) * cap * 16;   // 16 uint4 per cached row
    const uint4 *vrow = vc + ((size_t)b * nkv + kvh) * cap * 16;
    uint4 *stage0 = lds + wv * 1024, *stage1 = stage0 + 512;
    uint32_t vaddr[8];
    {
        const int R = g4 * 4 + (c16 >> 2);
        const uint32_t base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint4 *)stage0 + R * 256 +
                              ((c16 >> 1) & 1) * 16 + (c16 & 1) * 8;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) vaddr[dt] = base + ((dt ^ (R & 7)) << 5);
    }

    float m_run = -INFINITY, l_run = 0.f;   // of head c16
    f32x4_t o[8];                            // O^T: head c16, d = dt*16 + g4*4 + r
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) o[dt] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    // This wavefront's 32-key blocks, one stream: block i is block i % 4 of chunk wv + 4 (i / 4).  Only
    // the sequence's last chunk can be short, so masking against n_keys is all the blocks need.  (One
    // flat loop with the same shape as the per-chunk kernel's: the K registers and V stages that are
    // in flight across the back edge are the same ones in every iteration.)
    const int my_chunks = wv < nch ? (nch - wv + 3) / 4 : 0;
    const int last_blocks = (n_keys - (nch - 1) * chunk_keys + 31) / 32;
    const int my_blocks = my_chunks == 0 ? 0 : (((nch - 1) & 3) == wv ? (my_chunks - 1) * 4 + last_blocks : my_chunks * 4);
    auto key0 = [&](int i) { return (wv + 4 * (i >> 2)) * chunk_keys + (i & 3) * 32; };
    u32x4_t ka[2][4], kb2[2][4];
    if (my_blocks > 0) {
        dm_load_k(krow, key0(0), n_keys, c16, g4, ka);
        dm_issue_v(vrow, key0(0), n_keys, lane, stage0);
        dm_wait_all(ka);
        for (int i = 0;; i += 2) {
            const bool more1 = i + 1 < my_blocks;
            if (more1) {
                dm_load_k(krow, key0(i + 1), n_keys, c16, g4, kb2);
                dm_issue_v(vrow, key0(i + 1), n_keys, lane, stage1);
            }
            dm_block<0>(ka, qf, vaddr, key0(i), n_keys, g4, sc, m_run, l_run, o);
            if (!more1) break;
            dm_wait_all(kb2);
            const bool more2 = i + 2 < my_blocks;
            if (more2) {
                dm_load_k(krow, key0(i + 2), n_keys, c16, g4, ka);
                dm_issue_v(vrow, key0(i + 2), n_keys, lane, stage0);
            }
            dm_block<1>(kb2, qf, vaddr, key0(i + 1), n_keys, g4, sc, m_run, l_run, o);
            if (!more2) break;
            dm_wait_all(ka);
        }
    }
    l_run += __shfl_xor(l_run, 16, 64);
    l_run += __shfl_xor(l_run, 32, 64);

    // merge the four wavefronts in wavefront order: part[w][head] = (max, sum, 128 values), kDecPart floats each
    __syncthreads();   // every wavefront is done with its V stages
    float *part = (float *)lds;
    if (c16 < G) {
        float *p = part + (wv * G + c16) * kDecPart;
        if (g4 == 0) {
            p[0] = m_run;
            p[1] = l_run;
        }
#pragma unroll
        for (int dt = 0; dt < 8; ++dt)
            *(float4 *)(p + 4 + dt * 16 + g4 * 4) = make_float4(o[dt][0], o[dt][1], o[dt][2], o[dt][3]);
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < G * 128; idx += 256) {
        const int h = idx >> 7, c = idx & 127;
        const float *p = part + h * kDecPart;
        float M = p[0];                       // wavefront 0 always holds chunk 0, which has a key
#pragma unroll
        for (int w = 1; w < 4; ++w) M = fmaxf(M, p[w * G * kDecPart]);
        float L = 0.f, a = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float *q = p + w * G * kDecPart;
            const float wgt = fast_exp2(q[0] - M);   // a wavefront without a chunk has max -inf: weight 0
            L = fmaf(q[1], wgt, L);
            a = fmaf(q[4 + c], wgt, a);
        }
        out[packed_index(b, (kvh * G + h) * 128 + c, (nq * 128) >> 5)] = f2bf(a / L);
    }
}
#undef DM_TR

// Merge the chunk partials of one (sequence, head) in chunk order; thread c owns value c.  The
// (max, sum, value) loads of 16 chunks are all issued before anything is used, so a sequence of up to
// 16 chunks (2048 keys) costs one memory round trip; longer ones carry a running maximum from block
// to block of 16.
__global__ __launch_bounds__(128) void attn_combine_kernel(const float *__restrict__ part,
                                                           bf16_t *__restrict__ out, int nq,
                                                           const int32_t *__restrict__ lens, int nchunks,
                                                           int chunk_keys)
{
    const int b = blockIdx.x / nq, h = blockIdx.x % nq, c = threadIdx.x;
    const int n = min((max(lens[b], 0) + chunk_keys) / chunk_keys, nchunks);
    const float *p = part + ((size_t)b * nq + h) * nchunks * kDecPart;
    float M = -INFINITY, L = 0.f, a = 0.f;
    for (int i0 = 0; i0 < n; i0 += 16) {
        float m[16], l[16], v[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const bool ok = i0 + e < n;
            const float *q = p + (size_t)(ok ? i0 + e : 0) * kDecPart;
            m[e] = q[0];
            l[e] = q[1];
            v[e] = q[4 + c];
            if (!ok) m[e] = -INFINITY;   // weight 0
        }
        float Mb = m[0];
#pragma unroll
        for (int e = 1; e < 16; ++e) Mb = fmaxf(Mb, m[e]);
        const float Mn = fmaxf(M, Mb);                 // chunk 0 always has a key: Mn is finite
        const float keep = fast_exp2(M - Mn);          // 0 for the first block (M = -inf), 1 when the maximum stays
        L *= keep;
        a *= keep;
        M = Mn;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const float w = fast_exp2(m[e] - M);
            L = fmaf(l[e], w, L);
            a = fmaf(v[e], w, a);
        }
    }
    out[packed_index(b, h * 128 + c, (nq * 128) >> 5)] = f2bf(a / L);
}

// One workgroup per (sequence, kv head) with the merge inside (no partial sums, no combine launch)
// when the module has many kv heads; a property of the module's shape, never of the batch.
bool attn_decode_is_whole(int nq, int nkv) { return nkv >= 16 && nq / nkv <= 8; }

hipError_t launch_attn_decode_main(const void *qkv, float *partials, void *out_packed, int n_seqs, int nq, int nkv,
                                   const int32_t *lens_dev, const void *k_cache,
                                   const void *v_cache, int cap, hipStream_t st)
{
    if (n_seqs <= 0) return hipSuccess;
    const int chunk_keys = dec_chunk_keys(nq, nkv), nchunks = dec_chunks(cap, chunk_keys), G = nq / nkv;
    if (attn_decode_is_whole(nq, nkv)) {
        dim3 wgrid((unsigned)n_seqs * nkv);
#define CCS_WHOLE(GV)                                                                                      \
    hipLaunchKernelGGL((attn_decode_whole_kernel<GV>), wgrid, dim3(256), 65536, st, (const bf16_t *)qkv,   \
                       (bf16_t *)out_packed, n_seqs, nq, nkv, lens_dev, (const uint4 *)k_cache,            \
                       (const uint4 *)v_cache, cap, chunk_keys)
        switch (G) {
            case 1: CCS_WHOLE(1); break;
            case 2: CCS_WHOLE(2); break;
            case 4: CCS_WHOLE(4); break;
            case 8: CCS_WHOLE(8); break;
            default: return hipErrorInvalidValue;
        }
#undef CCS_WHOLE
        return hipGetLastError();
    }
    const long units = (long)n_seqs * nkv * nchunks;
    dim3 grid((unsigned)((units + 3) / 4)), block(256);
#define CCS_GQA(GV)                                                                                        \
    do {                                                                                                   \
        hipLaunchKernelGGL((attn_decode_mfma_kernel<GV>), grid, block, 65536, st, (const bf16_t *)qkv,     \
                           partials, n_seqs, nq, nkv, lens_dev, (const uint4 *)k_cache,                    \
                           (const uint4 *)v_cache, cap, nchunks, chunk_keys);                              \
    } while (0)
    switch (G) {
        case 1: CCS_GQA(1); break;
        case 2: CCS_GQA(2); break;
        case 4: CCS_GQA(4); break;
        case 8: CCS_GQA(8); break;
        default: return hipErrorInvalidValue;
    }
#undef CCS_GQA
    return hipGetLastError();
}

hipError_t launch_attn_decode_combine(const float *partials, void *out_packed, int n_seqs, int nq, int nkv,
                                      const int32_t *lens_dev, int cap, hipStream_t st)
{
    if (n_seqs <= 0) return hipSuccess;
    const int chunk_keys = dec_chunk_keys(nq, nkv), nchunks = dec_chunks(cap, chunk_keys);
    hipLaunchKernelGGL(attn_combine_kernel, dim3(n_seqs * nq), dim3(128), 0, st, partials, (bf16_t *)out_packed,
                       nq, lens_dev, nchunks, chunk_keys);
    return hipGetLastError();
}

// Function attributes (dynamic LDS sizes) of this file's kernels; once per process, outside any
// stream capture (ccs_module_create calls it).
hipError_t init_attention_kernels()
{
    const int attr = (int)hipFuncAttributeMaxDynamicSharedMemorySize;
    hipError_t e = hipFuncSetAttribute((const void *)attn_prefill_mfma_kernel, (hipFuncAttribute)attr, kPfStages * kPfStageU4 * 16);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void *)attn_decode_mfma_kernel<1>, (hipFuncAttribute)attr, 65536);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void *)attn_decode_mfma_kernel<2>, (hipFuncAttribute)attr, 65536);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void *)attn_decode_mfma_kernel<4>, (hipFuncAttribute)attr, 65536);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void *)attn_decode_mfma_kernel<8>, (hipFuncAttribute)attr, 65536);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void *)attn_decode_whole_kernel<1>, (hipFuncAttribute)attr, 65536);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void *)attn_decode_whole_kernel<2>, (hipFuncAttribute)attr, 65536);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void *)attn_decode_whole_kernel<4>, (hipFuncAttribute)attr, 65536);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void *)attn_decode_whole_kernel<8>, (hipFuncAttribute)attr, 65536);
    // the generic kernel keeps one score per key in LDS: allow it the whole 160 KiB here, so that no
    // forward (which a caller may be capturing into a graph) has to change a kernel attribute
    if (e == hipSuccess) e = hipFuncSetAttribute((const void *)attn_generic_kernel<float>, (hipFuncAttribute)attr, 160 * 1024);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void *)attn_generic_kernel<bf16_t>, (hipFuncAttribute)attr, 160 * 1024);
    return e;
}

}  // namespace ccs
