// HBM-bound kernels of the decoder-layer path: replica clone (streaming copy), weight packing,
// RMSNorm, rotary embedding + KV-cache append, SwiGLU (f32 path).
#include "ccs_common.h"
#include "ccs_kernels.h"

namespace ccs {

// ---------------------------------------------------------------------------------------------
// Replica clone: the replica-instantiation step of module replication / migration (paper,
// Section 3.1 "Implementation": the module is duplicated with its weights).  Pure HBM traffic:
// `bytes` read + `bytes` written.  One 16-byte streaming load and one streaming store per lane,
// one wavefront per workgroup: on this device a flat grid of tiny workgroups beats every
// persistent / unrolled grid-stride form that was measured (83 % of the HBM peak against 55-73 %),
// and the runtime's own device-to-device copy (61 %).
// ---------------------------------------------------------------------------------------------
constexpr int kCloneThreads = 64;

__global__ __launch_bounds__(kCloneThreads) void clone_kernel(uint4 *__restrict__ dst,
                                                              const uint4 *__restrict__ src,
                                                              size_t n16)
{
    const size_t i = (size_t)blockIdx.x * kCloneThreads + threadIdx.x;
    if (i < n16) st_stream(dst + i, ld_stream(src + i));
}

__global__ void clone_tail_kernel(uint8_t *dst, const uint8_t *src, size_t from, size_t bytes)
{
    size_t i = from + threadIdx.x;
    if (i < bytes) dst[i] = src[i];
}

hipError_t launch_clone(void *dst, const void *src, size_t bytes, hipStream_t st)
{
    if (bytes == 0) return hipSuccess;
    size_t n16 = bytes / 16;
    if (n16) {
        const size_t blocks = (n16 + kCloneThreads - 1) / kCloneThreads;
        if (blocks > 0x7fffffffull) return hipErrorInvalidValue;  // > 2 TiB in one call
        hipLaunchKernelGGL(clone_kernel, dim3((unsigned)blocks), dim3(kCloneThreads), 0, st, (uint4 *)dst,
                           (const uint4 *)src, n16);
    }
    if (bytes % 16)
        hipLaunchKernelGGL(clone_tail_kernel, dim3(1), dim3(16), 0, st, (uint8_t *)dst,
                           (const uint8_t *)src, n16 * 16, bytes);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Packing: row-major [N, K] bf16 -> fragment-packed (activations) or grouped fragment-packed
// (weights, module_create).  One thread per 16-byte slot of the OUTPUT, a wavefront per 1 KiB
// fragment: the writes are whole contiguous fragments, the reads 64-byte pieces of 16 rows (the
// other way round - reads in row order, 16-byte writes 256 bytes apart - ran at a third of the rate).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void pack_bf16_kernel(const uint4 *__restrict__ src,
                                                        uint4 *__restrict__ dst, int N, int K,
                                                        int blk_stride, int blk_offset, int grouped,
                                                        const uint4 *__restrict__ gain)
{
    const int kchunks = K >> 3, kfrags = K >> 5;
    const int lane = threadIdx.x & 63;
    const size_t n_frags = (size_t)((N + 15) >> 4) * kfrags;
    for (size_t f = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6); f < n_frags; f += (size_t)gridDim.x * 4) {
        const int rb = (int)(f / kfrags), kb = (int)(f % kfrags);
        const int n = rb * 16 + (lane & 15), kc = kb * 4 + (lane >> 4);
        if (n >= N) continue;   // rows past the end of the last block stay as they are (never part of a result)
        uint4 v = src[(size_t)n * kchunks + kc];
        if (gain) {   // fold the gains of the RMSNorm in front of this projection into the weight
            const uint4 g = gain[kc];
            v.x = pack2bf(bf_lo(v.x) * bf_lo(g.x), bf_hi(v.x) * bf_hi(g.x));
            v.y = pack2bf(bf_lo(v.y) * bf_lo(g.y), bf_hi(v.y) * bf_hi(g.y));
            v.z = pack2bf(bf_lo(v.z) * bf_lo(g.z), bf_hi(v.z) * bf_hi(g.z));
            v.w = pack2bf(bf_lo(v.w) * bf_lo(g.w), bf_hi(v.w) * bf_hi(g.w));
        }
        const int nb = rb * blk_stride + blk_offset;
        const size_t frag = grouped ? weight_fragment(nb, kb, kfrags) : (size_t)nb * kfrags + kb;
        dst[frag * 64 + lane] = v;
    }
}

hipError_t launch_pack_bf16(const void *src, void *dst_packed, int N, int K, int blk_stride,
                            int blk_offset, bool grouped, const void *gain, hipStream_t st)
{
    const size_t frags = (size_t)((N + 15) / 16) * (K / 32);
    if (!frags) return hipSuccess;
    int blocks = (int)((frags + 3) / 4 < 16384 ? (frags + 3) / 4 : 16384);
    hipLaunchKernelGGL(pack_bf16_kernel, dim3(blocks), dim3(256), 0, st, (const uint4 *)src,
                       (uint4 *)dst_packed, N, K, blk_stride, blk_offset, grouped ? 1 : 0, (const uint4 *)gain);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// RMSNorm.  A row's arithmetic depends on H alone: not on how many rows the launch has, nor on
// where the row sits in it.
//
// Block form (bf16, rows up to 8192 wide): a workgroup of 8 waves owns one 16-row block of the
// packed output and wave w owns its 1 KiB fragments w, w + 8, ...  Lane (r, q) = (lane & 15,
// lane >> 4) reads the 16-byte chunk 4 f + q of row r, which is exactly slot `lane` of fragment
// f, so every store instruction writes one whole contiguous fragment (the row-per-wave form
// writes 16-byte pieces 256 bytes apart).  The row stays in registers between the two passes,
// all loads are in flight together, and the sum of squares is put together in a fixed order:
// a lane's fragments in sequence, the four k quarters by two butterfly steps, the eight waves
// in index order through LDS.
// ---------------------------------------------------------------------------------------------
constexpr int kNormWaves = 8;

template <int HOLD>   // fragments a wave keeps in registers: kfrags <= 8 * HOLD
__global__ __launch_bounds__(512) void rmsnorm_bf16_block_kernel(const uint4 *__restrict__ x,
                                                                 const uint4 *__restrict__ g,
                                                                 uint4 *__restrict__ out, int rows,
                                                                 int H, float eps)
{
    __shared__ float part[kNormWaves][16];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int r = lane & 15, q = lane >> 4;
    const int row = blockIdx.x * 16 + r;
    const bool live = row < rows;
    const int chunks = H >> 3, kfrags = H >> 5;
    const uint4 *xr = x + (size_t)(live ? row : 0) * chunks + q;
    uint4 v[HOLD];
#pragma unroll
    for (int i = 0; i < HOLD; ++i) {
        const int f = w + kNormWaves * i;
        v[i] = (live && f < kfrags) ? xr[4 * f] : make_uint4(0, 0, 0, 0);
    }
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < HOLD; ++i) {
        const uint32_t e[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float a = bf_lo(e[j]), b = bf_hi(e[j]);
            ss = fmaf(a, a, ss);
            ss = fmaf(b, b, ss);
        }
    }
    ss += __shfl_xor(ss, 16);
    ss += __shfl_xor(ss, 32);
    if (q == 0) part[w][r] = ss;
    __syncthreads();
    float tot = 0.f;
#pragma unroll
    for (int j = 0; j < kNormWaves; ++j) tot += part[j][r];
    const float rs = 1.0f / sqrtf(tot / (float)H + eps);
    uint4 *oblk = out + (size_t)blockIdx.x * kfrags * 64 + lane;
#pragma unroll
    for (int i = 0; i < HOLD; ++i) {
        const int f = w + kNormWaves * i;
        if (f < kfrags) {
            const uint4 gv = g ? g[4 * f + q] : make_uint4(0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u);   // bf16 1.0
            const uint32_t e[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
            const uint32_t ge[4] = {gv.x, gv.y, gv.z, gv.w};
            uint4 o;
            o.x = pack2bf(bf_lo(e[0]) * rs * bf_lo(ge[0]), bf_hi(e[0]) * rs * bf_hi(ge[0]));
            o.y = pack2bf(bf_lo(e[1]) * rs * bf_lo(ge[1]), bf_hi(e[1]) * rs * bf_hi(ge[1]));
            o.z = pack2bf(bf_lo(e[2]) * rs * bf_lo(ge[2]), bf_hi(e[2]) * rs * bf_hi(ge[2]));
            o.w = pack2bf(bf_lo(e[3]) * rs * bf_lo(ge[3]), bf_hi(e[3]) * rs * bf_hi(ge[3]));
            oblk[(size_t)f * 64] = o;
        }
    }
}

// Row-per-wave form for wider rows: two passes, the second re-reads the row from L1/L2.
__global__ __launch_bounds__(256) void rmsnorm_bf16_kernel(const uint4 *__restrict__ x,
                                                           const uint4 *__restrict__ g,
                                                           uint4 *__restrict__ out, int rows, int H,
                                                           float eps)
{
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const int chunks = H >> 3;
    const uint4 *xr = x + (size_t)row * chunks;
    const int kfrags = H >> 5;
    uint4 *orow = out + (size_t)(row >> 4) * kfrags * 64 + (row & 15);   // + (c >> 2) * 64 + 16 * (c & 3)
    float ss = 0.f;
    for (int c = lane; c < chunks; c += 64) {
        uint4 v = xr[c];
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float a = bf_lo(w[j]), b = bf_hi(w[j]);
            ss = fmaf(a, a, ss);
            ss = fmaf(b, b, ss);
        }
    }
    ss = wave_sum(ss);
    const float r = 1.0f / sqrtf(ss / (float)H + eps);
    for (int c = lane; c < chunks; c += 64) {
        uint4 v = xr[c], gv = g ? g[c] : make_uint4(0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
        const uint32_t gw[4] = {gv.x, gv.y, gv.z, gv.w};
        uint32_t o[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            o[j] = pack2bf(bf_lo(w[j]) * r * bf_lo(gw[j]), bf_hi(w[j]) * r * bf_hi(gw[j]));
        orow[(size_t)(c >> 2) * 64 + 16 * (c & 3)] = make_uint4(o[0], o[1], o[2], o[3]);
    }
}

__global__ __launch_bounds__(256) void rmsnorm_f32_kernel(const float *__restrict__ x,
                                                          const float *__restrict__ g,
                                                          float *__restrict__ out, int rows, int H,
                                                          float eps)
{
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const float *xr = x + (size_t)row * H;
    float ss = 0.f;
    for (int c = lane; c < H; c += 64) ss = fmaf(xr[c], xr[c], ss);
    ss = wave_sum(ss);
    const float r = 1.0f / sqrtf(ss / (float)H + eps);
    for (int c = lane; c < H; c += 64) out[(size_t)row * H + c] = xr[c] * r * g[c];
}

hipError_t launch_rmsnorm(int dtype, const void *x, const void *g, void *out, int rows, int H,
                          float eps, hipStream_t st)
{
    if (rows <= 0) return hipSuccess;
    dim3 grid((rows + 3) / 4), block(256);
    if (dtype == DT_BF16 && H <= 8192) {
        const dim3 g16((rows + 15) / 16), b512(512);
        const int per_wave = ((H >> 5) + kNormWaves - 1) / kNormWaves;
#define CCS_NORM_BLOCK(HOLD)                                                                              \
    hipLaunchKernelGGL(rmsnorm_bf16_block_kernel<HOLD>, g16, b512, 0, st, (const uint4 *)x, (const uint4 *)g, \
                       (uint4 *)out, rows, H, eps)
        if (per_wave <= 8) CCS_NORM_BLOCK(8);
        else if (per_wave <= 16) CCS_NORM_BLOCK(16);
        else if (per_wave <= 24) CCS_NORM_BLOCK(24);
        else CCS_NORM_BLOCK(32);
#undef CCS_NORM_BLOCK
    }
    else if (dtype == DT_BF16)
        hipLaunchKernelGGL(rmsnorm_bf16_kernel, grid, block, 0, st, (const uint4 *)x, (const uint4 *)g,
                           (uint4 *)out, rows, H, eps);
    else
        hipLaunchKernelGGL(rmsnorm_f32_kernel, grid, block, 0, st, (const float *)x, (const float *)g,
                           (float *)out, rows, H, eps);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Prefill without the padding (bf16): the valid rows of a right-padded batch [n_seqs, seq_pad, H]
// are moved into one dense [sum len, H] matrix, sequence after sequence, before the first layer,
// and moved back (padded rows written as zeros) after the last; every kernel in between works on
// valid rows only.  offs[b] = number of valid rows before sequence b, from the device copy of the
// lengths clamped into [0, seq_pad], and capped at `total`, the row count the host sized the dense
// buffers for from its own copy of the lengths.  Every later kernel takes a sequence's length as
// offs[b + 1] - offs[b], so no dense row index can reach `total` even if the two copies disagree.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void prefill_offsets_kernel(const int32_t *__restrict__ lens, int n_seqs,
                                                              int seq_pad, int total, int32_t *__restrict__ offs)
{
    __shared__ int part[256];
    const int per = (n_seqs + 255) / 256;
    const int lo = min(n_seqs, (int)threadIdx.x * per), hi = min(n_seqs, lo + per);
    int s = 0;
    for (int i = lo; i < hi; ++i) s += min(max(lens[i], 0), seq_pad);
    part[threadIdx.x] = s;
    __syncthreads();
    int before = 0;
    for (int t = 0; t < (int)threadIdx.x; ++t) before += part[t];
    for (int i = lo; i < hi; ++i) {
        offs[i] = min(before, total);
        before += min(max(lens[i], 0), seq_pad);
    }
    if (hi == n_seqs && lo < n_seqs) offs[n_seqs] = min(before, total);
}

// n_seqs x ceil(seq_pad / 4) workgroups, one wavefront per row.  expand = 0: dense[offs[b] + s] = padded[b, s]
// for s < len_b; expand = 1: padded[b, s] = dense[offs[b] + s] for s < len_b, zero otherwise.
__global__ __launch_bounds__(256) void prefill_rows_kernel(uint4 *__restrict__ padded, uint4 *__restrict__ dense,
                                                           const int32_t *__restrict__ offs, int seq_pad,
                                                           int chunks, int expand)
{
    const int per_seq = (seq_pad + 3) >> 2;
    const int b = blockIdx.x / per_seq, s = (blockIdx.x % per_seq) * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (s >= seq_pad) return;
    const int len = offs[b + 1] - offs[b];
    uint4 *prow = padded + ((size_t)b * seq_pad + s) * chunks;
    uint4 *drow = dense + (size_t)(offs[b] + min(s, max(len - 1, 0))) * chunks;
    if (!expand) {
        if (s < len)
            for (int c = lane; c < chunks; c += 64) drow[c] = ld_stream(prow + c);
    } else if (s < len) {
        for (int c = lane; c < chunks; c += 64) st_stream(prow + c, drow[c]);
    } else {
        for (int c = lane; c < chunks; c += 64) st_stream(prow + c, make_uint4(0, 0, 0, 0));
    }
}

hipError_t launch_prefill_offsets(const int32_t *lens_dev, int n_seqs, int seq_pad, int total, int32_t *offs,
                                  hipStream_t st)
{
    if (n_seqs <= 0) return hipSuccess;
    hipLaunchKernelGGL(prefill_offsets_kernel, dim3(1), dim3(256), 0, st, lens_dev, n_seqs, seq_pad, total, offs);
    return hipGetLastError();
}

hipError_t launch_prefill_rows(void *padded, void *dense, const int32_t *offs, int n_seqs, int seq_pad, int H,
                               bool expand, hipStream_t st)
{
    if (n_seqs <= 0) return hipSuccess;
    hipLaunchKernelGGL(prefill_rows_kernel, dim3((unsigned)n_seqs * ((seq_pad + 3) / 4)), dim3(256), 0, st, (uint4 *)padded,
                       (uint4 *)dense, offs, seq_pad, H / 8, expand ? 1 : 0);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Rotary embedding + KV-cache append.  One workgroup per row, thread i owns the pair
// (i, i + d/2) of every head; sine and cosine of pos * base^(-2i/d) come from the module's fp32
// head + tail table of inverse frequencies (rope_cs in ccs_common.h) and are applied in fp32.
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(64) void rope_kernel(T *__restrict__ qkv, int nq, int nkv, int d,
                                                  const float2 *__restrict__ tab, int decode, int seq_pad,
                                                  const int32_t *__restrict__ lens,
                                                  T *__restrict__ k_cache, T *__restrict__ v_cache,
                                                  int cap)
{
    const int row = blockIdx.x;
    const int half = d >> 1;
    const int width = (nq + 2 * nkv) * d;
    T *r = qkv + (size_t)row * width;
    int seq, pos, len;
    if (decode) { seq = row; pos = cap > 0 ? cached_len(lens, row, cap) : max(lens[row], 0); len = pos + 1; }
    else { seq = row / seq_pad; pos = row % seq_pad; len = lens[seq]; }
    const bool store = (k_cache != nullptr) && (pos < len) && (pos < cap);
    for (int i = threadIdx.x; i < half; i += 64) {
        float c, s;
        rope_cs(tab, i, pos, c, s);
        for (int h = 0; h < nq + nkv; ++h) {
            T *z = r + (size_t)h * d;
            float a = io<T>::ld(z + i), b = io<T>::ld(z + i + half);
            float ra = a * c - b * s, rb = b * c + a * s;
            io<T>::st(z + i, ra);
            io<T>::st(z + i + half, rb);
            if (store && h >= nq) {
                T *kc = k_cache + (((size_t)seq * nkv + (h - nq)) * cap + pos) * d;
                io<T>::st(kc + i, ra);
                io<T>::st(kc + i + half, rb);
            }
        }
        if (store) {
            for (int h = 0; h < nkv; ++h) {
                const T *v = r + (size_t)(nq + nkv + h) * d;
                T *vc = v_cache + (((size_t)seq * nkv + h) * cap + pos) * d;
                vc[i] = v[i];
                vc[i + half] = v[i + half];
            }
        }
    }
}

// Prefill, bf16, head_dim 128: rotate q in place and write the rotated keys and the values in
// the operand order of the MFMA attention kernel (ccs_attention.hip):
//   kp  per (sequence, kv head): matrix [S32 keys, 128] in the fragment-packed layout;
//   vtp per (sequence, kv head): V transposed, per 32-key block 8 fragments (one per 16 values
//       of d); lane = d % 16 + 16 * ((key % 16) / 4) holds 8 keys: slots 0..3 = keys
//       (key % 16) / 4 * 4 + 0..3 of the first 16 keys of the block, slots 4..7 the same of the
//       second 16 - the order in which the score accumulators of that kernel hold them.
// One workgroup = (sequence, block of 32 positions, group of 8 head slots); thread = (position,
// 8 consecutive d of the first half + their partners 64 up), so every global access is 16 bytes:
// q in place, K straight into packed chunks, V through a 32 x 128 LDS tile that is read back
// transposed.  The rows are dense (sequence b = rows offs[b] .. offs[b + 1] - 1 of qkv); only
// blocks that hold a valid position are written, and positions past the sequence's length inside
// the last block write zeros, so that masked products stay finite.  Optionally fills the
// row-major caches.
constexpr int kRopeHeadsPerGroup = 8;

__global__ __launch_bounds__(256) void rope_pack_prefill_kernel(
    bf16_t *__restrict__ qkv, bf16_t *__restrict__ kp, bf16_t *__restrict__ vtp, int nq, int nkv,
    const float2 *__restrict__ tab, int S32, int groups, const int32_t *__restrict__ offs,
    bf16_t *__restrict__ k_cache, bf16_t *__restrict__ v_cache, int cap)
{
    __shared__ bf16_t vt[32][128 + 2];
    const int blocks_per_seq = (S32 >> 5) * groups;
    const int seq = blockIdx.x / blocks_per_seq, rem = blockIdx.x % blocks_per_seq;
    const int kb = rem / groups, hg = rem % groups;
    const int tid = threadIdx.x, pl = tid >> 3, c = tid & 7;
    const int pos = kb * 32 + pl;
    const int len = offs[seq + 1] - offs[seq];
    if (kb * 32 >= len) return;   // the attention kernel reads key blocks up to the one holding key len - 1
    const bool valid = pos < len;
    const bool store = valid && (k_cache != nullptr) && (pos < cap);
    const int slots = nq + 2 * nkv, width = slots * 128;
    const int h_lo = hg * kRopeHeadsPerGroup, h_hi = min(slots, h_lo + kRopeHeadsPerGroup);
    const size_t head_elems = (size_t)S32 * 128;
    bf16_t *row = qkv + ((size_t)offs[seq] + (valid ? pos : 0)) * width;

    float cs[8], sn[8];
    if (h_lo < nq + nkv) {
#pragma unroll
        for (int e = 0; e < 8; ++e) rope_cs(tab, c * 8 + e, pos, cs[e], sn[e]);
    }
    for (int hs = h_lo; hs < h_hi; ++hs) {
        bf16_t *z = row + (size_t)hs * 128 + c * 8;
        uint4 lo = make_uint4(0, 0, 0, 0), hi = make_uint4(0, 0, 0, 0);
        if (valid) { lo = *(const uint4 *)z; hi = *(const uint4 *)(z + 64); }
        if (hs < nq + nkv) {
            const uint32_t lw[4] = {lo.x, lo.y, lo.z, lo.w}, hw[4] = {hi.x, hi.y, hi.z, hi.w};
            uint32_t ol[4], oh[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float a0 = bf_lo(lw[j]), b0 = bf_lo(hw[j]), a1 = bf_hi(lw[j]), b1 = bf_hi(hw[j]);
                ol[j] = pack2bf(a0 * cs[2 * j] - b0 * sn[2 * j], a1 * cs[2 * j + 1] - b1 * sn[2 * j + 1]);
                oh[j] = pack2bf(b0 * cs[2 * j] + a0 * sn[2 * j], b1 * cs[2 * j + 1] + a1 * sn[2 * j + 1]);
            }
            lo = make_uint4(ol[0], ol[1], ol[2], ol[3]);
            hi = make_uint4(oh[0], oh[1], oh[2], oh[3]);
            if (hs < nq) {
                if (valid) { *(uint4 *)z = lo; *(uint4 *)(z + 64) = hi; }
            } else {
                bf16_t *kh = kp + ((size_t)seq * nkv + (hs - nq)) * head_elems;
                *(uint4 *)(kh + packed_index(pos, c * 8, 4)) = lo;
                *(uint4 *)(kh + packed_index(pos, 64 + c * 8, 4)) = hi;
                if (store) {
                    bf16_t *kc = k_cache + (((size_t)seq * nkv + (hs - nq)) * cap + pos) * 128 + c * 8;
                    *(uint4 *)kc = lo;
                    *(uint4 *)(kc + 64) = hi;
                }
            }
        } else {
            const int vh = hs - nq - nkv;
            if (store) {
                bf16_t *vc = v_cache + (((size_t)seq * nkv + vh) * cap + pos) * 128 + c * 8;
                *(uint4 *)vc = lo;
                *(uint4 *)(vc + 64) = hi;
            }
            __syncthreads();  // previous head's tile fully read
            {
                uint32_t *d0 = (uint32_t *)&vt[pl][c * 8], *d1 = (uint32_t *)&vt[pl][64 + c * 8];
                d0[0] = lo.x; d0[1] = lo.y; d0[2] = lo.z; d0[3] = lo.w;
                d1[0] = hi.x; d1[1] = hi.y; d1[2] = hi.z; d1[3] = hi.w;
            }
            __syncthreads();
            uint4 *vth = (uint4 *)(vtp + ((size_t)seq * nkv + vh) * head_elems) + (size_t)kb * 8 * 64;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int q2 = tid + 256 * j, dt = q2 >> 6, ln = q2 & 63;
                const int dd = dt * 16 + (ln & 15), g = ln >> 4;
                uint32_t w[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int k0 = (e >> 1) * 16 + g * 4 + (e & 1) * 2;   // slots 2e, 2e+1
                    w[e] = (uint32_t)vt[k0][dd] | ((uint32_t)vt[k0 + 1][dd] << 16);
                }
                vth[dt * 64 + ln] = make_uint4(w[0], w[1], w[2], w[3]);
            }
        }
    }
}

hipError_t launch_rope_pack_prefill(void *qkv, void *kp, void *vtp, int n_seqs, int seq_pad, int nq, int nkv,
                                    const void *tab, const int32_t *offs, void *k_cache, void *v_cache, int cap,
                                    hipStream_t st)
{
    if (n_seqs <= 0) return hipSuccess;
    const int S32 = (seq_pad + 31) / 32 * 32;
    const int groups = (nq + 2 * nkv + kRopeHeadsPerGroup - 1) / kRopeHeadsPerGroup;
    hipLaunchKernelGGL(rope_pack_prefill_kernel, dim3(n_seqs * (S32 / 32) * groups), dim3(256), 0, st, (bf16_t *)qkv,
                       (bf16_t *)kp, (bf16_t *)vtp, nq, nkv, (const float2 *)tab, S32, groups, offs, (bf16_t *)k_cache,
                       (bf16_t *)v_cache, cap);
    return hipGetLastError();
}

hipError_t launch_rope(int dtype, void *qkv, int rows, int nq, int nkv, int d, const void *tab,
                       int decode, int seq_pad, const int32_t *lens_dev, void *k_cache,
                       void *v_cache, int cap, hipStream_t st)
{
    if (rows <= 0) return hipSuccess;
    if (dtype == DT_BF16)
        hipLaunchKernelGGL(rope_kernel<bf16_t>, dim3(rows), dim3(64), 0, st, (bf16_t *)qkv, nq, nkv, d,
                           (const float2 *)tab, decode, seq_pad, lens_dev, (bf16_t *)k_cache, (bf16_t *)v_cache, cap);
    else
        hipLaunchKernelGGL(rope_kernel<float>, dim3(rows), dim3(64), 0, st, (float *)qkv, nq, nkv, d,
                           (const float2 *)tab, decode, seq_pad, lens_dev, (float *)k_cache, (float *)v_cache, cap);
    return hipGetLastError();
}

// Inverse-frequency table of the rotary embedding: tab[i] = (head, tail) of base^(-2i/d) in fp32,
// evaluated in fp64 once per module (it lives in the weight arena and is cloned with it).
__global__ void rope_table_kernel(float2 *tab, int d, float base)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= d / 2) return;
    const double theta = pow((double)base, -2.0 * (double)i / (double)d);
    const float hi = (float)theta;
    tab[i] = make_float2(hi, (float)(theta - (double)hi));
}

hipError_t launch_rope_table(void *tab, int d, float base, hipStream_t st)
{
    hipLaunchKernelGGL(rope_table_kernel, dim3((d / 2 + 63) / 64), dim3(64), 0, st, (float2 *)tab, d, base);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Decode, bf16, head_dim 128: what follows a K-split Q/K/V projection of raw rows.  Sums the K
// segments' partials in segment order, scales by the row's RMSNorm factor (from the segments' sums of
// squares, also in segment order), rotates q and k to position lens[row], stores q (bf16) into the
// row-major qkv buffer and appends the rotated key and the value at cache slot lens[row].  One
// thread owns 4 columns of the first half of a head and their partners 64 up.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void qkv_partials_rope_decode_kernel(
    const float *__restrict__ part, const float *__restrict__ ssq, int S, int M, int nq, int nkv, int K, float eps,
    const float2 *__restrict__ tab, const int32_t *__restrict__ lens, bf16_t *__restrict__ qkv,
    bf16_t *__restrict__ k_cache, bf16_t *__restrict__ v_cache, int cap)
{
    const int heads = nq + 2 * nkv, width = heads * 128;
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= M * heads * 16) return;
    const int m = idx / (heads * 16), hu = idx % (heads * 16);
    const int head = hu >> 4, c = (hu & 15) * 4;
    const size_t seg = (size_t)M * width;
    const float *p = part + (size_t)m * width + head * 128 + c;
    float4 lo = *(const float4 *)p, hi = *(const float4 *)(p + 64);
    float tot = ssq[m];
    for (int k = 1; k < S; ++k) {
        const float4 a = *(const float4 *)(p + k * seg), b = *(const float4 *)(p + k * seg + 64);
        lo.x += a.x; lo.y += a.y; lo.z += a.z; lo.w += a.w;
        hi.x += b.x; hi.y += b.y; hi.z += b.z; hi.w += b.w;
        tot += ssq[k * M + m];
    }
    const float rs = 1.0f / sqrtf(tot / (float)K + eps);
    const int pos = cached_len(lens, m, cap);
    float l[4] = {lo.x * rs, lo.y * rs, lo.z * rs, lo.w * rs}, h[4] = {hi.x * rs, hi.y * rs, hi.z * rs, hi.w * rs};
    if (head < nq + nkv) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float cs, sn;
            rope_cs(tab, c + e, pos, cs, sn);
            const float a = l[e], b = h[e];
            l[e] = a * cs - b * sn;
            h[e] = b * cs + a * sn;
        }
    }
    const uint2 plo = make_uint2(pack2bf(l[0], l[1]), pack2bf(l[2], l[3]));
    const uint2 phi = make_uint2(pack2bf(h[0], h[1]), pack2bf(h[2], h[3]));
    bf16_t *dst;
    if (head < nq) dst = qkv + (size_t)m * width + head * 128 + c;
    else if (head < nq + nkv) dst = k_cache + (((size_t)m * nkv + (head - nq)) * cap + pos) * 128 + c;
    else dst = v_cache + (((size_t)m * nkv + (head - nq - nkv)) * cap + pos) * 128 + c;
    *(uint2 *)dst = plo;
    *(uint2 *)(dst + 64) = phi;
}

hipError_t launch_qkv_partials_rope_decode(const float *partials, const float *ssq_partials, int S, int M, int nq,
                                           int nkv, int K, float eps, const void *tab, const int32_t *lens_dev,
                                           void *qkv, void *k_cache, void *v_cache, int cap, hipStream_t st)
{
    if (M <= 0) return hipSuccess;
    const int total = M * (nq + 2 * nkv) * 16;
    hipLaunchKernelGGL(qkv_partials_rope_decode_kernel, dim3((total + 255) / 256), dim3(256), 0, st, partials, ssq_partials, S,
                       M, nq, nkv, K, eps, (const float2 *)tab, lens_dev, (bf16_t *)qkv, (bf16_t *)k_cache,
                       (bf16_t *)v_cache, cap);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void swiglu_f32_kernel(const float *__restrict__ gu,
                                                         float *__restrict__ u, size_t total, int I)
{
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    size_t t = i / I;
    int j = (int)(i % I);
    float g = gu[t * 2 * I + j], up = gu[t * 2 * I + I + j];
    u[i] = g / (1.0f + expf(-g)) * up;
}

hipError_t launch_swiglu_f32(const float *gu, float *u, int rows, int I, hipStream_t st)
{
    size_t total = (size_t)rows * I;
    if (!total) return hipSuccess;
    hipLaunchKernelGGL(swiglu_f32_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, gu, u,
                       total, I);
    return hipGetLastError();
}

}  // namespace ccs
