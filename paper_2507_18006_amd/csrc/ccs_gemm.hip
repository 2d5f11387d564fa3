// Projection GEMMs of the decoder layer (paper, Section 2.1: Q/K/V/O and the three FFN
// projections are linear maps; Table 1 puts ~99 % of a layer's FLOPs in them).
//
// y[m, n] = sum_k x[m, k] * W[n, k].  On the bf16 path both operands are fragment-packed
// (ccs_common.h) and every variant uses v_mfma_f32_16x16x32_bf16 with the weight fragment as
// the A operand and the activation fragment as the B operand, so one accumulator register
// quartet holds 4 consecutive n for one row m.
//
//  * gemm_tiled:  LDS-tiled, double-buffered, for compute-bound row counts (prefill).
//  * gemm_skinny: weight-streaming for <= 64 rows (decode): no LDS staging of operands, each
//    wavefront streams 1 KiB weight fragments straight into MFMA operands; K is cut into
//    segments whose count depends on the weight shape only and partial sums are reduced in a
//    fixed order, so a row's bits never depend on which other rows share the launch.
//  * gemm_f32: plain FMA kernel for the fp32 path.
#include "ccs_common.h"
#include "ccs_kernels.h"

namespace ccs {

__device__ __forceinline__ f32x4_t mfma16(const uint4 &a, const uint4 &b, f32x4_t c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                   __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

// =============================================================================================
// fp32 GEMM: 16x16 outputs per workgroup, K walked in order 0..K-1 for every output.
// =============================================================================================
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float *__restrict__ x,
                                                       const float *__restrict__ W,
                                                       const float *__restrict__ res,
                                                       float *__restrict__ y, int M, int N, int K)
{
    __shared__ float xs[16][17];
    __shared__ float ws[16][17];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int m = blockIdx.y * 16 + ty, n = blockIdx.x * 16 + tx;
    const int wn = blockIdx.x * 16 + ty;
    float acc = 0.f;
    for (int k0 = 0; k0 < K; k0 += 16) {
        xs[ty][tx] = (m < M && k0 + tx < K) ? x[(size_t)m * K + k0 + tx] : 0.f;
        ws[ty][tx] = (wn < N && k0 + tx < K) ? W[(size_t)wn * K + k0 + tx] : 0.f;
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) acc = fmaf(xs[ty][kk], ws[tx][kk], acc);
        __syncthreads();
    }
    if (m < M && n < N) y[(size_t)m * N + n] = res ? acc + res[(size_t)m * N + n] : acc;
}

hipError_t launch_gemm_f32(const float *x, const float *W, const float *res, float *y, int M,
                           int N, int K, hipStream_t st)
{
    if (M <= 0 || N <= 0) return hipSuccess;
    hipLaunchKernelGGL(gemm_f32_kernel, dim3((N + 15) / 16, (M + 15) / 16), dim3(256), 0, st, x, W, res,
                       y, M, N, K);
    return hipGetLastError();
}

// =============================================================================================
// Weight-streaming GEMM (decode-sized row counts)
// =============================================================================================
constexpr int kSkNB = 4;     // 16-row weight blocks per wavefront (64 output columns)
constexpr int kSkWaves = 4;  // wavefronts per workgroup, each a contiguous part of the segment
constexpr int kSkU = 4;      // k-fragments in flight per wavefront

static inline int sk_tiles(int N) { return (N / 16 + kSkNB - 1) / kSkNB; }

int skinny_segments(int N, int K)
{
    const int kfrags = K / 32, tiles = sk_tiles(N);
    int S = (512 + tiles - 1) / tiles;  // aim for >= 2 workgroups per CU
    if (S > 4) S = 4;
    int max_s = kfrags / (kSkWaves * 2);  // at least 2 fragments per wavefront
    if (S > max_s) S = max_s;
    if (S < 1) S = 1;
    const int per = (kfrags + S - 1) / S;
    return (kfrags + per - 1) / per;
}

size_t skinny_partial_bytes(int M, int N, int K)
{
    return (size_t)skinny_segments(N, K) * (size_t)M * (size_t)N * sizeof(float);
}

template <int MB>
__global__ __launch_bounds__(kSkWaves * 64) void gemm_skinny_kernel(
    const uint4 *__restrict__ Wp, const uint4 *__restrict__ Xp, float *__restrict__ part, int nblk,
    int kfrags, int ntiles, int kf_seg, int M, int N)
{
    __shared__ float red[kSkWaves - 1][kSkNB * MB * 4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int tile = blockIdx.x % ntiles, seg = blockIdx.x / ntiles;
    const int nb0 = tile * kSkNB;
    const int seg_lo = seg * kf_seg;
    const int seg_hi = min(kfrags, seg_lo + kf_seg);
    const int per_wave = (seg_hi - seg_lo + kSkWaves - 1) / kSkWaves;
    const int kb_lo = min(seg_hi, seg_lo + wave * per_wave);
    const int kb_hi = min(seg_hi, kb_lo + per_wave);

    const uint4 *wp[kSkNB];
#pragma unroll
    for (int j = 0; j < kSkNB; ++j) {
        int nb = min(nb0 + j, nblk - 1);  // clamped blocks are computed and dropped
        wp[j] = Wp + (size_t)nb * kfrags * 64 + lane;
    }
    const uint4 *xp[MB];
#pragma unroll
    for (int i = 0; i < MB; ++i) xp[i] = Xp + (size_t)i * kfrags * 64 + lane;

    f32x4_t acc[kSkNB][MB];
#pragma unroll
    for (int j = 0; j < kSkNB; ++j)
#pragma unroll
        for (int i = 0; i < MB; ++i) acc[j][i] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    int kb = kb_lo;
    for (; kb + kSkU <= kb_hi; kb += kSkU) {
        uint4 w[kSkU][kSkNB], xv[kSkU][MB];
#pragma unroll
        for (int u = 0; u < kSkU; ++u) {
#pragma unroll
            for (int j = 0; j < kSkNB; ++j) w[u][j] = ld_stream(wp[j] + (size_t)(kb + u) * 64);
#pragma unroll
            for (int i = 0; i < MB; ++i) xv[u][i] = xp[i][(size_t)(kb + u) * 64];
        }
#pragma unroll
        for (int u = 0; u < kSkU; ++u)
#pragma unroll
            for (int j = 0; j < kSkNB; ++j)
#pragma unroll
                for (int i = 0; i < MB; ++i) acc[j][i] = mfma16(w[u][j], xv[u][i], acc[j][i]);
    }
    for (; kb < kb_hi; ++kb) {
        uint4 w[kSkNB], xv[MB];
#pragma unroll
        for (int j = 0; j < kSkNB; ++j) w[j] = ld_stream(wp[j] + (size_t)kb * 64);
#pragma unroll
        for (int i = 0; i < MB; ++i) xv[i] = xp[i][(size_t)kb * 64];
#pragma unroll
        for (int j = 0; j < kSkNB; ++j)
#pragma unroll
            for (int i = 0; i < MB; ++i) acc[j][i] = mfma16(w[j], xv[i], acc[j][i]);
    }

    // in-workgroup reduction, fixed order wave 0 + wave 1 + wave 2 + wave 3
    if (wave > 0) {
#pragma unroll
        for (int j = 0; j < kSkNB; ++j)
#pragma unroll
            for (int i = 0; i < MB; ++i)
#pragma unroll
                for (int r = 0; r < 4; ++r) red[wave - 1][(j * MB + i) * 4 + r][lane] = acc[j][i][r];
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
        for (int j = 0; j < kSkNB; ++j) {
            const int nb = nb0 + j;
#pragma unroll
            for (int i = 0; i < MB; ++i) {
                float v[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    float s = acc[j][i][r];
#pragma unroll
                    for (int w = 0; w < kSkWaves - 1; ++w) s += red[w][(j * MB + i) * 4 + r][lane];
                    v[r] = s;
                }
                const int m = i * 16 + (lane & 15);
                if (nb < nblk && m < M) {
                    float4 *dst = (float4 *)(part + ((size_t)seg * M + m) * N + nb * 16 + (lane >> 4) * 4);
                    *dst = make_float4(v[0], v[1], v[2], v[3]);
                }
            }
        }
    }
}

// Fixed-order sum over the K segments + epilogue.  One thread per 4 consecutive outputs.
__global__ __launch_bounds__(256) void skinny_reduce_kernel(const float *__restrict__ part, int S, int M,
                                                            int N, int epi,
                                                            const bf16_t *__restrict__ res,
                                                            bf16_t *__restrict__ out)
{
    const int ncols = (epi == EPI_SWIGLU_PACKED) ? N / 2 : N;  // output columns
    const int q_per_row = ncols / 4;
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= M * q_per_row) return;
    const int m = idx / q_per_row, c = (idx % q_per_row) * 4;
    const size_t seg_stride = (size_t)M * N;
    if (epi == EPI_STORE_RM) {
        const float *p = part + (size_t)m * N + c;
        float4 s = *(const float4 *)p;
        for (int k = 1; k < S; ++k) {
            float4 t = *(const float4 *)(p + k * seg_stride);
            s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
        }
        if (res) {
            uint2 r = *(const uint2 *)(res + (size_t)m * N + c);
            s.x += bf_lo(r.x); s.y += bf_hi(r.x); s.z += bf_lo(r.y); s.w += bf_hi(r.y);
        }
        *(uint2 *)(out + (size_t)m * N + c) = make_uint2(pack2bf(s.x, s.y), pack2bf(s.z, s.w));
    } else {
        // gate columns of output block jb live at packed-weight block 2*jb, up columns at 2*jb+1
        const int gcol = (c >> 4) * 32 + (c & 15);
        const float *pg = part + (size_t)m * N + gcol;
        float4 g = *(const float4 *)pg, u = *(const float4 *)(pg + 16);
        for (int k = 1; k < S; ++k) {
            float4 tg = *(const float4 *)(pg + k * seg_stride), tu = *(const float4 *)(pg + 16 + k * seg_stride);
            g.x += tg.x; g.y += tg.y; g.z += tg.z; g.w += tg.w;
            u.x += tu.x; u.y += tu.y; u.z += tu.z; u.w += tu.w;
        }
        float o0 = g.x / (1.0f + __expf(-g.x)) * u.x, o1 = g.y / (1.0f + __expf(-g.y)) * u.y;
        float o2 = g.z / (1.0f + __expf(-g.z)) * u.z, o3 = g.w / (1.0f + __expf(-g.w)) * u.w;
        *(uint2 *)(out + packed_index(m, c, ncols >> 5)) = make_uint2(pack2bf(o0, o1), pack2bf(o2, o3));
    }
}

hipError_t launch_gemm_skinny_main(const void *Wp, const void *Xp, float *partials, int M, int N,
                                   int K, hipStream_t st)
{
    if (M <= 0) return hipSuccess;
    if (M > kSkinnyMaxRows) return hipErrorInvalidValue;
    const int kfrags = K / 32, nblk = N / 16, ntiles = sk_tiles(N);
    const int S = skinny_segments(N, K);
    const int kf_seg = (kfrags + S - 1) / S;
    dim3 grid(ntiles * S), block(kSkWaves * 64);
    const int mb = (M + 15) / 16;
#define CCS_SK(MBV)                                                                                    \
    hipLaunchKernelGGL(gemm_skinny_kernel<MBV>, grid, block, 0, st, (const uint4 *)Wp, (const uint4 *)Xp, \
                       partials, nblk, kfrags, ntiles, kf_seg, M, N)
    switch (mb) {
        case 1: CCS_SK(1); break;
        case 2: CCS_SK(2); break;
        case 3: CCS_SK(3); break;
        default: CCS_SK(4); break;
    }
#undef CCS_SK
    return hipGetLastError();
}

hipError_t launch_gemm_skinny_reduce(const float *partials, int epi, const void *res, void *out,
                                     int M, int N, int K, hipStream_t st)
{
    if (M <= 0) return hipSuccess;
    const int S = skinny_segments(N, K);
    const int ncols = (epi == EPI_SWIGLU_PACKED) ? N / 2 : N;
    const int total = M * (ncols / 4);
    hipLaunchKernelGGL(skinny_reduce_kernel, dim3((total + 255) / 256), dim3(256), 0, st, partials, S, M, N,
                       epi, (const bf16_t *)res, (bf16_t *)out);
    return hipGetLastError();
}

// =============================================================================================
// LDS-tiled MFMA GEMM (prefill-sized row counts)
// =============================================================================================
// Workgroup tile BN (weight rows) x BM (activation rows) x 64 (k), WN x WM wavefronts, each
// owning (BN/WN) x (BM/WM) outputs as 16x16 accumulator tiles.  Packed fragments are copied
// global -> registers -> LDS verbatim (1 KiB per fragment, conflict-free both ways); the copy of
// k-tile t+1 is in flight while k-tile t is multiplied.  K is walked in order for every output
// element and there is no split over K, so results do not depend on M or on the tile an
// element lands in.
template <int BN, int BM, int WN, int WM>
struct TiledCfg {
    static constexpr int KB = 2;                 // k-fragments per k-tile (BK = 64)
    static constexpr int TN = BN / 16, TM = BM / 16;
    static constexpr int FN = TN / WN, FM = TM / WM;
    static constexpr int THREADS = WN * WM * 64;
    static constexpr int W_CHUNKS = TN * KB * 64, X_CHUNKS = TM * KB * 64;  // uint4 per stage
    static constexpr int W_LD = W_CHUNKS / THREADS, X_LD = X_CHUNKS / THREADS;
    static constexpr size_t LDS_BYTES = 2 * (size_t)(W_CHUNKS + X_CHUNKS) * 16;
    static_assert(W_CHUNKS % THREADS == 0 && X_CHUNKS % THREADS == 0, "tile/threads mismatch");
    static_assert(FN % 2 == 0, "gate/up pairs must stay inside one wavefront");
};

template <int BN, int BM, int WN, int WM>
__global__ __launch_bounds__(WN *WM * 64) void gemm_tiled_kernel(
    const uint4 *__restrict__ Wp, const uint4 *__restrict__ Xp, int epi, const bf16_t *__restrict__ res,
    bf16_t *__restrict__ out, int M, int N, int kfrags, int tiles_m)
{
    using C = TiledCfg<BN, BM, WN, WM>;
    extern __shared__ uint4 lds[];
    constexpr int STAGE = C::W_CHUNKS + C::X_CHUNKS;  // stage s: weights at s*STAGE, activations behind

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wn = wave % WN, wm = wave / WN;
    const int tm = blockIdx.x % tiles_m, tn = blockIdx.x / tiles_m;
    const int nb0 = tn * C::TN, mb0 = tm * C::TM;
    const int nblk = N >> 4, mblk = (M + 15) >> 4;
    const int ktiles = (kfrags + C::KB - 1) / C::KB;

    uint4 gw[C::W_LD], gx[C::X_LD];
    auto fetch = [&](int kt) {
#pragma unroll
        for (int it = 0; it < C::W_LD; ++it) {
            const int c = it * C::THREADS + tid;
            const int frag = c >> 6, nbl = frag / C::KB, kb = kt * C::KB + frag % C::KB;
            gw[it] = (nb0 + nbl < nblk && kb < kfrags)
                         ? Wp[((size_t)(nb0 + nbl) * kfrags + kb) * 64 + (c & 63)]
                         : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int it = 0; it < C::X_LD; ++it) {
            const int c = it * C::THREADS + tid;
            const int frag = c >> 6, mbl = frag / C::KB, kb = kt * C::KB + frag % C::KB;
            gx[it] = (mb0 + mbl < mblk && kb < kfrags)
                         ? Xp[((size_t)(mb0 + mbl) * kfrags + kb) * 64 + (c & 63)]
                         : make_uint4(0, 0, 0, 0);
        }
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int it = 0; it < C::W_LD; ++it) lds[buf * STAGE + it * C::THREADS + tid] = gw[it];
#pragma unroll
        for (int it = 0; it < C::X_LD; ++it) lds[buf * STAGE + C::W_CHUNKS + it * C::THREADS + tid] = gx[it];
    };

    f32x4_t acc[C::FN][C::FM];
#pragma unroll
    for (int j = 0; j < C::FN; ++j)
#pragma unroll
        for (int i = 0; i < C::FM; ++i) acc[j][i] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    fetch(0);
    stash(0);
    __syncthreads();
    for (int kt = 0; kt < ktiles; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < ktiles) fetch(kt + 1);
#pragma unroll
        for (int kb = 0; kb < C::KB; ++kb) {
            uint4 a[C::FN], b[C::FM];
#pragma unroll
            for (int j = 0; j < C::FN; ++j) a[j] = lds[cur * STAGE + ((wn * C::FN + j) * C::KB + kb) * 64 + lane];
#pragma unroll
            for (int i = 0; i < C::FM; ++i) b[i] = lds[cur * STAGE + C::W_CHUNKS + ((wm * C::FM + i) * C::KB + kb) * 64 + lane];
#pragma unroll
            for (int j = 0; j < C::FN; ++j)
#pragma unroll
                for (int i = 0; i < C::FM; ++i) acc[j][i] = mfma16(a[j], b[i], acc[j][i]);
        }
        if (kt + 1 < ktiles) stash(cur ^ 1);
        __syncthreads();
    }

    // epilogue: acc[j][i][r] is y[m][n] with n = nb*16 + (lane/16)*4 + r, m = mb*16 + lane%16
    const int mrow = lane & 15, nq = (lane >> 4) * 4;
    if (epi == EPI_STORE_RM) {
#pragma unroll
        for (int j = 0; j < C::FN; ++j) {
            const int nb = nb0 + wn * C::FN + j;
            if (nb >= nblk) continue;
#pragma unroll
            for (int i = 0; i < C::FM; ++i) {
                const int m = (mb0 + wm * C::FM + i) * 16 + mrow;
                if (m >= M) continue;
                const size_t o = (size_t)m * N + nb * 16 + nq;
                float v0 = acc[j][i][0], v1 = acc[j][i][1], v2 = acc[j][i][2], v3 = acc[j][i][3];
                if (res) {
                    uint2 r = *(const uint2 *)(res + o);
                    v0 += bf_lo(r.x); v1 += bf_hi(r.x); v2 += bf_lo(r.y); v3 += bf_hi(r.y);
                }
                *(uint2 *)(out + o) = make_uint2(pack2bf(v0, v1), pack2bf(v2, v3));
            }
        }
    } else {
        const int ifrags = N >> 6;  // I / 32
#pragma unroll
        for (int j = 0; j < C::FN; j += 2) {
            const int nb = nb0 + wn * C::FN + j;  // even: gate block, nb + 1: up block
            if (nb + 1 >= nblk) continue;
#pragma unroll
            for (int i = 0; i < C::FM; ++i) {
                const int m = (mb0 + wm * C::FM + i) * 16 + mrow;
                if (m >= M) continue;
                float o[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float g = acc[j][i][r];
                    o[r] = g / (1.0f + __expf(-g)) * acc[j + 1][i][r];
                }
                const int col = (nb >> 1) * 16 + nq;
                *(uint2 *)(out + packed_index(m, col, ifrags)) = make_uint2(pack2bf(o[0], o[1]), pack2bf(o[2], o[3]));
            }
        }
    }
}

template <int BN, int BM, int WN, int WM>
static hipError_t launch_tiled_cfg(const void *Wp, const void *Xp, int epi, const void *res, void *out,
                                   int M, int N, int K, hipStream_t st)
{
    using C = TiledCfg<BN, BM, WN, WM>;
    static bool attr_done = false;
    auto kern = gemm_tiled_kernel<BN, BM, WN, WM>;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)C::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(C::THREADS), C::LDS_BYTES, st, (const uint4 *)Wp,
                       (const uint4 *)Xp, epi, (const bf16_t *)res, (bf16_t *)out, M, N, K / 32, tiles_m);
    return hipGetLastError();
}

hipError_t launch_gemm_tiled(const void *Wp, const void *Xp, int epi, const void *res, void *out,
                             int M, int N, int K, hipStream_t st)
{
    if (M <= 0) return hipSuccess;
    return launch_tiled_cfg<256, 256, 2, 4>(Wp, Xp, epi, res, out, M, N, K, st);
}

}  // namespace ccs
