// Projection GEMMs of the decoder layer (paper, Section 2.1: Q/K/V/O and the three FFN
// projections are linear maps; Table 1 puts ~99 % of a layer's FLOPs in them).
//
// y[m, n] = sum_k x[m, k] * W[n, k].  On the bf16 path both operands are fragment-packed
// (ccs_common.h): 1 KiB fragments of 16 rows x 32 k in the operand register layout of the matrix
// cores, the weight as the A operand and the activation as the B operand.
//
//  * gemm_tiled_dma: LDS-tiled, for compute-bound row counts (prefill): 256 x 128 x 32 workgroup
//    tiles of v_mfma_f32_32x32x16_bf16, operands brought in by direct-to-LDS loads through a
//    3-stage ring, optional deterministic K split for launches that cannot fill the GPU.
//  * skinny_reduce: fixed-order sum of K-split partial sums + epilogue (the weight-streaming
//    projections for <= 64 rows live in ccs_gemm_stream.hip).
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
// Reduction of K-split partial sums (both the LDS-tiled GEMM and the weight-streaming projections)
// =============================================================================================
// Fixed-order sum over the K segments + epilogue.  One thread per 4 consecutive outputs.
__global__ __launch_bounds__(256) void skinny_reduce_kernel(const float *__restrict__ part, int S, int M,
                                                            int N, int epi,
                                                            const bf16_t *__restrict__ res,
                                                            bf16_t *__restrict__ out,
                                                            bf16_t *__restrict__ out_packed)
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
        const uint2 o = make_uint2(pack2bf(s.x, s.y), pack2bf(s.z, s.w));
        *(uint2 *)(out + (size_t)m * N + c) = o;
        if (out_packed) *(uint2 *)(out_packed + packed_index(m, c, N >> 5)) = o;
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

hipError_t launch_partial_reduce(const float *partials, int S, int epi, const void *res, void *out, void *out_packed,
                                 int M, int N, hipStream_t st)
{
    if (M <= 0) return hipSuccess;
    const int ncols = (epi == EPI_SWIGLU_PACKED) ? N / 2 : N;
    const int total = M * (ncols / 4);
    hipLaunchKernelGGL(skinny_reduce_kernel, dim3((total + 255) / 256), dim3(256), 0, st, partials, S, M, N,
                       epi, (const bf16_t *)res, (bf16_t *)out, (bf16_t *)out_packed);
    return hipGetLastError();
}

// =============================================================================================
// LDS-tiled MFMA GEMM (prefill-sized row counts)
// =============================================================================================
// ---------------------------------------------------------------------------------------------
// Main prefill GEMM: 256 (weight rows) x BM (activation rows, 256 or 128) x 32 (k) workgroup
// tile, 4 wavefronts (2 x 2), each owning 128 x BM/2 outputs as accumulator tiles of
// v_mfma_f32_32x32x16_bf16 (256 or 128 accumulator registers).  The shipped configuration is
// BM = 128 with a 3-stage ring, which fits two workgroups (two wavefronts per SIMD) on a CU.
//
// Packed fragments go global -> LDS with direct-to-LDS loads (global_load_lds_dwordx4: one
// instruction moves one 1 KiB fragment; no staging registers, no ds_write) into a ring of NST
// stages; NST - 1 k-tiles are in flight while one is multiplied, which is what hides the
// L2-miss latency (with two stages the kernel ran at the latency of the slowest load per
// k-tile).  The fragments of the next 16-wide k-step are read from LDS while the MFMAs of the
// current step issue.  Unit rates this is sized against (measured, per CU): MFMA 32x32x16
// reaches the bf16 peak with one wavefront per SIMD (16x16x32 needs two); LDS reads ~240 B/clk;
// the vector-memory path (L2 hits, to registers or LDS alike) ~60 B/clk, which a 256 x 256 tile
// loads to ~53 % of the MFMA time.
//
// A 32x32x16 operand is assembled from the 16 x 32 packed fragments: lane l takes row l%32
// (16-row block (l%32)/16) and the 16-byte chunk (l%16) + 16*(2*half + l/32); every group of 16
// lanes reads 256 contiguous bytes, so the LDS reads are conflict free.
//
// The LDS reads and waits of the main loop are inline assembly: the compiler serialises every
// ds_read behind all outstanding direct-to-LDS loads (it cannot prove the stages do not alias)
// and does not prefetch fragments across MFMAs.  Each k-tile issues the same number of loads per
// lane (out-of-range blocks are clamped to the last valid block; their products land in
// accumulators that are never stored), so `s_waitcnt vmcnt(n)` counts whole k-tiles.
// Needs K % 32 == 0 (always true for packed operands).
// ---------------------------------------------------------------------------------------------
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;

template <int BM, int NST>
struct DmaCfg {
    static constexpr int TN = 16, TM = BM / 16;         // 16-row blocks per stage
    static constexpr int FM = BM / 64;                  // 32-row activation fragments per wavefront
    static constexpr int FPW = (TN + TM) / 4;           // fragments each wavefront loads per k-tile
    static constexpr int STAGE = (TN + TM) * 64;        // uint4 per stage
    static constexpr size_t LDS_BYTES = (size_t)NST * STAGE * 16;
    static constexpr int WAIT_STEADY = (NST - 2) * FPW; // loads that may stay in flight at the barrier
    static constexpr int WAIT_PROLOGUE = (NST - 1) * FPW;
    static_assert(LDS_BYTES <= 160 * 1024, "LDS ring too large");
    static_assert(WAIT_PROLOGUE < 64, "vmcnt is a 6-bit counter");
};

#define CCS_STR2(x) #x
#define CCS_STR(x) CCS_STR2(x)

__device__ __forceinline__ void dma_one(const uint4 *src, uint4 *lds_dst)
{
    __builtin_amdgcn_global_load_lds(src, lds_dst, 16, 0, 0);
}

template <int FPW>
__device__ __forceinline__ void dma_issue(const uint4 *const *src, const int *kstep, int kt, uint4 *lds_dst)
{
#pragma unroll
    for (int i = 0; i < FPW; ++i)
        __builtin_amdgcn_global_load_lds(src[i] + (size_t)kt * kstep[i], lds_dst + i * 64, 16, 0, 0);
}

template <int BM, int NST>
__global__ __launch_bounds__(256, (BM == 128 && NST <= 3) ? 2 : 1) void gemm_tiled_dma_kernel(
    const uint4 *__restrict__ Wp, const uint4 *__restrict__ Xp, int epi, const bf16_t *__restrict__ res,
    bf16_t *__restrict__ out, int M, int N, int kfrags, int tiles_m, int tiles, float *__restrict__ part,
    int kt_per_seg, int x_rows)
{
    using C = DmaCfg<BM, NST>;
    extern __shared__ uint4 lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wn = wave & 1, wm = wave >> 1;
    // K segment of this workgroup (one segment unless the launch is split over K: then the
    // fp32 partial sums of segment `seg` go to part[seg][M][N] and a reduction kernel follows)
    // Workgroups go to the 8 XCDs round-robin by index and every XCD has its own L2: give XCD x a
    // contiguous range of the (tile, K segment) list, so that the row tiles that share a weight
    // panel run on one XCD at about the same time and the panel is fetched into one L2 once.
    const int nwg = gridDim.x, xcd = blockIdx.x & 7, in_xcd = blockIdx.x >> 3;
    const int logical = xcd * (nwg >> 3) + min(xcd, nwg & 7) + in_xcd;
    const int tile_id = logical % tiles, seg = logical / tiles;
    const int tm = tile_id % tiles_m, tn = tile_id / tiles_m;
    const int nb0 = tn * C::TN, mb0 = tm * C::TM;
    const int nblk = N >> 4, mblk = (M + 15) >> 4;
    const int kt0 = seg * kt_per_seg;
    const int ktiles = min(kfrags, kt0 + kt_per_seg) - kt0;

    // fragment f of a stage: f < TN -> weight block nb0 + f (grouped weight order: the next k-tile
    // of a block is kWGroup fragments further), else activation block mb0 + f - TN (plain order)
    const uint4 *src[C::FPW];
    int kstep[C::FPW];  // uint4 from one k-tile to the next
#pragma unroll
    for (int i = 0; i < C::FPW; ++i) {
        const int f = wave * C::FPW + i;
        const bool is_x = f >= C::TN;
        const int blk = is_x ? min(mb0 + f - C::TN, mblk - 1) : min(nb0 + f, nblk - 1);
        src[i] = is_x ? Xp + ((size_t)blk * kfrags + kt0) * 64 + lane : Wp + weight_fragment(blk, kt0, kfrags) * 64 + lane;
        kstep[i] = is_x ? 64 : kWGroup * 64;
        if (is_x && x_rows) {
            // activations as plain row-major rows [M, K]: fragment slot `lane` (row lane % 16, k quarter
            // lane / 16) is 16 contiguous bytes of its row, so the direct-to-LDS load can fetch it from
            // there (the LDS side stays in fragment order); rows past M repeat the last row, never stored
            const int row = min(blk * 16 + (lane & 15), M - 1);
            src[i] = Xp + (size_t)row * kfrags * 4 + (size_t)kt0 * 4 + (lane >> 4);
            kstep[i] = 4;
        }
    }
    // (a __device__ helper, not a lambda: the host pass cannot instantiate a lambda that holds the
    // direct-to-LDS builtin and then silently drops the kernel's launch stub)
#define dma(kt, stage) dma_issue<C::FPW>(src, kstep, kt, lds + (stage) * C::STAGE + wave * C::FPW * 64)

    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint4 *)lds;
    const int sub = ((lane & 31) >> 4) * 64 + (lane & 15) + 16 * (lane >> 5);
    const uint32_t a_addr = lds0 + (uint32_t)(wn * 8 * 64 + sub) * 16;                       // + j * 2048 per fragment
    const uint32_t b_addr = lds0 + (uint32_t)((C::TN + wm * C::FM * 2) * 64 + sub) * 16;     // + i * 2048
    constexpr uint32_t kStageBytes = C::STAGE * 16;

    f32x16_t acc[4][C::FM];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < C::FM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[j][i][r] = 0.f;

    // two fragment register sets: k-step s multiplies set s % 2 while set (s + 1) % 2 is being read.
    // A wavefront issues in order and is alone on its SIMD, so every LDS read and every
    // direct-to-LDS load is placed in the shadow of an MFMA (2 MFMAs, then one read and at most
    // one load): issued in a block in front of the MFMAs they cost their full issue time.
    u32x4_t fa0[4], fb0[4], fa1[4], fb1[4];
    constexpr int MPG = (4 * C::FM) / 8;  // MFMAs per group, 8 groups per k-step
#define CCS_LDS_READ(dst, addr, OFF) \
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "i"(OFF) : "memory")
#define CCS_WAIT_SET(fa, fb)                                                                                  \
    do {                                                                                                      \
        if (C::FM > 2)                                                                                        \
            asm volatile("s_waitcnt lgkmcnt(0)"                                                               \
                         : "+v"(fa[0]), "+v"(fa[1]), "+v"(fa[2]), "+v"(fa[3]), "+v"(fb[0]), "+v"(fb[1]),      \
                           "+v"(fb[2]), "+v"(fb[3])::"memory");                                               \
        else                                                                                                  \
            asm volatile("s_waitcnt lgkmcnt(0)"                                                               \
                         : "+v"(fa[0]), "+v"(fa[1]), "+v"(fa[2]), "+v"(fa[3]), "+v"(fb[0]), "+v"(fb[1])::"memory"); \
    } while (0)
    // one k-step: multiply (ca, cb); if do_read, fetch (na, nb) from abase/bbase + OFF; if do_dma,
    // issue this wavefront's loads of k-tile kt_dma into stage st_dma
#define CCS_STEP(ca, cb, na, nb, abase, bbase, OFF, do_read, do_dma, kt_dma, st_dma)                           \
    do {                                                                                                       \
        __builtin_amdgcn_sched_barrier(0);                                                                     \
        _Pragma("unroll") for (int q = 0; q < 8; ++q) {                                                        \
            _Pragma("unroll") for (int e = 0; e < MPG; ++e) {                                                  \
                const int idx = q * MPG + e, j = idx / C::FM, i = idx % C::FM;                                 \
                acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                                           \
                    __builtin_bit_cast(bf16x8_t, ca[j]), __builtin_bit_cast(bf16x8_t, cb[i]), acc[j][i], 0, 0, 0); \
            }                                                                                                  \
            __builtin_amdgcn_sched_barrier(0);                                                                 \
            if (do_read) {                                                                     \
                if (q < 4) CCS_LDS_READ(na[q & 3], (abase) + (q & 3) * 2048u, OFF);                            \
                else if (q - 4 < C::FM) CCS_LDS_READ(nb[q & 3], (bbase) + (q & 3) * 2048u, OFF);               \
            }                                                                                                  \
            if ((do_dma) && q < C::FPW)                                                          \
                dma_one(src[q < C::FPW ? q : 0] + (size_t)(kt_dma) * kstep[q < C::FPW ? q : 0],                \
                        lds + (st_dma) * C::STAGE + (wave * C::FPW + q) * 64);                                 \
            __builtin_amdgcn_sched_barrier(0);                                                                 \
        }                                                                                                      \
    } while (0)

#pragma unroll
    for (int t = 0; t < NST; ++t) dma(min(t, ktiles - 1), t);
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(C::WAIT_PROLOGUE) : "memory");
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 4; ++q) CCS_LDS_READ(fa0[q], a_addr + q * 2048u, 0);
#pragma unroll
    for (int q = 0; q < C::FM; ++q) CCS_LDS_READ(fb0[q], b_addr + q * 2048u, 0);
    CCS_WAIT_SET(fa0, fb0);
    int stage = 0;
    for (int kt = 0; kt < ktiles; ++kt) {
        const int nstage = (stage + 1 == NST) ? 0 : stage + 1;
        const uint32_t ab = a_addr + stage * kStageBytes, bb = b_addr + stage * kStageBytes;
        const uint32_t an = a_addr + nstage * kStageBytes, bn = b_addr + nstage * kStageBytes;
        // k-step 0 (half 0 of the fragments); half 1 (+512 B) is read meanwhile
        CCS_STEP(fa0, fb0, fa1, fb1, ab, bb, 512, true, false, 0, 0);
        CCS_WAIT_SET(fa1, fb1);
        // this wavefront is done reading `stage`; k-tile kt + 1 must have landed for everybody
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(C::WAIT_STEADY) : "memory");
        __syncthreads();
        // k-step 1: refill `stage` with k-tile kt + NST, read step 0 of k-tile kt + 1 meanwhile
        // (past the end the refill re-loads the last k-tile into a stage nobody reads and the
        // fragment read fetches values nobody multiplies: the loop body has no branches)
        CCS_STEP(fa1, fb1, fa0, fb0, an, bn, 0, true, true, min(kt + NST, ktiles - 1), stage);
        CCS_WAIT_SET(fa0, fb0);
        stage = nstage;
    }
#undef CCS_STEP
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // no load may land in LDS after this workgroup is gone
#undef CCS_LDS_READ
#undef CCS_WAIT_SET
#undef dma

    // Epilogue.  acc[j][i][r] = y[m][n] with m = 32-row block base + lane % 32 and
    // n = 32-row weight tile base + (r / 4) * 8 + (lane / 32) * 4 + r % 4: a lane owns 4 consecutive
    // n of one row, so direct stores would be 8-byte pieces scattered over 32 rows.  Every
    // wavefront therefore turns its outputs through its own LDS region, one 32-row block at a
    // time, and stores full 256-byte row segments (row-major output) or whole 1 KiB fragments
    // (packed output): 16 bytes per lane, fully coalesced.
    __syncthreads();  // every wavefront's loads have landed: the stages can be reused
    const int mlane = lane & 31, nsub = (lane >> 5) * 4;
    if (epi == EPI_STORE_RM || part != nullptr) {
        constexpr int ROWB = 128 * 4 + 16;  // padded fp32 row: 16 lanes x 16 B hit 64 different banks
        char *reg = (char *)lds + wave * (32 * ROWB);
        const int n_wave = (nb0 + wn * 8) * 16;  // first output column of this wavefront
#pragma unroll
        for (int i = 0; i < C::FM; ++i) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g)
                    *(float4 *)(reg + mlane * ROWB + (j * 32 + g * 8 + nsub) * 4) =
                        make_float4(acc[j][i][g * 4 + 0], acc[j][i][g * 4 + 1], acc[j][i][g * 4 + 2], acc[j][i][g * 4 + 3]);
            const int m0 = (mb0 + (wm * C::FM + i) * 2) * 16;
            const int n = n_wave + (lane & 15) * 8;
#pragma unroll
            for (int rr = 0; rr < 8; ++rr) {
                const int row = rr * 4 + (lane >> 4), m = m0 + row;
                const float4 lo = *(const float4 *)(reg + row * ROWB + (lane & 15) * 32);
                const float4 hi = *(const float4 *)(reg + row * ROWB + (lane & 15) * 32 + 16);
                if (m < M && n < N && part != nullptr) {
                    float *o = part + ((size_t)seg * M + m) * N + n;
                    *(float4 *)o = lo;
                    *(float4 *)(o + 4) = hi;
                } else if (m < M && n < N) {
                    const size_t o = (size_t)m * N + n;
                    float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
                    if (res) {
                        const uint4 r = *(const uint4 *)(res + o);
                        v[0] += bf_lo(r.x); v[1] += bf_hi(r.x); v[2] += bf_lo(r.y); v[3] += bf_hi(r.y);
                        v[4] += bf_lo(r.z); v[5] += bf_hi(r.z); v[6] += bf_lo(r.w); v[7] += bf_hi(r.w);
                    }
                    *(uint4 *)(out + o) = make_uint4(pack2bf(v[0], v[1]), pack2bf(v[2], v[3]), pack2bf(v[4], v[5]),
                                                     pack2bf(v[6], v[7]));
                }
            }
        }
    } else {
        // SwiGLU: rows 0..15 of a 32-row weight tile are a gate block, rows 16..31 the matching up
        // block, so acc[..][r] and acc[..][r + 8] pair up; a wavefront produces 64 columns of u per
        // 32-row block = 2 x 2 packed fragments, assembled in LDS in packed order.
        char *reg = (char *)lds + wave * 4096;
        const int ifrags = N >> 6;                     // I / 32
        const int cb0 = (nb0 >> 1) / 2 + wn * 2;       // first 32-column fragment of u of this wavefront
#pragma unroll
        for (int i = 0; i < C::FM; ++i) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int g = 0; g < 2; ++g) {
                    float o[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const float gt = acc[j][i][g * 4 + r];
                        o[r] = gt / (1.0f + __expf(-gt)) * acc[j][i][8 + g * 4 + r];
                    }
                    const int c = j * 16 + g * 8 + nsub;  // column within the wavefront's 64
                    const int off = ((mlane >> 4) * 2 + (c >> 5)) * 1024 + ((mlane & 15) + 16 * ((c & 31) >> 3)) * 16 + (c & 7) * 2;
                    *(uint2 *)(reg + off) = make_uint2(pack2bf(o[0], o[1]), pack2bf(o[2], o[3]));
                }
            const int mb = mb0 + (wm * C::FM + i) * 2;  // first 16-row block of this 32-row block
#pragma unroll
            for (int f = 0; f < 4; ++f) {
                const uint4 v = *(const uint4 *)(reg + f * 1024 + lane * 16);
                const int mbf = mb + (f >> 1), cb = cb0 + (f & 1);
                if (mbf < mblk && cb < ifrags) ((uint4 *)out)[((size_t)mbf * ifrags + cb) * 64 + lane] = v;
            }
        }
    }
}

template <int BM, int NST>
hipError_t launch_gemm_tiled_dma(const void *Wp, const void *Xp, int epi, const void *res, void *out,
                                 int M, int N, int K, float *part, int S, bool x_rows, hipStream_t st)
{
    using C = DmaCfg<BM, NST>;
    auto kern = gemm_tiled_dma_kernel<BM, NST>;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + 255) / 256, tiles = tiles_m * tiles_n;
    const int kfrags = K / 32, per = (kfrags + S - 1) / S;
    hipLaunchKernelGGL(kern, dim3(tiles * S), dim3(256), C::LDS_BYTES, st, (const uint4 *)Wp, (const uint4 *)Xp, epi,
                       (const bf16_t *)res, (bf16_t *)out, M, N, kfrags, tiles_m, tiles, part, per, x_rows ? 1 : 0);
    return hipGetLastError();
}

// K segments of the LDS-tiled GEMM: 1 when the launch fills the GPU; otherwise (few hundred rows
// against a narrow weight: fewer than 192 workgroup tiles) K is cut to fill whole rounds of CUs.
// The count is taken from the row count of the FULL batch (variant_rows), never from the slice a
// replica gets, so every replica count reduces in the same order.
int tiled_segments(int N, int K, long variant_rows)
{
    const long tiles = (long)((N + 255) / 256) * ((variant_rows + 127) / 128);
    if (tiles >= 192) return 1;
    const int kfrags = K / 32;
    // rounds of 256 one-per-CU workgroups, each 1/S of the K loop, plus what the split costs (a
    // second launch, S partial buffers written and read back)
    int best = 1;
    double best_cost = (double)((tiles + 255) / 256);
    for (int S = 2; S <= 8 && S <= kfrags / 16; ++S) {
        const double cost = (double)((tiles * S + 255) / 256) / S + 0.08 + 0.02 * (S - 1);
        if (cost < best_cost) { best_cost = cost; best = S; }
    }
    const int per = (kfrags + best - 1) / best;
    return (kfrags + per - 1) / per;
}

size_t tiled_partial_bytes(int M, int N, int K, long variant_rows)
{
    const int S = tiled_segments(N, K, variant_rows);
    return S > 1 ? (size_t)S * M * N * sizeof(float) : 0;
}

hipError_t launch_gemm_tiled(const void *Wp, const void *Xp, bool x_rows, int epi, const void *res, void *out,
                             int M, int N, int K, long variant_rows, float *partials, hipStream_t st)
{
    if (M <= 0) return hipSuccess;
    const int S = tiled_segments(N, K, variant_rows);
    if (S > 1) {
        hipError_t e = launch_gemm_tiled_dma<128, 3>(Wp, Xp, epi, nullptr, nullptr, M, N, K, partials, S, x_rows, st);
        if (e != hipSuccess) return e;
        return launch_partial_reduce(partials, S, epi, res, out, nullptr, M, N, st);
    }
    // 256 x 128 tiles, 3-stage ring (72 KiB): two workgroups share a CU, so one's epilogue and
    // prologue run under the other's main loop - measured 5-20 % faster than one 256 x 256 or
    // 256 x 128 workgroup per CU with a deeper ring on every projection shape of the 13B layer.
    return launch_gemm_tiled_dma<128, 3>(Wp, Xp, epi, res, out, M, N, K, nullptr, 1, x_rows, st);
}

// Function attributes (dynamic LDS sizes) of this file's kernels; once per process, outside any
// stream capture (ccs_module_create calls it).
hipError_t init_gemm_kernels()
{
    hipError_t e = hipFuncSetAttribute((const void *)gemm_tiled_dma_kernel<128, 3>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)DmaCfg<128, 3>::LDS_BYTES);
    if (e == hipSuccess) e = init_gemm_stream_kernels();
    return e;
}

}  // namespace ccs
