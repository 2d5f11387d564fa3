// Weight-streaming projections for decode-sized row counts (<= 64 rows): the Q/K/V, O, gate/up and
// down projections of a decode step and a small-batch single projection (paper, Section 2.1: decode
// is memory-bound; Section 3.1: a replica runs the unmodified module on its slice).
//
// One launch per projection, nothing left for a second kernel:
//   * a workgroup owns NB 16-column blocks of the output over the WHOLE K range; its 4 wavefronts
//     stream contiguous quarters of K (1 KiB weight fragments straight into MFMA A operands, two
//     rolling register sets so that loads stay in flight under the MFMAs) and their accumulators
//     are added through LDS in the fixed order (0 + 2) + (1 + 3);
//   * the activation operand is fragment-packed, or (XROWS) the plain row-major rows of the caller:
//     then a wavefront fetches its k-steps with coalesced loads (four lanes per 64-byte row piece)
//     and turns them into fragment order through a private, XOR-swizzled piece of LDS (one
//     conflict-free 16-byte write and read per lane and fragment) - fetching fragment slots
//     straight from the rows costs the address unit four times as many cycles, which made a
//     32-row launch 60 % slower.  With `norm` the kernel is also the RMSNorm in
//     front of the projection: the weights carry the norm's gains already (folded in when the
//     module is created), the activations are the raw rows of the residual stream, the row's sum
//     of squares comes from one extra MFMA per fragment (the diagonal of X X^T, accumulated in
//     fp32 in a fixed order) and the accumulators are scaled by rsqrt(mean square + eps) in the
//     epilogue - a row's scale is a scalar, so it commutes with the projection;
//   * epilogues: store (+ residual) row-major, optionally also fragment-packed for the next
//     projection; SwiGLU into a fragment-packed u; and for the decode Q/K/V projection the rotary
//     embedding, the q store and the KV-cache append (a tile is made of whole rotary pairs: dims
//     [16 s, 16 s + 16) and their partners 64 up, plus - in the 3-block form - 16 dims of a v head).
//   * tile shapes: a compute unit sustains only so many outstanding misses, so a launch streams
//     at a rate proportional to the compute units it keeps busy - every launcher below picks tiles
//     that leave all 256 of them about the same number of blocks (two passes over NB + NB2 blocks
//     when one pass would need too many accumulators); and narrow tiles re-read the activations
//     once per tile through the same L1, so where K is long enough (SPLIT) tiles stay wide, K is
//     cut over 2..4 workgroups per tile and the workgroup that finishes last adds the partial
//     tiles in segment order inside the launch (device-coherent stores and loads, an arrival
//     counter per tile; nobody waits, so nothing can hang);
//   * column-split form (COLS; gate/up of a 33..64-row batch with five to eight (gate, up) pairs per
//     workgroup): the wavefronts share K and split the tile's columns, the activation fragments
//     are fetched once per workgroup and handed round through LDS - NB / 4 x MB accumulator tiles
//     per wavefront instead of NB x MB, so 14 blocks fit ONE pass where the K-split form needs
//     two passes that fetch the activations twice (70B gate/up at 64 rows: 152 -> 143 us);
//   * GS_PARTIALS: the same cut with fp32 partial sums (and per-segment sums of squares) left for a
//     small second kernel that adds them in segment order and applies the epilogue - kept where
//     that kernel has more to do than add (rotary + cache append for 33..64 rows) or measured
//     faster (K > 8192 at 33..64 rows).
// Tile shape, K cut and everything else about the launch depend on the weight shape and on the row
// count of the full batch only, and every output row is computed from its own input row alone,
// so a row's bits do not depend on the batch.
#include "ccs_common.h"
#include "ccs_kernels.h"

namespace ccs {

namespace {


__device__ __forceinline__ f32x4_t gs_mfma(const uint4 &a, const uint4 &b, f32x4_t c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c,
                                                   0, 0, 0);
}

// k-steps per register set: enough bytes in flight per wavefront without spilling
constexpr int gs_u(int MB, int NB) { return (NB + MB) <= 3 ? 6 : (NB + MB) <= 6 ? 4 : 2; }

// floats of LDS the reduction and the row statistics take: W / 2 tile buffers, per-wavefront sums of squares, scales
constexpr int gs_red_floats(int MB, int NB, int W, int COLS = 0) { return (COLS ? 1 : W / 2) * MB * 16 * (NB * 16 + 4) + W * MB * 16 + MB * 16 + 4; }

struct GsArgs {
    const uint4 *Wp;      // grouped fragment-packed weight
    int kfrags;           // K / 32
    int G;                // 16-row blocks per weight group (layout of Wp)
    const uint4 *X;       // fragment-packed rows [M16, K]; XROWS: row-major bf16 rows [M, K]
    int norm;             // X holds raw rows: scale row m of the result by rsqrt(mean_k x[m, k]^2 + eps)
    float eps;
    int M, N;             // rows; valid output columns
    const bf16_t *res;    // GS_STORE: optional residual, row-major [M, N]
    bf16_t *out;
    bf16_t *out_packed;   // GS_STORE: optional second copy of the result, fragment-packed [M16, N]
    // K segments over workgroups (GS_PARTIALS; otherwise one segment = all of K)
    int ntiles;           // column tiles of the launch: workgroup b works on tile b % ntiles, segment b / ntiles
    int kf_seg;           // k-steps per segment
    float *part;          // fp32 partial sums [S, M, N]
    float *ssq_part;      // optional: the rows' sums of squares per segment [S, M]
    // SPLIT: K cut over nseg workgroups per tile, summed by the workgroup of a tile that finishes last
    int nseg;
    int *cnt;
    int nbt;              // COLS: blocks of a tile that exist (<= NB); tile t starts at block t * nbt             // one arrival counter per tile; zero between launches
    // GS_QKV_DECODE
    int nq, nkv;
    const float2 *tab;
    const int32_t *lens;
    bf16_t *kc, *vc;
    int cap;
};

// One tile of a launch: the NB 16-column blocks blk0 .. blk0 + NB - 1 of the weight (GS_QKV_DECODE:
// the blocks that `tile` names, see below) over K segment `seg`, from the first load to the last store.
template <int MB, int NB, int EPI, int kGsWaves, int U, int XROWS, int SPLIT, int COLS = 0>
__device__ __forceinline__ void gs_pass(const GsArgs &a, float *red, const int blk0, const int tile, const int seg)
{
    static_assert(!COLS || (MB == 4 && kGsWaves == 4 && NB % 4 == 0 && !XROWS && EPI != GS_QKV_DECODE && EPI != GS_PARTIALS),
                  "column-split form: 64 rows, four wavefronts, packed activations");
    constexpr int ROWF = NB * 16 + 4;      // floats per padded LDS row: conflict-free 16-byte accesses
    constexpr int BUF = MB * 16 * ROWF;    // floats per reduction buffer
    constexpr bool QKV3 = EPI == GS_QKV_DECODE && NB == 3;   // one rotary pair of blocks of a q or k head + one block of a v head
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int kfrags = a.kfrags, G = a.G;
    const int seg_lo = seg * a.kf_seg, seg_hi = min(kfrags, seg_lo + a.kf_seg);
    const int per_wave = (seg_hi - seg_lo + kGsWaves - 1) / kGsWaves;
    const int kb_lo = min(seg_hi, seg_lo + wave * per_wave);
    const int kb_hi = min(seg_hi, kb_lo + per_wave);

    // 16-row weight blocks of this tile
    constexpr int HH = QKV3 ? 1 : NB >= 2 ? NB / 2 : 1;   // GS_QKV_DECODE: blocks per half of the head
    constexpr int PARTS = QKV3 ? 4 : NB >= 8 ? 1 : 8 / NB;
    const int hs = tile / PARTS, part = tile % PARTS;   // head slot and part of the head (GS_QKV_DECODE)
    const int last_blk = (a.N >> 4) - 1;               // blocks past the weight repeat the last one; never stored
    const bool norm = a.norm != 0;
    constexpr int HALF = kGsWaves / 2;
    constexpr int NRB = COLS ? 1 : HALF;       // reduction buffers
    float *wssq = red + NRB * BUF;             // [wavefronts][MB * 16 rows]
    float *rsv = wssq + kGsWaves * MB * 16;    // [MB * 16]: rsqrt(mean square + eps) per row
    const int nbt = COLS ? a.nbt : NB;         // blocks of this tile that exist
    if constexpr (COLS) {
        // Column-split form (64 rows): the wavefronts share K and split the tile's COLUMNS - wavefront w
        // owns blocks w * NB / 4 .. - so a wavefront keeps NB / 4 x MB accumulator tiles instead of
        // NB x MB and a tile can be 14 or 16 blocks wide in ONE pass; the activation fragments, which
        // every wavefront needs, are fetched once per workgroup (wavefront w loads row block w) and
        // handed round through LDS, one set of U k-steps per barrier, double-buffered.
        constexpr int NBW = NB / 4;
        const uint4 *wq[NBW];
#pragma unroll
        for (int j = 0; j < NBW; ++j) {
            const int nb = min(blk0 + min(wave * NBW + j, nbt - 1), last_blk);   // blocks past the tile repeat its last one; never stored
            wq[j] = a.Wp + (((size_t)(nb / G) * kfrags) * G + (nb % G)) * 64 + lane;
        }
        const size_t wstep = (size_t)G * 64;
        const uint4 *xmine = a.X + (size_t)min(wave, (a.M - 1) >> 4) * kfrags * 64 + lane;   // row block `wave`
        uint4 *xs = (uint4 *)(red + gs_red_floats(MB, NB, kGsWaves, 1));                      // [2 stages][U][MB][64]
        f32x4_t acc[NBW][MB];
#pragma unroll
        for (int j = 0; j < NBW; ++j)
#pragma unroll
            for (int i = 0; i < MB; ++i) acc[j][i] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        f32x4_t sqw = f32x4_t{0.f, 0.f, 0.f, 0.f};   // X X^T of row block `wave`
        uint4 w0[U][NBW], xr0[U], w1[U][NBW], xr1[U];
        const int n_sets = (seg_hi - seg_lo + U - 1) / U;
#define GC_LOAD(W_, XR_, SET)                                                                              \
    _Pragma("unroll") for (int u = 0; u < U; ++u) {                                                        \
        const int kk = min(seg_lo + (SET) * U + u, seg_hi - 1);                                            \
        _Pragma("unroll") for (int j = 0; j < NBW; ++j) W_[u][j] = ld_stream(wq[j] + (size_t)kk * wstep);  \
        XR_[u] = xmine[(size_t)kk * 64];                                                                   \
    }
#define GC_PUBLISH(XR_, STAGE)                                                                             \
    _Pragma("unroll") for (int u = 0; u < U; ++u) xs[(((STAGE) * U + u) * MB + wave) * 64 + lane] = XR_[u];
        // set SET: X of all row blocks from stage STAGE, own weights W_, own row block XR_ for the sum of
        // squares; then the next set's X (XN_, loaded a step ago) goes into the other stage, this set's
        // registers are refilled two sets ahead, and the workgroup meets
#define GC_STEP(W_, XR_, XN_, SET, STAGE)                                                                  \
    {                                                                                                      \
        uint4 xf[U][MB];                                                                                   \
        _Pragma("unroll") for (int u = 0; u < U; ++u)                                                      \
            _Pragma("unroll") for (int i = 0; i < MB; ++i) xf[u][i] = xs[(((STAGE) * U + u) * MB + i) * 64 + lane]; \
        _Pragma("unroll") for (int u = 0; u < U; ++u) {                                                    \
            if (seg_lo + (SET) * U + u < seg_hi) {                                                         \
                _Pragma("unroll") for (int j = 0; j < NBW; ++j)                                             \
                    _Pragma("unroll") for (int i = 0; i < MB; ++i) acc[j][i] = gs_mfma(W_[u][j], xf[u][i], acc[j][i]); \
                if (EPI == GS_SWIGLU || norm) sqw = gs_mfma(XR_[u], XR_[u], sqw);                          \
            }                                                                                              \
        }                                                                                                  \
        GC_PUBLISH(XN_, 1 - (STAGE));                                                                      \
        GC_LOAD(W_, XR_, (SET) + 2);                                                                       \
        __syncthreads();                                                                                   \
    }
        GC_LOAD(w0, xr0, 0);
        GC_PUBLISH(xr0, 0);
        GC_LOAD(w1, xr1, 1);
        __syncthreads();
        for (int s = 0; s < n_sets; s += 2) {
            GC_STEP(w0, xr0, xr1, s, 0);
            GC_STEP(w1, xr1, xr0, s + 1, 1);
        }
#undef GC_LOAD
#undef GC_PUBLISH
#undef GC_STEP
        // every wavefront puts its columns into the one tile buffer; its row block's sums of squares, zeros for the others
        float *slot0 = red + (lane & 15) * ROWF + (lane >> 4) * 4;
#pragma unroll
        for (int j = 0; j < NBW; ++j) {
            const int cb = wave * NBW + j;
            if (cb < nbt) {
#pragma unroll
                for (int i = 0; i < MB; ++i)
                    *(float4 *)(slot0 + i * 16 * ROWF + cb * 16) = make_float4(acc[j][i][0], acc[j][i][1], acc[j][i][2], acc[j][i][3]);
            }
        }
        const int m16 = lane & 15;
        if ((lane >> 4) == (m16 >> 2)) {
            const float sv = (m16 & 3) == 0 ? sqw[0] : (m16 & 3) == 1 ? sqw[1] : (m16 & 3) == 2 ? sqw[2] : sqw[3];
#pragma unroll
            for (int i = 0; i < MB; ++i) wssq[wave * (MB * 16) + i * 16 + m16] = i == wave ? sv : 0.f;
        }
        __syncthreads();
    } else {
        const uint4 *wp[NB];
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            int nb;
            if (QKV3) nb = j < 2 ? hs * 8 + j * 4 + part : (a.nq + a.nkv) * 8 + tile;
            else if (EPI == GS_QKV_DECODE) nb = hs * 8 + (j / HH) * 4 + part * HH + (j % HH);
            else nb = min(blk0 + j, last_blk);
            wp[j] = a.Wp + (((size_t)(nb / G) * kfrags) * G + (nb % G)) * 64 + lane;
        }
        const size_t wstep = (size_t)G * 64;   // uint4 from one k-step of a block to the next

        const uint4 *xp[MB];
#pragma unroll
        for (int i = 0; i < MB; ++i) {
            if (XROWS) {   // lane -> row i * 16 + lane / 4, 16-byte piece lane % 4 of the k-step's 64 bytes
                const int row = min(i * 16 + (lane >> 2), a.M - 1);   // rows past the batch repeat the last one; never stored
                xp[i] = a.X + (size_t)row * kfrags * 4 + (lane & 3);
            } else {
                const int blk = min(i, (a.M - 1) >> 4);   // row blocks past the batch repeat the last one; never stored
                xp[i] = a.X + (size_t)blk * kfrags * 64 + lane;
            }
        }
        constexpr int XSTEP = XROWS ? 4 : 64;   // uint4 per k-step
        // XROWS: this wavefront's staging area, one 1 KiB fragment per (k-step of a set, row block), behind
        // the reduction buffers.  Row r's piece c sits at slot 4 r + (c ^ (r / 4 % 4)): the writes (lane =
        // 4 r + c) and the reads in fragment order (lane = r + 16 c) both touch every bank once per 16 lanes.
        uint4 *stage = (uint4 *)(red + gs_red_floats(MB, NB, kGsWaves)) + wave * (U * MB * 64);
        const int st_wr = ((lane >> 2) << 2) + ((lane & 3) ^ ((lane >> 4) & 3));
        const int st_rd = ((lane & 15) << 2) + ((lane >> 4) ^ (((lane & 15) >> 2) & 3));

        f32x4_t acc[NB][MB];
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int i = 0; i < MB; ++i) acc[j][i] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        f32x4_t sq[MB];   // X X^T per row block; the diagonal is the rows' sum of squares
#pragma unroll
        for (int i = 0; i < MB; ++i) sq[i] = f32x4_t{0.f, 0.f, 0.f, 0.f};

        // Two register sets of U k-steps each, rolling: while one set is multiplied the other is in
        // flight.  The loop body has no branch around a load - past the end a set re-loads the last
        // k-step (a cache hit) and is not multiplied - so that the compiler's wait counts stay exact.
        // (Starting each tile's K walk at a different offset, so that the workgroups do not ask the L2
        // for the same activation lines at the same moment, was measured: no gain.)
        uint4 w0[U][NB], x0[U][MB], w1[U][NB], x1[U][MB];
        const int n_sets = (kb_hi - kb_lo + U - 1) / U;
#define GS_LOAD(W_, X_, SET)                                                                              \
        _Pragma("unroll") for (int u = 0; u < U; ++u) {                                                       \
            const int kk = min(kb_lo + (SET) * U + u, kb_hi - 1);                                             \
            _Pragma("unroll") for (int j = 0; j < NB; ++j) W_[u][j] = ld_stream(wp[j] + (size_t)kk * wstep);  \
            _Pragma("unroll") for (int i = 0; i < MB; ++i) X_[u][i] = xp[i][(size_t)kk * XSTEP];              \
        }
#define GS_MUL(W_, X_, SET)                                                                               \
        if (XROWS) {   /* row pieces -> fragment order through the wavefront's own LDS */                     \
            _Pragma("unroll") for (int u = 0; u < U; ++u)                                                     \
                _Pragma("unroll") for (int i = 0; i < MB; ++i) stage[(u * MB + i) * 64 + st_wr] = X_[u][i];   \
            _Pragma("unroll") for (int u = 0; u < U; ++u)                                                     \
                _Pragma("unroll") for (int i = 0; i < MB; ++i) X_[u][i] = stage[(u * MB + i) * 64 + st_rd];   \
        }                                                                                                     \
        _Pragma("unroll") for (int u = 0; u < U; ++u) {                                                       \
            if (kb_lo + (SET) * U + u < kb_hi) {                                                              \
                _Pragma("unroll") for (int j = 0; j < NB; ++j)                                                 \
                    _Pragma("unroll") for (int i = 0; i < MB; ++i) acc[j][i] = gs_mfma(W_[u][j], X_[u][i], acc[j][i]); \
                if (EPI == GS_SWIGLU || EPI == GS_QKV_DECODE || norm) {                                       \
                    _Pragma("unroll") for (int i = 0; i < MB; ++i) sq[i] = gs_mfma(X_[u][i], X_[u][i], sq[i]); \
                }                                                                                             \
            }                                                                                                 \
        }
        if (n_sets > 0) {
            GS_LOAD(w0, x0, 0);
            GS_LOAD(w1, x1, 1);
            for (int s = 0; s < n_sets; s += 2) {
                GS_MUL(w0, x0, s);
                GS_LOAD(w0, x0, s + 2);
                GS_MUL(w1, x1, s + 1);
                GS_LOAD(w1, x1, s + 3);
            }
        }
#undef GS_LOAD
#undef GS_MUL

        if (XROWS) __syncthreads();   // (kept apart from the staging areas anyway; the wavefronts meet here before the epilogue)
        // In-workgroup reduction through kGsWaves / 2 LDS buffers of row-major [row][NB * 16 columns]
        // tiles: the upper half of the wavefronts write their accumulators, the lower half add them to
        // their own (w + (w + kGsWaves / 2)) and write the sums; then every thread adds the buffers in
        // index order for the outputs it stores.
        float *slot = red + (wave % HALF) * BUF + (lane & 15) * ROWF + (lane >> 4) * 4;   // + i * 16 * ROWF + j * 16
        if (wave >= HALF) {
#pragma unroll
            for (int j = 0; j < NB; ++j)
#pragma unroll
                for (int i = 0; i < MB; ++i)
                    *(float4 *)(slot + i * 16 * ROWF + j * 16) = make_float4(acc[j][i][0], acc[j][i][1], acc[j][i][2], acc[j][i][3]);
        }
        {
            // a row's sum of squares over this wavefront's part of K: element (m, m) of X X^T, which lane
            // m + 16 * (m / 4) holds in register m % 4; the wavefronts are added in index order below
            const int m16 = lane & 15;
            if ((lane >> 4) == (m16 >> 2)) {
#pragma unroll
                for (int i = 0; i < MB; ++i) {
                    const float s = (m16 & 3) == 0 ? sq[i][0] : (m16 & 3) == 1 ? sq[i][1] : (m16 & 3) == 2 ? sq[i][2] : sq[i][3];
                    wssq[wave * (MB * 16) + i * 16 + m16] = s;
                }
            }
        }
        __syncthreads();
        if (wave < HALF) {
#pragma unroll
            for (int j = 0; j < NB; ++j)
#pragma unroll
                for (int i = 0; i < MB; ++i) {
                    float4 *p = (float4 *)(slot + i * 16 * ROWF + j * 16);
                    const float4 t = *p;
                    *p = make_float4(acc[j][i][0] + t.x, acc[j][i][1] + t.y, acc[j][i][2] + t.z, acc[j][i][3] + t.w);
                }
        }
    }
    if (threadIdx.x < MB * 16) {
        const int m = threadIdx.x;
        float tot = wssq[m];
#pragma unroll
        for (int w = 1; w < kGsWaves; ++w) tot += wssq[w * (MB * 16) + m];
        rsv[m] = (norm && EPI != GS_PARTIALS) ? 1.0f / sqrtf(tot / (float)(kfrags * 32) + a.eps) : 1.0f;
        if (EPI == GS_PARTIALS && a.ssq_part && blk0 == 0 && m < a.M) a.ssq_part[seg * a.M + m] = tot;
        if (SPLIT) rsv[m] = tot;   // this segment's part of the sum of squares, published below
    }
    __syncthreads();
    constexpr int QUADS = MB * 16 * (NB * 4);   // float4 outputs of the tile
    constexpr int NBUF = SPLIT ? 1 : NRB;       // buffers `fetch` adds
    if (SPLIT) {
        // K is cut over a.nseg workgroups per tile.  Every workgroup publishes its partial tile and
        // its part of the rows' sums of squares with device-coherent (write-through) stores, waits
        // until they are performed, and bumps the tile's arrival counter; the workgroup that finds
        // nseg - 1 earlier arrivals reads all partial tiles back with device-coherent loads, adds
        // them in SEGMENT order (its own included, so the sum does not depend on who came last) and
        // runs the epilogue.  Nobody waits for anybody: there is no spinning.
        constexpr int TILEF = MB * 16 * NB * 16;
        constexpr int NT = kGsWaves * 64, QPT = (QUADS + NT - 1) / NT;
        const int nseg = a.nseg;   // 2 .. 4
        f32x4_t *mine = (f32x4_t *)(a.part + ((size_t)seg * a.ntiles + tile) * TILEF);
        for (int q = threadIdx.x; q < QUADS; q += NT) {
            const int m = q / (NB * 4), c = (q % (NB * 4)) * 4;
            float4 v = *(const float4 *)(red + m * ROWF + c);
#pragma unroll
            for (int w = 1; w < NRB; ++w) {
                const float4 t = *(const float4 *)(red + w * BUF + m * ROWF + c);
                v.x += t.x; v.y += t.y; v.z += t.z; v.w += t.w;
            }
            const f32x4_t vv = {v.x, v.y, v.z, v.w};
            asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(mine + q), "v"(vv) : "memory");
        }
        float *ssq_all = a.ssq_part + (size_t)tile * 4 * 64;   // [segment][row] of this tile
        if (norm && threadIdx.x < MB * 16)
            asm volatile("global_store_dword %0, %1, off sc1" ::"v"(ssq_all + seg * 64 + threadIdx.x), "v"(rsv[threadIdx.x]) : "memory");
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the stores above are performed device-wide
        __syncthreads();
        int *arrived = (int *)(rsv + MB * 16);
        if (threadIdx.x == 0) *arrived = __hip_atomic_fetch_add(a.cnt + tile, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        if (*arrived != nseg - 1) return;   // the same for the whole workgroup
        // All loads are issued before the one wait (straight-line code: a register with a load in
        // flight must not reach a control-flow join, where the compiler may copy it).  Segments past
        // nseg repeat the last one and are not added.
        f32x4_t r[QPT][4];
#pragma unroll
        for (int t = 0; t < QPT; ++t) {
            const int q = min((int)threadIdx.x + t * NT, QUADS - 1);
#pragma unroll
            for (int sg = 0; sg < 4; ++sg) {
                const f32x4_t *src = (const f32x4_t *)(a.part + ((size_t)min(sg, nseg - 1) * a.ntiles + tile) * TILEF) + q;
                asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(r[t][sg]) : "v"(src) : "memory");
            }
        }
#pragma unroll
        for (int t = 0; t < QPT; ++t)
            asm volatile("s_waitcnt vmcnt(0)" : "+v"(r[t][0]), "+v"(r[t][1]), "+v"(r[t][2]), "+v"(r[t][3])::"memory");
#pragma unroll
        for (int t = 0; t < QPT; ++t) {
            const int q = threadIdx.x + t * NT;
            f32x4_t v = r[t][0] + r[t][1];
            if (nseg > 2) v += r[t][2];
            if (nseg > 3) v += r[t][3];
            if (q < QUADS) *(float4 *)(red + (q / (NB * 4)) * ROWF + (q % (NB * 4)) * 4) = make_float4(v[0], v[1], v[2], v[3]);
        }
        if (norm) {   // the rows' sums of squares, the same way (one more round trip; only projections with the norm in front)
            float sv[4];
#pragma unroll
            for (int sg = 0; sg < 4; ++sg) {
                const float *sp = ssq_all + min(sg, nseg - 1) * 64 + (threadIdx.x & 63);
                asm volatile("global_load_dword %0, %1, off sc1" : "=v"(sv[sg]) : "v"(sp) : "memory");
            }
            asm volatile("s_waitcnt vmcnt(0)" : "+v"(sv[0]), "+v"(sv[1]), "+v"(sv[2]), "+v"(sv[3])::"memory");
            float tot = sv[0] + sv[1];
            if (nseg > 2) tot += sv[2];
            if (nseg > 3) tot += sv[3];
            if (threadIdx.x < MB * 16) rsv[threadIdx.x] = 1.0f / sqrtf(tot / (float)(kfrags * 32) + a.eps);
        } else if (threadIdx.x < MB * 16) {
            rsv[threadIdx.x] = 1.0f;
        }
        if (threadIdx.x == 0) __hip_atomic_store(a.cnt + tile, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next launch
        __syncthreads();
    }
    // value of the tile at (row m, column c of NB * 16), scaled by the row's norm factor
    auto fetch = [&](int m, int c) -> float4 {
        float4 v = *(const float4 *)(red + m * ROWF + c);
#pragma unroll
        for (int w = 1; w < NBUF; ++w) {
            const float4 t = *(const float4 *)(red + w * BUF + m * ROWF + c);
            v.x += t.x; v.y += t.y; v.z += t.z; v.w += t.w;
        }
        const float r = rsv[m];
        v.x *= r; v.y *= r; v.z *= r; v.w *= r;
        return v;
    };
    if (EPI == GS_PARTIALS) {
        for (int q = threadIdx.x; q < QUADS; q += kGsWaves * 64) {
            const int m = q / (NB * 4), c = (q % (NB * 4)) * 4;
            const int n = blk0 * 16 + c;
            if (m < a.M && n < a.N) *(float4 *)(a.part + ((size_t)seg * a.M + m) * a.N + n) = fetch(m, c);
        }
    } else if (EPI == GS_STORE) {
        for (int q = threadIdx.x; q < QUADS; q += kGsWaves * 64) {
            const int m = q / (NB * 4), c = (q % (NB * 4)) * 4;
            const int n = blk0 * 16 + c;
            if (m >= a.M || n >= a.N || c >= nbt * 16) continue;
            float4 v = fetch(m, c);
            if (a.res) {
                const uint2 r = *(const uint2 *)(a.res + (size_t)m * a.N + n);
                v.x += bf_lo(r.x); v.y += bf_hi(r.x); v.z += bf_lo(r.y); v.w += bf_hi(r.y);
            }
            const uint2 o = make_uint2(pack2bf(v.x, v.y), pack2bf(v.z, v.w));
            *(uint2 *)(a.out + (size_t)m * a.N + n) = o;
            if (a.out_packed) *(uint2 *)(a.out_packed + packed_index(m, n, a.N >> 5)) = o;
        }
    } else if (EPI == GS_SWIGLU) {   // the tile's blocks are (gate, up) pairs: NB / 2 blocks of u
        for (int q = threadIdx.x; q < QUADS / 2; q += kGsWaves * 64) {
            const int m = q / (NB * 2), pr = (q % (NB * 2)) / 4, c4 = (q % 4) * 4;
            const int col = (blk0 / 2 + pr) * 16 + c4;   // column of u
            if (m >= a.M || col >= a.N / 2 || pr * 2 >= nbt) continue;
            const float4 g = fetch(m, pr * 32 + c4), u = fetch(m, pr * 32 + 16 + c4);
            const float o0 = g.x / (1.0f + __expf(-g.x)) * u.x, o1 = g.y / (1.0f + __expf(-g.y)) * u.y;
            const float o2 = g.z / (1.0f + __expf(-g.z)) * u.z, o3 = g.w / (1.0f + __expf(-g.w)) * u.w;
            *(uint2 *)(a.out + packed_index(m, col, (a.N / 2) >> 5)) = make_uint2(pack2bf(o0, o1), pack2bf(o2, o3));
        }
    } else if (QKV3) {   // columns [0, 16): dims d0 + c of a q or k head, [16, 32): their rotary partners 64 up, [32, 48): 16 dims of a v head
        const int width = (a.nq + 2 * a.nkv) * 128;
        const int d0 = part * 16;
        for (int q = threadIdx.x; q < MB * 16 * 8; q += kGsWaves * 64) {
            const int m = q >> 3, e4 = q & 7;
            if (m >= a.M) continue;
            const int pos = cached_len(a.lens, m, a.cap);
            if (e4 < 4) {   // the rotary pair
                const int c = e4 * 4;
                const float4 lo4 = fetch(m, c), hi4 = fetch(m, c + 16);
                float l[4] = {lo4.x, lo4.y, lo4.z, lo4.w}, h[4] = {hi4.x, hi4.y, hi4.z, hi4.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float cs, sn;
                    rope_cs(a.tab, d0 + c + e, pos, cs, sn);
                    const float x0v = l[e], x1v = h[e];
                    l[e] = x0v * cs - x1v * sn;
                    h[e] = x1v * cs + x0v * sn;
                }
                bf16_t *dst = hs < a.nq ? a.out + (size_t)m * width + hs * 128 + d0 + c
                                        : a.kc + (((size_t)m * a.nkv + (hs - a.nq)) * a.cap + pos) * 128 + d0 + c;
                *(uint2 *)dst = make_uint2(pack2bf(l[0], l[1]), pack2bf(l[2], l[3]));
                *(uint2 *)(dst + 64) = make_uint2(pack2bf(h[0], h[1]), pack2bf(h[2], h[3]));
            } else {        // the v block: block tile % 8 of v head tile / 8
                const int c = (e4 - 4) * 4;
                const float4 v = fetch(m, 32 + c);
                bf16_t *dst = a.vc + (((size_t)m * a.nkv + (tile >> 3)) * a.cap + pos) * 128 + (tile & 7) * 16 + c;
                *(uint2 *)dst = make_uint2(pack2bf(v.x, v.y), pack2bf(v.z, v.w));
            }
        }
    } else {   // GS_QKV_DECODE: columns [0, NB * 8) are dims d0 + c, columns [NB * 8, NB * 16) their rotary partners 64 up
        const int width = (a.nq + 2 * a.nkv) * 128;
        const int d0 = part * (NB * 8);
        for (int q = threadIdx.x; q < QUADS / 2; q += kGsWaves * 64) {
            const int m = q / (NB * 2), c = (q % (NB * 2)) * 4;
            if (m >= a.M) continue;
            const float4 lo4 = fetch(m, c), hi4 = fetch(m, c + NB * 8);
            float l[4] = {lo4.x, lo4.y, lo4.z, lo4.w}, h[4] = {hi4.x, hi4.y, hi4.z, hi4.w};
            const int pos = cached_len(a.lens, m, a.cap);
            const int dim = d0 + c;
            if (hs < a.nq + a.nkv) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float cs, sn;
                    rope_cs(a.tab, dim + e, pos, cs, sn);
                    const float x0v = l[e], x1v = h[e];
                    l[e] = x0v * cs - x1v * sn;
                    h[e] = x1v * cs + x0v * sn;
                }
            }
            const uint2 plo = make_uint2(pack2bf(l[0], l[1]), pack2bf(l[2], l[3]));
            const uint2 phi = make_uint2(pack2bf(h[0], h[1]), pack2bf(h[2], h[3]));
            bf16_t *dst;
            if (hs < a.nq) dst = a.out + (size_t)m * width + hs * 128 + dim;
            else if (hs < a.nq + a.nkv) dst = a.kc + (((size_t)m * a.nkv + (hs - a.nq)) * a.cap + pos) * 128 + dim;
            else dst = a.vc + (((size_t)m * a.nkv + (hs - a.nq - a.nkv)) * a.cap + pos) * 128 + dim;
            *(uint2 *)dst = plo;
            *(uint2 *)(dst + 64) = phi;
        }
    }
}

// The kernel: workgroup b works on column tile b % ntiles and K segment b / ntiles.  With NB2 > 0 a
// tile is NB + NB2 blocks wide and is done in two passes (NB blocks, then NB2), which lets a launch
// give every compute unit the same number of blocks when that number is too large for one pass's registers.
template <int MB, int NB, int EPI, int kGsWaves, int U, int XROWS, int NB2, int SPLIT, int COLS>
__global__ __launch_bounds__(kGsWaves * 64, (MB * NB <= 8 && kGsWaves == 4) ? 2 : 1) void gemm_stream_kernel(const GsArgs a)
{
    extern __shared__ float red[];
    const int tile = blockIdx.x % a.ntiles, seg = blockIdx.x / a.ntiles;
    if constexpr (COLS) {
        gs_pass<MB, NB, EPI, kGsWaves, U, XROWS, SPLIT, 1>(a, red, tile * a.nbt, tile, seg);
    } else {
        gs_pass<MB, NB, EPI, kGsWaves, U, XROWS, SPLIT>(a, red, tile * (NB + NB2), tile, seg);
        if (NB2 > 0) {
            constexpr int NBB = NB2 > 0 ? NB2 : 1;
            if ((tile * (NB + NB2) + NB) * 16 < a.N) {   // the same for the whole workgroup
                __syncthreads();
                gs_pass<MB, NBB, EPI, kGsWaves, gs_u(MB, NBB), XROWS, 0>(a, red, tile * (NB + NB2) + NB, tile, seg);
            }
        }
    }
}

constexpr int gs_lds_bytes(int MB, int NB, int W, int U, int XROWS)
{
    return gs_red_floats(MB, NB, W) * (int)sizeof(float) + (XROWS ? W * U * MB * 1024 : 0);
}
constexpr int gs_lds_bytes2(int MB, int NB, int NB2, int W, int XROWS)
{
    const int a = gs_lds_bytes(MB, NB, W, gs_u(MB, NB), XROWS);
    const int b = NB2 > 0 ? gs_lds_bytes(MB, NB2, W, gs_u(MB, NB2), XROWS) : 0;
    return a > b ? a : b;
}
// column-split form: one tile buffer, two stages of U k-steps of all MB row blocks
constexpr int kGsColsU = 4;   // k-steps per set: 16 KiB of weights per wavefront and set with 16-block tiles
constexpr int gs_lds_bytes_cols(int MB, int NB, int W) { return gs_red_floats(MB, NB, W, 1) * (int)sizeof(float) + 2 * kGsColsU * MB * 1024; }

// wavefronts per workgroup of every instantiation (eight were measured: never faster)
constexpr int kGsW = 4;

template <int MB, int NB, int EPI, int XROWS, int NB2 = 0, int SPLIT = 0>
hipError_t gs_launch(int grid, const GsArgs &a, hipStream_t st)
{
    hipLaunchKernelGGL((gemm_stream_kernel<MB, NB, EPI, kGsW, gs_u(MB, NB), XROWS, NB2, SPLIT, 0>), dim3(grid), dim3(kGsW * 64),
                       gs_lds_bytes2(MB, NB, NB2, kGsW, XROWS), st, a);
    return hipGetLastError();
}

// column-split form (64-row launches with wide tiles)
template <int NB, int EPI, int SPLIT>
hipError_t gs_launch_cols(int grid, const GsArgs &a, hipStream_t st)
{
    hipLaunchKernelGGL((gemm_stream_kernel<4, NB, EPI, kGsW, kGsColsU, 0, 0, SPLIT, 1>), dim3(grid), dim3(kGsW * 64),
                       gs_lds_bytes_cols(4, NB, kGsW), st, a);
    return hipGetLastError();
}
template <int NB, int EPI, int SPLIT>
hipError_t gs_attr_cols()
{
    return hipFuncSetAttribute((const void *)gemm_stream_kernel<4, NB, EPI, kGsW, kGsColsU, 0, 0, SPLIT, 1>,
                               hipFuncAttributeMaxDynamicSharedMemorySize, gs_lds_bytes_cols(4, NB, kGsW));
}

template <int NB, int EPI, int XROWS, int NB2 = 0, int SPLIT = 0>
hipError_t gs_launch_mb(int grid, const GsArgs &a, hipStream_t st)
{
    const int mb = (a.M + 15) / 16;
    if (mb <= 1) return gs_launch<1, NB, EPI, XROWS, NB2, SPLIT>(grid, a, st);
    if (mb == 2) return gs_launch<2, NB, EPI, XROWS, NB2, SPLIT>(grid, a, st);
    return gs_launch<4, NB, EPI, XROWS, NB2, SPLIT>(grid, a, st);
}

template <int MB, int NB, int EPI, int XROWS, int NB2, int SPLIT>
hipError_t gs_attr()
{
    return hipFuncSetAttribute((const void *)gemm_stream_kernel<MB, NB, EPI, kGsW, gs_u(MB, NB), XROWS, NB2, SPLIT, 0>,
                               hipFuncAttributeMaxDynamicSharedMemorySize, gs_lds_bytes2(MB, NB, NB2, kGsW, XROWS));
}
template <int NB, int EPI, int NB2 = 0, int SPLIT = 0>
hipError_t gs_attr_mb()
{
    hipError_t e = gs_attr<1, NB, EPI, 0, NB2, SPLIT>();
    if (e == hipSuccess) e = gs_attr<2, NB, EPI, 0, NB2, SPLIT>();
    if (e == hipSuccess) e = gs_attr<4, NB, EPI, 0, NB2, SPLIT>();
    if (e == hipSuccess) e = gs_attr<1, NB, EPI, 1, NB2, SPLIT>();
    if (e == hipSuccess) e = gs_attr<2, NB, EPI, 1, NB2, SPLIT>();
    if (e == hipSuccess) e = gs_attr<4, NB, EPI, 1, NB2, SPLIT>();
    return e;
}

}  // namespace

// Shape of a store-type projection [N, K] for a batch of `variant_rows` rows (of the FULL batch).
// Unsplit: tiles of the widest of 8, 4, 2, 1 blocks that still gives about one workgroup per
// compute unit.  Narrow tiles re-read the activations once per tile, which is what bounds them when
// the batch has more than 16 rows; so when K is long enough to leave every wavefront at least 20
// k-steps, tiles of 8, 4 or 2 blocks with K cut over 2..4 workgroups (about 256 workgroups again)
// and the sum taken inside the launch are faster (measured, 32 rows: 4096 x 11008 20.2 against
// 23.8 us; 64 rows: 8192 x 8192 28.9 against 31.7 us; 4096 x 4096 gains nothing).
StoreShape stream_store_shape(int N, int K, long variant_rows)
{
    const int nblk = (N + 15) / 16, kfrags = K / 32;
    StoreShape sh{1, 1};
    for (int nb = 8; nb > 1; nb >>= 1)
        if (nblk / nb >= 192) { sh.nb = nb; break; }
    if (variant_rows > 16) {
        for (int nb = 8; nb >= 2; nb >>= 1) {
            const int tiles = (nblk + nb - 1) / nb;
            int S = 256 / tiles;
            if (S > 4) S = 4;
            if (S < 2 || tiles * S < 192 || kfrags / (4 * S) < 20) continue;
            sh.nb = nb;
            sh.nseg = S;
            break;
        }
    }
    return sh;
}

static int mb_of(int rows) { const int mb = (rows + 15) / 16; return mb <= 1 ? 1 : mb == 2 ? 2 : 4; }

// fp32 partial tiles of a split store-type projection (0 when it is not split)
size_t stream_store_partial_bytes(int N, int K, long variant_rows, int rows)
{
    const StoreShape sh = stream_store_shape(N, K, variant_rows);
    if (sh.nseg < 2) return 0;
    const size_t tiles = ((N + 15) / 16 + sh.nb - 1) / sh.nb;
    return (size_t)sh.nseg * tiles * mb_of(rows) * 16 * sh.nb * 16 * sizeof(float);
}

// Blocks a compute unit ends up with when `tiles` tiles of `nb` blocks are dealt to 256 of them.
static int blocks_per_cu(int tiles, int nb) { return ((tiles + 255) / 256) * nb; }

// The decode Q/K/V projection works on whole rotary pairs: whole heads (8 blocks), half heads (4), or -
// when there are as many q + k rotary pairs of blocks as v blocks, i.e. n_q == n_kv - one pair with one
// v block (3).  The choice that leaves the fewest blocks on the busiest compute unit wins, the wider
// tile on a tie (a 32-head module: 256 tiles of 3 blocks instead of 192 of 4).
static int stream_qkv_nb(int nq, int nkv)
{
    const int heads = nq + 2 * nkv;
    int best = 8, cost = blocks_per_cu(heads, 8);
    if (blocks_per_cu(heads * 2, 4) < cost) { best = 4; cost = blocks_per_cu(heads * 2, 4); }
    if (nq == nkv && blocks_per_cu(nkv * 8, 3) < cost) best = 3;
    return best;
}

// Gate/up: (gate, up) pairs of blocks per workgroup so that 256 workgroups cover the weight; up to 4
// pairs are one pass, 5 and 7 are two passes (6 + 4, 8 + 6 blocks), anything else tiles of 3 or 4 pairs.
static void stream_gu_shape(int N2, int *nb1, int *nb2)
{
    const int pairs = N2 / 32, c = (pairs + 255) / 256;
    *nb2 = 0;
    if (c <= 4) *nb1 = 2 * c;
    else if (c == 5) { *nb1 = 6; *nb2 = 4; }
    else if (c == 6) *nb1 = 6;
    else if (c == 7) { *nb1 = 8; *nb2 = 6; }
    else *nb1 = 8;
}

hipError_t launch_gemm_stream_store(const void *Wp, StoreShape sh, const void *X, bool x_rows, bool norm, float eps,
                                    const void *res, void *out, void *out_packed, int M, int N, int K, float *partials,
                                    int *counters, hipStream_t st)
{
    if (M <= 0) return hipSuccess;
    if (M > kSkinnyMaxRows || (K & 31) || (N & 15)) return hipErrorInvalidValue;
    const int nb = sh.nb;
    if (nb != 1 && nb != 2 && nb != 4 && nb != 8) return hipErrorInvalidValue;
    GsArgs a{};
    a.Wp = (const uint4 *)Wp; a.kfrags = K / 32; a.G = kWGroup; a.X = (const uint4 *)X; a.norm = norm ? 1 : 0; a.eps = eps;
    a.M = M; a.N = N; a.res = (const bf16_t *)res; a.out = (bf16_t *)out; a.out_packed = (bf16_t *)out_packed;
    const int tiles = ((N / 16) + nb - 1) / nb;
    a.ntiles = tiles; a.kf_seg = a.kfrags;
    if (sh.nseg > 1) {
        // K over nseg workgroups per tile, summed inside the launch; only without the norm (no per-segment sums of squares here)
        if (sh.nseg > 4 || norm || !partials || !counters || tiles > kStreamCounters || nb < 2) return hipErrorInvalidValue;
        a.nseg = sh.nseg; a.kf_seg = (a.kfrags + sh.nseg - 1) / sh.nseg;
        if (a.kf_seg * (sh.nseg - 1) >= a.kfrags) return hipErrorInvalidValue;   // no empty segment
        a.part = partials; a.cnt = counters;
        const int grid = tiles * sh.nseg;
#define CCS_GS(NBV) (x_rows ? gs_launch_mb<NBV, GS_STORE, 1, 0, 1>(grid, a, st) : gs_launch_mb<NBV, GS_STORE, 0, 0, 1>(grid, a, st))
        switch (nb) {
            case 2: return CCS_GS(2);
            case 4: return CCS_GS(4);
            default: return CCS_GS(8);
        }
#undef CCS_GS
    }
#define CCS_GS(NBV) (x_rows ? gs_launch_mb<NBV, GS_STORE, 1>(tiles, a, st) : gs_launch_mb<NBV, GS_STORE, 0>(tiles, a, st))
    switch (nb) {
        case 1: return CCS_GS(1);
        case 2: return CCS_GS(2);
        case 4: return CCS_GS(4);
        default: return CCS_GS(8);
    }
#undef CCS_GS
}

// gate/up takes the column-split form when the FULL batch has 33..64 rows, the activations are packed and a
// workgroup gets five to eight (gate, up) pairs
static bool stream_gu_cols(int N2, long variant_rows, bool x_rows)
{
    const int per_wg = (N2 / 32 + 255) / 256;
    return variant_rows > 32 && !x_rows && per_wg >= 5 && per_wg <= 8;
}

hipError_t launch_gemm_stream_swiglu(const void *Wp, const void *X, bool x_rows, float eps, void *u_packed, int M, int N2,
                                     int K, long variant_rows, hipStream_t st)
{
    if (M <= 0) return hipSuccess;
    if (M > kSkinnyMaxRows || (K & 31) || (N2 & 31)) return hipErrorInvalidValue;
    GsArgs a{};
    a.Wp = (const uint4 *)Wp; a.kfrags = K / 32; a.G = kWGroup; a.X = (const uint4 *)X; a.norm = 1; a.eps = eps;
    a.M = M; a.N = N2; a.out = (bf16_t *)u_packed;
    const int pairs = N2 / 32, per_wg = (pairs + 255) / 256;
    if (stream_gu_cols(N2, variant_rows, x_rows)) {
        // 33..64 rows in the full batch: one pass over all of a workgroup's pairs in the column-split form (two passes
        // would fetch the activations twice)
        a.nbt = 2 * per_wg;
        a.ntiles = (pairs + per_wg - 1) / per_wg; a.kf_seg = a.kfrags;
        return gs_launch_cols<16, GS_SWIGLU, 0>(a.ntiles, a, st);
    }
    int nb1, nb2;
    stream_gu_shape(N2, &nb1, &nb2);
    const int tiles = ((N2 / 16) + nb1 + nb2 - 1) / (nb1 + nb2);
    a.ntiles = tiles; a.kf_seg = a.kfrags;
#define CCS_GS(NB1, NB2) (x_rows ? gs_launch_mb<NB1, GS_SWIGLU, 1, NB2>(tiles, a, st) : gs_launch_mb<NB1, GS_SWIGLU, 0, NB2>(tiles, a, st))
    if (nb2 == 4) return CCS_GS(6, 4);
    if (nb2 == 6) return CCS_GS(8, 6);
    switch (nb1) {
        case 2: return CCS_GS(2, 0);
        case 4: return CCS_GS(4, 0);
        case 6: return CCS_GS(6, 0);
        default: return CCS_GS(8, 0);
    }
#undef CCS_GS
}

hipError_t launch_gemm_stream_qkv_decode(const void *Wp, const void *X, bool x_rows, float eps, void *qkv, int M, int nq,
                                         int nkv, int K, const void *tab, const int32_t *lens_dev, void *k_cache,
                                         void *v_cache, int cap, hipStream_t st)
{
    if (M <= 0) return hipSuccess;
    if (M > kSkinnyMaxRows || (K & 31)) return hipErrorInvalidValue;
    GsArgs a{};
    a.Wp = (const uint4 *)Wp; a.kfrags = K / 32; a.G = kWGroup; a.X = (const uint4 *)X; a.norm = 1; a.eps = eps;
    a.M = M; a.N = (nq + 2 * nkv) * 128; a.out = (bf16_t *)qkv;
    a.nq = nq; a.nkv = nkv; a.tab = (const float2 *)tab; a.lens = lens_dev; a.kc = (bf16_t *)k_cache; a.vc = (bf16_t *)v_cache;
    a.cap = cap;
    const int heads = nq + 2 * nkv;
    a.kf_seg = a.kfrags;
#define CCS_GS(NBV) (x_rows ? gs_launch_mb<NBV, GS_QKV_DECODE, 1>(a.ntiles, a, st) : gs_launch_mb<NBV, GS_QKV_DECODE, 0>(a.ntiles, a, st))
    switch (stream_qkv_nb(nq, nkv)) {
        case 8: a.ntiles = heads; return CCS_GS(8);
        case 4: a.ntiles = heads * 2; return CCS_GS(4);
        default: a.ntiles = nkv * 8; return CCS_GS(3);
    }
#undef CCS_GS
}

// K segments of the GS_PARTIALS form for a [N, K] weight: from the weight shape alone.  Measured sweeps
// (32 and 64 rows, 33 MB to 940 MB weights): about one workgroup per compute unit with long streams
// beats more, shorter ones, so K is cut into floor(256 / tiles) segments of at least 32 k-steps.
int skinny_segments(int N, int K)
{
    const int kfrags = K / 32, tiles = ((N + 15) / 16 + 7) / 8;
    int S = 256 / tiles;
    const int max_s = kfrags / 32;
    if (S > max_s) S = max_s;
    if (S > 64) S = 64;
    if (S < 1) S = 1;
    const int per = (kfrags + S - 1) / S;
    return (kfrags + per - 1) / per;
}

size_t skinny_partial_bytes(int M, int N, int K)
{
    return (size_t)skinny_segments(N, K) * (size_t)M * (size_t)N * sizeof(float);
}

hipError_t launch_gemm_stream_partials(const void *Wp, const void *X, bool x_rows, bool norm, float *partials,
                                       float *ssq_partials, int M, int N, int K, hipStream_t st)
{
    if (M <= 0) return hipSuccess;
    if (M > kSkinnyMaxRows || (K & 31) || (N & 15)) return hipErrorInvalidValue;
    GsArgs a{};
    a.Wp = (const uint4 *)Wp; a.kfrags = K / 32; a.G = kWGroup; a.X = (const uint4 *)X; a.norm = norm ? 1 : 0;
    a.M = M; a.N = N; a.part = partials; a.ssq_part = norm ? ssq_partials : nullptr;
    const int S = skinny_segments(N, K);
    a.ntiles = ((N / 16) + 7) / 8;
    a.kf_seg = (a.kfrags + S - 1) / S;
    const int grid = a.ntiles * S;
    return x_rows ? gs_launch_mb<8, GS_PARTIALS, 1>(grid, a, st) : gs_launch_mb<8, GS_PARTIALS, 0>(grid, a, st);
}

hipError_t init_gemm_stream_kernels()
{
    hipError_t e = gs_attr_mb<1, GS_STORE>();
    if (e == hipSuccess) e = gs_attr_mb<2, GS_STORE>();
    if (e == hipSuccess) e = gs_attr_mb<4, GS_STORE>();
    if (e == hipSuccess) e = gs_attr_mb<8, GS_STORE>();
    if (e == hipSuccess) e = gs_attr_mb<2, GS_STORE, 0, 1>();
    if (e == hipSuccess) e = gs_attr_mb<4, GS_STORE, 0, 1>();
    if (e == hipSuccess) e = gs_attr_mb<8, GS_STORE, 0, 1>();
    if (e == hipSuccess) e = gs_attr_mb<2, GS_SWIGLU>();
    if (e == hipSuccess) e = gs_attr_mb<4, GS_SWIGLU>();
    if (e == hipSuccess) e = gs_attr_mb<6, GS_SWIGLU>();
    if (e == hipSuccess) e = gs_attr_mb<8, GS_SWIGLU>();
    if (e == hipSuccess) e = gs_attr_mb<6, GS_SWIGLU, 4>();
    if (e == hipSuccess) e = gs_attr_mb<8, GS_SWIGLU, 6>();
    if (e == hipSuccess) e = gs_attr_mb<8, GS_PARTIALS>();
    if (e == hipSuccess) e = gs_attr_mb<8, GS_QKV_DECODE>();
    if (e == hipSuccess) e = gs_attr_mb<4, GS_QKV_DECODE>();
    if (e == hipSuccess) e = gs_attr_mb<3, GS_QKV_DECODE>();
    if (e == hipSuccess) e = gs_attr_cols<16, GS_SWIGLU, 0>();
    return e;
}

}  // namespace ccs
