// Host-side launchers of the gfx950 kernels.  Every launcher only enqueues on `st` and
// returns the launch status; shapes are validated by the caller (ccs_module.cpp).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace ccs {

enum { DT_F32 = 0, DT_BF16 = 1 };

// One-time function attributes (dynamic LDS sizes); not capturable, so not part of a forward.
hipError_t init_gemm_kernels();
hipError_t init_attention_kernels();

// ---- streaming / elementwise (ccs_elementwise.hip) -----------------------------------------
// dst[0:bytes) = src[0:bytes), both 16-byte aligned, device memory, no overlap.
hipError_t launch_clone(void *dst, const void *src, size_t bytes, hipStream_t st);
// Row-major bf16 [N, K] -> fragment-packed rows; 16-row block nb of the source lands at packed
// block nb * blk_stride + blk_offset of a packed matrix with K/32 fragments per block row.
// `grouped`: weight order (groups of 8 blocks, see ccs_common.h); the caller zeroes the padding.
// `gain` (bf16 [K], may be null): every row is multiplied element-wise by it on the way (rounded to
// bf16) - how the gains of the RMSNorm in front of a projection are folded into its weight.
hipError_t launch_pack_bf16(const void *src, void *dst_packed, int N, int K, int blk_stride,
                            int blk_offset, bool grouped, const void *gain, hipStream_t st);
// out[t,:] = x[t,:] * rsqrt(mean(x[t,:]^2) + eps) * g.  x row-major [rows, H].
// bf16: out is fragment-packed [rows16, H] and g may be null (gains folded into the next weight);
// f32: out row-major.
hipError_t launch_rmsnorm(int dtype, const void *x, const void *g, void *out, int rows, int H,
                          float eps, hipStream_t st);
// Inverse-frequency table of the rotary embedding, d/2 float2 entries (fp32 head and tail of
// base^(-2i/d)); part of the weight arena.  All rope kernels take it as `tab`.
hipError_t launch_rope_table(void *tab, int d, float base, hipStream_t st);
// Rotary embedding (split-half pairs) in place on the q and k parts of qkv [rows, (nq+2nkv)*d]
// row-major.  prefill (decode == 0): position = row % seq_pad; when caches are non-null the
// rotated k and v of rows with position < lens[row / seq_pad] are stored at slot = position.
// decode: position = lens[row]; rotated k and v stored at slot lens[row] of sequence `row`.
hipError_t launch_rope(int dtype, void *qkv, int rows, int nq, int nkv, int d, const void *tab,
                       int decode, int seq_pad, const int32_t *lens_dev, void *k_cache,
                       void *v_cache, int cap, hipStream_t st);
// bf16 prefill without padding: offs[b] = valid rows before sequence b (n_seqs + 1 entries), from
// the device copy of the lengths clamped into [0, seq_pad] and capped at `total` (the dense row
// count the host planned for); the kernels below take len_b = offs[b + 1] - offs[b].
// launch_prefill_rows moves the valid rows of a padded [n_seqs, seq_pad, H] batch into a dense
// [offs[n_seqs], H] matrix (expand = false) or back, writing the padded rows as zeros (expand = true).
hipError_t launch_prefill_offsets(const int32_t *lens_dev, int n_seqs, int seq_pad, int total, int32_t *offs,
                                  hipStream_t st);
hipError_t launch_prefill_rows(void *padded, void *dense, const int32_t *offs, int n_seqs, int seq_pad, int H,
                               bool expand, hipStream_t st);
// bf16 prefill with head_dim 128 on dense rows (sequence b = rows offs[b] .. offs[b] + len_b - 1 of
// qkv): rotate q in place and emit K (fragment-packed per kv head) and V (transposed, in the key
// order of the MFMA prefill-attention kernel) into kp / vtp, each n_seqs * nkv * S32 * 128
// elements, S32 = seq_pad rounded up to 32, for the 32-key blocks that hold a valid key (keys
// past len_b inside the last block are written as zeros); optional row-major caches.
hipError_t launch_rope_pack_prefill(void *qkv, void *kp, void *vtp, int n_seqs, int seq_pad, int nq, int nkv,
                                    const void *tab, const int32_t *offs, void *k_cache, void *v_cache, int cap,
                                    hipStream_t st);
// f32 path: u[t,j] = silu(gu[t,j]) * gu[t, I + j], gu row-major [rows, 2I].
hipError_t launch_swiglu_f32(const float *gu, float *u, int rows, int I, hipStream_t st);

// ---- GEMMs (ccs_gemm.hip) ------------------------------------------------------------------
// f32: y[m,n] = sum_k x[m,k] W[n,k] (+ res[m,n]); everything row-major.
hipError_t launch_gemm_f32(const float *x, const float *W, const float *res, float *y, int M,
                           int N, int K, hipStream_t st);

enum GemmEpilogue {
    EPI_STORE_RM = 0,   // y row-major bf16 [M, N], optional residual (row-major bf16 [M, N])
    EPI_SWIGLU_PACKED = 1  // N = 2I with gate/up interleaved in 16-row blocks; u fragment-packed [M16, I]
};
// Largest row count the weight-streaming variants accept in one launch.
constexpr int kSkinnyMaxRows = 64;
// The same with a K split, for the projections whose one-launch form is slower (33..64 rows against
// a large weight): 128-column tiles, K cut into skinny_segments(N, K) segments (a function of the
// weight shape only), fp32 partial sums [S, M, N] into `partials` and, with `norm`, the rows' sums of
// squares per segment [S, M] into `ssq_partials`; the caller follows with launch_partial_reduce or
// launch_qkv_partials_rope_decode.
int skinny_segments(int N, int K);
size_t skinny_partial_bytes(int M, int N, int K);
hipError_t launch_gemm_stream_partials(const void *Wp, const void *X, bool x_rows, bool norm, float *partials,
                                       float *ssq_partials, int M, int N, int K, hipStream_t st);
// Decode Q/K/V (head_dim 128) behind a K-split projection of raw rows: segment sums in segment order,
// the RMSNorm scale rsqrt(sum_s ssq[s, m] / K + eps), rotary embedding at position lens[m], q store
// and KV-cache append at slot lens[m].
hipError_t launch_qkv_partials_rope_decode(const float *partials, const float *ssq_partials, int S, int M, int nq,
                                           int nkv, int K, float eps, const void *tab, const int32_t *lens_dev,
                                           void *qkv, void *k_cache, void *v_cache, int cap, hipStream_t st);
// Fixed-order sum of S partial buffers (fp32 [S, M, N]) + epilogue; used by both GEMM variants.
// EPI_STORE_RM: out_packed (may be null) receives a second, fragment-packed copy of the result.
hipError_t launch_partial_reduce(const float *partials, int S, int epi, const void *res, void *out, void *out_packed,
                                 int M, int N, hipStream_t st);
// bf16 LDS-tiled MFMA GEMM for any M (Xp fragment-packed and readable up to M rounded up to 16 rows,
// or, with x_rows, the plain row-major bf16 rows [M, K]).  When the batch
// is too small to fill the GPU, K is cut into tiled_segments(N, K, variant_rows) segments whose
// partial sums go through `partials` (tiled_partial_bytes) and launch_partial_reduce;
// variant_rows is the row count of the full batch the launch belongs to.
int tiled_segments(int N, int K, long variant_rows);
size_t tiled_partial_bytes(int M, int N, int K, long variant_rows);
hipError_t launch_gemm_tiled(const void *Wp, const void *Xp, bool x_rows, int epi, const void *res, void *out,
                             int M, int N, int K, long variant_rows, float *partials, hipStream_t st);

// ---- weight-streaming projections, one launch each (ccs_gemm_stream.hip) -----------------------
// For M <= kSkinnyMaxRows rows.  Weights are fragment-packed in groups of kWGroup 16-row blocks
// (ccs_common.h), x is fragment-packed [M16, K] or (x_rows) plain row-major bf16 rows [M, K], which
// the kernel turns into fragments itself.  With `norm` x holds the raw rows of the residual
// stream and the kernel is also the RMSNorm in front of the projection (the weight already carries
// the norm's gains): row m of the result is scaled by rsqrt(mean_k x[m, k]^2 + eps).  A row's
// result depends on that row alone.
enum { GS_STORE = 0, GS_SWIGLU = 1, GS_QKV_DECODE = 2, GS_PARTIALS = 3 };
hipError_t init_gemm_stream_kernels();
// Shape of a store-type projection [N, K] for a batch of `variant_rows` rows (the FULL batch's count):
// tiles of nb 16-column blocks (1, 2, 4 or 8) and, when nseg > 1, K cut over nseg workgroups per
// tile whose partial tiles the last of them to finish adds in segment order inside the launch.
struct StoreShape { int nb, nseg; };
StoreShape stream_store_shape(int N, int K, long variant_rows);
// bytes of fp32 partial tiles a split launch of `rows` rows needs (0 when the shape is not split)
size_t stream_store_partial_bytes(int N, int K, long variant_rows, int rows);
constexpr int kStreamCounters = 256;   // arrival counters (int32) a split launch may use; all zero between launches
// out[m, n] = sum_k x'[m, k] W[n, k] (+ res[m, n]) as row-major bf16 [M, N] and, when out_packed
// is not null, also fragment-packed [M16, N] (the operand of the next projection).  A split shape
// needs `partials` (stream_store_partial_bytes) and `counters` (kStreamCounters zeroed int32, left
// zeroed) and no norm.
hipError_t launch_gemm_stream_store(const void *Wp, StoreShape sh, const void *X, bool x_rows, bool norm, float eps,
                                    const void *res, void *out, void *out_packed, int M, int N, int K, float *partials,
                                    int *counters, hipStream_t st);
// u = silu(gate) * up of RMSNorm(x), fragment-packed [M16, N2 / 2]; weight [N2, K] with gate / up
// interleaved in 16-row blocks; x raw.
hipError_t launch_gemm_stream_swiglu(const void *Wp, const void *X, bool x_rows, float eps, void *u_packed, int M, int N2,
                                     int K, long variant_rows, hipStream_t st);
// Decode Q/K/V projection (head_dim 128, weight [Wq; Wk; Wv]: one head = one weight group) of
// RMSNorm(x), x raw, and behind it the rotary embedding at position lens[m], the q store into the
// row-major qkv buffer [M, (nq + 2 nkv) * 128] and the append of the rotated key and the value at
// cache slot lens[m] (caches [M, nkv, cap, 128]).
hipError_t launch_gemm_stream_qkv_decode(const void *Wp, const void *X, bool x_rows, float eps, void *qkv, int M, int nq,
                                         int nkv, int K, const void *tab, const int32_t *lens_dev, void *k_cache,
                                         void *v_cache, int cap, hipStream_t st);

// ---- attention (ccs_attention.hip) ---------------------------------------------------------
// Generic (slow, any head_dim <= 256) softmax attention: one wavefront per query row.
// Query rows come from qkv row-major [rows, (nq+2nkv)*d].  prefill: keys/values are the k/v
// parts of qkv of the same sequence, key j visible to row position t iff j <= t; rows with
// position >= lens[b] are skipped.  decode: keys/values are cache slots 0..lens[b].
// Output: f32 row-major [rows, nq*d]; bf16 fragment-packed [rows16, nq*d].
hipError_t launch_attn_generic(int dtype, const void *qkv, void *out, int rows, int nq, int nkv,
                               int d, int decode, int seq_pad, const int32_t *lens_dev,
                               const void *k_cache, const void *v_cache, int cap, hipStream_t st);
// bf16, head_dim 128 causal prefill attention on the matrix cores over dense rows: q rows from
// qkv (rotated, row major, sequence b at rows offs[b]..), keys/values from the kp / vtp buffers of
// launch_rope_pack_prefill; output fragment packed [rows16, nq*128] at the same dense rows.
hipError_t launch_attn_prefill_mfma(const void *qkv, const void *kp, const void *vtp, void *out_packed,
                                    int n_seqs, int seq_pad, int nq, int nkv, const int32_t *offs, hipStream_t st);
// bf16, head_dim 128 decode attention.  Modules with few kv heads (attn_decode_is_whole false): one
// wavefront per (sequence, kv head, 128-key chunk) leaves fp32 partials and launch_attn_decode_combine
// merges them in chunk order.  Modules with many kv heads: one workgroup per (sequence, kv head)
// merges inside and writes out_packed itself; the combine launch is then skipped.
size_t attn_decode_partial_bytes(int n_seqs, int nq, int cap);
bool attn_decode_is_whole(int nq, int nkv);
hipError_t launch_attn_decode_main(const void *qkv, float *partials, void *out_packed, int n_seqs, int nq, int nkv,
                                   const int32_t *lens_dev, const void *k_cache,
                                   const void *v_cache, int cap, hipStream_t st);
hipError_t launch_attn_decode_combine(const float *partials, void *out_packed, int n_seqs, int nq, int nkv,
                                      const int32_t *lens_dev, int cap, hipStream_t st);

}  // namespace ccs
