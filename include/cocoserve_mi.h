/*
 * cocoserve_mi.h - C ABI of the module-replica hot path for AMD Instinct MI355X (gfx950).
 *
 * The library implements the data-parallel core of CoCoServe's module scaling on ONE GPU:
 *   - a *module* is a LLaMA-style decoder layer, a run of consecutive decoder layers, or a
 *     single projection (the paper's module definition: Section 1, footnote on modules;
 *     Section 2.1 lists the projections; Section 3.1: for consecutive replicated layers the
 *     scatter and gather only happen at the two ends of the run);
 *   - *replication* clones the module's weights and runs the unmodified module on contiguous
 *     slices of the batch (15 requests -> 7 and 8), collecting the outputs in batch order
 *     (Section 3.1 "Replication");
 *   - *migration* copies a module to a new place and drops the old copy (Section 3.1
 *     "Migration" and "Implementation").
 * Replicas live in separate weight arenas of the same GPU's HBM and run on separate HIP
 * streams; there is no second device and no collective.
 *
 * Conventions (all entry points)
 *   - Every pointer argument says "host" or "device".  All device memory (weight arenas,
 *     workspaces, activations, KV caches) and all streams are owned by the CALLER; the library
 *     owns only the handle, its events and host-side metadata.
 *   - Streams are passed as `void*` holding a `hipStream_t`.
 *   - Calls enqueue work and return; ordering is by stream and event.  `ccs_module_sync`
 *     waits for everything the module has enqueued.
 *   - Every call returns a `ccs_status`; nothing throws across the ABI.  `ccs_last_error()`
 *     returns a thread-local description of the last non-OK return on this thread.
 *   - There is no CPU fallback: without a usable HIP device calls fail with CCS_EHIP.
 *
 * Data layouts
 *   - Caller-side weights are row-major [out_features, in_features]; a forward computes
 *     y = x W^T, no bias (Section 2.1: projections are linear maps).
 *   - Activations x / y are row-major [rows, features] in the module's dtype.
 *   - KV caches are [n_seqs, n_kv_heads, cache_cap, head_dim] in the module's dtype per layer
 *     (layer l of a run starts cache_layer_stride bytes after layer l - 1); keys are stored
 *     after the rotary embedding.
 *   - `ccs_module_create` re-packs the weights into the arena in the library's own streaming
 *     order; a clone is one contiguous copy of `ccs_module_arena_bytes` bytes.
 */
#ifndef COCOSERVE_MI_H
#define COCOSERVE_MI_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ccs_module ccs_module; /* opaque, library-owned */

typedef enum ccs_status {
    CCS_OK = 0,
    CCS_EINVAL = -1,       /* bad argument (null pointer, bad shape, lens out of range, ...) */
    CCS_ESTATE = -2,       /* call not legal in the module's state (replica not instantiated) */
    CCS_ENOMEM = -3,       /* a caller-provided buffer is too small / host allocation failed */
    CCS_EUNSUPPORTED = -4, /* shape outside what the kernels support */
    CCS_EHIP = -5          /* a HIP runtime call failed; message holds the HIP error string */
} ccs_status;

/* Module kinds (Section 3.3, Table 1 analyses the decoder layer, its self-attention and FFN parts and the
 * single projections as modules of their own).  The two halves of a layer carry their norm and
 * their residual, so that an attention block followed by an FFN block IS the layer:
 *   CCS_ATTN_BLOCK: y = x + Attention(RMSNorm(x; g1)) Wo^T   (uses wq, wk, wv, wo, g1; PREFILL / DECODE)
 *   CCS_FFN_BLOCK:  y = x + (silu(h Wg^T) * (h Wu^T)) Wd^T, h = RMSNorm(x; g2)   (wgate, wup, wdown, g2; ROWS) */
typedef enum ccs_kind { CCS_DECODER_LAYER = 0, CCS_LINEAR = 1, CCS_ATTN_BLOCK = 2, CCS_FFN_BLOCK = 3 } ccs_kind;
typedef enum ccs_dtype { CCS_F32 = 0, CCS_BF16 = 1 } ccs_dtype;
typedef enum ccs_mode {
    CCS_PREFILL = 0, /* whole prompts, causal, right padding masked (Section 2.1 "prefill") */
    CCS_DECODE = 1,  /* one new token per sequence against the KV cache (Section 2.1 "decode") */
    CCS_ROWS = 2     /* CCS_LINEAR and CCS_FFN_BLOCK modules: independent token rows */
} ccs_mode;

enum { CCS_MAX_REPLICAS = 16 };

/* Shape of a module.  Decoder layer: hidden, heads, head_dim, intermediate (SwiGLU width),
 * rms_eps, rope_base; requires n_q_heads % n_kv_heads == 0 and head_dim even.  The bf16 path
 * additionally needs hidden, n_q_heads*head_dim and intermediate to be multiples of 32,
 * n_kv_heads*head_dim a multiple of 16 and head_dim == 128 (else CCS_EUNSUPPORTED); the f32 path takes
 * any shape with head_dim <= 256.  n_layers (0 is read as 1, at most CCS_MAX_LAYERS) makes
 * the module a run of that many consecutive decoder layers of this shape, each with its own
 * weights: the output of layer l is the input of layer l + 1 and a replica runs the whole run
 * on its slice.  Linear: in_features, out_features (bf16: in % 32 == 0, out % 16 == 0). */
enum { CCS_MAX_LAYERS = 128 };
typedef struct ccs_module_desc {
    int32_t kind;  /* ccs_kind */
    int32_t dtype; /* ccs_dtype: storage type of weights, activations and caches */
    int32_t hidden, n_q_heads, n_kv_heads, head_dim, intermediate;
    int32_t in_features, out_features;
    float rms_eps, rope_base;
    int32_t n_layers; /* decoder layers in the run; 0 or 1: a single layer */
} ccs_module_desc;

/* Device pointers to the caller's weights in the module's dtype, row-major [out, in].
 * Decoder layer: wq [n_q*d, H], wk/wv [n_kv*d, H], wo [H, n_q*d], wgate/wup [I, H],
 * wdown [H, I], g1/g2 [H] (RMSNorm gains).  Linear: w [out, in]; the others are ignored.
 * A run of n_layers layers takes an array of n_layers of these, first layer first.
 * Read only during ccs_module_create. */
typedef struct ccs_weights {
    const void *wq, *wk, *wv, *wo, *wgate, *wup, *wdown, *g1, *g2;
    const void *w;
} ccs_weights;

/* One batch (or one contiguous slice of it).
 *   PREFILL: x, y are [n_seqs, seq_pad, hidden]; lens[b] in [1, seq_pad] is the prompt length,
 *            rows t >= lens[b] are padding: never read (bf16 modules gather the valid rows
 *            into a dense matrix and compute those alone); their y rows are written as zeros
 *            by bf16 modules and hold unspecified finite values for fp32 modules.
 *            If k_cache/v_cache are non-null the rotated keys and the values of
 *            positions < lens[b] are stored there (cache_cap >= lens[b]).
 *   DECODE:  x, y are [n_seqs, hidden]; lens[b] >= 0 is the number of cached positions; the
 *            new token is position lens[b]: its key/value are stored at slot lens[b] and the
 *            query attends over slots 0..lens[b] (cache_cap >= lens[b] + 1).  The caches are
 *            required.  lens itself is not advanced by the library.
 *   ROWS:    x is [n_seqs, in_features], y is [n_seqs, out_features] (an FFN block: both
 *            [n_seqs, hidden]); seq_pad, lens and the caches are ignored.
 * A run of layers: every layer has caches of this shape; k_cache / v_cache point at the first
 * layer's and layer l's start cache_layer_stride BYTES further each (at least the bytes of one
 * layer's cache for the WHOLE batch the slice belongs to; ignored for a single layer).
 * lens_host and lens_dev hold the same n_seqs values (host copy for validation and launch
 * planning, device copy for the kernels).  n_seqs == 0 is a legal no-op. */
typedef struct ccs_batch {
    int32_t mode; /* ccs_mode */
    int32_t n_seqs, seq_pad;
    const void *x;            /* device */
    void *y;                  /* device */
    const int32_t *lens_host; /* host   */
    const int32_t *lens_dev;  /* device */
    void *k_cache, *v_cache;  /* device */
    int32_t cache_cap;
    int64_t cache_layer_stride; /* bytes between consecutive layers' caches (runs of layers) */
} ccs_batch;

/* Bytes of one replica's packed weights (what a clone copies); 0 if the desc is invalid.
 * Table 1 of the paper counts the same bytes for a layer (projections only) - the arena adds
 * the two norm-gain vectors and alignment padding.  Host-only, no GPU needed. */
size_t ccs_module_arena_bytes(const ccs_module_desc *desc);

/* Bytes of scratch one replica needs to run batches of at most max_seqs sequences with
 * max_seq_pad rows each (1 for DECODE and ROWS) and caches of at most max_cache_cap slots.
 * Host-only.  0 if the desc is invalid. */
size_t ccs_module_workspace_bytes(const ccs_module_desc *desc, int32_t max_seqs,
                                  int32_t max_seq_pad, int32_t max_cache_cap);

/* Section 1 (footnote on modules) and Section 2.1: a module - decoder layer, attention or FFN
 * block, projection - is the unit that is replicated and migrated; Section 3.1: the original
 * instance keeps serving while replicas are added beside it.
 * Create a module with ONE instance (replica 0, "the original"): packs `weights` (host array of
 * max(1, n_layers) structs holding device pointers) into
 * `arena0` (device, >= ccs_module_arena_bytes, 256-byte aligned) on `stream`, and remembers
 * `workspace0` (device, workspace_bytes long, 256-byte aligned) and `stream` as replica 0's.
 * A workspace belongs to its replica from here on: the call clears its first KiB on `stream`
 * (arrival counters that the replica's launches use and leave at zero); the caller must not
 * write to it, nor hand it to another replica or module, while the replica exists.
 * The caller's weight buffers may be released after the stream has been synchronised.
 * Errors: CCS_EINVAL (null/misaligned pointers, bad desc), CCS_EUNSUPPORTED, CCS_EHIP. */
int ccs_module_create(const ccs_module_desc *desc, const ccs_weights *weights, void *arena0,
                      void *workspace0, size_t workspace_bytes, void *stream, ccs_module **out);

/* Set the number of instances to k (1 <= k <= CCS_MAX_REPLICAS).  For every replica j that
 * does not exist yet, arenas[j], workspaces[j] (device) and streams[j] are taken over and the
 * weights of replica 0 are cloned into arenas[j] by a streaming HBM->HBM copy enqueued on
 * streams[j] (after replica 0's pending pack/clone), and the first KiB of workspaces[j] is
 * cleared there as ccs_module_create does for replica 0's; replica j's forwards are ordered
 * after both.  Entries of existing replicas (j < current k, including 0) are ignored and may
 * be null.  Shrinking (k below the current count) waits for the dropped replicas' work and
 * forgets them; their buffers go back to the caller.  Section 3.1 "Replication".
 * Errors: CCS_EINVAL, CCS_EHIP. */
int ccs_module_replicate(ccs_module *m, int32_t k, void *const *arenas, void *const *workspaces,
                         size_t workspace_bytes, void *const *streams);

/* Number of instances the module currently has (>= 1), or CCS_EINVAL. */
int ccs_module_replicas(const ccs_module *m);

/* Section 3.1 "Replication": every instance runs the UNMODIFIED module on its contiguous slice of
 * the batch; Section 2.1: the module's arithmetic in prefill and decode.
 * Run the module on ONE replica over one contiguous slice, on that replica's stream.
 * `slice` (host struct; its pointers as documented above) already points at the slice's first
 * row / sequence.  Errors: CCS_EINVAL (bad replica index, bad batch), CCS_ESTATE, CCS_ENOMEM
 * (workspace too small for this batch), CCS_EHIP. */
int ccs_module_forward(ccs_module *m, int32_t replica, const ccs_batch *slice);

/* For callers that cannot allocate or bring a workspace (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): ccs_module_forward with everything the
 * kernels keep between launches - normalised rows, q/k/v, attention output, SwiGLU output, the
 * fp32 partial sums of the split-K projections and of the split-KV attention - in an array of
 * CCS_STATIC_WORKSPACE_BYTES that is part of the library's code object (every GPU the library
 * runs on holds one copy until the process ends) instead of the replica's workspace.  The call
 * makes no allocation of any kind and records no per-kernel timing.  Same kernels, same
 * arithmetic, same bits as ccs_module_forward.  A batch whose plan does not fit the array is
 * rejected with CCS_ENOMEM and a message that gives both sizes (64 MiB hold every decode step of
 * the 7B / 13B / 70B shapes up to 64 sequences x 2048 cached positions and projections of a few
 * hundred rows; a 13B prefill of thousands of rows does not fit).  Nothing in the array has to
 * start at zero: every partial sum a kernel reads was written by the launch before it.  ALL
 * calls on one GPU share that GPU's array - of every module and replica: two calls whose kernels
 * may overlap in time (different streams without an ordering between them) race; keep them on
 * one stream or order them with events.  Other errors as ccs_module_forward. */
enum { CCS_STATIC_WORKSPACE_BYTES = 64 * 1024 * 1024 };
int ccs_module_forward_static(ccs_module *m, int32_t replica, const ccs_batch *slice);

/* CCS_STATIC_WORKSPACE_BYTES as the built library has it. */
size_t ccs_static_workspace_bytes(void);

/* The replicated forward of Section 3.1: cut the batch into k = ccs_module_replicas(m)
 * contiguous slices [floor(j n / k), floor((j+1) n / k)) - over sequences for a decoder layer,
 * over token rows for a projection.  Slice 0 runs on `caller_stream` itself with replica 0's
 * weights and workspace; for j >= 1 the call orders `caller_stream` -> replica j's stream (fork
 * event), runs slice j there, and orders that stream -> `caller_stream` (join event).  Outputs
 * land in `full->y` at their batch positions, so the gather is free.  Output rows are
 * bit-identical for every k at a fixed batch.  `caller_stream` is ordered after the work that
 * created or migrated replica 0, and copies / migrations / the next forward of replica 0 on
 * another stream are ordered after this slice 0; two replicated forwards of one module issued from
 * DIFFERENT caller streams without an ordering between them still share replica 0's workspace:
 * keep them on one stream or order them.  If a slice fails after others were forked, the forked
 * streams are joined before the error is returned.  The call only enqueues (kernel launches, event record / wait), so it may be
 * recorded into a HIP graph by capturing `caller_stream`. */
int ccs_module_forward_split(ccs_module *m, const ccs_batch *full, void *caller_stream);

/* The same with uneven shares: slice j is the next counts[j] sequences (rows for a projection),
 * j = 0 .. k-1 in batch order; counts (host, k entries, >= 0) must add up to full->n_seqs.
 * Section 4.1, Eq. 1: a replica's share bs_ij follows its capacity, and the layer takes as long
 * as its slowest replica.  Results are bit-identical to any other partition of the batch.
 * Errors as ccs_module_forward_split, plus CCS_EINVAL for bad counts. */
int ccs_module_forward_shares(ccs_module *m, const ccs_batch *full, const int32_t *counts,
                              void *caller_stream);

/* Section 3.1 "Implementation": instantiating a replica duplicates the module with its weights;
 * Section 6.5, Table 2 prices that step.
 * Clone replica `replica`'s packed weights into `dst_arena` (device, arena_bytes) on `stream`
 * (ordered after that replica's pending work, including a slice 0 that a replicated forward
 * ran on a caller's stream); the source stays in use.  Errors: CCS_EINVAL, CCS_ESTATE, CCS_EHIP. */
int ccs_module_copy(ccs_module *m, int32_t replica, void *dst_arena, void *stream);

/* Migrate: clone as ccs_module_copy, then make `dst_arena` the replica's arena; later
 * forwards on the replica are ordered after the copy.  The old arena belongs to the caller
 * again once `stream` has been synchronised (Section 3.1 "Implementation": replicate to the
 * destination, remove the local copy). */
int ccs_module_migrate(ccs_module *m, int32_t replica, void *dst_arena, void *stream);

/* Copy / migrate a KV cache that travels with its layer (Section 3.1 "Implementation":
 * optional migration of the KV cache): a streaming copy of `bytes` bytes device->device on
 * `stream`.  src and dst must not overlap; both 16-byte aligned. */
int ccs_cache_copy(void *dst, const void *src, size_t bytes, void *stream);

/* Device address of replica `replica`'s arena (for tests and for freeing after migrate). */
int ccs_module_arena(const ccs_module *m, int32_t replica, void **arena_out);

/* Kernels of one replica forward, for per-kernel device timing.  The weight-streaming GEMM
 * variant is one launch when K is not split (its epilogue runs in the kernel) and two otherwise
 * (main + REDUCE); the LDS-tiled variant reports everything under the main stage.  A projection
 * module reports PACK_X and GEMM_DOWN(+_REDUCE).  In a run of layers a stage accumulates over
 * the layers. */
typedef enum ccs_stage {
    CCS_ST_RMSNORM1 = 0,
    CCS_ST_GEMM_QKV = 1, CCS_ST_GEMM_QKV_REDUCE = 2,
    CCS_ST_ROPE = 3,
    CCS_ST_ATTN = 4, CCS_ST_ATTN_COMBINE = 5,
    CCS_ST_GEMM_O = 6, CCS_ST_GEMM_O_REDUCE = 7,
    CCS_ST_RMSNORM2 = 8,
    CCS_ST_GEMM_GU = 9, CCS_ST_GEMM_GU_REDUCE = 10,
    CCS_ST_GEMM_DOWN = 11, CCS_ST_GEMM_DOWN_REDUCE = 12,
    CCS_ST_PACK_X = 13,
    CCS_ST_CLONE = 14,
    CCS_ST_COMPACT = 15,   /* bf16 prefill: valid rows of the padded batch gathered into dense rows */
    CCS_ST_EXPAND = 16,    /* ... and the output rows put back, padded rows zeroed */
    CCS_N_STAGES = 17
} ccs_stage;

/* Per-kernel timing (the paper's Monitor gathers latencies with event timers, Section 5
 * "Metrics Monitor").  While bit s of stage_mask is set, every launch of stage s is bracketed
 * by a pair of HIP events on the stream it is enqueued on; 0 switches timing off (default).
 * Recording stops silently after 65536 unread pairs per replica. */
int ccs_module_profile(ccs_module *m, uint32_t stage_mask);

/* Wait for the recorded pairs of `replica`, and return per stage the summed kernel time in
 * milliseconds (ms_sum, host, CCS_N_STAGES doubles) and the number of launches (count, host,
 * CCS_N_STAGES int64) accumulated since the last reset; reset != 0 clears them afterwards. */
int ccs_module_profile_read(ccs_module *m, int32_t replica, double *ms_sum, int64_t *count,
                            int32_t reset);

/* Section 3.1 (correctness of scaling operations): an instance is only dropped or moved once its
 * work has finished.  Block the host until every stream of the module has drained, including
 * caller streams that ran slice 0 of a replicated forward. */
int ccs_module_sync(ccs_module *m);

/* Section 3.1 "Migration": removing an instance hands its memory back.  Wait for the module's
 * work, release events and host metadata.  Device buffers stay with the caller. */
int ccs_module_destroy(ccs_module *m);

/* ---- scale-up planning (Section 4.1), host-only: no GPU, no module handle ----------------------- */

/* Eq. 4, homogeneous devices and even splits: S = 1 / (gamma + (1 - gamma) / n * sum_i 1 / p_i),
 * p[i] >= 1 the number of instances of layer i (host array, n entries), gamma = delta C / (d B).
 * Returns 0 for bad arguments. */
double ccs_speedup_homo(const int32_t *p, int32_t n, double gamma);

/* Eq. 1-3, general form: S = W(P0) / (W(P) + T(P)) with W(P) = sum_i max_j d^2 bs_ij l / C_ij and
 * T(P) = delta sum_i sum_{j>=1} d bs_ij l / B_ij.  bs, capacity, bandwidth are host arrays
 * flattened over (layer i, instance j < p[i]), instance 0 being the original (its bandwidth
 * entry is ignored); W(P0) runs each layer's whole batch on its original.  Returns 0 for bad
 * arguments. */
double ccs_speedup(const int32_t *p, int32_t n, const double *bs, const double *capacity,
                   const double *bandwidth, double d, double l, double delta);

/* Section 4.1, Eq. 1: a layer takes as long as its slowest instance, max_j d^2 bs_ij l / C_ij, so an
 * instance's share of the batch should follow its capacity.  Computes the integer shares
 * counts_out[j] >= 0 (host, k entries, sum n) that MINIMISE max_j counts[j] / capacity[j] for the
 * k instances' capacities (host, k positive finite doubles; only their ratios matter), ready for
 * ccs_module_forward_shares.  Among the optimal answers it returns the one reached from the
 * capacity-weighted contiguous split - boundaries floor(n (C_0 + .. + C_{j-1}) / C_total), which for
 * equal capacities is the paper's floor(j n / k) rule (15 -> 7 + 8) - by handing single units from
 * a slowest instance to the instance that stays fastest.  Host-only.
 * Errors: CCS_EINVAL (null pointers, k outside [1, CCS_MAX_REPLICAS], n < 0, a capacity <= 0). */
int ccs_shares_from_capacity(int64_t n, int32_t k, const double *capacity, int32_t *counts_out);

/* Algorithm 1 (greedy scale-up).  p_in: current instances per layer (n entries, >= 1).  Node g
 * (n_nodes of them, visited in order) has node_available[g] free resource units; it is eligible
 * if at least one replica of replica_size units fits, and takes at most available / size replicas.
 * placed_in (optional, [n_nodes][n] bytes): which layers node g already holds a replica of.
 * For each eligible node the candidate layers are ordered by continuity - repeatedly the free
 * layer that gives the node its longest run of consecutive layers, the lower index on ties - and
 * a replica is added whenever Eq. 4 improves.  Outputs: p_out (n entries), placed_out
 * ([n_nodes][n] bytes, caller-allocated), speedup_out (optional).  The call only plans; the
 * caller instantiates the replicas.  Errors: CCS_EINVAL. */
int ccs_plan_scale_up(const int32_t *p_in, int32_t n, double gamma, const int64_t *node_available,
                      int32_t n_nodes, int64_t replica_size, const uint8_t *placed_in,
                      int32_t *p_out, uint8_t *placed_out, double *speedup_out);

/* Thread-local, never null; valid until the next library call on this thread. */
const char *ccs_last_error(void);

/* Library version string. */
const char *ccs_version(void);

#ifdef __cplusplus
}
#endif
#endif /* COCOSERVE_MI_H */
