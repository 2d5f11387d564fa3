// Host runtime and C ABI (include/cocoserve_mi.h): module handle, weight-arena and workspace
// plans, replica streams/events, the batch-slice planner and the fork/join of the replicated
// forward (paper, Section 3.1 "Replication" / "Migration" / "Implementation").
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/cocoserve_mi.h"
#include "ccs_common.h"
#include "ccs_kernels.h"

// Workspace of ccs_module_forward_static: one array per GPU, inside the code object, so that the
// entry point needs no caller workspace and no allocation.  Host code never uses this name as an
// address (on the host it is only a stand-in for the symbol): static_workspace() asks the runtime
// for the device address once per device and everything else goes through that pointer.
static __device__ __align__(256) unsigned char g_static_ws[CCS_STATIC_WORKSPACE_BYTES];

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

#define CCS_HIP(expr)                                                                       \
    do {                                                                                    \
        hipError_t e__ = (expr);                                                            \
        if (e__ != hipSuccess) return fail(CCS_EHIP, "%s: %s", #expr, hipGetErrorString(e__)); \
    } while (0)

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Device address of g_static_ws on the current device (every GPU holds its own copy of the array at
// its own address); resolved on first use per device, then cached.
constexpr int kMaxDevices = 64;
std::mutex g_static_ws_mutex;
void *g_static_ws_ptr[kMaxDevices] = {nullptr};

int static_workspace(void **out)
{
    int dev = -1;
    CCS_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(CCS_EUNSUPPORTED, "device index %d beyond %d", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_static_ws_mutex);
    if (!g_static_ws_ptr[dev]) {
        void *p = nullptr;
        CCS_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_ws)));
        if (!p || ((uintptr_t)p & 255)) return fail(CCS_EHIP, "static workspace symbol resolved to %p", p);
        g_static_ws_ptr[dev] = p;
    }
    *out = g_static_ws_ptr[dev];
    return CCS_OK;
}

struct Dims {
    int H, nq, nkv, d, I, QD, KD, W3;  // W3 = QD + 2 KD
    int in_f, out_f;
    int L;  // decoder layers in the run (1 for a single layer or a projection)
    size_t esz;
};

// a decoder layer and its two halves (Section 3.3, Table 1 lists self-attention and FFN as modules of
// their own) share shapes, kernels and plans
inline bool is_layerlike(int kind) { return kind == CCS_DECODER_LAYER || kind == CCS_ATTN_BLOCK || kind == CCS_FFN_BLOCK; }
inline bool has_attn(int kind) { return kind == CCS_DECODER_LAYER || kind == CCS_ATTN_BLOCK; }
inline bool has_ffn(int kind) { return kind == CCS_DECODER_LAYER || kind == CCS_FFN_BLOCK; }

struct ArenaPlan {
    size_t qkv, o, gu, dn, g1, g2, rope, w;  // offsets inside one layer
    size_t layer;                            // bytes of one layer (256-byte multiple)
    size_t total;                            // layers * layer
};

struct WsPlan {
    // h: normalised rows (LDS-tiled path); xp, x1p: fragment-packed raw rows of the layer input and of
    // the residual stream after the attention block (weight-streaming path: the projections apply the
    // norm themselves); xa, xb: activations between layers of a run; xc, yc, offs: dense prefill
    // rows in / out and their per-sequence offsets
    size_t h, qkv, a, x1, gu, u, xp, x1p, kp, vtp, xa, xb, xc, yc, offs, ssqp, scratch, scratch_bytes, total;   // ssqp: per-segment sums of squares of a K-split projection
    size_t cnt;   // arrival counters of split weight-streaming launches: always at offset 0, zeroed when the workspace is attached
};

// A store-type projection (O, down, a single projection) of a batch of `variant_rows` <= 64 rows runs
// as one launch over narrow tiles, except for 33..64 rows against a long K, where 128-column tiles
// with a K split and a reduction kernel stream faster (measured on the 70B down projection: 80 us
// against 102 us).  Decided from the weight shape and the FULL batch's row count.
inline bool store_split(int K, long long variant_rows) { return variant_rows > 32 && K > 8192; }
// The decode Q/K/V projection likewise: one launch over half-head tiles up to 32 rows; for 33..64 rows
// whole-head tiles with a K split and a reduction kernel that also rotates and appends (measured on
// the 70B shape: 41 us against 55 us).
inline bool qkv_split(long long variant_rows) { return variant_rows > 32; }
// A single projection of up to this many rows (of the FULL batch) reads the caller's row-major rows in
// the LDS-tiled GEMM itself; larger batches are packed first.
constexpr long long kDirectRowsMax = 512;
// first bytes of every workspace: arrival counters of split weight-streaming launches
constexpr size_t kCounterBytes = (size_t)ccs::kStreamCounters * sizeof(int32_t);
constexpr long long kLinearStreamRowsMax = 32;
// A single projection streams its weight in one launch up to 32 rows (of the FULL batch), and up to
// 64 rows when the weight's shape lets that launch cut K over workgroups (wide tiles: measured on
// 11008 -> 4096 at 64 rows 22.9 us in one launch, against 32.9 us over narrow tiles and 26 us for
// the LDS-tiled GEMM with its reduction launch).
inline bool linear_streams(int out_f, int in_f, long long variant_rows)
{
    if (variant_rows <= kLinearStreamRowsMax) return true;
    return variant_rows <= ccs::kSkinnyMaxRows && ccs::stream_store_shape(out_f, in_f, (long)variant_rows).nseg > 1;
}

int check_desc(const ccs_module_desc *D, Dims *out)
{
    if (!D) return fail(CCS_EINVAL, "desc is null");
    if (D->dtype != CCS_F32 && D->dtype != CCS_BF16) return fail(CCS_EINVAL, "unknown dtype %d", D->dtype);
    Dims d{};
    d.esz = D->dtype == CCS_BF16 ? 2 : 4;
    d.L = 1;
    if (D->n_layers < 0 || D->n_layers > CCS_MAX_LAYERS) return fail(CCS_EINVAL, "n_layers must be in [0, %d]", (int)CCS_MAX_LAYERS);
    if (is_layerlike(D->kind)) {
        if (D->kind != CCS_DECODER_LAYER && D->n_layers > 1) return fail(CCS_EINVAL, "n_layers applies to whole decoder layers only");
        d.L = D->n_layers > 1 ? D->n_layers : 1;
        if (D->hidden <= 0 || D->n_q_heads <= 0 || D->n_kv_heads <= 0 || D->head_dim <= 0 || D->intermediate <= 0)
            return fail(CCS_EINVAL, "decoder-layer dimensions must be positive");
        if (D->n_q_heads % D->n_kv_heads) return fail(CCS_EINVAL, "n_q_heads %% n_kv_heads != 0");
        if (D->head_dim & 1) return fail(CCS_EINVAL, "head_dim must be even");
        if (!(D->rms_eps >= 0.f) || !(D->rope_base > 0.f)) return fail(CCS_EINVAL, "bad rms_eps / rope_base");
        d.H = D->hidden; d.nq = D->n_q_heads; d.nkv = D->n_kv_heads; d.d = D->head_dim; d.I = D->intermediate;
        d.QD = d.nq * d.d; d.KD = d.nkv * d.d; d.W3 = d.QD + 2 * d.KD;
        if (d.d > 256) return fail(CCS_EUNSUPPORTED, "head_dim > 256");
        if (D->dtype == CCS_BF16) {
            if (d.H % 32 || d.QD % 32 || d.I % 32 || d.KD % 16)
                return fail(CCS_EUNSUPPORTED, "bf16 path: hidden, n_q*d, intermediate must be multiples of 32, n_kv*d of 16");
            if (d.d != 128) return fail(CCS_EUNSUPPORTED, "bf16 path: head_dim must be 128");
            const int G = d.nq / d.nkv;
            if (G != 1 && G != 2 && G != 4 && G != 8) return fail(CCS_EUNSUPPORTED, "bf16 path: n_q/n_kv must be 1, 2, 4 or 8");
        }
    } else if (D->kind == CCS_LINEAR) {
        if (D->n_layers > 1) return fail(CCS_EINVAL, "n_layers applies to decoder layers only");
        if (D->in_features <= 0 || D->out_features <= 0) return fail(CCS_EINVAL, "linear dimensions must be positive");
        d.in_f = D->in_features; d.out_f = D->out_features;
        if (D->dtype == CCS_BF16 && (d.in_f % 32 || d.out_f % 16))
            return fail(CCS_EUNSUPPORTED, "bf16 path: in_features %% 32 and out_features %% 16 must be 0");
    } else {
        return fail(CCS_EINVAL, "unknown kind %d", D->kind);
    }
    if (out) *out = d;
    return CCS_OK;
}

ArenaPlan arena_plan(const ccs_module_desc *D, const Dims &d)
{
    ArenaPlan p{};
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    // bf16 weights are fragment-packed in groups of 8 row blocks (padded to a whole group)
    auto wbytes = [&](int N, int K) { return D->dtype == CCS_BF16 ? ccs::packed_weight_bytes(N, K) : (size_t)N * K * 4; };
    if (D->kind == CCS_LINEAR) {
        p.w = take(wbytes(d.out_f, d.in_f));
    } else {
        if (has_attn(D->kind)) {
            p.qkv = take(wbytes(d.W3, d.H));
            p.o = take(wbytes(d.H, d.QD));
            p.g1 = take((size_t)d.H * d.esz);
            p.rope = take((size_t)(d.d / 2) * 2 * sizeof(float));  // inverse-frequency table (fp32 head + tail)
        }
        if (has_ffn(D->kind)) {
            p.gu = take(wbytes(2 * d.I, d.H));
            p.dn = take(wbytes(d.H, d.I));
            p.g2 = take((size_t)d.H * d.esz);
        }
    }
    p.layer = off;
    p.total = off * (size_t)d.L;
    return p;
}

inline size_t max_sz(size_t a, size_t b) { return a > b ? a : b; }

// Scratch one forward over `rows` rows (n_seqs sequences, caches of `cap` slots) needs.
// `skinny`: the weight-streaming GEMM variant is in use (rows <= kSkinnyMaxRows).
// `vrows`: row count of the full batch (selects the K split of the LDS-tiled GEMM).
WsPlan ws_plan(const ccs_module_desc *D, const Dims &d, size_t rows, int n_seqs, int cap, bool skinny,
               bool decode, int prefill_seq_pad = 0, long vrows = -1)
{
    if (vrows < 0) vrows = (long)rows;
    WsPlan p{};
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    const size_t r16 = align_up(rows, 16);
    p.cnt = take(kCounterBytes);
    if (D->kind == CCS_LINEAR) {
        if (D->dtype == CCS_BF16) {
            p.xp = take(r16 * d.in_f * 2);
            p.scratch_bytes = linear_streams(d.out_f, d.in_f, vrows) ? ccs::stream_store_partial_bytes(d.out_f, d.in_f, vrows, (int)rows)
                                                            : ccs::tiled_partial_bytes((int)rows, d.out_f, d.in_f, vrows);
            p.scratch = take(p.scratch_bytes);
        }
    } else if (D->dtype == CCS_BF16) {
        p.h = take(r16 * d.H * 2);
        p.xp = take(r16 * d.H * 2);
        p.x1p = take(r16 * d.H * 2);
        p.qkv = take(rows * d.W3 * 2);
        p.a = take(r16 * d.QD * 2);
        p.x1 = take(rows * d.H * 2);
        p.u = take(r16 * d.I * 2);
        if (prefill_seq_pad > 0) {  // K / V^T in matrix-core operand order for the prefill attention
            const size_t s32 = align_up((size_t)prefill_seq_pad, 32);
            p.kp = take((size_t)n_seqs * d.nkv * s32 * d.d * 2);
            p.vtp = take((size_t)n_seqs * d.nkv * s32 * d.d * 2);
            p.xc = take(rows * d.H * 2);   // the batch's valid rows without the padding, and the output before it is padded again
            p.yc = take(rows * d.H * 2);
            p.offs = take(((size_t)n_seqs + 1) * 4);
        }
        if (d.L > 1) {
            p.xa = take(rows * d.H * 2);
            p.xb = take(rows * d.H * 2);
        }
        size_t s = 0;
        p.ssqp = take((size_t)64 * ccs::kSkinnyMaxRows * sizeof(float));
        if (skinny) {   // partial sums of the projections that may take the K-split form
            s = max_sz(s, ccs::skinny_partial_bytes((int)rows, d.W3, d.H));
            s = max_sz(s, ccs::skinny_partial_bytes((int)rows, d.H, d.QD));
            s = max_sz(s, ccs::skinny_partial_bytes((int)rows, d.H, d.I));
            s = max_sz(s, ccs::stream_store_partial_bytes(d.H, d.QD, vrows, (int)rows));
            s = max_sz(s, ccs::stream_store_partial_bytes(d.H, d.I, vrows, (int)rows));
        } else {
            s = max_sz(s, ccs::tiled_partial_bytes((int)rows, d.W3, d.H, vrows));
            s = max_sz(s, ccs::tiled_partial_bytes((int)rows, d.H, d.QD, vrows));
            s = max_sz(s, ccs::tiled_partial_bytes((int)rows, 2 * d.I, d.H, vrows));
            s = max_sz(s, ccs::tiled_partial_bytes((int)rows, d.H, d.I, vrows));
        }
        if (decode) s = max_sz(s, ccs::attn_decode_partial_bytes(n_seqs, d.nq, cap));
        p.scratch_bytes = s;
        p.scratch = take(s);
    } else {
        p.h = take(rows * d.H * 4);
        p.qkv = take(rows * d.W3 * 4);
        p.a = take(rows * d.QD * 4);
        p.x1 = take(rows * d.H * 4);
        p.gu = take(rows * 2 * d.I * 4);
        p.u = take(rows * d.I * 4);
        if (d.L > 1) {
            p.xa = take(rows * d.H * 4);
            p.xb = take(rows * d.H * 4);
        }
    }
    p.total = off;
    return p;
}

// Per-kernel device timing with HIP events on the replica's own stream (the paper's Monitor
// collects latencies with event timers, Section 5 "Metrics Monitor").
struct ProfPair {
    hipEvent_t a, b;
    int stage;
};
struct Prof {
    std::vector<ProfPair> pending;
    std::vector<ProfPair> pool;
    double ms[CCS_N_STAGES] = {0};
    int64_t count[CCS_N_STAGES] = {0};
};

struct Replica {
    Prof *prof = nullptr;
    void *arena = nullptr;
    void *ws = nullptr;
    size_t ws_bytes = 0;
    hipStream_t stream = nullptr;
    hipEvent_t ready = nullptr;  // arena contents complete (pack / clone / migrate)
    hipEvent_t done = nullptr;   // last forward_split slice finished
};

}  // namespace

struct ccs_module {
    ccs_module_desc desc;
    Dims dims;
    ArenaPlan ap;
    int k = 0;
    Replica rep[CCS_MAX_REPLICAS];
    hipEvent_t fork = nullptr;
    hipEvent_t slice0_done = nullptr;   // end of the last slice 0 that ran on a caller's stream other than replica 0's
    bool slice0_recorded = false;
    uint32_t prof_mask = 0;
};

namespace {

int make_event(hipEvent_t *ev)
{
    CCS_HIP(hipEventCreateWithFlags(ev, hipEventDisableTiming));
    return CCS_OK;
}

void drop_events(Replica &R)
{
    if (R.ready) (void)hipEventDestroy(R.ready);
    if (R.done) (void)hipEventDestroy(R.done);
    R.ready = R.done = nullptr;
}

constexpr size_t kProfMaxPending = 1u << 16;

ProfPair *prof_begin(ccs_module *m, Replica &R, int stage, hipStream_t st)
{
    if (!(m->prof_mask & (1u << stage))) return nullptr;
    if (!R.prof) R.prof = new (std::nothrow) Prof();
    if (!R.prof || R.prof->pending.size() >= kProfMaxPending) return nullptr;
    ProfPair p{nullptr, nullptr, stage};
    if (!R.prof->pool.empty()) {
        p = R.prof->pool.back();
        p.stage = stage;
        R.prof->pool.pop_back();
    } else if (hipEventCreate(&p.a) != hipSuccess || hipEventCreate(&p.b) != hipSuccess) {
        if (p.a) (void)hipEventDestroy(p.a);
        return nullptr;
    }
    if (hipEventRecord(p.a, st) != hipSuccess) {
        R.prof->pool.push_back(p);   // keep the pair for a later launch
        return nullptr;
    }
    R.prof->pending.push_back(p);
    return &R.prof->pending.back();
}

void prof_end(ProfPair *p, hipStream_t st)
{
    if (p) (void)hipEventRecord(p->b, st);
}

void prof_free(Replica &R)
{
    if (!R.prof) return;
    for (auto &p : R.prof->pending) { (void)hipEventDestroy(p.a); (void)hipEventDestroy(p.b); }
    for (auto &p : R.prof->pool) { (void)hipEventDestroy(p.a); (void)hipEventDestroy(p.b); }
    delete R.prof;
    R.prof = nullptr;
}

#define CCS_STAGE(sid, expr)                              \
    do {                                                  \
        ProfPair *pp__ = prof_on ? prof_begin(m, R, (sid), st) : nullptr; \
        hipError_t se__ = (expr);                         \
        prof_end(pp__, st);                               \
        if (se__ != hipSuccess) return fail(CCS_EHIP, "%s: %s", #expr, hipGetErrorString(se__)); \
    } while (0)

int check_batch(const ccs_module *m, const ccs_batch *b)
{
    if (!b) return fail(CCS_EINVAL, "batch is null");
    if (b->n_seqs < 0) return fail(CCS_EINVAL, "n_seqs < 0");
    const Dims &d = m->dims;
    if (m->desc.kind == CCS_LINEAR || m->desc.kind == CCS_FFN_BLOCK) {
        if (b->mode != CCS_ROWS) return fail(CCS_EINVAL, "a projection or FFN block takes mode CCS_ROWS");
        if (b->n_seqs > 0 && (!b->x || !b->y)) return fail(CCS_EINVAL, "x / y is null");
        return CCS_OK;
    }
    if (b->mode != CCS_PREFILL && b->mode != CCS_DECODE)
        return fail(CCS_EINVAL, "a decoder layer or attention block takes mode CCS_PREFILL or CCS_DECODE");
    if (b->n_seqs == 0) return CCS_OK;
    if (!b->x || !b->y) return fail(CCS_EINVAL, "x / y is null");
    if (!b->lens_host || !b->lens_dev) return fail(CCS_EINVAL, "lens_host / lens_dev is null");
    if ((b->k_cache == nullptr) != (b->v_cache == nullptr)) return fail(CCS_EINVAL, "k_cache and v_cache must come together");
    if (b->mode == CCS_PREFILL) {
        if (b->seq_pad < 1) return fail(CCS_EINVAL, "seq_pad < 1");
        if ((long long)b->n_seqs * b->seq_pad > 0x7fffffffLL / 4) return fail(CCS_EUNSUPPORTED, "too many rows");
        for (int i = 0; i < b->n_seqs; ++i) {
            const int len = b->lens_host[i];
            if (len < 1 || len > b->seq_pad) return fail(CCS_EINVAL, "lens[%d] = %d outside [1, seq_pad = %d]", i, len, b->seq_pad);
            if (b->k_cache && len > b->cache_cap) return fail(CCS_EINVAL, "lens[%d] = %d exceeds cache_cap %d", i, len, b->cache_cap);
        }
        if (b->seq_pad > 8192) return fail(CCS_EUNSUPPORTED, "seq_pad > 8192");
    } else {
        if (!b->k_cache) return fail(CCS_EINVAL, "decode needs k_cache / v_cache");
        if (b->cache_cap < 1) return fail(CCS_EINVAL, "cache_cap < 1");
        for (int i = 0; i < b->n_seqs; ++i) {
            const int len = b->lens_host[i];
            if (len < 0 || len + 1 > b->cache_cap) return fail(CCS_EINVAL, "lens[%d] = %d needs cache_cap > %d (have %d)", i, len, len, b->cache_cap);
        }
        if (m->desc.dtype == CCS_F32 && b->cache_cap > 8192) return fail(CCS_EUNSUPPORTED, "f32 decode: cache_cap > 8192");
    }
    if (d.L > 1 && b->k_cache) {
        const long long one = (long long)b->n_seqs * d.nkv * b->cache_cap * d.d * (long long)d.esz;
        if (b->cache_layer_stride < one) return fail(CCS_EINVAL, "cache_layer_stride %lld is less than one layer's cache (%lld bytes)", (long long)b->cache_layer_stride, one);
        if (b->cache_layer_stride % 16) return fail(CCS_EINVAL, "cache_layer_stride must be a multiple of 16 bytes");
    }
    return CCS_OK;
}

// Rows the kernels work on: for a bf16 prefill the sum of the (validated) lengths, otherwise
// every row of the batch.
long long valid_rows(const ccs_batch *b)
{
    long long t = 0;
    for (int i = 0; i < b->n_seqs; ++i) t += b->lens_host[i] < b->seq_pad ? b->lens_host[i] : b->seq_pad;
    return t;
}
long long batch_rows(const ccs_module *m, const ccs_batch *b)
{
    if (b->mode != CCS_PREFILL) return b->n_seqs;
    return m->desc.dtype == CCS_BF16 ? valid_rows(b) : (long long)b->n_seqs * b->seq_pad;
}

// One replica, one slice.  variant_rows: row count that selects the GEMM variant (the full
// batch's for a replicated forward, so that every replica count produces the same bits).
// ws_static: run in this workspace of ws_static_bytes bytes instead of the replica's own, and
// record no per-kernel timing (that path creates events); used by ccs_module_forward_static.
int forward_one(ccs_module *m, int r, const ccs_batch *b, long long variant_rows, bool on_caller_stream = false,
                hipStream_t caller_stream = nullptr, void *ws_static = nullptr, size_t ws_static_bytes = 0)
{
    using namespace ccs;
    Replica &R = m->rep[r];
    const Dims &d = m->dims;
    const ccs_module_desc &D = m->desc;
    hipStream_t st = on_caller_stream ? caller_stream : R.stream;
    if (b->n_seqs == 0) return CCS_OK;
    const bool bf = D.dtype == CCS_BF16;
    const bool skinny = bf && variant_rows <= kSkinnyMaxRows;
    const bool prof_on = ws_static == nullptr;
    char *ws = ws_static ? (char *)ws_static : (char *)R.ws;
    const size_t ws_bytes = ws_static ? ws_static_bytes : R.ws_bytes;
    const char *A0 = (const char *)R.arena;

    if (D.kind == CCS_LINEAR) {
        const char *A = A0;
        const int M = b->n_seqs;
        // small batches stream the weight in one launch (see linear_streams), larger ones take the LDS-tiled GEMM
        const bool skinny = bf && linear_streams(d.out_f, d.in_f, variant_rows);
        if (!bf) {
            CCS_STAGE(CCS_ST_GEMM_DOWN, launch_gemm_f32((const float *)b->x, (const float *)(A + m->ap.w), nullptr, (float *)b->y, M, d.out_f, d.in_f, st));
            return CCS_OK;
        }
        WsPlan p = ws_plan(&D, d, M, 0, 0, skinny, false, 0, (long)variant_rows);
        if (p.total > ws_bytes) return fail(CCS_ENOMEM, "%s workspace has %zu bytes, batch needs %zu", ws_static ? "the static" : "the replica's", ws_bytes, p.total);
        if (skinny) {   // one launch, straight from the caller's rows
            CCS_STAGE(CCS_ST_GEMM_DOWN, launch_gemm_stream_store(A + m->ap.w, stream_store_shape(d.out_f, d.in_f, (long)variant_rows), b->x, true, false, 0.f, nullptr, b->y, nullptr, M, d.out_f, d.in_f, (float *)(ws + p.scratch), (int *)(ws + p.cnt), st));
            return CCS_OK;
        }
        if (variant_rows <= kDirectRowsMax) {
            // LDS-tiled; its direct-to-LDS loads fetch the fragments straight from the caller's rows.  Those
            // are 16-byte pieces 64 lanes apart, four times the address unit's work of a packed fragment:
            // worth it while the launch is short (it saves the packing launch), a loss of 10 % at 1024 rows
            CCS_STAGE(CCS_ST_GEMM_DOWN, launch_gemm_tiled(A + m->ap.w, b->x, true, EPI_STORE_RM, nullptr, b->y, M, d.out_f, d.in_f, (long)variant_rows, (float *)(ws + p.scratch), st));
            return CCS_OK;
        }
        CCS_STAGE(CCS_ST_PACK_X, launch_pack_bf16(b->x, ws + p.xp, M, d.in_f, 1, 0, false, nullptr, st));
        CCS_STAGE(CCS_ST_GEMM_DOWN, launch_gemm_tiled(A + m->ap.w, ws + p.xp, false, EPI_STORE_RM, nullptr, b->y, M, d.out_f, d.in_f, (long)variant_rows, (float *)(ws + p.scratch), st));
        return CCS_OK;
    }

    const bool attn = has_attn(D.kind), ffn = has_ffn(D.kind);
    const bool decode = b->mode == CCS_DECODE;
    const bool rows_mode = b->mode == CCS_ROWS;   // FFN block: independent token rows
    const int seq_pad = (decode || rows_mode) ? 1 : b->seq_pad;
    // bf16 prefill drops the padding: the kernels see the sum of the lengths as one dense row range
    const bool dense = bf && !decode && !rows_mode;
    const int T = dense ? (int)valid_rows(b) : b->n_seqs * seq_pad;
    WsPlan p = ws_plan(&D, d, T, b->n_seqs, b->cache_cap, skinny, decode, (decode || rows_mode) ? 0 : seq_pad, (long)variant_rows);
    if (p.total > ws_bytes) return fail(CCS_ENOMEM, "%s workspace has %zu bytes, batch needs %zu", ws_static ? "the static" : "the replica's", ws_bytes, p.total);
    const int dt = bf ? DT_BF16 : DT_F32;

    // A run of layers: layer l reads x_in and writes x_out, ping-ponging between two workspace
    // buffers; the first layer reads the batch's x, the last writes its y (Section 3.1: inside a
    // run of consecutive layers nothing is scattered or gathered).
    const int32_t *offs = (const int32_t *)(ws + p.offs);
    if (dense) {
        CCS_STAGE(CCS_ST_COMPACT, launch_prefill_offsets(b->lens_dev, b->n_seqs, seq_pad, T, (int32_t *)(ws + p.offs), st));
        CCS_STAGE(CCS_ST_COMPACT, launch_prefill_rows(const_cast<void *>(b->x), ws + p.xc, offs, b->n_seqs, seq_pad, d.H, false, st));
    }
    bool xp_ready = false;   // weight-streaming path: xp already holds the packed rows of x_in (written by the previous layer's down projection)
    for (int l = 0; l < d.L; ++l) {
        const char *A = A0 + (size_t)l * m->ap.layer;
        const void *x_first = dense ? (const void *)(ws + p.xc) : b->x;
        void *y_last = dense ? (void *)(ws + p.yc) : b->y;
        const void *x_in = l == 0 ? x_first : (const void *)(ws + ((l & 1) ? p.xa : p.xb));
        void *x_out = l == d.L - 1 ? y_last : (void *)(ws + ((l & 1) ? p.xb : p.xa));
        void *kc = b->k_cache ? (char *)b->k_cache + (size_t)l * (size_t)b->cache_layer_stride : nullptr;
        void *vc = b->v_cache ? (char *)b->v_cache + (size_t)l * (size_t)b->cache_layer_stride : nullptr;
        const bool last = l == d.L - 1;

        // x1: the residual stream between the two blocks (the block's input when attention is absent,
        // the module's output when the FFN is absent)
        const void *x1_in = attn ? (ffn ? (const void *)(ws + p.x1) : (const void *)x_out) : x_in;
        void *x1_out = ffn ? (void *)(ws + p.x1) : x_out;
        const void *tab = A + m->ap.rope;
        float *scratch = (float *)(ws + p.scratch);
        if (bf && skinny) {
            // Weight-streaming path (at most 64 rows in the full batch): every projection is one launch
            // that also applies the RMSNorm in front of it (the gains are folded into the weights) and
            // whatever follows it - rotary embedding and cache append, residual, SwiGLU - so a decode
            // step is five launches per layer when the attention kernel merges its own chunks (six
            // with the combine launch, up to eight when Q/K/V and down split K over workgroups).
            // x of the first projection: the packed copy the previous layer of a run left, else the rows themselves
            const void *xq = xp_ready ? (const void *)(ws + p.xp) : x_in;
            const bool xq_rows = !xp_ready;
            if (attn) {
                if (decode && qkv_split(variant_rows)) {
                    CCS_STAGE(CCS_ST_GEMM_QKV, launch_gemm_stream_partials(A + m->ap.qkv, xq, xq_rows, true, scratch, (float *)(ws + p.ssqp), T, d.W3, d.H, st));
                    CCS_STAGE(CCS_ST_GEMM_QKV_REDUCE, launch_qkv_partials_rope_decode(scratch, (const float *)(ws + p.ssqp), skinny_segments(d.W3, d.H), T, d.nq, d.nkv, d.H, D.rms_eps, tab, b->lens_dev, ws + p.qkv, kc, vc, b->cache_cap, st));
                }
                if (decode) {
                    if (!qkv_split(variant_rows))
                        CCS_STAGE(CCS_ST_GEMM_QKV, launch_gemm_stream_qkv_decode(A + m->ap.qkv, xq, xq_rows, D.rms_eps, ws + p.qkv, T, d.nq, d.nkv, d.H, tab, b->lens_dev, kc, vc, b->cache_cap, st));
                    CCS_STAGE(CCS_ST_ATTN, launch_attn_decode_main(ws + p.qkv, scratch, ws + p.a, b->n_seqs, d.nq, d.nkv, b->lens_dev, kc, vc, b->cache_cap, st));
                    if (!attn_decode_is_whole(d.nq, d.nkv)) CCS_STAGE(CCS_ST_ATTN_COMBINE, launch_attn_decode_combine(scratch, ws + p.a, b->n_seqs, d.nq, d.nkv, b->lens_dev, b->cache_cap, st));
                } else {
                    CCS_STAGE(CCS_ST_GEMM_QKV, launch_gemm_stream_store(A + m->ap.qkv, StoreShape{kWGroup, 1}, xq, xq_rows, true, D.rms_eps, nullptr, ws + p.qkv, nullptr, T, d.W3, d.H, nullptr, nullptr, st));
                    CCS_STAGE(CCS_ST_ROPE, launch_rope_pack_prefill(ws + p.qkv, ws + p.kp, ws + p.vtp, b->n_seqs, seq_pad, d.nq, d.nkv, tab, offs, kc, vc, b->cache_cap, st));
                    CCS_STAGE(CCS_ST_ATTN, launch_attn_prefill_mfma(ws + p.qkv, ws + p.kp, ws + p.vtp, ws + p.a, b->n_seqs, seq_pad, d.nq, d.nkv, offs, st));
                }
                CCS_STAGE(CCS_ST_GEMM_O, launch_gemm_stream_store(A + m->ap.o, stream_store_shape(d.H, d.QD, (long)variant_rows), ws + p.a, false, false, 0.f, x_in, x1_out, ffn ? ws + p.x1p : nullptr, T, d.H, d.QD, scratch, (int *)(ws + p.cnt), st));
            }
            if (ffn) {
                if (attn) CCS_STAGE(CCS_ST_GEMM_GU, launch_gemm_stream_swiglu(A + m->ap.gu, ws + p.x1p, false, D.rms_eps, ws + p.u, T, 2 * d.I, d.H, (long)variant_rows, st));
                else CCS_STAGE(CCS_ST_GEMM_GU, launch_gemm_stream_swiglu(A + m->ap.gu, x_in, true, D.rms_eps, ws + p.u, T, 2 * d.I, d.H, (long)variant_rows, st));
                void *next_xp = last ? nullptr : (void *)(ws + p.xp);   // inside a run: the next layer's packed input rows
                if (store_split(d.I, variant_rows)) {
                    CCS_STAGE(CCS_ST_GEMM_DOWN, launch_gemm_stream_partials(A + m->ap.dn, ws + p.u, false, false, scratch, nullptr, T, d.H, d.I, st));
                    CCS_STAGE(CCS_ST_GEMM_DOWN_REDUCE, launch_partial_reduce(scratch, skinny_segments(d.H, d.I), EPI_STORE_RM, x1_in, x_out, next_xp, T, d.H, st));
                } else {
                    CCS_STAGE(CCS_ST_GEMM_DOWN, launch_gemm_stream_store(A + m->ap.dn, stream_store_shape(d.H, d.I, (long)variant_rows), ws + p.u, false, false, 0.f, x1_in, x_out, next_xp, T, d.H, d.I, scratch, (int *)(ws + p.cnt), st));
                }
                xp_ready = !last;
            }
        } else if (bf) {
            // LDS-tiled path: normalised rows h (no gains: they are folded into the weights), one launch
            // per projection (two when K is split)
#define CCS_GEMM(sid, woff, xoff, epi, res, out, N, K) \
    CCS_STAGE(sid, launch_gemm_tiled(A + (woff), ws + (xoff), false, (epi), (res), (out), T, (N), (K), (long)variant_rows, scratch, st))
            CCS_STAGE(attn ? CCS_ST_RMSNORM1 : CCS_ST_RMSNORM2, launch_rmsnorm(dt, x_in, nullptr, ws + p.h, T, d.H, D.rms_eps, st));
            if (attn) {
                CCS_GEMM(CCS_ST_GEMM_QKV, m->ap.qkv, p.h, EPI_STORE_RM, nullptr, ws + p.qkv, d.W3, d.H);
                if (decode) {
                    CCS_STAGE(CCS_ST_ROPE, launch_rope(dt, ws + p.qkv, T, d.nq, d.nkv, d.d, tab, decode, seq_pad, b->lens_dev, kc, vc, b->cache_cap, st));
                    CCS_STAGE(CCS_ST_ATTN, launch_attn_decode_main(ws + p.qkv, scratch, ws + p.a, b->n_seqs, d.nq, d.nkv, b->lens_dev, kc, vc, b->cache_cap, st));
                    if (!attn_decode_is_whole(d.nq, d.nkv)) CCS_STAGE(CCS_ST_ATTN_COMBINE, launch_attn_decode_combine(scratch, ws + p.a, b->n_seqs, d.nq, d.nkv, b->lens_dev, b->cache_cap, st));
                } else {
                    CCS_STAGE(CCS_ST_ROPE, launch_rope_pack_prefill(ws + p.qkv, ws + p.kp, ws + p.vtp, b->n_seqs, seq_pad, d.nq, d.nkv, tab, offs, kc, vc, b->cache_cap, st));
                    CCS_STAGE(CCS_ST_ATTN, launch_attn_prefill_mfma(ws + p.qkv, ws + p.kp, ws + p.vtp, ws + p.a, b->n_seqs, seq_pad, d.nq, d.nkv, offs, st));
                }
                CCS_GEMM(CCS_ST_GEMM_O, m->ap.o, p.a, EPI_STORE_RM, x_in, x1_out, d.H, d.QD);
                if (ffn) CCS_STAGE(CCS_ST_RMSNORM2, launch_rmsnorm(dt, ws + p.x1, nullptr, ws + p.h, T, d.H, D.rms_eps, st));
            }
            if (ffn) {
                CCS_GEMM(CCS_ST_GEMM_GU, m->ap.gu, p.h, EPI_SWIGLU_PACKED, nullptr, ws + p.u, 2 * d.I, d.H);
                CCS_GEMM(CCS_ST_GEMM_DOWN, m->ap.dn, p.u, EPI_STORE_RM, x1_in, x_out, d.H, d.I);
            }
#undef CCS_GEMM
        } else {
            auto W = [&](size_t off) { return (const float *)(A + off); };
            CCS_STAGE(attn ? CCS_ST_RMSNORM1 : CCS_ST_RMSNORM2, launch_rmsnorm(dt, x_in, A + (attn ? m->ap.g1 : m->ap.g2), ws + p.h, T, d.H, D.rms_eps, st));
            if (attn) {
                CCS_STAGE(CCS_ST_GEMM_QKV, launch_gemm_f32((const float *)(ws + p.h), W(m->ap.qkv), nullptr, (float *)(ws + p.qkv), T, d.W3, d.H, st));
                CCS_STAGE(CCS_ST_ROPE, launch_rope(dt, ws + p.qkv, T, d.nq, d.nkv, d.d, tab, decode, seq_pad, b->lens_dev, kc, vc, b->cache_cap, st));
                CCS_STAGE(CCS_ST_ATTN, launch_attn_generic(dt, ws + p.qkv, ws + p.a, T, d.nq, d.nkv, d.d, decode, seq_pad, b->lens_dev, kc, vc, b->cache_cap, st));
                CCS_STAGE(CCS_ST_GEMM_O, launch_gemm_f32((const float *)(ws + p.a), W(m->ap.o), (const float *)x_in, (float *)x1_out, T, d.H, d.QD, st));
                if (ffn) CCS_STAGE(CCS_ST_RMSNORM2, launch_rmsnorm(dt, ws + p.x1, A + m->ap.g2, ws + p.h, T, d.H, D.rms_eps, st));
            }
            if (ffn) {
                CCS_STAGE(CCS_ST_GEMM_GU, launch_gemm_f32((const float *)(ws + p.h), W(m->ap.gu), nullptr, (float *)(ws + p.gu), T, 2 * d.I, d.H, st));
                CCS_STAGE(CCS_ST_GEMM_GU_REDUCE, launch_swiglu_f32((const float *)(ws + p.gu), (float *)(ws + p.u), T, d.I, st));
                CCS_STAGE(CCS_ST_GEMM_DOWN, launch_gemm_f32((const float *)(ws + p.u), W(m->ap.dn), (const float *)x1_in, (float *)x_out, T, d.H, d.I, st));
            }
        }
    }
    if (dense) CCS_STAGE(CCS_ST_EXPAND, launch_prefill_rows(b->y, ws + p.yc, offs, b->n_seqs, seq_pad, d.H, true, st));
    return CCS_OK;
}

// Order `st` after a slice 0 that a replicated forward ran on a caller's stream.
int wait_slice0(ccs_module *m, int replica, hipStream_t st)
{
    if (replica == 0 && m->slice0_recorded) CCS_HIP(hipStreamWaitEvent(st, m->slice0_done, 0));
    return CCS_OK;
}

}  // namespace

extern "C" {

const char *ccs_last_error(void) { return g_err; }
const char *ccs_version(void) { return "cocoserve_mi 0.1 (gfx950)"; }

size_t ccs_module_arena_bytes(const ccs_module_desc *desc)
{
    Dims d;
    if (check_desc(desc, &d) != CCS_OK) return 0;
    return arena_plan(desc, d).total;
}

size_t ccs_module_workspace_bytes(const ccs_module_desc *desc, int32_t max_seqs, int32_t max_seq_pad,
                                  int32_t max_cache_cap)
{
    Dims d;
    if (check_desc(desc, &d) != CCS_OK) return 0;
    if (max_seqs < 0 || max_seq_pad < 1 || max_cache_cap < 0) {
        fail(CCS_EINVAL, "negative sizes");
        return 0;
    }
    const size_t rows = (size_t)max_seqs * max_seq_pad;
    const bool skinny = rows <= (size_t)ccs::kSkinnyMaxRows;
    const bool layer = has_attn(desc->kind);
    // cover every plan a batch within these limits can take: prefill (max_seq_pad rows per
    // sequence), decode (one row per sequence, when a cache size is given), either GEMM variant
    size_t need = ws_plan(desc, d, rows, max_seqs, max_cache_cap, skinny, false, layer ? max_seq_pad : 0).total;
    // smaller batches may split K in the tiled GEMM: the partial buffer grows with the split
    for (size_t v = 128; v < rows && v <= 4096; v += 128) {
        // (a bf16 prefill works on the valid rows only, so few rows can come with many sequences)
        need = max_sz(need, ws_plan(desc, d, v, max_seqs, max_cache_cap, false, false, layer ? max_seq_pad : 0).total);
    }
    if (!skinny) {
        need = max_sz(need, ws_plan(desc, d, ccs::kSkinnyMaxRows, max_seqs, max_cache_cap, true, false, layer ? max_seq_pad : 0).total);
    }
    if (desc->kind == CCS_LINEAR && rows > (size_t)kLinearStreamRowsMax)   // a small batch takes the weight-streaming launch, which may split K
        need = max_sz(need, ws_plan(desc, d, rows < (size_t)ccs::kSkinnyMaxRows ? rows : (size_t)ccs::kSkinnyMaxRows, max_seqs, 0, true, false, 0).total);
    if (layer && max_cache_cap > 0) {
        const bool dsk = max_seqs <= ccs::kSkinnyMaxRows;
        need = max_sz(need, ws_plan(desc, d, max_seqs, max_seqs, max_cache_cap, dsk, true, 0).total);
        if (!dsk) need = max_sz(need, ws_plan(desc, d, ccs::kSkinnyMaxRows, ccs::kSkinnyMaxRows, max_cache_cap, true, true, 0).total);
    }
    return need ? need : 256;
}

int ccs_module_create(const ccs_module_desc *desc, const ccs_weights *w, void *arena0, void *workspace0,
                      size_t workspace_bytes, void *stream, ccs_module **out)
{
    using namespace ccs;
    if (!out) return fail(CCS_EINVAL, "out is null");
    *out = nullptr;
    Dims d;
    int rc = check_desc(desc, &d);
    if (rc != CCS_OK) return rc;
    if (!w || !arena0 || !workspace0) return fail(CCS_EINVAL, "weights / arena0 / workspace0 is null");
    if (((uintptr_t)arena0 & 255) || ((uintptr_t)workspace0 & 255)) return fail(CCS_EINVAL, "arena0 / workspace0 must be 256-byte aligned");
    if (desc->kind == CCS_LINEAR) {
        if (!w->w) return fail(CCS_EINVAL, "weights.w is null");
    } else {
        for (int l = 0; l < d.L; ++l) {
            if (has_attn(desc->kind) && (!w[l].wq || !w[l].wk || !w[l].wv || !w[l].wo || !w[l].g1))
                return fail(CCS_EINVAL, "an attention weight pointer of layer %d is null", l);
            if (has_ffn(desc->kind) && (!w[l].wgate || !w[l].wup || !w[l].wdown || !w[l].g2))
                return fail(CCS_EINVAL, "an FFN weight pointer of layer %d is null", l);
        }
    }
    int ndev = 0;
    CCS_HIP(hipGetDeviceCount(&ndev));
    if (ndev < 1) return fail(CCS_EHIP, "no HIP device");
    {   // kernel attributes: once per process, here rather than in a forward (which may be captured)
        static std::once_flag once;
        static hipError_t init_err = hipSuccess;
        std::call_once(once, [] {
            init_err = ccs::init_gemm_kernels();
            if (init_err == hipSuccess) init_err = ccs::init_attention_kernels();
        });
        if (init_err != hipSuccess) return fail(CCS_EHIP, "kernel attributes: %s", hipGetErrorString(init_err));
    }

    {   // the static workspace's address on this device, resolved at set-up rather than in a forward
        void *sws = nullptr;
        rc = static_workspace(&sws);
        if (rc != CCS_OK) return rc;
    }
    ccs_module *m = new (std::nothrow) ccs_module();
    if (!m) return fail(CCS_ENOMEM, "host allocation failed");
    m->desc = *desc;
    m->dims = d;
    m->ap = arena_plan(desc, d);
    hipStream_t st = (hipStream_t)stream;
    const bool bf = desc->dtype == CCS_BF16;
    hipError_t e = hipSuccess;
    for (int l = 0; l < d.L; ++l) {
        char *A = (char *)arena0 + (size_t)l * m->ap.layer;
        const ccs_weights *wl = w + l;
        auto rm_copy = [&](size_t off, const void *src, size_t bytes) { if (e == hipSuccess) e = launch_clone(A + off, src, bytes, st); };
        // gain: the gains of the RMSNorm in front of the projection, folded into its weight
        // (W[n, k] * g[k], rounded to bf16): RMSNorm(x; g) W^T = (x / rms(x)) (W diag(g))^T
        auto pack = [&](size_t off, const void *src, int N, int K, int stride, int blk_off, const void *gain = nullptr) {
            if (e == hipSuccess) e = launch_pack_bf16(src, A + off, N, K, stride, blk_off, true, gain, st);
        };
        // padding fragments of a weight whose block count is not a multiple of the group must be zero
        auto zero_if_padded = [&](size_t off, int N, int K) {
            if (e == hipSuccess && bf && ccs::packed_weight_bytes(N, K) != (size_t)N * K * 2)
                e = hipMemsetAsync(A + off, 0, ccs::packed_weight_bytes(N, K), st);
        };
        if (desc->kind == CCS_LINEAR) {
            zero_if_padded(m->ap.w, d.out_f, d.in_f);
            if (bf) pack(m->ap.w, wl->w, d.out_f, d.in_f, 1, 0);
            else rm_copy(m->ap.w, wl->w, (size_t)d.out_f * d.in_f * 4);
        } else if (bf) {
            if (has_attn(desc->kind)) {
                zero_if_padded(m->ap.qkv, d.W3, d.H);
                zero_if_padded(m->ap.o, d.H, d.QD);
                pack(m->ap.qkv, wl->wq, d.QD, d.H, 1, 0, wl->g1);
                pack(m->ap.qkv, wl->wk, d.KD, d.H, 1, d.QD / 16, wl->g1);
                pack(m->ap.qkv, wl->wv, d.KD, d.H, 1, (d.QD + d.KD) / 16, wl->g1);
                pack(m->ap.o, wl->wo, d.H, d.QD, 1, 0);
                rm_copy(m->ap.g1, wl->g1, (size_t)d.H * 2);
            }
            if (has_ffn(desc->kind)) {
                zero_if_padded(m->ap.gu, 2 * d.I, d.H);
                zero_if_padded(m->ap.dn, d.H, d.I);
                pack(m->ap.gu, wl->wgate, d.I, d.H, 2, 0, wl->g2);  // gate blocks even, up blocks odd
                pack(m->ap.gu, wl->wup, d.I, d.H, 2, 1, wl->g2);
                pack(m->ap.dn, wl->wdown, d.H, d.I, 1, 0);
                rm_copy(m->ap.g2, wl->g2, (size_t)d.H * 2);
            }
        } else {
            const size_t rowb = (size_t)d.H * 4;
            if (has_attn(desc->kind)) {
                rm_copy(m->ap.qkv, wl->wq, d.QD * rowb);
                rm_copy(m->ap.qkv + d.QD * rowb, wl->wk, d.KD * rowb);
                rm_copy(m->ap.qkv + (d.QD + d.KD) * rowb, wl->wv, d.KD * rowb);
                rm_copy(m->ap.o, wl->wo, (size_t)d.H * d.QD * 4);
                rm_copy(m->ap.g1, wl->g1, rowb);
            }
            if (has_ffn(desc->kind)) {
                rm_copy(m->ap.gu, wl->wgate, d.I * rowb);
                rm_copy(m->ap.gu + d.I * rowb, wl->wup, d.I * rowb);
                rm_copy(m->ap.dn, wl->wdown, (size_t)d.H * d.I * 4);
                rm_copy(m->ap.g2, wl->g2, rowb);
            }
        }
        if (e == hipSuccess && has_attn(desc->kind)) e = launch_rope_table(A + m->ap.rope, d.d, desc->rope_base, st);
    }
    if (e != hipSuccess) {
        delete m;
        return fail(CCS_EHIP, "packing weights: %s", hipGetErrorString(e));
    }
    Replica &R = m->rep[0];
    R.arena = arena0; R.ws = workspace0; R.ws_bytes = workspace_bytes; R.stream = st;
    auto drop = [&] {
        drop_events(R);
        if (m->fork) (void)hipEventDestroy(m->fork);
        if (m->slice0_done) (void)hipEventDestroy(m->slice0_done);
        prof_free(R);
        delete m;
    };
    if (make_event(&R.ready) != CCS_OK || make_event(&R.done) != CCS_OK || make_event(&m->fork) != CCS_OK ||
        make_event(&m->slice0_done) != CCS_OK) {
        drop();
        return CCS_EHIP;
    }
    e = workspace_bytes >= kCounterBytes ? hipMemsetAsync(workspace0, 0, kCounterBytes, st) : hipSuccess;
    if (e == hipSuccess) e = hipEventRecord(R.ready, st);
    if (e != hipSuccess) { drop(); return fail(CCS_EHIP, "attaching the workspace: %s", hipGetErrorString(e)); }
    m->k = 1;
    *out = m;
    return CCS_OK;
}

int ccs_module_replicate(ccs_module *m, int32_t k, void *const *arenas, void *const *workspaces,
                         size_t workspace_bytes, void *const *streams)
{
    if (!m) return fail(CCS_EINVAL, "module is null");
    if (k < 1 || k > CCS_MAX_REPLICAS) return fail(CCS_EINVAL, "k = %d outside [1, %d]", k, (int)CCS_MAX_REPLICAS);
    if (k < m->k) {
        for (int j = k; j < m->k; ++j) {
            Replica &R = m->rep[j];
            CCS_HIP(hipStreamSynchronize(R.stream));
            if (R.ready) (void)hipEventDestroy(R.ready);
            if (R.done) (void)hipEventDestroy(R.done);
            prof_free(R);
            R = Replica();
        }
        m->k = k;
        return CCS_OK;
    }
    if (k == m->k) return CCS_OK;
    if (!arenas || !workspaces || !streams) return fail(CCS_EINVAL, "arenas / workspaces / streams is null");
    for (int j = m->k; j < k; ++j) {
        if (!arenas[j] || !workspaces[j]) return fail(CCS_EINVAL, "arena / workspace of replica %d is null", j);
        if (((uintptr_t)arenas[j] & 255) || ((uintptr_t)workspaces[j] & 255)) return fail(CCS_EINVAL, "buffers of replica %d must be 256-byte aligned", j);
        for (int i = 0; i < j; ++i) {
            void *other = i < m->k ? m->rep[i].arena : arenas[i];
            if (other == arenas[j]) return fail(CCS_EINVAL, "replica %d would share replica %d's arena", j, i);
        }
    }
    for (int j = m->k; j < k; ++j) {
        Replica R;
        R.arena = arenas[j]; R.ws = workspaces[j]; R.ws_bytes = workspace_bytes; R.stream = (hipStream_t)streams[j];
        int rc = make_event(&R.ready);
        if (rc == CCS_OK) rc = make_event(&R.done);
        if (rc == CCS_OK) {
            m->rep[j] = R;
            m->k = j + 1;
        } else {
            drop_events(R);
            return rc;
        }
        Replica &N = m->rep[j];
        auto undo = [&] { prof_free(N); drop_events(N); N = Replica(); m->k = j; };   // earlier new replicas stay
        hipError_t e = hipStreamWaitEvent(N.stream, m->rep[0].ready, 0);
        if (e == hipSuccess) {
            ProfPair *pp = prof_begin(m, N, CCS_ST_CLONE, N.stream);
            e = ccs::launch_clone(N.arena, m->rep[0].arena, m->ap.total, N.stream);
            prof_end(pp, N.stream);
        }
        if (e == hipSuccess && N.ws_bytes >= kCounterBytes) e = hipMemsetAsync(N.ws, 0, kCounterBytes, N.stream);
        if (e == hipSuccess) e = hipEventRecord(N.ready, N.stream);
        if (e != hipSuccess) {
            undo();
            return fail(CCS_EHIP, "cloning replica %d: %s", j, hipGetErrorString(e));
        }
    }
    return CCS_OK;
}

int ccs_module_replicas(const ccs_module *m)
{
    if (!m) return fail(CCS_EINVAL, "module is null");
    return m->k;
}

int ccs_module_forward(ccs_module *m, int32_t replica, const ccs_batch *slice)
{
    if (!m) return fail(CCS_EINVAL, "module is null");
    if (replica < 0 || replica >= CCS_MAX_REPLICAS) return fail(CCS_EINVAL, "replica index %d out of range", replica);
    if (replica >= m->k) return fail(CCS_ESTATE, "replica %d is not instantiated (module has %d)", replica, m->k);
    int rc = check_batch(m, slice);
    if (rc != CCS_OK) return rc;
    rc = wait_slice0(m, replica, m->rep[replica].stream);
    if (rc != CCS_OK) return rc;
    return forward_one(m, replica, slice, batch_rows(m, slice));
}

int ccs_module_forward_static(ccs_module *m, int32_t replica, const ccs_batch *slice)
{
    if (!m) return fail(CCS_EINVAL, "module is null");
    if (replica < 0 || replica >= CCS_MAX_REPLICAS) return fail(CCS_EINVAL, "replica index %d out of range", replica);
    if (replica >= m->k) return fail(CCS_ESTATE, "replica %d is not instantiated (module has %d)", replica, m->k);
    int rc = check_batch(m, slice);
    if (rc != CCS_OK) return rc;
    void *ws = nullptr;
    rc = static_workspace(&ws);
    if (rc != CCS_OK) return rc;
    rc = wait_slice0(m, replica, m->rep[replica].stream);
    if (rc != CCS_OK) return rc;
    return forward_one(m, replica, slice, batch_rows(m, slice), false, nullptr, ws, (size_t)CCS_STATIC_WORKSPACE_BYTES);
}

size_t ccs_static_workspace_bytes(void) { return (size_t)CCS_STATIC_WORKSPACE_BYTES; }

// Slice j = sequences [bounds[j], bounds[j + 1]) on replica j; slice 0 on the caller's stream.
static int forward_bounds(ccs_module *m, const ccs_batch *full, const long long *bounds, hipStream_t cs)
{
    const int k = m->k;
    const long long n = full->n_seqs;
    if (n == 0) return CCS_OK;
    const bool prefill = full->mode == CCS_PREFILL;
    const long long rows_per_seq = prefill ? full->seq_pad : 1;
    const long long full_rows = batch_rows(m, full);   // selects the kernel variants of every slice
    const Dims &d = m->dims;
    const size_t esz = d.esz;
    const size_t x_row = (m->desc.kind == CCS_LINEAR ? (size_t)d.in_f : (size_t)d.H) * esz;
    const size_t y_row = (m->desc.kind == CCS_LINEAR ? (size_t)d.out_f : (size_t)d.H) * esz;
    const size_t cache_seq = (size_t)d.nkv * (size_t)full->cache_cap * d.d * esz;

    // Slice 0 uses replica 0's arena and workspace from the caller's stream.  When that is not
    // replica 0's own stream, order it after whatever filled or moved the arena, and leave an event
    // behind that copies, migrations and later forwards of replica 0 wait for.  (Not while the
    // caller is capturing: events recorded outside a capture cannot be tied into it, and an event
    // recorded inside one must not leak out; a capturing caller orders these itself.)
    const bool foreign = cs != m->rep[0].stream;
    bool capturing = false;
    if (foreign) {
        hipStreamCaptureStatus cst = hipStreamCaptureStatusNone;
        CCS_HIP(hipStreamIsCapturing(cs, &cst));
        capturing = cst != hipStreamCaptureStatusNone;
        if (!capturing) {
            CCS_HIP(hipEventRecord(m->rep[0].done, m->rep[0].stream));   // replica 0's own earlier forwards
            CCS_HIP(hipStreamWaitEvent(cs, m->rep[0].done, 0));
            CCS_HIP(hipStreamWaitEvent(cs, m->rep[0].ready, 0));
        }
    }
    if (k > 1) CCS_HIP(hipEventRecord(m->fork, cs));
    for (int j = 0; j < k; ++j) {
        const long long lo = bounds[j], hi = bounds[j + 1];
        if (hi == lo) continue;
        Replica &R = m->rep[j];
        ccs_batch s = *full;
        s.n_seqs = (int32_t)(hi - lo);
        s.x = (const char *)full->x + (size_t)lo * rows_per_seq * x_row;
        s.y = (char *)full->y + (size_t)lo * rows_per_seq * y_row;
        if (full->lens_host) s.lens_host = full->lens_host + lo;
        if (full->lens_dev) s.lens_dev = full->lens_dev + lo;
        if (full->k_cache) {
            s.k_cache = (char *)full->k_cache + (size_t)lo * cache_seq;
            s.v_cache = (char *)full->v_cache + (size_t)lo * cache_seq;
        }
        // slice 0 runs on the caller's stream itself (no events at k = 1); the others fork and join
        const bool inline_ = (j == 0) || R.stream == cs;
        if (!inline_) CCS_HIP(hipStreamWaitEvent(R.stream, m->fork, 0));
        const int rc = forward_one(m, j, &s, full_rows, inline_, cs);
        if (!inline_) {
            // join also when the slice failed half-way: the stream was forked, and a caller that
            // captures must get every forked stream back
            const hipError_t e1 = hipEventRecord(R.done, R.stream);
            const hipError_t e2 = e1 == hipSuccess ? hipStreamWaitEvent(cs, R.done, 0) : e1;
            if (rc == CCS_OK && e2 != hipSuccess) return fail(CCS_EHIP, "joining replica %d: %s", j, hipGetErrorString(e2));
        }
        if (rc != CCS_OK) return rc;   // earlier slices are already joined
    }
    if (foreign && !capturing && bounds[1] > bounds[0]) {
        CCS_HIP(hipEventRecord(m->slice0_done, cs));
        m->slice0_recorded = true;
    }
    return CCS_OK;
}


int ccs_module_forward_split(ccs_module *m, const ccs_batch *full, void *caller_stream)
{
    if (!m) return fail(CCS_EINVAL, "module is null");
    int rc = check_batch(m, full);
    if (rc != CCS_OK) return rc;
    long long bounds[CCS_MAX_REPLICAS + 1];
    const long long n = full->n_seqs;
    for (int j = 0; j <= m->k; ++j) bounds[j] = j * n / m->k;  // slice j = [floor(jn/k), floor((j+1)n/k))
    return forward_bounds(m, full, bounds, (hipStream_t)caller_stream);
}

int ccs_module_forward_shares(ccs_module *m, const ccs_batch *full, const int32_t *counts, void *caller_stream)
{
    if (!m) return fail(CCS_EINVAL, "module is null");
    if (!counts) return fail(CCS_EINVAL, "counts is null");
    int rc = check_batch(m, full);
    if (rc != CCS_OK) return rc;
    long long bounds[CCS_MAX_REPLICAS + 1];
    bounds[0] = 0;
    for (int j = 0; j < m->k; ++j) {
        if (counts[j] < 0) return fail(CCS_EINVAL, "counts[%d] = %d is negative", j, counts[j]);
        bounds[j + 1] = bounds[j] + counts[j];
    }
    if (bounds[m->k] != full->n_seqs)
        return fail(CCS_EINVAL, "counts add up to %lld, the batch has %d", bounds[m->k], full->n_seqs);
    return forward_bounds(m, full, bounds, (hipStream_t)caller_stream);
}

int ccs_module_copy(ccs_module *m, int32_t replica, void *dst_arena, void *stream)
{
    if (!m) return fail(CCS_EINVAL, "module is null");
    if (replica < 0 || replica >= CCS_MAX_REPLICAS) return fail(CCS_EINVAL, "replica index %d out of range", replica);
    if (replica >= m->k) return fail(CCS_ESTATE, "replica %d is not instantiated", replica);
    if (!dst_arena || ((uintptr_t)dst_arena & 255)) return fail(CCS_EINVAL, "dst_arena is null or not 256-byte aligned");
    Replica &R = m->rep[replica];
    if (dst_arena == R.arena) return fail(CCS_EINVAL, "dst_arena is the replica's own arena");
    hipStream_t st = (hipStream_t)stream;
    if (st != R.stream) {
        // order after everything the replica has enqueued so far (its pack/clone included)
        CCS_HIP(hipEventRecord(R.done, R.stream));
        CCS_HIP(hipStreamWaitEvent(st, R.done, 0));
    }
    {   // ... and after a slice 0 that ran on some caller's stream
        const int rc0 = wait_slice0(m, replica, st);
        if (rc0 != CCS_OK) return rc0;
    }
    const bool prof_on = true;
    CCS_STAGE(CCS_ST_CLONE, ccs::launch_clone(dst_arena, R.arena, m->ap.total, st));
    return CCS_OK;
}

int ccs_module_migrate(ccs_module *m, int32_t replica, void *dst_arena, void *stream)
{
    int rc = ccs_module_copy(m, replica, dst_arena, stream);
    if (rc != CCS_OK) return rc;
    Replica &R = m->rep[replica];
    hipStream_t st = (hipStream_t)stream;
    CCS_HIP(hipEventRecord(R.ready, st));
    if (st != R.stream) CCS_HIP(hipStreamWaitEvent(R.stream, R.ready, 0));
    R.arena = dst_arena;
    return CCS_OK;
}

int ccs_cache_copy(void *dst, const void *src, size_t bytes, void *stream)
{
    if (bytes == 0) return CCS_OK;
    if (!dst || !src) return fail(CCS_EINVAL, "dst / src is null");
    if (((uintptr_t)dst & 15) || ((uintptr_t)src & 15)) return fail(CCS_EINVAL, "dst / src must be 16-byte aligned");
    const char *s = (const char *)src;
    char *t = (char *)dst;
    if ((s < t + bytes) && (t < s + bytes)) return fail(CCS_EINVAL, "src and dst overlap");
    CCS_HIP(ccs::launch_clone(dst, src, bytes, (hipStream_t)stream));
    return CCS_OK;
}

int ccs_module_arena(const ccs_module *m, int32_t replica, void **arena_out)
{
    if (!m || !arena_out) return fail(CCS_EINVAL, "null argument");
    if (replica < 0 || replica >= m->k) return fail(CCS_ESTATE, "replica %d is not instantiated", replica);
    *arena_out = m->rep[replica].arena;
    return CCS_OK;
}

int ccs_module_profile(ccs_module *m, uint32_t stage_mask)
{
    if (!m) return fail(CCS_EINVAL, "module is null");
    if (stage_mask >> CCS_N_STAGES) return fail(CCS_EINVAL, "stage_mask has bits beyond CCS_N_STAGES");
    m->prof_mask = stage_mask;
    return CCS_OK;
}

int ccs_module_profile_read(ccs_module *m, int32_t replica, double *ms_sum, int64_t *count, int32_t reset)
{
    if (!m || !ms_sum || !count) return fail(CCS_EINVAL, "null argument");
    if (replica < 0 || replica >= m->k) return fail(CCS_ESTATE, "replica %d is not instantiated", replica);
    Replica &R = m->rep[replica];
    for (int i = 0; i < CCS_N_STAGES; ++i) { ms_sum[i] = 0.0; count[i] = 0; }
    if (!R.prof) return CCS_OK;
    Prof &P = *R.prof;
    for (auto &p : P.pending) {
        CCS_HIP(hipEventSynchronize(p.b));
        float ms = 0.f;
        CCS_HIP(hipEventElapsedTime(&ms, p.a, p.b));
        P.ms[p.stage] += ms;
        P.count[p.stage] += 1;
        P.pool.push_back(p);
    }
    P.pending.clear();
    for (int i = 0; i < CCS_N_STAGES; ++i) { ms_sum[i] = P.ms[i]; count[i] = P.count[i]; }
    if (reset)
        for (int i = 0; i < CCS_N_STAGES; ++i) { P.ms[i] = 0.0; P.count[i] = 0; }
    return CCS_OK;
}

int ccs_module_sync(ccs_module *m)
{
    if (!m) return fail(CCS_EINVAL, "module is null");
    for (int j = 0; j < m->k; ++j) CCS_HIP(hipStreamSynchronize(m->rep[j].stream));
    if (m->slice0_recorded) CCS_HIP(hipEventSynchronize(m->slice0_done));
    return CCS_OK;
}

int ccs_module_destroy(ccs_module *m)
{
    if (!m) return fail(CCS_EINVAL, "module is null");
    for (int j = 0; j < m->k; ++j) {
        Replica &R = m->rep[j];
        (void)hipStreamSynchronize(R.stream);
        if (R.ready) (void)hipEventDestroy(R.ready);
        if (R.done) (void)hipEventDestroy(R.done);
        prof_free(R);
    }
    if (m->slice0_recorded) (void)hipEventSynchronize(m->slice0_done);
    if (m->fork) (void)hipEventDestroy(m->fork);
    if (m->slice0_done) (void)hipEventDestroy(m->slice0_done);
    delete m;
    return CCS_OK;
}

}  // extern "C"
