/*
 * CPU oracle for the module-replica hot path (TEST INFRASTRUCTURE ONLY).
 *
 * This file is the slow, plain definition of what one module forward computes
 * and of how a batch is split over replicas and gathered back.  It exists so
 * that the GPU library can be checked against something that shares no code
 * with it.  Only tests, the smoke check and the benchmark's CPU-baseline leg
 * may load it; the product path never does.
 *
 * What the paper fixes (and where):
 *   - a module is a decoder layer, its attention / FFN block, one projection,
 *     or a KV cache (Section 1 footnote on modules; Section 2.1 lists the
 *     q/k/v/o and the three FFN projections with their dimensions);
 *   - replication runs the unmodified module on contiguous slices of the
 *     batch, 15 requests becoming 7 and 8, and collects the outputs in order
 *     (Section 3.1 "Replication"); model semantics must be preserved
 *     (Section 3.1, correctness paragraph);
 *   - prefill handles a whole prompt, decode one token against the KV cache
 *     (Section 2.1).
 * The paper never writes the layer arithmetic down; it is the public
 * LLaMA-2 pre-norm layer: RMSNorm, q/k/v projections, split-half rotary
 * embedding, causal softmax attention (grouped-query when n_kv < n_q),
 * o projection + residual, RMSNorm, silu(gate)*up, down projection + residual.
 *
 * Precision: inputs and outputs are fp32 arrays; every intermediate value and
 * every accumulation is fp64 and nothing is rounded between steps.
 * There is no tiling, fusion or reordering: each function is the definition.
 *
 * Parity pins (tests/test_oracle_*.py): rotary closed forms, softmax/attention
 * invariants and a pure-Python brute force, library fp64 routines for the
 * projections, norm, silu and attention, prefill == prefill + one decode step,
 * split == unsplit, and the parameter/byte/FLOP figures of Table 1.
 * Whole-layer values at 7B/13B/70B shapes are printed nowhere in the paper:
 * at those sizes parity rests on the pinned pieces ("parity unpinned" for the
 * full-size layer as a whole).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int hidden;        /* H */
    int n_q_heads;     /* query heads */
    int n_kv_heads;    /* key/value heads, divides n_q_heads */
    int head_dim;      /* d, even */
    int intermediate;  /* I, SwiGLU width */
    double rms_eps;
    double rope_base;
} orc_layer_desc;

/* all matrices [out_features, in_features] row-major, y = x W^T */
typedef struct {
    const float *wq, *wk, *wv, *wo, *wgate, *wup, *wdown, *g1, *g2;
} orc_layer_weights;

/* ---- split rule: Section 3.1 "Replication" (15 -> 7 + 8) ---------------- */
/* bounds[j] = floor(j*n/k), j = 0..k; slice j is [bounds[j], bounds[j+1]). */
void orc_split_bounds(int64_t n, int k, int64_t *bounds)
{
    for (int j = 0; j <= k; ++j) bounds[j] = (j * n) / k;
}

/* ---- RMSNorm: "layer normalization" of Section 2.1, LLaMA form ---------- */
/* out[t,c] = x[t,c] / sqrt(mean_c x[t,c]^2 + eps) * g[c] */
void orc_rmsnorm_f64(const double *x, const float *g, double eps, int64_t T, int H, double *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        const double *xr = x + t * H;
        double ss = 0.0;
        for (int c = 0; c < H; ++c) ss += xr[c] * xr[c];
        double r = 1.0 / sqrt(ss / (double)H + eps);
        for (int c = 0; c < H; ++c) out[t * H + c] = xr[c] * r * (double)g[c];
    }
}

/* ---- projection: a linear map without bias (Section 2.1) ---------------- */
/* y[t,n] = sum_k x[t,k] * W[n,k] */
void orc_linear_f64(const double *x, const float *W, int64_t T, int K, int N, double *y)
{
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        const float *wr = W + (int64_t)n * K;
        for (int64_t t = 0; t < T; ++t) {
            const double *xr = x + t * K;
            double acc = 0.0;
#pragma omp simd reduction(+ : acc)
            for (int k = 0; k < K; ++k) acc += xr[k] * (double)wr[k];
            y[t * N + n] = acc;
        }
    }
}

/* ---- rotary embedding, split-half pairing (i, i + d/2) ------------------ */
/* theta_i = base^(-2i/d); pair rotated by angle pos * theta_i. */
void orc_rope_f64(double *z, int d, int64_t pos, double base)
{
    int half = d / 2;
    for (int i = 0; i < half; ++i) {
        double theta = pow(base, -2.0 * (double)i / (double)d);
        double ang = (double)pos * theta;
        double c = cos(ang), s = sin(ang);
        double a = z[i], b = z[i + half];
        z[i] = a * c - b * s;
        z[i + half] = b * c + a * s;
    }
}

/* ---- one query against n_keys visible keys ------------------------------ */
/* s_j = q.k_j / sqrt(d); p = softmax(s); out = sum_j p_j v_j.
 * keys/vals: row j at keys + j*stride.  probs (optional) receives p. */
static void attend_one(const double *q, const double *keys, const double *vals, int64_t n_keys,
                       int d, int64_t stride, double *out, double *probs)
{
    double *s = (double *)malloc(sizeof(double) * (size_t)n_keys);
    double inv = 1.0 / sqrt((double)d), mx = -INFINITY;
    for (int64_t j = 0; j < n_keys; ++j) {
        double acc = 0.0;
        for (int c = 0; c < d; ++c) acc += q[c] * keys[j * stride + c];
        s[j] = acc * inv;
        if (s[j] > mx) mx = s[j];
    }
    double den = 0.0;
    for (int64_t j = 0; j < n_keys; ++j) { s[j] = exp(s[j] - mx); den += s[j]; }
    for (int c = 0; c < d; ++c) out[c] = 0.0;
    for (int64_t j = 0; j < n_keys; ++j) {
        double p = s[j] / den;
        if (probs) probs[j] = p;
        for (int c = 0; c < d; ++c) out[c] += p * vals[j * stride + c];
    }
    free(s);
}

void orc_attend_f64(const double *q, const double *keys, const double *vals, int64_t n_keys, int d,
                    int64_t stride, double *out, double *probs)
{
    attend_one(q, keys, vals, n_keys, d, stride, out, probs);
}

static double silu(double z) { return z / (1.0 + exp(-z)); }

/* The layer's two halves (Section 3.3, Table 1 treats self-attention and FFN as modules of
 * their own).  Each half carries its norm and its residual, so the layer is the attention
 * block followed by the FFN block.  rows: T. */
/* x1 = x + a Wo^T, a = the attention output of RMSNorm(x; g1) */
static void attention_output(const orc_layer_desc *D, const orc_layer_weights *w, const double *x,
                             const double *a, int64_t T, double *x1)
{
    int H = D->hidden, QD = D->n_q_heads * D->head_dim;
    orc_linear_f64(a, w->wo, T, QD, H, x1);
    for (int64_t i = 0; i < T * H; ++i) x1[i] += x[i];
}

/* y = x1 + (silu(h2 Wg^T) * (h2 Wu^T)) Wd^T, h2 = RMSNorm(x1; g2) */
static void ffn_block(const orc_layer_desc *D, const orc_layer_weights *w, const double *x1, int64_t T,
                      double *y)
{
    int H = D->hidden, I = D->intermediate;
    double *h2 = (double *)malloc(sizeof(double) * (size_t)(T * H));
    double *gt = (double *)malloc(sizeof(double) * (size_t)(T * I));
    double *up = (double *)malloc(sizeof(double) * (size_t)(T * I));
    orc_rmsnorm_f64(x1, w->g2, D->rms_eps, T, H, h2);
    orc_linear_f64(h2, w->wgate, T, H, I, gt);
    orc_linear_f64(h2, w->wup, T, H, I, up);
    for (int64_t i = 0; i < T * I; ++i) gt[i] = silu(gt[i]) * up[i];
    orc_linear_f64(gt, w->wdown, T, I, H, y);
    for (int64_t i = 0; i < T * H; ++i) y[i] += x1[i];
    free(h2); free(gt); free(up);
}

/* Steps after attention, shared by prefill and decode because the layer is the
 * same in both phases.  parts: 1 = stop after the attention block (y = x1), 3 = whole layer. */
static void post_attention(const orc_layer_desc *D, const orc_layer_weights *w, const double *x,
                           const double *a, int64_t T, double *y, int parts)
{
    int H = D->hidden;
    if (!(parts & 2)) {
        attention_output(D, w, x, a, T, y);
        return;
    }
    double *x1 = (double *)malloc(sizeof(double) * (size_t)(T * H));
    attention_output(D, w, x, a, T, x1);
    ffn_block(D, w, x1, T, y);
    free(x1);
}

/* FFN block on independent token rows: x, y [T, H] fp32 */
void orc_ffn_block(const orc_layer_desc *D, const orc_layer_weights *w, const float *x, int64_t T, float *y)
{
    int H = D->hidden;
    double *xd = (double *)malloc(sizeof(double) * (size_t)(T * H));
    double *yd = (double *)malloc(sizeof(double) * (size_t)(T * H));
    for (int64_t i = 0; i < T * H; ++i) xd[i] = (double)x[i];
    ffn_block(D, w, xd, T, yd);
    for (int64_t i = 0; i < T * H; ++i) y[i] = (float)yd[i];
    free(xd); free(yd);
}

/* ---- decoder layer, prefill phase (Section 2.1) -------------------------- */
/* x, y: [B, S, H] fp32.  lens[b] in [1, S]: tokens t >= lens[b] are right padding; their
 * output rows are written as 0 and are not part of the result.  Query t of sequence b sees
 * keys j <= t (causal), all of which are < lens[b] for a valid t.
 * k_cache/v_cache (optional, [B, n_kv, cap, d] fp32): receive the rotated keys and the
 * values of positions 0..lens[b]-1, which is what a later decode step reads. */
static int layer_prefill(const orc_layer_desc *D, const orc_layer_weights *w, const float *x,
                         const int32_t *lens, int B, int S, float *y, float *k_cache,
                         float *v_cache, int cap, int parts)
{
    int H = D->hidden, d = D->head_dim, nq = D->n_q_heads, nkv = D->n_kv_heads;
    if (nkv <= 0 || nq % nkv || (d & 1)) return -1;
    int QD = nq * d, KD = nkv * d, grp = nq / nkv;
    for (int b = 0; b < B; ++b) {
        int len = lens[b];
        if (len < 1 || len > S || (k_cache && len > cap)) return -1;
        const float *xb = x + (int64_t)b * S * H;
        float *yb = y + (int64_t)b * S * H;
        memset(yb, 0, sizeof(float) * (size_t)S * H);
        double *xd = (double *)malloc(sizeof(double) * (size_t)len * H);
        double *h = (double *)malloc(sizeof(double) * (size_t)len * H);
        double *q = (double *)malloc(sizeof(double) * (size_t)len * QD);
        double *k = (double *)malloc(sizeof(double) * (size_t)len * KD);
        double *v = (double *)malloc(sizeof(double) * (size_t)len * KD);
        double *a = (double *)malloc(sizeof(double) * (size_t)len * QD);
        double *yd = (double *)malloc(sizeof(double) * (size_t)len * H);
        for (int64_t i = 0; i < (int64_t)len * H; ++i) xd[i] = (double)xb[i];
        orc_rmsnorm_f64(xd, w->g1, D->rms_eps, len, H, h);
        orc_linear_f64(h, w->wq, len, H, QD, q);
        orc_linear_f64(h, w->wk, len, H, KD, k);
        orc_linear_f64(h, w->wv, len, H, KD, v);
        for (int t = 0; t < len; ++t) {
            for (int hh = 0; hh < nq; ++hh) orc_rope_f64(q + (int64_t)t * QD + hh * d, d, t, D->rope_base);
            for (int hh = 0; hh < nkv; ++hh) orc_rope_f64(k + (int64_t)t * KD + hh * d, d, t, D->rope_base);
        }
        if (k_cache && v_cache) {
            for (int t = 0; t < len; ++t)
                for (int hh = 0; hh < nkv; ++hh)
                    for (int c = 0; c < d; ++c) {
                        int64_t o = (((int64_t)b * nkv + hh) * cap + t) * d + c;
                        k_cache[o] = (float)k[(int64_t)t * KD + hh * d + c];
                        v_cache[o] = (float)v[(int64_t)t * KD + hh * d + c];
                    }
        }
#pragma omp parallel for collapse(2) schedule(dynamic, 4)
        for (int t = 0; t < len; ++t)
            for (int hh = 0; hh < nq; ++hh) {
                int kvh = hh / grp;
                attend_one(q + (int64_t)t * QD + hh * d, k + kvh * d, v + kvh * d, t + 1, d, KD,
                           a + (int64_t)t * QD + hh * d, NULL);
            }
        post_attention(D, w, xd, a, len, yd, parts);
        for (int64_t i = 0; i < (int64_t)len * H; ++i) yb[i] = (float)yd[i];
        free(xd); free(h); free(q); free(k); free(v); free(a); free(yd);
    }
    return 0;
}

int orc_decoder_layer_prefill(const orc_layer_desc *D, const orc_layer_weights *w, const float *x,
                              const int32_t *lens, int B, int S, float *y, float *k_cache,
                              float *v_cache, int cap)
{
    return layer_prefill(D, w, x, lens, B, S, y, k_cache, v_cache, cap, 3);
}

/* the attention block alone: y = x + Attention(RMSNorm(x; g1)) Wo^T */
int orc_attention_block_prefill(const orc_layer_desc *D, const orc_layer_weights *w, const float *x,
                                const int32_t *lens, int B, int S, float *y, float *k_cache,
                                float *v_cache, int cap)
{
    return layer_prefill(D, w, x, lens, B, S, y, k_cache, v_cache, cap, 1);
}

/* ---- decoder layer, decode phase (Section 2.1) --------------------------- */
/* x, y: [B, H] fp32, one new token per sequence.  lens[b] = L_b entries already cached
 * (post-rotation keys).  The new token sits at position L_b: its rotated key and its value
 * are stored at cache slot L_b and the query attends over slots 0..L_b (L_b + 1 keys).
 * Caches [B, n_kv, cap, d] fp32 are updated in place; cap >= L_b + 1. */
static int layer_decode(const orc_layer_desc *D, const orc_layer_weights *w, const float *x,
                        const int32_t *lens, int B, float *k_cache, float *v_cache, int cap,
                        float *y, int parts)
{
    int H = D->hidden, d = D->head_dim, nq = D->n_q_heads, nkv = D->n_kv_heads;
    if (nkv <= 0 || nq % nkv || (d & 1)) return -1;
    for (int b = 0; b < B; ++b)
        if (lens[b] < 0 || lens[b] + 1 > cap) return -1;
    int QD = nq * d, KD = nkv * d, grp = nq / nkv;
    double *xd = (double *)malloc(sizeof(double) * (size_t)B * H);
    double *h = (double *)malloc(sizeof(double) * (size_t)B * H);
    double *q = (double *)malloc(sizeof(double) * (size_t)B * QD);
    double *k = (double *)malloc(sizeof(double) * (size_t)B * KD);
    double *v = (double *)malloc(sizeof(double) * (size_t)B * KD);
    double *a = (double *)malloc(sizeof(double) * (size_t)B * QD);
    double *yd = (double *)malloc(sizeof(double) * (size_t)B * H);
    for (int64_t i = 0; i < (int64_t)B * H; ++i) xd[i] = (double)x[i];
    orc_rmsnorm_f64(xd, w->g1, D->rms_eps, B, H, h);
    orc_linear_f64(h, w->wq, B, H, QD, q);
    orc_linear_f64(h, w->wk, B, H, KD, k);
    orc_linear_f64(h, w->wv, B, H, KD, v);
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b)
        for (int kvh = 0; kvh < nkv; ++kvh) {
            int L = lens[b];
            orc_rope_f64(k + (int64_t)b * KD + kvh * d, d, L, D->rope_base);
            /* visible keys/values of this (sequence, kv head): cached slots then the new one */
            double *kk = (double *)malloc(sizeof(double) * (size_t)(L + 1) * d);
            double *vv = (double *)malloc(sizeof(double) * (size_t)(L + 1) * d);
            float *kc = k_cache + ((int64_t)b * nkv + kvh) * cap * d;
            float *vc = v_cache + ((int64_t)b * nkv + kvh) * cap * d;
            for (int64_t i = 0; i < (int64_t)L * d; ++i) { kk[i] = (double)kc[i]; vv[i] = (double)vc[i]; }
            for (int c = 0; c < d; ++c) {
                kk[(int64_t)L * d + c] = k[(int64_t)b * KD + kvh * d + c];
                vv[(int64_t)L * d + c] = v[(int64_t)b * KD + kvh * d + c];
                kc[(int64_t)L * d + c] = (float)kk[(int64_t)L * d + c];
                vc[(int64_t)L * d + c] = (float)vv[(int64_t)L * d + c];
            }
            for (int g = 0; g < grp; ++g) {
                int hh = kvh * grp + g;
                double *qh = q + (int64_t)b * QD + hh * d;
                orc_rope_f64(qh, d, L, D->rope_base);
                attend_one(qh, kk, vv, L + 1, d, d, a + (int64_t)b * QD + hh * d, NULL);
            }
            free(kk); free(vv);
        }
    post_attention(D, w, xd, a, B, yd, parts);
    for (int64_t i = 0; i < (int64_t)B * H; ++i) y[i] = (float)yd[i];
    free(xd); free(h); free(q); free(k); free(v); free(a); free(yd);
    return 0;
}

int orc_decoder_layer_decode(const orc_layer_desc *D, const orc_layer_weights *w, const float *x,
                             const int32_t *lens, int B, float *k_cache, float *v_cache, int cap,
                             float *y)
{
    return layer_decode(D, w, x, lens, B, k_cache, v_cache, cap, y, 3);
}

int orc_attention_block_decode(const orc_layer_desc *D, const orc_layer_weights *w, const float *x,
                               const int32_t *lens, int B, float *k_cache, float *v_cache, int cap,
                               float *y)
{
    return layer_decode(D, w, x, lens, B, k_cache, v_cache, cap, y, 1);
}

/* ---- single projection module: y = x W^T (Section 3.1 "Migration": projections are
 * modules of their own) ---------------------------------------------------- */
void orc_linear_module(const float *x, const float *W, int64_t T, int K, int N, float *y)
{
    double *xd = (double *)malloc(sizeof(double) * (size_t)(T * K));
    double *yd = (double *)malloc(sizeof(double) * (size_t)(T * N));
    for (int64_t i = 0; i < T * K; ++i) xd[i] = (double)x[i];
    orc_linear_f64(xd, W, T, K, N, yd);
    for (int64_t i = 0; i < T * N; ++i) y[i] = (float)yd[i];
    free(xd); free(yd);
}

/* ---- fp32-array conveniences for the piece-wise tests -------------------- */
void orc_rmsnorm(const float *x, const float *g, double eps, int64_t T, int H, float *out)
{
    double *xd = (double *)malloc(sizeof(double) * (size_t)(T * H));
    double *od = (double *)malloc(sizeof(double) * (size_t)(T * H));
    for (int64_t i = 0; i < T * H; ++i) xd[i] = (double)x[i];
    orc_rmsnorm_f64(xd, g, eps, T, H, od);
    for (int64_t i = 0; i < T * H; ++i) out[i] = (float)od[i];
    free(xd); free(od);
}

/* number of OpenMP threads the loops above will use */
int orc_omp_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
