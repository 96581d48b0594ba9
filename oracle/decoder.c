/*
 * CPU oracle of the LLM forward that ANPD verifies drafts with.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call this file;
 * it exists so that tests, the smoke check and the benchmark's cpu_baseline
 * leg have a slow, plain statement of what the verification forward computes.
 * It shares no code with the HIP library.
 *
 * What is computed (paper, Section 3.1, "Parallel Decoding", step 2): one
 * forward of a decoder-only LLM over the window x_{i+1..i+K} against the cached
 * (k,v)_1..(k,v)_i, giving one next-token prediction per window row.  The
 * paper wraps a LLaMA model without describing its layer; the layer below is
 * the public LLaMA architecture: RMSNorm, rotary position embedding in the
 * half-split pairing (i, i + head_dim/2), causal softmax attention with scale
 * 1/sqrt(head_dim), SwiGLU feed-forward, no biases, untied LM head.  Keys and
 * values may be shared by groups of query heads (grouped-query attention, the
 * arrangement of the ChatGLM model the paper also evaluates): with n_kv_heads
 * key/value heads, query head h reads key/value head h / (n_heads / n_kv_heads).
 *
 * Arithmetic is IEEE double throughout.  Storage formats are part of the
 * problem and are modelled: weights arrive either as float32 or as bfloat16
 * bit patterns and are widened exactly; when kv_bf16 is set, K (after the
 * rotation) and V are rounded to float32 and then to bfloat16, round to
 * nearest even, at the moment they enter the cache.
 *
 * There is no blocking or reordering: every sum runs over its index in
 * increasing order.  OpenMP, when enabled, only distributes independent
 * output elements over threads.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORC_F32 = 0, ORC_BF16 = 1 };

typedef struct {
    int32_t n_layers, d_model, n_heads, head_dim, d_ffn, vocab;
    double rms_eps, rope_base;
    int32_t w_dtype; /* ORC_F32 or ORC_BF16: element type behind every weight pointer */
    int32_t kv_bf16; /* round cached K and V to bfloat16 */
    int32_t n_kv_heads; /* key/value heads; 0 means n_heads (one per query head) */
} orc_cfg;

typedef struct {
    const void *embed, *final_norm, *lm_head;
    const void *const *attn_norm, *const *wq, *const *wk, *const *wv, *const *wo;
    const void *const *ffn_norm, *const *w_gate, *const *w_up, *const *w_down;
} orc_weights;

typedef struct {
    orc_cfg cfg;
    orc_weights w;
} orc_model;

typedef struct {
    int32_t max_tokens, len;
    int32_t n_layers, d_model; /* d_model here: width of a cached row = n_kv_heads * head_dim */
    double *k, *v; /* [layer][max_tokens][n_kv_heads * head_dim] */
} orc_kv;

/* ---- storage formats ---------------------------------------------------- */

static double widen(const void *p, int dt, size_t i)
{
    if (dt == ORC_BF16) {
        uint32_t bits = (uint32_t)((const uint16_t *)p)[i] << 16;
        float f;
        memcpy(&f, &bits, 4);
        return (double)f;
    }
    return (double)((const float *)p)[i];
}

/* double -> float32 -> bfloat16 (round to nearest, ties to even) -> double */
double orc_round_bf16(double x)
{
    float f = (float)x;
    uint32_t bits;
    memcpy(&bits, &f, 4);
    if ((bits & 0x7fffffffu) > 0x7f800000u) return (double)f; /* NaN stays NaN */
    uint32_t lsb = (bits >> 16) & 1u;
    bits += 0x7fffu + lsb;
    bits &= 0xffff0000u;
    memcpy(&f, &bits, 4);
    return (double)f;
}

/* ---- the pieces of one layer -------------------------------------------- */

/* rmsnorm(x, g)_i = x_i * g_i / sqrt(mean_j x_j^2 + eps) */
void orc_rmsnorm(const double *x, const void *g, int g_dtype, int d, double eps, double *out)
{
    double ss = 0.0;
    for (int j = 0; j < d; ++j) ss += x[j] * x[j];
    double r = 1.0 / sqrt(ss / (double)d + eps);
    for (int i = 0; i < d; ++i) out[i] = x[i] * widen(g, g_dtype, (size_t)i) * r;
}

/* Y[m][n] = sum_k X[m][k] * W[n][k];  W is [N][K] row-major (out, in). */
void orc_linear(const double *X, int M, int K, const void *W, int w_dtype, int N, double *Y)
{
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int m = 0; m < M; ++m) {
            double acc = 0.0;
            const double *x = X + (size_t)m * K;
            for (int k = 0; k < K; ++k) acc += x[k] * widen(W, w_dtype, (size_t)n * K + k);
            Y[(size_t)m * N + n] = acc;
        }
    }
}

/* Rotary embedding of one token's H heads at absolute position pos.
 * Pair (i, i + dh/2) of each head is rotated by the angle pos * base^(-2i/dh). */
void orc_rope(double *v, int H, int dh, int pos, double base)
{
    int half = dh / 2;
    for (int h = 0; h < H; ++h) {
        double *p = v + (size_t)h * dh;
        for (int i = 0; i < half; ++i) {
            double ang = (double)pos * pow(base, -2.0 * (double)i / (double)dh);
            double c = cos(ang), s = sin(ang);
            double a = p[i], b = p[i + half];
            p[i] = a * c - b * s;
            p[i + half] = b * c + a * s;
        }
    }
}

/* One query token (H heads) against cached positions 0..n_keys-1, the keys and values held as Hkv
 * heads (H a multiple of Hkv): query head h reads key/value head h / (H / Hkv).
 * Kc, Vc: [n_keys][Hkv*dh].  out: [H*dh]. */
void orc_attention_grouped(const double *q, const double *Kc, const double *Vc, int n_keys, int H, int Hkv, int dh,
                           double *out)
{
    int d = Hkv * dh, group = H / Hkv;
    double scale = 1.0 / sqrt((double)dh);
    double *s = (double *)malloc(sizeof(double) * (size_t)n_keys);
    for (int h = 0; h < H; ++h) {
        const double *qh = q + (size_t)h * dh;
        const int hk = h / group;
        double mx = -INFINITY;
        for (int j = 0; j < n_keys; ++j) {
            const double *kj = Kc + (size_t)j * d + (size_t)hk * dh;
            double acc = 0.0;
            for (int i = 0; i < dh; ++i) acc += qh[i] * kj[i];
            s[j] = acc * scale;
            if (s[j] > mx) mx = s[j];
        }
        double denom = 0.0;
        for (int j = 0; j < n_keys; ++j) {
            s[j] = exp(s[j] - mx);
            denom += s[j];
        }
        for (int i = 0; i < dh; ++i) {
            double acc = 0.0;
            for (int j = 0; j < n_keys; ++j) acc += s[j] * Vc[(size_t)j * d + (size_t)hk * dh + i];
            out[(size_t)h * dh + i] = acc / denom;
        }
    }
    free(s);
}

/* The same with one key/value head per query head. */
void orc_attention(const double *q, const double *Kc, const double *Vc, int n_keys, int H, int dh,
                   double *out)
{
    orc_attention_grouped(q, Kc, Vc, n_keys, H, H, dh, out);
}

/* SwiGLU: out_i = silu(gate_i) * up_i, silu(z) = z / (1 + exp(-z)) */
void orc_swiglu(const double *gate, const double *up, int n, double *out)
{
    for (int i = 0; i < n; ++i) out[i] = gate[i] / (1.0 + exp(-gate[i])) * up[i];
}

/* Greedy choice: index of the largest logit after rounding to float32 (the
 * precision the device decides in); the lowest index wins ties. */
int32_t orc_argmax(const double *logits, int n)
{
    int32_t best = 0;
    float bv = (float)logits[0];
    for (int i = 1; i < n; ++i) {
        float v = (float)logits[i];
        if (v > bv) { bv = v; best = i; }
    }
    return best;
}

/* ---- model / cache objects ---------------------------------------------- */

orc_model *orc_model_create(const orc_cfg *cfg, const orc_weights *w)
{
    orc_model *m = (orc_model *)calloc(1, sizeof(orc_model));
    m->cfg = *cfg;
    m->w = *w;
    return m;
}

void orc_model_destroy(orc_model *m) { free(m); }

orc_kv *orc_kv_create(const orc_model *m, int32_t max_tokens)
{
    orc_kv *kv = (orc_kv *)calloc(1, sizeof(orc_kv));
    kv->max_tokens = max_tokens;
    kv->n_layers = m->cfg.n_layers;
    kv->d_model = (m->cfg.n_kv_heads > 0 ? m->cfg.n_kv_heads : m->cfg.n_heads) * m->cfg.head_dim;
    size_t n = (size_t)kv->n_layers * (size_t)max_tokens * (size_t)kv->d_model;
    kv->k = (double *)calloc(n, sizeof(double));
    kv->v = (double *)calloc(n, sizeof(double));
    if (!kv->k || !kv->v) { free(kv->k); free(kv->v); free(kv); return NULL; }
    return kv;
}

void orc_kv_destroy(orc_kv *kv)
{
    if (!kv) return;
    free(kv->k);
    free(kv->v);
    free(kv);
}

int32_t orc_kv_len(const orc_kv *kv) { return kv->len; }

/* Commit or roll back: positions >= new_len are dead. */
int32_t orc_kv_set_len(orc_kv *kv, int32_t new_len)
{
    if (new_len < 0 || new_len > kv->max_tokens) return -1;
    kv->len = new_len;
    return 0;
}

/* Overwrite cached entries of one layer at positions pos0..pos0+n-1 with the
 * given values (float32, [n][d_model]); used to seed a cache with synthetic
 * contents.  Does not change the length. */
int32_t orc_kv_load(orc_kv *kv, int32_t layer, int32_t pos0, int32_t n, const float *kdata,
                    const float *vdata)
{
    if (layer < 0 || layer >= kv->n_layers || pos0 < 0 || pos0 + n > kv->max_tokens) return -1;
    size_t base = ((size_t)layer * kv->max_tokens + pos0) * kv->d_model;
    for (size_t i = 0; i < (size_t)n * kv->d_model; ++i) {
        kv->k[base + i] = (double)kdata[i];
        kv->v[base + i] = (double)vdata[i];
    }
    return 0;
}

/* Read back cached entries (for rollback tests). */
int32_t orc_kv_read(const orc_kv *kv, int32_t layer, int32_t pos0, int32_t n, double *kout,
                    double *vout)
{
    if (layer < 0 || layer >= kv->n_layers || pos0 < 0 || pos0 + n > kv->max_tokens) return -1;
    size_t base = ((size_t)layer * kv->max_tokens + pos0) * kv->d_model;
    memcpy(kout, kv->k + base, sizeof(double) * (size_t)n * kv->d_model);
    memcpy(vout, kv->v + base, sizeof(double) * (size_t)n * kv->d_model);
    return 0;
}

/*
 * Forward over a window of n tokens placed at positions len..len+n-1.
 * Writes their K and V into the cache (the length is NOT advanced: the caller
 * commits with orc_kv_set_len once it knows how many rows it keeps) and
 * returns logits[n][vocab].  Row r attends to positions 0..len+r, which makes
 * the window causal within itself.
 * Returns 0, or -1 on a bad token id / capacity overflow.
 */
int32_t orc_forward(const orc_model *mdl, orc_kv *kv, const int32_t *tokens, int32_t n,
                    double *logits)
{
    const orc_cfg *c = &mdl->cfg;
    const orc_weights *w = &mdl->w;
    const int d = c->d_model, H = c->n_heads, dh = c->head_dim, F = c->d_ffn, V = c->vocab;
    const int L = kv->len, wd = c->w_dtype;
    const int Hkv = c->n_kv_heads > 0 ? c->n_kv_heads : H, dkv = Hkv * dh;
    if (n < 1 || L + n > kv->max_tokens || H * dh != d || H % Hkv != 0 || kv->d_model != dkv) return -1;
    for (int r = 0; r < n; ++r)
        if (tokens[r] < 0 || tokens[r] >= V) return -1;

    double *x = (double *)malloc(sizeof(double) * (size_t)n * d);
    double *h = (double *)malloc(sizeof(double) * (size_t)n * d);
    double *q = (double *)malloc(sizeof(double) * (size_t)n * d);
    double *kk = (double *)malloc(sizeof(double) * (size_t)n * dkv);
    double *vv = (double *)malloc(sizeof(double) * (size_t)n * dkv);
    double *att = (double *)malloc(sizeof(double) * (size_t)n * d);
    double *y = (double *)malloc(sizeof(double) * (size_t)n * d);
    double *g = (double *)malloc(sizeof(double) * (size_t)n * F);
    double *u = (double *)malloc(sizeof(double) * (size_t)n * F);
    double *a = (double *)malloc(sizeof(double) * (size_t)n * F);

    for (int r = 0; r < n; ++r)
        for (int i = 0; i < d; ++i) x[(size_t)r * d + i] = widen(w->embed, wd, (size_t)tokens[r] * d + i);

    for (int l = 0; l < c->n_layers; ++l) {
        double *Kc = kv->k + (size_t)l * kv->max_tokens * dkv;
        double *Vc = kv->v + (size_t)l * kv->max_tokens * dkv;
        for (int r = 0; r < n; ++r)
            orc_rmsnorm(x + (size_t)r * d, w->attn_norm[l], wd, d, c->rms_eps, h + (size_t)r * d);
        orc_linear(h, n, d, w->wq[l], wd, d, q);
        orc_linear(h, n, d, w->wk[l], wd, dkv, kk);
        orc_linear(h, n, d, w->wv[l], wd, dkv, vv);
        for (int r = 0; r < n; ++r) {
            int pos = L + r;
            orc_rope(q + (size_t)r * d, H, dh, pos, c->rope_base);
            orc_rope(kk + (size_t)r * dkv, Hkv, dh, pos, c->rope_base);
            for (int i = 0; i < dkv; ++i) {
                double kval = kk[(size_t)r * dkv + i], vval = vv[(size_t)r * dkv + i];
                if (c->kv_bf16) { kval = orc_round_bf16(kval); vval = orc_round_bf16(vval); }
                Kc[(size_t)pos * dkv + i] = kval;
                Vc[(size_t)pos * dkv + i] = vval;
            }
        }
#pragma omp parallel for schedule(static)
        for (int r = 0; r < n; ++r)
            orc_attention_grouped(q + (size_t)r * d, Kc, Vc, L + r + 1, H, Hkv, dh, att + (size_t)r * d);
        orc_linear(att, n, d, w->wo[l], wd, d, y);
        for (size_t i = 0; i < (size_t)n * d; ++i) x[i] += y[i];
        for (int r = 0; r < n; ++r)
            orc_rmsnorm(x + (size_t)r * d, w->ffn_norm[l], wd, d, c->rms_eps, h + (size_t)r * d);
        orc_linear(h, n, d, w->w_gate[l], wd, F, g);
        orc_linear(h, n, d, w->w_up[l], wd, F, u);
        orc_swiglu(g, u, n * F, a);
        orc_linear(a, n, F, w->w_down[l], wd, d, y);
        for (size_t i = 0; i < (size_t)n * d; ++i) x[i] += y[i];
    }
    for (int r = 0; r < n; ++r)
        orc_rmsnorm(x + (size_t)r * d, w->final_norm, wd, d, c->rms_eps, h + (size_t)r * d);
    orc_linear(h, n, d, w->lm_head, wd, V, logits);

    free(x); free(h); free(q); free(kk); free(vv); free(att); free(y); free(g); free(u); free(a);
    return 0;
}

int32_t orc_num_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
