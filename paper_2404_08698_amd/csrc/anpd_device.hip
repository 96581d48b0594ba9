// Device half of the C ABI: model / cache objects and the verification step.
//
// One step (paper, Section 3.1 "Parallel Decoding" step 2; Algorithm 1) is a
// fixed sequence of kernel launches on the caller's stream.  Everything that
// varies from step to step (cache length, page table, window tokens) is read
// from device memory, and the only host <-> device traffic of a step is the
// window upload and the (accepted, next, predictions) read-back.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <new>
#include <vector>

#include "anpd_common.h"
#include "anpd_kernels.h"

using namespace anpd;

#define HIP_TRY(expr)                                                                             \
    do {                                                                                          \
        hipError_t e_ = (expr);                                                                   \
        if (e_ != hipSuccess) return fail(ANPD_E_HIP, "%s: %s", #expr, hipGetErrorString(e_));    \
    } while (0)

namespace {

size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

struct Layout {  // byte offsets into the model workspace
    size_t rope_tab, tok, result, counter, x, h, y, qkv, att, gu, a, logits, hs, atts, as, part, total;
    int max_splits;
};

bool cfg_ok(const anpd_model_cfg *c, const char **why)
{
#define REQ(cond, msg) if (!(cond)) { *why = msg; return false; }
    REQ(c, "cfg is NULL");
    REQ(c->n_layers >= 1 && c->d_model >= 8 && c->n_heads >= 1 && c->d_ffn >= 8 && c->vocab >= 1, "non-positive dimension");
    REQ(c->n_heads * c->head_dim == c->d_model, "d_model must equal n_heads * head_dim");
    REQ(c->head_dim == 64 || c->head_dim == 128, "head_dim must be 64 or 128");
    REQ(c->d_model % 16 == 0 && c->d_ffn % 16 == 0 && c->vocab % 16 == 0, "d_model, d_ffn and vocab must be multiples of 16");
    REQ(c->dtype == ANPD_F32 || c->dtype == ANPD_BF16, "dtype must be ANPD_F32 or ANPD_BF16");
    REQ(c->page_tokens >= 8 && c->page_tokens <= 256 && (c->page_tokens & (c->page_tokens - 1)) == 0, "page_tokens must be a power of two in 8..256");
    REQ(c->max_window >= 1 && c->max_window <= ANPD_MAX_WINDOW, "max_window must be in 1..ANPD_MAX_WINDOW");
    REQ(c->max_positions >= 1 && c->max_positions <= (1 << 20), "max_positions must be in 1..2^20");
    REQ(c->gemm_path >= ANPD_GEMM_AUTO && c->gemm_path <= ANPD_GEMM_MFMA, "unknown gemm_path");
    REQ(!(c->gemm_path == ANPD_GEMM_MFMA && c->dtype != ANPD_BF16), "the MFMA path needs bf16 weights");
    REQ(c->rms_eps > 0.f && c->rope_base > 1.f, "rms_eps / rope_base out of range");
#undef REQ
    return true;
}

Layout make_layout(const anpd_model_cfg *c)
{
    Layout L;
    const size_t MW = (size_t)c->max_window, d = (size_t)c->d_model, F = (size_t)c->d_ffn, V = (size_t)c->vocab;
    const size_t tiles = 64;  // split operand: up to 4 tiles of 16 rows
    L.max_splits = (c->max_positions + kAttnSplit - 1) / kAttnSplit + 1;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes); return at; };
    L.rope_tab = take((size_t)c->max_positions * (c->head_dim / 2) * sizeof(float2));
    L.tok = take(ANPD_MAX_WINDOW * sizeof(int32_t));
    L.result = take((2 + ANPD_MAX_WINDOW) * sizeof(int32_t));
    L.counter = take(sizeof(uint32_t));
    L.x = take(MW * d * 4);
    L.h = take(MW * d * 4);
    L.y = take(MW * d * 4);
    L.qkv = take(MW * 3 * d * 4);
    L.att = take(MW * d * 4);
    L.gu = take(MW * 2 * F * 4);
    L.a = take(MW * F * 4);
    L.logits = take(MW * V * 4);
    L.hs = take(tiles * d * 2);
    L.atts = take(tiles * d * 2);
    L.as = take(tiles * F * 2);
    L.part = take((size_t)c->n_heads * L.max_splits * MW * (c->head_dim + 2) * 4);
    L.total = o;
    return L;
}

}  // namespace

struct anpd_model {
    anpd_model_cfg cfg;
    Layout lay;
    char *ws;
    bool mfma;
    const void *embed, *final_norm, *lm_head;
    std::vector<const void *> attn_norm, wq, wk, wv, wo, ffn_norm, w_gate, w_up, w_down;
    int32_t *pin;  // pinned host staging: [0..32) window, [32..66) result
};

struct anpd_kv {
    const anpd_model *m;
    char *pool;
    int32_t n_pages, max_tokens, len;
    size_t page_bytes;
    std::vector<int32_t> table;      // logical -> physical, -1 = none
    std::vector<int32_t> dev_table;  // what the device copy currently holds
    std::vector<int32_t> free_list;  // physical pages, handed out from the back
    int32_t *d_table, *d_len;
    int32_t *pin;                    // pinned staging: [0] length, [1..] table
    bool table_dirty;
};

namespace {

size_t page_bytes_of(const anpd_model_cfg &c)
{
    return (size_t)c.n_layers * 2 * c.d_model * c.page_tokens * (c.dtype == ANPD_BF16 ? 2 : 4);
}

// ---- GEMM dispatch -----------------------------------------------------------

int32_t launch_gemm_dot(const float *X, int M, int K, const void *W0, const void *W1, const void *W2, int nseg,
                        int n_seg, float *Y, int ldy, int dtype, hipStream_t st)
{
    constexpr int R = 4;
    int n_total = nseg * n_seg;
    dim3 grid((unsigned)((n_total + 4 * R - 1) / (4 * R)));
    if (dtype == ANPD_BF16)
        hipLaunchKernelGGL((gemm_dot_kernel<bf16_t, R>), grid, dim3(256), 0, st, X, M, K, (const bf16_t *)W0,
                           (const bf16_t *)W1, (const bf16_t *)W2, n_seg, n_total, Y, ldy);
    else
        hipLaunchKernelGGL((gemm_dot_kernel<float, R>), grid, dim3(256), 0, st, X, M, K, (const float *)W0,
                           (const float *)W1, (const float *)W2, n_seg, n_total, Y, ldy);
    HIP_TRY(hipGetLastError());
    return ANPD_OK;
}

int32_t launch_gemm_mfma(const bf16_t *Xs, int M, int K, const void *W0, const void *W1, const void *W2, int nseg,
                         int n_seg, float *Y, int ldy, hipStream_t st)
{
    const int cls = window_class(M);
    const int tiles = nseg * n_seg / 16;
    // More waves per block when there are few blocks, so every SIMD still has loads in flight.
    // The wave count fixes the summation order, so it may depend on the matrix shape only,
    // never on the window size.
    int nw = tiles >= 1024 ? 4 : (tiles >= 512 ? 8 : 16);
    const int nks = (K + 31) / 32;
    while (nw > 1 && (nw - 1) * kMfmaU >= nks) nw >>= 1;
    dim3 grid((unsigned)tiles), block((unsigned)nw * 64);
    size_t smem = (size_t)nw * (cls / 8) * 64 * 4 * sizeof(float);
    const bf16_t *w0 = (const bf16_t *)W0, *w1 = (const bf16_t *)W1, *w2 = (const bf16_t *)W2;
    if (cls == 8)
        hipLaunchKernelGGL((gemm_mfma_kernel<8>), grid, block, smem, st, Xs, M, K, w0, w1, w2, n_seg, Y, ldy);
    else if (cls == 16)
        hipLaunchKernelGGL((gemm_mfma_kernel<16>), grid, block, smem, st, Xs, M, K, w0, w1, w2, n_seg, Y, ldy);
    else
        hipLaunchKernelGGL((gemm_mfma_kernel<32>), grid, block, smem, st, Xs, M, K, w0, w1, w2, n_seg, Y, ldy);
    HIP_TRY(hipGetLastError());
    return ANPD_OK;
}

int32_t gemm(const anpd_model *m, const float *X, const bf16_t *Xs, int M, int K, const void *W0, const void *W1,
             const void *W2, int nseg, int n_seg, float *Y, int ldy, hipStream_t st)
{
    if (m->mfma) return launch_gemm_mfma(Xs, M, K, W0, W1, W2, nseg, n_seg, Y, ldy, st);
    return launch_gemm_dot(X, M, K, W0, W1, W2, nseg, n_seg, Y, ldy, m->cfg.dtype, st);
}

// ---- cache pages ---------------------------------------------------------------

// Make sure logical pages covering positions [0, upto) exist; refresh the device table if needed.
int32_t ensure_pages(anpd_kv *kv, int32_t upto, hipStream_t st)
{
    const int pt = kv->m->cfg.page_tokens;
    const int need = (upto + pt - 1) / pt;
    for (int lp = 0; lp < need; ++lp) {
        if (kv->table[(size_t)lp] >= 0) continue;
        if (kv->free_list.empty()) return fail(ANPD_E_CAPACITY, "KV pool has no free page");
        kv->table[(size_t)lp] = kv->free_list.back();
        kv->free_list.pop_back();
        if (kv->table[(size_t)lp] != kv->dev_table[(size_t)lp]) kv->table_dirty = true;
    }
    if (kv->table_dirty) {
        // the staging buffer is free: every call that uses it synchronises before returning
        for (size_t i = 0; i < kv->table.size(); ++i) {
            if (kv->table[i] >= 0) kv->dev_table[i] = kv->table[i];
            kv->pin[1 + i] = kv->dev_table[i] < 0 ? 0 : kv->dev_table[i];
        }
        HIP_TRY(hipMemcpyAsync(kv->d_table, kv->pin + 1, kv->table.size() * sizeof(int32_t), hipMemcpyHostToDevice, st));
        kv->table_dirty = false;
    }
    return ANPD_OK;
}

// Return pages wholly beyond `len` to the free list.
void release_pages(anpd_kv *kv, int32_t len)
{
    const int pt = kv->m->cfg.page_tokens;
    const int keep = (len + pt - 1) / pt;
    for (int lp = (int)kv->table.size() - 1; lp >= keep; --lp) {
        if (kv->table[(size_t)lp] >= 0) {
            kv->free_list.push_back(kv->table[(size_t)lp]);
            kv->table[(size_t)lp] = -1;
        }
    }
}

template <typename KT>
int32_t run_step(anpd_model *m, anpd_kv *kv, int M, int mode, hipStream_t st)
{
    const anpd_model_cfg &c = m->cfg;
    const Layout &L = m->lay;
    char *ws = m->ws;
    const int d = c.d_model, F = c.d_ffn, V = c.vocab, H = c.n_heads, dh = c.head_dim;
    const int cls = window_class(M);
    float *x = (float *)(ws + L.x), *h = (float *)(ws + L.h), *y = (float *)(ws + L.y);
    float *qkv = (float *)(ws + L.qkv), *att = (float *)(ws + L.att), *gu = (float *)(ws + L.gu);
    float *a = (float *)(ws + L.a), *logits = (float *)(ws + L.logits), *part = (float *)(ws + L.part);
    bf16_t *hs = m->mfma ? (bf16_t *)(ws + L.hs) : nullptr;
    bf16_t *atts = m->mfma ? (bf16_t *)(ws + L.atts) : nullptr;
    bf16_t *as = m->mfma ? (bf16_t *)(ws + L.as) : nullptr;
    const float2 *rope = (const float2 *)(ws + L.rope_tab);
    const int32_t *tok = (const int32_t *)(ws + L.tok);
    int32_t *result = (int32_t *)(ws + L.result);
    uint32_t *counter = (uint32_t *)(ws + L.counter);
    KT *pool = (KT *)kv->pool;
    const float scale = 1.0f / sqrtf((float)dh);
    const int n_splits = (kv->len + M + kAttnSplit - 1) / kAttnSplit;
    int32_t rc;

    hipLaunchKernelGGL((embed_kernel<KT>), dim3(M), dim3(256), 0, st, (const KT *)m->embed, tok, x, d);
    for (int l = 0; l < c.n_layers; ++l) {
        hipLaunchKernelGGL((addnorm_kernel<KT>), dim3(M), dim3(256), 0, st, x, l == 0 ? (const float *)nullptr : y,
                           (const KT *)m->attn_norm[l], h, hs, d, c.rms_eps, cls);
        if ((rc = gemm(m, h, hs, M, d, m->wq[l], m->wk[l], m->wv[l], 3, d, qkv, 3 * d, st)) != ANPD_OK) return rc;
        hipLaunchKernelGGL((rope_kv_kernel<KT>), dim3(M), dim3(256), 0, st, qkv, rope, pool, kv->d_table, kv->d_len, l,
                           c.n_layers, H, dh, c.page_tokens);
        if (dh == 128) {
            hipLaunchKernelGGL((attn_kernel<KT, 128>), dim3(H, n_splits), dim3(256), 0, st, qkv, pool, kv->d_table,
                               kv->d_len, M, l, c.n_layers, H, c.page_tokens, c.max_window, L.max_splits, scale, part);
            hipLaunchKernelGGL((attn_combine_kernel<128>), dim3(M, H), dim3(128), 0, st, part, kv->d_len, H,
                               c.max_window, L.max_splits, att, atts, cls);
        } else {
            hipLaunchKernelGGL((attn_kernel<KT, 64>), dim3(H, n_splits), dim3(256), 0, st, qkv, pool, kv->d_table,
                               kv->d_len, M, l, c.n_layers, H, c.page_tokens, c.max_window, L.max_splits, scale, part);
            hipLaunchKernelGGL((attn_combine_kernel<64>), dim3(M, H), dim3(64), 0, st, part, kv->d_len, H, c.max_window,
                               L.max_splits, att, atts, cls);
        }
        if ((rc = gemm(m, att, atts, M, d, m->wo[l], nullptr, nullptr, 1, d, y, d, st)) != ANPD_OK) return rc;
        hipLaunchKernelGGL((addnorm_kernel<KT>), dim3(M), dim3(256), 0, st, x, y, (const KT *)m->ffn_norm[l], h, hs, d,
                           c.rms_eps, cls);
        if ((rc = gemm(m, h, hs, M, d, m->w_gate[l], m->w_up[l], nullptr, 2, F, gu, 2 * F, st)) != ANPD_OK) return rc;
        hipLaunchKernelGGL(swiglu_kernel, dim3((F + 255) / 256, M), dim3(256), 0, st, gu, a, as, F, cls);
        if ((rc = gemm(m, a, as, M, F, m->w_down[l], nullptr, nullptr, 1, d, y, d, st)) != ANPD_OK) return rc;
    }
    hipLaunchKernelGGL((addnorm_kernel<KT>), dim3(M), dim3(256), 0, st, x, y, (const KT *)m->final_norm, h, hs, d,
                       c.rms_eps, cls);
    if ((rc = gemm(m, h, hs, M, d, m->lm_head, nullptr, nullptr, 1, V, logits, V, st)) != ANPD_OK) return rc;
    hipLaunchKernelGGL(argmax_accept_kernel, dim3(M), dim3(1024), 0, st, logits, V, M, tok, mode, result, kv->d_len,
                       counter);
    HIP_TRY(hipGetLastError());
    return ANPD_OK;
}

}  // namespace

extern "C" {

size_t anpd_model_workspace_bytes(const anpd_model_cfg *cfg)
{
    const char *why;
    if (!cfg_ok(cfg, &why)) { fail(ANPD_E_INVAL, "anpd_model_workspace_bytes: %s", why); return 0; }
    return make_layout(cfg).total;
}

int32_t anpd_model_create(const anpd_model_cfg *cfg, const anpd_weights *w, void *workspace, size_t workspace_bytes,
                          void *stream, anpd_model_t **out)
{
    if (!out) return fail(ANPD_E_INVAL, "anpd_model_create: out is NULL");
    *out = nullptr;
    const char *why;
    if (!cfg_ok(cfg, &why)) return fail(ANPD_E_INVAL, "anpd_model_create: %s", why);
    if (!w || !workspace) return fail(ANPD_E_INVAL, "anpd_model_create: NULL weights or workspace");
    if (((uintptr_t)workspace & 255) != 0) return fail(ANPD_E_INVAL, "anpd_model_create: workspace must be 256-byte aligned");
    Layout lay = make_layout(cfg);
    if (workspace_bytes < lay.total)
        return fail(ANPD_E_CAPACITY, "anpd_model_create: workspace has %zu bytes, %zu needed", workspace_bytes, lay.total);
    if (!w->embed || !w->final_norm || !w->lm_head || !w->attn_norm || !w->wq || !w->wk || !w->wv || !w->wo ||
        !w->ffn_norm || !w->w_gate || !w->w_up || !w->w_down)
        return fail(ANPD_E_INVAL, "anpd_model_create: a weight pointer is NULL");
    for (int l = 0; l < cfg->n_layers; ++l)
        if (!w->attn_norm[l] || !w->wq[l] || !w->wk[l] || !w->wv[l] || !w->wo[l] || !w->ffn_norm[l] || !w->w_gate[l] ||
            !w->w_up[l] || !w->w_down[l])
            return fail(ANPD_E_INVAL, "anpd_model_create: a weight pointer of layer %d is NULL", l);

    anpd_model *m = new (std::nothrow) anpd_model;
    if (!m) return fail(ANPD_E_NOMEM, "anpd_model_create: out of memory");
    m->cfg = *cfg;
    m->lay = lay;
    m->ws = (char *)workspace;
    m->mfma = cfg->gemm_path == ANPD_GEMM_MFMA || (cfg->gemm_path == ANPD_GEMM_AUTO && cfg->dtype == ANPD_BF16);
    m->embed = w->embed;
    m->final_norm = w->final_norm;
    m->lm_head = w->lm_head;
    const size_t nl = (size_t)cfg->n_layers;
    m->attn_norm.assign(w->attn_norm, w->attn_norm + nl);
    m->wq.assign(w->wq, w->wq + nl);
    m->wk.assign(w->wk, w->wk + nl);
    m->wv.assign(w->wv, w->wv + nl);
    m->wo.assign(w->wo, w->wo + nl);
    m->ffn_norm.assign(w->ffn_norm, w->ffn_norm + nl);
    m->w_gate.assign(w->w_gate, w->w_gate + nl);
    m->w_up.assign(w->w_up, w->w_up + nl);
    m->w_down.assign(w->w_down, w->w_down + nl);
    m->pin = nullptr;

    hipStream_t st = (hipStream_t)stream;
    // cos/sin of pos * base^(-2i/head_dim), evaluated in double, stored as float
    const int half = cfg->head_dim / 2;
    std::vector<float2> tab((size_t)cfg->max_positions * half);
    for (int i = 0; i < half; ++i) {
        double theta = std::pow((double)cfg->rope_base, -2.0 * (double)i / (double)cfg->head_dim);
        for (int p = 0; p < cfg->max_positions; ++p) {
            double ang = (double)p * theta;
            tab[(size_t)p * half + i] = make_float2((float)std::cos(ang), (float)std::sin(ang));
        }
    }
    hipError_t e = hipHostMalloc((void **)&m->pin, 128 * sizeof(int32_t), hipHostMallocDefault);
    if (e != hipSuccess) { delete m; return fail(ANPD_E_HIP, "hipHostMalloc: %s", hipGetErrorString(e)); }
    e = hipMemsetAsync(m->ws, 0, lay.total, st);
    if (e == hipSuccess) e = hipMemcpyAsync(m->ws + lay.rope_tab, tab.data(), tab.size() * sizeof(float2), hipMemcpyHostToDevice, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) {
        (void)hipHostFree(m->pin);
        delete m;
        return fail(ANPD_E_HIP, "anpd_model_create: %s", hipGetErrorString(e));
    }
    *out = m;
    return ANPD_OK;
}

void anpd_model_destroy(anpd_model_t *m)
{
    if (!m) return;
    if (m->pin) (void)hipHostFree(m->pin);
    delete m;
}

size_t anpd_kv_pool_bytes(const anpd_model_t *m, int32_t max_tokens)
{
    if (!m || max_tokens < 1 || max_tokens > m->cfg.max_positions) {
        fail(ANPD_E_INVAL, "anpd_kv_pool_bytes: bad argument");
        return 0;
    }
    const int pt = m->cfg.page_tokens;
    size_t pages = (size_t)(max_tokens + pt - 1) / pt;
    return align_up(pages * page_bytes_of(m->cfg)) + align_up((pages + 1) * sizeof(int32_t));
}

int32_t anpd_kv_create(const anpd_model_t *m, void *pool, size_t pool_bytes, int32_t max_tokens, anpd_kv_t **out)
{
    if (!out) return fail(ANPD_E_INVAL, "anpd_kv_create: out is NULL");
    *out = nullptr;
    if (!m || !pool) return fail(ANPD_E_INVAL, "anpd_kv_create: NULL model or pool");
    if (max_tokens < 1 || max_tokens > m->cfg.max_positions)
        return fail(ANPD_E_CAPACITY, "anpd_kv_create: max_tokens %d outside 1..max_positions (%d)", max_tokens, m->cfg.max_positions);
    if (((uintptr_t)pool & 255) != 0) return fail(ANPD_E_INVAL, "anpd_kv_create: pool must be 256-byte aligned");
    size_t need = anpd_kv_pool_bytes(m, max_tokens);
    if (pool_bytes < need) return fail(ANPD_E_CAPACITY, "anpd_kv_create: pool has %zu bytes, %zu needed", pool_bytes, need);
    anpd_kv *kv = new (std::nothrow) anpd_kv;
    if (!kv) return fail(ANPD_E_NOMEM, "anpd_kv_create: out of memory");
    const int pt = m->cfg.page_tokens;
    kv->m = m;
    kv->pool = (char *)pool;
    kv->n_pages = (max_tokens + pt - 1) / pt;
    kv->max_tokens = max_tokens;
    kv->len = 0;
    kv->page_bytes = page_bytes_of(m->cfg);
    kv->table.assign((size_t)kv->n_pages, -1);
    kv->dev_table.assign((size_t)kv->n_pages, -1);
    for (int p = kv->n_pages - 1; p >= 0; --p) kv->free_list.push_back(p);  // page 0 is handed out first
    char *tail = kv->pool + align_up((size_t)kv->n_pages * kv->page_bytes);
    kv->d_len = (int32_t *)tail;
    kv->d_table = kv->d_len + 1;
    kv->table_dirty = true;
    kv->pin = nullptr;
    hipError_t e = hipHostMalloc((void **)&kv->pin, ((size_t)kv->n_pages + 1) * sizeof(int32_t), hipHostMallocDefault);
    if (e == hipSuccess) {
        kv->pin[0] = 0;
        e = hipMemcpy(kv->d_len, kv->pin, sizeof(int32_t), hipMemcpyHostToDevice);
    }
    if (e != hipSuccess) {
        if (kv->pin) (void)hipHostFree(kv->pin);
        delete kv;
        return fail(ANPD_E_HIP, "anpd_kv_create: %s", hipGetErrorString(e));
    }
    *out = kv;
    return ANPD_OK;
}

void anpd_kv_destroy(anpd_kv_t *kv)
{
    if (!kv) return;
    if (kv->pin) (void)hipHostFree(kv->pin);
    delete kv;
}

int32_t anpd_kv_length(const anpd_kv_t *kv) { return kv ? kv->len : fail(ANPD_E_INVAL, "anpd_kv_length: NULL handle"); }

int32_t anpd_kv_num_pages(const anpd_kv_t *kv) { return kv ? kv->n_pages : fail(ANPD_E_INVAL, "anpd_kv_num_pages: NULL handle"); }

int32_t anpd_kv_set_page_order(anpd_kv_t *kv, const int32_t *perm, int32_t n_pages)
{
    if (!kv || !perm) return fail(ANPD_E_INVAL, "anpd_kv_set_page_order: NULL argument");
    if (n_pages != kv->n_pages) return fail(ANPD_E_INVAL, "anpd_kv_set_page_order: expected %d entries", kv->n_pages);
    if ((int)kv->free_list.size() != kv->n_pages) return fail(ANPD_E_INVAL, "anpd_kv_set_page_order: cache is not empty");
    std::vector<char> seen((size_t)n_pages, 0);
    for (int i = 0; i < n_pages; ++i) {
        if (perm[i] < 0 || perm[i] >= n_pages || seen[(size_t)perm[i]])
            return fail(ANPD_E_INVAL, "anpd_kv_set_page_order: not a permutation");
        seen[(size_t)perm[i]] = 1;
    }
    for (int i = 0; i < n_pages; ++i) kv->free_list[(size_t)(n_pages - 1 - i)] = perm[i];
    return ANPD_OK;
}

int32_t anpd_kv_truncate(anpd_kv_t *kv, int32_t new_len, void *stream)
{
    if (!kv) return fail(ANPD_E_INVAL, "anpd_kv_truncate: NULL handle");
    if (new_len < 0 || new_len > kv->max_tokens)
        return fail(ANPD_E_CAPACITY, "anpd_kv_truncate: length %d outside 0..%d", new_len, kv->max_tokens);
    hipStream_t st = (hipStream_t)stream;
    int32_t rc = ensure_pages(kv, new_len, st);
    if (rc != ANPD_OK) return rc;
    kv->pin[0] = new_len;
    HIP_TRY(hipMemcpyAsync(kv->d_len, kv->pin, sizeof(int32_t), hipMemcpyHostToDevice, st));
    HIP_TRY(hipStreamSynchronize(st));
    kv->len = new_len;
    release_pages(kv, new_len);
    return ANPD_OK;
}

static int32_t kv_copy(anpd_kv *kv, int32_t layer, int32_t pos0, int32_t n, float *k, float *v, bool to_cache, void *stream)
{
    if (!kv || ((!k || !v) && n != 0)) return fail(ANPD_E_INVAL, "anpd_kv_read/write: NULL argument");
    const anpd_model_cfg &c = kv->m->cfg;
    if (layer < 0 || layer >= c.n_layers || pos0 < 0 || n < 0 || pos0 + n > kv->max_tokens)
        return fail(ANPD_E_CAPACITY, "anpd_kv_read/write: layer %d, positions %d..%d out of range", layer, pos0, pos0 + n);
    if (n == 0) return ANPD_OK;
    hipStream_t st = (hipStream_t)stream;
    if (to_cache) {
        int32_t rc = ensure_pages(kv, pos0 + n, st);
        if (rc != ANPD_OK) return rc;
    } else {
        const int pt = c.page_tokens;
        for (int lp = pos0 / pt; lp <= (pos0 + n - 1) / pt; ++lp)
            if (kv->table[(size_t)lp] < 0) return fail(ANPD_E_INVAL, "anpd_kv_read: position %d has no page", lp * pt);
    }
#define KV_COPY(KT, TO)                                                                                          \
    hipLaunchKernelGGL((kv_copy_kernel<KT, TO>), dim3(n), dim3(256), 0, st, (KT *)kv->pool, kv->d_table, k, v, pos0, \
                       layer, c.n_layers, c.n_heads, c.head_dim, c.page_tokens)
    if (c.dtype == ANPD_BF16) { if (to_cache) KV_COPY(bf16_t, true); else KV_COPY(bf16_t, false); }
    else { if (to_cache) KV_COPY(float, true); else KV_COPY(float, false); }
#undef KV_COPY
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipStreamSynchronize(st));
    return ANPD_OK;
}

int32_t anpd_kv_write(anpd_kv_t *kv, int32_t layer, int32_t pos0, int32_t n, const float *k, const float *v, void *stream)
{
    return kv_copy(kv, layer, pos0, n, const_cast<float *>(k), const_cast<float *>(v), true, stream);
}

int32_t anpd_kv_read(const anpd_kv_t *kv, int32_t layer, int32_t pos0, int32_t n, float *k, float *v, void *stream)
{
    return kv_copy(const_cast<anpd_kv *>(kv), layer, pos0, n, k, v, false, stream);
}

int32_t anpd_verify(anpd_model_t *m, anpd_kv_t *kv, const int32_t *window, int32_t n_window, int32_t mode,
                    int32_t *out_accepted, int32_t *out_next, int32_t *out_predicts, float *out_logits, void *stream)
{
    if (!m || !kv || !window || !out_accepted || !out_next) return fail(ANPD_E_INVAL, "anpd_verify: NULL argument");
    if (kv->m != m) return fail(ANPD_E_INVAL, "anpd_verify: the cache belongs to another model");
    if (mode != ANPD_VERIFY && mode != ANPD_APPEND) return fail(ANPD_E_INVAL, "anpd_verify: unknown mode %d", mode);
    if (n_window < 1) return fail(ANPD_E_INVAL, "anpd_verify: n_window must be >= 1");
    if (n_window > m->cfg.max_window)
        return fail(ANPD_E_CAPACITY, "anpd_verify: n_window %d exceeds max_window %d", n_window, m->cfg.max_window);
    if (kv->len + n_window > kv->max_tokens)
        return fail(ANPD_E_CAPACITY, "anpd_verify: length %d + window %d exceeds capacity %d", kv->len, n_window, kv->max_tokens);
    for (int i = 0; i < n_window; ++i)
        if (window[i] < 0 || window[i] >= m->cfg.vocab)
            return fail(ANPD_E_RANGE, "anpd_verify: token %d at window[%d] outside [0, %d)", window[i], i, m->cfg.vocab);

    hipStream_t st = (hipStream_t)stream;
    int32_t rc = ensure_pages(kv, kv->len + n_window, st);
    if (rc != ANPD_OK) return rc;
    std::memcpy(m->pin, window, sizeof(int32_t) * (size_t)n_window);
    HIP_TRY(hipMemcpyAsync(m->ws + m->lay.tok, m->pin, sizeof(int32_t) * (size_t)n_window, hipMemcpyHostToDevice, st));
    rc = m->cfg.dtype == ANPD_BF16 ? run_step<bf16_t>(m, kv, n_window, mode, st) : run_step<float>(m, kv, n_window, mode, st);
    if (rc != ANPD_OK) return rc;
    int32_t *res = m->pin + 32;
    HIP_TRY(hipMemcpyAsync(res, m->ws + m->lay.result, sizeof(int32_t) * (size_t)(2 + n_window), hipMemcpyDeviceToHost, st));
    if (out_logits)
        HIP_TRY(hipMemcpyAsync(out_logits, m->ws + m->lay.logits, sizeof(float) * (size_t)n_window * m->cfg.vocab,
                               hipMemcpyDeviceToDevice, st));
    HIP_TRY(hipStreamSynchronize(st));
    *out_accepted = res[0];
    *out_next = res[1];
    if (out_predicts) std::memcpy(out_predicts, res + 2, sizeof(int32_t) * (size_t)n_window);
    kv->len += 1 + res[0];
    release_pages(kv, kv->len);
    return ANPD_OK;
}

size_t anpd_linear_workspace_bytes(int32_t M, int32_t K)
{
    if (M < 1 || M > ANPD_MAX_WINDOW || K < 8) return 0;
    return align_up((size_t)64 * (size_t)K * sizeof(bf16_t));
}

int32_t anpd_linear(const float *X, const void *W, float *Y, int32_t M, int32_t N, int32_t K, int32_t dtype,
                    int32_t path, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!X || !W || !Y) return fail(ANPD_E_INVAL, "anpd_linear: NULL argument");
    if (M < 1 || M > ANPD_MAX_WINDOW || K < 8 || K % 8 != 0 || N < 16 || N % 16 != 0)
        return fail(ANPD_E_INVAL, "anpd_linear: need 1 <= M <= %d, K %% 8 == 0, N %% 16 == 0", ANPD_MAX_WINDOW);
    if (dtype != ANPD_F32 && dtype != ANPD_BF16) return fail(ANPD_E_INVAL, "anpd_linear: unknown dtype");
    hipStream_t st = (hipStream_t)stream;
    if (path == ANPD_GEMM_DOT) return launch_gemm_dot(X, M, K, W, nullptr, nullptr, 1, N, Y, N, dtype, st);
    if (path != ANPD_GEMM_MFMA) return fail(ANPD_E_INVAL, "anpd_linear: path must be ANPD_GEMM_DOT or ANPD_GEMM_MFMA");
    if (dtype != ANPD_BF16) return fail(ANPD_E_INVAL, "anpd_linear: the MFMA path needs bf16 weights");
    if (!workspace || workspace_bytes < anpd_linear_workspace_bytes(M, K))
        return fail(ANPD_E_CAPACITY, "anpd_linear: workspace too small");
    const int cls = window_class(M);
    hipLaunchKernelGGL(split_kernel, dim3((K + 255) / 256, M), dim3(256), 0, st, X, (bf16_t *)workspace, M, K, cls);
    return launch_gemm_mfma((const bf16_t *)workspace, M, K, W, nullptr, nullptr, 1, N, Y, N, st);
}

}  // extern "C"
