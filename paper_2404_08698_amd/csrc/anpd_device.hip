// Device half of the C ABI: model / cache objects and the verification step.
//
// One step (paper, Section 3.1 "Parallel Decoding" step 2; Algorithm 1) is a
// fixed sequence of kernel launches on the caller's stream.  Everything that
// varies from step to step (cache length, page table, window tokens) is read
// from device memory, and the only host <-> device traffic of a step is the
// window upload and the (accepted, next, predictions) read-back.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "anpd_common.h"
#include "anpd_kernels.h"
#include "anpd_fast.h"
#include "anpd_mega.h"
#include "anpd_prefill.h"

using namespace anpd;

#define HIP_TRY(expr)                                                                             \
    do {                                                                                          \
        hipError_t e_ = (expr);                                                                   \
        if (e_ != hipSuccess) return fail(ANPD_E_HIP, "%s: %s", #expr, hipGetErrorString(e_));    \
    } while (0)

namespace {

size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

int kv_heads_of(const anpd_model_cfg &c) { return c.n_kv_heads > 0 ? c.n_kv_heads : c.n_heads; }
int kv_dim_of(const anpd_model_cfg &c) { return kv_heads_of(c) * c.head_dim; }

struct Layout {  // byte offsets into the model workspace
    size_t rope_tab, tok, tree, batch, result, counter, x, h, y, qkv, att, gu, a, logits, part;
    // fast path: packed operands, partial sums of squares, packed weights
    size_t xp_d, xp_att, xp_f, ssp_a, ssp_b, qp, head_ctr, layer_tab, amax, row_ctr, bar, wp_lm, total;
    size_t xp_layers, xp_stride;   // the one-kernel step's operands (bytes; stride between the layers' sets in bf16 elements: 0, one set)
    std::vector<size_t> wp_qkv, wp_o, wp_gu, wp_down;
    int max_splits;
};

bool wants_mfma(const anpd_model_cfg *c)
{
    return c->gemm_path == ANPD_GEMM_MFMA || c->gemm_path == ANPD_GEMM_MFMA_LAUNCHES ||
           (c->gemm_path == ANPD_GEMM_AUTO && c->dtype == ANPD_BF16);
}

size_t packed_bytes(size_t n_tiles, int K) { return n_tiles * (size_t)((K + 31) / 32) * 1024; }

bool wants_mfma(const anpd_model_cfg *c);

bool cfg_ok(const anpd_model_cfg *c, const char **why)
{
#define REQ(cond, msg) if (!(cond)) { *why = msg; return false; }
    REQ(c, "cfg is NULL");
    REQ(c->n_layers >= 1 && c->d_model >= 8 && c->n_heads >= 1 && c->d_ffn >= 8 && c->vocab >= 1, "non-positive dimension");
    REQ(c->n_heads * c->head_dim == c->d_model, "d_model must equal n_heads * head_dim");
    REQ(c->n_kv_heads >= 0 && (c->n_kv_heads == 0 || c->n_heads % c->n_kv_heads == 0), "n_kv_heads must be 0 or divide n_heads");
    REQ(c->head_dim == 64 || c->head_dim == 128, "head_dim must be 64 or 128");
    REQ(c->d_model % 16 == 0 && c->d_ffn % 16 == 0 && c->vocab % 16 == 0, "d_model, d_ffn and vocab must be multiples of 16");
    REQ(c->dtype == ANPD_F32 || c->dtype == ANPD_BF16, "dtype must be ANPD_F32 or ANPD_BF16");
    REQ(c->page_tokens >= 8 && c->page_tokens <= 256 && (c->page_tokens & (c->page_tokens - 1)) == 0, "page_tokens must be a power of two in 8..256");
    REQ(c->max_window >= 1 && c->max_window <= ANPD_MAX_WINDOW, "max_window must be in 1..ANPD_MAX_WINDOW");
    REQ(c->max_positions >= 1 && c->max_positions <= (1 << 20), "max_positions must be in 1..2^20");
    REQ(c->gemm_path == ANPD_GEMM_AUTO || c->gemm_path == ANPD_GEMM_DOT || c->gemm_path == ANPD_GEMM_MFMA ||
            c->gemm_path == ANPD_GEMM_MFMA_LAUNCHES, "unknown gemm_path");
    REQ(!((c->gemm_path == ANPD_GEMM_MFMA || c->gemm_path == ANPD_GEMM_MFMA_LAUNCHES) && c->dtype != ANPD_BF16),
        "the MFMA path needs bf16 weights");
    REQ(c->rms_eps > 0.f && c->rope_base > 1.f, "rms_eps / rope_base out of range");
    REQ(!(wants_mfma(c) && c->page_tokens != 16), "the MFMA path needs page_tokens == 16");
#undef REQ
    return true;
}

Layout make_layout(const anpd_model_cfg *c)
{
    Layout L;
    const size_t MW = (size_t)c->max_window, d = (size_t)c->d_model, F = (size_t)c->d_ffn, V = (size_t)c->vocab;
    const size_t kvd = (size_t)kv_dim_of(*c);
    L.max_splits = (c->max_positions + kAttnSplit - 1) / kAttnSplit + 1;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes); return at; };
    L.rope_tab = take((size_t)c->max_positions * (c->head_dim / 2) * sizeof(float2));
    L.tok = take(ANPD_MAX_WINDOW * sizeof(int32_t));
    L.tree = take(3 * ANPD_MAX_WINDOW * sizeof(int32_t));                 // draft tree: parent, depth, visibility mask
    L.batch = take(ANPD_MAX_WINDOW * sizeof(int32_t) + ANPD_MAX_WINDOW * sizeof(SeqRef));   // batched step: sequence of every row, sequences
    // accepted, next, predictions, accepted path of a tree, (accepted, next) of every sequence of a batch
    L.result = take((2 + ANPD_MAX_WINDOW + ANPD_MAX_WINDOW + 1 + 2 * ANPD_MAX_WINDOW) * sizeof(int32_t));
    L.counter = take(sizeof(uint32_t));
    L.x = take(MW * d * 4);
    L.h = take(MW * d * 4);
    L.y = take(MW * d * 4);
    L.qkv = take(MW * (d + 2 * kvd) * 4);
    L.att = take(MW * d * 4);
    L.gu = take(MW * 2 * F * 4);
    L.a = take(MW * F * 4);
    L.logits = take(MW * V * 4);
    L.part = take((size_t)c->n_heads * L.max_splits * (wants_mfma(c) ? 32 : MW) * (c->head_dim + 2) * 4);
    L.xp_d = L.xp_att = L.xp_f = L.ssp_a = L.ssp_b = L.qp = L.head_ctr = L.wp_lm = 0;
    L.layer_tab = L.amax = L.row_ctr = L.bar = 0;
    L.xp_layers = L.xp_stride = 0;
    if (wants_mfma(c)) {
        L.xp_d = take(((d + 31) / 32) * 4 * 1024);
        L.xp_att = take(((d + 31) / 32) * 4 * 1024);
        L.xp_f = take(((F + 31) / 32) * 4 * 1024);
        // one set of the four operands for all layers (a set per layer, 48 MB at the 7B shape, cost 0.6 % of the
        // step at 640 cached positions and 1.6 % at 2048: lines that come round once per step are cold when
        // they are written)
        L.xp_stride = 0;
        L.xp_layers = take((3 * x_operand_elems((int)d) + x_operand_elems((int)F)) * sizeof(bf16_t));
        L.ssp_a = take((d / 16) * 32 * 4);
        L.ssp_b = take((d / 16) * 32 * 4);
        L.qp = take((size_t)c->n_heads * 4 * (c->head_dim / 32) * 1024);
        L.head_ctr = take((size_t)c->n_heads * kCounterStride * sizeof(uint32_t));
        L.layer_tab = take((size_t)c->n_layers * sizeof(LayerW));
        L.amax = take((V / 16) * 32 * sizeof(unsigned long long));
        L.row_ctr = take(sizeof(uint32_t));
        L.bar = take(kBarStride * 9 * sizeof(uint32_t) + (size_t)c->n_heads * kCounterStride * sizeof(uint32_t));   // barrier words, then per-head QKV counters
        L.wp_lm = take(packed_bytes(V / 16, (int)d));
        for (int l = 0; l < c->n_layers; ++l) {
            L.wp_qkv.push_back(take(packed_bytes((d + 2 * kvd) / 16, (int)d)));
            L.wp_o.push_back(take(packed_bytes(d / 16, (int)d)));
            L.wp_gu.push_back(take(packed_bytes(F / 8, (int)d)));
            L.wp_down.push_back(take(packed_bytes(d / 16, (int)F)));
        }
    }
    L.total = o;
    return L;
}

struct PrefillLayout {  // byte offsets into the caller's prefill workspace
    size_t tok, x, part, xq, xq_att, xq_f, qp, total;
};

// Sized for the worst alignment of the first row inside its cache page.
PrefillLayout make_prefill_layout(const anpd_model_cfg &c, int n_tokens)
{
    PrefillLayout L;
    const size_t G = ((size_t)n_tokens + 30) / 16, d = (size_t)c.d_model, F = (size_t)c.d_ffn;
    const size_t nks_d = (d + 31) / 32, nks_f = (F + 31) / 32;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes); return at; };
    L.tok = take((size_t)n_tokens * sizeof(int32_t));
    L.x = take(G * 16 * d * sizeof(float));
    L.part = take((size_t)kPgSplit * G * 16 * d * sizeof(float));
    L.xq = take(G * nks_d * 2048);
    L.xq_att = take(G * nks_d * 2048);
    L.xq_f = take(G * nks_f * 2048);
    L.qp = take((size_t)c.n_heads * G * (size_t)(c.head_dim / 32) * 2048);
    L.total = o;
    return L;
}

}  // namespace

struct anpd_model {
    anpd_model_cfg cfg;
    Layout lay;
    char *ws;
    bool mfma;
    int n_cu;
    bool mega;            // the one-kernel step is available
    bool mega_tree;       // ... and so is its draft-tree form
    bool mega_batch;      // ... and its several-sequences form
    bool mega_rows16;     // ... and its form for windows of 9 to 16 rows
    int mega_kc;          // k-steps per wave per work item of the one-kernel step (8: d_model <= 4096, 10: <= 5120)
    long long *trace;     // optional device buffer for barrier timestamps
    int mega_grid;
    bool plain_launch;    // launch the one-kernel step without the cooperative-launch API (profiling aid)
    int32_t spin_limit;   // polls before a grid-barrier wait gives up
    uint32_t bar_epoch;
    uint32_t ready_epoch;  // QKV phases run by the one-kernel step so far
    const void *embed, *final_norm, *lm_head;
    std::vector<const void *> attn_norm, wq, wk, wv, wo, ffn_norm, w_gate, w_up, w_down;
    int32_t *pin;  // pinned host staging: [0..32) window, [32..99) result and accepted path, [100] error flag of the
                   // persistent kernel, [128..224) draft tree (parent, depth, mask), [256..320) results of a batch,
                   // [384..416) sequence of every row of a batch, [512..768) its sequences (SeqRef)
    int32_t *pin_dev;  // the same memory as the device addresses it
    // optional per-kernel timing with events on the launch stream
    bool prof;
    std::vector<hipEvent_t> ev;
    std::vector<int> ev_cat;
    int ev_used;
    double prof_ms[ANPD_PROF_NCAT];
    int64_t prof_launches[ANPD_PROF_NCAT];
    int64_t prof_steps;
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
    return (size_t)c.n_layers * 2 * kv_dim_of(c) * c.page_tokens * (c.dtype == ANPD_BF16 ? 2 : 4);
}

// ---- GEMM dispatch -----------------------------------------------------------

// Up to three weight matrices side by side: n0 rows of W0, n1 of W1 (0 if absent), n2 of W2.
int32_t launch_gemm_dot(const float *X, int M, int K, const void *W0, const void *W1, const void *W2, int n0, int n1,
                        int n2, float *Y, int ldy, int dtype, hipStream_t st)
{
    constexpr int R = 4;
    int n_total = n0 + n1 + n2;
    dim3 grid((unsigned)((n_total + 4 * R - 1) / (4 * R)));
    if (dtype == ANPD_BF16)
        hipLaunchKernelGGL((gemm_dot_kernel<bf16_t, R>), grid, dim3(256), 0, st, X, M, K, (const bf16_t *)W0,
                           (const bf16_t *)W1, (const bf16_t *)W2, n0, n1, n_total, Y, ldy);
    else
        hipLaunchKernelGGL((gemm_dot_kernel<float, R>), grid, dim3(256), 0, st, X, M, K, (const float *)W0,
                           (const float *)W1, (const float *)W2, n0, n1, n_total, Y, ldy);
    HIP_TRY(hipGetLastError());
    return ANPD_OK;
}

// ---- fast path: packed MFMA GEMMs ---------------------------------------------

template <int EPI>
int32_t launch_fast(FastArgs &a, int n_cu, bool force_stream, hipStream_t st)
{
    const int kpw = (a.nks + kFastWaves - 1) / kFastWaves;
    if (a.cls == 8 && kpw <= 20 && !force_stream) {
        dim3 grid((unsigned)(a.n_tiles < n_cu ? a.n_tiles : n_cu)), block(kFastWaves * 64);
        if (kpw <= 2) hipLaunchKernelGGL((gemm_xs_kernel<2, EPI>), grid, block, 0, st, a);
        else if (kpw <= 4) hipLaunchKernelGGL((gemm_xs_kernel<4, EPI>), grid, block, 0, st, a);
        else if (kpw <= 8) hipLaunchKernelGGL((gemm_xs_kernel<8, EPI>), grid, block, 0, st, a);
        else if (kpw <= 16) hipLaunchKernelGGL((gemm_xs_kernel<16, EPI>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((gemm_xs_kernel<20, EPI>), grid, block, 0, st, a);
    } else if (a.cls == 8 || (a.cls == 16 && a.n_tiles <= n_cu)) {
        // one block per tile; several blocks share a compute unit.  Also the faster form for 9..16 rows when
        // there is only one tile per compute unit (grouping would leave half of them idle).
        dim3 grid((unsigned)a.n_tiles), block(kFastWaves * 64);
        const int nt = a.cls / 8;
        size_t smem = (size_t)kFastWaves * nt * 256 * sizeof(float);
        if (nt == 1) hipLaunchKernelGGL((gemm_stream_kernel<1, EPI>), grid, block, smem, st, a);
        else hipLaunchKernelGGL((gemm_stream_kernel<2, EPI>), grid, block, smem, st, a);
    } else {
        // windows of 9..32 rows: every block takes a contiguous range of at least two tiles, so that an
        // activation fragment is loaded once for several weight tiles
        const int nt = a.cls / 8;
        int blocks = a.n_tiles / 2 < n_cu ? a.n_tiles / 2 : n_cu;
        // (two fragments, between one and two tiles per compute unit: every compute unit gets a block of one or
        // two tiles rather than half of them a block of two: 13B shape, 9 rows: -0.8 % per step)
        if (nt == 2 && a.n_tiles < 2 * n_cu) blocks = a.n_tiles < n_cu ? a.n_tiles : n_cu;
        if (blocks < 1) blocks = 1;
        dim3 grid((unsigned)blocks), block(kFastWaves * 64);
        const int per_block = (a.n_tiles + blocks - 1) / blocks;
        if (nt == 2 && per_block <= 2) {
            size_t smem = (size_t)2 * kFastWaves * 2 * 256 * sizeof(float);
            hipLaunchKernelGGL((gemm_group_kernel<2, 2, EPI>), grid, block, smem, st, a);
        } else if (nt == 2 && per_block > 4) {
            // six, seven or eight tiles per pass: the smallest form that takes the block's tiles in one pass
            // (the eight-tile form sits at the register limit)
#define ANPD_GROUP2(TG_)                                                                                                          \
    do {                                                                                                                          \
        size_t smem = (size_t)TG_ * kFastWaves * 2 * 256 * sizeof(float);                                                         \
        static bool attr_set_g = false;                                                                                           \
        if (!attr_set_g) {                                                                                                        \
            HIP_TRY(hipFuncSetAttribute((const void *)gemm_group_kernel<2, TG_, EPI>, hipFuncAttributeMaxDynamicSharedMemorySize, \
                                        (int)smem));                                                                              \
            attr_set_g = true;                                                                                                    \
        }                                                                                                                         \
        hipLaunchKernelGGL((gemm_group_kernel<2, TG_, EPI>), grid, block, smem, st, a);                                           \
    } while (0)
            if (per_block <= 6) ANPD_GROUP2(6);
            else if (per_block == 7) ANPD_GROUP2(7);
            else ANPD_GROUP2(8);
#undef ANPD_GROUP2
        } else if (nt == 2) {
            size_t smem = (size_t)4 * kFastWaves * 2 * 256 * sizeof(float);
            static bool attr_set2 = false;
            if (!attr_set2) {
                HIP_TRY(hipFuncSetAttribute((const void *)gemm_group_kernel<2, 4, EPI>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
                attr_set2 = true;
            }
            hipLaunchKernelGGL((gemm_group_kernel<2, 4, EPI>), grid, block, smem, st, a);
        } else if (per_block <= 2) {
            size_t smem = (size_t)2 * kFastWaves * 4 * 256 * sizeof(float);
            hipLaunchKernelGGL((gemm_group_kernel<4, 2, EPI>), grid, block, smem, st, a);
        } else {
            size_t smem = (size_t)4 * kFastWaves * 4 * 256 * sizeof(float);
            static bool attr_set = false;
            if (!attr_set) {
                HIP_TRY(hipFuncSetAttribute((const void *)gemm_group_kernel<4, 4, EPI>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
                attr_set = true;
            }
            hipLaunchKernelGGL((gemm_group_kernel<4, 4, EPI>), grid, block, smem, st, a);
        }
    }
    HIP_TRY(hipGetLastError());
    return ANPD_OK;
}

int32_t launch_pack(const void *s0, const void *s1, const void *s2, void *dst, int mode, int n_tiles, int K, int d,
                    int head_dim, int kvd, hipStream_t st)
{
    const int nks = (K + 31) / 32;
    size_t total = (size_t)n_tiles * nks * 64;
    hipLaunchKernelGGL(pack_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, (const bf16_t *)s0,
                       (const bf16_t *)s1, (const bf16_t *)s2, (uint4 *)dst, mode, n_tiles, K, nks, d, head_dim, kvd);
    HIP_TRY(hipGetLastError());
    return ANPD_OK;
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

// Timing mark: an event after the launches of category `cat` (-1 = start of the step).
inline void mark(anpd_model *m, int cat, hipStream_t st)
{
    if (!m->prof) return;
    if (m->ev_used == (int)m->ev.size()) {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) return;
        m->ev.push_back(e);
        m->ev_cat.push_back(cat);
    }
    m->ev_cat[(size_t)m->ev_used] = cat;
    (void)hipEventRecord(m->ev[(size_t)m->ev_used], st);
    m->ev_used += 1;
}

// After the stream has been synchronised: add the intervals between this call's marks to the sums.
void collect_marks(anpd_model *m)
{
    if (!m->prof) return;
    for (int i = 1; i < m->ev_used; ++i) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, m->ev[(size_t)i - 1], m->ev[(size_t)i]) == hipSuccess) {
            m->prof_ms[m->ev_cat[(size_t)i]] += (double)ms;
            m->prof_launches[m->ev_cat[(size_t)i]] += 1;
        }
    }
    m->prof_steps += 1;
}

// tree: the window is a draft tree whose parent / depth / mask arrays are in the workspace
template <typename KT>
int32_t run_step_generic(anpd_model *m, anpd_kv *kv, int M, int mode, hipStream_t st, bool tree = false)
{
    const anpd_model_cfg &c = m->cfg;
    const Layout &L = m->lay;
    char *ws = m->ws;
    const int d = c.d_model, F = c.d_ffn, V = c.vocab, H = c.n_heads, dh = c.head_dim;
    const int Hkv = kv_heads_of(c), kvd = kv_dim_of(c);
    float *x = (float *)(ws + L.x), *h = (float *)(ws + L.h), *y = (float *)(ws + L.y);
    float *qkv = (float *)(ws + L.qkv), *att = (float *)(ws + L.att), *gu = (float *)(ws + L.gu);
    float *a = (float *)(ws + L.a), *logits = (float *)(ws + L.logits), *part = (float *)(ws + L.part);
    const float2 *rope = (const float2 *)(ws + L.rope_tab);
    const int32_t *tok = (const int32_t *)(ws + L.tok);
    int32_t *result = (int32_t *)(ws + L.result);
    uint32_t *counter = (uint32_t *)(ws + L.counter);
    KT *pool = (KT *)kv->pool;
    const float scale = 1.0f / sqrtf((float)dh);
    const int n_splits = (kv->len + M + kAttnSplit - 1) / kAttnSplit;
    const int32_t *t_parent = (const int32_t *)(ws + L.tree), *t_depth = tree ? t_parent + ANPD_MAX_WINDOW : nullptr;
    const uint32_t *t_mask = tree ? (const uint32_t *)(t_parent + 2 * ANPD_MAX_WINDOW) : nullptr;
    int32_t rc;

    m->ev_used = 0;
    mark(m, -1, st);
    hipLaunchKernelGGL((embed_kernel<KT>), dim3(M), dim3(256), 0, st, (const KT *)m->embed, tok, x, d);
    for (int l = 0; l < c.n_layers; ++l) {
        hipLaunchKernelGGL((addnorm_kernel<KT>), dim3(M), dim3(256), 0, st, x, l == 0 ? (const float *)nullptr : y,
                           (const KT *)m->attn_norm[l], h, d, c.rms_eps);
        mark(m, ANPD_PROF_OTHER, st);
        if ((rc = launch_gemm_dot(h, M, d, m->wq[l], m->wk[l], m->wv[l], d, kvd, kvd, qkv, d + 2 * kvd, c.dtype, st)) != ANPD_OK) return rc;
        mark(m, ANPD_PROF_GEMM_QKV, st);
        hipLaunchKernelGGL((rope_kv_kernel<KT>), dim3(M), dim3(256), 0, st, qkv, rope, pool, kv->d_table, kv->d_len, l,
                           c.n_layers, H, Hkv, dh, c.page_tokens, t_depth);
        mark(m, ANPD_PROF_OTHER, st);
        if (dh == 128) {
            hipLaunchKernelGGL((attn_kernel<KT, 128>), dim3(H, n_splits), dim3(256), 0, st, qkv, d + 2 * kvd, pool, kv->d_table,
                               kv->d_len, M, l, c.n_layers, H, Hkv, c.page_tokens, c.max_window, L.max_splits, scale, part, t_mask);
            hipLaunchKernelGGL((attn_combine_kernel<128>), dim3(M, H), dim3(128), 0, st, part, kv->d_len, H,
                               c.max_window, L.max_splits, att, (bf16_t *)nullptr, 8);
        } else {
            hipLaunchKernelGGL((attn_kernel<KT, 64>), dim3(H, n_splits), dim3(256), 0, st, qkv, d + 2 * kvd, pool, kv->d_table,
                               kv->d_len, M, l, c.n_layers, H, Hkv, c.page_tokens, c.max_window, L.max_splits, scale, part, t_mask);
            hipLaunchKernelGGL((attn_combine_kernel<64>), dim3(M, H), dim3(64), 0, st, part, kv->d_len, H, c.max_window,
                               L.max_splits, att, (bf16_t *)nullptr, 8);
        }
        mark(m, ANPD_PROF_ATTN, st);
        if ((rc = launch_gemm_dot(att, M, d, m->wo[l], nullptr, nullptr, d, 0, 0, y, d, c.dtype, st)) != ANPD_OK) return rc;
        mark(m, ANPD_PROF_GEMM_O, st);
        hipLaunchKernelGGL((addnorm_kernel<KT>), dim3(M), dim3(256), 0, st, x, y, (const KT *)m->ffn_norm[l], h, d,
                           c.rms_eps);
        mark(m, ANPD_PROF_OTHER, st);
        if ((rc = launch_gemm_dot(h, M, d, m->w_gate[l], m->w_up[l], nullptr, F, F, 0, gu, 2 * F, c.dtype, st)) != ANPD_OK) return rc;
        mark(m, ANPD_PROF_GEMM_GATE_UP, st);
        hipLaunchKernelGGL(swiglu_kernel, dim3((F + 255) / 256, M), dim3(256), 0, st, gu, a, F);
        mark(m, ANPD_PROF_OTHER, st);
        if ((rc = launch_gemm_dot(a, M, F, m->w_down[l], nullptr, nullptr, d, 0, 0, y, d, c.dtype, st)) != ANPD_OK) return rc;
        mark(m, ANPD_PROF_GEMM_DOWN, st);
    }
    hipLaunchKernelGGL((addnorm_kernel<KT>), dim3(M), dim3(256), 0, st, x, y, (const KT *)m->final_norm, h, d,
                       c.rms_eps);
    mark(m, ANPD_PROF_OTHER, st);
    if ((rc = launch_gemm_dot(h, M, d, m->lm_head, nullptr, nullptr, V, 0, 0, logits, V, c.dtype, st)) != ANPD_OK) return rc;
    mark(m, ANPD_PROF_GEMM_LM_HEAD, st);
    hipLaunchKernelGGL(argmax_accept_kernel, dim3(M), dim3(1024), 0, st, logits, V, M, tok, mode, result, kv->d_len,
                       counter);
    if (tree) {
        hipLaunchKernelGGL(accept_tree_kernel, dim3(1), dim3(64), 0, st, tok, t_parent, t_depth, M, result, kv->d_len, kv->len);
        hipLaunchKernelGGL((kv_compact_kernel<KT>), dim3((unsigned)(c.n_layers * 2 * Hkv)), dim3(128), 0, st, pool, kv->d_table,
                           (const int32_t *)result, kv->len, c.n_layers, Hkv, dh, c.page_tokens);
    }
    mark(m, ANPD_PROF_OTHER, st);
    HIP_TRY(hipGetLastError());
    return ANPD_OK;
}

// The fused bf16 step: per layer QKV(+norm, RoPE, cache write) -> attention -> combine -> O(+residual)
// -> gate/up(+norm, SwiGLU) -> down(+residual); then LM head(+norm) -> argmax / accept.
// A batched step: the sequences' descriptions are in the workspace (Layout::batch); `kv` is unused.
struct BatchLaunch {
    int n_seq, n_blocks /* (split, sequence) blocks per head */, grid_splits /* splits of the longest sequence */;
};

int32_t run_step_fast(anpd_model *m, anpd_kv *kv, int M, int mode, hipStream_t st, bool tree = false,
                      const BatchLaunch *batch = nullptr)
{
    const anpd_model_cfg &c = m->cfg;
    const Layout &L = m->lay;
    char *ws = m->ws;
    const int d = c.d_model, F = c.d_ffn, V = c.vocab, H = c.n_heads, dh = c.head_dim;
    const int Hkv = kv_heads_of(c), kvd = kv_dim_of(c);
    const int cls = window_class(M);
    float *x = (float *)(ws + L.x);
    float *logits = (float *)(ws + L.logits), *part = (float *)(ws + L.part);
    bf16_t *qp = (bf16_t *)(ws + L.qp);
    uint32_t *head_ctr = (uint32_t *)(ws + L.head_ctr);
    bf16_t *xp_d = (bf16_t *)(ws + L.xp_d), *xp_att = (bf16_t *)(ws + L.xp_att), *xp_f = (bf16_t *)(ws + L.xp_f);
    float *ssp_a = (float *)(ws + L.ssp_a), *ssp_b = (float *)(ws + L.ssp_b);
    const int32_t *tok = (const int32_t *)(ws + L.tok);
    int32_t *result = (int32_t *)(ws + L.result);
    uint32_t *counter = (uint32_t *)(ws + L.counter);
    const float scale = 1.0f / sqrtf((float)dh);
    const int n_splits = batch ? batch->grid_splits : n_splits_of(kv->len + M);
    const bool one_page = n_splits <= kSmallSplits;
    const int nks_d = (d + 31) / 32, nks_f = (F + 31) / 32;
    const int32_t *b_row_seq = (const int32_t *)(ws + L.batch);
    const SeqRef *b_seqs = (const SeqRef *)(ws + L.batch + ANPD_MAX_WINDOW * sizeof(int32_t));
    int32_t *dummy_len = (int32_t *)(ws + L.counter) + 16;   // the per-row argmax kernel's length update goes nowhere in a batch
    const int32_t *t_parent = (const int32_t *)(ws + L.tree), *t_depth = t_parent + ANPD_MAX_WINDOW;
    const uint32_t *t_mask = (const uint32_t *)(t_parent + 2 * ANPD_MAX_WINDOW);
    int32_t rc;

    FastArgs base;
    std::memset(&base, 0, sizeof(base));
    base.M = M;
    base.cls = cls;
    base.inv_d = 1.0f / (float)d;
    base.eps = c.rms_eps;
    base.n_ss = d / 16;
    base.d = d;
    base.x = x;
    if (!batch) {
        base.pool = (bf16_t *)kv->pool;
        base.page_table = kv->d_table;
        base.len_ptr = kv->d_len;
    }
    base.rope = (const float2 *)(ws + L.rope_tab);
    base.n_layers = c.n_layers;
    base.n_heads = H;
    base.n_kv_heads = Hkv;
    base.head_dim = dh;

    m->ev_used = 0;
    mark(m, -1, st);
    {
        FastArgs a = base;
        a.gain = (const bf16_t *)m->attn_norm[0];
        a.xp_next = xp_d;
        a.ssp_next = ssp_a;
        hipLaunchKernelGGL(embed_fast_kernel, dim3(d / 16), dim3(64), 0, st, (const bf16_t *)m->embed, tok, a);
    }
    mark(m, ANPD_PROF_OTHER, st);
    for (int l = 0; l < c.n_layers; ++l) {
        {
            FastArgs a = base;
            a.Wp = (const uint4 *)(ws + L.wp_qkv[(size_t)l]);
            a.Xp = (const uint4 *)xp_d;
            a.nks = nks_d;
            a.n_tiles = (d + 2 * kvd) / 16;
            a.ssp = ssp_a;
            a.qp = qp;
            a.layer = l;
            a.depth = t_depth;
            a.seqs = b_seqs;
            a.row_seq = b_row_seq;
            rc = batch ? launch_fast<EPI_QKV_BATCH>(a, m->n_cu, false, st)
                       : (tree ? launch_fast<EPI_QKV_TREE>(a, m->n_cu, false, st) : launch_fast<EPI_QKV>(a, m->n_cu, false, st));
            if (rc != ANPD_OK) return rc;
        }
        mark(m, ANPD_PROF_GEMM_QKV, st);
        // (n_splits <= kSmallSplits: every split of the step has one page per wave: the leaner instantiation)
        if (batch) {
#define ANPD_ATTN_B(DH_, MAXP_)                                                                                            \
    hipLaunchKernelGGL((attn_batch_kernel<DH_, MAXP_>), dim3(H, n_splits, batch->n_seq), dim3(kFastThreads), 0, st,      \
                       (const uint4 *)qp, b_seqs, b_row_seq, batch->n_blocks, M, l, c.n_layers, H, Hkv, L.max_splits, scale, part, \
                       head_ctr, xp_att, cls)
            if (dh == 128) { if (one_page) ANPD_ATTN_B(128, 1); else ANPD_ATTN_B(128, kFastPages); }
            else if (one_page) ANPD_ATTN_B(64, 1);
            else ANPD_ATTN_B(64, kFastPages);
#undef ANPD_ATTN_B
        } else {
#define ANPD_ATTN(DH_, TREE_, MAXP_)                                                                                       \
    hipLaunchKernelGGL((attn_fast_kernel<DH_, TREE_, MAXP_>), dim3(H, n_splits), dim3(kFastThreads), 0, st, (const uint4 *)qp,  \
                       (const bf16_t *)kv->pool, kv->d_table, kv->d_len, M, l, c.n_layers, H, Hkv, L.max_splits, scale, part,   \
                       head_ctr, xp_att, cls, t_mask)
#define ANPD_ATTN_T(DH_, MAXP_) do { if (tree) ANPD_ATTN(DH_, true, MAXP_); else ANPD_ATTN(DH_, false, MAXP_); } while (0)
            if (dh == 128) { if (one_page) ANPD_ATTN_T(128, 1); else ANPD_ATTN_T(128, kFastPages); }
            else if (one_page) ANPD_ATTN_T(64, 1);
            else ANPD_ATTN_T(64, kFastPages);
#undef ANPD_ATTN_T
#undef ANPD_ATTN
        }
        mark(m, ANPD_PROF_ATTN, st);
        {
            FastArgs a = base;
            a.Wp = (const uint4 *)(ws + L.wp_o[(size_t)l]);
            a.Xp = (const uint4 *)xp_att;
            a.nks = nks_d;
            a.n_tiles = d / 16;
            a.gain = (const bf16_t *)m->ffn_norm[l];
            a.xp_next = xp_d;
            a.ssp_next = ssp_b;
            if ((rc = launch_fast<EPI_RESIDUAL>(a, m->n_cu, false, st)) != ANPD_OK) return rc;
        }
        mark(m, ANPD_PROF_GEMM_O, st);
        {
            FastArgs a = base;
            a.Wp = (const uint4 *)(ws + L.wp_gu[(size_t)l]);
            a.Xp = (const uint4 *)xp_d;
            a.nks = nks_d;
            a.n_tiles = F / 8;
            a.ssp = ssp_b;
            a.ap = xp_f;
            if ((rc = launch_fast<EPI_GATE_UP>(a, m->n_cu, false, st)) != ANPD_OK) return rc;
        }
        mark(m, ANPD_PROF_GEMM_GATE_UP, st);
        {
            FastArgs a = base;
            a.Wp = (const uint4 *)(ws + L.wp_down[(size_t)l]);
            a.Xp = (const uint4 *)xp_f;
            a.nks = nks_f;
            a.n_tiles = d / 16;
            a.gain = (const bf16_t *)(l + 1 < c.n_layers ? m->attn_norm[(size_t)l + 1] : m->final_norm);
            a.xp_next = xp_d;
            a.ssp_next = ssp_a;
            if ((rc = launch_fast<EPI_RESIDUAL>(a, m->n_cu, false, st)) != ANPD_OK) return rc;
        }
        mark(m, ANPD_PROF_GEMM_DOWN, st);
    }
    {
        FastArgs a = base;
        a.Wp = (const uint4 *)(ws + L.wp_lm);
        a.Xp = (const uint4 *)xp_d;
        a.nks = nks_d;
        a.n_tiles = V / 16;
        a.ssp = ssp_a;
        a.Y = logits;
        a.ldy = V;
        if ((rc = launch_fast<EPI_LOGITS>(a, m->n_cu, false, st)) != ANPD_OK) return rc;
    }
    mark(m, ANPD_PROF_GEMM_LM_HEAD, st);
    hipLaunchKernelGGL(argmax_accept_kernel, dim3(M), dim3(1024), 0, st, logits, V, M, tok, batch ? (int)ANPD_APPEND : mode, result,
                       batch ? dummy_len : kv->d_len, counter);
    if (batch) hipLaunchKernelGGL(accept_batch_kernel, dim3(1), dim3(64), 0, st, tok, b_seqs, batch->n_seq, mode, result);
    if (tree) {
        hipLaunchKernelGGL(accept_tree_kernel, dim3(1), dim3(64), 0, st, tok, t_parent, t_depth, M, result, kv->d_len, kv->len);
        hipLaunchKernelGGL(kvf_compact_kernel, dim3((unsigned)(c.n_layers * 2 * Hkv)), dim3(128), 0, st, (bf16_t *)kv->pool,
                           kv->d_table, (const int32_t *)result, kv->len, c.n_layers, Hkv, dh);
    }
    mark(m, ANPD_PROF_OTHER, st);
    HIP_TRY(hipGetLastError());
    return ANPD_OK;
}

// The step as one persistent kernel (window class 8).
// tree (nullable): the pinned draft-tree arrays parent[32], depth[32], mask[32] of a window of at most 8 rows.
// batch (nullable): several sequences side by side (kv is null then): seqs[n_seq], row_seq[M] and the lengths the host
// knows them to have.
struct MegaBatch {
    int n_seq;
    const SeqRef *seqs;
    const int32_t *row_seq;
    const int32_t *len;
};
int32_t run_step_mega(anpd_model *m, anpd_kv *kv, const int32_t *window, int M, int mode, bool want_logits, hipStream_t st,
                      const int32_t *tree = nullptr, const MegaBatch *batch = nullptr)
{
    const anpd_model_cfg &c = m->cfg;
    const Layout &L = m->lay;
    char *ws = m->ws;
    MegaArgs g;
    std::memset(&g, 0, sizeof(g));
    g.layers = (const LayerW *)(ws + L.layer_tab);
    g.n_layers = c.n_layers;
    g.wp_lm = (const uint4 *)(ws + L.wp_lm);
    g.final_gain = (const bf16_t *)m->final_norm;
    g.embed = (const bf16_t *)m->embed;
    g.d = c.d_model; g.F = c.d_ffn; g.V = c.vocab; g.n_heads = c.n_heads; g.n_kv_heads = kv_heads_of(c); g.head_dim = c.head_dim;
    g.M = M; g.mode = mode;
    g.inv_d = 1.0f / (float)c.d_model; g.eps = c.rms_eps; g.scale = 1.0f / sqrtf((float)c.head_dim);
    g.x = (float *)(ws + L.x);
    g.xp_layers = (bf16_t *)(ws + L.xp_layers);
    g.xp_stride = L.xp_stride;
    g.qp = (bf16_t *)(ws + L.qp);
    g.ssp_a = (float *)(ws + L.ssp_a); g.ssp_b = (float *)(ws + L.ssp_b); g.part = (float *)(ws + L.part);
    g.head_counter = (uint32_t *)(ws + L.head_ctr);
    if (kv) { g.pool = (bf16_t *)kv->pool; g.page_table = kv->d_table; g.len_ptr = kv->d_len; }
    g.rope = (const float2 *)(ws + L.rope_tab);
    g.max_splits = L.max_splits;
    g.logits = want_logits ? (float *)(ws + L.logits) : nullptr;
    g.amax = (unsigned long long *)(ws + L.amax);
    for (int i = 0; i < 16; ++i) g.tok[i] = i < M ? window[i] : 0;
    g.result = (int32_t *)(ws + L.result);
    g.host_result = m->pin_dev + 32;
    g.row_counter = (uint32_t *)(ws + L.row_ctr);
    g.bar = (uint32_t *)(ws + L.bar);
    g.bar_epoch = m->bar_epoch;
    g.error = m->pin_dev + 100;
    g.spin_limit = m->spin_limit;
    g.qkv_ready = (uint32_t *)(ws + L.bar) + kBarStride * 9;
    g.ready_epoch = m->ready_epoch;
    g.trace = m->trace;
    if (tree)
        for (int i = 0; i < 8; ++i) {
            g.parent[i] = tree[i];
            g.depth[i] = tree[ANPD_MAX_WINDOW + i];
            g.mask[i] = (uint32_t)tree[2 * ANPD_MAX_WINDOW + i];
        }
    if (batch) {
        g.n_seq = batch->n_seq;
        g.host_batch = m->pin_dev + 256;
        int tasks = 0;
        for (int s = 0; s < batch->n_seq; ++s) {
            g.seqs[s] = batch->seqs[s];
            g.task0[s] = tasks;
            const int splits = n_splits_of(batch->len[s] + batch->seqs[s].n_rows);
            tasks += splits * c.n_heads;
            g.n_att_blocks += splits;
        }
        g.task0[batch->n_seq] = tasks;
        for (int i = 0; i < M; ++i) g.row_seq[i] = batch->row_seq[i];
    }
    m->ev_used = 0;
    mark(m, -1, st);
    void *args[] = {&g};
    const int form = batch ? MEGA_BATCH : (tree ? MEGA_TREE : MEGA_CHAIN);
    const void *fn128[] = {(const void *)verify_mega_kernel<128, MEGA_CHAIN>, (const void *)verify_mega_kernel<128, MEGA_TREE>,
                           (const void *)verify_mega_kernel<128, MEGA_BATCH>};
    const void *fn64[] = {(const void *)verify_mega_kernel<64, MEGA_CHAIN>, (const void *)verify_mega_kernel<64, MEGA_TREE>,
                          (const void *)verify_mega_kernel<64, MEGA_BATCH>};
    const void *fn = c.head_dim == 128 ? fn128[form] : fn64[form];
    if (M > 8)   // windows of 9 to 16 rows (chains only; the caller has checked mega_rows16)
        fn = c.head_dim == 128 ? (const void *)verify_mega_kernel<128, MEGA_CHAIN, 2> : (const void *)verify_mega_kernel<64, MEGA_CHAIN, 2>;
    else if (m->mega_kc == 10)   // d_model above 4096 (chains only)
        fn = c.head_dim == 128 ? (const void *)verify_mega_kernel<128, MEGA_CHAIN, 1, 10> : (const void *)verify_mega_kernel<64, MEGA_CHAIN, 1, 10>;
    if (m->plain_launch) {
        // profiling aid (see anpd_model_create): an ordinary launch of the same grid
        HIP_TRY(hipLaunchKernel(fn, dim3((unsigned)m->mega_grid), dim3(kFastThreads), args, 0, st));
    } else {
        HIP_TRY(hipLaunchCooperativeKernel(fn, dim3((unsigned)m->mega_grid), dim3(kFastThreads), args, 0, st));
    }
    m->bar_epoch += (uint32_t)kMegaBarriers(c.n_layers);
    m->ready_epoch += (uint32_t)c.n_layers;
    if (tree) {
        // the winning path's K and V to consecutive positions (a no-op kernel when it is the first candidate)
        hipLaunchKernelGGL(kvf_compact_kernel, dim3((unsigned)(c.n_layers * 2 * kv_heads_of(c))), dim3(128), 0, st, (bf16_t *)kv->pool,
                           kv->d_table, (const int32_t *)(ws + L.result), kv->len, c.n_layers, kv_heads_of(c), c.head_dim);
        HIP_TRY(hipGetLastError());
    }
    mark(m, ANPD_PROF_STEP, st);
    return ANPD_OK;
}

// ---- prompt processing on the matrix cores ------------------------------------

template <int EPI, int TN>
int32_t launch_prefill_gemm_tn(const PrefillArgs &a, int n_bt, int n_br, hipStream_t st)
{
    static bool attr_set = false;   // per instantiation
    if (!attr_set) {
        HIP_TRY(hipFuncSetAttribute((const void *)prefill_gemm_kernel<EPI, TN>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kPgLdsBytes));
        attr_set = true;
    }
    hipLaunchKernelGGL((prefill_gemm_kernel<EPI, TN>), dim3((unsigned)(n_bt * a.S * n_br)), dim3(kPgThreads), kPgLdsBytes, st, a);
    HIP_TRY(hipGetLastError());
    return ANPD_OK;
}

// Blocks of 256 or of 192 output features, whichever takes fewer rounds of the chip's compute units, a
// round of the smaller block counted as kPfSmallBlock of the larger one's (measured at the 7B shape: 0.85 - 0.89).
constexpr double kPfSmallBlock = 0.87;
template <int EPI>
int32_t launch_prefill_gemm(const PrefillArgs &a, int n_cu, hipStream_t st)
{
    const int n_br = (a.G + 7) / 8;
    const int bt4 = (a.n_tiles + 15) / 16, bt3 = (a.n_tiles + 11) / 12;
    const int rounds4 = (bt4 * a.S * n_br + n_cu - 1) / n_cu, rounds3 = (bt3 * a.S * n_br + n_cu - 1) / n_cu;
    const bool small = kPfSmallBlock * rounds3 < (double)rounds4;
    return small ? launch_prefill_gemm_tn<EPI, 3>(a, bt3, n_br, st) : launch_prefill_gemm_tn<EPI, 4>(a, bt4, n_br, st);
}

// All P rows at once; per layer norm -> QKV(+RoPE, cache write) -> attention -> O(+residual) -> norm ->
// gate/up(+SwiGLU) -> down(+residual); the last row then goes through the step's LM head and argmax.
int32_t run_prefill_mfma(anpd_model *m, anpd_kv *kv, int P, char *pws, const PrefillLayout &PL, hipStream_t st)
{
    const anpd_model_cfg &c = m->cfg;
    const Layout &L = m->lay;
    char *ws = m->ws;
    const int d = c.d_model, F = c.d_ffn, V = c.vocab, H = c.n_heads, dh = c.head_dim;
    const int len = kv->len, r0 = len & 15;
    const int G = (r0 + P + 15) / 16;
    const int nks_d = (d + 31) / 32, nks_f = (F + 31) / 32;
    const int32_t *tok = (const int32_t *)(pws + PL.tok);
    float *x = (float *)(pws + PL.x), *part = (float *)(pws + PL.part);
    bf16_t *xq = (bf16_t *)(pws + PL.xq), *xq_att = (bf16_t *)(pws + PL.xq_att), *xq_f = (bf16_t *)(pws + PL.xq_f);
    bf16_t *qp = (bf16_t *)(pws + PL.qp);
    const float inv_d = 1.0f / (float)d, scale = 1.0f / sqrtf((float)dh);
    int32_t rc;

    PrefillArgs base;
    std::memset(&base, 0, sizeof(base));
    base.G = G;
    base.L = len;
    base.P = P;
    base.S = 1;
    base.part = part;
    base.d = d;
    base.qp = qp;
    base.pool = (bf16_t *)kv->pool;
    base.page_table = kv->d_table;
    base.rope = (const float2 *)(ws + L.rope_tab);
    base.n_layers = c.n_layers;
    base.n_heads = H;
    base.n_kv_heads = kv_heads_of(c);
    base.head_dim = dh;

    m->ev_used = 0;
    mark(m, -1, st);
    // columns F .. 32 * nks_f of the down projection's operand meet zero weights: they must not hold NaN patterns
    if (F % 32 != 0) HIP_TRY(hipMemsetAsync(xq_f, 0, (size_t)G * nks_f * 2048, st));
    hipLaunchKernelGGL((prefill_norm_kernel<true>), dim3((unsigned)(G * 16)), dim3(256), 0, st, (const bf16_t *)m->embed, tok, x,
                       (const float *)nullptr, 0, (const bf16_t *)m->attn_norm[0], xq, nks_d, d, len, P, inv_d, c.rms_eps);
    mark(m, ANPD_PROF_OTHER, st);
    for (int l = 0; l < c.n_layers; ++l) {
        {
            PrefillArgs a = base;
            a.Wp = (const uint4 *)(ws + L.wp_qkv[(size_t)l]);
            a.Xq = (const uint4 *)xq;
            a.nks = nks_d;
            a.n_tiles = (d + 2 * kv_dim_of(c)) / 16;
            a.layer = l;
            if ((rc = launch_prefill_gemm<EPI_QKV>(a, m->n_cu, st)) != ANPD_OK) return rc;
        }
        mark(m, ANPD_PROF_GEMM_QKV, st);
        if (dh == 128)
            hipLaunchKernelGGL((prefill_attn_kernel<128>), dim3((unsigned)H, (unsigned)((G + 3) / 4)), dim3(256), 0, st, (const uint4 *)qp,
                               (const bf16_t *)kv->pool, kv->d_table, G, len, P, l, c.n_layers, H, kv_heads_of(c), scale, xq_att, nks_d);
        else
            hipLaunchKernelGGL((prefill_attn_kernel<64>), dim3((unsigned)H, (unsigned)((G + 3) / 4)), dim3(256), 0, st, (const uint4 *)qp,
                               (const bf16_t *)kv->pool, kv->d_table, G, len, P, l, c.n_layers, H, kv_heads_of(c), scale, xq_att, nks_d);
        mark(m, ANPD_PROF_ATTN, st);
        {
            PrefillArgs a = base;
            a.Wp = (const uint4 *)(ws + L.wp_o[(size_t)l]);
            a.Xq = (const uint4 *)xq_att;
            a.nks = nks_d;
            a.n_tiles = d / 16;
            a.S = kPgSplit;
            if ((rc = launch_prefill_gemm<EPI_RESIDUAL>(a, m->n_cu, st)) != ANPD_OK) return rc;
        }
        mark(m, ANPD_PROF_GEMM_O, st);
        hipLaunchKernelGGL((prefill_norm_kernel<false>), dim3((unsigned)(G * 16)), dim3(256), 0, st, (const bf16_t *)nullptr, tok, x,
                           (const float *)part, kPgSplit, (const bf16_t *)m->ffn_norm[l], xq, nks_d, d, len, P, inv_d, c.rms_eps);
        mark(m, ANPD_PROF_OTHER, st);
        {
            PrefillArgs a = base;
            a.Wp = (const uint4 *)(ws + L.wp_gu[(size_t)l]);
            a.Xq = (const uint4 *)xq;
            a.nks = nks_d;
            a.n_tiles = F / 8;
            a.out = xq_f;
            a.out_nks = nks_f;
            if ((rc = launch_prefill_gemm<EPI_GATE_UP>(a, m->n_cu, st)) != ANPD_OK) return rc;
        }
        mark(m, ANPD_PROF_GEMM_GATE_UP, st);
        {
            PrefillArgs a = base;
            a.Wp = (const uint4 *)(ws + L.wp_down[(size_t)l]);
            a.Xq = (const uint4 *)xq_f;
            a.nks = nks_f;
            a.n_tiles = d / 16;
            a.S = kPgSplit;
            if ((rc = launch_prefill_gemm<EPI_RESIDUAL>(a, m->n_cu, st)) != ANPD_OK) return rc;
        }
        mark(m, ANPD_PROF_GEMM_DOWN, st);
        if (l + 1 < c.n_layers) {
            hipLaunchKernelGGL((prefill_norm_kernel<false>), dim3((unsigned)(G * 16)), dim3(256), 0, st, (const bf16_t *)nullptr, tok,
                               x, (const float *)part, kPgSplit, (const bf16_t *)m->attn_norm[(size_t)l + 1], xq, nks_d, d, len, P, inv_d, c.rms_eps);
            mark(m, ANPD_PROF_OTHER, st);
        }
    }
    // last row -> the step's LM head, argmax and length update (one appended row)
    hipLaunchKernelGGL(prefill_last_kernel, dim3((unsigned)(d / 16)), dim3(64), 0, st, x + (size_t)(r0 + P - 1) * d,
                       (const float *)(part + (size_t)(r0 + P - 1) * d), kPgSplit, (size_t)G * 16 * d, (const bf16_t *)m->final_norm, (bf16_t *)(ws + L.xp_d), (float *)(ws + L.ssp_a), kv->d_len, len + P - 1);
    mark(m, ANPD_PROF_OTHER, st);
    {
        FastArgs a;
        std::memset(&a, 0, sizeof(a));
        a.M = 1;
        a.cls = 8;
        a.inv_d = inv_d;
        a.eps = c.rms_eps;
        a.n_ss = d / 16;
        a.d = d;
        a.Wp = (const uint4 *)(ws + L.wp_lm);
        a.Xp = (const uint4 *)(ws + L.xp_d);
        a.nks = nks_d;
        a.n_tiles = V / 16;
        a.ssp = (const float *)(ws + L.ssp_a);
        a.Y = (float *)(ws + L.logits);
        a.ldy = V;
        if ((rc = launch_fast<EPI_LOGITS>(a, m->n_cu, false, st)) != ANPD_OK) return rc;
    }
    mark(m, ANPD_PROF_GEMM_LM_HEAD, st);
    hipLaunchKernelGGL(argmax_accept_kernel, dim3(1), dim3(1024), 0, st, (const float *)(ws + L.logits), V, 1,
                       (const int32_t *)(ws + L.tok), (int)ANPD_APPEND, (int32_t *)(ws + L.result), kv->d_len,
                       (uint32_t *)(ws + L.counter));
    mark(m, ANPD_PROF_OTHER, st);
    HIP_TRY(hipGetLastError());
    return ANPD_OK;
}

// After the stream has been synchronised: did a grid barrier of the one-kernel step give up?  Then the
// counters are no longer in step: start them over.
bool barrier_gave_up(anpd_model *m, hipStream_t st)
{
    if (m->pin[100] == 0) return false;
    m->pin[100] = 0;
    (void)hipMemsetAsync(m->ws + m->lay.bar, 0, kBarStride * 9 * sizeof(uint32_t) + (size_t)m->cfg.n_heads * kCounterStride * sizeof(uint32_t), st);
    (void)hipStreamSynchronize(st);
    m->bar_epoch = 0;
    m->ready_epoch = 0;
    return true;
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
    m->mfma = wants_mfma(cfg);
    {
        int dev = 0;
        hipDeviceProp_t prop;
        m->n_cu = 256;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
            m->n_cu = prop.multiProcessorCount;
    }
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
    m->prof = false;
    m->ev_used = 0;
    m->prof_steps = 0;
    for (int i = 0; i < ANPD_PROF_NCAT; ++i) { m->prof_ms[i] = 0.0; m->prof_launches[i] = 0; }

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
    hipError_t e = hipHostMalloc((void **)&m->pin, 1024 * sizeof(int32_t), hipHostMallocDefault);
    if (e != hipSuccess) { delete m; return fail(ANPD_E_HIP, "hipHostMalloc: %s", hipGetErrorString(e)); }
    std::memset(m->pin, 0, 1024 * sizeof(int32_t));
    e = hipHostGetDevicePointer((void **)&m->pin_dev, m->pin, 0);
    if (e != hipSuccess) { (void)hipHostFree(m->pin); delete m; return fail(ANPD_E_HIP, "hipHostGetDevicePointer: %s", hipGetErrorString(e)); }
    e = hipMemsetAsync(m->ws, 0, m->mfma ? lay.wp_lm : lay.total, st);
    if (e == hipSuccess) e = hipMemcpyAsync(m->ws + lay.rope_tab, tab.data(), tab.size() * sizeof(float2), hipMemcpyHostToDevice, st);
    int32_t prc = ANPD_OK;
    m->mega = false;
    m->mega_tree = false;
    m->mega_batch = false;
    m->trace = nullptr;
    m->mega_grid = 0;
    m->bar_epoch = 0;
    m->ready_epoch = 0;
    m->spin_limit = 1 << 21;
    // ANPD_MEGA_PLAIN_LAUNCH=1: an ordinary launch of the same grid.  Only for profilers that cannot
    // cope with the cooperative queue; all blocks are resident only if nothing else runs on the device
    // (otherwise a barrier wait times out and anpd_verify reports it).
    {
        const char *pl = std::getenv("ANPD_MEGA_PLAIN_LAUNCH");
        m->plain_launch = pl && pl[0] == '1';
    }
    m->mega_rows16 = false;
    m->mega_kc = (cfg->d_model + 31) / 32 <= 2 * kChunk * kFastWaves ? kChunk : 10;
    if (e == hipSuccess && m->mfma && cfg->gemm_path != ANPD_GEMM_MFMA_LAUNCHES && (cfg->d_model + 31) / 32 <= 2 * 10 * kFastWaves) {
        // the persistent step needs every block resident at once: one block per compute unit
        int per_cu = 0;
        hipError_t oe;
        if (m->mega_kc == kChunk)
            oe = cfg->head_dim == 128 ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, verify_mega_kernel<128>, kFastThreads, 0)
                                      : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, verify_mega_kernel<64>, kFastThreads, 0);
        else
            oe = cfg->head_dim == 128
                     ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, verify_mega_kernel<128, MEGA_CHAIN, 1, 10>, kFastThreads, 0)
                     : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, verify_mega_kernel<64, MEGA_CHAIN, 1, 10>, kFastThreads, 0);
        if (oe == hipSuccess && per_cu >= 1) {
            std::vector<LayerW> tab((size_t)cfg->n_layers);
            for (int l = 0; l < cfg->n_layers; ++l) {
                tab[(size_t)l].qkv = (const uint4 *)(m->ws + lay.wp_qkv[(size_t)l]);
                tab[(size_t)l].o = (const uint4 *)(m->ws + lay.wp_o[(size_t)l]);
                tab[(size_t)l].gu = (const uint4 *)(m->ws + lay.wp_gu[(size_t)l]);
                tab[(size_t)l].down = (const uint4 *)(m->ws + lay.wp_down[(size_t)l]);
                tab[(size_t)l].attn_gain = (const bf16_t *)m->attn_norm[(size_t)l];
                tab[(size_t)l].ffn_gain = (const bf16_t *)m->ffn_norm[(size_t)l];
            }
            e = hipMemcpyAsync(m->ws + lay.layer_tab, tab.data(), tab.size() * sizeof(LayerW), hipMemcpyHostToDevice, st);
            if (e == hipSuccess) e = hipStreamSynchronize(st);  // `tab` is about to go out of scope
            m->mega = true;
            m->mega_grid = m->n_cu;
            int per_cu_t = 0;
            hipError_t te = cfg->head_dim == 128
                                ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu_t, verify_mega_kernel<128, MEGA_TREE>, kFastThreads, 0)
                                : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu_t, verify_mega_kernel<64, MEGA_TREE>, kFastThreads, 0);
            m->mega_tree = te == hipSuccess && per_cu_t >= 1 && m->mega_kc == kChunk;
            if (te != hipSuccess) (void)hipGetLastError();
            int per_cu_b = 0;
            te = cfg->head_dim == 128
                     ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu_b, verify_mega_kernel<128, MEGA_BATCH>, kFastThreads, 0)
                     : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu_b, verify_mega_kernel<64, MEGA_BATCH>, kFastThreads, 0);
            m->mega_batch = te == hipSuccess && per_cu_b >= 1 && m->mega_kc == kChunk;
            if (te != hipSuccess) (void)hipGetLastError();
            int per_cu_r = 0;
            te = cfg->head_dim == 128
                     ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu_r, verify_mega_kernel<128, MEGA_CHAIN, 2>, kFastThreads, 0)
                     : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu_r, verify_mega_kernel<64, MEGA_CHAIN, 2>, kFastThreads, 0);
            m->mega_rows16 = te == hipSuccess && per_cu_r >= 1 && m->mega_kc == kChunk;
            if (te != hipSuccess) (void)hipGetLastError();

        } else {
            (void)hipGetLastError();
        }
    }
    if (e == hipSuccess && m->mfma) {
        // repack every matrix into MFMA-fragment order inside the workspace
        const int d = cfg->d_model, F = cfg->d_ffn, dh = cfg->head_dim, kvd = kv_dim_of(*cfg);
        for (int l = 0; l < cfg->n_layers && prc == ANPD_OK; ++l) {
            prc = launch_pack(m->wq[l], m->wk[l], m->wv[l], m->ws + lay.wp_qkv[(size_t)l], PACK_QKV, (d + 2 * kvd) / 16, d, d, dh, kvd, st);
            if (prc == ANPD_OK) prc = launch_pack(m->wo[l], nullptr, nullptr, m->ws + lay.wp_o[(size_t)l], PACK_PLAIN, d / 16, d, d, dh, kvd, st);
            if (prc == ANPD_OK) prc = launch_pack(m->w_gate[l], m->w_up[l], nullptr, m->ws + lay.wp_gu[(size_t)l], PACK_GATE_UP, F / 8, d, d, dh, kvd, st);
            if (prc == ANPD_OK) prc = launch_pack(m->w_down[l], nullptr, nullptr, m->ws + lay.wp_down[(size_t)l], PACK_PLAIN, d / 16, F, d, dh, kvd, st);
        }
        if (prc == ANPD_OK) prc = launch_pack(m->lm_head, nullptr, nullptr, m->ws + lay.wp_lm, PACK_PLAIN, cfg->vocab / 16, d, d, dh, kvd, st);
    }
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess || prc != ANPD_OK) {
        (void)hipHostFree(m->pin);
        delete m;
        return prc != ANPD_OK ? prc : fail(ANPD_E_HIP, "anpd_model_create: %s", hipGetErrorString(e));
    }
    *out = m;
    return ANPD_OK;
}

void anpd_model_destroy(anpd_model_t *m)
{
    if (!m) return;
    if (m->pin) (void)hipHostFree(m->pin);
    for (hipEvent_t e : m->ev) (void)hipEventDestroy(e);
    delete m;
}

int32_t anpd_model_trace(anpd_model_t *m, void *buffer, size_t bytes)
{
    if (!m) return fail(ANPD_E_INVAL, "anpd_model_trace: NULL handle");
    if (buffer && (!m->mega || bytes < (size_t)m->mega_grid * kTraceEvents * sizeof(long long)))
        return fail(ANPD_E_CAPACITY, "anpd_model_trace: needs %zu bytes and the one-kernel step",
                    (size_t)m->mega_grid * kTraceEvents * sizeof(long long));
    m->trace = (long long *)buffer;
    return m->mega ? m->mega_grid : 0;
}

int32_t anpd_model_set_barrier_spin_limit(anpd_model_t *m, int32_t spins)
{
    if (!m) return fail(ANPD_E_INVAL, "anpd_model_set_barrier_spin_limit: NULL handle");
    if (spins < 0) return fail(ANPD_E_INVAL, "anpd_model_set_barrier_spin_limit: spins must be >= 0");
    m->spin_limit = spins == 0 ? (1 << 21) : spins;
    return ANPD_OK;
}

int32_t anpd_model_profile(anpd_model_t *m, int32_t enable)
{
    if (!m) return fail(ANPD_E_INVAL, "anpd_model_profile: NULL handle");
    m->prof = enable != 0;
    m->prof_steps = 0;
    for (int i = 0; i < ANPD_PROF_NCAT; ++i) { m->prof_ms[i] = 0.0; m->prof_launches[i] = 0; }
    return ANPD_OK;
}

int32_t anpd_model_profile_read(const anpd_model_t *m, double *out_ms, int64_t *out_launches, int64_t *out_steps)
{
    if (!m || !out_ms || !out_launches || !out_steps) return fail(ANPD_E_INVAL, "anpd_model_profile_read: NULL argument");
    for (int i = 0; i < ANPD_PROF_NCAT; ++i) { out_ms[i] = m->prof_ms[i]; out_launches[i] = m->prof_launches[i]; }
    *out_steps = m->prof_steps;
    return ANPD_OK;
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
    if (e == hipSuccess) e = hipMemset(kv->pool, 0, need);  // unwritten slots must read as zeros, never as NaN patterns
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
                       layer, c.n_layers, kv_heads_of(c), c.head_dim, c.page_tokens)
    if (kv->m->mfma) {
        if (to_cache)
            hipLaunchKernelGGL((kvf_copy_kernel<true>), dim3(n), dim3(256), 0, st, (bf16_t *)kv->pool, kv->d_table, k, v, pos0,
                               layer, c.n_layers, kv_heads_of(c), c.head_dim);
        else
            hipLaunchKernelGGL((kvf_copy_kernel<false>), dim3(n), dim3(256), 0, st, (bf16_t *)kv->pool, kv->d_table, k, v, pos0,
                               layer, c.n_layers, kv_heads_of(c), c.head_dim);
    } else if (c.dtype == ANPD_BF16) { if (to_cache) KV_COPY(bf16_t, true); else KV_COPY(bf16_t, false); }
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
    // The persistent kernel takes the window by value and writes its result and error flag into the
    // pinned buffer itself; the other paths go through copies.
    const bool one_kernel = m->mega && (n_window <= 8 || (n_window <= 16 && m->mega_rows16));
    int32_t *res = m->pin + 32;
    if (one_kernel) {
        rc = run_step_mega(m, kv, window, n_window, mode, out_logits != nullptr, st);
        if (rc != ANPD_OK) return rc;
    } else {
        std::memcpy(m->pin, window, sizeof(int32_t) * (size_t)n_window);
        HIP_TRY(hipMemcpyAsync(m->ws + m->lay.tok, m->pin, sizeof(int32_t) * (size_t)n_window, hipMemcpyHostToDevice, st));
        if (m->mfma) rc = run_step_fast(m, kv, n_window, mode, st);
        else if (m->cfg.dtype == ANPD_BF16) rc = run_step_generic<bf16_t>(m, kv, n_window, mode, st);
        else rc = run_step_generic<float>(m, kv, n_window, mode, st);
        if (rc != ANPD_OK) return rc;
        HIP_TRY(hipMemcpyAsync(res, m->ws + m->lay.result, sizeof(int32_t) * (size_t)(2 + n_window), hipMemcpyDeviceToHost, st));
    }
    if (out_logits)
        HIP_TRY(hipMemcpyAsync(out_logits, m->ws + m->lay.logits, sizeof(float) * (size_t)n_window * m->cfg.vocab,
                               hipMemcpyDeviceToDevice, st));
    HIP_TRY(hipStreamSynchronize(st));
    if (one_kernel && barrier_gave_up(m, st)) return fail(ANPD_E_HIP, "anpd_verify: the persistent kernel timed out at a grid barrier");
    collect_marks(m);
    *out_accepted = res[0];
    *out_next = res[1];
    if (out_predicts) std::memcpy(out_predicts, res + 2, sizeof(int32_t) * (size_t)n_window);
    kv->len += 1 + res[0];
    release_pages(kv, kv->len);
    return ANPD_OK;
}

int32_t anpd_verify_tree(anpd_model_t *m, anpd_kv_t *kv, const int32_t *window, const int32_t *parent, int32_t n_window,
                         int32_t *out_accepted, int32_t *out_next, int32_t *out_path, int32_t *out_predicts, float *out_logits,
                         void *stream)
{
    if (!m || !kv || !window || !parent || !out_accepted || !out_next) return fail(ANPD_E_INVAL, "anpd_verify_tree: NULL argument");
    if (kv->m != m) return fail(ANPD_E_INVAL, "anpd_verify_tree: the cache belongs to another model");
    if (n_window < 1) return fail(ANPD_E_INVAL, "anpd_verify_tree: n_window must be >= 1");
    if (n_window > m->cfg.max_window)
        return fail(ANPD_E_CAPACITY, "anpd_verify_tree: n_window %d exceeds max_window %d", n_window, m->cfg.max_window);
    if (kv->len + n_window > kv->max_tokens)
        return fail(ANPD_E_CAPACITY, "anpd_verify_tree: length %d + window %d exceeds capacity %d", kv->len, n_window, kv->max_tokens);
    if (parent[0] != -1) return fail(ANPD_E_INVAL, "anpd_verify_tree: parent[0] must be -1");
    for (int i = 0; i < n_window; ++i) {
        if (window[i] < 0 || window[i] >= m->cfg.vocab)
            return fail(ANPD_E_RANGE, "anpd_verify_tree: token %d at window[%d] outside [0, %d)", window[i], i, m->cfg.vocab);
        if (i > 0 && (parent[i] < 0 || parent[i] >= i))
            return fail(ANPD_E_INVAL, "anpd_verify_tree: parent[%d] = %d is not an earlier row", i, parent[i]);
    }
    hipStream_t st = (hipStream_t)stream;
    int32_t rc = ensure_pages(kv, kv->len + n_window, st);
    if (rc != ANPD_OK) return rc;
    // depth and visibility (self + ancestors) of every row
    int32_t *tp = m->pin + 128, *td = tp + ANPD_MAX_WINDOW;
    uint32_t *tm = (uint32_t *)(td + ANPD_MAX_WINDOW);
    for (int i = 0; i < ANPD_MAX_WINDOW; ++i) { tp[i] = 0; td[i] = 0; tm[i] = 0; }
    tp[0] = -1;
    tm[0] = 1u;
    for (int i = 1; i < n_window; ++i) {
        tp[i] = parent[i];
        td[i] = td[parent[i]] + 1;
        tm[i] = tm[parent[i]] | (1u << i);
    }
    int32_t *res = m->pin + 32;
    // windows of up to 8 rows: the one-kernel step in its draft-tree form (tokens and tree by value, result
    // written to pinned memory by the kernel); otherwise one launch per operation
    const bool one_kernel = m->mega && m->mega_tree && n_window <= 8;
    if (one_kernel) {
        rc = run_step_mega(m, kv, window, n_window, ANPD_APPEND, out_logits != nullptr, st, tp);
        if (rc != ANPD_OK) return rc;
    } else {
        std::memcpy(m->pin, window, sizeof(int32_t) * (size_t)n_window);
        HIP_TRY(hipMemcpyAsync(m->ws + m->lay.tok, m->pin, sizeof(int32_t) * (size_t)n_window, hipMemcpyHostToDevice, st));
        HIP_TRY(hipMemcpyAsync(m->ws + m->lay.tree, tp, sizeof(int32_t) * 3 * ANPD_MAX_WINDOW, hipMemcpyHostToDevice, st));
        if (m->mfma) rc = run_step_fast(m, kv, n_window, ANPD_APPEND, st, true);
        else if (m->cfg.dtype == ANPD_BF16) rc = run_step_generic<bf16_t>(m, kv, n_window, ANPD_APPEND, st, true);
        else rc = run_step_generic<float>(m, kv, n_window, ANPD_APPEND, st, true);
        if (rc != ANPD_OK) return rc;
        HIP_TRY(hipMemcpyAsync(res, m->ws + m->lay.result, sizeof(int32_t) * (size_t)(2 + 2 * ANPD_MAX_WINDOW + 1), hipMemcpyDeviceToHost, st));
    }
    if (out_logits)
        HIP_TRY(hipMemcpyAsync(out_logits, m->ws + m->lay.logits, sizeof(float) * (size_t)n_window * m->cfg.vocab,
                               hipMemcpyDeviceToDevice, st));
    HIP_TRY(hipStreamSynchronize(st));
    if (one_kernel && barrier_gave_up(m, st)) return fail(ANPD_E_HIP, "anpd_verify_tree: the persistent kernel timed out at a grid barrier");
    collect_marks(m);
    *out_accepted = res[0];
    *out_next = res[1];
    if (out_predicts) std::memcpy(out_predicts, res + 2, sizeof(int32_t) * (size_t)n_window);
    if (out_path) std::memcpy(out_path, res + 34, sizeof(int32_t) * (size_t)(res[0] + 1));
    kv->len += 1 + res[0];
    release_pages(kv, kv->len);
    return ANPD_OK;
}

int32_t anpd_verify_batch(anpd_model_t *m, anpd_kv_t *const *kvs, int32_t n_seq, const int32_t *const *windows,
                          const int32_t *n_windows, int32_t mode, int32_t *out_accepted, int32_t *out_next, float *out_logits,
                          void *stream)
{
    if (!m || !kvs || !windows || !n_windows || !out_accepted || !out_next) return fail(ANPD_E_INVAL, "anpd_verify_batch: NULL argument");
    if (mode != ANPD_VERIFY && mode != ANPD_APPEND) return fail(ANPD_E_INVAL, "anpd_verify_batch: unknown mode %d", mode);
    if (n_seq < 1 || n_seq > ANPD_MAX_WINDOW) return fail(ANPD_E_INVAL, "anpd_verify_batch: n_seq must be in 1..%d", ANPD_MAX_WINDOW);
    if (!m->mfma) return fail(ANPD_E_UNIMPLEMENTED, "anpd_verify_batch: needs the matrix-core path (bf16 weights)");
    int total = 0;
    for (int s = 0; s < n_seq; ++s) {
        anpd_kv *kv = kvs[s];
        if (!kv || !windows[s]) return fail(ANPD_E_INVAL, "anpd_verify_batch: NULL cache or window of sequence %d", s);
        if (kv->m != m) return fail(ANPD_E_INVAL, "anpd_verify_batch: cache %d belongs to another model", s);
        for (int t = 0; t < s; ++t)
            if (kvs[t] == kv) return fail(ANPD_E_INVAL, "anpd_verify_batch: sequences %d and %d share a cache", t, s);
        if (n_windows[s] < 1) return fail(ANPD_E_INVAL, "anpd_verify_batch: n_windows[%d] must be >= 1", s);
        if (kv->len + n_windows[s] > kv->max_tokens)
            return fail(ANPD_E_CAPACITY, "anpd_verify_batch: sequence %d: length %d + window %d exceeds capacity %d", s, kv->len,
                        n_windows[s], kv->max_tokens);
        for (int i = 0; i < n_windows[s]; ++i)
            if (windows[s][i] < 0 || windows[s][i] >= m->cfg.vocab)
                return fail(ANPD_E_RANGE, "anpd_verify_batch: token %d at window %d row %d outside [0, %d)", windows[s][i], s, i, m->cfg.vocab);
        total += n_windows[s];
        if (total > m->cfg.max_window)
            return fail(ANPD_E_CAPACITY, "anpd_verify_batch: %d rows in all exceed max_window %d", total, m->cfg.max_window);
    }
    hipStream_t st = (hipStream_t)stream;
    for (int s = 0; s < n_seq; ++s) {
        int32_t rc = ensure_pages(kvs[s], kvs[s]->len + n_windows[s], st);
        if (rc != ANPD_OK) return rc;
    }
    // joint window, sequence of every row, sequences
    int32_t *row_seq = m->pin + 384;
    SeqRef *seqs = (SeqRef *)(m->pin + 512);
    BatchLaunch bl = {n_seq, 0, 0};
    int row = 0;
    for (int s = 0; s < n_seq; ++s) {
        anpd_kv *kv = kvs[s];
        seqs[s].pool = (bf16_t *)kv->pool;
        seqs[s].page_table = kv->d_table;
        seqs[s].len_ptr = kv->d_len;
        seqs[s].row0 = row;
        seqs[s].n_rows = n_windows[s];
        const int splits = n_splits_of(kv->len + n_windows[s]);
        bl.n_blocks += splits;
        if (splits > bl.grid_splits) bl.grid_splits = splits;
        for (int i = 0; i < n_windows[s]; ++i, ++row) {
            m->pin[row] = windows[s][i];
            row_seq[row] = s;
        }
    }
    // At most 8 rows in all (decoding batches, short windows): the persistent kernel takes the sequences by
    // value and writes the results into the pinned buffer itself; otherwise copies and the fused launches.
    const bool one_kernel = m->mega && m->mega_batch && total <= 8;
    int32_t *res = m->pin + 256;
    int32_t rc;
    if (one_kernel) {
        int32_t lens[8];
        for (int s = 0; s < n_seq; ++s) lens[s] = kvs[s]->len;
        MegaBatch mb = {n_seq, seqs, row_seq, lens};
        rc = run_step_mega(m, nullptr, m->pin, total, mode, out_logits != nullptr, st, nullptr, &mb);
        if (rc != ANPD_OK) return rc;
    } else {
        HIP_TRY(hipMemcpyAsync(m->ws + m->lay.tok, m->pin, sizeof(int32_t) * (size_t)total, hipMemcpyHostToDevice, st));
        HIP_TRY(hipMemcpyAsync(m->ws + m->lay.batch, row_seq, sizeof(int32_t) * (size_t)total, hipMemcpyHostToDevice, st));
        HIP_TRY(hipMemcpyAsync(m->ws + m->lay.batch + ANPD_MAX_WINDOW * sizeof(int32_t), seqs, sizeof(SeqRef) * (size_t)n_seq,
                               hipMemcpyHostToDevice, st));
        rc = run_step_fast(m, nullptr, total, mode, st, false, &bl);
        if (rc != ANPD_OK) return rc;
        HIP_TRY(hipMemcpyAsync(res, m->ws + m->lay.result + 67 * sizeof(int32_t), sizeof(int32_t) * 2 * (size_t)n_seq, hipMemcpyDeviceToHost, st));
    }
    if (out_logits)
        HIP_TRY(hipMemcpyAsync(out_logits, m->ws + m->lay.logits, sizeof(float) * (size_t)total * m->cfg.vocab, hipMemcpyDeviceToDevice, st));
    HIP_TRY(hipStreamSynchronize(st));
    if (one_kernel && barrier_gave_up(m, st)) return fail(ANPD_E_HIP, "anpd_verify_batch: the persistent kernel timed out at a grid barrier");
    collect_marks(m);
    for (int s = 0; s < n_seq; ++s) {
        out_accepted[s] = res[2 * s];
        out_next[s] = res[2 * s + 1];
        kvs[s]->len += 1 + res[2 * s];
        release_pages(kvs[s], kvs[s]->len);
    }
    return ANPD_OK;
}

size_t anpd_prefill_workspace_bytes(const anpd_model_t *m, int32_t n_tokens)
{
    if (!m || n_tokens < 1 || n_tokens > m->cfg.max_positions) {
        fail(ANPD_E_INVAL, "anpd_prefill_workspace_bytes: bad argument");
        return 0;
    }
    return m->mfma ? make_prefill_layout(m->cfg, n_tokens).total : 0;
}

int32_t anpd_prefill(anpd_model_t *m, anpd_kv_t *kv, const int32_t *tokens, int32_t n_tokens, int32_t *out_next,
                     float *out_logits, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!m || !kv || !tokens || !out_next) return fail(ANPD_E_INVAL, "anpd_prefill: NULL argument");
    if (kv->m != m) return fail(ANPD_E_INVAL, "anpd_prefill: the cache belongs to another model");
    if (n_tokens < 1) return fail(ANPD_E_INVAL, "anpd_prefill: n_tokens must be >= 1");
    if (kv->len + n_tokens > kv->max_tokens)
        return fail(ANPD_E_CAPACITY, "anpd_prefill: length %d + %d tokens exceeds capacity %d", kv->len, n_tokens, kv->max_tokens);
    for (int i = 0; i < n_tokens; ++i)
        if (tokens[i] < 0 || tokens[i] >= m->cfg.vocab)
            return fail(ANPD_E_RANGE, "anpd_prefill: token %d at tokens[%d] outside [0, %d)", tokens[i], i, m->cfg.vocab);
    hipStream_t st = (hipStream_t)stream;
    const size_t V = (size_t)m->cfg.vocab;

    if (!m->mfma) {
        // dot-product models: the prompt goes through the step in windows of max_window appended rows
        int32_t acc = 0, last_n = 0;
        for (int i = 0; i < n_tokens; i += last_n) {
            last_n = n_tokens - i < m->cfg.max_window ? n_tokens - i : m->cfg.max_window;
            int32_t rc = anpd_verify(m, kv, tokens + i, last_n, ANPD_APPEND, &acc, out_next, nullptr, nullptr, stream);
            if (rc != ANPD_OK) return rc;
        }
        if (out_logits) {
            HIP_TRY(hipMemcpyAsync(out_logits, m->ws + m->lay.logits + (size_t)(last_n - 1) * V * sizeof(float), V * sizeof(float),
                                   hipMemcpyDeviceToDevice, st));
            HIP_TRY(hipStreamSynchronize(st));
        }
        return ANPD_OK;
    }

    if (m->cfg.d_model > 8192) return fail(ANPD_E_UNIMPLEMENTED, "anpd_prefill: d_model above 8192 is not supported in one pass");
    const PrefillLayout PL = make_prefill_layout(m->cfg, n_tokens);
    if (!workspace || ((uintptr_t)workspace & 255) != 0) return fail(ANPD_E_INVAL, "anpd_prefill: workspace must be a 256-byte aligned device buffer");
    if (workspace_bytes < PL.total)
        return fail(ANPD_E_CAPACITY, "anpd_prefill: workspace has %zu bytes, %zu needed", workspace_bytes, PL.total);
    int32_t rc = ensure_pages(kv, kv->len + n_tokens, st);
    if (rc != ANPD_OK) return rc;
    char *pws = (char *)workspace;
    HIP_TRY(hipMemcpyAsync(pws + PL.tok, tokens, sizeof(int32_t) * (size_t)n_tokens, hipMemcpyHostToDevice, st));
    rc = run_prefill_mfma(m, kv, n_tokens, pws, PL, st);
    if (rc != ANPD_OK) return rc;
    int32_t *res = m->pin + 32;
    HIP_TRY(hipMemcpyAsync(res, m->ws + m->lay.result, sizeof(int32_t) * 3, hipMemcpyDeviceToHost, st));
    if (out_logits)
        HIP_TRY(hipMemcpyAsync(out_logits, m->ws + m->lay.logits, V * sizeof(float), hipMemcpyDeviceToDevice, st));
    HIP_TRY(hipStreamSynchronize(st));
    collect_marks(m);
    *out_next = res[1];
    kv->len += n_tokens;
    return ANPD_OK;
}

size_t anpd_linear_workspace_bytes(int32_t M, int32_t K)
{
    if (M < 1 || M > ANPD_MAX_WINDOW || K < 8) return 0;
    return align_up((size_t)((K + 31) / 32) * 4 * 1024);
}

size_t anpd_packed_bytes(int32_t N, int32_t K)
{
    if (N < 16 || N % 16 != 0 || K < 8 || K % 8 != 0) return 0;
    return packed_bytes((size_t)N / 16, K);
}

int32_t anpd_pack_weights(const void *W, int32_t N, int32_t K, void *packed, size_t packed_bytes_given, void *stream)
{
    if (!W || !packed) return fail(ANPD_E_INVAL, "anpd_pack_weights: NULL argument");
    size_t need = anpd_packed_bytes(N, K);
    if (need == 0) return fail(ANPD_E_INVAL, "anpd_pack_weights: need N %% 16 == 0 and K %% 8 == 0");
    if (packed_bytes_given < need) return fail(ANPD_E_CAPACITY, "anpd_pack_weights: buffer has %zu bytes, %zu needed", packed_bytes_given, need);
    return launch_pack(W, nullptr, nullptr, packed, PACK_PLAIN, N / 16, K, 0, 0, 0, (hipStream_t)stream);
}

int32_t anpd_linear(const float *X, const void *W, float *Y, int32_t M, int32_t N, int32_t K, int32_t dtype,
                    int32_t path, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!X || !W || !Y) return fail(ANPD_E_INVAL, "anpd_linear: NULL argument");
    if (M < 1 || M > ANPD_MAX_WINDOW || K < 8 || K % 8 != 0 || N < 16 || N % 16 != 0)
        return fail(ANPD_E_INVAL, "anpd_linear: need 1 <= M <= %d, K %% 8 == 0, N %% 16 == 0", ANPD_MAX_WINDOW);
    if (dtype != ANPD_F32 && dtype != ANPD_BF16) return fail(ANPD_E_INVAL, "anpd_linear: unknown dtype");
    hipStream_t st = (hipStream_t)stream;
    if (path == ANPD_GEMM_DOT) return launch_gemm_dot(X, M, K, W, nullptr, nullptr, N, 0, 0, Y, N, dtype, st);
    if (path != ANPD_GEMM_MFMA && path != ANPD_GEMM_MFMA_STREAM)
        return fail(ANPD_E_INVAL, "anpd_linear: unknown path %d", path);
    if (dtype != ANPD_BF16) return fail(ANPD_E_INVAL, "anpd_linear: the MFMA path needs bf16 weights");
    if (!workspace || workspace_bytes < anpd_linear_workspace_bytes(M, K))
        return fail(ANPD_E_CAPACITY, "anpd_linear: workspace too small");
    int n_cu = 256, dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
        n_cu = prop.multiProcessorCount;
    const int cls = window_class(M);
    HIP_TRY(hipMemsetAsync(workspace, 0, anpd_linear_workspace_bytes(M, K), st));
    hipLaunchKernelGGL(split_packed_kernel, dim3((K / 4 + 255) / 256, M), dim3(256), 0, st, X, (bf16_t *)workspace, M, K, cls);
    FastArgs a;
    std::memset(&a, 0, sizeof(a));
    a.Wp = (const uint4 *)W;
    a.Xp = (const uint4 *)workspace;
    a.nks = (K + 31) / 32;
    a.n_tiles = N / 16;
    a.M = M;
    a.cls = cls;
    a.Y = Y;
    a.ldy = N;
    return launch_fast<EPI_PLAIN>(a, n_cu, path == ANPD_GEMM_MFMA_STREAM, st);
}

}  // extern "C"

// ---- anpd_linear without a workspace argument and without any allocation ---------------------
//
// The split form of X lives in a file-scope device array.  Each device holds its own copy of the
// array at its own address, so the address is looked up once per device (with that device current)
// and kept; host code never uses the array's name for anything but that lookup.
namespace {

constexpr size_t kStaticScratchBytes = (size_t)(ANPD_LINEAR_STATIC_MAX_K / 32) * 4 * 1024;
constexpr int kMaxDevices = 64;

struct StaticScratch {
    void *ptr;
    int n_cu;
};
StaticScratch g_static_scratch[kMaxDevices];   // zero-initialised: ptr == nullptr means "not looked up yet"

}  // namespace

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// Clears `n16` 16-byte words (a kernel rather than a memset node, so that a caller may capture the call).
__global__ __launch_bounds__(256) void fill_zero_kernel(uint4 *p, size_t n16)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n16) p[i] = make_uint4(0, 0, 0, 0);
}

extern "C" int32_t anpd_linear_static(const float *X, const void *W, float *Y, int32_t M, int32_t N, int32_t K, void *stream)
{
    if (!X || !W || !Y) return fail(ANPD_E_INVAL, "anpd_linear_static: NULL argument");
    if (M < 1 || M > ANPD_MAX_WINDOW || K < 8 || K % 8 != 0 || N < 16 || N % 16 != 0)
        return fail(ANPD_E_INVAL, "anpd_linear_static: need 1 <= M <= %d, K %% 8 == 0, N %% 16 == 0", ANPD_MAX_WINDOW);
    if (K > ANPD_LINEAR_STATIC_MAX_K)
        return fail(ANPD_E_CAPACITY, "anpd_linear_static: K = %d exceeds the built-in scratch (K <= %d); use anpd_linear with a workspace",
                    K, ANPD_LINEAR_STATIC_MAX_K);
    const size_t need = anpd_linear_workspace_bytes(M, K);
    if (need == 0 || need > kStaticScratchBytes) return fail(ANPD_E_CAPACITY, "anpd_linear_static: operand does not fit the built-in scratch");
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(ANPD_E_CAPACITY, "anpd_linear_static: device index %d not supported", dev);
    StaticScratch &sc = g_static_scratch[dev];
    if (!sc.ptr) {
        void *p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(ANPD_E_HIP, "anpd_linear_static: the scratch array has no address on device %d", dev);
        int n_cu = 0;
        HIP_TRY(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
        sc.n_cu = n_cu > 0 ? n_cu : 256;
        sc.ptr = p;
    }
    hipStream_t st = (hipStream_t)stream;
    const int cls = window_class(M);
    // the array keeps the previous call's operand: rows and k-steps this call does not write must read as zeros
    const size_t n16 = need / 16;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, st, (uint4 *)sc.ptr, n16);
    hipLaunchKernelGGL(split_packed_kernel, dim3((K / 4 + 255) / 256, M), dim3(256), 0, st, X, (bf16_t *)sc.ptr, M, K, cls);
    FastArgs a;
    std::memset(&a, 0, sizeof(a));
    a.Wp = (const uint4 *)W;
    a.Xp = (const uint4 *)sc.ptr;
    a.nks = (K + 31) / 32;
    a.n_tiles = N / 16;
    a.M = M;
    a.cls = cls;
    a.Y = Y;
    a.ldy = N;
    return launch_fast<EPI_PLAIN>(a, sc.n_cu, false, st);
}
