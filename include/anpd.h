/*
 * anpd.h - C ABI of the MI355X-native verification path of Adaptive N-gram
 * Parallel Decoding (ANPD, arXiv 2404.08698).
 *
 * Two halves:
 *   - a host-side adaptive multi-level N-gram table (the drafter), and
 *   - the device-side verification step: one LLaMA-shaped forward over the
 *     window [last accepted token, draft_1..draft_k] against the sequence's
 *     paged KV cache, greedy argmax per row, longest-matching-prefix
 *     acceptance, KV commit / rollback.
 *
 * Conventions
 *   - Every call returns int32_t: >= 0 on success (a count where documented),
 *     < 0 an ANPD_E_* code.  anpd_last_error() gives a thread-local message.
 *     No exceptions, no abort, nothing printed.
 *   - On error the object's state is unchanged (arguments are validated
 *     before anything is launched), except ANPD_E_HIP after a launch.
 *   - Handles are opaque, library-owned, and not thread-safe.  One sequence
 *     per anpd_kv_t.
 *   - "host" / "device" on a pointer says where the memory lives.  All
 *     buffers are caller-owned; the library never frees or reallocates them.
 *     Device memory (weights, KV page pool, workspace) is allocated by the
 *     caller and passed as raw device pointers; the library itself allocates
 *     only a few hundred bytes of pinned host memory per handle.
 *   - A stream is a hipStream_t passed as void* (NULL = the default stream).
 */
#ifndef ANPD_H
#define ANPD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    ANPD_OK = 0,
    ANPD_E_INVAL = -1,         /* bad argument */
    ANPD_E_RANGE = -2,         /* token id outside [0, vocab) */
    ANPD_E_CAPACITY = -3,      /* KV capacity, window size or workspace exceeded */
    ANPD_E_NOMEM = -4,         /* host allocation failed */
    ANPD_E_HIP = -5,           /* a HIP call failed; see anpd_last_error() */
    ANPD_E_UNIMPLEMENTED = -6
};

enum { ANPD_F32 = 0, ANPD_BF16 = 1 };               /* storage type of weights and of cached K/V */
enum { ANPD_VERIFY = 0, ANPD_APPEND = 1 };          /* anpd_verify modes */
/* GEMM forms.  DOT: wavefront dot products on the caller's row-major weights (any dtype).
 * MFMA: matrix cores on bf16 weights repacked into fragment order.  MFMA_STREAM (anpd_linear
 * only) forces the MFMA form that streams the activation operand instead of holding it in
 * registers; both MFMA forms give bit-identical results.  With MFMA, a window runs as ONE
 * persistent kernel per step when the model allows it: up to 16 rows for d_model <= 4096, up to
 * 8 rows for d_model <= 5120 (draft trees and several sequences: up to 8 rows, d_model <= 4096);
 * MFMA_LAUNCHES (model option) keeps the same arithmetic as one launch per operation. */
enum { ANPD_GEMM_AUTO = 0, ANPD_GEMM_DOT = 1, ANPD_GEMM_MFMA = 2, ANPD_GEMM_MFMA_STREAM = 3,
       ANPD_GEMM_MFMA_LAUNCHES = 4 };

#define ANPD_MAX_WINDOW 32

const char *anpd_last_error(void);

/* ------------------------------------------------------------------------
 * Host side: adaptive multi-level N-gram table.
 *
 * Paper, Section 3.1 "Token Level N-gram Module" (Initialize / Update /
 * Query over token ids) and Section 3.2 "Multi-Level N-gram" (Algorithm 2:
 * one table per level n in [n_min, n_max], queried from n_max downwards, the
 * first level that answers wins).  The Memory is built from the live context
 * only and grows with every committed token.
 *
 * Query semantics: for a context c of n-1 ids, the answer is the follower
 * seen most often after c in the committed ids; among equally frequent
 * followers the one seen most recently; NULL if c was never followed.
 * ---------------------------------------------------------------------- */
typedef struct anpd_ngram anpd_ngram_t;

/* 2 <= n_min <= n_max <= 16, vocab >= 1.  *out receives the handle. */
int32_t anpd_ngram_create(int32_t n_min, int32_t n_max, int32_t vocab, anpd_ngram_t **out);
void anpd_ngram_destroy(anpd_ngram_t *t);
/* Forget everything (new prompt => fresh Memory). */
int32_t anpd_ngram_reset(anpd_ngram_t *t);
/* Append n COMMITTED tokens (host array) to the context and count, at every
 * level, the tuple each of them completes.  Initialize(prompt) is reset +
 * update(prompt).  Drafts are never passed here: Algorithm 1 updates with
 * accepted tokens only.  ANPD_E_RANGE (nothing appended) on a bad id.
 * Returns the new context length. */
int32_t anpd_ngram_update(anpd_ngram_t *t, const int32_t *tokens, int64_t n);
/* Number of committed tokens. */
int64_t anpd_ngram_length(const anpd_ngram_t *t);
/* One multi-level query (Algorithm 2) on an explicit tail (host array of
 * tail_len ids, most recent last).  Returns 1 and sets *out_token, *out_level
 * on a hit, 0 on NULL. */
int32_t anpd_ngram_query(const anpd_ngram_t *t, const int32_t *tail, int32_t tail_len,
                         int32_t *out_token, int32_t *out_level);
/* Drafting loop of Algorithm 1: up to max_k iterative multi-level queries,
 * each on the committed context followed by the tokens drafted so far;
 * stops at the first NULL.  out_tokens: host, max_k ints.  out_levels
 * (nullable): host, max_k ints, the level that answered each draft.
 * Returns the number drafted (0..max_k). */
int32_t anpd_ngram_propose(const anpd_ngram_t *t, int32_t max_k, int32_t *out_tokens,
                           int32_t *out_levels);

/* Drafting for multi-candidate verification (see anpd_verify_tree): up to n_cand candidate
 * continuations of the committed context, as a tree whose root is the last accepted token.
 * Candidate first tokens: the levels are walked from n_max downwards; within a level the followers
 * of the context come most frequent first (most recent first among equally frequent); distinct
 * tokens only, until n_cand are found.  The first one is therefore the ordinary multi-level answer.
 * Each candidate is then continued by the drafting loop of Algorithm 1 to at most max_k tokens.
 * Candidates are written one after the other until max_drafts rows are used up.
 *   out_tokens, out_parents (host, max_drafts ints): draft i is window row i + 1;
 *   out_parents[i] = window row it continues (0 = the root).  out_levels: nullable.
 * Returns the number of drafts written; n_cand = 1 gives exactly anpd_ngram_propose's chain. */
int32_t anpd_ngram_propose_tree(const anpd_ngram_t *t, int32_t max_k, int32_t n_cand, int32_t max_drafts,
                                int32_t *out_tokens, int32_t *out_parents, int32_t *out_levels);

/* ------------------------------------------------------------------------
 * Device side: the verification step.
 *
 * Paper, Section 3.1 "Parallel Decoding", step 2 and Algorithm 1: the LLM
 * scores the window in a single forward that re-uses the cached (k, v) of
 * everything before it; draft j is accepted while it equals the prediction
 * made after window row j-1; the first mismatch discards that draft and
 * everything after it, and the LLM's own prediction at that row becomes the
 * next token.  The decoder layer is the public LLaMA one (RMSNorm, rotary
 * embedding in the half-split pairing, causal softmax attention, SwiGLU).
 * ---------------------------------------------------------------------- */
typedef struct anpd_model anpd_model_t;
typedef struct anpd_kv anpd_kv_t;

typedef struct {
    int32_t n_layers, d_model, n_heads, head_dim, d_ffn, vocab;
    float rms_eps, rope_base;
    int32_t dtype;          /* ANPD_F32 | ANPD_BF16: weights and cached K/V */
    int32_t page_tokens;    /* tokens per KV page (16) */
    int32_t max_window;     /* largest n_window, 1..ANPD_MAX_WINDOW */
    int32_t max_positions;  /* largest KV capacity any anpd_kv_t of this model may have */
    int32_t gemm_path;      /* ANPD_GEMM_*: AUTO = MFMA for bf16, dot products for f32 */
    int32_t n_kv_heads;     /* key / value heads shared by groups of n_heads / n_kv_heads query heads
                               (grouped-query attention, e.g. the ChatGLM model of the paper's Table 1:
                               query head h reads key / value head h / (n_heads / n_kv_heads));
                               0 = n_heads, one per query head.  Must divide n_heads. */
} anpd_model_cfg;

/* All pointers are DEVICE pointers to [out][in] row-major matrices (gains:
 * [d_model]) in cfg.dtype, borrowed for the model's lifetime.  wk and wv have
 * n_kv_heads * head_dim rows.  The per-layer
 * members are HOST arrays of n_layers device pointers (read at create). */
typedef struct {
    const void *embed, *final_norm, *lm_head;   /* [vocab][d], [d], [vocab][d] */
    const void *const *attn_norm, *const *wq, *const *wk, *const *wv, *const *wo;
    const void *const *ffn_norm, *const *w_gate, *const *w_up, *const *w_down;
} anpd_weights;

/* Bytes of device workspace anpd_model_create needs for cfg (0 on bad cfg).  With the MFMA
 * path this includes a repacked copy of every matrix (about the size of the model): after
 * anpd_model_create returns, only `embed` and the norm gains are still read from the
 * caller's tensors. */
size_t anpd_model_workspace_bytes(const anpd_model_cfg *cfg);
/* workspace: DEVICE, 256-byte aligned, >= anpd_model_workspace_bytes(cfg);
 * used for activations and tables for the model's lifetime.  stream: used to
 * initialise the tables; the call returns after that work has finished. */
int32_t anpd_model_create(const anpd_model_cfg *cfg, const anpd_weights *w, void *workspace,
                          size_t workspace_bytes, void *stream, anpd_model_t **out);
void anpd_model_destroy(anpd_model_t *m);

/* Bytes of device pool a cache of max_tokens positions needs (0 on bad args). */
size_t anpd_kv_pool_bytes(const anpd_model_t *m, int32_t max_tokens);
/* pool: DEVICE, 256-byte aligned, >= anpd_kv_pool_bytes(); cleared by this call.
 * Pages hold page_tokens positions of every layer's K and V as blocks
 * [page][layer][k|v][head] of page_tokens x head_dim elements in cfg.dtype; a page
 * table maps logical to physical pages.  Inside a block the DOT path stores
 * [token][dim]; the MFMA path (page_tokens == 16) stores K and V in the order the
 * matrix-core fragments want (use anpd_kv_read / anpd_kv_write to exchange
 * contents).  max_tokens <= cfg.max_positions. */
int32_t anpd_kv_create(const anpd_model_t *m, void *pool, size_t pool_bytes, int32_t max_tokens,
                       anpd_kv_t **out);
void anpd_kv_destroy(anpd_kv_t *kv);
/* Committed positions. */
int32_t anpd_kv_length(const anpd_kv_t *kv);
/* Explicit commit / rollback: 0 <= new_len <= max_tokens.  Growing is allowed
 * (positions written by anpd_kv_write or by a previous window become live).
 * Pages wholly beyond new_len go back to the cache's free list. */
int32_t anpd_kv_truncate(anpd_kv_t *kv, int32_t new_len, void *stream);
/* Order in which free physical pages are handed out: perm is a HOST array
 * holding a permutation of 0..n_pages-1.  Only valid while the cache is empty. */
int32_t anpd_kv_set_page_order(anpd_kv_t *kv, const int32_t *perm, int32_t n_pages);
int32_t anpd_kv_num_pages(const anpd_kv_t *kv);
/* Copy n positions of one layer between the cache and DEVICE float32 arrays
 * k, v of shape [n][n_kv_heads * head_dim] (values are converted to / from cfg.dtype).
 * Writing allocates pages as needed and does not change the length.
 * Synchronous with respect to the host. */
int32_t anpd_kv_write(anpd_kv_t *kv, int32_t layer, int32_t pos0, int32_t n, const float *k,
                      const float *v, void *stream);
int32_t anpd_kv_read(const anpd_kv_t *kv, int32_t layer, int32_t pos0, int32_t n, float *k,
                     float *v, void *stream);

/* One verification step.
 *   window (host, n_window ints): window[0] = last accepted token, not yet in
 *   the cache; window[1..] = drafts.  1 <= n_window <= cfg.max_window.
 *   ANPD_VERIFY: a = longest prefix with window[i+1] == argmax(logits[i]);
 *     rows 0..a are committed (length += 1 + a), the rest rolled back;
 *     *out_accepted = a, *out_next = argmax(logits[a]).
 *   ANPD_APPEND: all rows are committed without comparing (chunked prefill,
 *     teacher forcing); *out_accepted = n_window - 1, *out_next = argmax of
 *     the last row.
 *   out_predicts (nullable, host, n_window ints): argmax of every row.
 *   out_logits (nullable, DEVICE, n_window * vocab floats): all logits.
 *   argmax takes the lowest index among equal maxima.
 * n_window = 1 is plain greedy decoding.  Blocks until the result is on the
 * host (one stream synchronisation per step).
 * Errors: ANPD_E_RANGE (bad token), ANPD_E_CAPACITY (length + n_window >
 * max_tokens or n_window > max_window), ANPD_E_INVAL, ANPD_E_HIP. */
int32_t anpd_verify(anpd_model_t *m, anpd_kv_t *kv, const int32_t *window, int32_t n_window,
                    int32_t mode, int32_t *out_accepted, int32_t *out_next, int32_t *out_predicts,
                    float *out_logits, void *stream);

/* Multi-candidate verification: several candidate drafts scored in ONE forward.
 *
 * Paper, Section 5, "Future Works", item 2 (more than one candidate in the LLM's verification
 * pass); the accept rule is Algorithm 1's, applied along every root-to-leaf path.
 *   window (host): window[0] = last accepted token; window[r], r >= 1, is a draft that continues
 *   window row parent[r] (parent[0] = -1, 0 <= parent[r] < r): the window is a tree.
 *   Row r stands at position length + depth(r) and attends to the cache and to its own ancestors
 *   only, so its logits are what the linear window [root .. r] would give at its last row.
 *   Row r >= 1 is accepted iff its parent is accepted and window[r] == argmax(logits[parent[r]]).
 *   The deepest accepted row wins (lowest index among equally deep): *out_accepted = its depth a,
 *   *out_next = argmax of its logits, out_path (nullable, host, a + 1 ints) = the window rows
 *   root .. winner.  Their K and V end up in cache positions length .. length + a, everything else
 *   is rolled back: length += 1 + a.
 *   out_predicts / out_logits: as in anpd_verify, by window row.
 * A chain (parent[r] = r - 1) gives bit for bit the result of anpd_verify.  Other shapes give every
 * row the same keys in different cache slots: the same sums in another order, equal to rounding.
 * Windows of up to 8 rows run as the one-kernel step (its draft-tree form), larger ones as one launch
 * per operation; a small kernel then moves the winning path's K and V into place.
 * Errors: as anpd_verify; ANPD_E_INVAL for a parent that is not an earlier row. */
int32_t anpd_verify_tree(anpd_model_t *m, anpd_kv_t *kv, const int32_t *window, const int32_t *parent,
                         int32_t n_window, int32_t *out_accepted, int32_t *out_next, int32_t *out_path,
                         int32_t *out_predicts, float *out_logits, void *stream);

/* Several sequences in one step: their windows go through every weight matrix together, so the
 * weights are streamed once for all of them (the step is bound by that stream: measured at the 7B
 * shape, up to 8 rows cost a one-row step, 9 to 16 rows 1.3 and 17 to 32 rows 1.9 times that).  The
 * paper verifies one sequence at a time (Algorithm 1); this is the same step for n_seq independent
 * runs of it.
 *   kvs (host array of n_seq handles): one cache per sequence, all of model m, all different.
 *   windows[s] (host, n_windows[s] ints): window of sequence s as in anpd_verify; the rows of all
 *   windows together must not exceed cfg.max_window.  mode: ANPD_VERIFY or ANPD_APPEND, for all.
 *   out_accepted, out_next (host, n_seq ints): per sequence, as in anpd_verify; every cache's
 *   length advances by 1 + its own accepted count.
 *   out_logits (nullable, DEVICE, total rows * vocab floats): rows in sequence order.
 * A sequence's rows, results and cache contents are bit-identical to verifying it alone with
 * anpd_verify.  Batches of at most 8 rows in all run as the one-kernel step (its several-sequences
 * form), larger ones as one launch per operation.  Matrix-core path only (bf16 weights):
 * ANPD_E_UNIMPLEMENTED otherwise.
 * Errors: as anpd_verify; ANPD_E_INVAL if two sequences share a cache. */
int32_t anpd_verify_batch(anpd_model_t *m, anpd_kv_t *const *kvs, int32_t n_seq, const int32_t *const *windows,
                          const int32_t *n_windows, int32_t mode, int32_t *out_accepted, int32_t *out_next,
                          float *out_logits, void *stream);

/* Prompt processing.
 *
 * Paper, Section 3.1 "Parallel Decoding", step 1, and the opening of Algorithm 1: before any
 * drafting the LLM reads the whole prompt once; that fills the (k, v) cache and yields the first
 * generated token.  Same arithmetic as appending the rows with anpd_verify (same layer, same
 * bf16 storage of K and V, causal attention over everything cached so far), but all n_tokens rows
 * go through each weight matrix together, on the matrix cores, instead of in windows of at most
 * ANPD_MAX_WINDOW rows; the sums are formed in a different order, so results agree with the
 * windowed form to rounding, not bit for bit.
 *   tokens (host, n_tokens ints) are appended at positions length .. length + n_tokens - 1; the
 *   cache need not be empty (a prompt may be fed in pieces) and its length need not be a multiple
 *   of the page size.  All rows are committed: length += n_tokens.
 *   *out_next = argmax of the last row's logits (lowest index among equal maxima).
 *   out_logits (nullable, DEVICE, vocab floats): the last row's logits.
 *   workspace: DEVICE, 256-byte aligned, >= anpd_prefill_workspace_bytes(m, n_tokens) bytes,
 *   used only during the call (about 175 KB per token at the 7B shape).  Models on the
 *   dot-product path (f32 weights) process the prompt in windows of max_window rows and need no
 *   workspace: the size is 0 and workspace may be NULL.
 * Blocks until the result is on the host.
 * Errors: ANPD_E_RANGE (bad token), ANPD_E_CAPACITY (length + n_tokens > max_tokens, or the
 * workspace is too small), ANPD_E_INVAL, ANPD_E_HIP.  Nothing is launched on the first three. */
size_t anpd_prefill_workspace_bytes(const anpd_model_t *m, int32_t n_tokens);
int32_t anpd_prefill(anpd_model_t *m, anpd_kv_t *kv, const int32_t *tokens, int32_t n_tokens,
                     int32_t *out_next, float *out_logits, void *workspace, size_t workspace_bytes,
                     void *stream);

/* Per-kernel timing of anpd_verify and anpd_prefill with events recorded on the launch stream
 * between kernel groups.  While enabled, every step accumulates the elapsed
 * milliseconds and the number of timed intervals per category; enabling or
 * disabling resets the sums.  out_ms, out_launches: host arrays of
 * ANPD_PROF_NCAT entries; *out_steps: steps accumulated. */
enum {
    ANPD_PROF_GEMM_QKV = 0, ANPD_PROF_GEMM_O, ANPD_PROF_GEMM_GATE_UP, ANPD_PROF_GEMM_DOWN,
    ANPD_PROF_GEMM_LM_HEAD, ANPD_PROF_ATTN, ANPD_PROF_OTHER, ANPD_PROF_STEP /* the one-kernel step */,
    ANPD_PROF_NCAT
};
int32_t anpd_model_profile(anpd_model_t *m, int32_t enable);
int32_t anpd_model_profile_read(const anpd_model_t *m, double *out_ms, int64_t *out_launches,
                                int64_t *out_steps);

/* Barrier-level trace of the one-kernel step.  buffer: DEVICE, grid * 1024 int64 (NULL switches the
 * trace off).  While set, block b stores 100 MHz timestamps at buffer[b * 1024 + e]: e = 0 kernel
 * start, then for every phase boundary the moment the block reaches it and the moment its wait
 * ends (1 + 5 * n_layers + 1 pairs; the pair after a QKV phase is a per-head hand-off, not a grid barrier).
 * Returns the grid size (0 if this model does not use the one-kernel step). */
int32_t anpd_model_trace(anpd_model_t *m, void *buffer, size_t bytes);

/* Test hook for the failure path of the one-kernel step.  A block waits at a grid barrier for at
 * most `spins` polls (0 restores the default, a couple of seconds); a wait that gives up raises
 * the error flag, every block stops waiting, all phases still run to their end, and that
 * anpd_verify returns ANPD_E_HIP.  After such an error the cache contents and length are
 * undefined: truncate and recompute.  The next call starts with fresh barrier counters. */
int32_t anpd_model_set_barrier_spin_limit(anpd_model_t *m, int32_t spins);

/* The dominant kernel on its own, for per-kernel parity and bandwidth
 * measurement: Y[M][N] = X[M][K] * W[N][K]^T with fp32 accumulation.
 *   X: DEVICE float32 [M][K]; Y: DEVICE float32 [M][N];
 *   path ANPD_GEMM_DOT: W is DEVICE [N][K] row-major in `dtype`; workspace may be NULL.
 *   path ANPD_GEMM_MFMA / ANPD_GEMM_MFMA_STREAM (bf16 only): W is the DEVICE buffer
 *   written by anpd_pack_weights for the same N and K; workspace: DEVICE,
 *   >= anpd_linear_workspace_bytes(M, K) bytes (holds the split bf16 form of X).
 *   1 <= M <= ANPD_MAX_WINDOW, K % 8 == 0, N % 16 == 0.  Asynchronous on stream. */
size_t anpd_linear_workspace_bytes(int32_t M, int32_t K);
/* Bytes of the repacked form of an [N][K] bf16 matrix (0 on bad N, K). */
size_t anpd_packed_bytes(int32_t N, int32_t K);
/* Repack W (DEVICE, [N][K] row-major bf16) into MFMA-fragment order:
 * packed[tile][k-step][lane][8], lane = 16 * kg + r holding
 * W[16 * tile + r][32 * ks + 8 * kg .. + 8], K padded with zeros to a multiple of 32.
 * Asynchronous on stream. */
int32_t anpd_pack_weights(const void *W, int32_t N, int32_t K, void *packed, size_t packed_bytes,
                          void *stream);
int32_t anpd_linear(const float *X, const void *W, float *Y, int32_t M, int32_t N, int32_t K,
                    int32_t dtype, int32_t path, void *workspace, size_t workspace_bytes,
                    void *stream);

/* anpd_linear for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels and the same bits as
 * anpd_linear on path ANPD_GEMM_MFMA (bf16 weights packed by anpd_pack_weights), but the split form of X
 * is kept in a device array that is part of the library (2 MiB, held by every GPU the library runs on
 * until the process ends) instead of a workspace argument.  The call allocates and frees nothing and
 * calls no allocating routine; the array is cleared by a kernel, not by a memset.
 *   X, Y, W: DEVICE, as in anpd_linear.  1 <= M <= ANPD_MAX_WINDOW, N % 16 == 0, K % 8 == 0,
 *   K <= ANPD_LINEAR_STATIC_MAX_K (ANPD_E_CAPACITY beyond that, nothing is launched).
 * Asynchronous on stream.  All calls on one GPU share that GPU's array: calls that overlap on one GPU
 * (different streams, different threads) race; serialise them. */
#define ANPD_LINEAR_STATIC_MAX_K 16384
int32_t anpd_linear_static(const float *X, const void *W, float *Y, int32_t M, int32_t N, int32_t K,
                           void *stream);

#ifdef __cplusplus
}
#endif
#endif /* ANPD_H */
