// Host-side adaptive multi-level N-gram table: the drafter of ANPD.
//
// Paper, Section 3.1 "Token Level N-gram Module": Initialize / Update / Query
// over token-id tuples, built from the live context and updated with every
// accepted token.  Section 3.2, Algorithm 2: one module per level n in
// [n_min, n_max]; a query walks from the largest level down and stops at the
// first level that knows the context.
//
// Each level keeps a hash map from the (n-1)-tuple to its followers with their
// counts and latest positions, and caches the current winner so a query is a
// single lookup.  The winner is the most frequent follower; ties go to the
// follower seen most recently.
#include <cstring>
#include <new>
#include <unordered_map>
#include <vector>

#include "anpd_common.h"

namespace anpd {

char *error_buffer()
{
    static thread_local char buf[kErrorBufferBytes] = {0};
    return buf;
}

namespace {

constexpr int kMaxLevel = 16;

struct Context {
    int32_t ids[kMaxLevel - 1];
    int32_t len;
    bool operator==(const Context &o) const
    {
        return len == o.len && std::memcmp(ids, o.ids, sizeof(int32_t) * (size_t)len) == 0;
    }
};

struct ContextHash {
    size_t operator()(const Context &c) const
    {
        uint64_t h = 0x9E3779B97F4A7C15ull ^ (uint64_t)c.len;
        for (int i = 0; i < c.len; ++i) {
            h ^= (uint64_t)(uint32_t)c.ids[i] + 0x9E3779B97F4A7C15ull + (h << 6) + (h >> 2);
            h *= 0xFF51AFD7ED558CCDull;
            h ^= h >> 33;
        }
        return (size_t)h;
    }
};

struct Follower {
    int32_t token;
    int32_t count;
    int64_t latest;
};

struct Followers {
    std::vector<Follower> list;
    int32_t best = -1;  // index into list
};

using Level = std::unordered_map<Context, Followers, ContextHash>;

}  // namespace
}  // namespace anpd

struct anpd_ngram {
    int32_t n_min, n_max, vocab;
    std::vector<int32_t> ids;             // committed context
    std::vector<anpd::Level> levels;      // levels[n - n_min]
};

namespace {

using namespace anpd;

Context make_context(const int32_t *end, int len)
{
    Context c;
    c.len = len;
    std::memcpy(c.ids, end - len, sizeof(int32_t) * (size_t)len);
    return c;
}

// Count `tok` (at position pos) as a follower of the n-1 ids before it.
void bump(Level &level, const Context &ctx, int32_t tok, int64_t pos)
{
    Followers &f = level[ctx];
    int idx = -1;
    for (size_t i = 0; i < f.list.size(); ++i)
        if (f.list[i].token == tok) { idx = (int)i; break; }
    if (idx < 0) {
        f.list.push_back({tok, 0, pos});
        idx = (int)f.list.size() - 1;
    }
    f.list[(size_t)idx].count += 1;
    f.list[(size_t)idx].latest = pos;
    // `tok` now has the latest position of all followers: it wins every tie.
    if (f.best < 0 || f.list[(size_t)idx].count >= f.list[(size_t)f.best].count) f.best = idx;
}

// Algorithm 2 on a tail of tail_len ids ending at `end`.
bool mln_query(const anpd_ngram *t, const int32_t *end, int64_t tail_len, int32_t *tok, int32_t *lvl)
{
    for (int n = t->n_max; n >= t->n_min; --n) {
        if (tail_len < n - 1) continue;
        const Level &level = t->levels[(size_t)(n - t->n_min)];
        auto it = level.find(make_context(end, n - 1));
        if (it != level.end()) {
            *tok = it->second.list[(size_t)it->second.best].token;
            *lvl = n;
            return true;
        }
    }
    return false;
}

}  // namespace

extern "C" {

const char *anpd_last_error(void) { return anpd::error_buffer(); }

int32_t anpd_ngram_create(int32_t n_min, int32_t n_max, int32_t vocab, anpd_ngram_t **out)
{
    if (!out) return fail(ANPD_E_INVAL, "anpd_ngram_create: out is NULL");
    *out = nullptr;
    if (n_min < 2 || n_max < n_min || n_max > kMaxLevel || vocab < 1)
        return fail(ANPD_E_INVAL, "anpd_ngram_create: need 2 <= n_min <= n_max <= %d and vocab >= 1", kMaxLevel);
    anpd_ngram *t = new (std::nothrow) anpd_ngram;
    if (!t) return fail(ANPD_E_NOMEM, "anpd_ngram_create: out of memory");
    t->n_min = n_min;
    t->n_max = n_max;
    t->vocab = vocab;
    t->levels.resize((size_t)(n_max - n_min + 1));
    *out = t;
    return ANPD_OK;
}

void anpd_ngram_destroy(anpd_ngram_t *t) { delete t; }

int32_t anpd_ngram_reset(anpd_ngram_t *t)
{
    if (!t) return fail(ANPD_E_INVAL, "anpd_ngram_reset: NULL handle");
    t->ids.clear();
    for (auto &l : t->levels) l.clear();
    return ANPD_OK;
}

int32_t anpd_ngram_update(anpd_ngram_t *t, const int32_t *tokens, int64_t n)
{
    if (!t || n < 0 || (n > 0 && !tokens)) return fail(ANPD_E_INVAL, "anpd_ngram_update: bad argument");
    for (int64_t i = 0; i < n; ++i)
        if (tokens[i] < 0 || tokens[i] >= t->vocab)
            return fail(ANPD_E_RANGE, "anpd_ngram_update: token %d at index %lld outside [0, %d)", tokens[i],
                        (long long)i, t->vocab);
    if ((int64_t)t->ids.size() + n > INT32_MAX) return fail(ANPD_E_CAPACITY, "anpd_ngram_update: context too long");
    try {
        t->ids.reserve(t->ids.size() + (size_t)n);
        for (int64_t i = 0; i < n; ++i) {
            int64_t pos = (int64_t)t->ids.size();
            t->ids.push_back(tokens[i]);
            const int32_t *end = t->ids.data() + pos;  // the n-1 ids before `pos` end here
            for (int lv = t->n_min; lv <= t->n_max; ++lv) {
                if (pos < lv - 1) break;
                bump(t->levels[(size_t)(lv - t->n_min)], make_context(end, lv - 1), tokens[i], pos);
            }
        }
    } catch (const std::bad_alloc &) {
        return fail(ANPD_E_NOMEM, "anpd_ngram_update: out of memory");
    }
    return (int32_t)t->ids.size();
}

int64_t anpd_ngram_length(const anpd_ngram_t *t) { return t ? (int64_t)t->ids.size() : 0; }

int32_t anpd_ngram_query(const anpd_ngram_t *t, const int32_t *tail, int32_t tail_len, int32_t *out_token,
                         int32_t *out_level)
{
    if (!t || tail_len < 0 || (tail_len > 0 && !tail) || !out_token)
        return fail(ANPD_E_INVAL, "anpd_ngram_query: bad argument");
    int32_t tok = -1, lvl = 0;
    bool hit = mln_query(t, tail + tail_len, tail_len, &tok, &lvl);
    if (hit) *out_token = tok;
    if (out_level) *out_level = hit ? lvl : 0;
    return hit ? 1 : 0;
}

int32_t anpd_ngram_propose(const anpd_ngram_t *t, int32_t max_k, int32_t *out_tokens, int32_t *out_levels)
{
    if (!t || max_k < 0 || (max_k > 0 && !out_tokens)) return fail(ANPD_E_INVAL, "anpd_ngram_propose: bad argument");
    // Sliding tail: the last n_max-1 committed ids followed by the drafts so far.
    std::vector<int32_t> tail;
    size_t keep = (size_t)(t->n_max - 1);
    size_t have = t->ids.size() < keep ? t->ids.size() : keep;
    tail.reserve(have + (size_t)max_k);
    tail.assign(t->ids.end() - (long)have, t->ids.end());
    int32_t k = 0;
    for (; k < max_k; ++k) {
        int32_t tok, lvl;
        if (!mln_query(t, tail.data() + tail.size(), (int64_t)tail.size(), &tok, &lvl)) break;
        out_tokens[k] = tok;
        if (out_levels) out_levels[k] = lvl;
        tail.push_back(tok);
    }
    return k;
}

int32_t anpd_ngram_propose_tree(const anpd_ngram_t *t, int32_t max_k, int32_t n_cand, int32_t max_drafts, int32_t *out_tokens,
                                int32_t *out_parents, int32_t *out_levels)
{
    if (!t || max_k < 0 || n_cand < 1 || max_drafts < 0 || (max_drafts > 0 && max_k > 0 && (!out_tokens || !out_parents)))
        return fail(ANPD_E_INVAL, "anpd_ngram_propose_tree: bad argument");
    if (max_k == 0 || max_drafts == 0) return 0;
    size_t keep = (size_t)(t->n_max - 1);
    size_t have = t->ids.size() < keep ? t->ids.size() : keep;
    std::vector<int32_t> base(t->ids.end() - (long)have, t->ids.end());
    // first tokens of the candidates: walk the levels downwards; inside a level the followers of the
    // context by (count, latest position) descending; distinct tokens only
    struct First { int32_t token, level; };
    std::vector<First> firsts;
    for (int n = t->n_max; n >= t->n_min && (int)firsts.size() < n_cand; --n) {
        if ((int64_t)base.size() < n - 1) continue;
        const Level &level = t->levels[(size_t)(n - t->n_min)];
        auto it = level.find(make_context(base.data() + base.size(), n - 1));
        if (it == level.end()) continue;
        std::vector<Follower> fs = it->second.list;
        for (size_t i = 1; i < fs.size(); ++i) {   // insertion sort: a context has few followers
            Follower f = fs[i];
            size_t j = i;
            while (j > 0 && (fs[j - 1].count < f.count || (fs[j - 1].count == f.count && fs[j - 1].latest < f.latest))) {
                fs[j] = fs[j - 1];
                --j;
            }
            fs[j] = f;
        }
        for (const Follower &f : fs) {
            bool seen = false;
            for (const First &g : firsts) seen = seen || g.token == f.token;
            if (!seen && (int)firsts.size() < n_cand) firsts.push_back({f.token, n});
        }
    }
    int32_t rows = 0;   // drafts written so far; draft i is window row i + 1
    std::vector<int32_t> tail;
    for (const First &f : firsts) {
        if (rows >= max_drafts) break;
        tail = base;
        int32_t parent = 0, tok = f.token, lvl = f.level;
        for (int32_t k = 0; k < max_k && rows < max_drafts; ++k) {
            if (k > 0 && !mln_query(t, tail.data() + tail.size(), (int64_t)tail.size(), &tok, &lvl)) break;
            out_tokens[rows] = tok;
            out_parents[rows] = parent;
            if (out_levels) out_levels[rows] = lvl;
            parent = rows + 1;
            ++rows;
            tail.push_back(tok);
        }
    }
    return rows;
}

}  // extern "C"
