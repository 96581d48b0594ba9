// Fused bf16 fast path of the verification step for gfx950.
//
// Weights are repacked once, at model creation, into MFMA-fragment order:
//   Wp[tile][k-step][lane][8 bf16]        (1 KiB per 16-row x 32-k block)
// where lane = 16 * kg + r holds W[row(tile, r)][32 * ks + 8 * kg .. + 8].  A wave
// then loads the A operand of v_mfma_f32_16x16x32_bf16 with one fully
// coalesced 1 KiB read, and the row map lets each fused epilogue find its
// partner element in lane ^ 32:
//   QKV    tile rows 0..7 = dims 8j..8j+7 of a head, rows 8..15 = the same
//          dims + head_dim/2: the two halves of a rotary pair;
//   gate/up  rows 0..7 = gate rows 8t..8t+7, rows 8..15 = the matching up rows.
//
// Activations travel between kernels as a split-bf16 operand in the same
// fragment order, Xp[k-step][frag][lane][8] (see xp_offset), written by the
// producing epilogue.  RMSNorm is folded around the GEMM: the producer stores
// x * gain and per-tile partial sums of x^2; the consumer multiplies its
// accumulators by 1/sqrt(mean(x^2) + eps).
//
// Summation order of every output element: k-steps ks = wave + u * nw in
// increasing u inside a wave (MFMA accumulation), then waves in increasing
// order, then hi + lo.  nw depends on the matrix shape only, so a row's
// result is bit-identical for every window size and window class.
#pragma once
#include "anpd_kernels.h"

namespace anpd {

constexpr int kFastWaves = 8;   // waves per block of every fast-path kernel: part of the numerics
constexpr int kFastThreads = kFastWaves * 64;

// store four consecutive columns k..k+3 (k % 4 == 0) of row m as hi and lo terms
template <bool COH = false>
__device__ __forceinline__ void xp_store4(bf16_t *xp, int cls, int m, int k, f32x4 v)
{
    bf16_t hi[4], lo[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        // v is often a product formed by the caller.  The value is made opaque here so that the subtraction
        // below is never fused with that product: whether the compiler fuses depends on the code around
        // the call, and the same epilogue is instantiated in several kernels whose bits must agree.
        float t = v[i];
        asm volatile("" : "+v"(t));
        hi[i] = f32_to_bf16(t);
        lo[i] = f32_to_bf16(t - bf16_to_f32(hi[i]));
    }
    uint2 ph = make_uint2((uint32_t)hi[0] | ((uint32_t)hi[1] << 16), (uint32_t)hi[2] | ((uint32_t)hi[3] << 16));
    uint2 pl = make_uint2((uint32_t)lo[0] | ((uint32_t)lo[1] << 16), (uint32_t)lo[2] | ((uint32_t)lo[3] << 16));
    stc8<COH>(xp + xp_offset(cls, m, k, 0), ph);
    stc8<COH>(xp + xp_offset(cls, m, k, 1), pl);
}

// ------------------------------------------------------ fast-path KV cache
//
// The fast path keeps K and V in MFMA-fragment order inside each (page, layer,
// k|v, head) block of 16 tokens x head_dim (page_tokens is 16 on this path):
//   K: [dim / 32][lane = 16 * ((dim % 32) / 8) + token][dim % 8]     A operand of 16x16x32 (rows = keys)
//   V: [dim / 16][lane = 16 * (token / 4) + dim % 16][token % 4]     A operand of 16x16x16 (rows = dims)
// so a wave loads a page's K (and V) tile with fully coalesced reads.
__host__ __device__ __forceinline__ size_t kvf_base(int page, int layer, int n_layers, int kv, int head, int n_heads,
                                                    int head_dim)
{
    return ((((size_t)page * n_layers + layer) * 2 + kv) * n_heads + head) * ((size_t)16 * head_dim);
}
__host__ __device__ __forceinline__ size_t kf_elem(int tok, int dim)
{
    return ((size_t)(dim >> 5) * 64 + (size_t)((dim >> 3) & 3) * 16 + tok) * 8 + (dim & 7);
}
__host__ __device__ __forceinline__ size_t vf_elem(int tok, int dim)
{
    return ((size_t)(dim >> 4) * 64 + (size_t)(tok >> 2) * 16 + (dim & 15)) * 4 + (tok & 3);
}

// bf16-element offset of q (row m, head, dim, hi|lo) in the packed query operand
// qp[head][m / 8][dim / 32][lane][8]: groups of 8 window rows in class-8 packing.
__host__ __device__ __forceinline__ size_t qp_offset(int head, int head_dim, int m, int dim, int lo)
{
    const int nksq = head_dim >> 5;
    return ((((size_t)head * 4 + (m >> 3)) * nksq + (dim >> 5)) * 64 + (size_t)((dim >> 3) & 3) * 16 + (m & 7) + 8 * lo) * 8 +
           (dim & 7);
}

// ------------------------------------------------------------------ packing

enum { PACK_PLAIN = 0, PACK_QKV = 1, PACK_GATE_UP = 2 };

// One thread per 16-byte fragment slot of the packed matrix.
// PLAIN:   tile t row r = src0 row 16 t + r.
// QKV:     tiles [0,Tq) from src0 (q), [Tq,Tq+Tkv) from src1 (k), then Tkv from src2 (v), Tq = d / 16,
//          Tkv = kvd / 16 (kvd = key / value heads x head_dim);
//          q/k tile (head h, j): row r < 8 -> dim 8j + r, r >= 8 -> dim head_dim/2 + 8j + r - 8.
// GATE_UP: tile t row r < 8 -> src0 (gate) row 8t + r, r >= 8 -> src1 (up) row 8t + r - 8.
__global__ __launch_bounds__(256) void pack_kernel(const bf16_t *__restrict__ src0, const bf16_t *__restrict__ src1,
                                                    const bf16_t *__restrict__ src2, uint4 *__restrict__ dst, int mode,
                                                    int n_tiles, int K, int nks, int d, int head_dim, int kvd)
{
    size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    size_t total = (size_t)n_tiles * nks * 64;
    if (idx >= total) return;
    int lane = (int)(idx & 63);
    size_t rest = idx >> 6;
    int ks = (int)(rest % nks), tile = (int)(rest / nks);
    int r = lane & 15, kg = lane >> 4;
    const bf16_t *src = src0;
    int row;
    if (mode == PACK_PLAIN) {
        row = tile * 16 + r;
    } else if (mode == PACK_QKV) {
        int Tq = d / 16, Tkv = kvd / 16;
        int which = tile < Tq ? 0 : (tile < Tq + Tkv ? 1 : 2), t = tile - (which == 0 ? 0 : (which == 1 ? Tq : Tq + Tkv));
        src = which == 0 ? src0 : (which == 1 ? src1 : src2);
        if (which < 2) {
            int tph = head_dim / 16, h = t / tph, j = t - h * tph;
            int dim = r < 8 ? 8 * j + r : head_dim / 2 + 8 * j + (r - 8);
            row = h * head_dim + dim;
        } else {
            row = t * 16 + r;
        }
    } else {
        src = r < 8 ? src0 : src1;
        row = tile * 8 + (r & 7);
    }
    int k = ks * 32 + kg * 8;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (k < K) v = *reinterpret_cast<const uint4 *>(src + (size_t)row * K + k);
    dst[idx] = v;
}

// --------------------------------------------------------------- epilogues

enum { EPI_PLAIN = 0, EPI_QKV = 1, EPI_RESIDUAL = 2, EPI_GATE_UP = 3, EPI_LOGITS = 4, EPI_LM_ARGMAX = 5,
       EPI_QKV_TREE = 6 /* QKV of a draft tree: a row's rotary position is length + its depth, not length + its index */,
       EPI_QKV_BATCH = 7 /* QKV of several sequences' windows side by side: cache, page table and length per row */ };
__host__ __device__ constexpr bool epi_is_qkv(int epi) { return epi == EPI_QKV || epi == EPI_QKV_TREE || epi == EPI_QKV_BATCH; }
__host__ __device__ constexpr bool epi_has_norm(int epi) { return epi_is_qkv(epi) || epi == EPI_GATE_UP || epi == EPI_LOGITS; }

// One sequence of a batched step: its cache and the window rows it owns (consecutive rows of the joint window).
struct SeqRef {
    bf16_t *pool;
    const int32_t *page_table;
    int32_t *len_ptr;
    int32_t row0, n_rows;
};

struct FastArgs {
    // GEMM proper
    const uint4 *Wp;      // packed weights
    const uint4 *Xp;      // packed split operand
    int nks, n_tiles, M, cls;
    // RMSNorm folded around the GEMM (QKV, GATE_UP, LOGITS): partial sums of squares of the input rows
    const float *ssp;     // [n_ss][32]
    int n_ss;
    float inv_d, eps;
    // outputs
    float *Y;             // PLAIN / LOGITS: fp32 [M][ldy]
    int ldy;
    // QKV
    bf16_t *qp;           // packed split query operand (see qp_offset)
    bf16_t *pool;
    const int32_t *page_table, *len_ptr;
    const float2 *rope;
    int layer, n_layers, n_heads, head_dim;
    int n_kv_heads;       // key / value heads (query head h reads head h / (n_heads / n_kv_heads))
    // RESIDUAL
    float *x;             // residual stream fp32 [M][d], updated in place
    const bf16_t *gain;   // gain of the norm that follows
    bf16_t *xp_next;      // operand for the next GEMM: split(x * gain)
    float *ssp_next;      // [n_tiles][32] partial sums of x^2
    int d;
    // GATE_UP
    bf16_t *ap;           // operand of the down projection: split(silu(gate) * up)
    // LM_ARGMAX: Y (nullable) receives the logits; amax the per-tile best (value bits << 32 | index)
    unsigned long long *amax;  // [n_tiles][32]
    // QKV in the persistent kernel: per-head count of finished q / k / v tiles (nullable)
    uint32_t *ready;
    // QKV_TREE: depth of every window row in the draft tree
    const int32_t *depth;
    // QKV_BATCH: the sequences and, for every window row, the index of its sequence
    const SeqRef *seqs;
    const int32_t *row_seq;
};

// rinv[m] = 1 / sqrt(mean(x[m]^2) + eps) for the window rows, from the producer's per-tile partial
// sums.  The order of the additions is the same for every window class: the partials of tiles
// g, g + 64, g + 128, ... are added in increasing order for each of 64 groups g, then the 64 group
// sums in increasing g.  Class 8 gives each thread one (row, group) pair, the other classes four
// groups of one of 32 rows; all of a thread's loads are in flight together.  Ends with a block
// barrier.  scratch: 64 * 32 floats of LDS.
template <bool COH = false>
__device__ __forceinline__ void compute_rinv(const FastArgs &a, float *rinv /* LDS [32] */, float *scratch /* LDS [2048] */)
{
    constexpr int NG = 64, B = 4;
    const int tid = fresh_tid();
    const int rows = a.cls == 8 ? 8 : 32;
    const int slots = kFastThreads / rows;            // 64 or 16 threads per row
    const int m = tid % rows, g0 = tid / rows;
    for (int g = g0; g < NG; g += slots) {
        float s = 0.f;
        if (m < a.M) {
            for (int t0 = g; t0 < a.n_ss; t0 += B * NG) {
                float v[B];
#pragma unroll
                for (int u = 0; u < B; ++u) {
                    const int t = t0 + u * NG;
                    v[u] = ldf_at<COH>(a.ssp, (uint32_t)((t < a.n_ss ? t : t0) * 32 + m));
                }
#pragma unroll
                for (int u = 0; u < B; ++u) s += (t0 + u * NG < a.n_ss) ? v[u] : 0.f;
            }
        }
        scratch[g * 32 + m] = s;
    }
    block_sync_lds();
    if (tid < rows) {
        float tot = 0.f;
#pragma unroll 8
        for (int g = 0; g < NG; ++g) tot += scratch[g * 32 + tid];
        rinv[tid] = 1.0f / sqrtf(fmaf(tot, a.inv_d, a.eps));
    }
    block_sync_lds();
}

// compute_rinv in three steps for windows of 8 NF rows and at most 256 tiles of partial sums, so that the
// persistent kernel can request the sums when a phase starts and reduce them when the first
// epilogue needs them, after the first tile's MFMAs.  Same additions in the same order.
// A thread takes row tid % (8 NF) of group tid / (8 NF) and of the NF - 1 groups a pass further on.
template <bool COH, int NF = 1>
__device__ __forceinline__ void rinv_issue(const FastArgs &a, float (&v)[NF][4], int tid)
{
    constexpr int R = 8 * NF, GP = kFastThreads / R;
    const int m = tid % R, g0 = tid / R;
#pragma unroll
    for (int p = 0; p < NF; ++p)
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int t = g0 + p * GP + 64 * u;
            v[p][u] = (m < a.M && t < a.n_ss) ? ldf_at<COH>(a.ssp, (uint32_t)(t * 32 + m)) : 0.f;
        }
}
template <int NF = 1>
__device__ __forceinline__ void rinv_partial_to_lds(const float (&v)[NF][4], float *scratch /* LDS [2048] */, int tid)
{
    constexpr int R = 8 * NF, GP = kFastThreads / R;
#pragma unroll
    for (int p = 0; p < NF; ++p) {
        float s = 0.f;
#pragma unroll
        for (int u = 0; u < 4; ++u) s += v[p][u];
        scratch[(tid / R + p * GP) * 32 + tid % R] = s;
    }
}
template <int NF = 1>
__device__ __forceinline__ void rinv_from_lds(const FastArgs &a, float *rinv, const float *scratch, int tid)
{
    if (tid < 8 * NF) {
        float tot = 0.f;
#pragma unroll 8
        for (int g = 0; g < 64; ++g) tot += scratch[g * 32 + tid];
        rinv[tid] = 1.0f / sqrtf(fmaf(tot, a.inv_d, a.eps));
    }
}

// Operands an epilogue reads from memory.  The persistent kernel requests them when the tile starts:
// a wave's loads return in order, so a load issued at the epilogue would wait for the weight chunks
// requested before it, and the gain vector is a first touch that comes from HBM.
struct EpiPre {
    f32x4 x, g;       // RESIDUAL: residual row piece and gain
    float2 cs[4];     // QKV: cos / sin of the four rotary pairs
    int page;         // QKV: physical page of the row's position
};

// frag: which 8 rows of the window (rows 8 frag .. 8 frag + 7 sit in lanes with lane % 16 < 8)
template <int EPI>
__device__ __forceinline__ void epilogue_preload(const FastArgs &a, int tile, int lane, EpiPre &pre, int frag = 0)
{
    const int m = 8 * frag + (lane & 7), kg = lane >> 4;
    const bool valid = (lane & 15) < 8 && m < a.M;
    if (EPI == EPI_RESIDUAL) {
        const int n = tile * 16 + 4 * kg;
        pre.x = (f32x4){0.f, 0.f, 0.f, 0.f};
        pre.g = pre.x;
        if (valid) {
            pre.x = *reinterpret_cast<const f32x4 *>(a.x + (size_t)m * a.d + n);
            uint2 gb = *reinterpret_cast<const uint2 *>(a.gain + n);
            pre.g = (f32x4){__uint_as_float(gb.x << 16), __uint_as_float(gb.x & 0xffff0000u), __uint_as_float(gb.y << 16),
                            __uint_as_float(gb.y & 0xffff0000u)};
        }
    } else if (epi_is_qkv(EPI)) {
        const int Tq = a.n_heads * a.head_dim / 16, Tkv = a.n_kv_heads * a.head_dim / 16;
        const int which = tile < Tq ? 0 : (tile < Tq + Tkv ? 1 : 2), t = tile - (which == 0 ? 0 : (which == 1 ? Tq : Tq + Tkv));
        int pos = 0;
        pre.page = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) pre.cs[i] = make_float2(1.f, 0.f);
        if (valid) {
            if (EPI == EPI_QKV_BATCH) {
                const SeqRef sq = a.seqs[a.row_seq[m]];
                pos = *sq.len_ptr + (m - sq.row0);
                pre.page = sq.page_table[pos >> 4];
            } else {
                pos = *a.len_ptr + m;
                pre.page = a.page_table[pos >> 4];
            }
            if (which < 2) {
                const int tph = a.head_dim / 16, half = a.head_dim / 2;
                const int j = t % tph;
                const int i0 = 8 * j + 4 * (kg & 1);
                const int rpos = EPI == EPI_QKV_TREE ? *a.len_ptr + a.depth[m] : pos;
#pragma unroll
                for (int i = 0; i < 4; ++i) pre.cs[i] = a.rope[(size_t)rpos * half + i0 + i];
            }
        }
    }
}

// y: this lane's four outputs D[4 kg + i][m] of tile `tile` for window row m (valid says whether the row exists).
// Every lane of the wave must call this (the fused forms exchange values with lane ^ 32).
template <int EPI, bool COH = false>
__device__ __forceinline__ void epilogue(const FastArgs &a, int tile, int m, int kg, f32x4 y, bool valid,
                                         const float *rinv, const EpiPre *pre = nullptr)
{
    if (EPI == EPI_PLAIN) {
        if (valid) stc16<COH>(a.Y + (size_t)m * a.ldy + tile * 16 + 4 * kg, y);
    } else if (EPI == EPI_LOGITS) {
        if (valid) stc16<COH>(a.Y + (size_t)m * a.ldy + tile * 16 + 4 * kg, y * rinv[m]);
    } else if (EPI == EPI_LM_ARGMAX) {
        // besides (optionally) storing the logits, keep the best (value, lowest index) of the
        // tile's 16 columns for every row
        f32x4 v = y * (valid ? rinv[m] : 0.f);
        const int n = tile * 16 + 4 * kg;
        if (valid && a.Y) stc16<COH>(a.Y + (size_t)m * a.ldy + n, v);
        float best = v[0];
        int bi = n;
#pragma unroll
        for (int i = 1; i < 4; ++i)
            if (v[i] > best) { best = v[i]; bi = n + i; }
#pragma unroll
        for (int off = 16; off <= 32; off <<= 1) {
            float ov = __shfl_xor(best, off, kWave);
            int oi = __shfl_xor(bi, off, kWave);
            if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
        }
        if (valid && kg == 0)
            st_agent(a.amax + (size_t)tile * 32 + m, ((unsigned long long)__float_as_uint(best) << 32) | (uint32_t)bi);
    } else if (EPI == EPI_RESIDUAL) {
        const int n = tile * 16 + 4 * kg;
        f32x4 v = {0.f, 0.f, 0.f, 0.f};
        if (valid) {
            float *xr = a.x + (size_t)m * a.d + n;
            f32x4 g;
            if (pre) {
                v = pre->x + y;
                g = pre->g;
            } else {
                v = *reinterpret_cast<const f32x4 *>(xr) + y;
                uint2 gb = *reinterpret_cast<const uint2 *>(a.gain + n);
                g = (f32x4){__uint_as_float(gb.x << 16), __uint_as_float(gb.x & 0xffff0000u), __uint_as_float(gb.y << 16),
                            __uint_as_float(gb.y & 0xffff0000u)};
            }
            *reinterpret_cast<f32x4 *>(xr) = v;
            xp_store4<COH>(a.xp_next, a.cls, m, n, v * g);
        }
        float s = fmaf(v[3], v[3], fmaf(v[2], v[2], fmaf(v[1], v[1], v[0] * v[0])));
        s += __shfl_xor(s, 16, kWave);
        s += __shfl_xor(s, 32, kWave);
        if (valid && kg == 0) stc<COH>(a.ssp_next + (size_t)tile * 32 + m, s);
    } else if (epi_is_qkv(EPI)) {
        const float r = valid ? rinv[m] : 0.f;
        y = y * r;
        const int Tq = a.n_heads * a.head_dim / 16, Tkv = a.n_kv_heads * a.head_dim / 16;
        const int which = tile < Tq ? 0 : (tile < Tq + Tkv ? 1 : 2), t = tile - (which == 0 ? 0 : (which == 1 ? Tq : Tq + Tkv));
        f32x4 other;
#pragma unroll
        for (int i = 0; i < 4; ++i) other[i] = __shfl_xor(y[i], 32, kWave);
        if (!valid) return;
        int pos, page;          // the row's cache slot and the page it lies in
        bf16_t *pool = a.pool;
        if (EPI == EPI_QKV_BATCH) {
            const SeqRef sq = a.seqs[a.row_seq[m]];
            pos = *sq.len_ptr + (m - sq.row0);
            page = pre ? pre->page : sq.page_table[pos >> 4];
            pool = sq.pool;
        } else {
            pos = *a.len_ptr + m;
            page = pre ? pre->page : a.page_table[pos >> 4];
        }
        const int tok = pos & 15;
        if (which < 2) {
            const int tph = a.head_dim / 16, half = a.head_dim / 2;
            const int h = t / tph, j = t - h * tph;
            const int i0 = 8 * j + 4 * (kg & 1);
            const int rpos = EPI == EPI_QKV_TREE ? *a.len_ptr + a.depth[m] : pos;   // the row's rotary position
            f32x4 o;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float2 cs = pre ? pre->cs[i] : a.rope[(size_t)rpos * half + i0 + i];
                const float cross = other[i] * cs.y;   // (explicit fused form: see xp_store4)
                o[i] = kg < 2 ? fmaf(y[i], cs.x, -cross) : fmaf(y[i], cs.x, cross);
            }
            const int dim = i0 + (kg < 2 ? 0 : half);
            if (which == 0) {
                bf16_t hi[4], lo[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    hi[i] = f32_to_bf16(o[i]);
                    lo[i] = f32_to_bf16(o[i] - bf16_to_f32(hi[i]));
                }
                stc8<COH>(a.qp + qp_offset(h, a.head_dim, m, dim, 0),
                          make_uint2((uint32_t)hi[0] | ((uint32_t)hi[1] << 16), (uint32_t)hi[2] | ((uint32_t)hi[3] << 16)));
                stc8<COH>(a.qp + qp_offset(h, a.head_dim, m, dim, 1),
                          make_uint2((uint32_t)lo[0] | ((uint32_t)lo[1] << 16), (uint32_t)lo[2] | ((uint32_t)lo[3] << 16)));
            } else {
                bf16_t *dst = pool + kvf_base(page, a.layer, a.n_layers, 0, h, a.n_kv_heads, a.head_dim) + kf_elem(tok, dim);
                stc8<COH>(dst, make_uint2((uint32_t)f32_to_bf16(o[0]) | ((uint32_t)f32_to_bf16(o[1]) << 16),
                                          (uint32_t)f32_to_bf16(o[2]) | ((uint32_t)f32_to_bf16(o[3]) << 16)));
            }
        } else {
            const int n = t * 16 + 4 * kg, h = n / a.head_dim, dim = n - h * a.head_dim;
            bf16_t *dst = pool + kvf_base(page, a.layer, a.n_layers, 1, h, a.n_kv_heads, a.head_dim);
#pragma unroll
            for (int i = 0; i < 4; ++i) stc2<COH>(dst + vf_elem(tok, dim + i), f32_to_bf16(y[i]));
        }
    } else if (EPI == EPI_GATE_UP) {
        const float r = valid ? rinv[m] : 0.f;
        y = y * r;
        f32x4 up;
#pragma unroll
        for (int i = 0; i < 4; ++i) up[i] = __shfl_xor(y[i], 32, kWave);
        if (valid && kg < 2) {
            f32x4 act;
#pragma unroll
            for (int i = 0; i < 4; ++i) act[i] = y[i] / (1.0f + expf(-y[i])) * up[i];
            xp_store4<COH>(a.ap, a.cls, m, tile * 8 + 4 * kg, act);
        }
    }
}

// Sum the per-wave partial tiles (wave order), add hi + lo, run the epilogue.  One wave calls this.
template <int NT, int EPI, bool COH = false>
__device__ __forceinline__ void reduce_and_finish(const FastArgs &a, int tile, const float *red /* [nw][NT][256] */,
                                                  int nw, int lane, const float *rinv, const EpiPre *pre = nullptr)
{
    const int slot = lane & 15, kg = lane >> 4;
    f32x4 tot[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        tot[t] = *reinterpret_cast<const f32x4 *>(red + ((size_t)t * 64 + lane) * 4);
        for (int w = 1; w < nw; ++w)
            tot[t] += *reinterpret_cast<const f32x4 *>(red + (((size_t)w * NT + t) * 64 + lane) * 4);
    }
    if (NT == 1) {
        f32x4 lo;
#pragma unroll
        for (int i = 0; i < 4; ++i) lo[i] = row_down8(tot[0][i]);
        epilogue<EPI, COH>(a, tile, slot, kg, tot[0] + lo, slot < 8 && slot < a.M, rinv, pre);
    } else {
#pragma unroll
        for (int p = 0; p < NT / 2; ++p) {
            int m = p * 16 + slot;
            epilogue<EPI, COH>(a, tile, m, kg, tot[2 * p] + tot[2 * p + 1], m < a.M, rinv);
        }
    }
}

// The same for an operand of NF fragments in the class-8 arrangement (packed_class): fragment f holds rows
// 8 f .. 8 f + 7 as (hi | lo) slots, and its partial tiles are finished exactly like the one fragment of a
// window of up to 8 rows.  red: [nw][NF][256].  pre: the staged operands of every fragment, if any.
template <int NF, int EPI, bool COH = false>
__device__ __forceinline__ void reduce_and_finish_packed(const FastArgs &a, int tile, const float *red, int nw, int lane,
                                                         const float *rinv, const EpiPre *pre /* [NF] or null */ = nullptr)
{
    const int slot = lane & 15, kg = lane >> 4;
#pragma unroll
    for (int f = 0; f < NF; ++f) {
        f32x4 tot = *reinterpret_cast<const f32x4 *>(red + ((size_t)f * 64 + lane) * 4);
        for (int w = 1; w < nw; ++w) tot += *reinterpret_cast<const f32x4 *>(red + (((size_t)w * NF + f) * 64 + lane) * 4);
        f32x4 lo;
#pragma unroll
        for (int i = 0; i < 4; ++i) lo[i] = row_down8(tot[i]);
        const int m = 8 * f + (slot & 7);
        epilogue<EPI, COH>(a, tile, m, kg, tot + lo, slot < 8 && m < a.M, rinv, pre ? pre + f : nullptr);
    }
}

// ---------------------------------------------------- GEMM, X-stationary
//
// Window class 8 only.  One block per compute unit; a wave keeps its slice of
// the activation operand (k-steps wave, wave + 8, ...) in registers for the
// whole kernel and streams the weight tiles block, block + grid, ... past it,
// always one half-tile ahead, so the only memory traffic of the main loop is
// the weights.  The partial tiles of the 8 waves meet in LDS (double
// buffered, one barrier per tile); a different wave finishes each tile.
template <int KPW, int EPI>
__global__ __launch_bounds__(kFastThreads) void gemm_xs_kernel(FastArgs a)
{
    __shared__ float red[2][kFastWaves][256];
    __shared__ float rinv[32];
    constexpr int C = (KPW + 1) / 2;  // k-steps per pipeline stage
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nks = a.nks;
    int tile = blockIdx.x;
    uint4 w0[C], w1[KPW - C > 0 ? KPW - C : 1];
    // first stage of the first tile goes out before anything else
    if (tile < a.n_tiles) {
        const uint4 *W = a.Wp + (size_t)tile * nks * 64 + lane;
#pragma unroll
        for (int u = 0; u < C; ++u) {
            int ks = wave + u * kFastWaves;
            w0[u] = ks < nks ? ld_stream(W + (size_t)ks * 64) : make_uint4(0, 0, 0, 0);
        }
    }
    uint4 x[KPW];
#pragma unroll
    for (int u = 0; u < KPW; ++u) {
        int ks = wave + u * kFastWaves;
        x[u] = ks < nks ? a.Xp[(size_t)ks * 64 + lane] : make_uint4(0, 0, 0, 0);
    }
    if (epi_has_norm(EPI)) compute_rinv(a, rinv, &red[1][0][0]);

    for (int it = 0; tile < a.n_tiles; tile += gridDim.x, ++it) {
        const uint4 *W = a.Wp + (size_t)tile * nks * 64 + lane;
        if (KPW > C) {
#pragma unroll
            for (int u = C; u < KPW; ++u) {
                int ks = wave + u * kFastWaves;
                w1[u - C] = ks < nks ? ld_stream(W + (size_t)ks * 64) : make_uint4(0, 0, 0, 0);
            }
        }
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < C; ++u)
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, w0[u]),
                                                          __builtin_bit_cast(bf16x8, x[u]), acc, 0, 0, 0);
        const int next = tile + gridDim.x;
        if (next < a.n_tiles) {
            const uint4 *Wn = a.Wp + (size_t)next * nks * 64 + lane;
#pragma unroll
            for (int u = 0; u < C; ++u) {
                int ks = wave + u * kFastWaves;
                w0[u] = ks < nks ? ld_stream(Wn + (size_t)ks * 64) : make_uint4(0, 0, 0, 0);
            }
        }
        if (KPW > C) {
#pragma unroll
            for (int u = C; u < KPW; ++u)
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, w1[u - C]),
                                                              __builtin_bit_cast(bf16x8, x[u]), acc, 0, 0, 0);
        }
        float *r = &red[it & 1][0][0];
        *reinterpret_cast<f32x4 *>(r + ((size_t)wave * 64 + lane) * 4) = acc;
        block_sync_lds();
        if (wave == (it & (kFastWaves - 1))) reduce_and_finish<1, EPI>(a, tile, r, kFastWaves, lane, rinv);
    }
}

// ------------------------------------------------------ GEMM, streaming X
//
// Any window class and any K: one block per weight tile, the activation
// fragments are read from global memory (L2-resident) next to the weights.
// Same k-step assignment and summation order as the X-stationary form.
template <int NT, int EPI>
__global__ __launch_bounds__(kFastThreads) void gemm_stream_kernel(FastArgs a)
{
    extern __shared__ float red_dyn[];  // [kFastWaves][NT][256]
    __shared__ float rinv[32];
    constexpr int C = NT == 1 ? 4 : (NT == 2 ? 2 : 1);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nks = a.nks, tile = blockIdx.x;
    const uint4 *W = a.Wp + (size_t)tile * nks * 64 + lane;
    const uint4 *X = a.Xp + lane;
    if (epi_has_norm(EPI)) compute_rinv(a, rinv, red_dyn);
    f32x4 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = (f32x4){0.f, 0.f, 0.f, 0.f};
    for (int u0 = 0; wave + u0 * kFastWaves < nks; u0 += C) {
        uint4 wv[C], xv[C][NT];
#pragma unroll
        for (int c = 0; c < C; ++c) {
            int ks = wave + (u0 + c) * kFastWaves;
            bool ok = ks < nks;
            wv[c] = ok ? ld_stream(W + (size_t)ks * 64) : make_uint4(0, 0, 0, 0);
#pragma unroll
            for (int t = 0; t < NT; ++t) xv[c][t] = ok ? X[((size_t)ks * NT + t) * 64] : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int c = 0; c < C; ++c)
#pragma unroll
            for (int t = 0; t < NT; ++t)
                acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wv[c]),
                                                                 __builtin_bit_cast(bf16x8, xv[c][t]), acc[t], 0, 0, 0);
    }
#pragma unroll
    for (int t = 0; t < NT; ++t)
        *reinterpret_cast<f32x4 *>(red_dyn + (((size_t)wave * NT + t) * 64 + lane) * 4) = acc[t];
    __syncthreads();
    if (wave == 0) reduce_and_finish<NT, EPI>(a, tile, red_dyn, kFastWaves, lane, rinv);
}

// ------------------------------------------- GEMM, grouped tiles (windows of 9..32 rows)
//
// A window of more than 8 rows has NT = 2 or 4 activation fragments per
// k-step, too many to keep in registers, and reading them again for every
// weight tile makes the kernel wait for L2 rather than for HBM (NT times the
// weight bytes).  Here a block owns a contiguous range of tiles and takes up
// to TG of them per pass: every activation fragment it loads meets TG weight
// fragments, so the operand traffic is NT / TG of the weight traffic.  Two
// register stages of C k-steps keep the loads of the next stage in flight
// during the MFMAs of this one.  Same k-step assignment (wave, wave + 8, ...)
// and summation order as the other forms: bit-identical results.
template <int NT, int TG, int EPI>
__global__ __launch_bounds__(kFastThreads) void gemm_group_kernel(FastArgs a)
{
    extern __shared__ float red_dyn[];  // [TG][kFastWaves][NT][256]
    __shared__ float rinv[32];
    constexpr int C = (NT * TG >= 8) ? 2 : 4;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nks = a.nks;
    if (epi_has_norm(EPI)) compute_rinv(a, rinv, red_dyn);
    const int first = (int)(((long long)blockIdx.x * a.n_tiles) / gridDim.x);
    const int last = (int)(((long long)(blockIdx.x + 1) * a.n_tiles) / gridDim.x);
    const int n_mine = last - first;
    const int n_pass = (n_mine + TG - 1) / TG;
    const int per_pass = n_pass > 0 ? (n_mine + n_pass - 1) / n_pass : 0;
    const int kpw = (nks + kFastWaves - 1) / kFastWaves;
    const int n_it = (kpw + C - 1) / C;
    __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint4 *>(a.Xp), 0, nks * NT * 1024, 0x00020000);

    for (int t0 = first; t0 < last; t0 += per_pass) {
        const int ntl = last - t0 < per_pass ? last - t0 : per_pass;
        __amdgpu_buffer_rsrc_t rw[TG];
#pragma unroll
        for (int t = 0; t < TG; ++t) {
            const bool have = t < ntl;   // absent tiles: an empty buffer, reads zeros and fetches nothing
            rw[t] = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint4 *>(a.Wp + (size_t)(have ? t0 + t : 0) * nks * 64), 0,
                                                      have ? nks * 1024 : 0, 0x00020000);
        }
        f32x4 acc[TG][NT];
#pragma unroll
        for (int t = 0; t < TG; ++t)
#pragma unroll
            for (int f = 0; f < NT; ++f) acc[t][f] = (f32x4){0.f, 0.f, 0.f, 0.f};
        uint4 wA[TG][C], xA[NT][C], wB[TG][C], xB[NT][C];
        auto load = [&](uint4 (&w)[TG][C], uint4 (&x)[NT][C], int i) {
#pragma unroll
            for (int c = 0; c < C; ++c) {
                const int ks = wave + kFastWaves * (i * C + c);   // past the end: outside every buffer, reads zeros
#pragma unroll
                for (int t = 0; t < TG; ++t) {
                    u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(rw[t], (ks * 64 + lane) * 16, 0, kAuxStream);
                    w[t][c] = make_uint4(v.x, v.y, v.z, v.w);
                }
#pragma unroll
                for (int f = 0; f < NT; ++f) {
                    u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(rx, ((ks * NT + f) * 64 + lane) * 16, 0, 0);
                    x[f][c] = make_uint4(v.x, v.y, v.z, v.w);
                }
            }
        };
        auto mma = [&](const uint4 (&w)[TG][C], const uint4 (&x)[NT][C]) {
#pragma unroll
            for (int c = 0; c < C; ++c)
#pragma unroll
                for (int t = 0; t < TG; ++t)
#pragma unroll
                    for (int f = 0; f < NT; ++f)
                        acc[t][f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, w[t][c]),
                                                                            __builtin_bit_cast(bf16x8, x[f][c]), acc[t][f], 0, 0, 0);
        };
        load(wA, xA, 0);
        for (int i = 0; i < n_it; i += 2) {
            if (i + 1 < n_it) load(wB, xB, i + 1);
            mma(wA, xA);
            if (i + 2 < n_it) load(wA, xA, i + 2);
            if (i + 1 < n_it) mma(wB, xB);
        }
        __syncthreads();   // the previous pass's partial tiles have been consumed
#pragma unroll
        for (int t = 0; t < TG; ++t)
#pragma unroll
            for (int f = 0; f < NT; ++f)
                *reinterpret_cast<f32x4 *>(red_dyn + ((((size_t)t * kFastWaves + wave) * NT + f) * 64 + lane) * 4) = acc[t][f];
        __syncthreads();
        if (wave < ntl)
            reduce_and_finish<NT, EPI>(a, t0 + wave, red_dyn + (size_t)wave * kFastWaves * NT * 256, kFastWaves, lane, rinv);
    }
}

// ------------------------------------------------------------------ embed
//
// x[m] = E[token[m]] plus what the residual epilogue would leave behind for the
// first layer: split(x * attn_gain[0]) and the partial sums of squares.
// grid: d / 16 blocks of one wave.
template <bool COH>
__device__ __forceinline__ void embed_tile(const bf16_t *__restrict__ E, const int32_t *__restrict__ tok, const FastArgs &a,
                                           int tile, int lane)
{
    const int slot = lane & 15, kg = lane >> 4;
    const int n = tile * 16 + 4 * kg;
    for (int p = 0; p < (a.M + 15) / 16; ++p) {
        const int m = p * 16 + slot;
        const bool valid = m < a.M;
        f32x4 v = {0.f, 0.f, 0.f, 0.f};
        if (valid) {
            uint2 eb = *reinterpret_cast<const uint2 *>(E + (size_t)tok[m] * a.d + n);
            v = (f32x4){__uint_as_float(eb.x << 16), __uint_as_float(eb.x & 0xffff0000u), __uint_as_float(eb.y << 16),
                        __uint_as_float(eb.y & 0xffff0000u)};
            *reinterpret_cast<f32x4 *>(a.x + (size_t)m * a.d + n) = v;
            uint2 gb = *reinterpret_cast<const uint2 *>(a.gain + n);
            f32x4 g = {__uint_as_float(gb.x << 16), __uint_as_float(gb.x & 0xffff0000u), __uint_as_float(gb.y << 16),
                       __uint_as_float(gb.y & 0xffff0000u)};
            xp_store4<COH>(a.xp_next, a.cls, m, n, v * g);
        }
        float s = fmaf(v[3], v[3], fmaf(v[2], v[2], fmaf(v[1], v[1], v[0] * v[0])));
        s += __shfl_xor(s, 16, kWave);
        s += __shfl_xor(s, 32, kWave);
        if (valid && kg == 0) stc<COH>(a.ssp_next + (size_t)tile * 32 + m, s);
    }
}

__global__ __launch_bounds__(64) void embed_fast_kernel(const bf16_t *__restrict__ E, const int32_t *__restrict__ tok,
                                                         FastArgs a)
{
    embed_tile<false>(E, tok, a, blockIdx.x, threadIdx.x);
}

// fp32 [M][K] -> packed split operand (stand-alone linear entry point)
__global__ __launch_bounds__(256) void split_packed_kernel(const float *__restrict__ X, bf16_t *__restrict__ xp, int M,
                                                            int K, int cls)
{
    int m = blockIdx.y;
    int k = (blockIdx.x * 256 + threadIdx.x) * 4;
    if (m < M && k < K) xp_store4(xp, cls, m, k, *reinterpret_cast<const f32x4 *>(X + (size_t)m * K + k));
}


typedef short bf16x4s __attribute__((ext_vector_type(4)));

// Window-causal attention on the matrix cores.  The key positions are cut into splits at fixed absolute
// positions: 8 splits of 128 keys, then splits of 384 (split_begin).  A block works on one (head, split);
// wave w takes the 16-token pages w, w + 8, ... of the split (1 or 3 pages), one after the other.  Per group of 8 window rows and per page: S = K q^T with the query as a split-bf16 B operand
// (scores land with keys in registers and rows across lanes), P as a split-bf16 B operand straight from
// those registers, O += V^T P in the matrix cores' accumulators; the wave keeps a running (maximum,
// denominator, output) over its pages and rescales it when a page raises the maximum - no exchange with
// other waves until the wave's pages are done.  Then the waves' maxima meet in LDS, every wave scales its
// result to the block maximum and the tiles are added in a fixed order.  Each block stores (o, max,
// denominator) of its split; the last block of a head to finish merges the head's splits in increasing
// order and writes the packed operand of the output projection.  Short contexts get many small tasks (one
// page per wave, nothing sequential), long ones fewer and larger ones (17 per head at 4096 positions, where
// splits of 128 gave 33): a task costs a chain of round trips - query rows, reduction, stores, counter -
// whatever its size.  The cut depends on absolute key positions only, so a row's sums do not depend on the
// window size, on how a prompt was cut into pieces or on the cache's capacity.
// Scores are kept in the base-2 domain (scaled by log2 e) so that every exponential is one v_exp_f32.
// Row r sees keys 0..len + r; keys it must not see get weight exactly 0.
constexpr int kFastPages = 3;   // most pages per wave per task
constexpr int kSmallSplits = 8;   // splits of one page per wave: the first 1024 positions
__host__ __device__ constexpr int split_begin(int s)
{
    return s <= kSmallSplits ? s * 128 : 128 * kSmallSplits + (s - kSmallSplits) * 128 * kFastPages;
}
__host__ __device__ constexpr int split_pages(int s) { return s < kSmallSplits ? 1 : kFastPages; }   // per wave
__host__ __device__ constexpr int split_of(int key)
{
    return key < 128 * kSmallSplits ? key >> 7 : kSmallSplits + (key - 128 * kSmallSplits) / (128 * kFastPages);
}
// number of splits that hold at least one of the keys 0 .. n_keys - 1
__host__ __device__ constexpr int n_splits_of(int n_keys) { return n_keys <= 0 ? 0 : split_of(n_keys - 1) + 1; }
static_assert(split_begin(8) == 1024 && split_begin(9) == 1408 && split_of(1023) == 7 && split_of(1024) == 8 &&
              split_of(1407) == 8 && split_of(1408) == 9 && split_of(split_begin(12)) == 12 && split_of(split_begin(12) - 1) == 11,
              "cut of the key positions");
// uint32 words between per-head counters: one 256-byte line each.  Atomics of different heads on one
// line serialise at the memory side (measured with polled counters: +16 % step time when packed).
constexpr int kCounterStride = 64;

#ifdef ANPD_TIMING
__device__ long long *g_anpd_dbg = nullptr;
#define ANPD_STAMP(i) do { if (g_anpd_dbg && threadIdx.x == 0) g_anpd_dbg[(blockIdx.y * gridDim.x + blockIdx.x) * 16 + (i)] = wall_clock64(); } while (0)
#else
#define ANPD_STAMP(i) do { } while (0)
#endif

template <int DH>
struct AttnShared {
    float red[kFastWaves / 2][DH / 16][32][4];
    float wmax[kFastWaves][8], wden[kFastWaves][8];
    bool last;
};

struct NoPrefetch {
    __device__ __forceinline__ void operator()() const {}
};

// This wave's page of a (head, split) task: K and V fragments in registers.
template <int DH>
struct AttnKV {
    uint4 kf[DH / 32];
    uint2 vf[DH / 16];
    bool loaded;
};

// Pages 1 and 2 of a task, per wave, parked in LDS by a caller that requested them ahead of the task (the
// persistent kernel does: for a block's first task while the QKV weights stream, for its later tasks while
// the task before is reduced): a wave has registers for two pages at a time.  The pages go from memory straight into LDS, in the order the fragments have in memory, so
// every lane reads back the 16 / 8 bytes a register load would have given it.
struct AttnStash {
    uint4 k[2][kFastWaves][4][64];
    uint2 v[2][kFastWaves][8][64];
};
template <int DH>
__device__ __forceinline__ void stash_get(const AttnStash &st, int slot, AttnKV<DH> &kv, int wave, int lane)
{
#pragma unroll
    for (int i = 0; i < DH / 32; ++i) kv.kf[i] = st.k[slot][wave][i][lane];
#pragma unroll
    for (int i = 0; i < DH / 16; ++i) kv.vf[i] = st.v[slot][wave][i][lane];
    kv.loaded = true;
}

// Requests the wave's K / V page.  With only_old, only a page that lies wholly below position L:
// such a page was written by earlier steps, so the persistent kernel can request it before the
// barrier that ends the QKV phase (the window's own rows are written in that phase).
// `head` is the key / value head, one of n_kv_heads.
// j: which of the wave's pages of the split.
// ids: the page table's entries for the wave's pages, requested earlier (attn_page_ids), or null: a request
// that looks its entry up itself waits for it, and with it for everything the wave requested before.
struct AttnPageIds {
    int e[kFastPages];
};
__device__ __forceinline__ AttnPageIds attn_page_ids(int split, int L, int M, const int32_t *__restrict__ page_table)
{
    const int wave = fresh_tid() >> 6;
    AttnPageIds ids;
#pragma unroll
    for (int j = 0; j < kFastPages; ++j) {
        const int key0 = split_begin(split) + (wave + kFastWaves * j) * 16;
        ids.e[j] = (j < split_pages(split) && key0 < L + M) ? page_table[key0 >> 4] : 0;
    }
    return ids;
}
template <int DH, bool COH>
__device__ __forceinline__ void attn_load_kv(AttnKV<DH> &kv, int head, int split, int L, int M,
                                             const bf16_t *__restrict__ pool, const int32_t *__restrict__ page_table,
                                             int layer, int n_layers, int n_heads, bool only_old, int j = 0,
                                             const AttnPageIds *ids = nullptr)
{
    const int tid = fresh_tid();
    constexpr int NKS = DH / 32, NDT = DH / 16;
    const int lane = tid & 63, wave = tid >> 6;
    const int key0 = split_begin(split) + (wave + kFastWaves * j) * 16;
#pragma unroll
    for (int i = 0; i < NKS; ++i) kv.kf[i] = make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int i = 0; i < NDT; ++i) kv.vf[i] = make_uint2(0, 0);
    kv.loaded = false;
    if (key0 < L + M && (!only_old || key0 + 15 < L)) {
        const int page = __builtin_amdgcn_readfirstlane(ids ? ids->e[j] : page_table[key0 >> 4]);
        const uint4 *kp = reinterpret_cast<const uint4 *>(pool + kvf_base(page, layer, n_layers, 0, head, n_heads, DH));
        const uint2 *vp = reinterpret_cast<const uint2 *>(pool + kvf_base(page, layer, n_layers, 1, head, n_heads, DH));
#pragma unroll
        for (int i = 0; i < NKS; ++i) kv.kf[i] = ld16_at<COH>(kp, (uint32_t)(i * 64 + lane));
#pragma unroll
        for (int i = 0; i < NDT; ++i) kv.vf[i] = ld8_at<COH>(vp, (uint32_t)(i * 64 + lane));
        kv.loaded = true;
    }
}

// The query rows of row group rg of a head: the wave's B operand of the score MFMAs.
template <int DH, bool COH>
__device__ __forceinline__ void attn_load_q(uint4 (&qf)[DH / 32], const uint4 *__restrict__ qp, int head, int rg)
{
    const int lane = fresh_tid() & 63;
    const uint4 *q = qp + ((size_t)(head * 4 + rg) * (DH / 32)) * 64;
#pragma unroll
    for (int ks = 0; ks < DH / 32; ++ks) qf[ks] = ld16_at<COH>(q, (uint32_t)(ks * 64 + lane));
}
// Whether attn_park parks page j of wave `wave` of this split (the same answer wherever it is asked).
__device__ __forceinline__ bool attn_parks(int split, int L, int wave, int j)
{
    return split_begin(split) + (wave + kFastWaves * j) * 16 + 15 < L;
}
// Requests page j of this wave straight into slot `slot` of the stash, if the page lies wholly below
// position L (see attn_load_kv, only_old).  Returns whether it did (the same for the whole wave).
template <int DH>
__device__ __forceinline__ bool attn_park(AttnStash &st, int slot, int head, int split, int L, const bf16_t *__restrict__ pool,
                                          const int32_t *__restrict__ page_table, int layer, int n_layers, int n_heads, int j,
                                          const AttnPageIds *ids = nullptr)
{
    typedef __attribute__((address_space(3))) void *lds_ptr;
    const int tid = fresh_tid();
    const int lane = tid & 63, wave = tid >> 6;
    const int key0 = split_begin(split) + (wave + kFastWaves * j) * 16;
    if (!attn_parks(split, L, wave, j)) return false;
    const int page = __builtin_amdgcn_readfirstlane(ids ? ids->e[j] : page_table[key0 >> 4]);
    __amdgpu_buffer_rsrc_t rk = wave_buffer(pool + kvf_base(page, layer, n_layers, 0, head, n_heads, DH));
    __amdgpu_buffer_rsrc_t rv = wave_buffer(pool + kvf_base(page, layer, n_layers, 1, head, n_heads, DH));
    // K: DH / 32 fragments of 16 bytes per lane; V: DH / 16 fragments of 8 bytes per lane, the same number of bytes
#pragma unroll
    for (int i = 0; i < DH / 32; ++i)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rk, (lds_ptr)&st.k[slot][wave][i][0], 16, lane * 16, i * 1024, 0, kAuxCoherent);
#pragma unroll
    for (int i = 0; i < DH / 32; ++i)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rv, (lds_ptr)&st.v[slot][wave][2 * i][0], 16, lane * 16, i * 1024, 0, kAuxCoherent);
    return true;
}

// Partial results of the splits: outputs [head][split][32 rows][DH], then (maximum, denominator)
// pairs [head][split][32 rows][2].
__device__ __forceinline__ size_t part_o_index(int head, int split, int max_splits, int row, int DH)
{
    return (((size_t)head * max_splits + split) * 32 + row) * DH;
}
__device__ __forceinline__ size_t part_s_index(int n_heads, int head, int split, int max_splits, int row, int DH)
{
    return (size_t)n_heads * max_splits * 32 * DH + (((size_t)head * max_splits + split) * 32 + row) * 2;
}

// One (head, split) task; every thread of the block calls it.  kv holds the wave's first page if
// kv.loaded, else it is requested here; pages 1 and 2 are read from `stash` where stashed1 / stashed2 say so.
// q_lds: 16 * DH bytes of LDS for the copy of the query rows (or null); q_in_lds: the copy is there.
// more_tasks: after_values will request something.  `after_loads` runs right after the task's own loads have
// been issued (the persistent kernel puts its weight prefetch there, so that the prefetch queues
// behind the loads attention is waiting for, not in front of them).
// MODE 1 (tree): the window is a draft tree; row_mask[m] has bit r set if window row r is row m itself
// or one of its ancestors, and row m sees the cached positions plus exactly those rows.
// MODE 2 (batch): the window holds several sequences side by side; this task belongs to the sequence
// whose cache is (pool, page_table, L) and works on its rows [batch->row0, + n_rows) only; the head's
// splits of ALL sequences are merged by the last of batch->n_blocks blocks.
enum { ATTN_CHAIN = 0, ATTN_TREE = 1, ATTN_BATCH = 2 };
struct AttnBatch {
    int row0, n_rows, n_blocks;
    const SeqRef *seqs;
    const int32_t *row_seq;
};
// `publish`: see the merge step below.
// `after_values` runs once the task's last use of its K / V registers is behind it (the persistent kernel
// requests its next task's page there: into the same registers, while this task's partial results are
// reduced, stored and merged).
// MAXP: the most pages per wave that a split of this call can have (1: every key position lies below
// split_begin(kSmallSplits), so the code for further pages - a second set of page registers among it - is left
// out: the separate kernels then fit two blocks on a compute unit instead of one).
template <int DH, bool COH = false, typename AfterLoads = NoPrefetch, int MODE = ATTN_CHAIN, typename AfterValues = NoPrefetch,
          int MAXP = kFastPages>
__device__ __forceinline__ void attn_task(AttnShared<DH> &sh, AttnKV<DH> &kv, int head, int split, int L,
                                          const uint4 *__restrict__ qp, const bf16_t *__restrict__ pool,
                                          const int32_t *__restrict__ page_table, int M, int layer, int n_layers, int n_heads,
                                          int n_kv_heads, int max_splits, float scale, float *__restrict__ part,
                                          uint32_t *__restrict__ head_counter, bf16_t *__restrict__ xp_att, int cls,
                                          AfterLoads after_loads, const uint32_t *__restrict__ row_mask,
                                          const AttnBatch *batch, AfterValues after_values,
                                          int publish, const AttnStash *stash, bool stashed1, bool stashed2,
                                          uint4 *q_lds, bool q_in_lds, bool more_tasks)
{
    constexpr bool TREE = MODE == ATTN_TREE, BATCH = MODE == ATTN_BATCH;
    const int tid = fresh_tid();
    constexpr int NKS = DH / 32, NDT = DH / 16;
    const int lane = tid & 63, wave = tid >> 6, slot = lane & 15, kg = lane >> 4;
    const int row0 = BATCH ? batch->row0 : 0, row_end = BATCH ? batch->row0 + batch->n_rows : M;   // this task's rows
    const int rg0 = row0 >> 3;
    const int kv_head = head / (n_heads / n_kv_heads);
    ANPD_STAMP(0);

    // The wave has registers for two pages: kv (page 0, then page 2) and kvb (page 1).  What is not parked
    // in LDS is requested here; the requests go out before `after_loads`: loads come back in the order they
    // were issued, and what after_loads requests is further away.
    const int n_pages = MAXP == 1 ? 1 : split_pages(split);
    AttnKV<DH> kvb;
    kvb.loaded = false;
    auto request = [&](AttnKV<DH> &dst, int j) __attribute__((always_inline)) {
        attn_load_kv<DH, COH>(dst, kv_head, split, L, row_end - row0, pool, page_table, layer, n_layers, n_kv_heads, false, j);
    };
    if (!kv.loaded) request(kv, 0);
    // The separate kernels (COH = false) go through a split's pages with ONE set of page registers, each page
    // requested when the one before it has been used: a block's own waits get longer, but at 120 instead of 154
    // registers per lane two blocks share a compute unit and fill them.  Same arithmetic, same order.
    constexpr bool kOneSet = !COH;
    if (!kOneSet && n_pages > 1 && !stashed1) request(kvb, 1);
    // the query rows of the first row group: from memory, or from the copy an earlier task of this block left
    // in LDS (same head, same rows) - a block's later tasks then do not wait for memory before their first page
    uint4 qf[NKS];
    if (q_in_lds) {
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) qf[ks] = q_lds[ks * 64 + lane];
    } else {
        attn_load_q<DH, COH>(qf, qp, head, rg0);
    }
    // (a task of several pages waits for loads while it goes through them, and what after_loads requests
    // would be in front of those in the queue: there it is called once the pages are done)
    // (... nor when another task follows: its first requests wait for a table entry, and would wait for
    // everything requested before it)
    const bool loads_late = n_pages > 1 || more_tasks;
    if (!loads_late) after_loads();

    const float scale2 = scale * 1.44269504088896f;   // scores in the base-2 domain
    for (int rg = rg0; rg * 8 < row_end; ++rg) {
        if (rg > rg0) {
            attn_load_q<DH, COH>(qf, qp, head, rg);
            if (kOneSet ? n_pages > 1 : n_pages > 2) request(kv, 0);   // (otherwise every page is still in its registers)
        }
        const int m = rg * 8 + (slot & 7);
        const bool row_ok = slot < 8 && m < M && (!BATCH || (m >= row0 && m < row_end));
        uint32_t vis = 0;
        if (TREE) vis = row_mask[m < M ? m : 0];
        // running maximum and denominator of this wave's pages for row m; the output accumulates in the
        // matrix cores' layout (hi products in slots 0..7, lo products in 8..15, added once at the end)
        float m_run = kMasked, d_run = 0.f;
        f32x4 o_acc[NDT];
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt) o_acc[dt] = (f32x4){0.f, 0.f, 0.f, 0.f};
        // one page: scores, exponentials against the new running maximum, P, O += V^T P
        auto page = [&](const AttnKV<DH> &cur, int j) __attribute__((always_inline)) {
            const int key0 = split_begin(split) + (wave + kFastWaves * j) * 16;
            if (key0 >= L + (row_end - row0)) return;   // (whole wave) nothing of this page exists yet
            // ---- scores S[key][row]
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks)
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, cur.kf[ks]),
                                                              __builtin_bit_cast(bf16x8, qf[ks]), acc, 0, 0, 0);
            float sc[4], mx = kMasked;
            // a page wholly below the committed length is seen by every row (whole-wave branch)
            const bool all_seen = key0 + 15 < L;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float v = (acc[i] + row_down8(acc[i])) * scale2;
                bool ok = row_ok;
                if (!all_seen) {
                    const int key = key0 + 4 * kg + i;
                    const bool sees = TREE    ? (key < L || (key - L < 32 && ((vis >> (key - L)) & 1u)))
                                      : BATCH ? key <= L + (m - row0)
                                              : key <= L + m;
                    ok = ok && sees;
                }
                sc[i] = ok ? v : kMasked;
                mx = fmaxf(mx, sc[i]);
            }
            mx = rows_max(mx);
            // ---- the page's exponentials against the new running maximum
            const float m_new = fmaxf(m_run, mx);
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
            float p[4], den = 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                p[i] = sc[i] > 0.5f * kMasked ? __builtin_amdgcn_exp2f(sc[i] - m_new) : 0.f;
                den += p[i];
            }
            d_run = fmaf(d_run, alpha, den);   // (this lane's four keys of every page; the lanes' sums meet after the pages)
            m_run = m_new;
            // ---- what the wave has so far is rescaled only if some row's maximum went up (whole-wave
            // branch; a factor of exactly 1 changes nothing, so the result does not depend on it)
            if (__builtin_amdgcn_ballot_w64(alpha != 1.f) != 0) {
                const float up = row_up8(alpha);
                const float af = slot < 8 ? alpha : up;
#pragma unroll
                for (int dt = 0; dt < NDT; ++dt) o_acc[dt] = o_acc[dt] * af;
            }
            // ---- P operand (hi rows in slots 0..7, lo rows in 8..15)
            bf16x4s pb;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float up = row_up8(p[i]);
                float pv = slot < 8 ? p[i] : up;
                bf16_t hi = f32_to_bf16(pv);
                bf16_t o = slot < 8 ? hi : f32_to_bf16(pv - bf16_to_f32(hi));
                pb[i] = (short)o;
            }
            // ---- O[dim][row] += V^T P, one 16-dim tile at a time
#pragma unroll
            for (int dt = 0; dt < NDT; ++dt)
                o_acc[dt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(bf16x4s, cur.vf[dt]), pb, o_acc[dt], 0, 0, 0);
        };
        static_assert(kFastPages == 3, "page 2 takes the registers of page 0");
        page(kv, 0);
        if (kOneSet) {
            if (n_pages > 1) { request(kv, 1); page(kv, 1); }
            if (n_pages > 2) { request(kv, 2); page(kv, 2); }
        } else if (n_pages > 1) {
            if (stashed1) stash_get<DH>(*stash, 0, kvb, wave, lane);
            if (n_pages > 2 && !stashed2) request(kv, 2);
            page(kvb, 1);
        }
        if (!kOneSet && n_pages > 2) {
            if (stashed2) stash_get<DH>(*stash, 1, kv, wave, lane);
            page(kv, 2);
        }
        if (!q_in_lds && q_lds && more_tasks && wave == 0 && rg == rg0) {   // (read by later tasks: block barriers lie in between)
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) q_lds[ks * 64 + lane] = qf[ks];
        }
        if ((rg + 1) * 8 >= row_end) after_values();
        if (loads_late && rg == rg0) after_loads();
        ANPD_STAMP(1);
        // ---- the waves' maxima meet; every wave scales its result to the block maximum
        d_run = rows_sum(d_run);
        if (kg == 0 && slot < 8) sh.wmax[wave][slot] = m_run;
        block_sync_lds();
        float bm = sh.wmax[0][slot & 7];
#pragma unroll
        for (int w = 1; w < kFastWaves; ++w) bm = fmaxf(bm, sh.wmax[w][slot & 7]);
        const float wf = __builtin_amdgcn_exp2f(m_run - bm);
        if (kg == 0 && slot < 8) sh.wden[wave][slot] = d_run * wf;
        ANPD_STAMP(7);
        f32x4 ot[NDT];
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt) {
#pragma unroll
            for (int i = 0; i < 4; ++i) ot[dt][i] = (o_acc[dt][i] + row_down8(o_acc[dt][i])) * wf;
        }
        // ---- add the waves' tiles: wave w + H into wave w (H = half the waves), then waves 0..H-1 in
        // order, one or two dim tiles per wave.  LDS is addressed by compacted lane (kg * 8 + slot).
        const int cl = kg * 8 + (slot & 7);
        constexpr int HW = kFastWaves / 2;
        if (wave >= HW && slot < 8) {
#pragma unroll
            for (int dt = 0; dt < NDT; ++dt) *reinterpret_cast<f32x4 *>(&sh.red[wave - HW][dt][cl][0]) = ot[dt];
        }
        block_sync_lds();
        if (wave < HW && slot < 8) {
#pragma unroll
            for (int dt = 0; dt < NDT; ++dt) {
                f32x4 *r = reinterpret_cast<f32x4 *>(&sh.red[wave][dt][cl][0]);
                *r = ot[dt] + *r;
            }
        }
        block_sync_lds();
        ANPD_STAMP(9);
        for (int dt = wave; dt < NDT; dt += kFastWaves) {
            if (slot < 8) {
                const int row = rg * 8 + slot;
                f32x4 tot = *reinterpret_cast<const f32x4 *>(&sh.red[0][dt][cl][0]);
#pragma unroll
                for (int w = 1; w < HW; ++w) tot += *reinterpret_cast<const f32x4 *>(&sh.red[w][dt][cl][0]);
                if (row < M && row >= row0 && row < row_end)
                    stc16<true>(part + part_o_index(head, split, max_splits, row, DH) + 16 * dt + 4 * kg, tot);
            }
        }
        if (tid < 8 && rg * 8 + tid < M && rg * 8 + tid >= row0 && rg * 8 + tid < row_end) {
            const int mm = tid;
            float bmx = sh.wmax[0][mm], dsum = sh.wden[0][mm];
#pragma unroll
            for (int w = 1; w < kFastWaves; ++w) { bmx = fmaxf(bmx, sh.wmax[w][mm]); dsum += sh.wden[w][mm]; }
            stc8<true>(part + part_s_index(n_heads, head, split, max_splits, rg * 8 + mm, DH),
                       make_uint2(__float_as_uint(bmx), __float_as_uint(dsum)));
        }
        ANPD_STAMP(10);
        block_sync_lds();
        ANPD_STAMP(11);
    }

    // ---- the last block of this head merges the splits.  publish = number of finished tasks of this head
    // that this call reports (a block that runs several tasks of one head reports them together with the
    // last one: one wait for the stores and one trip to the counter instead of one per task); 0 = none yet.
    ANPD_STAMP(2);
    if (publish == 0) return;
    wait_stores();
    block_sync_lds();
    ANPD_STAMP(3);
    const int n_blocks = BATCH ? batch->n_blocks : n_splits_of(L + M);
    if (tid == 0)
        sh.last = __hip_atomic_fetch_add(&head_counter[head * kCounterStride], (uint32_t)publish, __ATOMIC_RELAXED,
                                         __HIP_MEMORY_SCOPE_AGENT) + (uint32_t)publish == (uint32_t)n_blocks;
    block_sync_lds();
    ANPD_STAMP(4);
    if (!sh.last) return;
    if (tid == 0) st_agent(&head_counter[head * kCounterStride], 0u);
    // Every thread merges four adjacent output elements of a row on its own: it reads the
    // (maximum, denominator) pair of each split of the row together with the split's outputs,
    // eight splits per round trip, and forms the row's global maximum and denominator itself.
    // Fixed order: splits ascending.
    constexpr int SB = 8, DQ = DH / 4;
    const uint4 *po = reinterpret_cast<const uint4 *>(part + part_o_index(head, 0, max_splits, 0, DH));
    const uint2 *ps = reinterpret_cast<const uint2 *>(part + part_s_index(n_heads, head, 0, max_splits, 0, DH));
    for (int idx = tid; idx < M * DQ; idx += kFastThreads) {
        const int row = idx / DQ, e4 = idx - row * DQ;
        int ns = split_of(L + row) + 1;
        if (BATCH) {   // the row's own sequence decides how many splits it has
            const SeqRef sq = batch->seqs[batch->row_seq[row]];
            ns = split_of(*sq.len_ptr + (row - sq.row0)) + 1;
        }
        float g = kMasked;
        if (ns > SB) {   // long contexts: the maximum needs a pass of its own, SB splits per round trip
            for (int s0 = 0; s0 < ns; s0 += SB) {
                float mv[SB];
#pragma unroll
                for (int j = 0; j < SB; ++j) mv[j] = __uint_as_float(ld8_at<true>(ps, (uint32_t)((s0 + j < ns ? s0 + j : s0) * 32 + row)).x);
#pragma unroll
                for (int j = 0; j < SB; ++j) g = fmaxf(g, mv[j]);
            }
        }
        f32x4 o = {0.f, 0.f, 0.f, 0.f};
        float den = 0.f;
        for (int s0 = 0; s0 < ns; s0 += SB) {
            uint4 ov[SB];
            uint2 st[SB];
#pragma unroll
            for (int j = 0; j < SB; ++j) {
                const int s2 = s0 + j < ns ? s0 + j : s0;
                ov[j] = ld16_at<true>(po, (uint32_t)((s2 * 32 + row) * DQ + e4));
                st[j] = ld8_at<true>(ps, (uint32_t)(s2 * 32 + row));
            }
            if (ns <= SB) {
#pragma unroll
                for (int j = 0; j < SB; ++j)
                    if (j < ns) g = fmaxf(g, __uint_as_float(st[j].x));
            }
#pragma unroll
            for (int j = 0; j < SB; ++j) {
                if (s0 + j < ns) {
                    const float wgt = __builtin_amdgcn_exp2f(__uint_as_float(st[j].x) - g);
                    den = fmaf(wgt, __uint_as_float(st[j].y), den);
                    o[0] = fmaf(wgt, __uint_as_float(ov[j].x), o[0]);
                    o[1] = fmaf(wgt, __uint_as_float(ov[j].y), o[1]);
                    o[2] = fmaf(wgt, __uint_as_float(ov[j].z), o[2]);
                    o[3] = fmaf(wgt, __uint_as_float(ov[j].w), o[3]);
                }
            }
        }
        o[0] /= den; o[1] /= den; o[2] /= den; o[3] /= den;
        xp_store4<COH>(xp_att, cls, row, head * DH + 4 * e4, o);
    }
    ANPD_STAMP(6);
}

// grid: (n_heads, n_splits_of(len + M)), kFastWaves waves.
template <int DH, bool TREE = false, int MAXP = kFastPages>
__global__ __launch_bounds__(kFastThreads) void attn_fast_kernel(const uint4 *__restrict__ qp, const bf16_t *__restrict__ pool,
                                                          const int32_t *__restrict__ page_table,
                                                          const int32_t *__restrict__ len_ptr, int M, int layer, int n_layers,
                                                          int n_heads, int n_kv_heads, int max_splits, float scale,
                                                          float *__restrict__ part, uint32_t *__restrict__ head_counter,
                                                          bf16_t *__restrict__ xp_att, int cls,
                                                          const uint32_t *__restrict__ row_mask)
{
    __shared__ AttnShared<DH> sh;
    const int L = *len_ptr;
    if (split_begin(blockIdx.y) >= L + M) return;
    AttnKV<DH> kv;
    kv.loaded = false;
    attn_task<DH, false, NoPrefetch, TREE ? ATTN_TREE : ATTN_CHAIN, NoPrefetch, MAXP>(sh, kv, blockIdx.x, blockIdx.y, L, qp, pool, page_table, M, layer,
                                                                    n_layers, n_heads, n_kv_heads, max_splits, scale, part,
                                                                    head_counter, xp_att, cls, NoPrefetch(), row_mask, nullptr,
                                                                    NoPrefetch(), 1, nullptr, false, false, nullptr, false, false);
}

// Several sequences' windows in one step: block (head, split, sequence) works on that sequence's rows
// against that sequence's cache.   grid: (n_heads, largest number of splits of any sequence, n_seq).
template <int DH, int MAXP = kFastPages>
__global__ __launch_bounds__(kFastThreads) void attn_batch_kernel(const uint4 *__restrict__ qp, const SeqRef *__restrict__ seqs,
                                                           const int32_t *__restrict__ row_seq, int n_blocks, int M, int layer,
                                                           int n_layers, int n_heads, int n_kv_heads, int max_splits,
                                                           float scale, float *__restrict__ part,
                                                           uint32_t *__restrict__ head_counter, bf16_t *__restrict__ xp_att,
                                                           int cls)
{
    __shared__ AttnShared<DH> sh;
    const SeqRef sq = seqs[blockIdx.z];
    const int L = *sq.len_ptr;
    if (split_begin(blockIdx.y) >= L + sq.n_rows) return;
    AttnKV<DH> kv;
    kv.loaded = false;
    AttnBatch bt = {sq.row0, sq.n_rows, n_blocks, seqs, row_seq};
    attn_task<DH, false, NoPrefetch, ATTN_BATCH, NoPrefetch, MAXP>(sh, kv, blockIdx.x, blockIdx.y, L, qp, sq.pool, sq.page_table, M, layer, n_layers,
                                                 n_heads, n_kv_heads, max_splits, scale, part, head_counter, xp_att, cls,
                                                 NoPrefetch(), nullptr, &bt, NoPrefetch(), 1, nullptr, false, false, nullptr, false, false);
}

// After a draft tree has been verified: the accepted path's rows path[1..a] sit in cache slots
// L + path[j]; move their K and V to slots L + j (path[j] >= j, so in increasing j a source is never
// overwritten before it is read).  result[0] = a; path = result + 34.  grid: n_layers * 2 * n_heads.
__global__ __launch_bounds__(128) void kvf_compact_kernel(bf16_t *__restrict__ pool, const int32_t *__restrict__ page_table,
                                                           const int32_t *__restrict__ result, int L, int n_layers, int n_heads,
                                                           int head_dim)
{
    const int head = blockIdx.x % n_heads, kv = (blockIdx.x / n_heads) & 1, layer = blockIdx.x / (2 * n_heads);
    const int a = result[0];
    const int32_t *path = result + 34;
    for (int j = 1; j <= a; ++j) {
        const int src = L + path[j], dst = L + j;
        if (src != dst && (int)threadIdx.x < head_dim) {
            const int e = threadIdx.x;
            const size_t so = kvf_base(page_table[src >> 4], layer, n_layers, kv, head, n_heads, head_dim) +
                              (kv == 0 ? kf_elem(src & 15, e) : vf_elem(src & 15, e));
            const size_t dofs = kvf_base(page_table[dst >> 4], layer, n_layers, kv, head, n_heads, head_dim) +
                                (kv == 0 ? kf_elem(dst & 15, e) : vf_elem(dst & 15, e));
            pool[dofs] = pool[so];
        }
        __syncthreads();
    }
}

// Acceptance for several sequences verified in one step, after argmax_accept_kernel has left the
// per-row predictions in result[2..]: Algorithm 1's rule inside every sequence's own rows.  Sequence s
// gets result[67 + 2 s] = accepted, result[68 + 2 s] = next, and its length advances by 1 + accepted.
// One thread.
__global__ void accept_batch_kernel(const int32_t *__restrict__ window, const SeqRef *__restrict__ seqs, int n_seq, int mode,
                                    int32_t *__restrict__ result)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    const int32_t *pred = result + 2;
    for (int s = 0; s < n_seq; ++s) {
        const int r0 = seqs[s].row0, n = seqs[s].n_rows;
        int a = 0;
        if (mode == 0) {
            while (a < n - 1 && window[r0 + a + 1] == pred[r0 + a]) ++a;
        } else {
            a = n - 1;
        }
        result[67 + 2 * s] = a;
        result[68 + 2 * s] = pred[r0 + a];
        *seqs[s].len_ptr += 1 + a;
    }
}

// Copies n positions of one layer between fp32 [n][d] arrays and the fast-path cache layout.
template <bool TO_CACHE>
__global__ __launch_bounds__(256) void kvf_copy_kernel(bf16_t *__restrict__ pool, const int32_t *__restrict__ page_table,
                                                        float *__restrict__ k, float *__restrict__ v, int pos0, int layer,
                                                        int n_layers, int n_heads, int head_dim)
{
    const int r = blockIdx.x, pos = pos0 + r, d = n_heads * head_dim;
    const int page = page_table[pos >> 4], tok = pos & 15;
    for (int e = threadIdx.x; e < d; e += 256) {
        int hd = e / head_dim, dim = e - hd * head_dim;
        size_t ko = kvf_base(page, layer, n_layers, 0, hd, n_heads, head_dim) + kf_elem(tok, dim);
        size_t vo = kvf_base(page, layer, n_layers, 1, hd, n_heads, head_dim) + vf_elem(tok, dim);
        if (TO_CACHE) {
            pool[ko] = f32_to_bf16(k[(size_t)r * d + e]);
            pool[vo] = f32_to_bf16(v[(size_t)r * d + e]);
        } else {
            k[(size_t)r * d + e] = bf16_to_f32(pool[ko]);
            v[(size_t)r * d + e] = bf16_to_f32(pool[vo]);
        }
    }
}

}  // namespace anpd
