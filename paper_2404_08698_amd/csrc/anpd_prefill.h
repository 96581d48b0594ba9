// Prompt processing for gfx950: the forward over all P prompt rows at once.
//
// Paper, Section 3.1 "Parallel Decoding", step 1, and the first lines of
// Algorithm 1: before any drafting the LLM reads the prompt once, which fills
// the (k, v) cache and yields the first generated token.  With hundreds of
// rows the GEMMs are bound by the matrix cores, not by weight streaming, so
// they get a form of their own: every wave owns a 64-feature x 64-row output
// tile over the whole K, and a weight fragment it loads meets 4 row groups
// (each as hi and lo term) instead of one.
//
// Shared with the verification step: the packed weights (MFMA-fragment order,
// weights as the A operand, activations as the B operand, so the fused
// epilogues find rotary and gate/up partners in lane ^ 32), the split-bf16
// activation operand, and the cache layout.
//
// Rows are indexed by page-aligned position: row m is absolute position
// (L & ~15) + m, where L is the cache length before the call, so a 16-row
// group is exactly one cache page and all 16 tokens of a page are written by
// one wave.  Rows in front of L (first group) or behind L + P (last group) are
// computed on zeros / leftovers and never stored.
//
// Activation operand of a GEMM with K = 32 * nks columns:
//   Xq[row group][k-step][hi|lo][lane = 16 * kg + (m & 15)][8]   bf16,
// lane holding columns 32 ks + 8 kg .. + 8 of row m: the B fragment of
// v_mfma_f32_16x16x32_bf16, loaded with one coalesced 1 KiB read.
#pragma once
#include "anpd_fast.h"

namespace anpd {

constexpr int kPfThreads = 256;       // 4 waves: 2 (features) x 2 (rows)
constexpr int kPfTN = 4, kPfTM = 4;   // wave tile: 4 weight tiles x 4 row groups

struct PrefillArgs {
    const uint4 *Wp;      // packed weights [n_tiles][nks][64]
    const uint4 *Xq;      // activation operand [G][nks][2][64]
    int nks, n_tiles, G;
    int L, P;             // cache length before the call, prompt rows
    // RESIDUAL
    float *x;             // residual stream fp32 [16 G][d], updated in place
    int d;
    // GATE_UP
    bf16_t *out;          // operand of the down projection
    int out_nks;
    // QKV
    bf16_t *qp;           // query operand [head][G][head_dim / 32][2][64][8]
    bf16_t *pool;
    const int32_t *page_table;
    const float2 *rope;
    int layer, n_layers, n_heads, head_dim;
};

__host__ __device__ __forceinline__ size_t xq_offset(int nks, int m, int k, int lo)
{
    return ((((size_t)(m >> 4) * nks + (k >> 5)) * 2 + lo) * 64 + (size_t)((k >> 3) & 3) * 16 + (m & 15)) * 8 + (k & 7);
}

// four consecutive columns k .. k + 3 (k % 4 == 0) of row m, as hi and lo terms
__device__ __forceinline__ void xq_store4(bf16_t *xq, int nks, int m, int k, f32x4 v)
{
    bf16_t hi[4], lo[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        hi[i] = f32_to_bf16(v[i]);
        lo[i] = f32_to_bf16(v[i] - bf16_to_f32(hi[i]));
    }
    *reinterpret_cast<uint2 *>(xq + xq_offset(nks, m, k, 0)) =
        make_uint2((uint32_t)hi[0] | ((uint32_t)hi[1] << 16), (uint32_t)hi[2] | ((uint32_t)hi[3] << 16));
    *reinterpret_cast<uint2 *>(xq + xq_offset(nks, m, k, 1)) =
        make_uint2((uint32_t)lo[0] | ((uint32_t)lo[1] << 16), (uint32_t)lo[2] | ((uint32_t)lo[3] << 16));
}

__device__ __forceinline__ f32x4 widen4(uint2 b)
{
    return (f32x4){__uint_as_float(b.x << 16), __uint_as_float(b.x & 0xffff0000u), __uint_as_float(b.y << 16),
                   __uint_as_float(b.y & 0xffff0000u)};
}

// ------------------------------------------------------------ RMSNorm rows
//
// Row m: h = x * g / sqrt(mean(x^2) + eps), stored as the split operand of the
// GEMM that follows.  EMBED: the row is first fetched from the embedding table
// (x[m] = E[token]).  Rows outside the prompt are stored as zeros.
// grid: 16 G blocks (one per row) of 256 threads.
template <bool EMBED>
__global__ __launch_bounds__(256) void prefill_norm_kernel(const bf16_t *__restrict__ E, const int32_t *__restrict__ tok,
                                                            float *__restrict__ x, const bf16_t *__restrict__ gain,
                                                            bf16_t *__restrict__ xq, int nks, int d, int L, int P, float inv_d,
                                                            float eps)
{
    __shared__ float part[4];
    const int m = blockIdx.x, r = m - (L & 15);
    const bool valid = r >= 0 && r < P;
    float *xr = x + (size_t)m * d;
    float ss = 0.f;
    if (valid) {
        const bf16_t *er = EMBED ? E + (size_t)tok[r] * d : nullptr;
        for (int k = 4 * threadIdx.x; k < d; k += 1024) {
            f32x4 v;
            if (EMBED) {
                v = widen4(*reinterpret_cast<const uint2 *>(er + k));
                *reinterpret_cast<f32x4 *>(xr + k) = v;
            } else {
                v = *reinterpret_cast<const f32x4 *>(xr + k);
            }
            ss = fmaf(v[3], v[3], fmaf(v[2], v[2], fmaf(v[1], v[1], fmaf(v[0], v[0], ss))));
        }
    }
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float rinv = 1.0f / sqrtf((part[0] + part[1] + part[2] + part[3]) * inv_d + eps);
    for (int k = 4 * threadIdx.x; k < d; k += 1024) {
        f32x4 h = {0.f, 0.f, 0.f, 0.f};
        if (valid) h = *reinterpret_cast<const f32x4 *>(xr + k) * rinv * widen4(*reinterpret_cast<const uint2 *>(gain + k));
        xq_store4(xq, nks, m, k, h);
    }
}

// --------------------------------------------------------------- epilogues

__host__ __device__ __forceinline__ size_t qpf_offset(int head, int G, int head_dim, int m, int dim, int lo)
{
    const int nksq = head_dim >> 5;
    return (((((size_t)head * G + (m >> 4)) * nksq + (dim >> 5)) * 2 + lo) * 64 + (size_t)((dim >> 3) & 3) * 16 + (m & 15)) * 8 +
           (dim & 7);
}

// y: this lane's four outputs (features 4 kg .. 4 kg + 3 of weight tile `tile`) for row m.
// Every lane of the wave must call this: the fused forms exchange values with lane ^ 32.
template <int EPI>
__device__ __forceinline__ void prefill_epilogue(const PrefillArgs &a, int tile, int m, int kg, f32x4 y, bool valid)
{
    if (EPI == EPI_RESIDUAL) {
        if (valid) {
            float *xr = a.x + (size_t)m * a.d + tile * 16 + 4 * kg;
            *reinterpret_cast<f32x4 *>(xr) = *reinterpret_cast<const f32x4 *>(xr) + y;
        }
    } else if (EPI == EPI_GATE_UP) {
        f32x4 up;
#pragma unroll
        for (int i = 0; i < 4; ++i) up[i] = __shfl_xor(y[i], 32, kWave);
        if (valid && kg < 2) {
            f32x4 act;
#pragma unroll
            for (int i = 0; i < 4; ++i) act[i] = y[i] / (1.0f + expf(-y[i])) * up[i];
            xq_store4(a.out, a.out_nks, m, tile * 8 + 4 * kg, act);
        }
    } else if (EPI == EPI_QKV) {
        const int T = a.n_heads * a.head_dim / 16;
        const int which = tile / T, t = tile - which * T;
        const int pos = (a.L & ~15) + m;
        f32x4 other;
#pragma unroll
        for (int i = 0; i < 4; ++i) other[i] = __shfl_xor(y[i], 32, kWave);
        if (!valid) return;
        const int page = a.page_table[pos >> 4], tk = pos & 15;
        if (which < 2) {
            const int tph = a.head_dim / 16, half = a.head_dim / 2;
            const int h = t / tph, j = t - h * tph;
            const int i0 = 8 * j + 4 * (kg & 1);
            f32x4 o;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float2 cs = a.rope[(size_t)pos * half + i0 + i];
                o[i] = kg < 2 ? y[i] * cs.x - other[i] * cs.y : y[i] * cs.x + other[i] * cs.y;
            }
            const int dim = i0 + (kg < 2 ? 0 : half);
            if (which == 0) {
                bf16_t hi[4], lo[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    hi[i] = f32_to_bf16(o[i]);
                    lo[i] = f32_to_bf16(o[i] - bf16_to_f32(hi[i]));
                }
                *reinterpret_cast<uint2 *>(a.qp + qpf_offset(h, a.G, a.head_dim, m, dim, 0)) =
                    make_uint2((uint32_t)hi[0] | ((uint32_t)hi[1] << 16), (uint32_t)hi[2] | ((uint32_t)hi[3] << 16));
                *reinterpret_cast<uint2 *>(a.qp + qpf_offset(h, a.G, a.head_dim, m, dim, 1)) =
                    make_uint2((uint32_t)lo[0] | ((uint32_t)lo[1] << 16), (uint32_t)lo[2] | ((uint32_t)lo[3] << 16));
            } else {
                bf16_t *dst = a.pool + kvf_base(page, a.layer, a.n_layers, 0, h, a.n_heads, a.head_dim) + kf_elem(tk, dim);
                *reinterpret_cast<uint2 *>(dst) = make_uint2((uint32_t)f32_to_bf16(o[0]) | ((uint32_t)f32_to_bf16(o[1]) << 16),
                                                             (uint32_t)f32_to_bf16(o[2]) | ((uint32_t)f32_to_bf16(o[3]) << 16));
            }
        } else {
            const int n = t * 16 + 4 * kg, h = n / a.head_dim, dim = n - h * a.head_dim;
            bf16_t *dst = a.pool + kvf_base(page, a.layer, a.n_layers, 1, h, a.n_heads, a.head_dim);
#pragma unroll
            for (int i = 0; i < 4; ++i) dst[vf_elem(tk, dim + i)] = f32_to_bf16(y[i]);
        }
    }
}

// -------------------------------------------------------------------- GEMM
//
// Y^T[features][rows] = W X^T with hi and lo terms of X accumulated into the
// same tile.  Block = 2 x 2 waves, 128 features x 128 rows; consecutive
// blocks share a weight range (rows run fastest).  A wave streams its 4
// weight fragments and 8 activation fragments per k-step straight into
// registers (buffer loads: absent tiles and row groups read zeros and fetch
// nothing), one k-step ahead of the matrix cores; two blocks per compute unit
// cover each other's waits.  Each wave owns its tile over the whole K, so
// there is no cross-wave reduction and every epilogue runs from registers.
// grid: ceil(n_tiles / 8) * ceil(G / 8) blocks.
template <int EPI>
__global__ __launch_bounds__(kPfThreads, 2) void prefill_gemm_kernel(PrefillArgs a)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n_br = (a.G + 2 * kPfTM - 1) / (2 * kPfTM);
    const int bt = blockIdx.x / n_br, br = blockIdx.x - bt * n_br;
    const int f0 = (bt * 2 + (wave & 1)) * kPfTN, g0 = (br * 2 + (wave >> 1)) * kPfTM;
    if (f0 >= a.n_tiles || g0 >= a.G) return;   // (no block-wide synchronisation below)
    const int nks = a.nks;

    __amdgpu_buffer_rsrc_t rw[kPfTN];
#pragma unroll
    for (int t = 0; t < kPfTN; ++t) {
        const bool have = f0 + t < a.n_tiles;
        rw[t] = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint4 *>(a.Wp + (size_t)(have ? f0 + t : 0) * nks * 64), 0,
                                                  have ? nks * 1024 : 0, 0x00020000);
    }
    // the wave's row groups as one buffer: groups beyond G lie outside it
    const int n_g = a.G - g0 < kPfTM ? a.G - g0 : kPfTM;
    __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint4 *>(a.Xq + (size_t)g0 * nks * 128), 0,
                                                                  n_g * nks * 2048, 0x00020000);
    f32x4 acc[kPfTN][kPfTM];
#pragma unroll
    for (int t = 0; t < kPfTN; ++t)
#pragma unroll
        for (int g = 0; g < kPfTM; ++g) acc[t][g] = (f32x4){0.f, 0.f, 0.f, 0.f};

    uint4 wA[kPfTN], xA[kPfTM][2], wB[kPfTN], xB[kPfTM][2];
    auto load = [&](uint4 (&w)[kPfTN], uint4 (&x)[kPfTM][2], int ks) {
#pragma unroll
        for (int t = 0; t < kPfTN; ++t) {
            u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(rw[t], (ks * 64 + lane) * 16, 0, 0);
            w[t] = make_uint4(v.x, v.y, v.z, v.w);
        }
#pragma unroll
        for (int g = 0; g < kPfTM; ++g)
#pragma unroll
            for (int hl = 0; hl < 2; ++hl) {
                u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(rx, (((g * nks + ks) * 2 + hl) * 64 + lane) * 16, 0, 0);
                x[g][hl] = make_uint4(v.x, v.y, v.z, v.w);
            }
    };
    auto mma = [&](const uint4 (&w)[kPfTN], const uint4 (&x)[kPfTM][2]) {
#pragma unroll
        for (int hl = 0; hl < 2; ++hl)
#pragma unroll
            for (int t = 0; t < kPfTN; ++t)
#pragma unroll
                for (int g = 0; g < kPfTM; ++g)
                    acc[t][g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, w[t]),
                                                                        __builtin_bit_cast(bf16x8, x[g][hl]), acc[t][g], 0, 0, 0);
    };
    load(wA, xA, 0);
    for (int ks = 0; ks < nks; ks += 2) {
        if (ks + 1 < nks) load(wB, xB, ks + 1);
        mma(wA, xA);
        if (ks + 2 < nks) load(wA, xA, ks + 2);
        if (ks + 1 < nks) mma(wB, xB);
    }

    const int slot = lane & 15, kg = lane >> 4;
    const int r0 = a.L & 15;
#pragma unroll
    for (int t = 0; t < kPfTN; ++t) {
        if (f0 + t >= a.n_tiles) break;   // wave-uniform
#pragma unroll
        for (int g = 0; g < kPfTM; ++g) {
            const int m = (g0 + g) * 16 + slot;
            const bool valid = g0 + g < a.G && m >= r0 && m < r0 + a.P;
            prefill_epilogue<EPI>(a, f0 + t, m, kg, acc[t][g], valid);
        }
    }
}

// --------------------------------------------------------------- attention
//
// Causal attention of the prompt rows over the cache (which by now holds the
// prompt's own K and V).  One wave per (head, 16-row group); the group is one
// cache page, so every earlier page is visible in full and only the last one
// needs the causal mask.  Per page: S = K q^T (query as hi + lo B operands;
// scores land with keys in registers and rows across lanes), online softmax
// per row, P as hi + lo B operands straight from those registers, O += V^T P.
// The next page's K and V are requested before this page's arithmetic.
// grid: (n_heads, ceil(G / 4)), 4 waves; later groups (more pages) start first.
template <int DH>
__global__ __launch_bounds__(256) void prefill_attn_kernel(const uint4 *__restrict__ qp, const bf16_t *__restrict__ pool,
                                                            const int32_t *__restrict__ page_table, int G, int L, int P,
                                                            int layer, int n_layers, int n_heads, float scale,
                                                            bf16_t *__restrict__ xq_att, int nks_d)
{
    constexpr int NKS = DH / 32, NDT = DH / 16;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, slot = lane & 15, kg = lane >> 4;
    const int head = blockIdx.x;
    const int g = ((int)gridDim.y - 1 - (int)blockIdx.y) * 4 + wave;
    if (g >= G) return;   // (no block-wide synchronisation below)
    const int last_page = (L >> 4) + g;

    uint4 qf[NKS][2];
    {
        const uint4 *q = qp + ((size_t)head * G + g) * NKS * 128;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
            for (int hl = 0; hl < 2; ++hl) qf[ks][hl] = q[(ks * 2 + hl) * 64 + lane];
    }
    uint4 kA[NKS], kB[NKS];
    uint2 vA[NDT], vB[NDT];
    auto load = [&](uint4 (&kf)[NKS], uint2 (&vf)[NDT], int pg) {
        const int page = __builtin_amdgcn_readfirstlane(page_table[pg]);
        const uint4 *kp = reinterpret_cast<const uint4 *>(pool + kvf_base(page, layer, n_layers, 0, head, n_heads, DH));
        const uint2 *vp = reinterpret_cast<const uint2 *>(pool + kvf_base(page, layer, n_layers, 1, head, n_heads, DH));
#pragma unroll
        for (int i = 0; i < NKS; ++i) kf[i] = kp[i * 64 + lane];
#pragma unroll
        for (int i = 0; i < NDT; ++i) vf[i] = vp[i * 64 + lane];
    };
    float mx = kMasked, den = 0.f;
    f32x4 o[NDT];
#pragma unroll
    for (int dt = 0; dt < NDT; ++dt) o[dt] = (f32x4){0.f, 0.f, 0.f, 0.f};
    auto page_step = [&](const uint4 (&kf)[NKS], const uint2 (&vf)[NDT], int pg) {
        f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kf[ks]), __builtin_bit_cast(bf16x8, qf[ks][0]), s, 0, 0, 0);
            s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kf[ks]), __builtin_bit_cast(bf16x8, qf[ks][1]), s, 0, 0, 0);
        }
        float sc[4], pm = kMasked;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const bool ok = pg < last_page || 4 * kg + i <= slot;   // on the row's own page: keys up to the row itself
            sc[i] = ok ? s[i] * scale : kMasked;
            pm = fmaxf(pm, sc[i]);
        }
        pm = fmaxf(pm, __shfl_xor(pm, 16, kWave));
        pm = fmaxf(pm, __shfl_xor(pm, 32, kWave));
        const float mnew = fmaxf(mx, pm);
        const float corr = expf(mx - mnew);
        mx = mnew;
        bf16x4s ph, pl;
        float psum = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float p = sc[i] > 0.5f * kMasked ? expf(sc[i] - mnew) : 0.f;
            psum += p;
            const bf16_t hi = f32_to_bf16(p);
            ph[i] = (short)hi;
            pl[i] = (short)f32_to_bf16(p - bf16_to_f32(hi));
        }
        den = fmaf(den, corr, psum);
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt) {
            f32x4 t = o[dt] * corr;
            t = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(bf16x4s, vf[dt]), ph, t, 0, 0, 0);
            o[dt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(bf16x4s, vf[dt]), pl, t, 0, 0, 0);
        }
    };
    load(kA, vA, 0);
    for (int pg = 0; pg <= last_page; pg += 2) {
        if (pg + 1 <= last_page) load(kB, vB, pg + 1);
        page_step(kA, vA, pg);
        if (pg + 2 <= last_page) load(kA, vA, pg + 2);
        if (pg + 1 <= last_page) page_step(kB, vB, pg + 1);
    }
    den += __shfl_xor(den, 16, kWave);
    den += __shfl_xor(den, 32, kWave);
    const int m = g * 16 + slot, r = m - (L & 15);
    const bool valid = r >= 0 && r < P;
    const float inv = valid ? 1.0f / den : 0.f;
#pragma unroll
    for (int dt = 0; dt < NDT; ++dt) {
        f32x4 v = {0.f, 0.f, 0.f, 0.f};
        if (valid) v = o[dt] * inv;
        xq_store4(xq_att, nks_d, m, head * DH + 16 * dt + 4 * kg, v);
    }
}

// ---------------------------------------------------- hand-over to the step
//
// The last prompt row is the only one whose logits are needed.  Leaves it
// where the step's LM-head GEMM expects its input (class-8 packed operand of
// x * gain in row 0, per-tile sums of squares) and sets the cache length to
// just below the row, so that the step's own argmax kernel, run for one
// appended row, finishes the job.   grid: d / 16 blocks of one wave.
__global__ __launch_bounds__(64) void prefill_last_kernel(const float *__restrict__ x_row, const bf16_t *__restrict__ gain,
                                                           bf16_t *__restrict__ xp, float *__restrict__ ssp,
                                                           int32_t *__restrict__ len_ptr, int len_before_row)
{
    const int lane = threadIdx.x, slot = lane & 15, kg = lane >> 4;
    const int tile = blockIdx.x, n = tile * 16 + 4 * kg;
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
    if (slot == 0) {
        v = *reinterpret_cast<const f32x4 *>(x_row + n);
        xp_store4<false>(xp, 8, 0, n, v * widen4(*reinterpret_cast<const uint2 *>(gain + n)));
    }
    float s = fmaf(v[3], v[3], fmaf(v[2], v[2], fmaf(v[1], v[1], v[0] * v[0])));
    s += __shfl_xor(s, 16, kWave);
    s += __shfl_xor(s, 32, kWave);
    if (lane == 0) ssp[(size_t)tile * 32] = s;
    if (blockIdx.x == 0 && lane == 0) *len_ptr = len_before_row;
}

}  // namespace anpd
