// Prompt processing for gfx950: the forward over all P prompt rows at once.
//
// Paper, Section 3.1 "Parallel Decoding", step 1, and the first lines of
// Algorithm 1: before any drafting the LLM reads the prompt once, which fills
// the (k, v) cache and yields the first generated token.  With hundreds of
// rows the GEMMs are bound by the matrix cores, not by weight streaming, so
// they get a form of their own: every wave owns a 64-feature x 64-row output
// tile, a weight fragment meets 4 row groups (each as hi and lo term) instead
// of one, and the eight waves of a block share their fragments through LDS.
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

constexpr int kPgThreads = 512;       // GEMM block: 8 waves, 4 (features) x 2 (rows)
constexpr int kPfTN = 4, kPfTM = 4;   // wave tile: 4 weight tiles x 4 row groups
constexpr int kPgStages = 4;          // LDS ring of k-steps
constexpr int kPgLead = 2;            // k-steps per block barrier (a round); the next round is requested one round ahead
constexpr int kPgUnits = 32;          // 1 KiB fragments per k-step: 16 weight tiles, 8 row groups x (hi, lo)
constexpr int kPgSplit = 4;           // K splits of the residual GEMMs
constexpr size_t kPgLdsBytes = (size_t)kPgStages * kPgUnits * 1024;

struct PrefillArgs {
    const uint4 *Wp;      // packed weights [n_tiles][nks][64]
    const uint4 *Xq;      // activation operand [G][nks][2][64]
    int nks, n_tiles, G;
    int L, P;             // cache length before the call, prompt rows
    int S;                // K splits (1 except RESIDUAL)
    // RESIDUAL
    float *part;          // partial products fp32 [S][16 G][d]
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
    int n_kv_heads;
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
// Row m: first x += the S partial products of the residual GEMM that ran
// before (in split order; S = 0: nothing to add), then
// h = x * g / sqrt(mean(x^2) + eps), stored as the split operand of the GEMM
// that follows.  EMBED: the row is fetched from the embedding table instead
// (x[m] = E[token]).  Rows outside the prompt are stored as zeros.
// grid: 16 G blocks (one per row) of 256 threads.
template <bool EMBED>
__global__ __launch_bounds__(256) void prefill_norm_kernel(const bf16_t *__restrict__ E, const int32_t *__restrict__ tok,
                                                            float *__restrict__ x, const float *__restrict__ part, int S,
                                                            const bf16_t *__restrict__ gain, bf16_t *__restrict__ xq, int nks,
                                                            int d, int L, int P, float inv_d, float eps)
{
    constexpr int NV = 8;   // 1024-column pieces of a row kept in registers (d <= 8192)
    __shared__ float red[4];
    const int m = blockIdx.x, r = m - (L & 15);
    const bool valid = r >= 0 && r < P;
    const size_t rows = (size_t)gridDim.x;
    float *xr = x + (size_t)m * d;
    f32x4 v[NV];
    float ss = 0.f;
    if (valid) {
        // every load of the row is requested before the first one is used
        const bf16_t *er = EMBED ? E + (size_t)tok[r] * d : nullptr;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int k = 4 * threadIdx.x + 1024 * i;
            v[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
            if (k < d) v[i] = EMBED ? widen4(*reinterpret_cast<const uint2 *>(er + k)) : *reinterpret_cast<const f32x4 *>(xr + k);
        }
        if (!EMBED) {
            for (int s = 0; s < S; ++s) {   // split order
                f32x4 p[NV];
#pragma unroll
                for (int i = 0; i < NV; ++i) {
                    const int k = 4 * threadIdx.x + 1024 * i;
                    p[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
                    if (k < d) p[i] = *reinterpret_cast<const f32x4 *>(part + ((size_t)s * rows + m) * d + k);
                }
#pragma unroll
                for (int i = 0; i < NV; ++i) v[i] += p[i];
            }
        }
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int k = 4 * threadIdx.x + 1024 * i;
            if (k < d) {
                if (EMBED || S > 0) *reinterpret_cast<f32x4 *>(xr + k) = v[i];
                ss = fmaf(v[i][3], v[i][3], fmaf(v[i][2], v[i][2], fmaf(v[i][1], v[i][1], fmaf(v[i][0], v[i][0], ss))));
            }
        }
    }
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float rinv = 1.0f / sqrtf((red[0] + red[1] + red[2] + red[3]) * inv_d + eps);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int k = 4 * threadIdx.x + 1024 * i;
        if (k < d) {
            f32x4 h = {0.f, 0.f, 0.f, 0.f};
            if (valid) h = v[i] * rinv * widen4(*reinterpret_cast<const uint2 *>(gain + k));
            xq_store4(xq, nks, m, k, h);
        }
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
__device__ __forceinline__ void prefill_epilogue(const PrefillArgs &a, int tile, int m, int kg, f32x4 y, bool valid, int sp)
{
    if (EPI == EPI_RESIDUAL) {
        if (valid) *reinterpret_cast<f32x4 *>(a.part + ((size_t)sp * a.G * 16 + m) * a.d + tile * 16 + 4 * kg) = y;
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
        const int Tq = a.n_heads * a.head_dim / 16, Tkv = a.n_kv_heads * a.head_dim / 16;
        const int which = tile < Tq ? 0 : (tile < Tq + Tkv ? 1 : 2), t = tile - (which == 0 ? 0 : (which == 1 ? Tq : Tq + Tkv));
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
                bf16_t *dst = a.pool + kvf_base(page, a.layer, a.n_layers, 0, h, a.n_kv_heads, a.head_dim) + kf_elem(tk, dim);
                *reinterpret_cast<uint2 *>(dst) = make_uint2((uint32_t)f32_to_bf16(o[0]) | ((uint32_t)f32_to_bf16(o[1]) << 16),
                                                             (uint32_t)f32_to_bf16(o[2]) | ((uint32_t)f32_to_bf16(o[3]) << 16));
            }
        } else {
            const int n = t * 16 + 4 * kg, h = n / a.head_dim, dim = n - h * a.head_dim;
            bf16_t *dst = a.pool + kvf_base(page, a.layer, a.n_layers, 1, h, a.n_kv_heads, a.head_dim);
#pragma unroll
            for (int i = 0; i < 4; ++i) dst[vf_elem(tk, dim + i)] = f32_to_bf16(y[i]);
        }
    }
}

// -------------------------------------------------------------------- GEMM
//
// Y^T[features][rows] = W X^T with hi and lo terms of X accumulated into the
// same tile.  Block = 4 x 2 waves, 256 features x 128 rows, each wave a
// 64 x 64 tile (4 weight fragments x 4 row groups).  Per k-step the block
// needs 16 weight fragments and 16 activation fragments of 1 KiB; each wave
// requests four of them straight into LDS (buffer loads with the LDS bit:
// lane i's 16 bytes land at base + 16 i, the fragment order itself; absent
// tiles and row groups read zeros and fetch nothing), one round of two k-steps
// ahead of the matrix cores through a ring of four stages, and every wave then
// reads its 12 fragments per k-step from LDS.  A fragment thus crosses the
// L2 -> CU path once per block instead of once per wave that uses it.
// One block barrier per round of two k-steps: it publishes the two stages
// whose loads the waves have just waited for, and frees the two stages read in
// the previous round for the requests that follow it (one barrier per k-step
// with three stages in flight measured 2 % slower).
// RESIDUAL GEMMs (few output features) are split S ways along K so that the
// grid fills the chip; the S partial tiles go to `part` and are added to the
// residual stream, in split order, by the norm kernel that follows.  S is
// fixed by the matrix, never by the number of rows: a row's sums are formed
// in the same order whatever else is in the batch.
// grid: ceil(n_tiles / 16) * S * ceil(G / 8) blocks; rows run fastest, so
// consecutive blocks share a weight range.
template <int OFF>
__device__ __forceinline__ u32x4_t lds_read16(uint32_t addr)
{
    u32x4_t v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
    return v;
}

// TN: weight fragments per wave (4: the 256-feature tile above; 3: 192 features).  The launcher picks the
// one whose grid fills the chip's compute units better (QKV of 512 rows: 192 blocks of 256 features, or 256
// blocks of 192); an output element's sums do not depend on it.
template <int EPI, int TN = kPfTN>
__global__ __launch_bounds__(kPgThreads) void prefill_gemm_kernel(PrefillArgs a)
{
    static_assert(TN == 3 || TN == 4, "a wave holds 3 or 4 weight fragments");
    extern __shared__ uint4 ring[];   // [kPgStages][kPgUnits][64]
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wf = wave & 3, wr = wave >> 2;
    const int n_br = (a.G + 7) / 8;
    // Blocks are dealt to the 8 XCDs in turn, and each XCD has its own L2.  Give XCD x a contiguous
    // range of the (weights, rows) order, so that the blocks sharing a weight range, and the row
    // blocks they all stream in step, meet in one L2 instead of being fetched into several.
    int id;
    {
        const int n = (int)gridDim.x, per = (n + 7) / 8, rem = n % 8;
        const int xcd = (int)blockIdx.x % 8, j = (int)blockIdx.x / 8;
        id = (rem == 0 || xcd < rem ? xcd * per : rem * per + (xcd - rem) * (per - 1)) + j;
    }
    const int br = id % n_br;
    id /= n_br;
    const int sp = id % a.S, bt = id / a.S;
    const int F0 = bt * 4 * TN, G0 = br * 8;
    const int nks = a.nks;
    const int ks0 = (int)((long long)sp * nks / a.S), n_it = (int)((long long)(sp + 1) * nks / a.S) - ks0;

    // this wave's share of a stage: units 4 wave .. 4 wave + 3 (waves 0..3 weights, 4..7 activations); with
    // TN = 3 a weight wave's fourth unit is an empty descriptor (zeros, nothing fetched): every wave still
    // issues four loads per stage, which is what the waits below count
    __amdgpu_buffer_rsrc_t rs[4];
    int uoff[4];
    const int ustride = wave < 4 ? 1024 : 2048;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        if (wave < 4) {
            const int tile = F0 + TN * wave + j;
            const bool have = j < TN && tile < a.n_tiles;
            rs[j] = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint4 *>(a.Wp + (size_t)(have ? tile : 0) * nks * 64), 0,
                                                      have ? nks * 1024 : 0, 0x00020000);
            uoff[j] = 0;
        } else {
            const int n_g = a.G - G0 < 8 ? a.G - G0 : 8;
            const int u = 4 * (wave - 4) + j;   // (row group, hi | lo)
            rs[j] = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint4 *>(a.Xq + (size_t)G0 * nks * 128), 0, n_g * nks * 2048,
                                                      0x00020000);
            uoff[j] = ((u >> 1) * nks * 2 + (u & 1)) * 1024;
        }
    }
    auto request = [&](int it) {
        uint4 *dst = ring + ((size_t)(it & (kPgStages - 1)) * kPgUnits + 4 * wave) * 64;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs[j], (__attribute__((address_space(3))) void *)(dst + j * 64), 16,
                                                     uoff[j] + (ks0 + it) * ustride + lane * 16, 0, 0, 0);
    };

    f32x4 acc[TN][kPfTM];
#pragma unroll
    for (int t = 0; t < TN; ++t)
#pragma unroll
        for (int g = 0; g < kPfTM; ++g) acc[t][g] = (f32x4){0.f, 0.f, 0.f, 0.f};
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void *)ring;

    // The fragment reads are written as assembly: reads the compiler can see would make it wait for
    // every outstanding load into LDS first (it cannot tell the ring's stages apart), and the ring
    // exists to keep three stages in flight.
    auto read_stage = [&](u32x4_t (&w)[4], u32x4_t (&xh)[kPfTM], u32x4_t (&xl)[kPfTM], int it) {
        const uint32_t sbase = lds_base + (uint32_t)(it & (kPgStages - 1)) * (kPgUnits * 1024) + (uint32_t)lane * 16;
        const uint32_t aw = sbase + (uint32_t)(4 * wf) * 1024, ax = sbase + (uint32_t)(16 + 8 * wr) * 1024;
        w[0] = lds_read16<0>(aw); w[1] = lds_read16<1024>(aw); w[2] = lds_read16<2048>(aw);
        if (TN == 4) w[3] = lds_read16<3072>(aw);
        else w[3] = w[2];
        xh[0] = lds_read16<0>(ax); xh[1] = lds_read16<2048>(ax); xh[2] = lds_read16<4096>(ax); xh[3] = lds_read16<6144>(ax);
        xl[0] = lds_read16<1024>(ax); xl[1] = lds_read16<3072>(ax); xl[2] = lds_read16<5120>(ax); xl[3] = lds_read16<7168>(ax);
    };
    auto wait_reads = [&](u32x4_t (&w)[4], u32x4_t (&xh)[kPfTM], u32x4_t (&xl)[kPfTM]) {
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : "+v"(w[0]), "+v"(w[1]), "+v"(w[2]), "+v"(w[3]), "+v"(xh[0]), "+v"(xh[1]), "+v"(xh[2]), "+v"(xh[3]),
                       "+v"(xl[0]), "+v"(xl[1]), "+v"(xl[2]), "+v"(xl[3]));
    };
    auto mma = [&](const u32x4_t (&w)[4], const u32x4_t (&xh)[kPfTM], const u32x4_t (&xl)[kPfTM]) {
#pragma unroll
        for (int t = 0; t < TN; ++t)
#pragma unroll
            for (int g = 0; g < kPfTM; ++g)
                acc[t][g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, w[t]), __builtin_bit_cast(bf16x8, xh[g]),
                                                                    acc[t][g], 0, 0, 0);
#pragma unroll
        for (int t = 0; t < TN; ++t)
#pragma unroll
            for (int g = 0; g < kPfTM; ++g)
                acc[t][g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, w[t]), __builtin_bit_cast(bf16x8, xl[g]),
                                                                    acc[t][g], 0, 0, 0);
    };
    // Two k-steps per block barrier.  The barrier of round j is reached by a wave once its own loads of
    // stages 2j and 2j + 1 have landed (at most the two younger stages still outstanding) and its reads of
    // the previous round's stages have returned; it publishes this round's stages and frees the previous
    // round's slots for stages 2j + 2 and 2j + 3.  All four slots are requested before the first round.
    u32x4_t wA[4], hA[kPfTM], lA[kPfTM], wB[4], hB[kPfTM], lB[kPfTM];
#pragma unroll
    for (int s = 0; s < kPgStages; ++s)
        if (s < n_it) request(s);
    for (int it = 0; it < n_it; it += 2) {
        // (the next round's stages are requested after this barrier, so only in round 0 is anything younger
        // than this round's stages outstanding: stages 2 and 3 from the prologue)
        if (it == 0 && n_it > 3) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        else if (it == 0 && n_it == 3) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        asm volatile("s_barrier" ::: "memory");
        if (it > 0) {
            if (it + 2 < n_it) request(it + 2);
            if (it + 3 < n_it) request(it + 3);
        }
        read_stage(wA, hA, lA, it);
        if (it + 1 < n_it) read_stage(wB, hB, lB, it + 1);
        wait_reads(wA, hA, lA);
        mma(wA, hA, lA);
        if (it + 1 < n_it) {
            wait_reads(wB, hB, lB);
            mma(wB, hB, lB);
        }
    }

    const int slot = lane & 15, kg = lane >> 4;
    const int r0 = a.L & 15;
    const int f0 = F0 + TN * wf, g0 = G0 + 4 * wr;
#pragma unroll
    for (int t = 0; t < TN; ++t) {
        if (f0 + t >= a.n_tiles) break;   // wave-uniform
#pragma unroll
        for (int g = 0; g < kPfTM; ++g) {
            const int m = (g0 + g) * 16 + slot;
            const bool valid = g0 + g < a.G && m >= r0 && m < r0 + a.P;
            prefill_epilogue<EPI>(a, f0 + t, m, kg, acc[t][g], valid, sp);
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
                                                            int layer, int n_layers, int n_heads, int n_kv_heads, float scale,
                                                            bf16_t *__restrict__ xq_att, int nks_d)
{
    constexpr int NKS = DH / 32, NDT = DH / 16;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, slot = lane & 15, kg = lane >> 4;
    const int head = blockIdx.x, kvh = head / (n_heads / n_kv_heads);
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
        const uint4 *kp = reinterpret_cast<const uint4 *>(pool + kvf_base(page, layer, n_layers, 0, kvh, n_kv_heads, DH));
        const uint2 *vp = reinterpret_cast<const uint2 *>(pool + kvf_base(page, layer, n_layers, 1, kvh, n_kv_heads, DH));
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
// The last prompt row is the only one whose logits are needed.  Adds the last
// down projection's partial products to it and leaves it where the step's
// LM-head GEMM expects its input (class-8 packed operand of x * gain in row 0,
// per-tile sums of squares); sets the cache length to just below the row, so
// that the step's own argmax kernel, run for one appended row, finishes the
// job.   grid: d / 16 blocks of one wave.
__global__ __launch_bounds__(64) void prefill_last_kernel(const float *__restrict__ x_row, const float *__restrict__ part_row,
                                                           int S, size_t part_stride, const bf16_t *__restrict__ gain,
                                                           bf16_t *__restrict__ xp, float *__restrict__ ssp,
                                                           int32_t *__restrict__ len_ptr, int len_before_row)
{
    const int lane = threadIdx.x, slot = lane & 15, kg = lane >> 4;
    const int tile = blockIdx.x, n = tile * 16 + 4 * kg;
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
    if (slot == 0) {
        v = *reinterpret_cast<const f32x4 *>(x_row + n);
        for (int s = 0; s < S; ++s) v += *reinterpret_cast<const f32x4 *>(part_row + (size_t)s * part_stride + n);
        xp_store4<false>(xp, 8, 0, n, v * widen4(*reinterpret_cast<const uint2 *>(gain + n)));
    }
    float s = fmaf(v[3], v[3], fmaf(v[2], v[2], fmaf(v[1], v[1], v[0] * v[0])));
    s += __shfl_xor(s, 16, kWave);
    s += __shfl_xor(s, 32, kWave);
    if (lane == 0) ssp[(size_t)tile * 32] = s;
    if (blockIdx.x == 0 && lane == 0) *len_ptr = len_before_row;
}

}  // namespace anpd
