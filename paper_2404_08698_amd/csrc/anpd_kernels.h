// HIP kernels of the ANPD verification step for gfx950 (MI355X, CDNA4).
//
// The step is one LLaMA-shaped forward over a window of M = k+1 rows (the last
// accepted token plus k drafts; paper Section 3.1, "Parallel Decoding", step 2)
// against a paged KV cache, ending in greedy argmax per row and the
// longest-matching-prefix acceptance of Algorithm 1.
//
// Every kernel computes a window row from that row's own data in an order
// that does not depend on M, so the result for a position is bit-identical
// whether it was verified in a 1-row or a 32-row window.  That is what makes
// ANPD on this path reproduce greedy decoding token for token.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace anpd {

typedef uint16_t bf16_t;  // bfloat16 storage
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kWave = 64;
constexpr int kAttnSplit = 64;        // keys per attention split (fixed: part of the numerics)
constexpr float kMasked = -1.0e30f;   // score of a key a row must not see

// ---------------------------------------------------------------- scalars

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float((uint32_t)b << 16); }

// round to nearest, ties to even (finite inputs)
__device__ __forceinline__ bf16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

__device__ __forceinline__ float load_f32(const float *p, size_t i) { return p[i]; }
__device__ __forceinline__ float load_f32(const bf16_t *p, size_t i) { return bf16_to_f32(p[i]); }
__device__ __forceinline__ void store_kv(float *p, size_t i, float v) { p[i] = v; }
__device__ __forceinline__ void store_kv(bf16_t *p, size_t i, float v) { p[i] = f32_to_bf16(v); }

// eight consecutive elements, widened to float
__device__ __forceinline__ void load8(const float *p, float (&o)[8])
{
    float4 a = *reinterpret_cast<const float4 *>(p);
    float4 b = *reinterpret_cast<const float4 *>(p + 4);
    o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w;
    o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
}
__device__ __forceinline__ void load8(const bf16_t *p, float (&o)[8])
{
    uint4 r = *reinterpret_cast<const uint4 *>(p);
    o[0] = __uint_as_float(r.x << 16); o[1] = __uint_as_float(r.x & 0xffff0000u);
    o[2] = __uint_as_float(r.y << 16); o[3] = __uint_as_float(r.y & 0xffff0000u);
    o[4] = __uint_as_float(r.z << 16); o[5] = __uint_as_float(r.z & 0xffff0000u);
    o[6] = __uint_as_float(r.w << 16); o[7] = __uint_as_float(r.w & 0xffff0000u);
}

// Device-coherent accesses (relaxed, agent scope): the store is written through and the load is
// served from the coherence point, so blocks on different XCDs can hand small results to each
// other through a counter without cache-wide write-back / invalidate fences.
template <typename T>
__device__ __forceinline__ void st_agent(T *p, T v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
template <typename T>
__device__ __forceinline__ T ld_agent(const T *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
// The same at system scope, for words in pinned host memory.
template <typename T>
__device__ __forceinline__ void st_system(T *p, T v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM); }
template <typename T>
__device__ __forceinline__ T ld_system(const T *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM); }

// Accessors for data that one block writes and another block reads.  COH = false: ordinary
// accesses, for kernels whose producers ran in an earlier launch.  COH = true: device-coherent
// accesses (see st_agent / ld_agent), for the persistent kernel where producer and consumer run in
// the same launch on different XCDs.  Wider items are moved as 8-byte pieces.
template <bool COH>
__device__ __forceinline__ float ldc(const float *p) { return COH ? ld_agent(p) : *p; }
template <bool COH>
__device__ __forceinline__ void stc(float *p, float v)
{
    if (COH) st_agent(p, v);
    else *p = v;
}
template <bool COH>
__device__ __forceinline__ uint2 ldc8(const uint2 *p)
{
    if (!COH) return *p;
    unsigned long long v = ld_agent(reinterpret_cast<const unsigned long long *>(p));
    return make_uint2((uint32_t)v, (uint32_t)(v >> 32));
}
template <bool COH>
__device__ __forceinline__ void stc8(void *p, uint2 v)
{
    if (COH) st_agent(reinterpret_cast<unsigned long long *>(p), (unsigned long long)v.x | ((unsigned long long)v.y << 32));
    else *reinterpret_cast<uint2 *>(p) = v;
}
template <bool COH>
__device__ __forceinline__ uint4 ldc16(const uint4 *p)
{
    if (!COH) return *p;
    uint2 lo = ldc8<true>(reinterpret_cast<const uint2 *>(p)), hi = ldc8<true>(reinterpret_cast<const uint2 *>(p) + 1);
    return make_uint4(lo.x, lo.y, hi.x, hi.y);
}
template <bool COH>
__device__ __forceinline__ void stc16(float *p, f32x4 v)
{
    if (COH) {
        stc8<true>(p, make_uint2(__float_as_uint(v[0]), __float_as_uint(v[1])));
        stc8<true>(p + 2, make_uint2(__float_as_uint(v[2]), __float_as_uint(v[3])));
    } else {
        *reinterpret_cast<f32x4 *>(p) = v;
    }
}
// 2-byte store; the coherent form is the same instruction with the write-through bits set
template <bool COH>
__device__ __forceinline__ void stc2(bf16_t *p, bf16_t v)
{
    if (COH) asm volatile("global_store_short %0, %1, off sc0 sc1" ::"v"(p), "v"((uint32_t)v) : "memory");
    else *p = v;
}

// Indexed loads from a buffer whose base pointer is the same for the whole wave.  The coherent
// form uses buffer instructions with the sc0 sc1 bits, which the compiler can keep in flight
// together (atomic loads are issued one at a time); the plain form is an ordinary load.
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
constexpr int kAuxCoherent = 17;  // sc0 | sc1
// Weights are read once per step and never again before 13 GB of other weights have gone by: loads
// marked non-temporal stream them past the caches instead of displacing what is re-read (activations,
// the cache pages).  Measured on the weight access pattern alone: 7.1 TB/s against 6.4 TB/s unmarked.
constexpr int kAuxStream = 2;     // nt
__device__ __forceinline__ uint4 ld_stream(const uint4 *p)
{
    typedef unsigned int u4 __attribute__((ext_vector_type(4)));
    u4 v = __builtin_nontemporal_load(reinterpret_cast<const u4 *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ __amdgpu_buffer_rsrc_t wave_buffer(const void *base)
{
    // (said explicitly to be the same in every lane: a base that was computed on the vector ALU - an index
    // from an integer division, say - would otherwise make every load a loop over the distinct descriptors)
    const unsigned long long a = (unsigned long long)base;
    const unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)a);
    const unsigned hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(a >> 32));
    return __builtin_amdgcn_make_buffer_rsrc((void *)(((unsigned long long)hi << 32) | lo), 0, 0x7fffffff, 0x00020000);
}
template <bool COH>
__device__ __forceinline__ uint4 ld16_at(const uint4 *base, uint32_t idx)
{
    if (!COH) return base[idx];
    u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(wave_buffer(base), (int)(idx * 16u), 0, kAuxCoherent);
    return make_uint4(v.x, v.y, v.z, v.w);
}
template <bool COH>
__device__ __forceinline__ uint2 ld8_at(const uint2 *base, uint32_t idx)
{
    if (!COH) return base[idx];
    u32x2_t v = __builtin_amdgcn_raw_buffer_load_b64(wave_buffer(base), (int)(idx * 8u), 0, kAuxCoherent);
    return make_uint2(v.x, v.y);
}
template <bool COH>
__device__ __forceinline__ float ldf_at(const float *base, uint32_t idx)
{
    if (!COH) return base[idx];
    return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(wave_buffer(base), (int)(idx * 4u), 0, kAuxCoherent));
}

// threadIdx.x as a value the optimiser treats as new at every call.  In the persistent kernel,
// lane-dependent offsets derived from the plain threadIdx.x are loop invariant over the layers: they
// get computed once up front, by the dozen, and then live in scratch memory.
__device__ __forceinline__ int fresh_tid()
{
    int t = threadIdx.x;
    asm volatile("" : "+v"(t));
    return t;
}

// Block barrier that orders LDS traffic only.  __syncthreads() also waits for every outstanding
// global load of the wave, which would drain the weight prefetch at each tile boundary.
__device__ __forceinline__ void block_sync_lds() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Wait until this wave's outstanding global stores have been acknowledged.
__device__ __forceinline__ void wait_stores() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Value of lane + 8 / lane - 8 within each row of 16 lanes, as a DPP move on the vector ALU
// (no trip through the LDS crossbar).  Lanes whose source falls outside the row read 0.
__device__ __forceinline__ float row_down8(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x108, 0xF, 0xF, true));
}
__device__ __forceinline__ float row_up8(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x118, 0xF, 0xF, true));
}

// Maximum / sum over the four lanes l, l ^ 16, l ^ 32, l ^ 48 (one lane of each row of 16), the same value in
// all four: two row swaps on the vector ALU (v_permlane16_swap exchanges the odd rows of its first operand
// with the even rows of its second, v_permlane32_swap the upper half with the lower half), no trip through
// LDS.  The sum adds in the order of the xor-16, xor-32 butterfly.
__device__ __forceinline__ float rows_max(float v)
{
    auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
    auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float rows_sum(float v)
{
    auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = __uint_as_float(a[0]) + __uint_as_float(a[1]);
    auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
    return v;
}

// Window class: how many 16-row MFMA slots a window of M rows occupies (8 = half a tile).
__host__ __device__ __forceinline__ int window_class(int M) { return M <= 8 ? 8 : (M <= 16 ? 16 : 32); }

// The MFMA GEMMs take their activation operand as two bf16 terms, v ~= hi + lo
// (hi = bf16(v), lo = bf16(v - hi)), which keeps ~16 mantissa bits of the fp32
// activation, laid out in MFMA B-fragment order Xp[k-step][frag][lane][8]:
// lane = 16 * kg + slot holds columns 32 * ks + 8 * kg .. + 8 of the row in `slot`.
//   class 8:  one fragment; slot m = hi of row m, slot m + 8 = lo of row m;
//   class 16: fragments (hi, lo) of rows 0..15;
//   class 32: fragments (hi, lo) of rows 0..15, then (hi, lo) of rows 16..31;
//   packed_class(nf), nf >= 2: nf fragments in the class-8 arrangement, fragment f holding rows 8 f .. 8 f + 7
//   (slot m % 8 = hi, slot m % 8 + 8 = lo): the one-kernel step's form for windows of more than 8 rows.
// Returns the bf16-element offset of (row m, column k, hi|lo).
__host__ __device__ constexpr int packed_class(int nf) { return nf == 1 ? 8 : 1000 + nf; }
__host__ __device__ __forceinline__ size_t xp_offset(int cls, int m, int k, int lo)
{
    const int ks = k >> 5, kg = (k >> 3) & 3, j = k & 7;
    int nt, frag, slot;
    if (cls == 8) { nt = 1; frag = 0; slot = m + 8 * lo; }
    else if (cls >= 1000) { nt = cls - 1000; frag = m >> 3; slot = (m & 7) + 8 * lo; }
    else { nt = cls >> 3; frag = 2 * (m >> 4) + lo; slot = m & 15; }
    return ((((size_t)ks * nt + frag) * 64) + (size_t)kg * 16 + slot) * 8 + j;
}

// ------------------------------------------------------------------ embed

// x[r][:] = E[token[r]][:]   grid: M blocks
template <typename WT>
__global__ __launch_bounds__(256) void embed_kernel(const WT *__restrict__ E, const int32_t *__restrict__ tok,
                                                     float *__restrict__ x, int d)
{
    int r = blockIdx.x;
    const WT *src = E + (size_t)tok[r] * d;
    for (int i = threadIdx.x; i < d; i += blockDim.x) x[(size_t)r * d + i] = load_f32(src, (size_t)i);
}

// --------------------------------------------------- residual add + RMSNorm

// x[r] += y[r] (if y), then h[r] = x[r] * g / sqrt(mean(x[r]^2) + eps).
// grid: M blocks, one row each; the reduction order depends on d only.
template <typename WT>
__global__ __launch_bounds__(256) void addnorm_kernel(float *__restrict__ x, const float *__restrict__ y,
                                                       const WT *__restrict__ g, float *__restrict__ h, int d,
                                                       float eps)
{
    __shared__ float part[4];
    int r = blockIdx.x;
    float *xr = x + (size_t)r * d;
    float ss = 0.f;
    for (int i = threadIdx.x; i < d; i += 256) {
        float v = xr[i];
        if (y) {
            v += y[(size_t)r * d + i];
            xr[i] = v;
        }
        ss = fmaf(v, v, ss);
    }
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    float tot = ((part[0] + part[1]) + part[2]) + part[3];
    float rinv = 1.0f / sqrtf(tot / (float)d + eps);
    for (int i = threadIdx.x; i < d; i += 256) {
        float v = xr[i] * load_f32(g, (size_t)i) * rinv;
        h[(size_t)r * d + i] = v;
    }
}

// --------------------------------------------------------------- GEMM (dot)
//
// Wavefront dot-product form of Y[M][N] = X[M][K] * W[N][K]^T.  A wave owns R
// output columns; its 64 lanes stride over K in 8-element pieces (one 16-byte
// load of bf16 weights per lane per row), multiply against the fp32 rows of X
// and finish with a butterfly sum over the lanes.  Exact fp32 products, fp32
// accumulation.  The weight matrix may be given as up to three row segments
// (Wq|Wk|Wv or Wgate|Wup) of n_seg0, n_seg1 and the remaining rows (multiples of
// R), written side by side into Y.
// grid: n_total / (4 * R) blocks of 4 waves.
template <typename WT, int R>
__global__ __launch_bounds__(256) void gemm_dot_kernel(const float *__restrict__ X, int M, int K,
                                                        const WT *__restrict__ W0, const WT *__restrict__ W1,
                                                        const WT *__restrict__ W2, int n_seg0, int n_seg1, int n_total,
                                                        float *__restrict__ Y, int ldy)
{
    const int lane = threadIdx.x & 63;
    const int n0 = (blockIdx.x * 4 + (threadIdx.x >> 6)) * R;
    if (n0 >= n_total) return;
    const int seg = n0 < n_seg0 ? 0 : (n0 < n_seg0 + n_seg1 ? 1 : 2);
    const WT *W = (seg == 0 ? W0 : (seg == 1 ? W1 : W2)) + (size_t)(n0 - (seg == 0 ? 0 : (seg == 1 ? n_seg0 : n_seg0 + n_seg1))) * K;

    for (int m0 = 0; m0 < M; m0 += 8) {
        float acc[R][8];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int mm = 0; mm < 8; ++mm) acc[r][mm] = 0.f;

        for (int k = lane * 8; k < K; k += 64 * 8) {
            float w[R][8];
#pragma unroll
            for (int r = 0; r < R; ++r) load8(W + (size_t)r * K + k, w[r]);
#pragma unroll
            for (int mm = 0; mm < 8; ++mm) {
                if (m0 + mm < M) {
                    float xv[8];
                    load8(X + (size_t)(m0 + mm) * K + k, xv);
#pragma unroll
                    for (int r = 0; r < R; ++r)
#pragma unroll
                        for (int i = 0; i < 8; ++i) acc[r][mm] = fmaf(xv[i], w[r][i], acc[r][mm]);
                }
            }
        }
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int mm = 0; mm < 8; ++mm) {
                float v = wave_sum(acc[r][mm]);
                if (lane == 0 && m0 + mm < M) Y[(size_t)(m0 + mm) * ldy + n0 + r] = v;
            }
    }
}

// ------------------------------------------------------- RoPE + KV write
//
// Page layout: [page][layer][k|v][head][token in page][head_dim].
__device__ __forceinline__ size_t kv_offset(int page, int layer, int n_layers, int kv, int head, int n_heads,
                                            int tok_in_page, int page_tokens, int head_dim)
{
    return ((((size_t)page * n_layers + layer) * 2 + kv) * n_heads + head) * ((size_t)page_tokens * head_dim) +
           (size_t)tok_in_page * head_dim;
}

// A row of the fused qkv buffer is [q: n_heads * head_dim | k: n_kv_heads * head_dim | v: the same].
// Rotates q (in place, in the fused qkv buffer) and k by the row's absolute
// position len + r, pair (i, i + head_dim/2) by angle pos * base^(-2i/head_dim)
// (cos/sin from a table computed in double on the host), and writes k and v of
// the row into the cache in the storage type.  grid: M blocks.
template <typename KT>
__global__ __launch_bounds__(256) void rope_kv_kernel(float *__restrict__ qkv, const float2 *__restrict__ rope_tab,
                                                       KT *__restrict__ pool, const int32_t *__restrict__ page_table,
                                                       const int32_t *__restrict__ len_ptr, int layer, int n_layers,
                                                       int n_heads, int n_kv_heads, int head_dim, int page_tokens,
                                                       const int32_t *__restrict__ depth /* draft tree: nullable */)
{
    const int r = blockIdx.x, d = n_heads * head_dim, dkv = n_kv_heads * head_dim, half = head_dim >> 1;
    const int pos = *len_ptr + r;                              // the row's cache slot
    const int rpos = depth ? *len_ptr + depth[r] : pos;        // the row's rotary position
    const int page = page_table[pos / page_tokens], tip = pos % page_tokens;
    float *q = qkv + (size_t)r * (d + 2 * dkv), *k = q + d, *v = k + dkv;
    for (int idx = threadIdx.x; idx < n_heads * half; idx += 256) {
        int hd = idx / half, i = idx - hd * half;
        float2 cs = rope_tab[(size_t)rpos * half + i];
        int e0 = hd * head_dim + i, e1 = e0 + half;
        float qa = q[e0], qb = q[e1];
        q[e0] = qa * cs.x - qb * cs.y;
        q[e1] = qb * cs.x + qa * cs.y;
        if (hd >= n_kv_heads) continue;
        float ka = k[e0], kb = k[e1];
        size_t ko = kv_offset(page, layer, n_layers, 0, hd, n_kv_heads, tip, page_tokens, head_dim);
        size_t vo = kv_offset(page, layer, n_layers, 1, hd, n_kv_heads, tip, page_tokens, head_dim);
        store_kv(pool, ko + i, ka * cs.x - kb * cs.y);
        store_kv(pool, ko + i + half, kb * cs.x + ka * cs.y);
        store_kv(pool, vo + i, v[e0]);
        store_kv(pool, vo + i + half, v[e1]);
    }
}

// ------------------------------------------------------------- attention
//
// Window-causal attention of the M query rows over the paged cache.  Keys are
// cut into fixed splits of kAttnSplit absolute positions; block (head, split)
// computes, for each row, the split's score maximum, sum of exponentials and
// unnormalised weighted V sum; attn_combine_kernel merges the splits of a row
// in increasing order.  Row r sees keys 0..len + r; keys it must not see get
// weight exactly 0, so a row's numbers do not depend on M.
// Lane layout: a key's head_dim elements are spread over DH/8 lanes (16 bytes
// of bf16 each), so a wave reads 64*8 consecutive elements of the page.
// part: [head][split][max_window][DH + 2] = (o[DH], max, denominator).
// grid: (n_heads, n_splits), 4 waves.
template <typename KT, int DH>
__global__ __launch_bounds__(256) void attn_kernel(const float *__restrict__ qkv, int q_stride, const KT *__restrict__ pool,
                                                    const int32_t *__restrict__ page_table,
                                                    const int32_t *__restrict__ len_ptr, int M, int layer, int n_layers,
                                                    int n_heads, int n_kv_heads, int page_tokens, int max_window,
                                                    int max_splits, float scale, float *__restrict__ part,
                                                    const uint32_t *__restrict__ row_mask /* draft tree: nullable */)
{
    constexpr int LPK = DH / 8;        // lanes per key
    constexpr int KPG = 64 / LPK;      // keys per wave group
    constexpr int NG = kAttnSplit / KPG;
    __shared__ float sc[8][kAttnSplit];
    __shared__ float stat[8][2];
    __shared__ float red[4][8][DH];

    const int head = blockIdx.x, split = blockIdx.y;
    const int kvh = head / (n_heads / n_kv_heads);   // the key / value head this query head reads
    const int L = *len_ptr;
    const int s0 = split * kAttnSplit;
    if (s0 >= L + M) return;  // no key of this split exists for any row
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int ksub = lane / LPK, dg = lane % LPK;

    for (int m0 = 0; m0 < M; m0 += 8) {
        // ---- scores
        float qv[8][8];
#pragma unroll
        for (int mm = 0; mm < 8; ++mm) {
            if (m0 + mm < M) {
                load8(qkv + (size_t)(m0 + mm) * q_stride + head * DH + dg * 8, qv[mm]);
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) qv[mm][i] = 0.f;
            }
        }
        for (int g = wave; g < NG; g += 4) {
            const int jl = g * KPG + ksub, j = s0 + jl;
            const bool exists = j < L + M;
            float kv[8];
            if (exists) {
                int page = page_table[j / page_tokens];
                load8(pool + kv_offset(page, layer, n_layers, 0, kvh, n_kv_heads, j % page_tokens, page_tokens, DH) + dg * 8, kv);
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) kv[i] = 0.f;
            }
#pragma unroll
            for (int mm = 0; mm < 8; ++mm) {
                float p = 0.f;
#pragma unroll
                for (int i = 0; i < 8; ++i) p = fmaf(qv[mm][i], kv[i], p);
#pragma unroll
                for (int off = LPK / 2; off >= 1; off >>= 1) p += __shfl_xor(p, off, kWave);
                if (dg == 0) {
                    bool sees = j <= L + m0 + mm;
                    if (row_mask && m0 + mm < M) sees = j < L || (j - L < 32 && ((row_mask[m0 + mm] >> (j - L)) & 1u));
                    sc[mm][jl] = (exists && m0 + mm < M && sees) ? p * scale : kMasked;
                }
            }
        }
        __syncthreads();
        // ---- per-row maximum, exponentials, denominator (one key per lane)
        for (int mm = wave; mm < 8; mm += 4) {
            float s = sc[mm][lane];
            float mx = wave_max(s);
            float p = (s > 0.5f * kMasked) ? expf(s - mx) : 0.f;
            sc[mm][lane] = p;
            float den = wave_sum(p);
            if (lane == 0) { stat[mm][0] = mx; stat[mm][1] = den; }
        }
        __syncthreads();
        // ---- weighted V
        float acc[8][8];
#pragma unroll
        for (int mm = 0; mm < 8; ++mm)
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[mm][i] = 0.f;
        for (int g = wave; g < NG; g += 4) {
            const int jl = g * KPG + ksub, j = s0 + jl;
            if (j < L + M) {
                float vv[8];
                int page = page_table[j / page_tokens];
                load8(pool + kv_offset(page, layer, n_layers, 1, kvh, n_kv_heads, j % page_tokens, page_tokens, DH) + dg * 8, vv);
#pragma unroll
                for (int mm = 0; mm < 8; ++mm) {
                    float p = sc[mm][jl];
#pragma unroll
                    for (int i = 0; i < 8; ++i) acc[mm][i] = fmaf(p, vv[i], acc[mm][i]);
                }
            }
        }
        // sum the KPG key streams of the wave (lanes that differ in ksub), then the waves in order
#pragma unroll
        for (int mm = 0; mm < 8; ++mm)
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                float v = acc[mm][i];
#pragma unroll
                for (int off = 32; off >= LPK; off >>= 1) v += __shfl_xor(v, off, kWave);
                acc[mm][i] = v;
            }
        if (ksub == 0) {
#pragma unroll
            for (int mm = 0; mm < 8; ++mm)
#pragma unroll
                for (int i = 0; i < 8; ++i) red[wave][mm][dg * 8 + i] = acc[mm][i];
        }
        __syncthreads();
        for (int idx = threadIdx.x; idx < 8 * DH; idx += 256) {
            int mm = idx / DH, e = idx - mm * DH;
            if (m0 + mm < M) {
                float o = ((red[0][mm][e] + red[1][mm][e]) + red[2][mm][e]) + red[3][mm][e];
                part[(((size_t)head * max_splits + split) * max_window + (m0 + mm)) * (DH + 2) + e] = o;
            }
        }
        if (threadIdx.x < 8 && m0 + threadIdx.x < M) {
            size_t base = (((size_t)head * max_splits + split) * max_window + (m0 + threadIdx.x)) * (DH + 2) + DH;
            part[base] = stat[threadIdx.x][0];
            part[base + 1] = stat[threadIdx.x][1];
        }
        __syncthreads();
    }
}

// Merge the splits of (row, head) in increasing split order.  Row r has keys in
// splits 0..(len + r) / kAttnSplit.  Writes att as fp32 and optionally as the
// split bf16 operand of the output projection.  grid: (M, n_heads), DH threads.
template <int DH>
__global__ __launch_bounds__(DH) void attn_combine_kernel(const float *__restrict__ part,
                                                           const int32_t *__restrict__ len_ptr, int n_heads,
                                                           int max_window, int max_splits, float *__restrict__ att,
                                                           bf16_t *__restrict__ atts, int cls)
{
    const int r = blockIdx.x, head = blockIdx.y, e = threadIdx.x;
    const int ns = (*len_ptr + r) / kAttnSplit + 1;
    const float *p = part + (((size_t)head * max_splits) * max_window + r) * (DH + 2);
    const size_t stride = (size_t)max_window * (DH + 2);
    float gm = kMasked;
    for (int s = 0; s < ns; ++s) gm = fmaxf(gm, p[s * stride + DH]);
    float o = 0.f, den = 0.f;
    for (int s = 0; s < ns; ++s) {
        float w = expf(p[s * stride + DH] - gm);
        o = fmaf(w, p[s * stride + e], o);
        den = fmaf(w, p[s * stride + DH + 1], den);
    }
    float v = o / den;
    const int d = n_heads * DH;
    att[(size_t)r * d + head * DH + e] = v;
    if (atts) {
        bf16_t hi = f32_to_bf16(v);
        atts[xp_offset(cls, r, head * DH + e, 0)] = hi;
        atts[xp_offset(cls, r, head * DH + e, 1)] = f32_to_bf16(v - bf16_to_f32(hi));
    }
}

// ------------------------------------------------------------------ SwiGLU

// a[r][i] = silu(gu[r][i]) * gu[r][F + i]    grid: (ceil(F/256), M)
__global__ __launch_bounds__(256) void swiglu_kernel(const float *__restrict__ gu, float *__restrict__ a,
                                                      int F)
{
    int r = blockIdx.y, i = blockIdx.x * 256 + threadIdx.x;
    if (i >= F) return;
    float g = gu[(size_t)r * 2 * F + i], u = gu[(size_t)r * 2 * F + F + i];
    float v = g / (1.0f + expf(-g)) * u;
    a[(size_t)r * F + i] = v;
}

// ------------------------------------------- argmax + acceptance + commit
//
// Block r finds argmax(logits[r]) (lowest index among equal maxima).  The last
// block to finish applies Algorithm 1's accept rule: a = longest prefix with
// window[i + 1] == pred[i]; next = pred[a]; the cache length advances by 1 + a
// (rejected rows are simply left beyond the length and overwritten later).
// result: [0] = a, [1] = next, [2..2+M) = pred.   grid: M blocks of 1024.
__global__ __launch_bounds__(1024) void argmax_accept_kernel(const float *__restrict__ logits, int V, int M,
                                                              const int32_t *__restrict__ window, int mode,
                                                              int32_t *__restrict__ result, int32_t *__restrict__ len_ptr,
                                                              uint32_t *__restrict__ counter)
{
    __shared__ float bv[16];
    __shared__ int bi[16];
    __shared__ bool last;
    const int r = blockIdx.x;
    const float *row = logits + (size_t)r * V;
    float best = -INFINITY;
    int besti = 0x7fffffff;
    for (int i = threadIdx.x; i < V; i += 1024) {
        float v = row[i];
        if (v > best || besti == 0x7fffffff) { best = v; besti = i; }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        float ov = __shfl_xor(best, off, kWave);
        int oi = __shfl_xor(besti, off, kWave);
        if (ov > best || (ov == best && oi < besti)) { best = ov; besti = oi; }
    }
    if ((threadIdx.x & 63) == 0) { bv[threadIdx.x >> 6] = best; bi[threadIdx.x >> 6] = besti; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 16; ++w)
            if (bv[w] > best || (bv[w] == best && bi[w] < besti)) { best = bv[w]; besti = bi[w]; }
        st_agent(result + 2 + r, (int32_t)besti);
        wait_stores();
        last = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == (uint32_t)(M - 1);
    }
    __syncthreads();
    if (last && threadIdx.x == 0) {
        const int32_t *pred = result + 2;
        int a = 0;
        if (mode == 0) {
            while (a < M - 1 && window[a + 1] == ld_agent(pred + a)) ++a;
        } else {
            a = M - 1;
        }
        result[0] = a;
        result[1] = ld_agent(pred + a);
        *len_ptr += 1 + a;
        st_agent(counter, 0u);
    }
}

// Acceptance over a draft tree, after argmax_accept_kernel has left the per-row predictions in
// result[2..] (run in APPEND mode on a copy of the length).  Row r > 0 is accepted iff its parent
// is and window[r] equals the prediction made at the parent; the deepest accepted row wins (lowest
// index among equally deep).  result[0] = its depth a, result[1] = the prediction at that row,
// result[34 + j] = the window row at depth j of the accepted path; length += 1 + a.   One thread.
__global__ void accept_tree_kernel(const int32_t *__restrict__ window, const int32_t *__restrict__ parent,
                                   const int32_t *__restrict__ depth, int M, int32_t *__restrict__ result,
                                   int32_t *__restrict__ len_ptr, int len_before)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    const int32_t *pred = result + 2;
    uint32_t acc = 1u;
    int best = 0;
    for (int r = 1; r < M; ++r) {
        const int p = parent[r];
        if (((acc >> p) & 1u) && window[r] == pred[p]) {
            acc |= 1u << r;
            if (depth[r] > depth[best]) best = r;
        }
    }
    const int a = depth[best];
    for (int r = best, j = a; j >= 0; --j, r = parent[r]) result[34 + j] = r;
    result[0] = a;
    result[1] = pred[best];
    *len_ptr = len_before + 1 + a;
}

// Generic-layout counterpart of kvf_compact_kernel.   grid: n_layers * 2 * n_heads blocks.
template <typename KT>
__global__ __launch_bounds__(128) void kv_compact_kernel(KT *__restrict__ pool, const int32_t *__restrict__ page_table,
                                                          const int32_t *__restrict__ result, int L, int n_layers, int n_heads,
                                                          int head_dim, int page_tokens)
{
    const int head = blockIdx.x % n_heads, kv = (blockIdx.x / n_heads) & 1, layer = blockIdx.x / (2 * n_heads);
    const int a = result[0];
    const int32_t *path = result + 34;
    for (int j = 1; j <= a; ++j) {
        const int src = L + path[j], dst = L + j;
        if (src != dst && (int)threadIdx.x < head_dim) {
            const size_t so = kv_offset(page_table[src / page_tokens], layer, n_layers, kv, head, n_heads, src % page_tokens,
                                        page_tokens, head_dim);
            const size_t dofs = kv_offset(page_table[dst / page_tokens], layer, n_layers, kv, head, n_heads, dst % page_tokens,
                                          page_tokens, head_dim);
            pool[dofs + threadIdx.x] = pool[so + threadIdx.x];
        }
        __syncthreads();
    }
}

// ----------------------------------------------------- cache import/export

// Copies n positions of one layer between fp32 [n][d] arrays and the cache.
template <typename KT, bool TO_CACHE>
__global__ __launch_bounds__(256) void kv_copy_kernel(KT *__restrict__ pool, const int32_t *__restrict__ page_table,
                                                       float *__restrict__ k, float *__restrict__ v, int pos0, int layer,
                                                       int n_layers, int n_heads, int head_dim, int page_tokens)
{
    const int r = blockIdx.x, pos = pos0 + r, d = n_heads * head_dim;
    const int page = page_table[pos / page_tokens], tip = pos % page_tokens;
    for (int e = threadIdx.x; e < d; e += 256) {
        int hd = e / head_dim, i = e - hd * head_dim;
        size_t ko = kv_offset(page, layer, n_layers, 0, hd, n_heads, tip, page_tokens, head_dim) + i;
        size_t vo = kv_offset(page, layer, n_layers, 1, hd, n_heads, tip, page_tokens, head_dim) + i;
        if (TO_CACHE) {
            store_kv(pool, ko, k[(size_t)r * d + e]);
            store_kv(pool, vo, v[(size_t)r * d + e]);
        } else {
            k[(size_t)r * d + e] = load_f32(pool, ko);
            v[(size_t)r * d + e] = load_f32(pool, vo);
        }
    }
}

}  // namespace anpd
