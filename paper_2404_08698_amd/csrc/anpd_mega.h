// The whole verification step as ONE persistent kernel (window class 8, d_model <= 4096).
//
// One 8-wave block per compute unit runs every phase of the step - embed, then
// per layer QKV / attention / O / gate-up / down, then LM head and argmax+accept
// (paper, Section 3.1 "Parallel Decoding" step 2; Algorithm 1) - separated by
// grid barriers.  Because the weights do not depend on activations, a block
// issues the loads of its first weight tile of the NEXT phase before it waits at
// a barrier, so HBM keeps streaming across phase boundaries and through the
// latency-bound attention phase; that is what separate launches cannot do.
//
// Blocks exchange activations through global memory with device-coherent
// accesses (write-through stores, loads served at the coherence point): the
// XCDs' L2 caches are not coherent with each other inside a launch, and
// cache-wide write-back / invalidate fences cost tens of microseconds here.
// The barrier is a two-level counter (groups of blocks, then one word every
// block polls); counters only grow, the host passes the epoch.  Waits are
// bounded: a block that gives up raises an error flag and every phase still
// runs to its end, so the grid always drains.
//
// The arithmetic of every phase is the code of the multi-kernel fast path
// (same tiles, same k-step assignment, same summation orders), so both paths
// give bit-identical results.
#pragma once
#include "anpd_fast.h"

namespace anpd {

struct LayerW {
    const uint4 *qkv, *o, *gu, *down;     // packed weights
    const bf16_t *attn_gain, *ffn_gain;
};

struct MegaArgs {
    const LayerW *layers;
    int n_layers;
    const uint4 *wp_lm;
    const bf16_t *final_gain, *embed;
    int d, F, V, n_heads, n_kv_heads, head_dim, M, mode;
    float inv_d, eps, scale;
    float *x;
    // Activation operands, one set per layer so that no address is written twice in a launch (see x_operand):
    // xp_layers + l * xp_stride holds, in this order, the QKV operand of layer l, the attention output, the
    // gate / up operand (d_model columns each) and the down projection's operand (d_ffn columns); the set after
    // the last layer holds the LM head's operand.  Sized for kMaxFrags fragments per k-step.
    bf16_t *xp_layers;
    size_t xp_stride;       // bf16 elements per layer
    bf16_t *qp;
    float *ssp_a, *ssp_b, *part;
    uint32_t *head_counter;
    bf16_t *pool;
    const int32_t *page_table;
    int32_t *len_ptr;
    const float2 *rope;
    int max_splits;
    float *logits;          // nullable: all logits [M][V]
    unsigned long long *amax;  // [V / 16][32] per-tile (value bits << 32 | index) of the best logit
    int32_t tok[16];        // the window's tokens, by value (no upload before the launch)
    int32_t *result;        // device: [0] accepted, [1] next, [2 + r] prediction of row r
    int32_t *host_result;   // pinned host memory, same layout: written at the end, read by the host after the launch
    uint32_t *row_counter;  // argmax phase hand-off
    uint32_t *bar;          // [0] = top counter, [kBarStride * (1 + g)] = group g
    uint32_t bar_epoch;     // barriers completed by earlier launches
    int32_t *error;         // pinned host memory: set to 1 if a barrier wait gave up
    int32_t spin_limit;     // polls before a barrier wait gives up
    uint32_t *qkv_ready;    // [n_heads] finished q / k / v tiles of the head, counted up over layers and launches
    uint32_t ready_epoch;   // QKV phases completed by earlier launches
    long long *trace;       // nullable: [grid][kTraceEvents] timestamps (100 MHz) at barrier arrive / wait-done
    // draft tree (multi-candidate verification), by value like the tokens: parent row, depth, and the
    // rows a row sees (itself and its ancestors) as a bit mask
    int32_t parent[8], depth[8];
    uint32_t mask[8];
    // several sequences in one step, by value as well: the sequences, the sequence of every row, and the
    // first attention task of every sequence (tasks run sequence by sequence: n_heads * splits each)
    SeqRef seqs[8];
    int32_t row_seq[8];
    int32_t task0[9];
    int32_t n_seq;
    int32_t n_att_blocks;    // (split, sequence) pairs per head
    int32_t *host_batch;     // pinned host memory: (accepted, next) of every sequence
};

constexpr int kTraceEvents = 1024;

// Cache policy of the activation-operand loads: at the coherence point (the operands of all layers share
// their addresses, see x_operand, so an XCD's L2 may hold the previous layer's version of a line).
constexpr int kAuxOperand = kAuxCoherent;
#ifndef ANPD_MEGA_STREAM_LDS
#define ANPD_MEGA_STREAM_LDS false
#endif

constexpr int kBarStride = 256;  // uint32 words between barrier counters (1 KiB: separate channels)
// embed, then attention / O / gate-up / down of every layer, then the LM head (the QKV phase hands over
// per head, not through the grid barrier)
constexpr int kMegaBarriers(int n_layers) { return 1 + 4 * n_layers + 1; }

struct GridBarrier {
    uint32_t *ctr;
    uint32_t done;   // barriers this block has arrived at, including earlier launches
    int32_t *error;
    int grp, gsize, ngroups;
    long long *trace;
    int n_ev;
    bool failed;     // (thread 0) a wait of this block gave up, or it saw the error flag: later waits do not spin
    int spin_limit;
};

template <typename ArgsPtr>
__device__ __forceinline__ void bar_init(GridBarrier &b, ArgsPtr a)
{
    b.ctr = a->bar;
    b.done = a->bar_epoch;
    b.error = a->error;
    b.ngroups = (gridDim.x % 8 == 0) ? 8 : 1;
    b.gsize = gridDim.x / b.ngroups;
    b.grp = blockIdx.x % b.ngroups;
    b.trace = a->trace ? a->trace + (size_t)blockIdx.x * kTraceEvents : nullptr;
    b.n_ev = 0;
    b.failed = false;
    b.spin_limit = a->spin_limit;
}

__device__ __forceinline__ void bar_stamp(GridBarrier &b)
{
    if (b.trace) {
        if (threadIdx.x == 0 && b.n_ev < kTraceEvents) b.trace[b.n_ev] = wall_clock64();
        b.n_ev += 1;
    }
}

// One thread per block calls it once every store of the phase that other blocks will read has
// been acknowledged (wait_stores() in the storing waves).  Counts arrival number b.done + 1.
__device__ __forceinline__ void bar_signal(const GridBarrier &b)
{
    uint32_t old = __hip_atomic_fetch_add(b.ctr + kBarStride * (1 + b.grp), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (old == (b.done + 1u) * (uint32_t)b.gsize - 1u)
        __hip_atomic_fetch_add(b.ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// All threads call it after their last store of the phase (phases without per-tile accounting).
__device__ __forceinline__ void bar_arrive(GridBarrier &b)
{
    bar_stamp(b);
    wait_stores();
    block_sync_lds();
    if (threadIdx.x == 0) bar_signal(b);
    b.done += 1;
}

// All threads call it before their first load of data produced in the previous phase.  Does not
// wait for this wave's outstanding loads (the weight prefetch stays in flight).
__device__ __forceinline__ void bar_wait(GridBarrier &b)
{
    if (threadIdx.x == 0 && !b.failed) {
        const uint32_t target = b.done * (uint32_t)b.ngroups;
        int spins = 0;
        while ((int32_t)(ld_agent(b.ctr) - target) < 0) {
            __builtin_amdgcn_s_sleep(4);
            ++spins;
            if ((spins & 4095) == 0 && ld_system(b.error) != 0) {   // some block has given up: stop waiting everywhere
                b.failed = true;
                break;
            }
            if (spins > b.spin_limit) {  // by default seconds: something is wrong, do not hang the GPU
                st_system(b.error, 1);
                b.failed = true;
                break;
            }
        }
    }
    block_sync_lds();
    bar_stamp(b);
}

// Bounded wait for a counter that only grows (same give-up rules as bar_wait).  Thread 0 only.
__device__ __forceinline__ void wait_count(GridBarrier &b, const uint32_t *p, uint32_t target)
{
    int spins = 0;
    while (!b.failed && (int32_t)(ld_agent(p) - target) < 0) {
        __builtin_amdgcn_s_sleep(4);
        ++spins;
        if ((spins & 4095) == 0 && ld_system(b.error) != 0) b.failed = true;
        if (spins > b.spin_limit) {
            st_system(b.error, 1);
            b.failed = true;
        }
    }
}

struct WSrc {
    const uint4 *Wp;
    int nks, n_tiles;
};

constexpr int kChunk = 8;   // k-steps per wave per pipeline item (half a tile when K = 4096)

// k-steps wave + 8 * (KC c + u), u = 0..KC-1, of tile `tile`.  Buffer loads: the descriptor covers exactly
// the tile's nks blocks, so k-steps past the end (and tiles that do not exist) read as zeros
// without a branch, and one offset register per thread serves every load.
template <int KC>
__device__ __forceinline__ void load_wchunk(uint4 (&w)[KC], const WSrc &s, int tile, int c, int wave, int lane)
{
    const bool have = tile < s.n_tiles;
    const uint4 *base = s.Wp + (size_t)(have ? tile : 0) * s.nks * 64;
    __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint4 *>(base), 0, have ? s.nks * 1024 : 0, 0x00020000);
    const int voff = (wave * 64 + lane) * 16;
#pragma unroll
    for (int u = 0; u < KC; ++u) {
        u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(r, voff, (KC * c + u) * kFastWaves * 1024, kAuxStream);
        w[u] = make_uint4(v.x, v.y, v.z, v.w);
    }
}

// Tiles are dealt out in rounds of one per block.  An incomplete last round goes to the even-numbered
// blocks first: blocks are placed on the eight XCDs in turn, and the odd XCDs are served about a tenth
// slower by the memory system (stand-alone streaming probe: equal work ends 10-12 % later there), so a
// round that does not reach every block should not end on them.
__device__ __forceinline__ int deal_rank()   // position of this block in an incomplete round
{
    const int b = blockIdx.x, grid = gridDim.x;
    return (b & 1) ? (grid + 1) / 2 + (b >> 1) : (b >> 1);
}
// Number of tiles of this block in a phase of n_tiles tiles, its tile number i, and its first tile
// (>= n_tiles if it has none).
__device__ __forceinline__ int block_tiles(int n_tiles)
{
    const int grid = gridDim.x;
    return n_tiles / grid + (deal_rank() < n_tiles % grid ? 1 : 0);
}
__device__ __forceinline__ int block_tile(int n_tiles, int i)
{
    const int grid = gridDim.x, full_rounds = n_tiles / grid;
    return i < full_rounds ? (int)blockIdx.x + i * grid : full_rounds * grid + deal_rank();
}
__device__ __forceinline__ int first_tile(const WSrc &s)
{
    return s.n_tiles >= (int)gridDim.x ? (int)blockIdx.x : deal_rank();
}

// The same k-steps of the activation operand, NF fragments each (Xp[k-step][fragment][lane]).
template <int NF, int KC>
__device__ __forceinline__ void load_xchunk(uint4 (&x)[NF][KC], const uint4 *Xp, int nks, int c, int wave, int lane, bool have = true)
{
    __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint4 *>(Xp), 0, have ? nks * NF * 1024 : 0, 0x00020000);
    const int voff = (wave * NF * 64 + lane) * 16;
#pragma unroll
    for (int u = 0; u < KC; ++u)
#pragma unroll
        for (int f = 0; f < NF; ++f) {
            u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(r, voff, ((KC * c + u) * kFastWaves * NF + f) * 1024, kAuxOperand);
            x[f][u] = make_uint4(v.x, v.y, v.z, v.w);
        }
}

// Epilogue operands of a block's first tiles, staged in LDS by the wave that will finish the
// tile.  They do not depend on the previous phase (a weight vector, tables of the step, and the
// residual rows this same block wrote), so they are requested before the phase barrier and are
// there when the epilogue runs: a load issued at the epilogue would queue behind the weight
// loads in flight, and the gain vector comes from HBM.
// (the residual epilogue and the QKV epilogues need different operands and never run in the same phase)
constexpr int pre_tiles(int nf) { return nf == 1 ? 3 : 1;}   // tiles per block whose epilogue operands are staged
constexpr int kMaxFrags = 2;   // activation fragments per k-step the one-kernel step is built for (windows of up to 16 rows)
struct EpiPreLds {
    union {
        struct { f32x4 x[64], g[64]; } res;
        struct { float2 cs[4][64]; int page[64]; } qkv;
    };
};
template <int EPI>
__device__ __forceinline__ void pre_to_lds(EpiPreLds &d, const EpiPre &p, int lane)
{
    if (EPI == EPI_RESIDUAL) {
        d.res.x[lane] = p.x;
        d.res.g[lane] = p.g;
    } else if (epi_is_qkv(EPI)) {
#pragma unroll
        for (int i = 0; i < 4; ++i) d.qkv.cs[i][lane] = p.cs[i];
        d.qkv.page[lane] = p.page;
    }
}
template <int EPI>
__device__ __forceinline__ void pre_from_lds(EpiPre &p, const EpiPreLds &d, int lane)
{
    if (EPI == EPI_RESIDUAL) {
        p.x = d.res.x[lane];
        p.g = d.res.g[lane];
    } else if (epi_is_qkv(EPI)) {
#pragma unroll
        for (int i = 0; i < 4; ++i) p.cs[i] = d.qkv.cs[i][lane];
        p.page = d.qkv.page[lane];
    }
}

// NF: operand fragments per k-step (see gemm_phase).  With NF > 1 the partial tiles have one buffer instead of
// two and the epilogue operands of one tile instead of three are staged, which leaves room for the second
// chunk of the resident operand (x1: per wave its KC k-steps x NF fragments).
template <int NF>
struct MegaShared {
    static constexpr int kRedBufs = NF == 1 ? 2 : 1;
    union {
        float red[kRedBufs][kFastWaves][NF][256];
        AttnShared<128> attn128;
        AttnShared<64> attn64;
    };
    float rinv[32];
    int tiles_done;   // epilogues finished by this block since the kernel started
    EpiPreLds pre[pre_tiles(NF)][NF];
    float rscratch[2048];   // group sums of the RMSNorm partials (see rinv_partial_to_lds)
    union {
        uint4 x1[NF == 1 ? 1 : kFastWaves * NF * kChunk * 64];
        AttnStash stash;   // attention phase only: no GEMM operand is staged while it runs
    };
};

template <int DH, int NF>
__device__ __forceinline__ AttnShared<DH> &attn_shared(MegaShared<NF> &sh)
{
    if constexpr (DH == 128) return sh.attn128;
    else return sh.attn64;
}

// One fragment (16 bytes per lane) from LDS, as assembly: the compiler does not see the read, so it does not
// make it wait for loads in flight that write LDS.  The caller waits (lds_wait) before it uses the value.
template <int OFF>
__device__ __forceinline__ u32x4_t lds_frag(uint32_t addr)
{
    u32x4_t v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
    return v;
}
// fragment number i (compile-time after unrolling) of a wave's chunk in LDS
__device__ __forceinline__ u32x4_t lds_frag_at(uint32_t addr, int i)
{
    u32x4_t v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "i"(i * 1024) : "memory");
    return v;
}
// Waits until at most PENDING of this wave's LDS reads are outstanding; the fragments are operands so that
// nothing that uses them is moved in front of the wait.
template <int PENDING, int NF>
__device__ __forceinline__ void lds_wait(u32x4_t (&t)[NF])
{
    static_assert(NF <= 2, "operand list written for at most two fragments");
    if constexpr (NF == 1) asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(t[0]) : "n"(PENDING));
    else asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(t[0]), "+v"(t[1]) : "n"(PENDING));
}
// A chunk of the activation operand straight into LDS (no registers while in flight): fragment (u, f) of this
// wave goes to dst[(u * NF + f) * 64 + lane].
template <int NF, int KC>
__device__ __forceinline__ void dma_xchunk(uint4 *dst, const uint4 *Xp, int nks, int c, int wave, int lane, bool have = true)
{
    __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint4 *>(Xp), 0, have ? nks * NF * 1024 : 0, 0x00020000);
    const int voff = (wave * NF * 64 + lane) * 16;
#pragma unroll
    for (int u = 0; u < KC; ++u)
#pragma unroll
        for (int f = 0; f < NF; ++f)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (__attribute__((address_space(3))) void *)(dst + (u * NF + f) * 64), 16, voff,
                                                     ((KC * c + u) * kFastWaves * NF + f) * 1024, 0, kAuxOperand);
}

// One GEMM phase.  On entry pf holds (or has in flight) the weights of this block's first work
// item, loaded by the previous phase; on exit those of the next phase's first item are in flight
// (issued after this block has arrived at the phase barrier, so the arrival does not wait for them).
// A work item is a chunk of KC k-steps per wave of one tile.
// STATIONARY: K needs at most two chunks; the activation operand stays in registers for all tiles.
// BARRIER = false (QKV): the phase does not end in a grid barrier; its consumers wait for per-head tile
// counts (a.ready).  The barrier's counters assume that no block is more than one barrier ahead of
// another, so a barrier that is not waited for must not be signalled either.
// NF: fragments of the activation operand per k-step, each holding 8 window rows as (hi | lo) slots like
// the one fragment of a window of up to 8 rows, so rows 8 f .. 8 f + 7 go through exactly the arithmetic
// of that window.  NF = 2 (9 to 16 rows) doubles the operand; with both of its chunks and a ring of weight
// items in registers the kernel spilled 70 to 160 registers per lane around the epilogues, and a reload from
// scratch memory queues behind the weights in flight (7B shape, 9 rows: 4.33 ms against 3.39 ms as separate
// launches).  So the second of the two operand buffers lives in LDS: requested straight into LDS (no
// registers while in flight) and read fragment by fragment next to the MFMAs that use it.  In a stationary
// phase that is chunk 1 of the operand; in a streaming phase (down projection) the chunks of the odd steps.
// KC: k-steps per wave per item; 2 KC * 8 k-steps must cover d_model for the stationary phases (8 up to
// d_model 4096, 10 up to 5120).
template <int EPI, bool STATIONARY, bool BARRIER = true, int NF = 1, int KC = kChunk>
__device__ __forceinline__ void gemm_phase(const FastArgs &a, const WSrc &next, uint4 (&pf)[KC], MegaShared<NF> &sh,
                                           GridBarrier &bar, int &tiles_before)
{
    // weight items in flight per wave, and how many steps ahead a streamed operand chunk is requested
    // kStreamLds: a streaming phase with NF > 1 passes the chunks of its odd steps through LDS and keeps a ring
    // of three.  Otherwise it has a ring of two and ONE operand buffer in registers, refilled for the next step
    // as soon as a step's MFMAs have read it (with two items in flight the operand of step s + 1 may be
    // requested behind the weights of step s + 1 without holding anything back: a wave's loads return in order).
    constexpr bool kStreamLds = ANPD_MEGA_STREAM_LDS;
    constexpr int RING = NF == 1 ? (KC <= 8 ? 3 : 2) : ((STATIONARY || kStreamLds) ? 3 : 2);
    constexpr int XLOOK = (NF > 1 && !STATIONARY && !kStreamLds) ? 1 : 2;
    constexpr bool kX1Lds = NF > 1 && (STATIONARY || kStreamLds);   // the second operand buffer (x1) lives in LDS
    static_assert(NF == 1 || KC == kChunk, "the LDS copy of the operand is sized for items of kChunk k-steps");
    const int tid = fresh_tid();
    const int lane = tid & 63, wave = tid >> 6;
    const WSrc cur = {a.Wp, a.nks, a.n_tiles};
    const int n_chunks = (((a.nks + kFastWaves - 1) / kFastWaves) + KC - 1) / KC;
    const int my_tiles = block_tiles(cur.n_tiles);
    auto tile_at = [&](int i) { return block_tile(cur.n_tiles, i); };
    const int tiles_after = tiles_before + my_tiles;
    // Waves that finish tiles in this phase have stores to wait for at its end; they fetch their share
    // of the next phase's first weights only after that wait, so the wait stays short.
    const bool reducer = wave < my_tiles;
    uint4 wb[KC], wc[KC], x0[NF][KC], x1[NF][KC];   // (wc is unused with a ring of two)

    // work items of this block: (tile, chunk) in order; pf holds item 0, wb (and wc) the one(s) after it
    int ti = 0, c = 0;     // item being computed: chunk c of the block's tile number ti
    int li = 0, lc = 0;    // last item whose weights have been requested
    bool next_issued = false;         // the next phase's first chunk has been requested
    // may_cross: the request may go to the next phase's first chunk when this phase has nothing left
    // (only on entry: later it would sit in front of the last epilogue's stores)
    // Every call issues KC loads, also past the block's last item (an empty descriptor: zeros, nothing
    // is fetched): the compiler counts the loads issued after the ones it waits for, and a request that
    // may or may not have been made counts as not made, which turns every wait into a wait for all loads.
    auto fetch = [&](uint4 (&dst)[KC], bool may_cross) {
        if (++lc == n_chunks) { lc = 0; ++li; }
        if (may_cross && !(li < my_tiles) && !next_issued && !reducer) {
            load_wchunk<KC>(dst, next, first_tile(next), 0, wave, lane);
            next_issued = true;
        } else {
            load_wchunk<KC>(dst, cur, li < my_tiles ? tile_at(li) : cur.n_tiles, lc, wave, lane);
        }
    };
    constexpr bool kHasPre = (EPI == EPI_RESIDUAL || epi_is_qkv(EPI));
    constexpr int kPreTiles = pre_tiles(NF);
    const bool stages = kHasPre && wave < kPreTiles && wave < my_tiles;   // this wave finishes tile number `wave`
    EpiPre pre0[NF];
    if (stages) {
#pragma unroll
        for (int f = 0; f < NF; ++f) epilogue_preload<EPI>(a, tile_at(wave), lane, pre0[f], f);
    }
    if constexpr (RING == 3) {
        fetch(wb, false);
        fetch(wc, true);
    } else {
        fetch(wb, true);
    }
    // at most RING - 1 items: the last buffer of the ring holds the next phase's first item (the same for
    // a whole wave: told to the compiler, or it takes everything a step does under this flag for lane-dependent)
    const bool cross_last = __builtin_amdgcn_readfirstlane((int)next_issued) != 0;
    if (stages) {
#pragma unroll
        for (int f = 0; f < NF; ++f) pre_to_lds<EPI>(sh.pre[wave][f], pre0[f], lane);
    }

    bar_wait(bar);
    if (BARRIER && my_tiles == 0 && tid == 0) bar_signal(bar);
    // STATIONARY: both chunks of the operand stay in x0 / x1.  Otherwise x0 / x1 alternate: a step's MFMAs
    // free one of them, and the operand chunk of the step after next is requested into it right away,
    // BEFORE the weights requested at the end of the step, so that no step's operand waits behind
    // weights of later steps (a wave's loads return in order).
    const int n_steps = my_tiles * n_chunks;
    uint4 *const x1_lds = sh.x1 + (kX1Lds ? wave * NF * KC * 64 : 0);
    // (chunk 1 goes straight into LDS; the block's first step waits for it, see do_step)
    if (kX1Lds) dma_xchunk<NF, KC>(x1_lds, a.Xp, a.nks, STATIONARY ? 1 : 1 % n_chunks, wave, lane, STATIONARY || 1 < n_steps);
    load_xchunk<NF, KC>(x0, a.Xp, a.nks, 0, wave, lane);
    if (!kX1Lds && XLOOK == 2 && (STATIONARY || 1 < n_steps))
        load_xchunk<NF, KC>(x1, a.Xp, a.nks, STATIONARY ? 1 : 1 % n_chunks, wave, lane);
    // the RMSNorm scale is needed by the first epilogue only: its partial sums are requested here and
    // reduced after the first tile's MFMAs, off the path from the barrier to the first MFMA
    constexpr bool kNorm = (epi_has_norm(EPI) || EPI == EPI_LM_ARGMAX);
    const bool late_norm = kNorm && a.n_ss <= 256 && my_tiles > 0;
    float nv[NF][4];
    if (late_norm) rinv_issue<true, NF>(a, nv, tid);
    else if (kNorm) compute_rinv<true>(a, sh.rinv, sh.rscratch);

    f32x4 acc[NF];
#pragma unroll
    for (int f = 0; f < NF; ++f) acc[f] = (f32x4){0.f, 0.f, 0.f, 0.f};
    int it = 0;
    int step = 0;
    // The weight buffers form a ring: a step multiplies the oldest buffer and requests the item RING steps
    // ahead into the same registers, so RING items stay in flight per wave.  (Passing the items down a
    // chain pf <- wb <- wc by value makes every step wait for the load it has just issued.)
    // xs: the operand buffer of this step when the operand is streamed (x0 and x1 in turn).
    // active: the block still has an item for this step.  The loop has one exit, at its top, and every
    // step issues the same number of loads whether it is active or not (empty descriptors once the items
    // have run out): with several exits, or requests made on some paths only, the compiler must assume
    // that the buffer a step waits for was requested last, and makes every step wait for all loads.
    // keep: buf holds the next phase's first item and is not refilled.
    // the MFMAs of one item against an operand chunk in registers / in this wave's LDS buffer (fragments read
    // one k-step ahead of the MFMAs that use them)
    auto mfma_reg = [&](uint4 (&buf)[KC], uint4 (&xr)[NF][KC]) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < KC; ++u)
#pragma unroll
            for (int f = 0; f < NF; ++f)
                acc[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, buf[u]),
                                                                 __builtin_bit_cast(bf16x8, xr[f][u]), acc[f], 0, 0, 0);
    };
    auto mfma_lds = [&](uint4 (&buf)[KC]) __attribute__((always_inline)) {
        const uint32_t xa = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void *)x1_lds + (uint32_t)lane * 16;
        u32x4_t t[2][NF];
#pragma unroll
        for (int f = 0; f < NF; ++f) t[0][f] = lds_frag_at(xa, f);
#pragma unroll
        for (int u = 0; u < KC; ++u) {
            if (u + 1 < KC) {
#pragma unroll
                for (int f = 0; f < NF; ++f) t[(u + 1) & 1][f] = lds_frag_at(xa, (u + 1) * NF + f);
                lds_wait<NF>(t[u & 1]);
            } else {
                lds_wait<0>(t[u & 1]);
            }
#pragma unroll
            for (int f = 0; f < NF; ++f)
                acc[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, buf[u]),
                                                                 __builtin_bit_cast(bf16x8, t[u & 1][f]), acc[f], 0, 0, 0);
        }
    };
    // from_lds (streaming phases with kX1Lds): this step's operand chunk is the one in LDS
    auto do_step = [&](uint4 (&buf)[KC], uint4 (&xs)[NF][KC], bool active, bool keep, bool from_lds = false) __attribute__((always_inline)) {
        if (active) {
            if (STATIONARY) {
                if (c == 1) {
                    if constexpr (kX1Lds) mfma_lds(buf);
                    else mfma_reg(buf, x1);
                } else {
                    mfma_reg(buf, x0);
                }
            } else if (kX1Lds && from_lds) {
                // The chunk was requested into LDS two steps ago (or on entry).  The reads below are assembly the
                // compiler does not connect with that request, and it places the requests into LDS among the
                // register loads around them as it sees fit: counting the loads that the source issues after the
                // request proves nothing (it let a step read a fragment before it had arrived, one tile in some
                // ten thousand).  So the wait is for everything this wave has requested, the next step's weights
                // and operand included.
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                mfma_lds(buf);
            } else {
                mfma_reg(buf, xs);
            }
        }
        if (!STATIONARY) {
            if (kX1Lds && from_lds)
                dma_xchunk<NF, KC>(x1_lds, a.Xp, a.nks, (step + XLOOK) % n_chunks, wave, lane, active && step + XLOOK < n_steps);
            else
                load_xchunk<NF, KC>(xs, a.Xp, a.nks, (step + XLOOK) % n_chunks, wave, lane, active && step + XLOOK < n_steps);
        }
        if constexpr (STATIONARY && kX1Lds) {
            // Chunk 1 of the operand was requested into LDS when the phase began and is first read in the block's
            // second step.  That the source requests it before chunk 0, which has arrived, proves nothing (see
            // below: the compiler interleaves the two): wait here, before this step's refill goes out, when all
            // that is outstanding besides it are the weights of the next two steps and the norm's partial sums -
            // all of it needed in a moment anyway.
            if (step == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
        if (!keep) fetch(buf, false);
        if (active) {
            ++step;
            const bool tile_done = (c == n_chunks - 1);
            const int finished = tile_at(ti);
            if (++c == n_chunks) { c = 0; ++ti; }
            if (tile_done) {
                float *r = &sh.red[MegaShared<NF>::kRedBufs == 2 ? (it & 1) : 0][0][0][0];
                if (MegaShared<NF>::kRedBufs == 1) block_sync_lds();   // the previous tile's partial sums have been read
#pragma unroll
                for (int f = 0; f < NF; ++f)
                    *reinterpret_cast<f32x4 *>(r + (((size_t)wave * NF + f) * 64 + lane) * 4) = acc[f];
                if (late_norm && it == 0) rinv_partial_to_lds<NF>(nv, sh.rscratch, tid);
                block_sync_lds();
                if (late_norm && it == 0) rinv_from_lds<NF>(a, sh.rinv, sh.rscratch, tid);   // wave 0, which also finishes tile 0
                if (wave == (it & (kFastWaves - 1))) {
                    if (kHasPre && it < kPreTiles) {
                        EpiPre pre[NF];
#pragma unroll
                        for (int f = 0; f < NF; ++f) pre_from_lds<EPI>(pre[f], sh.pre[it][f], lane);
                        reduce_and_finish_packed<NF, EPI, true>(a, finished, r, kFastWaves, lane, sh.rinv, pre);
                    } else {
                        reduce_and_finish_packed<NF, EPI, true>(a, finished, r, kFastWaves, lane, sh.rinv);
                    }
                }
#pragma unroll
                for (int f = 0; f < NF; ++f) acc[f] = (f32x4){0.f, 0.f, 0.f, 0.f};
#ifdef ANPD_TRACE_FINE
                if (it == 0) bar_stamp(bar);   // the first tile's epilogue has been issued
#endif
                ++it;
            }
        }
    };
    // The loop is entered with the operand in registers (it is the youngest request, so the weight
    // items have arrived as well): inside the loop the compiler then sees that the buffer a step needs has
    // younger requests behind it and lets those stay in flight.
#pragma unroll
    for (int f = 0; f < NF; ++f)
#pragma unroll
        for (int u = 0; u < KC; ++u) {
            u32x4_t t0 = __builtin_bit_cast(u32x4_t, x0[f][u]);
            asm volatile("" : "+v"(t0));
            x0[f][u] = __builtin_bit_cast(uint4, t0);
            if (!kX1Lds && XLOOK == 2) {
                u32x4_t t1 = __builtin_bit_cast(u32x4_t, x1[f][u]);
                asm volatile("" : "+v"(t1));
                x1[f][u] = __builtin_bit_cast(uint4, t1);
            }
        }
#ifdef ANPD_TRACE_FINE
    bar_stamp(bar);   // the operand has arrived
#endif
    if constexpr (RING == 3) {
        while (ti < my_tiles) {
            do_step(pf, x0, true, false);
            do_step(wb, x1, ti < my_tiles, false, true);
            do_step(wc, x0, ti < my_tiles, cross_last);
            if (!STATIONARY) {   // three weight buffers, two operand buffers: the pattern repeats after six steps
                do_step(pf, x1, ti < my_tiles, false, true);
                do_step(wb, x0, ti < my_tiles, false);
                do_step(wc, x1, ti < my_tiles, cross_last, true);
            }
        }
        if (cross_last) {   // the next phase expects its first item in pf
#pragma unroll
            for (int u = 0; u < KC; ++u) pf[u] = wc[u];
        }
    } else {
        while (ti < my_tiles) {
            do_step(pf, x0, true, false);
            do_step(wb, XLOOK == 2 ? x1 : x0, ti < my_tiles, cross_last, true);
        }
        if (cross_last) {
#pragma unroll
            for (int u = 0; u < KC; ++u) pf[u] = wb[u];
        }
    }
#ifdef ANPD_TRACE_FINE
    if (my_tiles == 0) { bar_stamp(bar); }   // (keeps the number of stamps per phase fixed)
#endif
    // Order in this compute unit's memory queue at the end of a phase: the last epilogue's stores,
    // then the other waves' first chunk of the next phase, then (after the acknowledgement) the
    // barrier signal, and only then the rest of the next phase's requests.
    block_sync_lds();                       // the last epilogue's stores have been issued
    if (!reducer && !next_issued) load_wchunk<KC>(pf, next, first_tile(next), 0, wave, lane);
    if (reducer) {
        // this wave's epilogue stores must be out before the block counts its tiles as done; the wave
        // that completes the block's count signals the grid barrier
        wait_stores();
        if (BARRIER) {
            const int mine = (my_tiles - 1 - wave) / kFastWaves + 1;
            if (lane == 0 && atomicAdd(&sh.tiles_done, mine) + mine == tiles_after) bar_signal(bar);
        }
        if (epi_is_qkv(EPI) && a.ready && lane == 0) {
            // the attention tasks of a head wait for its 3 * head_dim / 16 tiles only (its own q tiles and the
            // k and v tiles of its key / value head), not for the whole grid: a k or v tile counts for every
            // query head of its group
            const int Tq = a.n_heads * a.head_dim / 16, Tkv = a.n_kv_heads * a.head_dim / 16, tph = a.head_dim / 16;
            const int grp = a.n_heads / a.n_kv_heads;
            for (int i = wave; i < my_tiles; i += kFastWaves) {
                const int t = tile_at(i);
                if (t < Tq) {
                    __hip_atomic_fetch_add(a.ready + kCounterStride * (t / tph), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                } else {
                    const int kvh = ((t - Tq) % Tkv) / tph;
                    for (int h = kvh * grp; h < (kvh + 1) * grp; ++h)
                        __hip_atomic_fetch_add(a.ready + kCounterStride * h, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        }
        load_wchunk<KC>(pf, next, first_tile(next), 0, wave, lane);
    }
    if (BARRIER) block_sync_lds();          // the block's signal (if it was this block's turn) has been issued
    if (BARRIER) {
        tiles_before = tiles_after;
        bar.done += 1;
    }
    bar_stamp(bar);
}

// The kernel's arguments stay in the kernarg segment.  Every phase reads the fields it needs
// through a pointer the optimiser cannot see through, so nothing read for one phase stays in
// registers across the others (kept live, these values push the weight pipeline into scratch
// memory, and a scratch reload queues behind the weight loads in flight).
typedef const MegaArgs __attribute__((address_space(4))) *MegaArgsK;

// The four activation operands of layer l (which = 0 QKV, 1 attention output, 2 gate / up, 3 down); the LM
// head's operand is set n_layers' first.  xp_stride = 0: every layer uses the same set.  (With a set per
// layer a compute unit's L2 cannot hold an older version of a line, and consumers could read through their
// XCD's L2 instead of at the coherence point: that gained nothing measurable, and writing 48 MB of lines
// that come round once per step cost 0.6 % of the step at 640 cached positions and 1.6 % at 2048, 7B shape.)
__host__ __device__ __forceinline__ size_t x_operand_elems(int columns) { return (size_t)((columns + 31) / 32) * kMaxFrags * 512; }
__device__ __forceinline__ bf16_t *x_operand(MegaArgsK g, int l, int which)
{
    return g->xp_layers + (size_t)l * g->xp_stride + (size_t)which * x_operand_elems(g->d);
}
typedef const LayerW __attribute__((address_space(4))) *LayerWK;
__device__ __forceinline__ MegaArgsK phase_args()
{
    MegaArgsK p = (MegaArgsK)__builtin_amdgcn_kernarg_segment_ptr();
    asm volatile("" : "+s"(p));
    return p;
}
__device__ __forceinline__ LayerW layer_weights(MegaArgsK g, int l)
{
    LayerWK t = (LayerWK)g->layers + l;   // the table is not written while the kernel runs
    LayerW w;
    w.qkv = t->qkv; w.o = t->o; w.gu = t->gu; w.down = t->down;
    w.attn_gain = t->attn_gain; w.ffn_gain = t->ffn_gain;
    return w;
}
template <int NF>
__device__ __forceinline__ FastArgs base_args(MegaArgsK g)
{
    FastArgs a = {};
    a.M = g->M;
    a.cls = packed_class(NF);
    a.inv_d = g->inv_d;
    a.eps = g->eps;
    a.n_ss = g->d / 16;
    a.d = g->d;
    a.x = g->x;
    a.pool = g->pool;
    a.page_table = g->page_table;
    a.len_ptr = g->len_ptr;
    a.rope = g->rope;
    a.n_layers = g->n_layers;
    a.n_heads = g->n_heads;
    a.n_kv_heads = g->n_kv_heads;
    a.head_dim = g->head_dim;
    a.qp = g->qp;
    return a;
}

// An attention task: (head, split) and the cache it works on.
struct AttTask {
    int head, split, L, rows, row0;
    const bf16_t *pool;
    const int32_t *table;
};
// Task t of the list that the blocks share out by turns: the last splits of a long context are the large
// ones and go first.  Several sequences: tasks run sequence by sequence, every sequence has a multiple of
// n_heads of them.
template <bool BATCH>
__device__ __forceinline__ AttTask attention_task(MegaArgsK g, int L, int t)
{
    const int n_heads = g->n_heads;
    AttTask k;
    if (BATCH) {
        int s = 0;
        while (s + 1 < g->n_seq && t >= g->task0[s + 1]) ++s;
        const int local = t - g->task0[s];
        k.L = *g->seqs[s].len_ptr;
        k.rows = g->seqs[s].n_rows;
        k.head = local % n_heads;
        k.split = n_splits_of(k.L + k.rows) - 1 - local / n_heads;
        k.row0 = g->seqs[s].row0;
        k.pool = g->seqs[s].pool;
        k.table = g->seqs[s].page_table;
    } else {
        k.head = t % n_heads;
        k.split = n_splits_of(L + g->M) - 1 - t / n_heads;
        k.L = L;
        k.rows = g->M;
        k.row0 = 0;
        k.pool = g->pool;
        k.table = g->page_table;
    }
    return k;
}
// The block's tasks in the order it runs them: every grid-th task of the list.  (Sharing a head's splits out
// among its blocks by size, longest first, was measured slower at every length: 2.62 against 2.60 ms per step
// at 512 positions, 3.25 against 3.18 at 4096, 7B shape.)
template <bool BATCH>
struct AttQueue {
    int t, n_tasks, grid;
    __device__ __forceinline__ AttQueue(MegaArgsK g, int L, int grid_)
    {
        grid = grid_;
        n_tasks = BATCH ? g->task0[g->n_seq] : g->n_heads * n_splits_of(L + g->M);
        t = blockIdx.x;
    }
    __device__ __forceinline__ bool have() const { return t < n_tasks; }
    __device__ __forceinline__ AttTask current(MegaArgsK g, int L) const { return attention_task<BATCH>(g, L, t); }
    __device__ __forceinline__ void advance() { t += grid; }
};

// MODE 1 (tree): the window is a draft tree (see MegaArgs::parent): rotary positions by depth, attention
// over ancestors only, acceptance along the paths.  MODE 2 (batch): the window holds several sequences
// side by side (MegaArgs::seqs): cache, length and position per row, attention per sequence, acceptance
// inside every sequence.  Separate instantiations, so the chain form keeps its registers.
// NF, KC: see gemm_phase (NF = 2: windows of 9 to 16 rows; KC = 10: d_model up to 5120).
enum { MEGA_CHAIN = 0, MEGA_TREE = 1, MEGA_BATCH = 2 };
template <int DH, int MODE = MEGA_CHAIN, int NF = 1, int KC = kChunk>
__global__ __launch_bounds__(kFastThreads) void verify_mega_kernel(MegaArgs /* read through phase_args() */)
{
    constexpr bool TREE = MODE == MEGA_TREE, BATCH = MODE == MEGA_BATCH;
    __shared__ MegaShared<NF> sh;
    __shared__ float bval[kFastWaves];
    __shared__ int bidx[kFastWaves];
    __shared__ bool last_row;
    const int grid = gridDim.x;
    GridBarrier bar;
    int tiles_before = 0, L, n_layers;
    uint4 pf[KC];
    {
        MegaArgsK g = phase_args();
        bar_init(bar, g);
        bar_stamp(bar);
        L = BATCH ? 0 : __builtin_amdgcn_readfirstlane(*g->len_ptr);   // (scalar: split and page indices derive from it)
        n_layers = g->n_layers;
        if (threadIdx.x == 0) sh.tiles_done = 0;   // ordered by the first block barrier below
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        const int d = g->d;
        const LayerW w0 = layer_weights(g, 0);
        {   // weights of the first QKV tile go out before anything else
            WSrc first = {w0.qkv, (d + 31) / 32, (d + 2 * g->n_kv_heads * g->head_dim) / 16};
            load_wchunk<KC>(pf, first, first_tile(first), 0, wave, lane);
        }
        // ---- embed (+ operand and sums of squares for the first norm)
        FastArgs a = base_args<NF>(g);
        a.gain = w0.attn_gain;
        a.xp_next = x_operand(g, 0, 0);
        a.ssp_next = g->ssp_a;
        if (wave == 0)
            // (the block that owns a tile of the residual stream here owns it in the O and down phases too)
            for (int i = 0; i < block_tiles(d / 16); ++i) embed_tile<true>(g->embed, (const int32_t *)g->tok, a, block_tile(d / 16, i), lane);
        bar_arrive(bar);
    }
    for (int l = 0; l < n_layers; ++l) {
        {   // QKV (+ norm, RoPE, cache write); then the O tile is put in flight
            MegaArgsK g = phase_args();
            const LayerW w = layer_weights(g, l);
            FastArgs a = base_args<NF>(g);
            const int nks_d = (g->d + 31) / 32;
            a.Wp = w.qkv; a.Xp = (const uint4 *)x_operand(g, l, 0); a.nks = nks_d;
            a.n_tiles = (g->d + 2 * g->n_kv_heads * g->head_dim) / 16;
            a.ssp = g->ssp_a; a.layer = l; a.ready = g->qkv_ready;
            if (TREE) a.depth = (const int32_t *)g->depth;
            if (BATCH) {
                a.seqs = (const SeqRef *)g->seqs;
                a.row_seq = (const int32_t *)g->row_seq;
            }
            WSrc none = {w.o, nks_d, 0};   // the O tile is requested by the attention phase
            gemm_phase<BATCH ? EPI_QKV_BATCH : (TREE ? EPI_QKV_TREE : EPI_QKV), true, false, NF, KC>(a, none, pf, sh, bar, tiles_before);
        }
        {   // attention: (head, split) tasks - per sequence when the step holds several; the O weights stream
            // in meanwhile.  Cache pages wholly below the committed length do not depend on this step: the
            // first task's page is requested before the barrier.
            MegaArgsK g = phase_args();
            const LayerW w = layer_weights(g, l);
            const int tid = fresh_tid();
            const int lane = tid & 63, wave = tid >> 6;
            const int M = g->M, n_heads = g->n_heads;
            const int grp = n_heads / g->n_kv_heads;
            typedef AttTask Task;
            AttQueue<BATCH> queue(g, L, grid);
            const int n_tasks = queue.n_tasks;
            auto have = [&]() { return queue.have(); };
            auto current = [&]() { return queue.current(g, L); };
            auto advance = [&]() { queue.advance(); };
            // the first task's pages are requested now, during the wait for the head: page 0 into registers, pages 1
            // and 2 into LDS.  (Requested when the QKV phase starts instead, the pages cost that phase more than
            // they save this one: 7B shape, 3.266 against 3.248 ms per step at 4096 positions, 2.627 against 2.618 at 512.)
            AttnKV<DH> kv;
            kv.loaded = false;
            bool stashed1 = false, stashed2 = false, q_in_lds = false;
            // (the RMSNorm scratch is idle between the QKV and the gate / up phase: room for the query rows)
            static_assert(sizeof(sh.rscratch) >= (DH / 32) * 64 * sizeof(uint4), "query rows of one row group");
            uint4 *const q_lds = reinterpret_cast<uint4 *>(sh.rscratch);
            if (have()) {
                const Task k = current();
                const int np = split_pages(k.split);
                const AttnPageIds ids = attn_page_ids(k.split, k.L, k.rows, k.table);
                attn_load_kv<DH, true>(kv, k.head / grp, k.split, k.L, k.rows, k.pool, k.table, l, n_layers, g->n_kv_heads, true, 0, &ids);
                if (np > 1) stashed1 = attn_park<DH>(sh.stash, 0, k.head / grp, k.split, k.L, k.pool, k.table, l, n_layers, g->n_kv_heads, 1, &ids);
                if (np > 2) stashed2 = attn_park<DH>(sh.stash, 1, k.head / grp, k.split, k.L, k.pool, k.table, l, n_layers, g->n_kv_heads, 2, &ids);
            }
            // The first O tile's weights go out now, behind the pages: requested inside the tasks they would
            // either queue in front of a task's own loads or still be in flight when the task waits for its
            // stores (one counter covers a wave's loads and stores).  The wait for the head below is longer
            // than their way from memory.
            const WSrc o_src = {w.o, (g->d + 31) / 32, g->d / 16};
            load_wchunk<KC>(pf, o_src, first_tile(o_src), 0, wave, lane);
            // No grid barrier here: a task needs the q / k / v tiles of its own head only, and every
            // block still arrives at the barrier that ends this phase after its QKV tiles, which is
            // what the O phase waits for.
            if (tid == 0) {
                const uint32_t target = (uint32_t)(3 * g->head_dim / 16) * (g->ready_epoch + (uint32_t)l + 1u);
                // (with the grid a multiple of the head count all of a block's tasks wait for the same head)
                if (grid % n_heads == 0) {
                    if (have()) wait_count(bar, g->qkv_ready + kCounterStride * ((int)blockIdx.x % n_heads), target);
                } else {
                    for (int tt = blockIdx.x; tt < n_tasks; tt += grid) wait_count(bar, g->qkv_ready + kCounterStride * (tt % n_heads), target);
                }
            }
            block_sync_lds();
            bar_stamp(bar);
            auto prefetch_o = NoPrefetch();
            // with the grid a multiple of the head count all tasks of a block belong to one head: they are
            // reported to the head's counter together, by the last one
            const bool one_head = grid % n_heads == 0;
            int unreported = 0;
            while (have()) {
                const Task k = current();
                advance();
                unreported += 1;
                const int publish = (!one_head || !have()) ? unreported : 0;
                if (publish) unreported = 0;
                // a block with several tasks (long contexts) requests the next task's page as soon as this
                // task has used its own: every wait for the block's counters is over by now
                // (and its further pages into the LDS slots this task has finished with)
                // The next task's page table entries are asked for now and read then: asked for then, they would
                // come back behind everything this task requests in between.
                bool next1 = false, next2 = false;
                AttnPageIds next_ids = {};
                if (have()) {
                    const Task k2 = current();
                    next_ids = attn_page_ids(k2.split, k2.L, k2.rows, k2.table);
                }
                auto next_page = [&]() {
                    if (have()) {
                        const Task k2 = current();
                        const int np = split_pages(k2.split);
                        attn_load_kv<DH, true>(kv, k2.head / grp, k2.split, k2.L, k2.rows, k2.pool, k2.table, l, n_layers, g->n_kv_heads,
                                               false, 0, &next_ids);
                        if (np > 1)
                            next1 = attn_park<DH>(sh.stash, 0, k2.head / grp, k2.split, k2.L, k2.pool, k2.table, l, n_layers, g->n_kv_heads, 1,
                                                  &next_ids);
                        if (np > 2)
                            next2 = attn_park<DH>(sh.stash, 1, k2.head / grp, k2.split, k2.L, k2.pool, k2.table, l, n_layers, g->n_kv_heads, 2,
                                                  &next_ids);
                    }
                };
                AttnBatch bt = {k.row0, k.rows, g->n_att_blocks, (const SeqRef *)g->seqs, (const int32_t *)g->row_seq};
                attn_task<DH, true, decltype(prefetch_o), BATCH ? ATTN_BATCH : (TREE ? ATTN_TREE : ATTN_CHAIN), decltype(next_page)>(
                    attn_shared<DH>(sh), kv, k.head, k.split, k.L, (const uint4 *)g->qp, k.pool, k.table, M, l, n_layers, n_heads,
                    g->n_kv_heads, g->max_splits, g->scale, g->part, g->head_counter, x_operand(g, l, 1), packed_class(NF), prefetch_o,
                    TREE ? (const uint32_t *)g->mask : nullptr, BATCH ? &bt : nullptr, next_page, publish, &sh.stash, stashed1,
                    stashed2, q_lds, q_in_lds, have());
                stashed1 = next1;
                stashed2 = next2;
                q_in_lds = one_head && !BATCH;   // (the block's later tasks: same head, same rows)
                block_sync_lds();
            }
            bar_arrive(bar);
        }
        {   // O (+ residual, operand and sums for the FFN norm)
            MegaArgsK g = phase_args();
            const LayerW w = layer_weights(g, l);
            FastArgs a = base_args<NF>(g);
            const int nks_d = (g->d + 31) / 32;
            a.Wp = w.o; a.Xp = (const uint4 *)x_operand(g, l, 1); a.nks = nks_d; a.n_tiles = g->d / 16;
            a.gain = w.ffn_gain; a.xp_next = x_operand(g, l, 2); a.ssp_next = g->ssp_b;
            WSrc next = {w.gu, nks_d, g->F / 8};
            gemm_phase<EPI_RESIDUAL, true, true, NF, KC>(a, next, pf, sh, bar, tiles_before);
        }
        {   // gate / up (+ norm, SwiGLU)
            MegaArgsK g = phase_args();
            const LayerW w = layer_weights(g, l);
            FastArgs a = base_args<NF>(g);
            a.Wp = w.gu; a.Xp = (const uint4 *)x_operand(g, l, 2); a.nks = (g->d + 31) / 32; a.n_tiles = g->F / 8;
            a.ap = x_operand(g, l, 3);
            a.ssp = g->ssp_b;
            WSrc next = {w.down, (g->F + 31) / 32, g->d / 16};
            gemm_phase<EPI_GATE_UP, true, true, NF, KC>(a, next, pf, sh, bar, tiles_before);
        }
        {   // down (+ residual, operand and sums for the next norm)
            MegaArgsK g = phase_args();
            const LayerW w = layer_weights(g, l);
            FastArgs a = base_args<NF>(g);
            a.Wp = w.down; a.Xp = (const uint4 *)x_operand(g, l, 3); a.nks = (g->F + 31) / 32; a.n_tiles = g->d / 16;
            const bool more = l + 1 < n_layers;
            a.gain = more ? layer_weights(g, l + 1).attn_gain : g->final_gain;
            a.xp_next = x_operand(g, l + 1, 0); a.ssp_next = g->ssp_a;
            WSrc next = {more ? layer_weights(g, l + 1).qkv : g->wp_lm, (g->d + 31) / 32, more ? (g->d + 2 * g->n_kv_heads * g->head_dim) / 16 : g->V / 16};
            gemm_phase<EPI_RESIDUAL, false, true, NF, KC>(a, next, pf, sh, bar, tiles_before);
        }
    }
    {   // LM head (+ final norm) with per-tile argmax
        MegaArgsK g = phase_args();
        FastArgs a = base_args<NF>(g);
        const int nks_d = (g->d + 31) / 32;
        a.Wp = g->wp_lm; a.Xp = (const uint4 *)x_operand(g, g->n_layers, 0); a.nks = nks_d; a.n_tiles = g->V / 16;
        a.ssp = g->ssp_a; a.Y = g->logits; a.ldy = g->V; a.amax = g->amax;
        WSrc none = {g->wp_lm, nks_d, 0};
        gemm_phase<EPI_LM_ARGMAX, true, true, NF, KC>(a, none, pf, sh, bar, tiles_before);
    }
    MegaArgsK g = phase_args();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // ---- argmax over the tile winners, acceptance, commit (blocks 0..M-1, one row each)
    bar_wait(bar);
    if ((int)blockIdx.x < g->M) {
        const int r = blockIdx.x, n_tiles = g->V / 16;
        float best = -INFINITY;
        int besti = 0x7fffffff;
        for (int t = threadIdx.x; t < n_tiles; t += kFastThreads) {
            uint2 pk = ld8_at<true>(reinterpret_cast<const uint2 *>(g->amax), (uint32_t)(t * 32 + r));
            float v = __uint_as_float(pk.y);
            int i = (int)pk.x;
            if (v > best || besti == 0x7fffffff || (v == best && i < besti)) { best = v; besti = i; }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            float ov = __shfl_xor(best, off, kWave);
            int oi = __shfl_xor(besti, off, kWave);
            if (ov > best || (ov == best && oi < besti)) { best = ov; besti = oi; }
        }
        if (lane == 0) { bval[wave] = best; bidx[wave] = besti; }
        __syncthreads();
        if (threadIdx.x == 0) {
            for (int w2 = 1; w2 < kFastWaves; ++w2)
                if (bval[w2] > best || (bval[w2] == best && bidx[w2] < besti)) { best = bval[w2]; besti = bidx[w2]; }
            st_agent(g->result + 2 + r, (int32_t)besti);
            wait_stores();
            last_row = __hip_atomic_fetch_add(g->row_counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == (uint32_t)(g->M - 1);
        }
        __syncthreads();
        if (last_row && threadIdx.x == 0) {
            const int32_t *pred = g->result + 2;
            int acc_n = 0;
            int32_t next;
            int32_t *hr = g->host_result;
            if (BATCH) {
                // Algorithm 1's rule inside every sequence's own rows
                for (int s = 0; s < g->n_seq; ++s) {
                    const int r0 = g->seqs[s].row0, n = g->seqs[s].n_rows;
                    int a = 0;
                    if (g->mode == 0) {
                        while (a < n - 1 && g->tok[r0 + a + 1] == ld_agent(pred + r0 + a)) ++a;
                    } else {
                        a = n - 1;
                    }
                    const int32_t nx = ld_agent(pred + r0 + a);
                    g->result[67 + 2 * s] = a;
                    g->result[68 + 2 * s] = nx;
                    st_system(g->host_batch + 2 * s, (int32_t)a);
                    st_system(g->host_batch + 2 * s + 1, nx);
                    *g->seqs[s].len_ptr += 1 + a;
                }
                next = 0;
            } else if (TREE) {
                // row r > 0 is accepted iff its parent is and its token is the prediction made there; the
                // deepest accepted row wins, the lowest index among equally deep ones
                uint32_t ok = 1u;
                int best = 0;
                for (int r = 1; r < g->M; ++r) {
                    const int p = g->parent[r];
                    if (((ok >> p) & 1u) && g->tok[r] == ld_agent(pred + p)) {
                        ok |= 1u << r;
                        if (g->depth[r] > g->depth[best]) best = r;
                    }
                }
                acc_n = g->depth[best];
                next = ld_agent(pred + best);
                for (int r = best, j = acc_n; j >= 0; --j, r = g->parent[r]) {
                    g->result[34 + j] = r;
                    st_system(hr + 34 + j, (int32_t)r);
                }
            } else {
                if (g->mode == 0) {
                    while (acc_n < g->M - 1 && g->tok[acc_n + 1] == ld_agent(pred + acc_n)) ++acc_n;
                } else {
                    acc_n = g->M - 1;
                }
                next = ld_agent(pred + acc_n);
            }
            g->result[0] = acc_n;
            g->result[1] = next;
            st_system(hr, (int32_t)acc_n);
            st_system(hr + 1, next);
            for (int i = 0; i < g->M; ++i) st_system(hr + 2 + i, ld_agent(pred + i));
            if (!BATCH) *g->len_ptr = L + 1 + acc_n;
            st_agent(g->row_counter, 0u);
        }
    }
}

}  // namespace anpd
