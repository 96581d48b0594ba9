// Stand-alone probe of the weight access pattern of the verification step (no arithmetic of the method):
// 256 blocks of 8 waves stream 128 KiB (or 344 KiB) tiles block, block + grid, ... with 1 KiB loads per
// wave, DEPTH chunks of 8 loads in flight, optionally with the per-tile LDS reduction and block barrier of
// the GEMM phases.  It answers three questions the kernels' design rests on: what the pattern reaches in
// steady state by cache policy of the loads, whether pipeline depth matters, and what a burst of the size
// of one GEMM phase reaches (in-kernel clock, first block start to last block end).
//
//   hipcc --offload-arch=gfx950 -O3 -o stream_probe stream_probe.hip && ./stream_probe
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_t;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e), __LINE__); exit(1); } } while (0)

// AUX: cache policy bits of the buffer loads (0 plain, 1 sc0, 2 nt, 16 sc1).  SYNC: per-tile LDS reduction.
template <int CH, int DEPTH, int AUX, int SYNC>
__global__ __launch_bounds__(512) void stream_kernel(const uint4 *Wp, int n_tiles, int nks, float *out, long long *clk)
{
    constexpr int W = 8;
    __shared__ float red[2][W][256];
    const long long t_start = wall_clock64();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, grid = gridDim.x;
    const int n_chunks = (((nks + W - 1) / W) + CH - 1) / CH;
    uint4 buf[DEPTH][CH];
    int lt = blockIdx.x, lc = 0, it = 0;
    // a tile past the end gets an empty descriptor: the loads return zeros and fetch nothing
    auto load = [&](uint4 (&dst)[CH], int tile, int c) {
        const bool have = tile < n_tiles;
        const uint4 *base = Wp + (size_t)(have ? tile : 0) * nks * 64;
        __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint4 *>(base), 0, have ? nks * 1024 : 0, 0x00020000);
        const int voff = (wave * 64 + lane) * 16;
#pragma unroll
        for (int u = 0; u < CH; ++u) {
            u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(r, voff, (CH * c + u) * W * 1024, AUX);
            dst[u] = make_uint4(v.x, v.y, v.z, v.w);
        }
    };
    auto advance = [&]() { if (++lc == n_chunks) { lc = 0; lt += grid; } };
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) { load(buf[d], lt, lc); advance(); }
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    const uint4 xc = make_uint4(0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u);
    int tile = blockIdx.x, c = 0;
    while (tile < n_tiles) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            if (tile < n_tiles) {
#pragma unroll
                for (int u = 0; u < CH; ++u)
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, buf[d][u]), __builtin_bit_cast(bf16x8, xc), acc, 0, 0, 0);
                load(buf[d], lt, lc);
                advance();
                if (++c == n_chunks) {
                    c = 0;
                    tile += grid;
                    if (SYNC) {
                        float *r = &red[it & 1][0][0];
                        *reinterpret_cast<f32x4 *>(r + ((size_t)wave * 64 + lane) * 4) = acc;
                        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
                        if (wave == (it & (W - 1))) {
                            f32x4 t = {0.f, 0.f, 0.f, 0.f};
                            for (int w = 0; w < W; ++w) t += *reinterpret_cast<const f32x4 *>(r + ((size_t)w * 64 + lane) * 4);
                            if (t[0] == 123.f) out[lane] = t[1];
                        }
                        acc = (f32x4){0.f, 0.f, 0.f, 0.f};
                        ++it;
                    }
                }
            }
        }
    }
    if (clk && threadIdx.x == 0) { clk[2 * blockIdx.x] = t_start; clk[2 * blockIdx.x + 1] = wall_clock64(); }
    if (acc[0] == 123.456f) out[threadIdx.x] = acc[0] + acc[1] + acc[2] + acc[3];
}

// steady state: the whole buffer per launch, timed with events
template <int CH, int DEPTH, int AUX, int SYNC>
void steady(const char *name, const uint4 *Wp, size_t bytes, int nks, float *out)
{
    const int n_tiles = (int)(bytes / ((size_t)nks * 1024));
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    float sum = 0.f;
    const int reps = 6;
    for (int i = 0; i < reps + 1; ++i) {
        CK(hipEventRecord(e0));
        stream_kernel<CH, DEPTH, AUX, SYNC><<<256, 512>>>(Wp, n_tiles, nks, out, nullptr);
        CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
        float ms; CK(hipEventElapsedTime(&ms, e0, e1));
        if (i) sum += ms;
    }
    printf("steady  %-44s chunk %2d depth %2d aux %2d tile %3d KiB: %.3f ms, %.0f GB/s\n", name, CH, DEPTH, AUX, nks, sum / reps, bytes / (sum / reps) / 1e6);
    fflush(stdout);
}

// a burst of `bytes` (a different part of the buffer every time), timed with the in-kernel 100 MHz clock
template <int CH, int DEPTH, int AUX, int SYNC>
void burst(const char *name, const uint4 *Wp, size_t total, size_t bytes, int nks, float *out, long long *clk)
{
    const int n_tiles = (int)(bytes / ((size_t)nks * 1024));
    double sum = 0, first = 0;
    int n = 0;
    for (int i = 0; i < 12; ++i) {
        const uint4 *base = Wp + (size_t)(i % (int)(total / bytes)) * (bytes / 16);
        stream_kernel<CH, DEPTH, AUX, SYNC><<<256, 512>>>(base, n_tiles, nks, out, clk);
        CK(hipDeviceSynchronize());
        long long h[512];
        CK(hipMemcpy(h, clk, sizeof(h), hipMemcpyDeviceToHost));
        long long mn = h[0], mx = h[1], mns = h[1];
        for (int b = 0; b < 256; ++b) {
            if (h[2 * b] < mn) mn = h[2 * b];
            if (h[2 * b + 1] > mx) mx = h[2 * b + 1];
            if (h[2 * b + 1] < mns) mns = h[2 * b + 1];
        }
        if (i >= 2) { sum += (mx - mn) / 100.0; first += (mns - mn) / 100.0; ++n; }
    }
    printf("burst   %-44s %5d tiles of %3d KiB, aux %2d: first block done after %6.2f us, last after %6.2f us: %.0f GB/s\n", name, n_tiles, nks, AUX,
           first / n, sum / n, bytes / (sum / n) / 1e3);
    fflush(stdout);
}

int main()
{
    const size_t bytes = (size_t)180355072 * 16;   // 16 gate/up matrices of the 7B shape: 2.9 GB, never cache-resident
    uint4 *Wp; float *out; long long *clk;
    CK(hipMalloc(&Wp, bytes)); CK(hipMalloc(&out, 4096)); CK(hipMalloc(&clk, 512 * 8));
    CK(hipMemset(Wp, 0x11, bytes));
    steady<8, 3, 0, 0>("plain loads", Wp, bytes, 128, out);
    steady<8, 3, 1, 0>("sc0", Wp, bytes, 128, out);
    steady<8, 3, 16, 0>("sc1", Wp, bytes, 128, out);
    steady<8, 3, 2, 0>("nt", Wp, bytes, 128, out);
    steady<8, 3, 18, 0>("sc1 nt", Wp, bytes, 128, out);
    steady<8, 2, 0, 0>("plain, two chunks in flight", Wp, bytes, 128, out);
    steady<8, 6, 0, 0>("plain, six chunks in flight", Wp, bytes, 128, out);
    steady<8, 2, 2, 1>("nt, two chunks, per-tile reduction + barrier", Wp, bytes, 128, out);
    steady<8, 3, 2, 1>("nt, three chunks, per-tile reduction + barrier", Wp, bytes, 128, out);
    steady<8, 4, 2, 1>("nt, four chunks, per-tile reduction + barrier", Wp, bytes, 128, out);
    steady<8, 3, 2, 1>("nt, K = 11008 tiles, reduction + barrier", Wp, bytes, 344, out);
    burst<8, 3, 2, 1>("gate/up phase (1376 tiles)", Wp, bytes, (size_t)1376 * 131072, 128, out, clk);
    burst<8, 3, 0, 1>("gate/up phase, plain loads", Wp, bytes, (size_t)1376 * 131072, 128, out, clk);
    burst<8, 3, 2, 1>("5 tiles per block", Wp, bytes, (size_t)1280 * 131072, 128, out, clk);
    burst<8, 3, 2, 1>("10 tiles per block", Wp, bytes, (size_t)2560 * 131072, 128, out, clk);
    burst<8, 3, 2, 1>("20 tiles per block", Wp, bytes, (size_t)5120 * 131072, 128, out, clk);
    burst<8, 3, 2, 1>("QKV phase (768 tiles)", Wp, bytes, (size_t)768 * 131072, 128, out, clk);
    burst<8, 3, 2, 1>("down phase (256 tiles of K = 11008)", Wp, bytes, (size_t)256 * 352256, 344, out, clk);
    return 0;
}
