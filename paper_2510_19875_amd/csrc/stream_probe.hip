// Micro-benchmarks behind the roofline statements of the Stream kernels (not part of the product
// library: built as libstream_probe.so and called by `bench.py --probes`).
//
//   mfma    the level kernel's tile product alone: 32 x (32x32x16 bf16 MFMA) per 64 x 64 x 128 tile
//           on register-resident operands holding random values, one or two wavefronts per SIMD,
//           for a short and a long run (the part lowers its clock under sustained matrix load);
//   clock   the shader clock during that long run: shader-clock counter against the constant
//           100 MHz real-time counter, read inside the kernel;
//   gather  the level kernel's K-tile fetch alone: 16 KiB tiles read as sixteen 1 KiB wave-wide
//           buffer loads from random tile positions inside a working set that fits the L2, the
//           Infinity Cache, or neither.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));

// One wavefront: `ntiles` tile products of 32 MFMAs each on operands held in registers.
// clk[2 * wave_id] / clk[2 * wave_id + 1]: elapsed shader clocks / elapsed 100 MHz ticks.
template <int OCC>
__global__ void __launch_bounds__(256, OCC) mfma_probe(const uint4 *in, float *out, int ntiles, long long *clk)
{
    const int lane = threadIdx.x & 63;
    uint4 q[2][8], kf[2][8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        q[0][i] = in[lane + 64 * i];
        q[1][i] = in[lane + 64 * (i + 8)];
        kf[0][i] = in[lane + 64 * (i + 16)];
        kf[1][i] = in[lane + 64 * (i + 24)];
    }
    const long long c0 = (long long)__builtin_amdgcn_s_memtime();
    const long long r0 = (long long)__builtin_amdgcn_s_memrealtime();
    float res = 0.f;
    for (int t = 0; t < ntiles; ++t) {
        floatx16 acc[2][2];
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;
#pragma unroll
        for (int fr = 0; fr < 8; ++fr)
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) {
#pragma unroll
                for (int rb = 0; rb < 2; ++rb)
                    acc[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, q[rb][fr]),
                                                                          __builtin_bit_cast(bf16x8, kf[cb][fr]),
                                                                          acc[rb][cb], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        res += acc[0][0][0] + acc[0][1][5] + acc[1][0][3] + acc[1][1][7];
        kf[0][0].x += 1;   // the products differ from tile to tile: nothing is hoisted
    }
    const long long c1 = (long long)__builtin_amdgcn_s_memtime();
    const long long r1 = (long long)__builtin_amdgcn_s_memrealtime();
    out[blockIdx.x * 256 + threadIdx.x] = res;
    if (lane == 0) {
        const long long w = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
        clk[2 * w] = c1 - c0;
        clk[2 * w + 1] = r1 - r0;
    }
}

// The same tile product from 16x16x32 MFMAs (64 per tile): does the smaller shape draw less power?
typedef float floatx4 __attribute__((ext_vector_type(4)));
__global__ void __launch_bounds__(256, 2) mfma16_probe(const uint4 *in, float *out, int ntiles, long long *clk)
{
    const int lane = threadIdx.x & 63;
    uint4 q[4][4], kf[4][4];     // [16-row group][32-wide slice of the contraction axis]
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            q[i][j] = in[lane + 64 * (i * 4 + j)];
            kf[i][j] = in[lane + 64 * (16 + i * 4 + j)];
        }
    const long long c0 = (long long)__builtin_amdgcn_s_memtime();
    const long long r0 = (long long)__builtin_amdgcn_s_memrealtime();
    float res = 0.f;
    for (int t = 0; t < ntiles; ++t) {
        floatx4 acc[4][4];
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b)
#pragma unroll
                for (int i = 0; i < 4; ++i) acc[a][b][i] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int cb = 0; cb < 4; ++cb) {
#pragma unroll
                for (int rb = 0; rb < 4; ++rb)
                    acc[rb][cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, q[rb][ks]),
                                                                          __builtin_bit_cast(bf16x8, kf[cb][ks]),
                                                                          acc[rb][cb], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b) res += acc[a][b][(a + b) & 3];   // every product is used
        kf[0][0].x += 1;
    }
    const long long c1 = (long long)__builtin_amdgcn_s_memtime();
    const long long r1 = (long long)__builtin_amdgcn_s_memrealtime();
    out[blockIdx.x * 256 + threadIdx.x] = res;
    if (lane == 0) {
        const long long w = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
        clk[2 * w] = c1 - c0;
        clk[2 * w + 1] = r1 - r0;
    }
}

// One wavefront reads `ntiles` tiles of 16 KiB (sixteen loads of 1 KiB in flight, refilled in
// place as the level kernel does) from pseudo-random tile positions below `tile_mask`.
__global__ void __launch_bounds__(256, 2) gather_probe(const char *base, unsigned region_bytes, int ntiles,
                                                       unsigned tile_mask, unsigned *out)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(base), 0, (int)region_bytes, 0x00020000);
    unsigned seed = (blockIdx.x * 4 + wave) * 2654435761u + 12345u;
    u32x4_t r[16];
    unsigned acc = 0;
    const unsigned lane_off = lane * 16;
    const unsigned t0 = (seed >> 8) & tile_mask;
    seed = seed * 1664525u + 1013904223u;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        r[j] = __builtin_amdgcn_raw_buffer_load_b128(rs, lane_off + (j & 3) * 1024, t0 * 16384u + (j >> 2) * 4096, 0);
        __builtin_amdgcn_sched_barrier(0);
    }
    for (int t = 0; t < ntiles; ++t) {
        const unsigned tn = __builtin_amdgcn_readfirstlane((seed >> 8) & tile_mask);
        seed = seed * 1664525u + 1013904223u;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            acc ^= r[j][0] ^ r[j][3];
            __builtin_amdgcn_sched_barrier(0);
            r[j] = __builtin_amdgcn_raw_buffer_load_b128(rs, lane_off + (j & 3) * 1024, tn * 16384u + (j >> 2) * 4096, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
#pragma unroll
    for (int j = 0; j < 16; ++j) acc ^= r[j][1];
    if (acc == 0x12345678u) out[0] = acc;   // (never true for the fill pattern: keeps the loads alive)
}

struct Timer {
    hipEvent_t e0, e1;
    Timer() { (void)hipEventCreate(&e0); (void)hipEventCreate(&e1); }
    ~Timer() { (void)hipEventDestroy(e0); (void)hipEventDestroy(e1); }
};

template <int OCC, bool SMALL = false>
int run_mfma(int ntiles, uint4 *in, float *out, long long *clk, double *tflops, double *mhz)
{
    const int wgs = 256 * OCC * 4;
    Timer tm;
    float ms = 0.f;
    for (int rep = 0; rep < 2; ++rep) {
        if (hipEventRecord(tm.e0) != hipSuccess) return 1;
        if constexpr (SMALL) hipLaunchKernelGGL(mfma16_probe, dim3(wgs), dim3(256), 0, 0, in, out, ntiles, clk);
        else hipLaunchKernelGGL(mfma_probe<OCC>, dim3(wgs), dim3(256), 0, 0, in, out, ntiles, clk);
        if (hipGetLastError() != hipSuccess) return 1;
        (void)hipEventRecord(tm.e1);
        if (hipEventSynchronize(tm.e1) != hipSuccess) return 1;
        (void)hipEventElapsedTime(&ms, tm.e0, tm.e1);
    }
    *tflops = (double)wgs * 4 * ntiles * 32 * 32768.0 / (ms * 1e-3) / 1e12;
    // shader clock = sum of shader clocks / sum of 100 MHz ticks over all wavefronts
    const int nw = wgs * 4;
    long long *h = new long long[2 * nw];
    if (hipMemcpy(h, clk, sizeof(long long) * 2 * nw, hipMemcpyDeviceToHost) != hipSuccess) { delete[] h; return 1; }
    double sc = 0, rt = 0;
    for (int i = 0; i < nw; ++i) { sc += (double)h[2 * i]; rt += (double)h[2 * i + 1]; }
    delete[] h;
    *mhz = rt > 0 ? sc / rt * 100.0 : 0.0;
    return 0;
}

}  // namespace

extern "C" {

// out[0..7]: MFMA-only TFLOP/s and shader clock (MHz) for {2 waves/SIMD short run, 2 waves/SIMD long
// run, 1 wave/SIMD short, 1 wave/SIMD long}; out[8 + 2i], out[9 + 2i]: tile-gather TB/s and bytes
// per launch for working sets of 2 MiB, 16 MiB, 64 MiB, 128 MiB, 1 GiB; out[18], out[19]: the long
// 2 waves/SIMD MFMA run again with all-zero operands; out[20], out[21] (if n >= 22): the long run built from
// 16x16x32 MFMAs on random operands.  Allocates its own buffers
// (1 GiB) and synchronises.  Returns 0 on success.
int stream_probe_run(double *out, int n)
{
    if (!out || n < 20) return 1;
    memset(out, 0, sizeof(double) * n);
    uint4 *in = nullptr;
    float *o = nullptr;
    long long *clk = nullptr;
    char *big = nullptr;
    unsigned *flag = nullptr;
    const size_t region = 1u << 30;
    if (hipMalloc(&in, 1 << 20) != hipSuccess) return 2;
    if (hipMalloc(&o, sizeof(float) * 256 * 8 * 256) != hipSuccess) return 2;
    if (hipMalloc(&clk, sizeof(long long) * 2 * 256 * 8 * 4) != hipSuccess) return 2;
    if (hipMalloc(&big, region) != hipSuccess) return 2;
    if (hipMalloc(&flag, 4) != hipSuccess) return 2;
    // operands: random bf16 values of both signs with magnitudes between 2^-7 and 2 (the power an
    // MFMA draws, and with it the clock the part sustains, depends on the data: zeros are cheap)
    {
        const size_t n16 = (1 << 20) / 2;
        unsigned short *h = new unsigned short[n16];
        unsigned long long st = 0x9E3779B97F4A7C15ull;
        for (size_t i = 0; i < n16; ++i) {
            st = st * 6364136223846793005ull + 1442695040888963407ull;
            const unsigned r = (unsigned)(st >> 33);
            h[i] = (unsigned short)(((r & 1u) << 15) | ((120u + ((r >> 1) & 7u)) << 7) | ((r >> 4) & 0x7fu));
        }
        const hipError_t e = hipMemcpy(in, h, n16 * 2, hipMemcpyHostToDevice);
        delete[] h;
        if (e != hipSuccess) return 2;
    }
    (void)hipMemset(big, 1, region);
    int rc = 0;
    // ~2 ms and ~60 ms of MFMA-only work
    rc |= run_mfma<2>(256, in, o, clk, &out[0], &out[1]);
    rc |= run_mfma<2>(8192, in, o, clk, &out[2], &out[3]);
    rc |= run_mfma<1>(512, in, o, clk, &out[4], &out[5]);
    rc |= run_mfma<1>(16384, in, o, clk, &out[6], &out[7]);
    if (n >= 22) rc |= run_mfma<2, true>(8192, in, o, clk, &out[20], &out[21]);   // 16x16x32 MFMAs, random operands
    // the same long run on all-zero operands: multipliers that do not toggle draw far less power
    if (hipMemset(in, 0, 1 << 20) != hipSuccess) return 2;
    rc |= run_mfma<2>(8192, in, o, clk, &out[18], &out[19]);
    const unsigned masks[5] = {127u, 1023u, 4095u, 8191u, 65535u};   // working sets in tiles of 16 KiB, minus one
    Timer tm;
    for (int i = 0; i < 5 && rc == 0; ++i) {
        const int wgs = 256 * 2 * 8, ntw = 256;
        const unsigned m = masks[i];
        float ms = 0.f;
        for (int rep = 0; rep < 2; ++rep) {
            (void)hipEventRecord(tm.e0);
            hipLaunchKernelGGL(gather_probe, dim3(wgs), dim3(256), 0, 0, big, (unsigned)region, ntw, m, flag);
            if (hipGetLastError() != hipSuccess) rc = 3;
            (void)hipEventRecord(tm.e1);
            if (hipEventSynchronize(tm.e1) != hipSuccess) rc = 3;
            (void)hipEventElapsedTime(&ms, tm.e0, tm.e1);
        }
        const double bytes = (double)wgs * 4 * ntw * 16384.0;
        out[8 + 2 * i] = bytes / (ms * 1e-3) / 1e12;
        out[9 + 2 * i] = (double)(m + 1) * 16384.0;
    }
    (void)hipFree(in); (void)hipFree(o); (void)hipFree(clk); (void)hipFree(big); (void)hipFree(flag);
    return rc;
}

}  // extern "C"
