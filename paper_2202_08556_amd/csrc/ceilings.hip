// Stand-alone ceilings of the memory system that bound the SpMM kernels (measurement tool, not
// part of libdaspmm.so):
//   ceilings stream                      HBM read and copy bandwidth, 1 GiB buffers
//   ceilings gather N k uniform|zipf     random gather of k rows of N floats (13 Mi indices), the
//                                        access pattern of the B operand, without values/FMA/C
//   ceilings file colind.bin k N [T]     the same over a real column-index stream (raw int32 file,
//                                        e.g. written by `python -m paper_2202_08556_amd.generators`);
//                                        with T also with every block of T indices sorted ascending
//   ceilings atomics                     fp32 atomic-add rate on random rows and on 16 hot rows
// The gather kernels use the staging scheme of the product kernels: a lane group loads a batch
// of indices coalesced, passes them round through LDS and issues 8 row gathers back to back.
#include <hip/hip_runtime.h>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>
#include <algorithm>

#define CK(x) do { hipError_t err_ = (x); if (err_ != hipSuccess) { \
    std::printf("HIP error %s at line %d\n", hipGetErrorString(err_), __LINE__); std::exit(1); } } while (0)

__global__ void copy_kernel(const float4* __restrict__ a, float4* __restrict__ b, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t st = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += st) b[i] = a[i];
}

__global__ void read_kernel(const float4* __restrict__ a, float* __restrict__ out, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t st = (size_t)gridDim.x * blockDim.x;
    float s = 0;
    for (; i < n; i += st) { const float4 v = a[i]; s += v.x + v.y + v.z + v.w; }
    if (s == 1.2345f) out[0] = s;
}

template <int V>
__device__ __forceinline__ void ldv(const float* p, float (&x)[V]) {
    if constexpr (V == 4) { const float4 t = *(const float4*)p; x[0] = t.x; x[1] = t.y; x[2] = t.z; x[3] = t.w; }
    else x[0] = *p;
}

__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// every group of G lanes gathers T rows (indices idx[group*T ..]); blockIdx.y = column tile
template <int V, int G>
__global__ __launch_bounds__(256) void gather_kernel(const int* __restrict__ idx, const float* __restrict__ B,
                                                     float* __restrict__ out, int N, int T, long ngroups, int pin)
{
    constexpr int U = 8, SB = G < U ? U : G;
    __shared__ int stage[4 * (64 / G) * SB];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, g = lane / G, j = lane % G;
    // pin > 0: 1-D grid, column tile = (blockIdx.x % 8) % pin, i.e. fixed per XCD
    int tile = blockIdx.y;
    long bx = blockIdx.x;
    if (pin > 0) { const int xcd = blockIdx.x & 7; tile = xcd % pin; bx = (long)(blockIdx.x >> 3) * (8 / pin) + xcd / pin; }
    const long group = (bx * 4 + wave) * (64 / G) + g;
    if (group >= ngroups) return;
    const int* my = idx + group * T;
    const float* Bn = B + (tile * G + j) * V;
    float acc[V];
    for (int v = 0; v < V; ++v) acc[v] = 0;
    int* st = stage + (wave * (64 / G) + g) * SB;
    for (int p0 = 0; p0 < T; p0 += SB) {
        for (int i = j; i < SB; i += G) st[i] = my[p0 + i];
        wave_lds_sync();
        for (int t0 = 0; t0 < SB; t0 += U) {
            float b[U][V];
#pragma unroll
            for (int u = 0; u < U; ++u) ldv<V>(Bn + (long)st[t0 + u] * N, b[u]);
#pragma unroll
            for (int u = 0; u < U; ++u) for (int v = 0; v < V; ++v) acc[v] += b[u][v];
        }
        wave_lds_sync();
    }
    float s = 0;
    for (int v = 0; v < V; ++v) s += acc[v];
    if (s == 1.2345f) out[0] = s;
}

__global__ void atomic_kernel(float* __restrict__ C, const int* __restrict__ idx, int n, int N) {
    const long w = ((long)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    if (w >= n) return;
    unsafeAtomicAdd(C + (long)idx[w] * N + lane, 1.0f);
}

template <class F>
float timeit(F f, int reps = 10) {
    hipEvent_t a, b;
    CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
    f(); f();
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(a));
    for (int i = 0; i < reps; ++i) f();
    CK(hipEventRecord(b));
    CK(hipEventSynchronize(b));
    float ms;
    CK(hipEventElapsedTime(&ms, a, b));
    return ms / reps;
}

template <int V, int G>
void run_gather(const int* didx, const float* dB, float* dout, int N, int T, long nidx) {
    if (N % (G * V) != 0 || T % (G < 8 ? 8 : G) != 0) return;
    const long ngroups = nidx / T, gpb = 4 * (64 / G);
    const int tiles = N / (G * V);
    for (int pin = 0; pin <= ((tiles == 2 || tiles == 4 || tiles == 8) ? 1 : 0); ++pin) {
        const long bx = (ngroups + gpb - 1) / gpb;
        const dim3 grid = pin ? dim3((unsigned)(8 * ((bx + 8 / tiles - 1) / (8 / tiles))), 1) : dim3((unsigned)bx, tiles);
        const int pinarg = pin ? tiles : 0;
        const float ms = timeit([&] { hipLaunchKernelGGL((gather_kernel<V, G>), grid, dim3(256), 0, 0, didx, dB, dout, N, T, ngroups, pinarg); });
        std::printf("  %d-byte loads, %2d lanes per row, %d column tile(s)%s, %d rows per lane group: %8.1f us  %6.2f TB/s\n",
                    4 * V, G, tiles, pin ? " pinned to XCDs" : "", T, ms * 1e3, (double)ngroups * T * N * 4 / ms / 1e9);
        std::fflush(stdout);
    }
}

void gather_all(const std::vector<int>& idx, long k, int N) {
    const long nidx = (long)idx.size() / 4096 * 4096;
    int* didx; float* dB; float* dout;
    CK(hipMalloc(&dout, 4));
    CK(hipMalloc(&didx, nidx * 4));
    CK(hipMalloc(&dB, (size_t)k * N * 4));
    CK(hipMemcpy(didx, idx.data(), nidx * 4, hipMemcpyHostToDevice));
    CK(hipMemset(dB, 0, (size_t)k * N * 4));
    if (N >= 128) { run_gather<4, 32>(didx, dB, dout, N, 256, nidx); run_gather<4, 8>(didx, dB, dout, N, 256, nidx); run_gather<1, 64>(didx, dB, dout, N, 512, nidx); }
    else if (N >= 64) { run_gather<4, 16>(didx, dB, dout, N, 256, nidx); run_gather<1, 64>(didx, dB, dout, N, 256, nidx); }
    else if (N >= 32) { run_gather<4, 8>(didx, dB, dout, N, 256, nidx); run_gather<1, 32>(didx, dB, dout, N, 256, nidx); }
    else if (N >= 16) { run_gather<4, 4>(didx, dB, dout, N, 256, nidx); run_gather<1, 16>(didx, dB, dout, N, 256, nidx); }
    else { run_gather<4, 2>(didx, dB, dout, N, 256, nidx); run_gather<1, 8>(didx, dB, dout, N, 256, nidx); }
    CK(hipFree(didx)); CK(hipFree(dB)); CK(hipFree(dout));
}

int main(int argc, char** argv)
{
    const char* mode = argc > 1 ? argv[1] : "stream";
    std::mt19937_64 rng(1);
    if (!std::strcmp(mode, "stream")) {
        const size_t n = (size_t)1 << 30;
        float4 *a, *b; float* out;
        CK(hipMalloc(&a, n)); CK(hipMalloc(&b, n)); CK(hipMalloc(&out, 4));
        CK(hipMemset(a, 1, n));
        for (int blocks : {2048, 8192, 32768}) {
            float ms = timeit([&] { hipLaunchKernelGGL(copy_kernel, dim3(blocks), dim3(256), 0, 0, a, b, n / 16); });
            std::printf("copy 1 GiB -> 1 GiB, %5d blocks: %.1f us  %.2f TB/s (read + write)\n", blocks, ms * 1e3, 2.0 * n / ms / 1e9);
            ms = timeit([&] { hipLaunchKernelGGL(read_kernel, dim3(blocks), dim3(256), 0, 0, a, out, n / 16); });
            std::printf("read 1 GiB,          %5d blocks: %.1f us  %.2f TB/s\n", blocks, ms * 1e3, 1.0 * n / ms / 1e9);
        }
    } else if (!std::strcmp(mode, "gather") && argc >= 5) {
        const int N = std::atoi(argv[2]);
        const long k = std::atol(argv[3]);
        const bool zipf = !std::strcmp(argv[4], "zipf");
        if (N < 8 || N % 8 || k < 1 || (size_t)k * N * 4 > ((size_t)3 << 30)) { std::printf("bad N or k\n"); return 1; }
        std::vector<int> idx(13 * 1024 * 1024);
        if (!zipf) {
            std::uniform_int_distribution<long> d(0, k - 1);
            for (auto& x : idx) x = (int)d(rng);
        } else {   // popularity rank r with P(r) ~ 1/r, mapped through a random permutation
            std::uniform_real_distribution<double> u(0, 1);
            std::vector<int> perm(k);
            for (long i = 0; i < k; ++i) perm[i] = (int)i;
            std::shuffle(perm.begin(), perm.end(), rng);
            for (auto& x : idx) {
                long r = (long)std::floor(std::exp(u(rng) * std::log(k + 1.0)));
                r = r < 1 ? 1 : (r > k ? k : r);
                x = perm[r - 1];
            }
        }
        std::printf("gather N=%d k=%ld (table %.1f MB) %s indices\n", N, k, (double)k * N * 4 / 1e6, zipf ? "zipf" : "uniform");
        gather_all(idx, k, N);
    } else if (!std::strcmp(mode, "file") && argc >= 5) {
        const long k = std::atol(argv[3]);
        const int N = std::atoi(argv[4]);
        FILE* f = std::fopen(argv[2], "rb");
        if (!f || N < 8 || N % 8 || k < 1) { std::printf("cannot open file or bad k / N\n"); return 1; }
        std::fseek(f, 0, SEEK_END);
        const long n = std::ftell(f) / 4;
        std::fseek(f, 0, SEEK_SET);
        std::vector<int> idx(n);
        if (std::fread(idx.data(), 4, n, f) != (size_t)n) { std::printf("short read\n"); return 1; }
        std::fclose(f);
        for (long i = 0; i < n; ++i)
            if (idx[i] < 0 || idx[i] >= k) { std::printf("index out of range\n"); return 1; }
        std::printf("gather over %s: %ld indices, k=%ld, N=%d\n", argv[2], n, k, N);
        gather_all(idx, k, N);
        if (argc >= 6) {
            // every lane group's T indices in ascending order: all groups then sweep the rows of B
            // from low to high addresses at about the same pace
            const long T = std::atol(argv[5]);
            if (T < 32 || T % 32) { std::printf("T must be a multiple of 32\n"); return 1; }
            for (long b = 0; b + T <= n; b += T) std::sort(idx.begin() + b, idx.begin() + b + T);
            std::printf("same stream, every block of %ld indices sorted ascending\n", T);
            const long nidx = n / T * T;
            int* didx; float* dB; float* dout;
            CK(hipMalloc(&dout, 4)); CK(hipMalloc(&didx, nidx * 4)); CK(hipMalloc(&dB, (size_t)k * N * 4));
            CK(hipMemcpy(didx, idx.data(), nidx * 4, hipMemcpyHostToDevice)); CK(hipMemset(dB, 0, (size_t)k * N * 4));
            if (N >= 128) { run_gather<4, 32>(didx, dB, dout, N, (int)T, nidx); run_gather<4, 8>(didx, dB, dout, N, (int)T, nidx); }
            else if (N >= 32) run_gather<4, 8>(didx, dB, dout, N, (int)T, nidx);
            else run_gather<1, 8>(didx, dB, dout, N, (int)T, nidx);
        }
    } else if (!std::strcmp(mode, "atomics")) {
        const int n = 1 << 20, N = 64;
        const long rows = 262144;
        float* C; int* didx;
        CK(hipMalloc(&C, rows * N * 4)); CK(hipMemset(C, 0, rows * N * 4)); CK(hipMalloc(&didx, n * 4));
        std::vector<int> idx(n);
        std::uniform_int_distribution<int> d(0, (int)rows - 1);
        for (auto& x : idx) x = d(rng);
        CK(hipMemcpy(didx, idx.data(), n * 4, hipMemcpyHostToDevice));
        float ms = timeit([&] { hipLaunchKernelGGL(atomic_kernel, dim3(n / 4), dim3(256), 0, 0, C, didx, n, N); });
        std::printf("atomic add, 64-float segments of random rows: %.1f us, %.1f G atomics/s\n", ms * 1e3, (double)n * 64 / ms / 1e6);
        for (auto& x : idx) x %= 16;
        CK(hipMemcpy(didx, idx.data(), n * 4, hipMemcpyHostToDevice));
        ms = timeit([&] { hipLaunchKernelGGL(atomic_kernel, dim3(n / 4), dim3(256), 0, 0, C, didx, n, N); });
        std::printf("atomic add, 16 hot rows: %.1f us, %.1f G atomics/s\n", ms * 1e3, (double)n * 64 / ms / 1e6);
    } else {
        std::printf("usage: ceilings stream | gather N k uniform|zipf | file colind.bin k N | atomics\n");
        return 1;
    }
    return hipDeviceSynchronize() == hipSuccess ? 0 : 1;
}
