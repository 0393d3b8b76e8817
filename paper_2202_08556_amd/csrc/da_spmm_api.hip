// Host side of libdaspmm.so: argument checks, choice of launch geometry, dispatch of the
// algorithm id to a kernel instantiation, the feature-extraction helper and the selector.
// The C ABI is declared and documented in include/da_spmm.h.
#include "da_spmm.h"
#include "da_spmm_kernels.hip"

#include <atomic>
#include <cmath>
#include <cstdio>
#include <cstring>

namespace {

using namespace daspmm;

thread_local char g_err[256] = "";

int fail(int code, const char* fmt, const char* a = "") {
    std::snprintf(g_err, sizeof g_err, fmt, a);
    return code;
}

int hip_fail(hipError_t e, const char* where) {
    std::snprintf(g_err, sizeof g_err, "%s: %s", where, hipGetErrorString(e));
    return DA_ERR_HIP;
}

// number of compute units of the current device (cached per device ordinal)
int cu_count() {
    static std::atomic<int> cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    int c = cached[dev].load(std::memory_order_relaxed);
    if (c == 0) {
        if (hipDeviceGetAttribute(&c, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || c <= 0)
            c = 256;
        cached[dev].store(c, std::memory_order_relaxed);
    }
    return c;
}

int pow2_ceil(long x) {
    int p = 1;
    while (p < x) p <<= 1;
    return p;
}

// widest per-lane vector (technique 2 of Sec. 4) that N and the base addresses allow
int pick_vec(int64_t N, const void* B, const void* C) {
    const uintptr_t a = reinterpret_cast<uintptr_t>(B) | reinterpret_cast<uintptr_t>(C);
    if (N % 4 == 0 && a % 16 == 0) return 4;
    if (N % 2 == 0 && a % 8 == 0) return 2;
    return 1;
}

struct Problem {
    int m, N;
    const int* rowptr;
    const int* colind;
    const float* vals;
    const float* B;
    float* C;
    hipStream_t stream;
    int64_t k;
};

enum Family { RB_SR, RB_PR, EB_SR, EB_PR };

constexpr int kEntriesPerWave = 512;   // EB: stored entries per wave and pass
constexpr int kMaxGridY = 65535;

template <int V, int G>
int launch(Family fam, const Problem& p) {
    const long tiles_l = (p.N + (long)G * V - 1) / ((long)G * V);
    if (tiles_l > kMaxGridY) return fail(DA_ERR_UNSUPPORTED, "N needs more than 65535 column tiles%s");
    const unsigned tiles = (unsigned)tiles_l;
    const dim3 block(kBlock);
    switch (fam) {
    case RB_SR: {
        const long rows_per_block = (long)kWavesPerBlock * (kWave / G);
        const dim3 grid((unsigned)((p.m + rows_per_block - 1) / rows_per_block), tiles);
        hipLaunchKernelGGL((rb_sr_kernel<V, G>), grid, block, 0, p.stream,
                           p.m, p.N, p.rowptr, p.colind, p.vals, p.B, p.C);
        break;
    }
    case RB_PR: {
        const dim3 grid((unsigned)((p.m + kWavesPerBlock - 1) / kWavesPerBlock), tiles);
        hipLaunchKernelGGL((rb_pr_kernel<V, G>), grid, block, 0, p.stream,
                           p.m, p.N, p.rowptr, p.colind, p.vals, p.B, p.C);
        break;
    }
    case EB_SR:
    case EB_PR: {
        // entries per worker: a lane group (SR) or a whole wave (PR)
        const int chunk = fam == EB_SR ? (kEntriesPerWave * G / kWave < 8 ? 8 : kEntriesPerWave * G / kWave)
                                       : kEntriesPerWave;
        const long entries_per_block = fam == EB_SR ? (long)chunk * kWavesPerBlock * (kWave / G)
                                                    : (long)chunk * kWavesPerBlock;
        // nnz is known only on the device; size the grid for a full machine, bounded by what the
        // matrix could hold at most
        long max_nnz = (long)p.m * (p.k < 1 ? 1 : p.k);
        if (max_nnz > 0x7fffffffL) max_nnz = 0x7fffffffL;
        long blocks = (max_nnz + entries_per_block - 1) / entries_per_block;
        const long full = (long)cu_count() * 8;
        if (blocks > full) blocks = full;
        if (blocks < 1) blocks = 1;
        // pre-pass: zero the rows that receive atomic additions, and the rows without entries
        {
            const int gz = pow2_ceil((p.N + V - 1) / V) > kWave ? kWave : pow2_ceil((p.N + V - 1) / V);
            const long rows_per_block = (long)kWavesPerBlock * (kWave / gz);
            const dim3 zgrid((unsigned)((p.m + rows_per_block - 1) / rows_per_block));
#define DA_ZERO(GZ) case GZ: hipLaunchKernelGGL((eb_zero_kernel<V, GZ>), zgrid, block, 0, p.stream, \
                                                p.m, p.N, p.rowptr, p.C, chunk); break;
            switch (gz) { DA_ZERO(1) DA_ZERO(2) DA_ZERO(4) DA_ZERO(8) DA_ZERO(16) DA_ZERO(32) DA_ZERO(64) }
#undef DA_ZERO
        }
        const dim3 grid((unsigned)blocks, tiles);
        if (fam == EB_SR)
            hipLaunchKernelGGL((eb_sr_kernel<V, G>), grid, block, 0, p.stream,
                               p.m, p.N, p.rowptr, p.colind, p.vals, p.B, p.C, chunk);
        else
            hipLaunchKernelGGL((eb_pr_kernel<V, G>), grid, block, 0, p.stream,
                               p.m, p.N, p.rowptr, p.colind, p.vals, p.B, p.C, chunk);
        break;
    }
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "kernel launch");
    return DA_OK;
}

template <int V>
int dispatch_g(Family fam, int G, const Problem& p) {
    switch (G) {
    case 1: return launch<V, 1>(fam, p);
    case 2: return launch<V, 2>(fam, p);
    case 4: return launch<V, 4>(fam, p);
    case 8: return launch<V, 8>(fam, p);
    case 16: return launch<V, 16>(fam, p);
    case 32: return launch<V, 32>(fam, p);
    case 64: return launch<V, 64>(fam, p);
    }
    return fail(DA_ERR_UNSUPPORTED, "bad lane group%s");
}

int dispatch(Family fam, int V, int G, const Problem& p) {
    switch (V) {
    case 4: return dispatch_g<4>(fam, G, p);
    case 2: return dispatch_g<2>(fam, G, p);
    default: return dispatch_g<1>(fam, G, p);
    }
}

const char* const kNames[DA_NUM_ALGOS] = {
    "RB+RM+SR", "RB+RM+PR", "RB+CM+SR", "RB+CM+PR", "EB+RM+SR", "EB+RM+PR", "EB+CM+SR", "EB+CM+PR"};

constexpr int kMaxGroupPR = 8;   // RM mapping under PR keeps at least 8 slots along the entries

}  // namespace

extern "C" {

int da_spmm(int64_t m, int64_t k, int64_t N, const int32_t* rowptr, const int32_t* colind,
            const float* vals, const float* B, float* C, int algo, void* stream)
{
    if (m < 0 || k < 0 || N < 0) return fail(DA_ERR_INVALID_ARG, "negative size%s");
    if (m > 0x7ffffffeLL || k > 0x7fffffffLL || N > 0x7fffffffLL)
        return fail(DA_ERR_INVALID_ARG, "size beyond the int32 index range%s");
    if (algo < 0 || algo >= DA_NUM_ALGOS) return fail(DA_ERR_BAD_ALGO, "algorithm id outside 0..7%s");
    if (m == 0 || N == 0) return DA_OK;
    if (!rowptr || !C) return fail(DA_ERR_INVALID_ARG, "null rowptr or C%s");
    // colind, vals and B are read only through stored entries; they may be null when nnz == 0,
    // which only the device knows

    Problem p{(int)m, (int)N, rowptr, colind, vals, B, C, (hipStream_t)stream, k};
    const int V = pick_vec(N, B, C);
    const bool eb = algo >= DA_EB_RM_SR;
    const bool cm = (algo & 2) != 0;
    const bool pr = (algo & 1) != 0;
    int G = 1;
    if (!cm) {
        G = pow2_ceil((N + V - 1) / V);
        const int cap = pr ? kMaxGroupPR : kWave;
        if (G > cap) G = cap;
    }
    const Family fam = eb ? (pr ? EB_PR : EB_SR) : (pr ? RB_PR : RB_SR);
    return dispatch(fam, V, G, p);
}

int da_spmm_features(int64_t m, int64_t N, const int32_t* rowptr, void* stream, da_features* out)
{
    if (!out) return fail(DA_ERR_INVALID_ARG, "null output%s");
    if (m < 0 || N < 0 || m > 0x7ffffffeLL) return fail(DA_ERR_INVALID_ARG, "bad size%s");
    std::memset(out, 0, sizeof *out);
    out->N = N;
    if (m == 0) return DA_OK;
    if (!rowptr) return fail(DA_ERR_INVALID_ARG, "null rowptr%s");
    hipStream_t st = (hipStream_t)stream;
    unsigned long long* dbuf = nullptr;
    hipError_t e = hipMalloc(&dbuf, 3 * sizeof(unsigned long long));
    if (e != hipSuccess) return hip_fail(e, "hipMalloc");
    unsigned long long h[3] = {0, 0, 0};
    e = hipMemsetAsync(dbuf, 0, sizeof h, st);
    if (e == hipSuccess) {
        long blocks = (m + kBlock - 1) / kBlock;
        const long cap = (long)cu_count() * 8;
        if (blocks > cap) blocks = cap;
        hipLaunchKernelGGL(features_kernel, dim3((unsigned)blocks), dim3(kBlock), 0, st, (int)m, rowptr, dbuf);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipMemcpyAsync(h, dbuf, sizeof h, hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    (void)hipFree(dbuf);
    if (e != hipSuccess) return hip_fail(e, "da_spmm_features");
    // population variance = (m * sum len^2 - nnz^2) / m^2, formed exactly in 128-bit integers
    const unsigned __int128 num = (unsigned __int128)(unsigned long long)m * h[0]
                                  - (unsigned __int128)h[2] * h[2];
    const double md = (double)m;
    const double mean = (double)h[2] / md;
    const double var = (double)num / (md * md);
    out->rows = m;
    out->nnz = (int64_t)h[2];
    out->row_nnz_mean = mean;
    out->row_nnz_std = std::sqrt(var);
    out->row_nnz_max = (double)h[1];
    return DA_OK;
}

const char* da_spmm_algo_name(int algo)
{
    return (algo >= 0 && algo < DA_NUM_ALGOS) ? kNames[algo] : nullptr;
}

const char* da_spmm_last_error(void) { return g_err; }

}  // extern "C"
