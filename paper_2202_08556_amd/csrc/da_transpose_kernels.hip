// CSR transpose for gfx950 (wave64): the CSR arrays of A^T from those of A, needed by the backward
// pass of a graph-convolution layer (the GCN application of Sec. 6), where the gradient of
// <G, A.X> with respect to X is A^T.G and is computed by the same SpMM kernels on A^T.
//
// Row j of A^T lists the stored entries of column j of A with ascending row numbers.  CSR stores
// entries row after row, so a STABLE sort of the entry numbers by column index is exactly that
// order, and it is deterministic (no atomic cursors).  The sort is a least-significant-digit radix
// sort with 10-bit digits; one pass is
//     radix_count_kernel    per-block digit histogram                       -> hist[digit][block]
//     scan_*_kernel         exclusive prefix sum over hist in that order    (three small kernels)
//     radix_scatter_kernel  stable scatter: position = scanned hist entry + number of earlier
//                           entries of the block with the same digit
// Inside a block each wave owns a contiguous run of entries and walks it 64 entries at a time; the
// lanes that hold the same digit find each other with one ballot per digit bit, so the rank of an
// entry among its peers is a population count and only one lane per distinct digit touches the
// wave's running counter in LDS.
// The last pass writes the transposed arrays directly (the row number of an entry comes from a
// binary search in rowptr, its value from vals) together with the sorted keys, from which the new
// row pointers follow by one lower-bound search per row.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace daspmm {

constexpr int kRadixBits = 10;
constexpr int kBins = 1 << kRadixBits;
constexpr int kSortBlock = 256;
constexpr int kSortWaves = kSortBlock / 64;
constexpr int kSortRounds = 32;                          // 64-entry rounds per wave and block
constexpr int kSortWaveRun = kSortRounds * 64;           // consecutive entries owned by one wave
constexpr int kSortTile = kSortWaves * kSortWaveRun;     // entries per block
constexpr int kScanPerThread = 16;
constexpr int kScanChunk = kSortBlock * kScanPerThread;  // ints per block in the scan kernels

__device__ __forceinline__ int digit_of(int key, int shift) { return (key >> shift) & (kBins - 1); }

// Lanes of the wave that are valid and hold the same digit as the caller (meaningless for a lane
// that is not valid).  Every lane of the wave must call it.
__device__ __forceinline__ unsigned long long digit_peers(int d, bool valid) {
    unsigned long long peers = __ballot(valid);
#pragma unroll
    for (int b = 0; b < kRadixBits; ++b) {
        const bool bit = (d >> b) & 1;
        const unsigned long long vote = __ballot(bit && valid);
        peers &= bit ? vote : ~vote;
    }
    return peers;
}

__device__ __forceinline__ int wave_inclusive_scan(int v, int lane) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int t = __shfl_up(v, d);
        if (lane >= d) v += t;
    }
    return v;
}

// Exclusive prefix of v over the 256 threads of the block; *total receives the block sum.
// sh: kSortWaves ints of LDS.  All threads must call it.
__device__ __forceinline__ int block_exclusive_scan(int v, int* sh, int* total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int inc = wave_inclusive_scan(v, lane);
    __syncthreads();                                     // sh may still be read from a previous call
    if (lane == 63) sh[wave] = inc;
    __syncthreads();
    int off = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kSortWaves; ++w) {
        const int s = sh[w];
        if (w < wave) off += s;
        tot += s;
    }
    *total = tot;
    return off + inc - v;
}

// ------------------------------------------------------------------------------------------
// exclusive prefix sum of an int array, in place: reduce per chunk, scan the chunk sums in one
// block, then scan every chunk with its base
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kSortBlock) void scan_reduce_kernel(const int* __restrict__ data, long len,
                                                                 int* __restrict__ part)
{
    __shared__ int sh[kSortWaves];
    const long base = (long)blockIdx.x * kScanChunk;
    int s = 0;
    for (int j = 0; j < kScanPerThread; ++j) {
        const long i = base + j * kSortBlock + threadIdx.x;
        if (i < len) s += data[i];
    }
    int total;
    block_exclusive_scan(s, sh, &total);
    if (threadIdx.x == 0) part[blockIdx.x] = total;
}

__global__ __launch_bounds__(kSortBlock) void scan_top_kernel(int* __restrict__ part, int count)
{
    __shared__ int sh[kSortWaves];
    int carry = 0;
    for (int base = 0; base < count; base += kSortBlock) {
        const int i = base + threadIdx.x;
        const int v = i < count ? part[i] : 0;
        int total;
        const int ex = block_exclusive_scan(v, sh, &total);
        if (i < count) part[i] = carry + ex;
        carry += total;
    }
}

__global__ __launch_bounds__(kSortBlock) void scan_apply_kernel(int* __restrict__ data, long len,
                                                                const int* __restrict__ part)
{
    __shared__ int sh[kSortWaves];
    const long first = (long)blockIdx.x * kScanChunk + (long)threadIdx.x * kScanPerThread;
    int x[kScanPerThread];
    int s = 0;
#pragma unroll
    for (int j = 0; j < kScanPerThread; ++j) {
        x[j] = first + j < len ? data[first + j] : 0;
        s += x[j];
    }
    int total;
    int run = part[blockIdx.x] + block_exclusive_scan(s, sh, &total);
#pragma unroll
    for (int j = 0; j < kScanPerThread; ++j) {
        if (first + j < len) data[first + j] = run;
        run += x[j];
    }
}

// ------------------------------------------------------------------------------------------
// one radix pass
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kSortBlock) void radix_count_kernel(const int* __restrict__ keys, int n, int shift,
                                                                 int* __restrict__ hist, int nblocks)
{
    __shared__ int cnt[kBins];
    for (int d = threadIdx.x; d < kBins; d += kSortBlock) cnt[d] = 0;
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const long wbase = (long)blockIdx.x * kSortTile + (long)wave * kSortWaveRun;
    for (int r = 0; r < kSortRounds; ++r) {
        const long e = wbase + r * 64 + lane;
        const bool valid = e < n;
        const int d = valid ? digit_of(keys[e], shift) : 0;
        const unsigned long long peers = digit_peers(d, valid);
        if (valid && lane == __ffsll((long long)peers) - 1) atomicAdd(&cnt[d], __popcll(peers));
    }
    __syncthreads();
    for (int d = threadIdx.x; d < kBins; d += kSortBlock) hist[(long)d * nblocks + blockIdx.x] = cnt[d];
}

// Smallest r in [0, m-1] with rowptr[r+1] > e: the row that owns stored entry e.
__device__ __forceinline__ int owner_row(const int* __restrict__ rowptr, int m, int e) {
    int lo = 0, hi = m - 1;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (rowptr[mid + 1] > e) hi = mid; else lo = mid + 1;
    }
    return lo;
}

// hist holds the exclusive prefix sums of the pass's histograms.  idx_in == nullptr means that the
// payload of entry e is e itself (first pass).  FINAL: besides the sorted keys, write the row
// number and value of every entry at its sorted position instead of the payload.
template <bool FINAL>
__global__ __launch_bounds__(kSortBlock) void radix_scatter_kernel(
    const int* __restrict__ keys_in, const int* __restrict__ idx_in, int n, int shift,
    const int* __restrict__ hist, int nblocks, int* __restrict__ keys_out, int* __restrict__ idx_out,
    const int* __restrict__ rowptr, int m, const float* __restrict__ vals,
    int* __restrict__ t_colind, float* __restrict__ t_vals)
{
    __shared__ int wcnt[kSortWaves][kBins];
    for (int d = threadIdx.x; d < kSortWaves * kBins; d += kSortBlock) (&wcnt[0][0])[d] = 0;
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const long wbase = (long)blockIdx.x * kSortTile + (long)wave * kSortWaveRun;
    // digits per wave
    for (int r = 0; r < kSortRounds; ++r) {
        const long e = wbase + r * 64 + lane;
        const bool valid = e < n;
        const int d = valid ? digit_of(keys_in[e], shift) : 0;
        const unsigned long long peers = digit_peers(d, valid);
        if (valid && lane == __ffsll((long long)peers) - 1) atomicAdd(&wcnt[wave][d], __popcll(peers));
    }
    __syncthreads();
    // counts -> first output position of every (wave, digit)
    for (int d = threadIdx.x; d < kBins; d += kSortBlock) {
        int b = hist[(long)d * nblocks + blockIdx.x];
#pragma unroll
        for (int w = 0; w < kSortWaves; ++w) {
            const int c = wcnt[w][d];
            wcnt[w][d] = b;
            b += c;
        }
    }
    __syncthreads();
    // stable scatter: rounds in order, peers ranked by lane number
    for (int r = 0; r < kSortRounds; ++r) {
        const long e = wbase + r * 64 + lane;
        const bool valid = e < n;
        const int key = valid ? keys_in[e] : 0;
        const int d = digit_of(key, shift);
        const unsigned long long peers = digit_peers(d, valid);
        const int leader = __ffsll((long long)peers) - 1;
        int first = 0;
        if (valid && lane == leader) first = atomicAdd(&wcnt[wave][d], __popcll(peers));
        first = __shfl(first, leader & 63);
        if (valid) {
            const int pos = first + __popcll(peers & ((1ull << lane) - 1ull));
            const int idx = idx_in ? idx_in[e] : (int)e;
            keys_out[pos] = key;
            if constexpr (FINAL) {
                t_colind[pos] = owner_row(rowptr, m, idx);
                t_vals[pos] = vals[idx];
            } else {
                idx_out[pos] = idx;
            }
        }
    }
}

// t_rowptr[c] = number of stored entries with column index < c, for c = 0..k.
__global__ __launch_bounds__(kSortBlock) void rowptr_from_sorted_kernel(const int* __restrict__ keys, int n, int k,
                                                                        int* __restrict__ t_rowptr)
{
    const long c = (long)blockIdx.x * kSortBlock + threadIdx.x;
    if (c > k) return;
    int lo = 0, hi = n;                                   // first position whose key is >= c
    while (lo < hi) {
        const int mid = (int)(((long)lo + hi) >> 1);
        if (keys[mid] < c) lo = mid + 1; else hi = mid;
    }
    t_rowptr[c] = lo;
}

}  // namespace daspmm
