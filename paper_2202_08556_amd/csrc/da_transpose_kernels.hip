// CSR transpose for gfx950 (wave64): the CSR arrays of A^T from those of A, needed by the backward
// pass of a graph-convolution layer (the GCN application of Sec. 6), where the gradient of
// <G, A.X> with respect to X is A^T.G and is computed by the same SpMM kernels on A^T.
//
// Row j of A^T lists the stored entries of column j of A with ascending row numbers.  CSR stores
// entries row after row, so a STABLE sort of the entries by column index is exactly that order,
// and it is deterministic (no atomic cursors on global memory).  The sort is a least-significant-
// digit radix sort of (column, row, value) triples with digits of at most 8 bits; one pass is
//     radix_count_kernel    per-block digit histogram                       -> hist[digit][block]
//     scan_*_kernel         exclusive prefix sum over hist in that order    (three small kernels)
//     radix_scatter_kernel  stable scatter: position = scanned hist entry + number of earlier
//                           entries of the block with the same digit
// Inside a block each wave owns a contiguous run of entries and walks it 64 entries at a time; the
// lanes that hold the same digit find each other with one ballot per digit bit, so the rank of an
// entry among its peers is a population count and only one lane per distinct digit touches the
// wave's running counter in LDS.  The block first orders its tile by digit in LDS and then copies
// it out, so that entries with the same digit leave as contiguous runs (coalesced stores) rather
// than as single 4-byte stores.
// The first pass reads colind / vals and derives the row number of every entry from rowptr; the
// last pass writes straight into the arrays of A^T (row numbers become its column indices) plus
// the sorted keys, from which the new row pointers follow by one lower-bound search per row.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace daspmm {

constexpr int kRadixBits = 8;                            // widest digit
constexpr int kBins = 1 << kRadixBits;
constexpr int kSortBlock = 256;                          // one thread per bin in the bookkeeping steps
constexpr int kSortWaves = kSortBlock / 64;
constexpr int kSortRounds = 16;                          // 64-entry rounds per wave and block
constexpr int kSortWaveRun = kSortRounds * 64;           // consecutive entries owned by one wave
constexpr int kSortTile = kSortWaves * kSortWaveRun;     // entries per block
constexpr int kScanPerThread = 16;
constexpr int kScanChunk = kSortBlock * kScanPerThread;  // ints per block in the scan kernels

static_assert(kBins == kSortBlock, "bookkeeping maps one thread to one bin");

__device__ __forceinline__ int digit_of(int key, int shift, int mask) { return (key >> shift) & mask; }

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
__device__ __forceinline__ void scan_reduce_body(unsigned bx, const int* __restrict__ data, long len,
                                                 int* __restrict__ part)
{
    __shared__ int sh[kSortWaves];
    const long base = (long)bx * kScanChunk;
    int s = 0;
    for (int j = 0; j < kScanPerThread; ++j) {
        const long i = base + j * kSortBlock + threadIdx.x;
        if (i < len) s += data[i];
    }
    int total;
    block_exclusive_scan(s, sh, &total);
    if (threadIdx.x == 0) part[bx] = total;
}

__global__ __launch_bounds__(kSortBlock) void scan_reduce_kernel(const int* __restrict__ data, long len,
                                                                 int* __restrict__ part)
{
    scan_reduce_body(blockIdx.x, data, len, part);
}

__device__ __forceinline__ void scan_top_body(int* __restrict__ part, int count)
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

__global__ __launch_bounds__(kSortBlock) void scan_top_kernel(int* __restrict__ part, int count)
{
    scan_top_body(part, count);
}

__device__ __forceinline__ void scan_apply_body(unsigned bx, int* __restrict__ data, long len,
                                                const int* __restrict__ part)
{
    __shared__ int sh[kSortWaves];
    const long first = (long)bx * kScanChunk + (long)threadIdx.x * kScanPerThread;
    int x[kScanPerThread];
    int s = 0;
#pragma unroll
    for (int j = 0; j < kScanPerThread; ++j) {
        x[j] = first + j < len ? data[first + j] : 0;
        s += x[j];
    }
    int total;
    int run = part[bx] + block_exclusive_scan(s, sh, &total);
#pragma unroll
    for (int j = 0; j < kScanPerThread; ++j) {
        if (first + j < len) data[first + j] = run;
        run += x[j];
    }
}

__global__ __launch_bounds__(kSortBlock) void scan_apply_kernel(int* __restrict__ data, long len,
                                                                const int* __restrict__ part)
{
    scan_apply_body(blockIdx.x, data, len, part);
}

// Smallest r in [lo, hi] with rowptr[r+1] > e: the row that owns stored entry e, given that it
// lies in [lo, hi].
__device__ __forceinline__ int owner_row(const int* __restrict__ rowptr, int lo, int hi, int e) {
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (rowptr[mid + 1] > e) hi = mid; else lo = mid + 1;
    }
    return lo;
}

// ------------------------------------------------------------------------------------------
// one radix pass; digit = (key >> shift) & mask with mask < kBins
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ void radix_count_body(unsigned bx, const int* __restrict__ keys, int n, int shift, int mask,
                                                 int* __restrict__ hist, int nblocks)
{
    __shared__ int cnt[kBins];
    cnt[threadIdx.x] = 0;
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const long wbase = (long)bx * kSortTile + (long)wave * kSortWaveRun;
    int key[kSortRounds];
#pragma unroll
    for (int r = 0; r < kSortRounds; ++r) {               // all loads of the lane in flight together;
        const long e = wbase + r * 64 + lane;             // clamped, so that they need no branch
        key[r] = keys[e < n ? e : n - 1];
    }
#pragma unroll
    for (int r = 0; r < kSortRounds; ++r) {
        const bool valid = wbase + r * 64 + lane < n;
        const int d = digit_of(key[r], shift, mask);
        const unsigned long long peers = digit_peers(d, valid);
        if (valid && lane == __ffsll((long long)peers) - 1) atomicAdd(&cnt[d], __popcll(peers));
        __builtin_amdgcn_sched_barrier(0);                // keep the ballots of one round together
    }
    __syncthreads();
    hist[(long)threadIdx.x * nblocks + bx] = cnt[threadIdx.x];
}

__global__ __launch_bounds__(kSortBlock) void radix_count_kernel(const int* __restrict__ keys, int n, int shift, int mask,
                                                                 int* __restrict__ hist, int nblocks)
{
    radix_count_body(blockIdx.x, keys, n, shift, mask, hist, nblocks);
}

// hist holds the exclusive prefix sums of the pass's histograms.  FIRST: the input is the matrix
// itself (keys_in = colind, vals_in = vals) and the row number of an entry is derived from rowptr;
// otherwise rows_in carries it.  The outputs of the last pass are the arrays of A^T.
template <bool FIRST>
__device__ __forceinline__ void radix_scatter_body(
    unsigned bx, const int* __restrict__ keys_in, const int* __restrict__ rows_in, const float* __restrict__ vals_in, int n,
    int shift, int mask, const int* __restrict__ hist, int nblocks,
    int* __restrict__ keys_out, int* __restrict__ rows_out, float* __restrict__ vals_out,
    const int* __restrict__ rowptr, int m)
{
    __shared__ int wcnt[kSortWaves][kBins];              // per wave and digit: count, then next slot in the tile
    __shared__ int gbase[kBins];                          // global position minus tile slot, per digit
    __shared__ int sh[kSortWaves];
    __shared__ int skey[kSortTile];
    __shared__ int srow[kSortTile];
    __shared__ float sval[kSortTile];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int w = 0; w < kSortWaves; ++w) wcnt[w][threadIdx.x] = 0;
    const long tbase = (long)bx * kSortTile;
    const long wbase = tbase + (long)wave * kSortWaveRun;
    const int tile_count = (int)min((long)kSortTile, (long)n - tbase);
    // the lane's 16 entries: every load is issued before the first one is used (indices clamped to
    // the last entry instead of branching; `valid` masks the surplus lanes of the last block)
    int key[kSortRounds], row[kSortRounds];
    float val[kSortRounds];
#pragma unroll
    for (int r = 0; r < kSortRounds; ++r) {
        const long e = wbase + r * 64 + lane;
        const long ec = e < n ? e : n - 1;
        key[r] = keys_in[ec];
        val[r] = vals_in[ec];
        if constexpr (!FIRST) row[r] = rows_in[ec];
    }
    if constexpr (FIRST) {
        // rows of the wave's run lie in [row_lo, row_hi]; the 16 searches of a lane advance together
        // so that their probes overlap
        int lo[kSortRounds], hi[kSortRounds];
        const long last = min(wbase + kSortWaveRun - 1, (long)n - 1);
        int row_lo = 0, row_hi = 0;
        if (wbase < n) {
            row_lo = owner_row(rowptr, 0, m - 1, (int)wbase);
            row_hi = owner_row(rowptr, row_lo, m - 1, (int)last);
        }
#pragma unroll
        for (int r = 0; r < kSortRounds; ++r) { lo[r] = row_lo; hi[r] = row_hi; }
        for (int span = row_hi - row_lo; span > 0; span >>= 1) {      // ceil(log2(span + 1)) steps
#pragma unroll
            for (int r = 0; r < kSortRounds; ++r) {
                const long e = wbase + r * 64 + lane;
                const int ec = (int)(e < last ? e : last);
                const int mid = (lo[r] + hi[r]) >> 1;
                if (rowptr[mid + 1] > ec) hi[r] = mid; else lo[r] = mid + 1;
            }
        }
#pragma unroll
        for (int r = 0; r < kSortRounds; ++r) row[r] = lo[r];
    }
    __syncthreads();
    // digits per wave; the peer masks are kept for the placement step
    unsigned long long peers[kSortRounds];
#pragma unroll
    for (int r = 0; r < kSortRounds; ++r) {
        const bool valid = wbase + r * 64 + lane < n;
        const int d = digit_of(key[r], shift, mask);
        peers[r] = valid ? digit_peers(d, valid) : 0ull;
        if (valid && lane == __ffsll((long long)peers[r]) - 1) atomicAdd(&wcnt[wave][d], __popcll(peers[r]));
        __builtin_amdgcn_sched_barrier(0);                // keep the ballots of one round together
    }
    __syncthreads();
    // thread d: counts of digit d -> first tile slot of every (wave, d), and the offset that turns
    // a tile slot of digit d into its global position
    {
        const int d = threadIdx.x;
        int c[kSortWaves], total = 0;
#pragma unroll
        for (int w = 0; w < kSortWaves; ++w) { c[w] = wcnt[w][d]; total += c[w]; }
        int all;
        int slot = block_exclusive_scan(total, sh, &all);
        gbase[d] = hist[(long)d * nblocks + bx] - slot;
#pragma unroll
        for (int w = 0; w < kSortWaves; ++w) { wcnt[w][d] = slot; slot += c[w]; }
    }
    __syncthreads();
    // stable placement inside the tile: rounds in order, peers ranked by lane number
#pragma unroll
    for (int r = 0; r < kSortRounds; ++r) {
        const bool valid = peers[r] != 0ull;              // a valid lane is its own peer
        const int d = digit_of(key[r], shift, mask);
        const int leader = __ffsll((long long)peers[r]) - 1;
        int first = 0;
        if (valid && lane == leader) first = atomicAdd(&wcnt[wave][d], __popcll(peers[r]));
        first = __shfl(first, leader & 63);
        if (valid) {
            const int slot = first + __popcll(peers[r] & ((1ull << lane) - 1ull));
            skey[slot] = key[r];
            srow[slot] = row[r];
            sval[slot] = val[r];
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    __syncthreads();
    // copy out: neighbouring tile slots of one digit are neighbouring global positions
    for (int i = threadIdx.x; i < tile_count; i += kSortBlock) {
        const int k2 = skey[i];
        const int pos = gbase[digit_of(k2, shift, mask)] + i;
        keys_out[pos] = k2;
        rows_out[pos] = srow[i];
        vals_out[pos] = sval[i];
    }
}

template <bool FIRST>
__global__ __launch_bounds__(kSortBlock) void radix_scatter_kernel(
    const int* __restrict__ keys_in, const int* __restrict__ rows_in, const float* __restrict__ vals_in, int n,
    int shift, int mask, const int* __restrict__ hist, int nblocks,
    int* __restrict__ keys_out, int* __restrict__ rows_out, float* __restrict__ vals_out,
    const int* __restrict__ rowptr, int m)
{
    radix_scatter_body<FIRST>(blockIdx.x, keys_in, rows_in, vals_in, n, shift, mask, hist, nblocks, keys_out, rows_out,
                              vals_out, rowptr, m);
}

// Sort keys of the EB schedule for unit u (the stored entries [u*unit, (u+1)*unit)), in [0, 2k).
// A unit inside one row covers a narrow column range and is keyed by the middle of that range,
// k + (first + last column index)/2: these units are swept over B in column order.  A unit that
// touches several rows is keyed by its first column index alone (units that start at the same
// place of rows of similar length walk the column range in step, so this aligns them too; for
// units of many short rows no order matters): all such units sort before the others and form a
// first segment of the schedule.  They walk row ends (stores, atomics, a row-pointer load each) and
// are latency-bound where the single-row units are bandwidth-bound; a wave that holds both kinds
// runs at the pace of the slower, so the kinds are kept apart, and the launch deals each segment
// to all XCDs.  count (one int, cleared first) receives the number of units of that segment.
// ids = 0, 1, 2, ...; the value slot of the triples the radix passes move carries, as a bit pattern,
// the row that owns the unit's first entry, so that the sort also delivers those rows in schedule order;
// rows_by_unit (may be null) receives the same rows indexed by unit number.
//
// Several schedules (one per chunk size) are built side by side: every kernel of the pipeline takes
// up to kMaxSortJobs jobs and blockIdx.y selects the job, so that the orders for all chunk sizes of
// a matrix cost the launches of one.
constexpr int kMaxSortJobs = 4;

struct SortJob {                       // one radix pass of one job (pointers change from pass to pass)
    const int* keys_in; const int* rows_in; const float* vals_in;
    int* keys_out; int* rows_out; float* vals_out;
    int* hist; int* part;
    long hist_len;
    int n, nblocks, parts;
};
struct SortJobs { SortJob j[kMaxSortJobs]; };

struct KeyJob {                        // key generation of one schedule
    int unit, nunits;
    int* keys; int* ids; float* pad; int* count; int* rows_by_unit;
};
struct KeyJobs { KeyJob j[kMaxSortJobs]; };

__global__ void schedule_clear_kernel(KeyJobs jobs, int njobs) {
    if ((int)threadIdx.x < njobs) *jobs.j[threadIdx.x].count = 0;
}

__global__ __launch_bounds__(kSortBlock) void radix_count_jobs_kernel(SortJobs jobs, int shift, int mask) {
    const SortJob J = jobs.j[blockIdx.y];
    if ((int)blockIdx.x < J.nblocks) radix_count_body(blockIdx.x, J.keys_in, J.n, shift, mask, J.hist, J.nblocks);
}
__global__ __launch_bounds__(kSortBlock) void scan_reduce_jobs_kernel(SortJobs jobs) {
    const SortJob J = jobs.j[blockIdx.y];
    if ((int)blockIdx.x < J.parts) scan_reduce_body(blockIdx.x, J.hist, J.hist_len, J.part);
}
__global__ __launch_bounds__(kSortBlock) void scan_top_jobs_kernel(SortJobs jobs) {
    const SortJob J = jobs.j[blockIdx.x];
    scan_top_body(J.part, J.parts);
}
__global__ __launch_bounds__(kSortBlock) void scan_apply_jobs_kernel(SortJobs jobs) {
    const SortJob J = jobs.j[blockIdx.y];
    if ((int)blockIdx.x < J.parts) scan_apply_body(blockIdx.x, J.hist, J.hist_len, J.part);
}
__global__ __launch_bounds__(kSortBlock) void radix_scatter_jobs_kernel(SortJobs jobs, int shift, int mask) {
    const SortJob J = jobs.j[blockIdx.y];
    if ((int)blockIdx.x < J.nblocks)
        radix_scatter_body<false>(blockIdx.x, J.keys_in, J.rows_in, J.vals_in, J.n, shift, mask, J.hist, J.nblocks, J.keys_out,
                                  J.rows_out, J.vals_out, nullptr, 0);
}

__global__ __launch_bounds__(kSortBlock) void schedule_keys_kernel(int m, int k, int nnz, const int* __restrict__ rowptr,
                                                                   const int* __restrict__ colind, KeyJobs jobs)
{
    const KeyJob J = jobs.j[blockIdx.y];
    const int unit = J.unit, nunits = J.nunits;
    int* __restrict__ keys = J.keys;
    int* __restrict__ ids = J.ids;
    float* __restrict__ pad = J.pad;
    int* __restrict__ count = J.count;
    int* __restrict__ rows_by_unit = J.rows_by_unit;
    const long u = (long)blockIdx.x * kSortBlock + threadIdx.x;
    if ((long)blockIdx.x * kSortBlock >= nunits) return;          // whole block beyond this job's units
    bool several = false;
    if (u < nunits) {
        const long c0 = u * unit;
        const long c1 = min(c0 + unit, (long)nnz) - 1;
        const int r0 = owner_row(rowptr, 0, m - 1, (int)c0);
        several = rowptr[r0 + 1] <= c1;
        keys[u] = several ? colind[c0] : k + (int)(((long)colind[c0] + (long)colind[c1]) >> 1);
        ids[u] = (int)u;
        pad[u] = __int_as_float(r0);
        if (rows_by_unit) rows_by_unit[u] = r0;
    }
    const unsigned long long vote = __ballot(several);
    if ((threadIdx.x & 63) == 0 && vote) atomicAdd(count, __popcll(vote));
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
