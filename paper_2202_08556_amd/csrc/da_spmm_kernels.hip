// HIP kernels of the DA-SpMM algorithm space for gfx950 (MI355X, wave64).
//
// Four kernel templates cover the 8 algorithms of the paper's Table 1:
//
//                     K-loop SR (Sec. 3.4 K1)        K-loop PR (Sec. 3.4 K2, Sec. 4)
//   M-loop RB (M1)    rb_sr_kernel<V,G>              rb_pr_kernel<V,G>
//   M-loop EB (M2)    eb_sr_kernel<V,G>              eb_pr_kernel<V,G>   (conditional reduction)
//
// The N-loop axis (Sec. 3.3) is the template parameter G = number of neighbouring lanes that share
// one stored entry and hold neighbouring column vectors of the B row it points to:
//   RM mapping: G = smallest power of two >= N/V (a lane group reads one contiguous B row segment)
//   CM mapping: G = 1 (neighbouring lanes hold different rows / entries; each lane owns a strip of
//               V columns; further strips are further grid.y tiles)
// V = 1, 2 or 4 is the number of consecutive columns a lane loads at once (the float2/float4
// technique of Sec. 4).  B and C are row-major in memory in every case.
//
// Column tiles: a lane group covers G*V columns; blockIdx.y selects the tile.
//
// No MFMA anywhere: every multiply-add consumes a freshly gathered B operand, there is no dense
// tile to contract.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace daspmm {

constexpr int kWave = 64;
constexpr int kBlock = 256;                 // 4 waves
constexpr int kWavesPerBlock = kBlock / kWave;

// ------------------------------------------------------------------------------------------
// small helpers
// ------------------------------------------------------------------------------------------
template <int V>
__device__ __forceinline__ void load_vec(const float* __restrict__ p, float (&x)[V]) {
    if constexpr (V == 4) {
        const float4 t = *reinterpret_cast<const float4*>(p);
        x[0] = t.x; x[1] = t.y; x[2] = t.z; x[3] = t.w;
    } else if constexpr (V == 2) {
        const float2 t = *reinterpret_cast<const float2*>(p);
        x[0] = t.x; x[1] = t.y;
    } else {
        x[0] = *p;
    }
}

template <int V>
__device__ __forceinline__ void store_vec(float* __restrict__ p, const float (&x)[V]) {
    if constexpr (V == 4) {
        *reinterpret_cast<float4*>(p) = make_float4(x[0], x[1], x[2], x[3]);
    } else if constexpr (V == 2) {
        *reinterpret_cast<float2*>(p) = make_float2(x[0], x[1]);
    } else {
        *p = x[0];
    }
}

// Rows shared between workers are combined with hardware fp32 atomic adds (Sec. 4: "atomic_add"
// for rows assigned to different workers); the return value is not used.
template <int V>
__device__ __forceinline__ void atomic_add_vec(float* __restrict__ p, const float (&x)[V]) {
#pragma unroll
    for (int v = 0; v < V; ++v) unsafeAtomicAdd(p + v, x[v]);
}

template <int V>
__device__ __forceinline__ void emit_vec(float* __restrict__ p, const float (&x)[V], bool atomic) {
    if (atomic) atomic_add_vec<V>(p, x); else store_vec<V>(p, x);
}

template <int V>
__device__ __forceinline__ void fma_vec(float (&acc)[V], float a, const float (&b)[V]) {
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] = fmaf(a, b[v], acc[v]);
}

// Orders LDS traffic of the lanes of one wave: the LDS unit serves one wave's requests in issue
// order, so only the compiler has to be kept from moving accesses across this point.
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Smallest r in [lo, hi] with rowptr[r+1] > q: the row that owns stored entry q (rows without
// entries are skipped).  Requires rowptr[lo] <= q < rowptr[hi+1].
__device__ __forceinline__ int row_of_entry(const int* __restrict__ rowptr, int lo, int hi, int q) {
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (rowptr[mid + 1] > q) hi = mid; else lo = mid + 1;
    }
    return lo;
}

// ------------------------------------------------------------------------------------------
// RB + SR : a lane group owns a row and adds its products one after another
// (Sec. 3.2 design M1, Sec. 3.4 design K1).  The group's G lanes load G stored entries with one
// coalesced request and pass them round through LDS so that every entry is fetched once and
// reused for all columns of the tile (the sparse-element cache of Sec. 4).
// ------------------------------------------------------------------------------------------
template <int V, int G>
__global__ __launch_bounds__(kBlock) void rb_sr_kernel(
    int m, int N, const int* __restrict__ rowptr, const int* __restrict__ colind,
    const float* __restrict__ vals, const float* __restrict__ B, float* __restrict__ C)
{
    constexpr int RPW = kWave / G;                       // rows per wave
    __shared__ int2 stage[G > 1 ? kBlock : 1];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int g = lane / G, j = lane % G;
    const long row = ((long)blockIdx.x * kWavesPerBlock + wave) * RPW + g;
    const int n0 = (blockIdx.y * G + j) * V;
    const bool nok = n0 < N;
    int start = 0, end = 0;
    if (row < m) { start = rowptr[row]; end = rowptr[row + 1]; }
    float acc[V];
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] = 0.f;
    const float* __restrict__ Bn = B + n0;

    if constexpr (G == 1) {
        if (nok) {
#pragma unroll 4
            for (int p = start; p < end; ++p) {
                const int c = colind[p];
                const float a = vals[p];
                float b[V];
                load_vec<V>(Bn + (long)c * N, b);
                fma_vec<V>(acc, a, b);
            }
        }
    } else {
        int2* st = stage + wave * kWave + g * G;
        for (int p0 = start; p0 < end; p0 += G) {
            const int p = p0 + j;
            int2 e = make_int2(0, 0);
            if (p < end) { e.x = colind[p]; e.y = __float_as_int(vals[p]); }
            st[j] = e;
            wave_lds_sync();
            const int cnt = min(G, end - p0);
            if (nok) {
#pragma unroll 4
                for (int t = 0; t < cnt; ++t) {
                    const int2 ee = st[t];
                    float b[V];
                    load_vec<V>(Bn + (long)ee.x * N, b);
                    fma_vec<V>(acc, __int_as_float(ee.y), b);
                }
            }
            wave_lds_sync();
        }
    }
    if (row < m && nok) store_vec<V>(C + row * N + n0, acc);
}

// ------------------------------------------------------------------------------------------
// RB + PR : a wave owns a row; its 64 lanes form S = 64/G slots along the row's stored entries
// (times G lanes along n).  Rows longer than S are walked with a for-loop (technique 1 of Sec. 4),
// lanes load V consecutive columns at once (technique 2), the wave's entries are fetched once and
// shared through LDS (technique 3), and the slots are combined by a reduction tree (Sec. 3.4 K2).
// ------------------------------------------------------------------------------------------
template <int V, int G>
__global__ __launch_bounds__(kBlock) void rb_pr_kernel(
    int m, int N, const int* __restrict__ rowptr, const int* __restrict__ colind,
    const float* __restrict__ vals, const float* __restrict__ B, float* __restrict__ C)
{
    constexpr int S = kWave / G;
    __shared__ int2 stage[G > 1 ? kBlock : 1];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int s = lane / G, j = lane % G;
    const long row = (long)blockIdx.x * kWavesPerBlock + wave;
    if (row >= m) return;                                 // whole wave leaves together
    const int n0 = (blockIdx.y * G + j) * V;
    const bool nok = n0 < N;
    const int start = rowptr[row], end = rowptr[row + 1];
    float acc[V];
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] = 0.f;
    const float* __restrict__ Bn = B + n0;

    if constexpr (G == 1) {
        if (nok) {
            for (int p = start + lane; p < end; p += kWave) {
                const int c = colind[p];
                const float a = vals[p];
                float b[V];
                load_vec<V>(Bn + (long)c * N, b);
                fma_vec<V>(acc, a, b);
            }
        }
    } else {
        int2* st = stage + wave * kWave;
        for (int p0 = start; p0 < end; p0 += kWave) {
            const int p = p0 + lane;
            int2 e = make_int2(0, 0);
            if (p < end) { e.x = colind[p]; e.y = __float_as_int(vals[p]); }
            st[lane] = e;
            wave_lds_sync();
            const int cnt = min(kWave, end - p0);
            if (nok) {
#pragma unroll 2
                for (int t = s; t < cnt; t += S) {
                    const int2 ee = st[t];
                    float b[V];
                    load_vec<V>(Bn + (long)ee.x * N, b);
                    fma_vec<V>(acc, __int_as_float(ee.y), b);
                }
            }
            wave_lds_sync();
        }
    }
    // reduction tree over the slots: lanes with equal j
#pragma unroll
    for (int d = kWave / 2; d >= G; d >>= 1) {
#pragma unroll
        for (int v = 0; v < V; ++v) acc[v] += __shfl_down(acc[v], d, kWave);
    }
    if (s == 0 && nok) store_vec<V>(C + row * N + n0, acc);
}

// ------------------------------------------------------------------------------------------
// EB pre-pass.  EB workers own fixed-size chunks of consecutive stored entries (Sec. 3.2 design
// M2).  A row whose entries all fall into one chunk is written by exactly one worker with a plain
// store; a row that straddles a chunk boundary receives atomic additions from several workers and
// must start from zero; a row without entries is touched by no worker.  This pass zeroes exactly
// those two kinds of rows so that C needs no full memset.  `chunk` is the number of entries per
// worker of the product kernel that follows.
// ------------------------------------------------------------------------------------------
template <int V, int G>
__global__ __launch_bounds__(kBlock) void eb_zero_kernel(
    int m, int N, const int* __restrict__ rowptr, float* __restrict__ C, int chunk)
{
    constexpr int RPW = kWave / G;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int g = lane / G, j = lane % G;
    const long row = ((long)blockIdx.x * kWavesPerBlock + wave) * RPW + g;
    if (row >= m) return;
    const int start = rowptr[row], end = rowptr[row + 1];
    const bool need = (end == start) || (start / chunk != (end - 1) / chunk);
    if (!need) return;
    float z[V];
#pragma unroll
    for (int v = 0; v < V; ++v) z[v] = 0.f;
    for (int n0 = j * V; n0 < N; n0 += G * V) store_vec<V>(C + row * N + n0, z);
}

// ------------------------------------------------------------------------------------------
// EB + SR : a lane group owns `chunk` consecutive stored entries and walks them in order,
// keeping (partial sum, row).  When the row changes the partial is written: plain store if the
// row lies wholly inside the chunk, atomic add for the first / last row when it is shared with the
// neighbouring chunk (the "partial sum aggregation among workers" of Sec. 3.2).  The row of the
// chunk's first entry is found by binary search in rowptr (the "row index calculation" overhead
// named there).  Workers stride over the chunks so that the grid size does not depend on nnz,
// which only the device knows.
// ------------------------------------------------------------------------------------------
template <int V, int G>
__global__ __launch_bounds__(kBlock) void eb_sr_kernel(
    int m, int N, const int* __restrict__ rowptr, const int* __restrict__ colind,
    const float* __restrict__ vals, const float* __restrict__ B, float* __restrict__ C, int chunk)
{
    constexpr int GPW = kWave / G;                        // workers per wave
    __shared__ int2 stage[G > 1 ? kBlock : 1];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int g = lane / G, j = lane % G;
    const int n0 = (blockIdx.y * G + j) * V;
    const bool nok = n0 < N;
    const float* __restrict__ Bn = B + n0;
    float* __restrict__ Cn = C + n0;
    const int nnz = rowptr[m];
    const long nworkers = (long)gridDim.x * kWavesPerBlock * GPW;
    const long worker = ((long)blockIdx.x * kWavesPerBlock + wave) * GPW + g;
    int2* st = stage + (G > 1 ? wave * kWave + g * G : 0);

    for (long c0l = worker * chunk; c0l < nnz; c0l += nworkers * chunk) {
        const int c0 = (int)c0l;
        const int c1 = (int)min(c0l + chunk, (long)nnz);
        int row = row_of_entry(rowptr, 0, m - 1, c0);
        int row_end = rowptr[row + 1];
        bool shared_with_prev = rowptr[row] < c0;          // only the chunk's first row can be
        float acc[V];
#pragma unroll
        for (int v = 0; v < V; ++v) acc[v] = 0.f;

        for (int q0 = c0; q0 < c1; q0 += G) {
            if constexpr (G > 1) {
                const int q = q0 + j;
                int2 e = make_int2(0, 0);
                if (q < c1) { e.x = colind[q]; e.y = __float_as_int(vals[q]); }
                st[j] = e;
                wave_lds_sync();
            }
            const int cnt = min(G, c1 - q0);
            int t = 0;
            while (t < cnt) {
                const int stop = min(cnt, row_end - q0);
                for (; t < stop; ++t) {
                    int2 ee;
                    if constexpr (G > 1) ee = st[t];
                    else ee = make_int2(colind[q0], __float_as_int(vals[q0]));
                    if (nok) {
                        float b[V];
                        load_vec<V>(Bn + (long)ee.x * N, b);
                        fma_vec<V>(acc, __int_as_float(ee.y), b);
                    }
                }
                if (q0 + t == row_end) {                   // the row is complete
                    if (nok) emit_vec<V>(Cn + (long)row * N, acc, shared_with_prev);
#pragma unroll
                    for (int v = 0; v < V; ++v) acc[v] = 0.f;
                    shared_with_prev = false;
                    if (q0 + t < c1) {
                        do { ++row; row_end = rowptr[row + 1]; } while (row_end <= q0 + t);
                    }
                }
            }
            if constexpr (G > 1) wave_lds_sync();
        }
        if (row_end > c1 && nok)                           // last row continues in the next chunk
            emit_vec<V>(Cn + (long)row * N, acc, true);
    }
}

// ------------------------------------------------------------------------------------------
// EB + PR : a wave owns `chunk` consecutive stored entries and takes them 64 at a time.  The
// lanes form S = 64/G slots (times G lanes along n); in one step slot s holds the product vector
// of one entry together with that entry's row index.  The slots are combined with the
// CONDITIONAL REDUCTION of Sec. 4 (Fig. 6(e)): a log-step network in which slot s adds the value
// of slot s+d only if both carry the same row index.  Because entries are stored row after row,
// afterwards the leftmost slot of every run of equal indices holds the sum of the run (the
// validity rule of Sec. 4).  Runs that end inside the step are written by their leftmost slot;
// the run that reaches the last slot and whose row is not finished is carried into the next step.
// Rows that are complete inside the chunk get one plain store; only the first and last row of a
// chunk, when shared with the neighbouring chunks, are combined with atomic adds.
// ------------------------------------------------------------------------------------------
template <int V, int G>
__global__ __launch_bounds__(kBlock) void eb_pr_kernel(
    int m, int N, const int* __restrict__ rowptr, const int* __restrict__ colind,
    const float* __restrict__ vals, const float* __restrict__ B, float* __restrict__ C, int chunk)
{
    constexpr int S = kWave / G;
    __shared__ int4 stage[G > 1 ? kBlock : 1];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int s = lane / G, j = lane % G;
    const int n0 = (blockIdx.y * G + j) * V;
    const bool nok = n0 < N;
    const float* __restrict__ Bn = B + n0;
    float* __restrict__ Cn = C + n0;
    const int nnz = rowptr[m];
    const long nwaves = (long)gridDim.x * kWavesPerBlock;
    const long wave_id = (long)blockIdx.x * kWavesPerBlock + wave;
    int4* st = stage + (G > 1 ? wave * kWave : 0);

    for (long c0l = wave_id * chunk; c0l < nnz; c0l += nwaves * chunk) {
        const int c0 = (int)c0l;
        const int c1 = (int)min(c0l + chunk, (long)nnz);
        const int row_lo = row_of_entry(rowptr, 0, m - 1, c0);
        const int row_hi = row_of_entry(rowptr, row_lo, m - 1, c1 - 1);
        float carry[V];
#pragma unroll
        for (int v = 0; v < V; ++v) carry[v] = 0.f;
        int carry_row = -1;
        bool carry_started = false;

        for (int q0 = c0; q0 < c1; q0 += kWave) {
            // every lane fetches one entry and finds its row (binary search restricted to the
            // rows of this chunk) and whether it is the first / last entry of that row
            const int q = q0 + lane;
            int4 mine = make_int4(0, 0, -1, 0);
            if (q < c1) {
                const int r = row_of_entry(rowptr, row_lo, row_hi, q);
                mine.x = colind[q];
                mine.y = __float_as_int(vals[q]);
                mine.z = r;
                mine.w = (q == rowptr[r] ? 1 : 0) | (q + 1 == rowptr[r + 1] ? 2 : 0);
            }
            if constexpr (G > 1) { st[lane] = mine; wave_lds_sync(); }
            const int cnt = min(kWave, c1 - q0);

            for (int t0 = 0; t0 < cnt; t0 += S) {
                int4 e;
                if constexpr (G > 1) e = st[t0 + s]; else e = mine;
                const bool evalid = t0 + s < cnt;
                const int er = e.z;
                float x[V];
#pragma unroll
                for (int v = 0; v < V; ++v) x[v] = 0.f;
                if (evalid && nok) {
                    float b[V];
                    load_vec<V>(Bn + (long)e.x * N, b);
                    const float a = __int_as_float(e.y);
#pragma unroll
                    for (int v = 0; v < V; ++v) x[v] = a * b[v];
                }
                // conditional reduction network over the slots
#pragma unroll
                for (int d = 1; d < S; d <<= 1) {
                    const int orow = __shfl_down(er, d * G, kWave);
                    const bool take = (s + d < S) && (orow == er);
#pragma unroll
                    for (int v = 0; v < V; ++v) {
                        const float ox = __shfl_down(x[v], d * G, kWave);
                        if (take) x[v] += ox;
                    }
                }
                const int prow = __shfl_up(er, G, kWave);
                const bool head = evalid && (s == 0 || prow != er);
                const int nv = min(S, cnt - t0);                       // valid slots in this step
                const int tail_lane = (nv - 1) * G;
                const int tail_row = __shfl(er, tail_lane, kWave);
                const bool tail_ended = (__shfl(e.w, tail_lane, kWave) & 2) != 0;
                bool started = (e.w & 1) != 0;
                if (s == 0 && carry_row == er) {                        // continue the carried run
#pragma unroll
                    for (int v = 0; v < V; ++v) x[v] += carry[v];
                    started = carry_started;
                }
                const bool in_tail_run = evalid && er == tail_row;
                if (head && nok && (!in_tail_run || tail_ended))
                    emit_vec<V>(Cn + (long)er * N, x, !started);
                if (!tail_ended) {
                    // leftmost slot of the tail run -> every slot keeps a copy of the carry
                    const unsigned long long mask = __ballot(in_tail_run);
                    const int src = (__ffsll((long long)mask) - 1) / G * G + j;
#pragma unroll
                    for (int v = 0; v < V; ++v) carry[v] = __shfl(x[v], src, kWave);
                    carry_started = __shfl((int)started, src, kWave) != 0;
                    carry_row = tail_row;
                } else {
                    carry_row = -1;
                }
            }
            if constexpr (G > 1) wave_lds_sync();
        }
        if (carry_row >= 0 && s == 0 && nok)                 // row continues in the next chunk
            emit_vec<V>(Cn + (long)carry_row * N, carry, true);
    }
}

// ------------------------------------------------------------------------------------------
// Input characteristics (Sec. 5.1, Table 2): sum of squared row lengths and the longest row,
// reduced exactly in integers.  out[0] += sum len^2, out[1] = max len, out[2] = nnz.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void features_kernel(
    int m, const int* __restrict__ rowptr, unsigned long long* __restrict__ out)
{
    __shared__ unsigned long long s_sq[kWavesPerBlock];
    __shared__ unsigned long long s_mx[kWavesPerBlock];
    unsigned long long sq = 0, mx = 0;
    for (long i = (long)blockIdx.x * kBlock + threadIdx.x; i < m; i += (long)gridDim.x * kBlock) {
        const unsigned long long len = (unsigned long long)(rowptr[i + 1] - rowptr[i]);
        sq += len * len;
        mx = len > mx ? len : mx;
    }
#pragma unroll
    for (int d = kWave / 2; d >= 1; d >>= 1) {
        sq += __shfl_down(sq, d, kWave);
        const unsigned long long o = __shfl_down(mx, d, kWave);
        mx = o > mx ? o : mx;
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) { s_sq[wave] = sq; s_mx[wave] = mx; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kWavesPerBlock; ++w) { sq += s_sq[w]; mx = s_mx[w] > mx ? s_mx[w] : mx; }
        atomicAdd(out + 0, sq);
        atomicMax(out + 1, mx);
        if (blockIdx.x == 0) out[2] = (unsigned long long)rowptr[m];
    }
}

}  // namespace daspmm
