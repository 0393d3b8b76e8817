// HIP kernels of the DA-SpMM algorithm space for gfx950 (MI355X, wave64).
//
// Four kernel templates cover the 8 algorithms of the paper's Table 1:
//
//                     K-loop SR (Sec. 3.4 K1)        K-loop PR (Sec. 3.4 K2, Sec. 4)
//   M-loop RB (M1)    rb_sr_kernel<V,G,NV>           rb_pr_kernel<V,G,NV>
//   M-loop EB (M2)    eb_sr_kernel<V,G,NV>           eb_pr_kernel<V,G,NV>  (conditional reduction)
//
// The N-loop axis (Sec. 3.3) is the lane mapping, set by the template parameters:
//   G   neighbouring lanes that share one stored entry and hold neighbouring column vectors of
//       the B row it points to.  RM mapping: G > 1 (a lane group reads one contiguous B row
//       segment, coalesced).  CM mapping: G = 1 (neighbouring lanes hold different rows / entries).
//   V   consecutive columns a lane loads at once (the float2/float4 technique of Sec. 4): 1 or 4.
//   NV  vectors of V columns a lane walks one after another (CM: the lane's own strip of columns;
//       RM uses NV = 1).
// A lane group covers G*V*NV columns; further column tiles are further blocks (see block_map).
// B and C are row-major in memory in every case.
//
// Memory-level parallelism: the hot loops fetch U entries' B segments back to back into registers
// before the first multiply-add consumes them, so that every wave keeps U gathers in flight; row
// bookkeeping (EB) happens while those loads are outstanding.
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
constexpr int kU = 8;                       // gathers in flight per lane (4 ... 16 measured within 1 % on EB+RM+SR)

// Element strides of the dense operands: B(r, n) is at B[r*rb + n*cb], C(i, n) at C[i*rc + n*cc].
// Row-major storage has cb = cc = 1 and rb, rc = leading dimension; column-major storage has
// rb = rc = 1 and cb, cc = leading dimension.  Vector loads / stores (V = 4) need cb = cc = 1.
struct Strides {
    long rb, cb, rc, cc;
};

// Order in which the EB workers take the chunks of stored entries: worker u takes chunk order[u]
// instead of chunk u.  The order is a permutation of 0..units-1 built for a matrix with `nnz`
// stored entries and the chunk size of the launch; a kernel that finds another nnz on the device
// ignores it (order == nullptr: no schedule).
// stripe > 0: the schedule is dealt in stripes to the XCDs that work on it (see sweep_block): all 8,
// or the 8 / pin_tiles XCDs that share a column tile when tiles are pinned to XCDs (nx_log2 = log2
// of that number).  The schedule may consist of two segments that are dealt separately, blocks
// [0, split) in stripes of `stripe` blocks and the rest in stripes of `stripe_b`, so that every XCD
// gets the same share of both (split == 0: one segment).  per_a = blocks of the first segment per
// XCD, rounded up to whole stripes; vblocks = number of block positions to walk (XCDs * blocks per
// XCD over both segments; positions that fall outside a segment find no chunk).  The grid's x
// extent must be a multiple of 8 so that a block stays on its XCD when it makes more than one pass.
struct Schedule {
    const int* order;
    int units;
    int nnz;
    int stripe, split, per_a, stripe_b, vblocks, nx_log2;
    // first_row[u] (may be null): the row that owned the first entry of chunk order[u] when the
    // order was built.  A hint only: a worker checks it against the row pointers it finds (two
    // independent loads) and searches when it does not hold, so stale contents cost speed, never
    // correctness.
    const int* first_row;
    // row_by_chunk[c] (may be null): the same hint indexed by chunk number; a worker on chunk c
    // reads row_by_chunk[c + 1], the row at the boundary that follows its chunk
    const int* row_by_chunk;
};

// The row that owns stored entry q according to the hint r, or -1 when the hint does not hold.
// *start / *end receive the row's pointers when it does.
__device__ __forceinline__ int hinted_row(const int* __restrict__ rowptr, int m, int r, int q, int* start, int* end) {
    if (r < 0 || r >= m) return -1;
    const int a = rowptr[r], b = rowptr[r + 1];
    if (a > q || q >= b) return -1;
    *start = a;
    *end = b;
    return r;
}

// ------------------------------------------------------------------------------------------
// small helpers
// ------------------------------------------------------------------------------------------
template <int V>
__device__ __forceinline__ void load_vec(const float* __restrict__ p, float (&x)[V]) {
    if constexpr (V == 4) {
        const float4 t = *reinterpret_cast<const float4*>(p);
        x[0] = t.x; x[1] = t.y; x[2] = t.z; x[3] = t.w;
    } else {
        static_assert(V == 1, "V is 1 or 4");
        x[0] = *p;
    }
}

typedef float floatx4 __attribute__((ext_vector_type(4)));

// C is written once and never read back by the kernels: its stores are marked non-temporal so
// that they do not push B rows out of L2.
template <int V>
__device__ __forceinline__ void store_vec(float* __restrict__ p, const float (&x)[V]) {
    if constexpr (V == 4) {
        floatx4 t = {x[0], x[1], x[2], x[3]};
        __builtin_nontemporal_store(t, reinterpret_cast<floatx4*>(p));
    } else {
        __builtin_nontemporal_store(x[0], p);
    }
}

// Rows shared between workers are combined with hardware fp32 atomic adds (Sec. 4: "atomic_add"
// for rows assigned to different workers); the return value is not used.
template <int V>
__device__ __forceinline__ void emit_vec(float* __restrict__ p, const float (&x)[V], bool atomic) {
    if (atomic) {
#pragma unroll
        for (int v = 0; v < V; ++v) unsafeAtomicAdd(p + v, x[v]);
    } else {
        store_vec<V>(p, x);
    }
}

// A lane's accumulators: NV vectors of V columns, vector i at column offset i*V from the lane's n0.
template <int V, int NV>
struct Acc {
    float a[NV][V];
    __device__ __forceinline__ void clear() {
#pragma unroll
        for (int i = 0; i < NV; ++i)
#pragma unroll
            for (int v = 0; v < V; ++v) a[i][v] = 0.f;
    }
    // Branch-free gather of the lane's vectors of one B row (nvalid >= 1).  Vectors past nvalid
    // re-read vector 0 (valid memory); their values are never written out.  cs = column stride.
    __device__ __forceinline__ void load(const float* __restrict__ p, int nvalid, long cs) {
#pragma unroll
        for (int i = 0; i < NV; ++i) load_vec<V>(p + (i < nvalid ? i : 0) * V * cs, a[i]);
    }
    __device__ __forceinline__ void fma(float s, const Acc& b) {
#pragma unroll
        for (int i = 0; i < NV; ++i)
#pragma unroll
            for (int v = 0; v < V; ++v) a[i][v] = fmaf(s, b.a[i][v], a[i][v]);
    }
    __device__ __forceinline__ void scale(float s) {
#pragma unroll
        for (int i = 0; i < NV; ++i)
#pragma unroll
            for (int v = 0; v < V; ++v) a[i][v] *= s;
    }
    __device__ __forceinline__ void add(const Acc& b) {
#pragma unroll
        for (int i = 0; i < NV; ++i)
#pragma unroll
            for (int v = 0; v < V; ++v) a[i][v] += b.a[i][v];
    }
    __device__ __forceinline__ void emit(float* __restrict__ p, int nvalid, bool atomic, long cs) const {
#pragma unroll
        for (int i = 0; i < NV; ++i)
            if (i < nvalid) emit_vec<V>(p + i * V * cs, a[i], atomic);
    }
};

// number of valid V-vectors of a lane whose first column is n0
template <int V, int NV>
__device__ __forceinline__ int valid_vectors(int n0, int N) {
    const int left = (N - n0 + V - 1) / V;          // V == 4 implies N % 4 == 0
    return left < 0 ? 0 : (left > NV ? NV : left);
}

// Address of the lane's first column in a row of B.  The gather address is the only per-entry
// integer work of the kernels, and in 64-bit form (sign extension, 64 x 64-bit multiply, 64-bit
// adds: about ten VALU operations, several of them quarter rate) it costs more issue slots than the
// four multiply-adds a 16-byte gather feeds.  WIDE = false: k < 2^24, row pitch < 16 MiB and B
// smaller than 4 GiB (checked by the host): byte offset = col * pitch + lane offset in one 24-bit
// multiply-add, added to the wave-uniform base by the load instruction itself.
template <bool WIDE>
struct BRows {
    const float* base;
    long rb;
    unsigned pitch_bytes, lane_bytes;
    __device__ __forceinline__ BRows(const float* __restrict__ B, int n0, const Strides& sd) {
        if constexpr (WIDE) {
            base = B + (long)n0 * sd.cb; rb = sd.rb; pitch_bytes = 0; lane_bytes = 0;
        } else {
            base = B; rb = 0;
            pitch_bytes = (unsigned)sd.rb * 4u;
            lane_bytes = (unsigned)n0 * (unsigned)sd.cb * 4u;
        }
    }
    __device__ __forceinline__ const float* row(int col) const {
        if constexpr (WIDE) {
            return base + (long)col * rb;
        } else {
            const unsigned off = __umul24((unsigned)col, pitch_bytes) + lane_bytes;
            return reinterpret_cast<const float*>(reinterpret_cast<const char*>(base) + off);
        }
    }
};

// Orders LDS traffic of the lanes of one wave: the LDS unit serves one wave's requests in issue
// order, so only the compiler has to be kept from moving accesses across this point.
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Sum over the lanes of a wave that share lane % G (the slots of a PR kernel); every lane ends up
// with the total.  Butterfly steps at distance 32 and 16 use the gfx950 lane-swap instructions,
// the steps inside a 16-lane row use DPP rotations fused into the add: no LDS round trips.
template <int CTRL>
__device__ __forceinline__ float dpp_add(float x) {
    return x + __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(x), CTRL, 0xf, 0xf, false));
}

template <int G>
__device__ __forceinline__ float slot_allreduce(float x) {
    if constexpr (G <= 32) {
        const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
        x = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    }
    if constexpr (G <= 16) {
        const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
        x = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    }
    if constexpr (G <= 8) x = dpp_add<0x128>(x);   // row_ror:8
    if constexpr (G <= 4) x = dpp_add<0x124>(x);   // row_ror:4
    if constexpr (G <= 2) x = dpp_add<0x122>(x);   // row_ror:2
    if constexpr (G <= 1) x = dpp_add<0x121>(x);   // row_ror:1
    return x;
}

// y[l] = x[l + D] for the lanes l < 64 - D of a wave (the other lanes receive unspecified values):
// the data movement of one step of the conditional reduction (Sec. 4, Fig. 6(e)), where a slot
// takes in the partial result of the slot D lanes to its right.  Distance 32 is one lane swap,
// distance 16 two swaps and a select, distance 1 a single DPP wave shift: no LDS round trip.
__device__ __forceinline__ unsigned lane_shift_down_32(unsigned x) {
    return __builtin_amdgcn_permlane32_swap(x, x, false, false)[1];      // lanes 0..31 <- lanes 32..63
}
__device__ __forceinline__ unsigned lane_shift_down_16(unsigned x) {
    // rows of 16 lanes [x0 x1 x2 x3] -> [x1 x2 x3 .]
    const unsigned z = lane_shift_down_32(x);                             // [x2 x3 x2 x3]
    const auto r = __builtin_amdgcn_permlane16_swap(x, z, false, false);  // [x0 x2 x2 x2], [x1 x3 x3 x3]
    return (threadIdx.x & 16) ? r[0] : r[1];
}
template <int D>
__device__ __forceinline__ float lane_shift_down(float xf) {
    static_assert(D == 1 || D == 2 || D == 4 || D == 8 || D == 16 || D == 32, "power of two below 64");
    const unsigned x = __float_as_uint(xf);
    if constexpr (D == 32) {
        return __uint_as_float(lane_shift_down_32(x));
    } else if constexpr (D == 16) {
        return __uint_as_float(lane_shift_down_16(x));
    } else if constexpr (D == 1) {
        return __uint_as_float(__builtin_amdgcn_update_dpp(0u, x, 0x130, 0xf, 0xf, false));   // wave_shl:1
    } else {
        // Distances 2, 4, 8 would take a DPP row rotation plus the rotation of the next row for the
        // lanes that wrap around (five operations); the LDS crossbar moves them in one and measured
        // faster (EB+RM+PR on the power-law matrix at N = 32: 249 against 261 us).
        return __shfl_down(xf, D, kWave);
    }
}

// The log-step network of the conditional reduction over the S = 64/G slots of a wave: in step DS
// (1, 2, 4, ...) slot s adds the value of slot s + DS when that slot belongs to the same run of
// equal row indices, i.e. when DS <= dist, the number of slots from s to the end of its run.
template <int G, int DS>
__device__ __forceinline__ void conditional_steps(float& x, int dist) {
    if constexpr (DS * G < kWave) {
        const float o = lane_shift_down<DS * G>(x);
        if (DS <= dist) x += o;
        conditional_steps<G, DS * 2>(x, dist);
    }
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

// The same search done by the G lanes of a group together: every step probes G rows at once and
// narrows [lo, hi] to 1/(G+1) of its width, so it takes log_{G+1}(m) dependent loads instead of
// log_2(m).  All lanes of the group must call it together with the same q; j = lane index inside
// the group, shift = index of the group's first lane in the wave.
template <int G>
__device__ __forceinline__ int row_of_entry_group(const int* __restrict__ rowptr, int lo, int hi, int q,
                                                  int j, int shift) {
    if constexpr (G < 4) {
        return row_of_entry(rowptr, lo, hi, q);
    } else {
        while (lo < hi) {
            const long len = hi - lo;
            const int r = lo + (int)((len * (j + 1)) / (G + 1));       // lo <= r < hi
            const bool above = rowptr[r + 1] > q;                      // owner row is <= r
            unsigned long long bits = __ballot(above) >> shift;
            if constexpr (G < 64) bits &= (1ull << G) - 1;
            const int nfalse = G - __popcll(bits);                     // probes 0..nfalse-1 are too low
            const int new_lo = nfalse == 0 ? lo : lo + (int)((len * nfalse) / (G + 1)) + 1;
            const int new_hi = nfalse == G ? hi : lo + (int)((len * (nfalse + 1)) / (G + 1));
            lo = new_lo;
            hi = new_hi;
        }
        return lo;
    }
}

// entries a lane group stages per batch
template <int G> struct StageBatch { static constexpr int value = G < 8 ? kU : (G < 32 ? 32 : G); };

template <int U> struct Count { static constexpr int value = U; };

// A lane's share of a staged batch of SB stored entries (lane j of the group holds entries j, j+G,
// ...).  The next batch is fetched into registers while the current one is being consumed from LDS,
// so the (colind, val) round trip is off the critical path.
template <int G, int SB>
struct BatchRegs {
    int2 e[SB / G];
    __device__ __forceinline__ void fetch(const int* __restrict__ colind, const float* __restrict__ vals,
                                          int p0, int end, int j) {
#pragma unroll
        for (int i = 0; i < SB / G; ++i) {
            const int p = p0 + j + i * G;
            e[i] = make_int2(0, 0);
            if (p < end) { e[i].x = colind[p]; e[i].y = __float_as_int(vals[p]); }
        }
    }
    __device__ __forceinline__ void put(int2* st, int j) const {
#pragma unroll
        for (int i = 0; i < SB / G; ++i) st[j + i * G] = e[i];
    }
};

// Which column tile a block works on and its rank among the blocks of that tile.
//   pin_tiles == 0: 2-D grid, blockIdx.y = tile.
//   pin_tiles in {2,4,8}: 1-D grid whose size is a multiple of 8.  Consecutive workgroups go to
//     consecutive XCDs (8 per device, each with its own L2), so tile = (blockIdx.x % 8) % pin_tiles
//     keeps every XCD on one tile: its L2 then caches only that tile's slice of B.
struct BlockMap { int tile; long bx; long nbx; };
__device__ __forceinline__ BlockMap block_map(int pin_tiles) {
    BlockMap b;
    if (pin_tiles <= 0) {
        b.tile = blockIdx.y; b.bx = blockIdx.x; b.nbx = gridDim.x;
    } else {
        const int xcd = blockIdx.x & 7, per = 8 / pin_tiles;
        b.tile = xcd % pin_tiles;
        b.bx = (long)(blockIdx.x >> 3) * per + xcd / pin_tiles;
        b.nbx = (long)(gridDim.x >> 3) * per;
    }
    return b;
}

// Position in the schedule of (virtual) block vb when the schedule is swept by nx XCDs together
// (nx = 8, or 8 / pin_tiles for the XCDs that share a pinned column tile).  Workgroups go
// round-robin to the 8 XCDs and block_map numbers the blocks of one tile so that block vb runs on
// the (vb % nx)-th of these XCDs and is that XCD's (vb / nx)-th block.  Stripe t of XCD x is stripe
// nx t + x of the segment: at any time the XCDs work on nx neighbouring stripes, each on its own,
// and the rows of B that one L2 has to hold are an nx-th of the band all running workers cover.
// Returns -1 for a position outside its segment.
__device__ __forceinline__ long sweep_block(long vb, const Schedule& sch) {
    const unsigned nx = 1u << sch.nx_log2;
    const unsigned x = (unsigned)vb & (nx - 1u);          // block counts fit 32 bits
    unsigned l = (unsigned)(vb >> sch.nx_log2);
    if (l < (unsigned)sch.per_a) {
        const unsigned st = (unsigned)sch.stripe, t = l / st;
        const long sb = (long)(t * nx + x) * st + (l - t * st);
        return (sch.split > 0 && sb >= sch.split) ? -1 : sb;
    }
    l -= (unsigned)sch.per_a;
    const unsigned st = (unsigned)sch.stripe_b, t = l / st;
    return sch.split + (long)(t * nx + x) * st + (l - t * st);
}

// Calls f(Count<UU>, t) for t covering [begin, cnt) in blocks of UMAX, then 8, 4, 2, 1 entries, so that
// every block is straight-line code of a compile-time size: its gathers carry no predicates and
// are all in flight before the first one is consumed.
template <int UMAX, class F>
__device__ __forceinline__ void for_blocks(int begin, int cnt, F&& f) {
    int t = begin;
    for (; t + UMAX <= cnt; t += UMAX) f(Count<UMAX>{}, t);
    static_assert(UMAX <= 16, "the remainder is covered by blocks of 8, 4, 2, 1");
    if constexpr (UMAX > 8) { if (t + 8 <= cnt) { f(Count<8>{}, t); t += 8; } }
    if constexpr (UMAX > 4) { if (t + 4 <= cnt) { f(Count<4>{}, t); t += 4; } }
    if constexpr (UMAX > 2) { if (t + 2 <= cnt) { f(Count<2>{}, t); t += 2; } }
    if constexpr (UMAX > 1) { if (t < cnt) f(Count<1>{}, t); }
}
template <int UMAX, class F>
__device__ __forceinline__ void for_blocks(int cnt, F&& f) { for_blocks<UMAX>(0, cnt, f); }

// ------------------------------------------------------------------------------------------
// RB + SR : a lane group owns a row and adds its products one after another
// (Sec. 3.2 design M1, Sec. 3.4 design K1).  For G > 1 the group's lanes load a batch of stored
// entries with coalesced requests and pass them round through LDS, so that every entry is fetched
// once and reused for all columns of the tile (the sparse-element cache of Sec. 4).
// ------------------------------------------------------------------------------------------
template <int V, int G, int NV, bool WIDE>
__global__ __launch_bounds__(kBlock) void rb_sr_kernel(
    int m, int N, Strides sd, const int* __restrict__ rowptr, const int* __restrict__ colind,
    const float* __restrict__ vals, const float* __restrict__ B, float* __restrict__ C, int pin_tiles)
{
    constexpr int RPW = kWave / G;                       // rows per wave
    constexpr int SB = StageBatch<G>::value;
    constexpr int UL = G == 1 ? kU / NV : kU;            // entries whose gathers are issued together
    __shared__ int2 stage[G > 1 ? kWavesPerBlock * RPW * SB : 1];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int g = lane / G, j = lane % G;
    const BlockMap bm = block_map(pin_tiles);
    const long row = (bm.bx * kWavesPerBlock + wave) * RPW + g;
    const int n0 = (bm.tile * G + j) * V * NV;
    const int nvec = valid_vectors<V, NV>(n0, N);
    int start = 0, end = 0;
    if (row < m) { start = rowptr[row]; end = rowptr[row + 1]; }
    Acc<V, NV> acc;
    acc.clear();
    const BRows<WIDE> brow(B, n0, sd);

    if constexpr (G == 1) {
        if (nvec > 0) {
            for_blocks<UL>(end - start, [&](auto uc, int t) {
                constexpr int UU = decltype(uc)::value;
                const int p0 = start + t;
                int c[UU];
                float a[UU];
                Acc<V, NV> b[UU];
#pragma unroll
                for (int u = 0; u < UU; ++u) { c[u] = colind[p0 + u]; a[u] = vals[p0 + u]; }
#pragma unroll
                for (int u = 0; u < UU; ++u) b[u].load(brow.row(c[u]), nvec, sd.cb);
#pragma unroll
                for (int u = 0; u < UU; ++u) acc.fma(a[u], b[u]);
            });
        }
    } else {
        int2* st = stage + (wave * RPW + g) * SB;
        BatchRegs<G, SB> next;
        next.fetch(colind, vals, start, end, j);
        for (int p0 = start; p0 < end; p0 += SB) {
            next.put(st, j);
            wave_lds_sync();
            if (p0 + SB < end) next.fetch(colind, vals, p0 + SB, end, j);
            if (nvec > 0) {
                for_blocks<UL>(min(SB, end - p0), [&](auto uc, int t) {
                    constexpr int UU = decltype(uc)::value;
                    int2 e[UU];
                    Acc<V, NV> b[UU];
#pragma unroll
                    for (int u = 0; u < UU; ++u) e[u] = st[t + u];
#pragma unroll
                    for (int u = 0; u < UU; ++u) b[u].load(brow.row(e[u].x), nvec, sd.cb);
#pragma unroll
                    for (int u = 0; u < UU; ++u) acc.fma(__int_as_float(e[u].y), b[u]);
                });
            }
            wave_lds_sync();
        }
    }
    if (row < m && nvec > 0) acc.emit(C + row * sd.rc + (long)n0 * sd.cc, nvec, false, sd.cc);
}

// ------------------------------------------------------------------------------------------
// RB + PR : a wave owns a row; its 64 lanes form S = 64/G slots along the row's stored entries
// (times G lanes along n).  Rows longer than S are walked with a for-loop (technique 1 of Sec. 4),
// lanes load V consecutive columns at once (technique 2), the wave's entries are fetched once and
// shared through LDS (technique 3), and the slots are combined by a reduction tree (Sec. 3.4 K2).
// In a batch of 64 staged entries slot s takes entries s, s+S, s+2S, ...
// ------------------------------------------------------------------------------------------
template <int V, int G, int NV, bool WIDE>
__global__ __launch_bounds__(kBlock) void rb_pr_kernel(
    int m, int N, Strides sd, const int* __restrict__ rowptr, const int* __restrict__ colind,
    const float* __restrict__ vals, const float* __restrict__ B, float* __restrict__ C, int pin_tiles)
{
    constexpr int S = kWave / G;
    constexpr int UL = G == 1 ? (NV > 2 ? 2 : 4) : (G < kU ? G : kU);
    __shared__ int2 stage[G > 1 ? kBlock : 1];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int s = lane / G, j = lane % G;
    const BlockMap bm = block_map(pin_tiles);
    const long row = bm.bx * kWavesPerBlock + wave;
    if (row >= m) return;                                 // whole wave leaves together
    const int n0 = (bm.tile * G + j) * V * NV;
    const int nvec = valid_vectors<V, NV>(n0, N);
    const int start = rowptr[row], end = rowptr[row + 1];
    Acc<V, NV> acc;
    acc.clear();
    const BRows<WIDE> brow(B, n0, sd);

    if constexpr (G == 1) {
        if (nvec > 0) {
            // steps in which all 64 lanes hold an entry, then one ragged step
            const int len = end - start;
            for_blocks<UL>(len / kWave, [&](auto uc, int t) {
                constexpr int UU = decltype(uc)::value;
                const int p0 = start + t * kWave + lane;
                int c[UU];
                float a[UU];
                Acc<V, NV> b[UU];
#pragma unroll
                for (int u = 0; u < UU; ++u) { c[u] = colind[p0 + u * kWave]; a[u] = vals[p0 + u * kWave]; }
#pragma unroll
                for (int u = 0; u < UU; ++u) b[u].load(brow.row(c[u]), nvec, sd.cb);
#pragma unroll
                for (int u = 0; u < UU; ++u) acc.fma(a[u], b[u]);
            });
            const int p = start + (len / kWave) * kWave + lane;
            if (p < end) {
                Acc<V, NV> b;
                b.load(brow.row(colind[p]), nvec, sd.cb);
                acc.fma(vals[p], b);
            }
        }
    } else {
        int2* st = stage + wave * kWave;
        BatchRegs<kWave, kWave> next;
        next.fetch(colind, vals, start, end, lane);
        for (int p0 = start; p0 < end; p0 += kWave) {
            next.put(st, lane);
            wave_lds_sync();
            if (p0 + kWave < end) next.fetch(colind, vals, p0 + kWave, end, lane);
            const int cnt = min(kWave, end - p0);
            if (nvec > 0) {
                for_blocks<UL>(cnt / S, [&](auto uc, int t) {
                    constexpr int UU = decltype(uc)::value;
                    int2 ee[UU];
                    Acc<V, NV> b[UU];
#pragma unroll
                    for (int u = 0; u < UU; ++u) ee[u] = st[(t + u) * S + s];
#pragma unroll
                    for (int u = 0; u < UU; ++u) b[u].load(brow.row(ee[u].x), nvec, sd.cb);
#pragma unroll
                    for (int u = 0; u < UU; ++u) acc.fma(__int_as_float(ee[u].y), b[u]);
                });
                const int t = (cnt / S) * S + s;              // ragged last step
                if (t < cnt) {
                    const int2 ee = st[t];
                    Acc<V, NV> b;
                    b.load(brow.row(ee.x), nvec, sd.cb);
                    acc.fma(__int_as_float(ee.y), b);
                }
            }
            wave_lds_sync();
        }
    }
    // reduction tree over the slots: lanes with equal j
#pragma unroll
    for (int i = 0; i < NV; ++i)
#pragma unroll
        for (int v = 0; v < V; ++v) acc.a[i][v] = slot_allreduce<G>(acc.a[i][v]);
    if (s == 0 && nvec > 0) acc.emit(C + row * sd.rc + (long)n0 * sd.cc, nvec, false, sd.cc);
}

// ------------------------------------------------------------------------------------------
// EB pre-pass.  EB workers own fixed-size chunks of consecutive stored entries (Sec. 3.2 design
// M2).  A row whose entries all fall into one chunk is written by exactly one worker with a plain
// store; a row that straddles a chunk boundary receives atomic additions from several workers and
// must start from zero; a row without entries is touched by no worker.  This pass zeroes exactly
// those two kinds of rows so that C needs no full memset.  `chunk` is the number of entries per
// worker of the product kernel that follows.  own_short: that kernel gives every row of at most
// `chunk` entries to a single worker (see eb_sr_kernel), so only longer rows are shared.  A wave inspects 64 rows (one per lane) and then
// clears the flagged ones together: one row at a time with full-width stores when a row takes
// more than 32 stores, several rows per store instruction otherwise.
// ------------------------------------------------------------------------------------------
template <int V>
__global__ __launch_bounds__(kBlock) void eb_zero_kernel(
    int m, int N, Strides sd, const int* __restrict__ rowptr, float* __restrict__ C, int chunk, int own_short)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const long base = ((long)blockIdx.x * kWavesPerBlock + wave) * kWave;
    if (base >= m) return;
    const long row = base + lane;
    bool need = false;
    if (row < m) {
        const int start = rowptr[row], end = rowptr[row + 1];
        need = (end == start) || (start / chunk != (end - 1) / chunk && (!own_short || end - start > chunk));
    }
    unsigned long long mask = __ballot(need);
    float z[V];
#pragma unroll
    for (int v = 0; v < V; ++v) z[v] = 0.f;
    const int vecs = (N + V - 1) / V;                     // stores per row
    if (vecs > kWave / 2) {
        while (mask) {
            const int r = __ffsll((long long)mask) - 1;
            mask &= mask - 1;
            float* __restrict__ crow = C + (base + r) * sd.rc;
            for (int n0 = lane * V; n0 < N; n0 += kWave * V) store_vec<V>(crow + (long)n0 * sd.cc, z);
        }
    } else {
        // short rows of C: T lanes per row, 64/T flagged rows per store instruction.  The flagged
        // lanes list themselves in LDS in lane order; lane group s then takes list entries
        // s, s + 64/T, ...
        __shared__ unsigned char listed[kWavesPerBlock][kWave];
        const int count = __popcll(mask);
        if (need) listed[wave][__popcll(mask & ((1ull << lane) - 1ull))] = (unsigned char)lane;
        wave_lds_sync();
        const int T = vecs <= 1 ? 1 : 1 << (32 - __clz(vecs - 1));   // power of two >= vecs, <= 32
        const int n0 = (lane & (T - 1)) * V;
        for (int s = lane / T; s < count; s += kWave / T) {
            const int r = listed[wave][s];
            if (n0 < N) store_vec<V>(C + (base + r) * sd.rc + (long)n0 * sd.cc, z);
        }
    }
}

// ------------------------------------------------------------------------------------------
// EB + SR : a lane group owns `chunk` consecutive stored entries and walks them in order,
// keeping (partial sum, row).  When the row changes the partial is written: plain store if the
// row lies wholly inside the chunk, atomic add for the first / last row when it is shared with the
// neighbouring chunk (the "partial sum aggregation among workers" of Sec. 3.2).  The row of the
// chunk's first entry is found by binary search in rowptr (the "row index calculation" overhead
// named there).  Workers stride over the chunks so that the grid size does not depend on nnz,
// which only the device knows.  With own_short the chunk boundaries give way to short rows: a row
// of at most `chunk` entries that straddles a boundary goes whole to the worker in whose chunk it
// starts, so that only rows longer than a chunk take atomic additions (eb_zero_kernel is told).
// ------------------------------------------------------------------------------------------
// Lane groups for which EB+SR can keep short rows whole (own_short): measured to pay for groups of
// 16 and 32 lanes (power-law N = 128 468 -> 460 us); for groups of 8 the extra bookkeeping costs
// registers and occupancy (power-law N = 32 144 -> 148 us), so those kernels are built without it.
template <int G> constexpr bool kOwnShortRows = G >= 16;

template <int V, int G, int NV, bool WIDE>
__global__ __launch_bounds__(kBlock) void eb_sr_kernel(
    int m, int N, Strides sd, const int* __restrict__ rowptr, const int* __restrict__ colind,
    const float* __restrict__ vals, const float* __restrict__ B, float* __restrict__ C, int chunk,
    int pin_tiles, Schedule sch, int own_short)
{
    constexpr int GPW = kWave / G;                        // workers per wave
    constexpr int SB = StageBatch<G>::value;
    constexpr int UL = G == 1 ? kU / NV : kU;             // entries whose gathers are issued together
    __shared__ int2 stage[G > 1 ? kWavesPerBlock * GPW * SB : 1];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int g = lane / G, j = lane % G;
    const BlockMap bm = block_map(pin_tiles);
    const int n0 = (bm.tile * G + j) * V * NV;
    const int nvec = valid_vectors<V, NV>(n0, N);
    const BRows<WIDE> brow(B, n0, sd);
    float* __restrict__ Cn = C + (long)n0 * sd.cc;
    const int nnz = rowptr[m];
    int2* st = stage + (G > 1 ? (wave * GPW + g) * SB : 0);

    const long nunits = ((unsigned)nnz + (unsigned)chunk - 1u) / (unsigned)chunk;   // nnz < 2^31
    const bool scheduled = sch.order != nullptr && sch.nnz == nnz && sch.units == nunits;
    const bool striped = scheduled && sch.stripe > 0;
    constexpr long WPB = kWavesPerBlock * GPW;            // workers per block
    const long nvb = striped ? sch.vblocks : (nunits + WPB - 1) / WPB;   // block positions to walk
    for (long vb = bm.bx; vb < nvb; vb += bm.nbx) {
        const long sb = striped ? sweep_block(vb, sch) : vb;
        const long u = sb * WPB + wave * GPW + g;
        if (sb < 0 || u >= nunits) continue;
        const long cid = scheduled ? (long)sch.order[u] : u;
        const long c0l = cid * chunk;
        const int c0 = (int)c0l;
        const int c1 = (int)min(c0l + chunk, (long)nnz);
        // the chunk's first row: from the plan's hint when it holds (one round trip), else by the
        // group's search (log_{G+1} m dependent loads)
        int row_start = 0, row_end = 0;
        int row = (scheduled && sch.first_row != nullptr) ? hinted_row(rowptr, m, sch.first_row[u], c0, &row_start, &row_end) : -1;
        if (row < 0) {
            row = row_of_entry_group<G>(rowptr, 0, m - 1, c0, j, g * G);
            row_start = rowptr[row];
            row_end = rowptr[row + 1];
        }
        BatchRegs<G, SB> next;
        // the first batch is fetched before the worker knows where exactly its entries begin and end
        if constexpr (G > 1) next.fetch(colind, vals, c0, (int)min(c0l + 2l * chunk, (long)nnz), j);
        // Rows of at most `chunk` entries are never split (own_short): the one that straddles the
        // chunk's end is finished by this worker, the one that straddles its start was finished by
        // the worker before.  Both workers read the same row pointers, so they agree; a worker then
        // owns the entries [lo, hi), between 0 and 2 * chunk - 1 of them, and only rows longer than a
        // chunk are combined with atomic additions.
        int lo = c0, hi = c1;
        if (kOwnShortRows<G> && own_short) {
            if (c1 < nnz) {
                int bs = 0, be = 0;
                int rb = (scheduled && sch.row_by_chunk != nullptr)
                             ? hinted_row(rowptr, m, sch.row_by_chunk[cid + 1], c1, &bs, &be) : -1;
                if (rb < 0) {
                    rb = row_of_entry_group<G>(rowptr, row, m - 1, c1, j, g * G);
                    bs = rowptr[rb];
                    be = rowptr[rb + 1];
                }
                if (bs < c1 && be - bs <= chunk) hi = be;
            }
            if (row_start < c0 && row_end - row_start <= chunk) {
                lo = row_end;
                if (lo < hi) {                                 // the next row with entries starts at lo
                    int walked = 0;
                    do { ++row; row_end = rowptr[row + 1]; } while (row_end <= lo && ++walked < 4);
                    if (row_end <= lo) {
                        row = row_of_entry_group<G>(rowptr, row + 1, m - 1, lo, j, g * G);
                        row_end = rowptr[row + 1];
                    }
                    row_start = lo;
                }
            }
        }
        if (lo >= hi) continue;
        bool shared_with_prev = row_start < lo;            // only the worker's first row can be
        Acc<V, NV> acc;
        acc.clear();

        int q0 = c0, skip = lo - c0;                       // entries of the first batch that are not ours
        if (skip >= SB) {                                  // the first batch holds none of ours: fetch again
            q0 = lo;
            skip = 0;
            if constexpr (G > 1) next.fetch(colind, vals, q0, hi, j);
        }
        for (; q0 < hi; q0 += SB, skip = 0) {
            if constexpr (G > 1) {
                next.put(st, j);
                wave_lds_sync();
                if (q0 + SB < hi) next.fetch(colind, vals, q0 + SB, hi, j);
            }
            for_blocks<UL>(skip, min(SB, hi - q0), [&](auto uc, int t) {
                constexpr int UU = decltype(uc)::value;
                int2 e[UU];
                Acc<V, NV> b[UU];
#pragma unroll
                for (int u = 0; u < UU; ++u) {
                    if constexpr (G > 1) e[u] = st[t + u];
                    else e[u] = make_int2(colind[q0 + t + u], __float_as_int(vals[q0 + t + u]));
                }
                if (nvec > 0) {
#pragma unroll
                    for (int u = 0; u < UU; ++u) b[u].load(brow.row(e[u].x), nvec, sd.cb);
                }
                if (row_end > q0 + t + UU) {
                    // the common case: the whole block lies inside the current row
                    if (nvec > 0) {
#pragma unroll
                        for (int u = 0; u < UU; ++u) acc.fma(__int_as_float(e[u].y), b[u]);
                    }
                } else {
                    // All products first, so that every gather has been waited for before the
                    // first store or atomic is issued: stores share the in-order memory counter
                    // with loads, and a store issued between a gather and its use would make the
                    // wave wait for the store's acknowledgement.
                    if (nvec > 0) {
#pragma unroll
                        for (int u = 0; u < UU; ++u) b[u].scale(__int_as_float(e[u].y));
                    }
#pragma unroll
                    for (int u = 0; u < UU; ++u) {
                        if (nvec > 0) acc.add(b[u]);
                        const int next = q0 + t + u + 1;
                        if (next == row_end) {                 // the row is complete
                            if (nvec > 0) acc.emit(Cn + (long)row * sd.rc, nvec, shared_with_prev, sd.cc);
                            acc.clear();
                            shared_with_prev = false;
                            if (next < hi) {
                                // the next row with entries: usually row + 1; after a few rows
                                // without entries search instead of walking (a run of thousands
                                // of empty rows would otherwise cost a dependent load each)
                                int walked = 0;
                                do { ++row; row_end = rowptr[row + 1]; } while (row_end <= next && ++walked < 4);
                                if (row_end <= next) {
                                    row = row_of_entry_group<G>(rowptr, row + 1, m - 1, next, j, g * G);
                                    row_end = rowptr[row + 1];
                                }
                            }
                        }
                    }
                }
            });
            if constexpr (G > 1) wave_lds_sync();
        }
        if (row_end > hi && nvec > 0)                      // last row continues with the next worker
            acc.emit(Cn + (long)row * sd.rc, nvec, true, sd.cc);
    }
}

// ------------------------------------------------------------------------------------------
// EB + PR : a wave owns `chunk` consecutive stored entries and takes them 64 at a time.  The
// lanes form S = 64/G slots (times G lanes along n); in one step slot s holds the product vector
// of one entry together with that entry's row index.
//
// A step whose entries all belong to one row needs no cross-lane traffic: every slot adds its
// product to its own partial sum of the current row (as the RB+PR kernel does); the slots are
// combined only when the row ends.  A step that contains a row boundary is combined with the
// CONDITIONAL REDUCTION of Sec. 4 (Fig. 6(e)): a log-step network in which slot s adds the value
// of slot s+d only if both belong to the same row.  Because entries are stored row after row,
// afterwards the leftmost slot of every run of equal row indices holds the sum of the run (the
// validity rule of Sec. 4); whether slot s+d is in the same run is decided once, from a ballot of
// the run heads, instead of comparing shuffled row indices in every step of the network.  The run
// that starts the step is merged with the partial sums carried so far, runs that end inside the
// step are written by their leftmost slot, and the run that reaches the end of the step
// unfinished becomes the new set of per-slot partial sums.  Rows that are complete inside the
// chunk get one plain store; only the first and last row of a chunk, when shared with the
// neighbouring chunks, are combined with atomic adds.
// ------------------------------------------------------------------------------------------
template <int V, int G, int NV>
__device__ __forceinline__ Acc<V, NV> slots_allreduce(Acc<V, NV> x) {
#pragma unroll
    for (int i = 0; i < NV; ++i)
#pragma unroll
        for (int v = 0; v < V; ++v) x.a[i][v] = slot_allreduce<G>(x.a[i][v]);
    return x;
}

// Inclusive prefix sum of v over the 64 lanes of a wave: log-step scan inside the rows of 16 lanes
// with DPP row shifts (zeros shifted in), then the totals of the rows below are added.
__device__ __forceinline__ int wave_inclusive_scan_dpp(int v) {
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);    // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);    // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true);    // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, true);    // row_shr:8
    const int t0 = __builtin_amdgcn_readlane(v, 15), t1 = __builtin_amdgcn_readlane(v, 31),
              t2 = __builtin_amdgcn_readlane(v, 47);
    const int row = (threadIdx.x >> 4) & 3;
    return v + (row >= 1 ? t0 : 0) + (row >= 2 ? t1 : 0) + (row >= 3 ? t2 : 0);
}

constexpr int kStagedChunk = 512;   // EB+PR: largest chunk whose row starts are staged in LDS

template <int V, int G, int NV, bool WIDE>
__global__ __launch_bounds__(kBlock) void eb_pr_kernel(
    int m, int N, Strides sd, const int* __restrict__ rowptr, const int* __restrict__ colind,
    const float* __restrict__ vals, const float* __restrict__ B, float* __restrict__ C, int chunk,
    int pin_tiles, Schedule sch)
{
    constexpr int S = kWave / G;
    constexpr int UU = G < 4 ? G : 4;                     // steps whose gathers are issued together (8 measured slower)
    __shared__ int4 stage[G > 1 ? kBlock : 1];
    __shared__ int starts[kWavesPerBlock][kStagedChunk + 2];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int s = lane / G, j = lane % G;
    const BlockMap bm = block_map(pin_tiles);
    const int n0 = (bm.tile * G + j) * V * NV;
    const int nvec = valid_vectors<V, NV>(n0, N);
    const BRows<WIDE> brow(B, n0, sd);
    float* __restrict__ Cn = C + (long)n0 * sd.cc;
    const int nnz = rowptr[m];
    int4* st = stage + (G > 1 ? wave * kWave : 0);
    int* cnt = starts[wave];

    const long nunits = ((unsigned)nnz + (unsigned)chunk - 1u) / (unsigned)chunk;   // nnz < 2^31
    const bool scheduled = sch.order != nullptr && sch.nnz == nnz && sch.units == nunits;
    const bool striped = scheduled && sch.stripe > 0;
    const long nvb = striped ? sch.vblocks : (nunits + kWavesPerBlock - 1) / kWavesPerBlock;   // block positions to walk
    for (long vb = bm.bx; vb < nvb; vb += bm.nbx) {
        const long sb = striped ? sweep_block(vb, sch) : vb;
        const long u = sb * kWavesPerBlock + wave;
        if (sb < 0 || u >= nunits) continue;
        const long c0l = (scheduled ? (long)sch.order[u] : u) * chunk;
        const int c0 = (int)c0l;
        const int c1 = (int)min(c0l + chunk, (long)nnz);
        int hint_start, hint_end;
        int row_lo = (scheduled && sch.first_row != nullptr) ? hinted_row(rowptr, m, sch.first_row[u], c0, &hint_start, &hint_end) : -1;
        if (row_lo < 0) row_lo = row_of_entry_group<kWave>(rowptr, 0, m - 1, c0, lane, 0);
        const int row_hi = row_of_entry_group<kWave>(rowptr, row_lo, m - 1, c1 - 1, lane, 0);
        Acc<V, NV> acc;                                    // per-slot partial sums of row `cur`
        acc.clear();
        int cur = -1;                                      // row being accumulated (wave-uniform)
        bool cur_started = false;                          // its first entry lies in this chunk

        // The row of every entry ("row index calculation" of Sec. 3.2).  The rows after the first
        // that begin inside the chunk are counted per chunk position in LDS, one coalesced pass
        // over their row pointers; the row of the entry at position p is then the first row plus
        // the number of row starts at positions 1..p, a prefix sum over the wave, and an entry is
        // the first / last of its row when a row starts at its own / the next position.  cnt[0]
        // holds whether the first row starts with the chunk, cnt[c1 - c0] whether the last one ends
        // with it.  A row range too long to stage (runs of rows without entries) falls back to a
        // binary search per entry; a chunk inside one row needs none of this.
        const int len = c1 - c0;
        const bool single = row_hi == row_lo;                  // the chunk lies inside one row (wave-uniform)
        const bool staged = !single && chunk <= kStagedChunk && row_hi - row_lo <= 4 * kStagedChunk;
        const int single_start = single ? rowptr[row_lo] : 0, single_end = single ? rowptr[row_lo + 1] : 0;
        int row_base = 0, carried = 0;
        if (staged) {
            for (int i = lane; i <= len; i += kWave) cnt[i] = 0;
            wave_lds_sync();
            for (int r = row_lo + 1 + lane; r <= row_hi; r += kWave) atomicAdd(&cnt[rowptr[r] - c0], 1);
            const int first_here = rowptr[row_lo] == c0 ? 1 : 0;
            if (lane == 0) { cnt[0] = first_here; cnt[len] = rowptr[row_hi + 1] == c1 ? 1 : 0; }
            wave_lds_sync();
            row_base = row_lo - first_here;
        }
        auto lookup = [&](int q) {
            int4 e = make_int4(0, 0, -1, 0);
            if (single) {
                if (q < c1) {
                    e.x = colind[q];
                    e.y = __float_as_int(vals[q]);
                    e.z = row_lo;
                    e.w = (q == single_start ? 1 : 0) | (q + 1 == single_end ? 2 : 0);
                }
            } else if (staged) {
                const bool valid = q < c1;
                const int here = valid ? cnt[q - c0] : 0, next = valid ? cnt[q - c0 + 1] : 0;
                const int upto = wave_inclusive_scan_dpp(here);
                if (valid) {
                    e.x = colind[q];
                    e.y = __float_as_int(vals[q]);
                    e.z = row_base + carried + upto;
                    e.w = (here > 0 ? 1 : 0) | (next > 0 ? 2 : 0);
                }
                carried += __builtin_amdgcn_readlane(upto, kWave - 1);
            } else if (q < c1) {
                const int r = row_of_entry(rowptr, row_lo, row_hi, q);
                e.x = colind[q];
                e.y = __float_as_int(vals[q]);
                e.z = r;
                e.w = (q == rowptr[r] ? 1 : 0) | (q + 1 == rowptr[r + 1] ? 2 : 0);
            }
            return e;
        };
        for (int q0 = c0; q0 < c1; q0 += kWave) {
            const int4 mine = lookup(q0 + lane);
            if constexpr (G > 1) { st[lane] = mine; wave_lds_sync(); }
            const int cnt = min(kWave, c1 - q0);

            for (int tb = 0; tb * S < cnt; tb += UU) {
                int4 e[UU];
                Acc<V, NV> b[UU];
#pragma unroll
                for (int u = 0; u < UU; ++u) {
                    if constexpr (G > 1) e[u] = st[((tb + u) * S + s) & (kWave - 1)]; else e[u] = mine;
                    if ((tb + u) * S + s >= cnt) e[u].z = -1;
                }
                // branch-free gathers: slots past the end of the chunk hold column 0
                if (nvec > 0) {
#pragma unroll
                    for (int u = 0; u < UU; ++u) b[u].load(brow.row(e[u].x), nvec, sd.cb);
                }
                // all products first: no store or atomic is issued while a gather is outstanding
                // (stores share the in-order memory counter with loads)
#pragma unroll
                for (int u = 0; u < UU; ++u) {
                    const bool ok = e[u].z >= 0 && nvec > 0;
                    const float a = __int_as_float(e[u].y);
#pragma unroll
                    for (int i = 0; i < NV; ++i)
#pragma unroll
                        for (int v = 0; v < V; ++v) b[u].a[i][v] = ok ? a * b[u].a[i][v] : 0.f;
                }
#pragma unroll
                for (int u = 0; u < UU; ++u) {
                    const int t0 = (tb + u) * S;                       // first entry of this step
                    if (t0 >= cnt) break;                              // wave-uniform
                    const int er = e[u].z;
                    const bool evalid = er >= 0;
                    const int nv = min(S, cnt - t0);                   // valid slots in this step
                    const int first_row = __builtin_amdgcn_readfirstlane(er);
                    const int first_flags = __builtin_amdgcn_readfirstlane(e[u].w);
                    const int last_row = __builtin_amdgcn_readlane(er, (nv - 1) * G);
                    const int last_flags = __builtin_amdgcn_readlane(e[u].w, (nv - 1) * G);

                    if (first_row == last_row) {
                        // one row in the whole step: no cross-lane work
                        if (cur < 0) { cur = first_row; cur_started = (first_flags & 1) != 0; }
                        acc.add(b[u]);
                        if (last_flags & 2) {                           // the row ends here
                            const Acc<V, NV> total = slots_allreduce<V, G, NV>(acc);
                            if (s == 0 && nvec > 0) total.emit(Cn + (long)cur * sd.rc, nvec, !cur_started, sd.cc);
                            acc.clear();
                            cur = -1;
                        }
                    } else {
                        // a row boundary inside the step: conditional reduction
                        const Acc<V, NV> p = b[u];                      // this slot's product
                        Acc<V, NV> x = p;
                        // run heads: a slot whose entry is the first of its row (entries are stored
                        // row after row, so its left neighbour then holds another row); the first
                        // slot past the valid ones counts as a head so that the last run ends there
                        const bool head = s <= nv && (s == 0 || s == nv || (e[u].w & 1) != 0);
                        const unsigned long long heads = __ballot(head);
                        // slots from s to the end of its run
                        int dist = S - 1 - s;
                        if (s < S - 1) {
                            const unsigned long long above = heads >> ((s + 1) * G);
                            if (above) dist = (__ffsll((long long)above) - 1) / G;
                        }
#pragma unroll
                        for (int i = 0; i < NV; ++i)
#pragma unroll
                            for (int v = 0; v < V; ++v) conditional_steps<G, 1>(x.a[i][v], dist);
                        // the run that starts the step continues the row accumulated so far
                        bool started = true;                            // runs that begin inside the step
                        if (cur >= 0) {
                            const Acc<V, NV> total = slots_allreduce<V, G, NV>(acc);
                            if (s == 0) { x.add(total); started = cur_started; }
                        } else if (s == 0) {
                            started = (first_flags & 1) != 0;
                        }
                        const bool last_ended = (last_flags & 2) != 0;
                        const bool in_last_run = evalid && er == last_row;
                        if (head && evalid && nvec > 0 && (!in_last_run || last_ended))
                            x.emit(Cn + (long)er * sd.rc, nvec, !started, sd.cc);
                        if (last_ended) {
                            acc.clear();
                            cur = -1;
                        } else {                                        // unfinished run -> new partial sums
#pragma unroll
                            for (int i = 0; i < NV; ++i)
#pragma unroll
                                for (int v = 0; v < V; ++v) acc.a[i][v] = in_last_run ? p.a[i][v] : 0.f;
                            cur = last_row;
                            cur_started = true;
                        }
                    }
                }
            }
            if constexpr (G > 1) wave_lds_sync();
        }
        if (cur >= 0) {                                       // row continues in the next chunk
            const Acc<V, NV> total = slots_allreduce<V, G, NV>(acc);
            if (s == 0 && nvec > 0) total.emit(Cn + (long)cur * sd.rc, nvec, true, sd.cc);
        }
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

// ------------------------------------------------------------------------------------------
// Well-formedness checks of the CSR arrays (debug aid).  flags[0] collects violation bits,
// flags[1] receives rowptr[m].  The column check must only run after the row-pointer check
// passed: it trusts rowptr[m] as the number of stored entries.
// ------------------------------------------------------------------------------------------
enum : unsigned { kBadFirst = 1u, kBadOrder = 2u, kBadColumn = 4u };

__global__ __launch_bounds__(kBlock) void validate_rowptr_kernel(int m, const int* __restrict__ rowptr,
                                                                 unsigned* __restrict__ flags)
{
    unsigned bad = 0;
    for (long i = (long)blockIdx.x * kBlock + threadIdx.x; i < m; i += (long)gridDim.x * kBlock)
        if (rowptr[i + 1] < rowptr[i]) bad |= kBadOrder;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        if (rowptr[0] != 0) bad |= kBadFirst;
        flags[1] = (unsigned)rowptr[m];
    }
    if (bad) atomicOr(flags, bad);
}

__global__ __launch_bounds__(kBlock) void validate_colind_kernel(int nnz, int k, const int* __restrict__ colind,
                                                                 unsigned* __restrict__ flags)
{
    unsigned bad = 0;
    for (long p = (long)blockIdx.x * kBlock + threadIdx.x; p < nnz; p += (long)gridDim.x * kBlock) {
        const int c = colind[p];
        if (c < 0 || c >= k) bad |= kBadColumn;
    }
    if (bad) atomicOr(flags, bad);
}

}  // namespace daspmm
