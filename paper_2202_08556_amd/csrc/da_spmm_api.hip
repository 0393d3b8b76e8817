// Host side of libdaspmm.so: argument checks, choice of launch geometry, dispatch of the
// algorithm id to a kernel instantiation, the feature-extraction helper and the selector.
// The C ABI is declared and documented in include/da_spmm.h.
#include "da_spmm.h"
#include "da_spmm_kernels.hip"
#include "da_transpose_kernels.hip"

#include <atomic>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <memory>
#include <mutex>

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

struct Problem {
    int m, N;
    Strides sd;
    const int* rowptr;
    const int* colind;
    const float* vals;
    const float* B;
    float* C;
    hipStream_t stream;
    int64_t k;
};

enum Family { RB_SR, RB_PR, EB_SR, EB_PR };

// Launch geometry of one call: lane mapping (V, G, NV as in da_spmm_kernels.hip) and, for EB,
// the number of stored entries per worker.
struct Geometry {
    int V, G, NV, chunk;
    bool pin;   // pin column tiles to XCDs when the tile count is 2, 4 or 8
    int stripe; // blocks per stripe when a prepared matrix's chunk order is dealt to the XCDs (0: off)
};

constexpr int kSweepStripe = 256;

constexpr int kMaxGridY = 65535;
constexpr int kMaxGroupPR = 32;        // PR needs at least two slots along the entries
constexpr int kDefaultGroupPR = 8;     // 4-byte accesses: at least 8 slots along the entries
constexpr int kEntriesPerWavePR = 512; // EB+PR: stored entries per wave and pass

int env_int(const char* name, int fallback) {
    const char* v = std::getenv(name);
    return (v && *v) ? std::atoi(v) : fallback;
}

bool is_pow2(int x) { return x > 0 && (x & (x - 1)) == 0; }

// nnz of matrices whose features were extracted, keyed by (rowptr address, m).  da_spmm uses it
// only to size EB grids; EB kernels stride over all chunks whatever the grid size, so a stale or
// missing hint costs speed, never correctness.
struct NnzHint { const void* rowptr; int64_t m; int64_t nnz; };
std::mutex g_hint_mu;
NnzHint g_hints[16];
int g_hint_next = 0;

void remember_nnz(const void* rowptr, int64_t m, int64_t nnz) {
    std::lock_guard<std::mutex> lk(g_hint_mu);
    for (auto& h : g_hints)
        if (h.rowptr == rowptr && h.m == m) { h.nnz = nnz; return; }
    g_hints[g_hint_next] = NnzHint{rowptr, m, nnz};
    g_hint_next = (g_hint_next + 1) % 16;
}

int64_t lookup_nnz(const void* rowptr, int64_t m) {
    std::lock_guard<std::mutex> lk(g_hint_mu);
    for (const auto& h : g_hints)
        if (h.rowptr == rowptr && h.m == m) return h.nnz;
    return -1;
}

// Chunk schedules of matrices prepared with da_spmm_prepare, keyed like the nnz hints.  The
// orders live in one library-owned device allocation per matrix, held through a reference count:
// a product call copies the reference under the mutex, launches outside it and drops the reference
// after the launch, so that a concurrent release / re-prepare / eviction can free the memory only
// once no call is between its lookup and its launch (hipFree itself waits for launched kernels).
constexpr int kPlanUnits[4] = {64, 128, 256, 512};
struct DeviceBlock {
    void* p = nullptr;
    ~DeviceBlock() { if (p) (void)hipFree(p); }
};
struct Plan {
    const void* rowptr = nullptr;
    const void* colind = nullptr;
    int64_t m = 0, nnz = 0;
    int* order[4] = {nullptr, nullptr, nullptr, nullptr};
    int* first_row[4] = {nullptr, nullptr, nullptr, nullptr};   // per schedule position: row of the chunk's first entry (hint)
    int* row_by_chunk[4] = {nullptr, nullptr, nullptr, nullptr}; // the same rows indexed by chunk number
    int units[4] = {0, 0, 0, 0};
    int first_units[4] = {0, 0, 0, 0};   // chunks of the first schedule segment (multi-row chunks)
    std::shared_ptr<DeviceBlock> block;
    bool captured = false;               // a stream capture recorded a kernel that reads the orders
};
std::mutex g_plan_mu;
Plan g_plans[16];
int g_plan_next = 0;

bool has_plan(const void* rowptr, const void* colind, int64_t m) {
    std::lock_guard<std::mutex> lk(g_plan_mu);
    for (const auto& pl : g_plans)
        if (pl.block && pl.rowptr == rowptr && pl.colind == colind && pl.m == m) return true;
    return false;
}

// Schedule of a prepared matrix for this chunk size; split holds the CHUNKS of the first segment
// here, the launch turns it into blocks.  *keep receives a reference to the plan's memory, to be
// held until the kernel that reads the order has been launched.  capturing: the launch is being
// recorded into a HIP graph, which will read the order on every replay: such a plan is never
// evicted or replaced behind the caller's back, only da_spmm_release frees it.
Schedule lookup_schedule(const void* rowptr, const void* colind, int64_t m, int chunk, bool capturing,
                         std::shared_ptr<DeviceBlock>* keep) {
    std::lock_guard<std::mutex> lk(g_plan_mu);
    for (auto& pl : g_plans)
        if (pl.block && pl.rowptr == rowptr && pl.colind == colind && pl.m == m)
            for (int i = 0; i < 4; ++i)
                if (kPlanUnits[i] == chunk) {
                    *keep = pl.block;
                    if (capturing) pl.captured = true;
                    return Schedule{pl.order[i], pl.units[i], (int)pl.nnz, 0, pl.first_units[i], 0, 0, 0, 3, pl.first_row[i], pl.row_by_chunk[i]};
                }
    return Schedule{nullptr, 0, 0, 0, 0, 0, 0, 0, 3, nullptr, nullptr};
}

// Default geometry per algorithm family and N.  Measured on MI355X: 16-byte and 4-byte gathers
// run at full rate, 8-byte gathers at about half, and narrow rows (N < 32) gather fastest with one
// column per lane.  Setting DA_SPMM_TUNE=1 lets DA_SPMM_V / _G / _NV / _CHUNK override the choice
// (for tuning runs only; invalid combinations are rejected).
int pick_geometry(bool cm, bool pr, bool eb, int64_t N, const void* B, const void* C, const Strides& sd,
                  int64_t known_nnz, bool prepared, Geometry* out) {
    const uintptr_t addr = reinterpret_cast<uintptr_t>(B) | reinterpret_cast<uintptr_t>(C);
    // 16-byte accesses need unit column strides and rows that start on 16-byte boundaries
    const bool vec4_ok = (N % 4 == 0) && (addr % 16 == 0) && sd.cb == 1 && sd.cc == 1 &&
                         sd.rb % 4 == 0 && sd.rc % 4 == 0;
    Geometry g{1, 1, 1, 0, false, kSweepStripe};
    if (cm) {
        g.V = vec4_ok ? 4 : 1;
        const long vecs = (N + g.V - 1) / g.V;
        g.NV = vecs >= 4 ? 4 : pow2_ceil(vecs);
        g.G = 1;
    } else {
        g.V = (vec4_ok && N >= 32) ? 4 : 1;
        g.G = pow2_ceil((N + g.V - 1) / g.V);
        // SR: at most 128 columns per tile (32 lanes of 4): at N = 256 two passes over 512-byte row
        // segments keep more rows of B in L2 than one pass over 1 KB rows and were never slower
        // PR keeps slots along the entries: with 16-byte accesses 2 under EB (wave per chunk; the
        // conditional reduction gets shallower as the group widens: power-law N = 128 823 / 645 /
        // 574 us for groups of 8 / 16 / 32) and 4 under RB (wave per row: 629 / 559 / 636 us)
        const int cap = g.V == 4 ? ((pr && !eb) ? 16 : 32) : (pr ? kDefaultGroupPR : kWave);
        if (g.G > cap) g.G = cap;
        g.NV = 1;
    }
    static const bool tune = std::getenv("DA_SPMM_TUNE") != nullptr;
    if (tune) {
        g.V = env_int("DA_SPMM_V", g.V);
        g.G = env_int("DA_SPMM_G", g.G);
        g.NV = env_int("DA_SPMM_NV", g.NV);
        g.pin = env_int("DA_SPMM_PIN", g.pin ? 1 : 0) != 0;
        g.stripe = env_int("DA_SPMM_STRIPE", g.stripe);
        if (g.stripe < 0 || g.stripe > 4096) return fail(DA_ERR_UNSUPPORTED, "DA_SPMM_STRIPE outside 0..4096%s");
        if ((g.V != 1 && g.V != 4) || (g.V == 4 && !vec4_ok) || !is_pow2(g.G) || g.G > kWave ||
            (pr && g.G > kMaxGroupPR) || (g.NV != 1 && g.NV != 2 && g.NV != 4) || (g.G > 1 && g.NV != 1))
            return fail(DA_ERR_UNSUPPORTED, "DA_SPMM_V/_G/_NV override is not a supported combination%s");
    }
    if (eb) {
        if (pr) g.chunk = kEntriesPerWavePR;
        // with a chunk schedule (prepared matrix) groups of 8 lanes do better on half-size chunks:
        // twice as many waves pass through the machine and the sweep has a time axis
        else g.chunk = g.G >= 16 ? 256 : (g.G == 8 ? (prepared ? 128 : 256) : (g.G == 4 ? 128 : 64));
        if (known_nnz >= 0) {
            // Small matrices: shrink the chunks until there are about four waves of workers per
            // SIMD, so that the chunk walk, a chain of dependent memory round trips, does not set
            // the run time.  Lane-sized workers (G < 8) keep their chunk: their search cost per
            // entry is already high.
            const long workers = (long)cu_count() * 16 * (pr ? 1 : kWave / g.G);
            const int floor_ = pr ? 64 : (g.G >= 8 ? 32 : g.chunk);
            long want = known_nnz / workers;
            want = (want + 7) / 8 * 8;
            if (want < floor_) want = floor_;
            if (want < g.chunk) g.chunk = (int)want;
        }
        if (tune) g.chunk = env_int("DA_SPMM_CHUNK", g.chunk);
        if (g.chunk < 8 || g.chunk > (1 << 20)) return fail(DA_ERR_UNSUPPORTED, "bad DA_SPMM_CHUNK%s");
    }
    *out = g;
    return DA_OK;
}

template <int V, int G, int NV, bool WIDE>
int launch_w(Family fam, const Problem& p, const Geometry& geo) {
    const int chunk = geo.chunk;
    const long tile_cols = (long)G * V * NV;
    const long tiles_l = (p.N + tile_cols - 1) / tile_cols;
    if (tiles_l > kMaxGridY) return fail(DA_ERR_UNSUPPORTED, "N needs more than 65535 column tiles%s");
    const unsigned tiles = (unsigned)tiles_l;
    const int pin = (geo.pin && (tiles == 2 || tiles == 4 || tiles == 8)) ? (int)tiles : 0;
    // grid for `bx` blocks per column tile
    auto grid_for = [&](long bx) {
        if (pin) { const long per = 8 / pin; return dim3((unsigned)(8 * ((bx + per - 1) / per)), 1); }
        return dim3((unsigned)bx, tiles);
    };
    const dim3 block(kBlock);
    switch (fam) {
    case RB_SR: {
        const long rows_per_block = (long)kWavesPerBlock * (kWave / G);
        hipLaunchKernelGGL((rb_sr_kernel<V, G, NV, WIDE>), grid_for((p.m + rows_per_block - 1) / rows_per_block),
                           block, 0, p.stream, p.m, p.N, p.sd, p.rowptr, p.colind, p.vals, p.B, p.C, pin);
        break;
    }
    case RB_PR: {
        if constexpr (G <= kMaxGroupPR) {
            hipLaunchKernelGGL((rb_pr_kernel<V, G, NV, WIDE>), grid_for((p.m + kWavesPerBlock - 1) / kWavesPerBlock),
                               block, 0, p.stream, p.m, p.N, p.sd, p.rowptr, p.colind, p.vals, p.B, p.C, pin);
        }
        break;
    }
    case EB_SR:
    case EB_PR: {
        // entries per block and pass: a lane group (SR) or a whole wave (PR) owns `chunk` entries
        const long entries_per_block = fam == EB_SR ? (long)chunk * kWavesPerBlock * (kWave / G)
                                                    : (long)chunk * kWavesPerBlock;
        // One chunk per worker when nnz is known from an earlier da_spmm_features call (the
        // hardware dispatcher then balances the blocks); otherwise nnz is known only on the
        // device and the grid is sized for a few waves of blocks over the whole machine, bounded
        // by what the matrix could hold at most.
        long blocks;
        const int64_t known = lookup_nnz(p.rowptr, p.m);
        if (known >= 0) {
            blocks = (known + entries_per_block - 1) / entries_per_block;
            if (blocks > (1L << 20)) blocks = 1L << 20;
        } else {
            long max_nnz = (long)p.m * (p.k < 1 ? 1 : p.k);
            if (max_nnz > 0x7fffffffL) max_nnz = 0x7fffffffL;
            blocks = (max_nnz + entries_per_block - 1) / entries_per_block;
            const long full = (long)cu_count() * 8 * 4;
            if (blocks > full) blocks = full;
        }
        if (blocks < 1) blocks = 1;
        // chunk order of a prepared matrix (column sweep), if one exists for this chunk size
        std::shared_ptr<DeviceBlock> keep;                 // dropped after the launch
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(p.stream, &cap) != hipSuccess) { (void)hipGetLastError(); cap = hipStreamCaptureStatusNone; }
        Schedule sch = env_int("DA_SPMM_NO_SCHEDULE", 0)
                           ? Schedule{nullptr, 0, 0, 0, 0, 0, 0, 0, 3, nullptr, nullptr}
                           : lookup_schedule(p.rowptr, p.colind, p.m, chunk, cap == hipStreamCaptureStatusActive, &keep);
        // EB+SR on a prepared matrix never splits rows of at most a chunk (the plan's row hints make
        // the second boundary look-up cheap); the zero pass and the product kernel are told alike
        const int own_short = (fam == EB_SR && kOwnShortRows<G> && sch.order != nullptr &&
                               env_int("DA_SPMM_SPLIT_SHORT_ROWS", 0) == 0) ? 1 : 0;
        // pre-pass: zero the rows that receive atomic additions, and the rows without entries
        const dim3 zgrid((unsigned)((p.m + kBlock - 1) / kBlock));
        hipLaunchKernelGGL((eb_zero_kernel<V>), zgrid, block, 0, p.stream, p.m, p.N, p.sd, p.rowptr, p.C, chunk, own_short);
        const int first_chunks = sch.split;
        sch.split = 0;
        if (sch.order && geo.stripe > 0) {
            // Deal the schedule in stripes (sweep_block) to the XCDs that work on it: all 8, or the
            // 8 / pin that share a pinned column tile.  Stripe length near geo.stripe such that whole
            // rounds of stripes cover a segment with next to no surplus (all XCDs then get the same
            // number of stripes).  When the schedule starts with a segment of multi-row chunks, that
            // segment and the rest are dealt separately: the two kinds of chunk cost differently,
            // and every XCD should get the same share of both.
            const long nx = pin ? 8 / pin : 8;
            sch.nx_log2 = nx == 8 ? 3 : (nx == 4 ? 2 : (nx == 2 ? 1 : 0));
            const long wpb = fam == EB_SR ? (long)kWavesPerBlock * (kWave / G) : (long)kWavesPerBlock;
            const long nvb = (sch.units + wpb - 1) / wpb;
            auto deal = [&](long nb, int* stripe_out) {        // blocks per XCD, rounded up to whole stripes
                const long per_xcd = (nb + nx - 1) / nx;
                long rounds = (per_xcd + geo.stripe / 2) / geo.stripe;
                if (rounds < 1) rounds = 1;
                *stripe_out = (int)((per_xcd + rounds - 1) / rounds);
                return (long)*stripe_out * rounds;
            };
            long split = env_int("DA_SPMM_NO_SPLIT", 0) ? 0 : first_chunks / wpb;
            if (split < 16 || nvb - split < 16) split = 0;
            if (nvb >= 16) {
                long per_b = 0;
                sch.split = (int)split;
                sch.per_a = (int)deal(split > 0 ? split : nvb, &sch.stripe);
                if (split > 0) per_b = deal(nvb - split, &sch.stripe_b); else sch.stripe_b = 1;
                sch.vblocks = (int)(nx * (sch.per_a + per_b));
                if (blocks >= nvb) blocks = sch.vblocks;      // one chunk per worker
            }
            if (!pin) blocks = (blocks + 7) / 8 * 8;       // block b stays on XCD b % 8 on every pass
        }
        if (fam == EB_SR) {
            hipLaunchKernelGGL((eb_sr_kernel<V, G, NV, WIDE>), grid_for(blocks), block, 0, p.stream,
                               p.m, p.N, p.sd, p.rowptr, p.colind, p.vals, p.B, p.C, chunk, pin, sch, own_short);
        } else {
            if constexpr (G <= kMaxGroupPR)
                hipLaunchKernelGGL((eb_pr_kernel<V, G, NV, WIDE>), grid_for(blocks), block, 0, p.stream,
                                   p.m, p.N, p.sd, p.rowptr, p.colind, p.vals, p.B, p.C, chunk, pin, sch);
        }
        break;
    }
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "kernel launch");
    return DA_OK;
}

// 32-bit gather offsets (BRows<false>) need column indices below 2^24, a row pitch below 16 MiB and
// every element of B within 4 GiB of its base; anything larger takes the 64-bit kernels.
template <int V, int G, int NV>
int launch(Family fam, const Problem& p, const Geometry& geo) {
    const unsigned long long last = (unsigned long long)(p.k > 0 ? p.k - 1 : 0) * (unsigned long long)p.sd.rb +
                                    (unsigned long long)(p.N > 0 ? p.N - 1 : 0) * (unsigned long long)p.sd.cb;
    const bool narrow = p.k <= (1 << 24) && p.sd.rb * 4 < (1 << 24) && (last + 4) * 4 < (1ull << 32) &&
                        env_int("DA_SPMM_WIDE", 0) == 0;
    return narrow ? launch_w<V, G, NV, false>(fam, p, geo) : launch_w<V, G, NV, true>(fam, p, geo);
}

template <int V>
int dispatch_v(Family fam, const Geometry& g, const Problem& p) {
    if (g.G == 1) {
        switch (g.NV) {
        case 1: return launch<V, 1, 1>(fam, p, g);
        case 2: return launch<V, 1, 2>(fam, p, g);
        case 4: return launch<V, 1, 4>(fam, p, g);
        }
    } else if (g.NV == 1) {
        switch (g.G) {
        case 2: return launch<V, 2, 1>(fam, p, g);
        case 4: return launch<V, 4, 1>(fam, p, g);
        case 8: return launch<V, 8, 1>(fam, p, g);
        case 16: return launch<V, 16, 1>(fam, p, g);
        case 32: return launch<V, 32, 1>(fam, p, g);
        case 64: return launch<V, 64, 1>(fam, p, g);
        }
    }
    return fail(DA_ERR_UNSUPPORTED, "unsupported lane mapping%s");
}

int dispatch(Family fam, const Geometry& g, const Problem& p) {
    if ((fam == RB_PR || fam == EB_PR) && g.G > kMaxGroupPR)
        return fail(DA_ERR_UNSUPPORTED, "PR lane group too wide%s");
    return g.V == 4 ? dispatch_v<4>(fam, g, p) : dispatch_v<1>(fam, g, p);
}

const char* const kNames[DA_NUM_ALGOS] = {
    "RB+RM+SR", "RB+RM+PR", "RB+CM+SR", "RB+CM+PR", "EB+RM+SR", "EB+RM+PR", "EB+CM+SR", "EB+CM+PR"};

// Workspace of da_csr_transpose: two buffers each of keys, row numbers and values (nnz elements)
// for the ping-pong of the radix passes, the per-block digit histograms of one pass, and the chunk
// sums of their prefix scan.  Every part starts on a 256-byte boundary.
struct TransposePlan {
    int passes, digit_bits, nblocks;
    long hist_len, parts;
    size_t off_keys[2], off_rows[2], off_vals[2], off_hist, off_part, bytes;
};

size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

TransposePlan plan_transpose(int64_t k, int64_t nnz) {
    TransposePlan t{};
    int bits = 1;
    while (bits < 31 && (int64_t(1) << bits) < k) ++bits;             // column indices are < 2^bits
    t.passes = (bits + kRadixBits - 1) / kRadixBits;
    t.digit_bits = (bits + t.passes - 1) / t.passes;                  // equal digits, at most kRadixBits wide
    t.nblocks = (int)((nnz + kSortTile - 1) / kSortTile);
    t.hist_len = (long)kBins * t.nblocks;
    t.parts = (t.hist_len + kScanChunk - 1) / kScanChunk;
    size_t off = 0;
    const size_t per = align256((size_t)nnz * 4);
    for (int i = 0; i < 2; ++i) { t.off_keys[i] = off; off += per; }
    for (int i = 0; i < 2; ++i) { t.off_rows[i] = off; off += per; }
    for (int i = 0; i < 2; ++i) { t.off_vals[i] = off; off += per; }
    t.off_hist = off; off += align256((size_t)t.hist_len * sizeof(int));
    t.off_part = off; off += align256((size_t)t.parts * sizeof(int));
    t.bytes = off > 0 ? off : 256;
    return t;
}

// One schedule to build: da_eb_schedule's outputs, and optionally the row of every chunk's first
// entry in schedule order (first_rows[u] belongs to chunk order[u]) and indexed by chunk number
// (rows_by_unit); all device pointers, the last three may be null
struct ScheduleJob {
    int unit;
    int32_t* order; int32_t* first_segment; int32_t* first_rows; int32_t* rows_by_unit;
    void* workspace; size_t workspace_bytes;
};
int enqueue_schedules(int64_t m, int64_t k, int64_t nnz, const int32_t* rowptr, const int32_t* colind,
                      const ScheduleJob* jobs, int njobs, void* stream);
int check_transpose_args(int64_t m, int64_t k, int64_t nnz, const int32_t* rowptr, const int32_t* colind,
                         const float* vals, int32_t* t_rowptr, int32_t* t_colind, float* t_vals);
int enqueue_transpose(int64_t m, int64_t k, int64_t nnz, const int32_t* rowptr, const int32_t* colind,
                      const float* vals, int32_t* t_rowptr, int32_t* t_colind, float* t_vals,
                      void* workspace, size_t workspace_bytes, void* stream);

// Scratch memory of the entry point that allocates nothing (da_csr_transpose_noalloc): a static
// device array, one copy per GPU, held from the moment the library is loaded on that GPU until the
// process ends.  In host code the array's name is only a handle for the runtime, not a device
// address: the address on the current device is asked for once per device and kept.
constexpr size_t kScratchBytes = size_t(32) << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices];

int scratch_address(void** out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return fail(DA_ERR_UNSUPPORTED, "device ordinal beyond 63%s");
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(scratch)");
        if (!p || reinterpret_cast<uintptr_t>(p) % 256 != 0) return fail(DA_ERR_HIP, "static scratch has no usable device address%s");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return DA_OK;
}

// DA_SPMM_DEBUG_VALIDATE=1 makes da_spmm / da_spmm_ex / da_csr_transpose check the CSR arrays on
// the device before they launch anything (this synchronises the stream)
bool debug_validate() {
    const char* v = std::getenv("DA_SPMM_DEBUG_VALIDATE");
    return v && *v && std::strcmp(v, "0") != 0;
}

}  // namespace

extern "C" {

int da_csr_validate(int64_t m, int64_t k, int64_t nnz, const int32_t* rowptr, const int32_t* colind, void* stream)
{
    if (m < 0 || k < 0 || nnz < -1) return fail(DA_ERR_INVALID_ARG, "negative size%s");
    if (m > 0x7ffffffeLL || k > 0x7fffffffLL || nnz > 0x7fffffffLL)
        return fail(DA_ERR_INVALID_ARG, "size beyond the int32 index range%s");
    if (m == 0) return nnz > 0 ? fail(DA_ERR_INVALID_ARG, "stored entries in a matrix without rows%s") : DA_OK;
    if (!rowptr) return fail(DA_ERR_INVALID_ARG, "null rowptr%s");
    hipStream_t st = (hipStream_t)stream;
    unsigned* dflags = nullptr;
    hipError_t e = hipMalloc(&dflags, 2 * sizeof(unsigned));
    if (e != hipSuccess) return hip_fail(e, "hipMalloc");
    unsigned h[2] = {0, 0};
    const long cap = (long)cu_count() * 8;
    auto blocks_for = [&](long n) { long b = (n + kBlock - 1) / kBlock; return (unsigned)(b > cap ? cap : (b < 1 ? 1 : b)); };
    e = hipMemsetAsync(dflags, 0, sizeof h, st);
    if (e == hipSuccess) {
        hipLaunchKernelGGL(validate_rowptr_kernel, dim3(blocks_for(m)), dim3(kBlock), 0, st, (int)m, rowptr, dflags);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipMemcpyAsync(h, dflags, sizeof h, hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    int status = DA_OK;
    if (e == hipSuccess) {
        const int64_t dev_nnz = (int64_t)(int32_t)h[1];
        if (h[0] & kBadFirst) status = fail(DA_ERR_INVALID_ARG, "malformed CSR: rowptr[0] != 0%s");
        else if (h[0] & kBadOrder) status = fail(DA_ERR_INVALID_ARG, "malformed CSR: rowptr decreases%s");
        else if (nnz >= 0 && dev_nnz != nnz) status = fail(DA_ERR_INVALID_ARG, "malformed CSR: rowptr[m] differs from nnz%s");
        else if (dev_nnz > 0 && !colind) status = fail(DA_ERR_INVALID_ARG, "null colind with stored entries%s");
        else if (dev_nnz > 0) {
            hipLaunchKernelGGL(validate_colind_kernel, dim3(blocks_for(dev_nnz)), dim3(kBlock), 0, st, (int)dev_nnz, (int)k,
                               colind, dflags);
            e = hipGetLastError();
            if (e == hipSuccess) e = hipMemcpyAsync(h, dflags, sizeof h, hipMemcpyDeviceToHost, st);
            if (e == hipSuccess) e = hipStreamSynchronize(st);
            if (e == hipSuccess && (h[0] & kBadColumn))
                status = fail(DA_ERR_INVALID_ARG, "malformed CSR: column index outside [0, k)%s");
        }
    }
    (void)hipFree(dflags);
    if (e != hipSuccess) return hip_fail(e, "da_csr_validate");
    return status;
}

int da_spmm_ex(int64_t m, int64_t k, int64_t N, const int32_t* rowptr, const int32_t* colind,
               const float* vals, const float* B, int64_t ldb, int layout_b, float* C, int64_t ldc,
               int layout_c, int algo, void* stream)
{
    if (m < 0 || k < 0 || N < 0) return fail(DA_ERR_INVALID_ARG, "negative size%s");
    if (m > 0x7ffffffeLL || k > 0x7fffffffLL || N > 0x7fffffffLL)
        return fail(DA_ERR_INVALID_ARG, "size beyond the int32 index range%s");
    if (algo < 0 || algo >= DA_NUM_ALGOS) return fail(DA_ERR_BAD_ALGO, "algorithm id outside 0..7%s");
    if ((layout_b != DA_ROW_MAJOR && layout_b != DA_COL_MAJOR) || (layout_c != DA_ROW_MAJOR && layout_c != DA_COL_MAJOR))
        return fail(DA_ERR_INVALID_ARG, "layout is neither DA_ROW_MAJOR nor DA_COL_MAJOR%s");
    if (ldb < (layout_b == DA_ROW_MAJOR ? N : k) || ldc < (layout_c == DA_ROW_MAJOR ? N : m))
        return fail(DA_ERR_INVALID_ARG, "leading dimension smaller than the extent it strides over%s");
    if (m == 0 || N == 0) return DA_OK;
    if (!rowptr || !C) return fail(DA_ERR_INVALID_ARG, "null rowptr or C%s");
    // colind, vals and B are read only through stored entries; they may be null when nnz == 0,
    // which only the device knows
    if (debug_validate()) {
        const int v = da_csr_validate(m, k, -1, rowptr, colind, stream);
        if (v != DA_OK) return v;
    }

    Strides sd;
    sd.rb = layout_b == DA_ROW_MAJOR ? ldb : 1;
    sd.cb = layout_b == DA_ROW_MAJOR ? 1 : ldb;
    sd.rc = layout_c == DA_ROW_MAJOR ? ldc : 1;
    sd.cc = layout_c == DA_ROW_MAJOR ? 1 : ldc;
    Problem p{(int)m, (int)N, sd, rowptr, colind, vals, B, C, (hipStream_t)stream, k};
    const bool eb = algo >= DA_EB_RM_SR;
    const bool cm = (algo & 2) != 0;
    const bool pr = (algo & 1) != 0;
    Geometry g;
    const int st = pick_geometry(cm, pr, eb, N, B, C, sd, eb ? lookup_nnz(rowptr, m) : -1,
                                 eb && has_plan(rowptr, colind, m), &g);
    if (st != DA_OK) return st;
    const Family fam = eb ? (pr ? EB_PR : EB_SR) : (pr ? RB_PR : RB_SR);
    return dispatch(fam, g, p);
}

int da_spmm(int64_t m, int64_t k, int64_t N, const int32_t* rowptr, const int32_t* colind,
            const float* vals, const float* B, float* C, int algo, void* stream)
{
    if (N < 0) return fail(DA_ERR_INVALID_ARG, "negative size%s");
    return da_spmm_ex(m, k, N, rowptr, colind, vals, B, N, DA_ROW_MAJOR, C, N, DA_ROW_MAJOR, algo, stream);
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
    remember_nnz(rowptr, m, out->nnz);
    out->row_nnz_mean = mean;
    out->row_nnz_std = std::sqrt(var);
    out->row_nnz_max = (double)h[1];
    return DA_OK;
}

int da_csr_transpose_workspace(int64_t m, int64_t k, int64_t nnz, size_t* bytes)
{
    if (!bytes) return fail(DA_ERR_INVALID_ARG, "null bytes%s");
    if (m < 0 || k < 0 || nnz < 0) return fail(DA_ERR_INVALID_ARG, "negative size%s");
    if (m > 0x7ffffffeLL || k > 0x7ffffffeLL || nnz > 0x7fffffffLL)
        return fail(DA_ERR_INVALID_ARG, "size beyond the int32 index range%s");
    *bytes = plan_transpose(k, nnz).bytes;
    return DA_OK;
}

int da_csr_transpose(int64_t m, int64_t k, int64_t nnz, const int32_t* rowptr, const int32_t* colind,
                     const float* vals, int32_t* t_rowptr, int32_t* t_colind, float* t_vals,
                     void* workspace, size_t workspace_bytes, void* stream)
{
    const int st = check_transpose_args(m, k, nnz, rowptr, colind, vals, t_rowptr, t_colind, t_vals);
    if (st != DA_OK) return st;
    if (debug_validate() && m > 0) {
        const int v = da_csr_validate(m, k, nnz, rowptr, colind, stream);
        if (v != DA_OK) return v;
    }
    return enqueue_transpose(m, k, nnz, rowptr, colind, vals, t_rowptr, t_colind, t_vals, workspace, workspace_bytes, stream);
}

int da_csr_transpose_noalloc(int64_t m, int64_t k, int64_t nnz, const int32_t* rowptr, const int32_t* colind,
                             const float* vals, int32_t* t_rowptr, int32_t* t_colind, float* t_vals, void* stream)
{
    const int st = check_transpose_args(m, k, nnz, rowptr, colind, vals, t_rowptr, t_colind, t_vals);
    if (st != DA_OK) return st;
    if (plan_transpose(k, nnz).bytes > kScratchBytes)
        return fail(DA_ERR_UNSUPPORTED,
                    "da_csr_transpose_noalloc: the sort needs more than the library's 32 MiB static scratch "
                    "(about 24 bytes per stored entry); use da_csr_transpose with a workspace%s");
    void* ptr = nullptr;
    const int sp = scratch_address(&ptr);
    if (sp != DA_OK) return sp;
    return enqueue_transpose(m, k, nnz, rowptr, colind, vals, t_rowptr, t_colind, t_vals, ptr, kScratchBytes, stream);
}

}  // extern "C"

namespace {

int check_transpose_args(int64_t m, int64_t k, int64_t nnz, const int32_t* rowptr, const int32_t* colind,
                         const float* vals, int32_t* t_rowptr, int32_t* t_colind, float* t_vals)
{
    if (m < 0 || k < 0 || nnz < 0) return fail(DA_ERR_INVALID_ARG, "negative size%s");
    if (m > 0x7ffffffeLL || k > 0x7ffffffeLL || nnz > 0x7fffffffLL)
        return fail(DA_ERR_INVALID_ARG, "size beyond the int32 index range%s");
    if (!t_rowptr) return fail(DA_ERR_INVALID_ARG, "null t_rowptr%s");
    if (nnz > 0 && (m == 0 || k == 0)) return fail(DA_ERR_INVALID_ARG, "stored entries in a matrix without rows or columns%s");
    if (nnz > 0 && (!rowptr || !colind || !vals || !t_colind || !t_vals))
        return fail(DA_ERR_INVALID_ARG, "null array with nnz > 0%s");
    return DA_OK;
}

// The radix passes of the transpose on the given scratch memory.  Every part of the scratch that
// a kernel reads was written earlier in the same call (keys / rows / values of the ping-pong, the
// whole histogram, every chunk sum), so stale contents of a reused buffer are never seen.
int enqueue_transpose(int64_t m, int64_t k, int64_t nnz, const int32_t* rowptr, const int32_t* colind,
                      const float* vals, int32_t* t_rowptr, int32_t* t_colind, float* t_vals,
                      void* workspace, size_t workspace_bytes, void* stream)
{
    const TransposePlan t = plan_transpose(k, nnz);
    if (nnz > 0 && (!workspace || workspace_bytes < t.bytes))
        return fail(DA_ERR_INVALID_ARG, "workspace missing or smaller than da_csr_transpose_workspace reports%s");
    if (nnz > 0 && reinterpret_cast<uintptr_t>(workspace) % 256 != 0)
        return fail(DA_ERR_INVALID_ARG, "workspace is not 256-byte aligned%s");
    hipStream_t s = (hipStream_t)stream;
    const int n = (int)nnz;
    char* ws = static_cast<char*>(workspace);
    const int* sorted_keys = nullptr;
    if (n > 0) {
        int* keys[2] = {reinterpret_cast<int*>(ws + t.off_keys[0]), reinterpret_cast<int*>(ws + t.off_keys[1])};
        int* rows[2] = {reinterpret_cast<int*>(ws + t.off_rows[0]), reinterpret_cast<int*>(ws + t.off_rows[1])};
        float* vbuf[2] = {reinterpret_cast<float*>(ws + t.off_vals[0]), reinterpret_cast<float*>(ws + t.off_vals[1])};
        int* hist = reinterpret_cast<int*>(ws + t.off_hist);
        int* part = reinterpret_cast<int*>(ws + t.off_part);
        const int mask = (1 << t.digit_bits) - 1;
        const int* keys_in = colind;
        const int* rows_in = nullptr;
        const float* vals_in = vals;
        for (int p = 0; p < t.passes; ++p) {
            const int shift = p * t.digit_bits;
            const bool last = p == t.passes - 1;
            int* keys_out = keys[p & 1];
            int* rows_out = last ? t_colind : rows[p & 1];
            float* vals_out = last ? t_vals : vbuf[p & 1];
            hipLaunchKernelGGL(radix_count_kernel, dim3(t.nblocks), dim3(kSortBlock), 0, s, keys_in, n, shift, mask, hist,
                               t.nblocks);
            hipLaunchKernelGGL(scan_reduce_kernel, dim3((unsigned)t.parts), dim3(kSortBlock), 0, s, hist, t.hist_len, part);
            hipLaunchKernelGGL(scan_top_kernel, dim3(1), dim3(kSortBlock), 0, s, part, (int)t.parts);
            hipLaunchKernelGGL(scan_apply_kernel, dim3((unsigned)t.parts), dim3(kSortBlock), 0, s, hist, t.hist_len, part);
            if (p == 0)
                hipLaunchKernelGGL(radix_scatter_kernel<true>, dim3(t.nblocks), dim3(kSortBlock), 0, s, keys_in, rows_in,
                                   vals_in, n, shift, mask, hist, t.nblocks, keys_out, rows_out, vals_out, rowptr, (int)m);
            else
                hipLaunchKernelGGL(radix_scatter_kernel<false>, dim3(t.nblocks), dim3(kSortBlock), 0, s, keys_in, rows_in,
                                   vals_in, n, shift, mask, hist, t.nblocks, keys_out, rows_out, vals_out, rowptr, (int)m);
            keys_in = keys_out;
            rows_in = rows_out;
            vals_in = vals_out;
        }
        sorted_keys = keys_in;
    }
    hipLaunchKernelGGL(rowptr_from_sorted_kernel, dim3((unsigned)((k + 1 + kSortBlock - 1) / kSortBlock)), dim3(kSortBlock),
                       0, s, sorted_keys, n, (int)k, t_rowptr);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "da_csr_transpose launch");
    return DA_OK;
}

}  // namespace

extern "C" {

int da_eb_schedule_workspace(int64_t k, int64_t nnz, int unit, size_t* bytes)
{
    if (!bytes) return fail(DA_ERR_INVALID_ARG, "null bytes%s");
    if (k < 0 || nnz < 0 || unit < 1) return fail(DA_ERR_INVALID_ARG, "negative size or unit < 1%s");
    if (k > 0x7ffffffeLL || nnz > 0x7fffffffLL) return fail(DA_ERR_INVALID_ARG, "size beyond the int32 index range%s");
    if (k > (1LL << 30)) return fail(DA_ERR_UNSUPPORTED, "more than 2^30 columns%s");
    *bytes = plan_transpose(2 * k, (nnz + unit - 1) / unit).bytes;        // sort keys lie in [0, 2k)
    return DA_OK;
}

int da_eb_schedule(int64_t m, int64_t k, int64_t nnz, const int32_t* rowptr, const int32_t* colind, int unit,
                   int32_t* order, int32_t* first_segment, void* workspace, size_t workspace_bytes, void* stream)
{
    const ScheduleJob job{unit, order, first_segment, nullptr, nullptr, workspace, workspace_bytes};
    return enqueue_schedules(m, k, nnz, rowptr, colind, &job, 1, stream);
}

}  // extern "C"

namespace {

// Builds up to kMaxSortJobs schedules of one matrix side by side: every stage is one launch whose
// blockIdx.y selects the schedule, so four chunk sizes cost the launches of one.  The number of
// radix passes depends on k alone and is therefore the same for every job.
int enqueue_schedules(int64_t m, int64_t k, int64_t nnz, const int32_t* rowptr, const int32_t* colind,
                      const ScheduleJob* jobs, int njobs, void* stream)
{
    if (m < 0 || k < 0 || nnz < 0) return fail(DA_ERR_INVALID_ARG, "negative size or unit < 1%s");
    if (m > 0x7ffffffeLL || k > 0x7ffffffeLL || nnz > 0x7fffffffLL)
        return fail(DA_ERR_INVALID_ARG, "size beyond the int32 index range%s");
    if (k > (1LL << 30)) return fail(DA_ERR_UNSUPPORTED, "more than 2^30 columns%s");
    if (njobs < 1 || njobs > kMaxSortJobs) return fail(DA_ERR_INVALID_ARG, "number of schedules out of range%s");
    for (int i = 0; i < njobs; ++i)
        if (jobs[i].unit < 1) return fail(DA_ERR_INVALID_ARG, "negative size or unit < 1%s");
    if (nnz == 0) return DA_OK;
    if (m == 0) return fail(DA_ERR_INVALID_ARG, "stored entries in a matrix without rows%s");
    if (!rowptr || !colind) return fail(DA_ERR_INVALID_ARG, "null rowptr, colind or order%s");
    TransposePlan t[kMaxSortJobs];
    int n[kMaxSortJobs];
    int *keys[kMaxSortJobs][2], *ids[kMaxSortJobs][2];
    float* pad[kMaxSortJobs][2];
    KeyJobs kj{};
    unsigned max_units_blocks = 0, max_nblocks = 0, max_parts = 0;
    for (int i = 0; i < njobs; ++i) {
        const ScheduleJob& J = jobs[i];
        if (!J.order) return fail(DA_ERR_INVALID_ARG, "null rowptr, colind or order%s");
        const int64_t nunits = (nnz + J.unit - 1) / J.unit;
        t[i] = plan_transpose(2 * k, nunits);
        if (!J.workspace || J.workspace_bytes < t[i].bytes)
            return fail(DA_ERR_INVALID_ARG, "workspace missing or smaller than da_eb_schedule_workspace reports%s");
        if (reinterpret_cast<uintptr_t>(J.workspace) % 256 != 0)
            return fail(DA_ERR_INVALID_ARG, "workspace is not 256-byte aligned%s");
        char* ws = static_cast<char*>(J.workspace);
        for (int b = 0; b < 2; ++b) {
            keys[i][b] = reinterpret_cast<int*>(ws + t[i].off_keys[b]);
            ids[i][b] = reinterpret_cast<int*>(ws + t[i].off_rows[b]);
            pad[i][b] = reinterpret_cast<float*>(ws + t[i].off_vals[b]);
        }
        n[i] = (int)nunits;
        int* part = reinterpret_cast<int*>(ws + t[i].off_part);
        // without a caller's counter the chunk sums serve: they are free until the first scan
        kj.j[i] = KeyJob{J.unit, n[i], keys[i][0], ids[i][0], pad[i][0], J.first_segment ? J.first_segment : part, J.rows_by_unit};
        const unsigned ub = (unsigned)((n[i] + kSortBlock - 1) / kSortBlock);
        max_units_blocks = ub > max_units_blocks ? ub : max_units_blocks;
        max_nblocks = (unsigned)t[i].nblocks > max_nblocks ? (unsigned)t[i].nblocks : max_nblocks;
        max_parts = (unsigned)t[i].parts > max_parts ? (unsigned)t[i].parts : max_parts;
    }
    hipStream_t s = (hipStream_t)stream;
    const unsigned nj = (unsigned)njobs;
    hipLaunchKernelGGL(schedule_clear_kernel, dim3(1), dim3(64), 0, s, kj, njobs);
    hipLaunchKernelGGL(schedule_keys_kernel, dim3(max_units_blocks, nj), dim3(kSortBlock), 0, s, (int)m, (int)k, (int)nnz, rowptr,
                       colind, kj);
    const int mask = (1 << t[0].digit_bits) - 1;
    for (int p = 0; p < t[0].passes; ++p) {
        const int shift = p * t[0].digit_bits;
        const int in = p & 1, out = in ^ 1;
        const bool last = p == t[0].passes - 1;
        SortJobs sj{};
        for (int i = 0; i < njobs; ++i) {
            char* ws = static_cast<char*>(jobs[i].workspace);
            SortJob& S = sj.j[i];
            S.keys_in = keys[i][in]; S.rows_in = ids[i][in]; S.vals_in = pad[i][in];
            S.keys_out = keys[i][out];
            S.rows_out = last ? jobs[i].order : ids[i][out];
            // the last pass delivers the first rows of the chunks, in schedule order, where the caller wants them
            S.vals_out = (last && jobs[i].first_rows) ? reinterpret_cast<float*>(jobs[i].first_rows) : pad[i][out];
            S.hist = reinterpret_cast<int*>(ws + t[i].off_hist);
            S.part = reinterpret_cast<int*>(ws + t[i].off_part);
            S.hist_len = t[i].hist_len;
            S.n = n[i]; S.nblocks = t[i].nblocks; S.parts = (int)t[i].parts;
        }
        hipLaunchKernelGGL(radix_count_jobs_kernel, dim3(max_nblocks, nj), dim3(kSortBlock), 0, s, sj, shift, mask);
        hipLaunchKernelGGL(scan_reduce_jobs_kernel, dim3(max_parts, nj), dim3(kSortBlock), 0, s, sj);
        hipLaunchKernelGGL(scan_top_jobs_kernel, dim3(nj), dim3(kSortBlock), 0, s, sj);
        hipLaunchKernelGGL(scan_apply_jobs_kernel, dim3(max_parts, nj), dim3(kSortBlock), 0, s, sj);
        hipLaunchKernelGGL(radix_scatter_jobs_kernel, dim3(max_nblocks, nj), dim3(kSortBlock), 0, s, sj, shift, mask);
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "da_eb_schedule launch");
    return DA_OK;
}

}  // namespace

extern "C" {

int da_spmm_release(const int32_t* rowptr)
{
    // the references are dropped outside the mutex: the last one frees device memory, which waits
    // for the device
    std::shared_ptr<DeviceBlock> dropped[16];
    {
        std::lock_guard<std::mutex> lk(g_plan_mu);
        int n = 0;
        for (auto& pl : g_plans)
            if (pl.block && (!rowptr || pl.rowptr == rowptr)) {
                dropped[n++] = std::move(pl.block);
                pl = Plan{};
            }
    }
    return DA_OK;
}

int da_spmm_prepare(int64_t m, int64_t k, int64_t nnz, const int32_t* rowptr, const int32_t* colind, void* stream)
{
    if (m < 0 || k < 0 || nnz < 0) return fail(DA_ERR_INVALID_ARG, "negative size%s");
    if (m > 0x7ffffffeLL || k > 0x7ffffffeLL || nnz > 0x7fffffffLL)
        return fail(DA_ERR_INVALID_ARG, "size beyond the int32 index range%s");
    if (m == 0 || nnz == 0) return DA_OK;
    if (!rowptr || !colind) return fail(DA_ERR_INVALID_ARG, "null rowptr or colind%s");
    if (debug_validate()) {
        const int v = da_csr_validate(m, k, nnz, rowptr, colind, stream);
        if (v != DA_OK) return v;
    }
    if (k > (1LL << 30)) { remember_nnz(rowptr, m, nnz); return DA_OK; }    // no schedule for such widths
    Plan pl;
    pl.rowptr = rowptr; pl.colind = colind; pl.m = m; pl.nnz = nnz;
    size_t ints = 64, ws_bytes = 0, ws_off[4];             // the first 4 ints receive the segment sizes
    for (int i = 0; i < 4; ++i) {
        pl.units[i] = (int)((nnz + kPlanUnits[i] - 1) / kPlanUnits[i]);
        ints += 3 * (size_t)((pl.units[i] + 63) & ~63);     // the order and, twice, the first rows of the chunks
        ws_off[i] = ws_bytes;                               // the four sorts run side by side, each in its own part
        ws_bytes += align256(plan_transpose(2 * k, pl.units[i]).bytes);
    }
    pl.block = std::make_shared<DeviceBlock>();
    DeviceBlock ws;
    hipError_t e = hipMalloc(&pl.block->p, ints * sizeof(int));
    if (e != hipSuccess) return hip_fail(e, "hipMalloc");
    e = hipMalloc(&ws.p, ws_bytes);
    if (e != hipSuccess) return hip_fail(e, "hipMalloc");
    size_t off = 64;
    int* seg = static_cast<int*>(pl.block->p);
    ScheduleJob jobs[4];
    for (int i = 0; i < 4; ++i) {
        pl.order[i] = seg + off;
        off += (size_t)((pl.units[i] + 63) & ~63);
        pl.first_row[i] = seg + off;
        off += (size_t)((pl.units[i] + 63) & ~63);
        pl.row_by_chunk[i] = seg + off;
        off += (size_t)((pl.units[i] + 63) & ~63);
        jobs[i] = ScheduleJob{kPlanUnits[i], pl.order[i], seg + i, pl.first_row[i], pl.row_by_chunk[i],
                              static_cast<char*>(ws.p) + ws_off[i], ws_bytes - ws_off[i]};
    }
    int status = enqueue_schedules(m, k, nnz, rowptr, colind, jobs, 4, stream);
    e = hipSuccess;
    if (status == DA_OK)
        e = hipMemcpyAsync(pl.first_units, seg, sizeof pl.first_units, hipMemcpyDeviceToHost, (hipStream_t)stream);
    if (e == hipSuccess) e = hipStreamSynchronize((hipStream_t)stream);
    if (status == DA_OK && e != hipSuccess) status = hip_fail(e, "da_spmm_prepare");
    if (status != DA_OK) return status;
    remember_nnz(rowptr, m, nnz);
    std::shared_ptr<DeviceBlock> old;                      // freed after the mutex is released
    {
        std::lock_guard<std::mutex> lk(g_plan_mu);
        Plan* slot = nullptr;
        for (auto& q : g_plans)
            if (q.block && q.rowptr == rowptr && q.m == m) { slot = &q; break; }  // an older plan of this matrix
        if (slot && slot->captured) {
            // A recorded graph reads the old orders on every replay: they stay.  When they describe
            // the same matrix shape the old plan simply remains in use; otherwise the new one takes
            // another slot and the old one lives on until da_spmm_release.
            if (slot->colind == colind && slot->nnz == nnz) return DA_OK;
            slot->rowptr = nullptr;                        // no longer found by lookups; memory kept
            slot = nullptr;
        }
        if (!slot) {
            for (int tries = 0; tries < 16 && !slot; ++tries) {
                Plan* cand = &g_plans[g_plan_next];
                g_plan_next = (g_plan_next + 1) % 16;
                if (!(cand->block && cand->captured)) slot = cand;
            }
            if (!slot) return DA_OK;                       // every slot is pinned by a graph: no plan for this matrix
        }
        old = std::move(slot->block);
        *slot = pl;
    }
    return DA_OK;
}

const char* da_spmm_algo_name(int algo)
{
    return (algo >= 0 && algo < DA_NUM_ALGOS) ? kNames[algo] : nullptr;
}

const char* da_spmm_last_error(void) { return g_err; }

}  // extern "C"
