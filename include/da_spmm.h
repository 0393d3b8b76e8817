/*
 * da_spmm.h -- C ABI of libdaspmm.so: data-aware CSR sparse x dense matrix multiply for
 * AMD MI355X (gfx950, wave64).
 *
 * The operation is the paper's problem statement (Sec. 3.1, Fig. 2(b)):  Y = A * X  with A an
 * M x K sparse matrix, X a K x N dense matrix and Y an M x N dense matrix; here named
 * C = A * B with A in CSR form (m x k), B (k x N) and C (m x N) dense, row-major.
 * Every algorithm id computes the same C (up to fp32 rounding order); the ids differ in how the
 * three loops of Fig. 2(a) are mapped onto the machine (Sec. 3.2-3.4, Table 1) and the selector
 * picks one of them from input characteristics (Sec. 5.1, Table 2).
 *
 * Conventions
 *   - every pointer is a DEVICE pointer unless the comment says "host";
 *   - buffers are borrowed for the duration of the stream-ordered execution of the call; the
 *     caller owns and frees them; B and C must not overlap;
 *   - calls only enqueue work on `stream` (a hipStream_t passed as void*, NULL = the default
 *     stream) and return without synchronising, except da_spmm_features which has to return
 *     values to the host;
 *   - every function returns a da_status (0 = success) and never throws or aborts;
 *     da_spmm_last_error() gives a thread-local text for the last failure.
 *
 * Environment switches (read at every call; for debugging and measurement, not for production)
 *   DA_SPMM_DEBUG_VALIDATE=1   check the CSR arrays on the device before every product / transpose
 *   DA_SPMM_NO_SCHEDULE=1      ignore the chunk orders of prepared matrices (da_spmm_prepare)
 *   DA_SPMM_NO_SPLIT=1         deal such an order to the XCDs as one segment instead of two
 *   DA_SPMM_SPLIT_SHORT_ROWS=1 EB+SR on prepared matrices: split short rows at chunk boundaries again
 *   DA_SPMM_WIDE=1             force the kernels with 64-bit gather addresses
 *   DA_SPMM_TUNE=1             honour DA_SPMM_V / _G / _NV / _CHUNK / _PIN / _STRIPE, which override the
 *                              launch geometry; unsupported combinations return DA_ERR_UNSUPPORTED
 */
#ifndef DA_SPMM_H
#define DA_SPMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DA_OK = 0,
    DA_ERR_INVALID_ARG = 1, /* negative size, size beyond the int32 index range, null rowptr / C */
    DA_ERR_BAD_ALGO = 2,    /* algorithm id outside 0..7                                        */
    DA_ERR_UNSUPPORTED = 3,
    DA_ERR_HIP = 4          /* a HIP runtime call or kernel launch failed                        */
} da_status;

/* Algorithm ids in the column order of the paper's Table 1:
 *   M-loop  RB = row balance: a worker owns whole rows              (Sec. 3.2, design M1)
 *           EB = element balance: a worker owns a fixed number of
 *                consecutive stored entries                          (Sec. 3.2, design M2)
 *   N-loop  RM = neighbouring lanes hold neighbouring columns n of one B row (coalesced row
 *                segments, Sec. 3.3 design N1); CM = neighbouring lanes hold different rows /
 *                entries and each lane walks its own strip of columns (Sec. 3.3 design N2).
 *                B and C are row-major in memory for every id; the axis is the lane->n mapping.
 *   K-loop  SR = one worker adds a row's products one after another  (Sec. 3.4, design K1)
 *           PR = the lanes of a wave hold different entries and combine them with a reduction
 *                tree; under EB this is the conditional reduction    (Sec. 3.4 design K2; Sec. 4)
 */
enum {
    DA_RB_RM_SR = 0, DA_RB_RM_PR = 1, DA_RB_CM_SR = 2, DA_RB_CM_PR = 3,
    DA_EB_RM_SR = 4, DA_EB_RM_PR = 5, DA_EB_CM_SR = 6, DA_EB_CM_PR = 7,
    DA_NUM_ALGOS = 8
};

/* Input characteristics used by the selector (Sec. 5.1, Table 2: nnz, matrix size, standard
 * deviation of the row lengths, N; extended by the mean and maximum row length).  Host struct. */
typedef struct {
    int64_t rows;          /* m                                                        */
    int64_t nnz;           /* stored entries of A                                      */
    double  row_nnz_mean;  /* nnz / m                                                  */
    double  row_nnz_std;   /* population standard deviation (divide by m) of row length */
    double  row_nnz_max;   /* longest row                                              */
    int64_t N;             /* width of B and C                                         */
} da_features;

/*
 * C = A * B  (Sec. 3.1, Fig. 2; algorithm space of Sec. 3.2-3.4 / Table 1, techniques of Sec. 4).
 *
 *   m, k, N   sizes; 0 <= m, k < 2^31, 0 <= N < 2^31.  m == 0 or N == 0 is a successful no-op.
 *   rowptr    int32[m+1], rowptr[0] == 0, non-decreasing, rowptr[m] == nnz < 2^31
 *   colind    int32[nnz], 0 <= colind[p] < k; need not be sorted inside a row; repeated (i,j)
 *             entries add
 *   vals      fp32[nnz]          (colind, vals and B may be NULL only when nnz == 0)
 *   B         fp32[k*N], row-major, leading dimension N
 *   C         fp32[m*N], row-major, leading dimension N; every element is OVERWRITTEN (rows
 *             without stored entries become +0)
 *   algo      0..7, see the enum above
 *   stream    hipStream_t (NULL = default stream)
 *
 * The contents of rowptr / colind are not validated (they live on the device); indices outside
 * their range are undefined behaviour.  EB ids enqueue two kernels (a pass that zeroes the rows
 * which will receive atomic additions, then the product); results of ids that use atomics can
 * differ in the last bits from run to run.  Returns DA_ERR_INVALID_ARG, DA_ERR_BAD_ALGO or
 * DA_ERR_HIP on failure; nothing is enqueued for the first two.
 */
int da_spmm(int64_t m, int64_t k, int64_t N,
            const int32_t *rowptr, const int32_t *colind, const float *vals,
            const float *B, float *C, int algo, void *stream);

/* Storage order of a dense operand. */
enum { DA_ROW_MAJOR = 0, DA_COL_MAJOR = 1 };

/*
 * The same product with explicit storage order and leading dimension of B and C: the paper's
 * literal N-loop axis (Sec. 3.3: X stored row- or column-major; "we have control on the
 * intermediate matrix layout").  Element (r, n) of B is at B[r*ldb + n] for DA_ROW_MAJOR
 * (ldb >= N) and at B[r + n*ldb] for DA_COL_MAJOR (ldb >= k); likewise C with ldc >= N or
 * ldc >= m.  Everything else is as for da_spmm, which equals
 * da_spmm_ex(..., B, N, DA_ROW_MAJOR, C, N, DA_ROW_MAJOR, ...).  Only the elements (r, n) with
 * r < m (k for B), n < N are read or written; padding between rows / columns is left untouched.
 * 16-byte accesses are used only for row-major operands whose leading dimensions are multiples
 * of 4 and whose bases are 16-byte aligned; any other combination runs with 4-byte accesses.
 * Returns DA_ERR_INVALID_ARG for an unknown layout or a leading dimension that is too small.
 */
int da_spmm_ex(int64_t m, int64_t k, int64_t N,
               const int32_t *rowptr, const int32_t *colind, const float *vals,
               const float *B, int64_t ldb, int layout_b,
               float *C, int64_t ldc, int layout_c, int algo, void *stream);

/*
 * Data-aware algorithm choice (Sec. 5.1): maps input characteristics to an algorithm id 0..7 by
 * walking a forest of boosted regression trees compiled into the library (trained offline on this
 * GPU on seeded synthetic matrices; each tree adds to a score per id, the best score wins).  `f` is a HOST pointer.  Pure and deterministic; no device work.
 * Returns the id, or a negative da_status (-DA_ERR_INVALID_ARG) when f is NULL or holds
 * negative / non-finite entries.
 */
int da_spmm_select(const da_features *f);

/*
 * Extract the selector's input characteristics (Sec. 5.1, Table 2) from the row pointers with one
 * device reduction.  rowptr is a device pointer (int32[m+1]); `out` is a HOST pointer.  Blocks
 * until the result is on the host (synchronises `stream`).  m == 0 gives all-zero features.
 * Side effect: the library remembers nnz for this (rowptr, m) pair in a small host table and
 * later da_spmm calls on the same matrix use it to size the grids of the EB algorithms (a
 * missing or stale entry only costs speed: EB kernels read nnz on the device and cover every
 * stored entry whatever the grid size).
 */
int da_spmm_features(int64_t m, int64_t N, const int32_t *rowptr, void *stream, da_features *out);

/*
 * Optional per-matrix preparation for the EB algorithms (Sec. 3.2 design M2).  An EB worker owns a
 * fixed number of consecutive stored entries; which worker takes which chunk does not change the
 * result, but it decides which rows of B are in flight together.  In a row much longer than a
 * chunk the sorted column indices make consecutive chunks cover successive column ranges, so
 * handing those chunks to the workers in the order of the columns they cover turns the random
 * gather of B into a sweep from low to high rows: concurrently running workers share a narrow
 * band of B that stays in the L2 caches.
 *
 * da_spmm_prepare builds those orders for the chunk sizes the EB kernels use, together with the row
 * that owns each chunk's first entry (a hint the kernels check against the row pointers before they
 * use it), and keeps them, keyed by (rowptr, colind, m), in library-owned device memory (about
 * nnz/11 ints) until da_spmm_release
 * (rowptr == NULL releases every matrix) or until 16 other matrices have been prepared.  Later
 * da_spmm / da_spmm_ex calls with the same rowptr, colind and m and an EB algorithm id pick the
 * order up by themselves; results are the same up to fp32 rounding order.  It also records nnz
 * like da_spmm_features does.  A kernel that finds another nnz on the device than the plan was
 * built for ignores the plan, so a stale plan costs speed, never correctness; the contents of
 * colind may change freely.  Allocates and frees temporary device memory, synchronises `stream`.
 * Prepare, release and the product calls may be issued from several host threads; product calls do
 * not serialise each other (the plan table is locked only for the lookup; the plan's memory is
 * reference-counted and freed only after every call that looked it up has launched, and the free
 * itself waits for launched kernels).
 * A HIP graph captured from an EB call on a prepared matrix holds the address of the plan's order.
 * The library notices the capture and from then on never frees that plan by itself (no eviction by
 * later prepares; a re-prepare of the same matrix keeps it): only da_spmm_release frees it, which
 * the caller must not do while the graph is still replayed.  da_spmm_release(NULL) also frees plans
 * that a re-prepare with another nnz has set aside.
 * These two host tables (nnz hints, plans) are the library's only mutable global state; both only
 * steer launch geometry and chunk order, never the result.
 *
 * da_eb_schedule is the building block: order[u], u = 0 .. ceil(nnz/unit)-1, lists the chunk
 * numbers (chunk c = stored entries [c*unit, (c+1)*unit)) sorted by a key in [0, 2k), ties in
 * ascending chunk number -- deterministic.  A chunk inside one row covers a narrow column range
 * and has the key k + (colind[first entry] + colind[last entry])/2: these chunks are swept over B
 * in column order.  A chunk that touches several rows has the key colind[first entry]: all such
 * chunks sort before the others and form a first segment of the schedule (they are latency-bound
 * where the others are bandwidth-bound, and a wave that holds both kinds runs at the pace of the
 * slower).  *first_segment (device, may be NULL) receives the number of chunks of that first
 * segment.  k <= 2^30 (DA_ERR_UNSUPPORTED beyond; da_spmm_prepare then
 * builds no order).  Caller workspace as for da_csr_transpose (size from
 * da_eb_schedule_workspace, 256-byte aligned); enqueues only.
 */
int da_spmm_prepare(int64_t m, int64_t k, int64_t nnz, const int32_t *rowptr, const int32_t *colind,
                    void *stream);
int da_spmm_release(const int32_t *rowptr);
int da_eb_schedule_workspace(int64_t k, int64_t nnz, int unit, size_t *bytes /* host, out */);
int da_eb_schedule(int64_t m, int64_t k, int64_t nnz, const int32_t *rowptr, const int32_t *colind,
                   int unit, int32_t *order, int32_t *first_segment,
                   void *workspace, size_t workspace_bytes, void *stream);

/*
 * Debug aid: check on the device that the CSR arrays are well formed -- rowptr[0] == 0, rowptr
 * non-decreasing, rowptr[m] == nnz (skipped when nnz is passed as -1), every colind in [0, k).
 * The product kernels trust these properties (Sec. 3.1 takes a valid CSR matrix as given) and a
 * violation can make them read out of bounds, so this call is the way to vet arrays of unknown
 * origin.  colind is only read after the row pointers passed, over rowptr[m] entries.
 * Allocates an 8-byte device buffer, synchronises `stream`, frees the buffer.  Returns DA_OK,
 * DA_ERR_INVALID_ARG (last error names the violated property) or DA_ERR_HIP.
 * Setting the environment variable DA_SPMM_DEBUG_VALIDATE=1 makes da_spmm, da_spmm_ex and
 * da_csr_transpose run this check first on every call (and return its error).
 */
int da_csr_validate(int64_t m, int64_t k, int64_t nnz, const int32_t *rowptr, const int32_t *colind,
                    void *stream);

/*
 * CSR arrays of the transpose.  The paper's GCN experiment (Sec. 6) runs the SpMM inside a graph
 * neural network layer; training such a layer needs the gradient of <G, A*X> with respect to X,
 * which is A^T * G -- the same sparse-times-dense product on the transposed matrix.  This call
 * builds A^T once per graph so that da_spmm (and the selector) serve the backward pass too.
 *
 *   A        m x k, CSR: rowptr int32[m+1], colind int32[nnz] (each in [0, k)), vals fp32[nnz];
 *            nnz is passed by the caller and must equal rowptr[m]
 *   A^T      k x m, CSR: t_rowptr int32[k+1], t_colind int32[nnz], t_vals fp32[nnz], written by
 *            the call; inside every row of A^T the indices ascend (entries of equal (row, column)
 *            keep their stored order), so the result is deterministic bit for bit
 *   workspace  device scratch of at least the size da_csr_transpose_workspace reports for the
 *            same (m, k, nnz) (about 24 bytes per stored entry), 256-byte aligned, owned by the
 *            caller, free for reuse once the stream has passed the call; may be NULL when nnz == 0
 * The call allocates nothing, only enqueues kernels on `stream` and does not synchronise.  Inputs
 * and outputs must not overlap.  As for da_spmm, the arrays are trusted to be well formed.
 * Errors: DA_ERR_INVALID_ARG (negative or too large sizes, null arrays with nnz > 0, workspace
 * missing / too small / misaligned), DA_ERR_HIP (launch failure).
 */
int da_csr_transpose_workspace(int64_t m, int64_t k, int64_t nnz, size_t *bytes /* host, out */);
int da_csr_transpose(int64_t m, int64_t k, int64_t nnz,
                     const int32_t *rowptr, const int32_t *colind, const float *vals,
                     int32_t *t_rowptr, int32_t *t_colind, float *t_vals,
                     void *workspace, size_t workspace_bytes, void *stream);

/*
 * da_csr_transpose for callers that cannot allocate device memory and have no workspace to hand
 * over: code that runs under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments (without the workspace), same kernels and bit-for-bit the same result
 * as da_csr_transpose; the radix passes run in a static device array of DA_NOALLOC_SCRATCH_BYTES
 * (32 MiB) that every GPU the library is loaded on holds until the process ends.  The call
 * allocates and frees nothing and does not synchronise; it skips the DA_SPMM_DEBUG_VALIDATE check
 * (which allocates).
 * Limit: da_csr_transpose_workspace(m, k, nnz) must not exceed DA_NOALLOC_SCRATCH_BYTES (about
 * 1.39 million stored entries); beyond it the call returns DA_ERR_UNSUPPORTED, enqueues nothing
 * and the last-error text says so.
 * All calls on one GPU share that GPU's array: calls whose execution can overlap on one GPU
 * (different streams, different host threads) race on it -- order them on one stream or with
 * events.  Nothing in the array needs clearing between calls (every part is written before it is
 * read within a call).  The first call on a device looks the array's address up
 * (hipGetSymbolAddress); make that first call outside a stream capture.
 */
#define DA_NOALLOC_SCRATCH_BYTES ((size_t)32 << 20)
int da_csr_transpose_noalloc(int64_t m, int64_t k, int64_t nnz,
                             const int32_t *rowptr, const int32_t *colind, const float *vals,
                             int32_t *t_rowptr, int32_t *t_colind, float *t_vals, void *stream);

/* "RB+RM+SR" ... "EB+CM+PR" (Table 1 naming); NULL for an id outside 0..7.  Host string, static. */
const char *da_spmm_algo_name(int algo);

/* Text describing the last failure on the calling thread ("" if none).  Host string, valid until
 * the next failing call on the same thread. */
const char *da_spmm_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* DA_SPMM_H */
