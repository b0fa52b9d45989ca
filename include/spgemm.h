/*
 * spgemm.h - C ABI of the MI355X (gfx950) row-wise sparse x sparse product library.
 *
 * The operation is the one the paper states in section 2.1, A_ij = sum_k B_ik C_kj
 * with every matrix in compressed sparse rows (pos/crd/val arrays, 0-based), run in
 * the row-wise loop order i -> k -> j of section 2.2 (Gustavson; "first-order
 * scattering").  In this header the product is written C = A * B.  The paper's four
 * workspace stages (section 4.3: insert, sort, merge, compress) are executed per
 * output row inside on-chip workspaces; the output structure is precomputed by a
 * symbolic phase, the route section 5.4 names for parallel workspaces.
 *
 * Conventions for every entry point
 *   - All matrix arrays are DEVICE pointers on the current HIP device unless a
 *     parameter says "host".  Input arrays are borrowed: never written, never freed.
 *   - rowptr is int64 (rows+1 entries, rowptr[0] == 0, non-decreasing,
 *     rowptr[rows] == nnz); colidx is int32 in [0, cols); values are float or double.
 *     Input rows need not be sorted and may repeat a column: a repeated entry simply
 *     contributes further products.
 *   - Result: CSR, 0-based, columns strictly ascending inside each row, no duplicates.
 *     An output coordinate is stored whenever at least one product lands on it, also
 *     when the sum is exactly zero (workspaces never drop components, section 4.3).
 *   - Every call returns an int status (0 = success, negative = spgemm_status below).
 *     Nothing throws or aborts across this boundary.  Argument checks run before the
 *     first HIP call, so they behave the same on a host without a GPU.
 *   - Work is enqueued on the stream given at spgemm_create.  A handle is not
 *     thread-safe; use one handle per host thread.
 */
#ifndef SPGEMM_H_
#define SPGEMM_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SPGEMM_OK = 0,
  SPGEMM_INVALID_ARG = -1,     /* null pointer, negative size, bad enum */
  SPGEMM_DIM_MISMATCH = -2,    /* A.cols != B.rows, or a plan used with other shapes */
  SPGEMM_DTYPE_MISMATCH = -3,  /* A and B value types differ */
  SPGEMM_UNSUPPORTED = -4,     /* a size this build cannot handle (see spgemm_symbolic) */
  SPGEMM_ALLOC_FAILED = -5,    /* allocator callback or hipMalloc returned null */
  SPGEMM_HIP_ERROR = -6,       /* a HIP runtime call failed; text in spgemm_last_error */
  SPGEMM_BAD_STATE = -7,       /* plan/handle misuse */
  SPGEMM_INVALID_INPUT = -8    /* device-side check: column out of range or rowptr not monotone */
} spgemm_status;

typedef enum { SPGEMM_F32 = 0, SPGEMM_F64 = 1 } spgemm_dtype;

/* One CSR operand (section 2.1's level formats Dense, Compressed). */
typedef struct {
  int64_t rows, cols, nnz;
  const int64_t* rowptr; /* device, rows+1 */
  const int32_t* colidx; /* device, nnz (may be null when nnz == 0) */
  const void* values;    /* device, nnz elements of dtype (may be null when nnz == 0) */
  int32_t dtype;         /* spgemm_dtype */
} spgemm_csr;

/* Device-memory callbacks.  alloc returns a device pointer aligned to at least 256
 * bytes or null; free releases one.  Both may be called from any API entry point on
 * the calling thread.  When no allocator is given the library uses hipMalloc/hipFree. */
typedef struct {
  void* (*alloc)(void* ctx, size_t bytes);
  void (*free)(void* ctx, void* ptr);
  void* ctx;
} spgemm_allocator;

typedef struct spgemm_context* spgemm_handle;
typedef struct spgemm_plan_s* spgemm_plan;

/* Kernel classes for statistics (per-class accumulated time and launch count). */
enum {
  SPGEMM_K_COUNT = 0,  /* per-row intermediate-product count + input checks */
  SPGEMM_K_BIN,        /* histogram, offsets, wavefront-scan scatter of row ids */
  SPGEMM_K_SYM_ESC,    /* symbolic, sorted-list workspace (expand, sort, count unique) */
  SPGEMM_K_SYM_HASH,   /* symbolic, LDS hash-set workspace */
  SPGEMM_K_SYM_DENSE,  /* symbolic, LDS dense flag (bitmap) workspace */
  SPGEMM_K_SCAN,       /* exclusive scan of row counts -> C.rowptr */
  SPGEMM_K_NUM_ESC,    /* numeric, sorted-list workspace (expand, sort, merge duplicates) */
  SPGEMM_K_NUM_HASH,   /* numeric, LDS hash workspace + sort */
  SPGEMM_K_NUM_DENSE,  /* numeric, LDS dense workspace over column tiles (direct or ranked) */
  SPGEMM_K_NUM_STAGED, /* numeric, coordinate list staged in LDS, windowed counting sort + merge */
  SPGEMM_K_BLOCK_PTR,  /* per-B-row column-block offsets used by the dense numeric kernel */
  SPGEMM_NUM_KERNEL_CLASSES
};

#define SPGEMM_NUM_BINS 8

typedef struct {
  int64_t ip_total;                     /* intermediate products, sum over rows */
  int64_t nnz_c;                        /* nonzeros of C */
  /* bins: symbolic 0,1 sorted list; 2,3 hash; 4,5,6 dense; 7 rows without products.
   *       numeric  0,1 sorted list; 2,3 hash; 4 staged list; 5,6 dense; 7 empty rows of C. */
  int64_t sym_bin_rows[SPGEMM_NUM_BINS];
  int64_t num_bin_rows[SPGEMM_NUM_BINS];
  int64_t sym_bin_ip[SPGEMM_NUM_BINS];   /* intermediate products per symbolic bin (rows beyond 2^31-1 products saturate) */
  int64_t num_bin_ip[SPGEMM_NUM_BINS];   /* intermediate products per numeric bin */
  int64_t num_bin_nnz[SPGEMM_NUM_BINS];  /* entries of C per numeric bin */
  double kernel_ms[SPGEMM_NUM_KERNEL_CLASSES];      /* summed HIP-event time of the last symbolic + numeric */
  int32_t kernel_launches[SPGEMM_NUM_KERNEL_CLASSES];
  int64_t dense_tiles;        /* column tiles planned for the dense numeric kernel */
  int64_t dense_direct_tiles; /* of those, tiles accumulated by column (one pass) */
  int64_t dense_runs;         /* work items (runs of tiles of one row) */
  int64_t dense_search_tiles; /* of the tiles, whole short rows whose ranks come from bisecting the column list */
  int64_t plan_bytes;         /* device memory the plan holds (per-row arrays, tile lists, block table, structure list) */
  int64_t plan_list_bytes;    /* of those, what the structure list (columns or flag words of the dense rows) was given */
  int64_t plan_list_used;     /* ... and what the symbolic phase filled of it */
} spgemm_stats;

/* Options for spgemm_set_option. */
enum {
  /* 1: bracket every kernel class with HIP events on the handle's stream; spgemm_get_stats
   * then waits for the recorded events and reports the times.  Default 0. */
  SPGEMM_OPT_TIMING = 1,
  /* Route rows through one workspace kind wherever its capacity allows (rows beyond that
   * capacity keep their normal route): 0 = normal binning (default), 1 = sorted-list,
   * 2 = hash, 3 = dense, 4 = staged coordinate list (numeric phase).  All routes compute the same function (the paper's table of
   * library algorithms, section 4.4); tests use this to compare them. */
  SPGEMM_OPT_FORCE_WORKSPACE = 2,
  /* Dense workspace tuning: a block of 8192 columns in which a row of C has at least this
   * many entries is accumulated in a dense array indexed by column (one pass over the
   * products); sparser blocks are grouped and accumulated by rank.  256 or more; default 6144.
   * Applies to the next spgemm_symbolic on the handle. */
  SPGEMM_OPT_DIRECT_MIN = 3,
  /* 1 (default): the plan keeps the column indices of the dense workspace's ranked tiles
   * (up to a third of the free device memory), which saves the numeric phase one pass over
   * those tiles' products; rows that do not fit fall back to the two-pass route.  0: never.
   * A value of 4096 or more limits the list to that many bytes. */
  SPGEMM_OPT_COLUMN_LIST = 4,
  /* 1 (default): for an ascending B the plan holds a table of per-row offsets at every 8192nd
   * column (when it fits 1 GiB), which turns the search for a tile's piece of a B row into two
   * loads.  0: never build it; pieces are found by bisection. */
  SPGEMM_OPT_BLOCK_TABLE = 5,
  /* A short dense row (at most 11264 entries, columns in the plan's list) whose products per entry do
   * not exceed this value is accumulated in one "searched" tile: a product finds its sum by bisection of
   * the row's column list, whatever the width of the row.  0: never.  Default 4. */
  SPGEMM_OPT_SEARCH_RATIO = 6
};

/* Create a handle bound to a HIP stream (hipStream_t passed as void*, null = default
 * stream) and an optional allocator (copied; null = hipMalloc/hipFree).  Makes no HIP call. */
int spgemm_create(spgemm_handle* out, void* hip_stream, const spgemm_allocator* alloc);
int spgemm_destroy(spgemm_handle h);
int spgemm_set_option(spgemm_handle h, int option, int64_t value);

/* Symbolic phase (the structure precomputation of section 5.4): counts intermediate
 * products per row, bins rows, computes |union_k cols(B_k)| per row in per-bin
 * workspaces and scans the counts.
 *   c_rowptr  device, A->rows + 1 int64, caller-owned, written.
 *   nnz_c     host, written with c_rowptr[A->rows].
 *   plan      out; library-owned scratch (row permutations, per-row counts) that
 *             spgemm_numeric needs.  Release with spgemm_plan_destroy.
 * Returns after the result is on the host (two stream synchronisations: after the row
 * classes are known, which sizes the plan's lists, and at the end).
 * SPGEMM_UNSUPPORTED: rows, cols or a B row length of 2^31 or more; a B row of 2^21 or more
 *   entries when some B row is not strictly ascending.
 * SPGEMM_INVALID_INPUT: a device-side check failed; c_rowptr contents are unspecified. */
int spgemm_symbolic(spgemm_handle h, const spgemm_csr* A, const spgemm_csr* B,
                    int64_t* c_rowptr, int64_t* nnz_c, spgemm_plan* plan);

/* Numeric phase: for every row inserts a_ik * b_kj into the row's workspace (section 4.3
 * insertion + deduplication), orders by column and writes the row at c_rowptr[i].
 *   c_rowptr            device, as produced by spgemm_symbolic for this plan.
 *   c_colidx, c_values  device, nnz_c elements each, caller-owned, written
 *                       (may be null when nnz_c == 0).
 * Only enqueues work (no synchronisation).  A plan may be
 * reused for further numeric calls with new values on the same structures.
 * Sums are accumulated in double for both value types and rounded once on output (one exception: the
 * staged coordinate list, taken on request only, stages each float product rounded to float).
 * The plan's scratch is read by the enqueued kernels: spgemm_plan_destroy waits for the stream when a
 * numeric phase is still in flight. */
int spgemm_numeric(spgemm_handle h, spgemm_plan plan, const spgemm_csr* A, const spgemm_csr* B,
                   const int64_t* c_rowptr, int32_t* c_colidx, void* c_values);

/* Whole product.  On success C->rows/cols/nnz/dtype are set and C->rowptr/colidx/values
 * are device buffers obtained from the handle's allocator (hipMalloc without one); the
 * caller owns them and releases them with its allocator's free or spgemm_free_device.
 * Synchronises twice: inside the symbolic phase, and before the plan's scratch is released. */
int spgemm(spgemm_handle h, const spgemm_csr* A, const spgemm_csr* B, spgemm_csr* C);

/* Whole product in a pipeline of row blocks (the GPU counterpart of the pipelining / double buffering
 * of section 5.3: while the workspace of one part of the result is being drained, the next part is
 * already being prepared): A is cut into nblocks blocks of consecutive rows of about equal numbers of
 * intermediate products; the symbolic phase of block t + 1 runs on a second stream of the same
 * priority while the numeric phase of block t runs on the handle's stream, and at most two plans are
 * alive at a time.  The result comes back as row blocks: C_blocks[t] (host array of nblocks structs,
 * written) is the CSR matrix of rows block_rows[t] .. block_rows[t+1] - 1 of C (block_rows: host,
 * nblocks + 1 entries, written), its row pointer starting at 0; stacked, the blocks are exactly the
 * matrix spgemm() returns.  Buffers come from the handle's allocator (three per block; release with
 * its free or spgemm_free_device).  Returns when everything is done. */
int spgemm_pipelined(spgemm_handle h, const spgemm_csr* A, const spgemm_csr* B, int nblocks, spgemm_csr* C_blocks,
                     int64_t* block_rows);

/* Release a device buffer that spgemm() obtained (routes to the allocator's free). */
int spgemm_free_device(spgemm_handle h, void* ptr);

/* Releases the plan's device memory (waits for the stream first when numeric work on the plan may still be
 * running).  A plan refers to its handle: destroy plans before spgemm_destroy of the handle they came from. */
int spgemm_plan_destroy(spgemm_plan plan);

/* Statistics of the plan's last symbolic and numeric runs (host struct, written).  With
 * SPGEMM_OPT_TIMING set this waits for the stream's outstanding timed launches. */
int spgemm_get_stats(spgemm_plan plan, spgemm_stats* out);

/* Text of the last error on this handle (never null; valid until the next call). */
const char* spgemm_last_error(spgemm_handle h);

/* ---- sparse tensor times sparse matrix through mode unfolding ------------------------------
 * Y = X x_mode M for a 3-tensor X(i,j,k) given as device coordinate arrays xi, xj, xk (int32) and
 * xval (nnz each, any order, borrowed): the coordinate of `mode` (1, 2 or 3) is contracted with the
 * rows of M and replaced by M's column l, e.g. mode 3: Y(i,j,l) = sum_k X(i,j,k) M(k,l).  It is
 * computed on the row-wise path through the unfolding of X over that mode (the index folding that
 * section 7.4 of the paper describes for its comparison system; the paper's own SpTTM of section 7.4
 * contracts one mode of a sparse tensor with a matrix into a sparse result, which is this operation):
 * the two kept coordinates fold into the row, the earlier mode major (mode 3: i*J + j, mode 2:
 * i*K + k, mode 1: j*K + k), the contracted coordinate is the column.  A coordinate that occurs
 * several times contributes several products.  The folded row extent and the extent of the contracted
 * mode must be below 2^31 - 1, nnz below 2^32 - 1.
 * Output matrices are device CSR whose buffers come from the handle's allocator (release with its
 * free or spgemm_free_device).  All calls synchronise the handle's stream except the fold calls,
 * which only enqueue.
 * SPGEMM_INVALID_INPUT: a coordinate outside [0,I) x [0,J) x [0,K). */

/* The unfolding itself: out = (product of the two kept extents) x (extent of `mode`) CSR, columns
 * ascending inside each row, repeated coordinates kept as separate entries in input order. */
int sptensor_unfold(spgemm_handle h, int mode, int64_t I, int64_t J, int64_t K, int64_t nnz, const int32_t* xi,
                    const int32_t* xj, const int32_t* xk, const void* xval, int32_t dtype, spgemm_csr* out);

/* Y = X x_mode M as the unfolded CSR matrix (rows as in sptensor_unfold, M->cols columns).
 * SPGEMM_DIM_MISMATCH: M->rows differs from the extent of `mode`. */
int spttm(spgemm_handle h, int mode, int64_t I, int64_t J, int64_t K, int64_t nnz, const int32_t* xi, const int32_t* xj,
          const int32_t* xk, const void* xval, int32_t dtype, const spgemm_csr* M, spgemm_csr* Y);

/* Folding back to a coordinate tensor: Y is the unfolding over `mode` of a tensor of extents I x J x K
 * (so Y->rows is the product of the two kept extents and Y->cols the extent of `mode`); entry p of Y
 * gets its three coordinates in yi[p], yj[p], yk[p] (device, Y->nnz each, caller-owned, written).
 * The values of the coordinate tensor are Y->values as they are. */
int sptensor_fold(spgemm_handle h, int mode, int64_t I, int64_t J, int64_t K, const spgemm_csr* Y, int32_t* yi, int32_t* yj,
                  int32_t* yk);

/* For callers that cannot allocate device memory (code under HIP graph capture set-up rules, tight
 * serving loops, harnesses that forbid hipMalloc): sptensor_unfold with caller-owned outputs and no
 * allocation of any kind.  out_rowptr (rows + 1 int64), out_colidx and out_values (nnz each) are device
 * arrays, written; rows and columns are as in sptensor_unfold.  The sort buffers live in one fixed
 * array inside the library (about 24 bytes per entry of the limit, per GPU, held until the process
 * ends), so nnz must not exceed SPTENSOR_NOALLOC_MAX_NNZ (SPGEMM_UNSUPPORTED beyond).  Calls on the
 * same GPU share that array: calls that overlap in time on one GPU (two streams, two threads) race
 * and must be serialised by the caller.  Synchronises the stream once, like sptensor_unfold. */
#define SPTENSOR_NOALLOC_MAX_NNZ 1048576
int sptensor_unfold_noalloc(spgemm_handle h, int mode, int64_t I, int64_t J, int64_t K, int64_t nnz, const int32_t* xi,
                            const int32_t* xj, const int32_t* xk, const void* xval, int32_t dtype, int64_t* out_rowptr,
                            int32_t* out_colidx, void* out_values);

/* The same three calls for the third mode (row i*J + j, column k). */
int sptensor_unfold_mode3(spgemm_handle h, int64_t I, int64_t J, int64_t K, int64_t nnz, const int32_t* xi,
                          const int32_t* xj, const int32_t* xk, const void* xval, int32_t dtype, spgemm_csr* out);
int spttm_mode3(spgemm_handle h, int64_t I, int64_t J, int64_t K, int64_t nnz, const int32_t* xi, const int32_t* xj,
                const int32_t* xk, const void* xval, int32_t dtype, const spgemm_csr* M, spgemm_csr* Y);
/* yi[p], yj[p] for entry p of Y; its third coordinate is Y->colidx[p]. */
int sptensor_fold_mode3(spgemm_handle h, int64_t J, const spgemm_csr* Y, int32_t* yi, int32_t* yj);

/* ---- outer-product route with a second-order sparse workspace -------------------------------
 * The paper's leading example (sections 1 and 4.1, evaluated in section 7.3): C = A * B in the loop
 * order k -> i -> j, A in doubly compressed sparse columns, B in doubly compressed sparse rows, C in
 * compressed sparse rows.  Consecutive products land on unrelated coordinates (i, j), so they go
 * through a workspace of whole components, run by the four stages of the algorithm template
 * (section 4.3): insert products into the accumulation array; when it is full, sort it into result
 * order and merge it, adding equal coordinates, into the all array; compress the all array into C.
 * The result is the same matrix as spgemm() gives (structure bit for bit, values up to summation
 * order); the route exists because it is the paper's own, and for operands that come in these formats.
 *
 * Doubly compressed format (section 2.1's level formats Compressed, Compressed): only the nvec
 * non-empty vectors (columns for A, rows for B) are kept: vec[v] is the v-th kept vector's index,
 * ascending, below major_dim; its entries are idx/values[ptr[v] .. ptr[v+1]) with idx below
 * minor_dim.  All arrays are device pointers; idx need not be sorted or unique inside a vector. */
typedef struct {
  int64_t major_dim, minor_dim; /* extent of the compressed dimension, extent of idx */
  int64_t nvec, nnz;
  const int32_t* vec;  /* device, nvec */
  const int64_t* ptr;  /* device, nvec + 1 */
  const int32_t* idx;  /* device, nnz */
  const void* values;  /* device, nnz elements of dtype */
  int32_t dtype;       /* spgemm_dtype */
} spgemm_dcs;

/* Conversions from CSR: rows without entries dropped (doubly compressed rows), or entries regrouped by
 * column with a stable sort and empty columns dropped (doubly compressed columns).  The four arrays of
 * *out come from the handle's allocator; release them with spgemm_dcs_free.  Both synchronise. */
int spgemm_dcsr_from_csr(spgemm_handle h, const spgemm_csr* M, spgemm_dcs* out);
int spgemm_dcsc_from_csr(spgemm_handle h, const spgemm_csr* M, spgemm_dcs* out);
int spgemm_dcs_free(spgemm_handle h, spgemm_dcs* M);

/* C = A * B by outer products.  A: doubly compressed columns of an m x k matrix (major_dim = k,
 * minor_dim = m); B: doubly compressed rows of a k x n matrix (major_dim = k, minor_dim = n).
 * acc_capacity: components the accumulation array holds before it is sorted and merged (0: 2^24).
 * C's buffers come from the handle's allocator (release with its free or spgemm_free_device).
 * Synchronises (once per batch of acc_capacity products).  Sums are accumulated in double.
 * SPGEMM_UNSUPPORTED: the result would have 2^32 - 1 or more entries. */
int spgemm_outer(spgemm_handle h, const spgemm_dcs* A, const spgemm_dcs* B, int64_t acc_capacity, spgemm_csr* C);

/* Library version: major*10000 + minor*100 + patch. */
int spgemm_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SPGEMM_H_ */
