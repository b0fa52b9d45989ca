// C ABI of the SpGEMM library (see include/spgemm.h): argument checks, plan scratch,
// kernel launches.  All device work is in the *_kernels.hpp headers beside this file.
#include "../../include/spgemm.h"

#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "common.hpp"
#include "setup_kernels.hpp"
#include "esc_kernels.hpp"
#include "hash_kernels.hpp"
#include "dense_kernels.hpp"
#include "staged_kernels.hpp"
#include "tensor_kernels.hpp"
#include "outer_kernels.hpp"

using namespace spg;

// a workgroup of the big kernels owns the whole LDS of a compute unit (160 KB)
static_assert(num_dense_lds<double>() <= 160 * 1024 && num_dense_lds<float>() <= 160 * 1024, "numeric dense kernel exceeds LDS");
static_assert(kSymDenseLds <= 160 * 1024, "symbolic dense kernel exceeds LDS");
static_assert(staged_lds<double>() <= 160 * 1024 && staged_lds<float>() <= 160 * 1024, "staged kernel exceeds LDS");

struct TimedLaunch {
  int cls;
  hipEvent_t start, stop;
};

struct spgemm_context {
  hipStream_t stream = nullptr;
  spgemm_allocator alloc{};
  bool has_alloc = false;
  int timing = 0;
  int force = 0;
  int direct_min = kDirectMinDefault;
  int64_t col_list = 1;   // 0 off, 1 automatic size, larger: byte limit
  int block_table = 1;    // 0: never build the block-offset table of B (pieces are bisected)
  int search_ratio = 4;   // searched tiles for rows with at most this many products per entry (0: never)
  int row_block = 0;      // 1: A is a block of rows of a larger matrix (row pointer values are that matrix's positions)
  std::string err = "";
  bool device_ready = false;
  int num_cus = 0;
  std::vector<TimedLaunch> timed;        // launches of the phase in flight
  std::vector<hipEvent_t> event_pool;
};

struct spgemm_plan_s {
  spgemm_context* h = nullptr;
  int64_t m = 0, k = 0, n = 0, nnz_a = 0, nnz_b = 0;
  int dtype = 0;
  void* scratch = nullptr;
  size_t scratch_bytes = 0, scratch2_bytes = 0, scratch3_bytes = 0;
  int* ip = nullptr;
  int* cnt = nullptr;
  int* perm_sym = nullptr;
  int* perm_num = nullptr;
  unsigned char* bin = nullptr;
  long long* partial = nullptr;
  void* scratch2 = nullptr;  // sized after the row classes are known: block offsets of B, tile and run lists
  int* blk_ptr = nullptr;    // rows(B) x blk_ptr_cols offsets, null when not needed or too large
  int blk_ptr_cols = 0;      // column blocks + 1
  TileRec* tiles = nullptr;
  RunRec* runs = nullptr;
  void* scratch3 = nullptr;  // column list of the ranked tiles (optional: sized from what the device has free)
  int32_t* col_list = nullptr;
  unsigned long long col_list_cap = 0;
  Control* ctl = nullptr;
  int64_t scan_blocks = 0;
  bool symbolic_done = false;
  bool numeric_pending = false;   // timed numeric launches not yet folded into stats
  bool numeric_in_flight = false; // numeric kernels were enqueued and the stream has not been waited for since
  spgemm_stats stats{};
};

namespace {

int fail(spgemm_context* h, int code, const std::string& msg) {
  if (h) h->err = msg;
  return code;
}

#define HIP_TRY(h, expr)                                                                 \
  do {                                                                                   \
    hipError_t e_ = (expr);                                                              \
    if (e_ != hipSuccess)                                                                \
      return fail((h), SPGEMM_HIP_ERROR, std::string(#expr) + ": " + hipGetErrorString(e_)); \
  } while (0)

int check_csr(spgemm_context* h, const spgemm_csr* M, const char* name) {
  if (!M) return fail(h, SPGEMM_INVALID_ARG, std::string(name) + " is null");
  if (M->rows < 0 || M->cols < 0 || M->nnz < 0) return fail(h, SPGEMM_INVALID_ARG, std::string(name) + ": negative size");
  if (M->dtype != SPGEMM_F32 && M->dtype != SPGEMM_F64) return fail(h, SPGEMM_INVALID_ARG, std::string(name) + ": unknown dtype");
  if (!M->rowptr) return fail(h, SPGEMM_INVALID_ARG, std::string(name) + ": rowptr is null");
  if (M->nnz > 0 && (!M->colidx || !M->values)) return fail(h, SPGEMM_INVALID_ARG, std::string(name) + ": colidx/values null with nnz > 0");
  if (M->rows >= 0x7fffffffLL || M->cols >= 0x7fffffffLL)
    return fail(h, SPGEMM_UNSUPPORTED, std::string(name) + ": rows and cols must be below 2^31 - 1");
  return SPGEMM_OK;
}

int check_pair(spgemm_context* h, const spgemm_csr* A, const spgemm_csr* B) {
  int rc = check_csr(h, A, "A");
  if (rc) return rc;
  rc = check_csr(h, B, "B");
  if (rc) return rc;
  if (A->cols != B->rows) return fail(h, SPGEMM_DIM_MISMATCH, "A.cols != B.rows");
  if (A->dtype != B->dtype) return fail(h, SPGEMM_DTYPE_MISMATCH, "A and B value types differ");
  return SPGEMM_OK;
}

void* dev_alloc(spgemm_context* h, size_t bytes) {
  if (bytes == 0) bytes = 256;
  if (h->has_alloc) return h->alloc.alloc(h->alloc.ctx, bytes);
  void* p = nullptr;
  if (hipMalloc(&p, bytes) != hipSuccess) return nullptr;
  return p;
}

void dev_free(spgemm_context* h, void* p) {
  if (!p) return;
  if (h->has_alloc) h->alloc.free(h->alloc.ctx, p);
  else (void)hipFree(p);
}

template <typename K>
int allow_lds(spgemm_context* h, K kernel, size_t bytes) {
  HIP_TRY(h, hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
  return SPGEMM_OK;
}

int ensure_device(spgemm_context* h) {
  if (h->device_ready) return SPGEMM_OK;
  int dev = 0;
  HIP_TRY(h, hipGetDevice(&dev));
  hipDeviceProp_t prop;
  HIP_TRY(h, hipGetDeviceProperties(&prop, dev));
  if (prop.warpSize != kWave) return fail(h, SPGEMM_UNSUPPORTED, "device is not wave64");
  h->num_cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  int rc;
  if ((rc = allow_lds(h, k_sym_dense, kSymDenseLds))) return rc;
  if ((rc = allow_lds(h, k_num_dense<float>, num_dense_lds<float>()))) return rc;
  if ((rc = allow_lds(h, k_num_dense<double>, num_dense_lds<double>()))) return rc;
  if ((rc = allow_lds(h, k_num_staged<float>, staged_lds<float>()))) return rc;
  if ((rc = allow_lds(h, k_num_staged<double>, staged_lds<double>()))) return rc;
  h->device_ready = true;
  return SPGEMM_OK;
}

hipEvent_t take_event(spgemm_context* h) {
  if (!h->event_pool.empty()) {
    hipEvent_t e = h->event_pool.back();
    h->event_pool.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  (void)hipEventCreate(&e);
  return e;
}

struct Timer {
  spgemm_context* h;
  int cls;
  TimedLaunch t{};
  Timer(spgemm_context* h_, int cls_) : h(h_), cls(cls_) {
    if (h->timing) {
      t.cls = cls;
      t.start = take_event(h);
      t.stop = take_event(h);
      (void)hipEventRecord(t.start, h->stream);
    }
  }
  ~Timer() {
    if (h->timing) {
      (void)hipEventRecord(t.stop, h->stream);
      h->timed.push_back(t);
    }
  }
};

// After a stream synchronisation: fold event times into the plan's statistics.
void collect_times(spgemm_context* h, spgemm_stats* st) {
  for (auto& t : h->timed) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, t.start, t.stop) == hipSuccess) {
      st->kernel_ms[t.cls] += ms;
      st->kernel_launches[t.cls] += 1;
    }
    h->event_pool.push_back(t.start);
    h->event_pool.push_back(t.stop);
  }
  h->timed.clear();
}

// Forget the launches timed so far (their events go back to the pool).
void drop_timed(spgemm_context* h) {
  for (auto& t : h->timed) { h->event_pool.push_back(t.start); h->event_pool.push_back(t.stop); }
  h->timed.clear();
}

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

inline unsigned grid_for(int64_t items, int64_t per_block, int64_t cap) {
  int64_t g = ceil_div(items > 0 ? items : 1, per_block);
  if (g > cap) g = cap;
  if (g < 1) g = 1;
  return (unsigned)g;
}

size_t align_up(size_t v) { return (v + 255) & ~(size_t)255; }

// Symbolic phase, first part: count, check, bin.  Ends with the control block on the host
// (one synchronisation): the second part sizes its lists and launches from the bin populations.
int run_setup(spgemm_context* h, spgemm_plan_s* p, const spgemm_csr* A, const spgemm_csr* B, Control* host) {
  hipStream_t s = h->stream;
  const int64_t m = p->m;
  {
    Timer t(h, SPGEMM_K_COUNT);
    hipLaunchKernelGGL(k_init_control, dim3(1), dim3(64), 0, s, p->ctl);
    hipLaunchKernelGGL(k_validate_b, dim3(grid_for(B->nnz > B->rows ? B->nnz : B->rows, 256 * 8, (int64_t)h->num_cus * 16)), dim3(256), 0, s,
                       B->rows, B->cols, B->nnz, B->rowptr, B->colidx, p->ctl);
    if (m > 0)
      hipLaunchKernelGGL(k_count_rows, dim3(grid_for(m, 256, (int64_t)h->num_cus * 8)), dim3(kCountThreads), 0, s, m, A->nnz, B->rows, A->rowptr, A->colidx,
                         B->rowptr, p->ip, p->bin, p->cnt, p->ctl, h->force, h->row_block);
  }
  {
    Timer t(h, SPGEMM_K_BIN);
    hipLaunchKernelGGL(k_bin_offsets, dim3(1), dim3(64), 0, s, p->ctl, 0);
    if (m > 0)
      hipLaunchKernelGGL(k_bin_scatter, dim3((unsigned)ceil_div(m, kScatterThreads)), dim3(kScatterThreads), 0, s, m, p->bin, p->perm_sym, p->ctl, 0);
  }
  HIP_TRY(h, hipGetLastError());
  HIP_TRY(h, hipMemcpyAsync(host, p->ctl, sizeof(Control), hipMemcpyDeviceToHost, s));
  HIP_TRY(h, hipStreamSynchronize(s));
  return SPGEMM_OK;
}

// Sizes and allocates what the dense kernels need beyond the per-row arrays: the tile and run
// lists (from an upper bound of the number of tiles) and the table of block offsets of B.
int alloc_dense_lists(spgemm_context* h, spgemm_plan_s* p, const spgemm_csr* B, const Control& host, unsigned* tile_cap,
                      unsigned* run_cap) {
  *tile_cap = 0; *run_cap = 0;
  double rows_d = 0, ip_d = 0;
  for (int b = 4; b <= 6; ++b) { rows_d += host.hist[0][b]; ip_d += (double)host.bin_ip[0][b]; }
  if (rows_d == 0) return SPGEMM_OK;
  const double n = (double)B->cols;
  const double blocks = (double)ceil_div(B->cols, kBlkCols);
  const double spans = (double)ceil_div(B->cols, (int64_t)kSymFlagWords * 32);
  // direct tiles hold at least direct_min entries each and there is at most one per block;
  // of two neighbouring ranked tiles at least one pair exceeds the tile budget together
  double direct = rows_d * blocks;
  if (ip_d / h->direct_min < direct) direct = ip_d / h->direct_min;
  const double entries = ip_d < rows_d * n ? ip_d : rows_d * n;
  const double weight = rows_d * blocks * kRankBlkBytes + (double)kRankEntryBytes * entries;
  // (+ a slab per workgroup of the symbolic kernel: what a workgroup has drawn and not used)
  const double wgs = (double)grid_for((int64_t)rows_d, 1, h->num_cus) + 1.0;
  const double tiles = 2.0 * direct + 2.0 * weight / kTileBudget + 4.0 * rows_d * spans + 16.0 + wgs * kTileSlab;
  const double runs = (tiles - wgs * kTileSlab) / kRunTiles + rows_d * spans + 16.0 + wgs * kRunSlab;
  if (tiles > 4.0e9) return fail(h, SPGEMM_UNSUPPORTED, "tile list of the dense workspace would exceed 2^32 records");
  *tile_cap = (unsigned)tiles;
  *run_cap = (unsigned)runs;
  p->blk_ptr_cols = (int)blocks + 1;
  const size_t bp_bytes = (size_t)B->rows * (size_t)p->blk_ptr_cols * 4;
  const bool with_bp = h->block_table && host.b_sorted && B->nnz > 0 && bp_bytes <= ((size_t)1 << 30);
  size_t off = 0;
  const size_t o_tiles = off; off = align_up(off + (size_t)*tile_cap * sizeof(TileRec));
  const size_t o_runs = off; off = align_up(off + (size_t)*run_cap * sizeof(RunRec));
  const size_t o_bp = off; if (with_bp) off = align_up(off + bp_bytes);
  p->scratch2 = dev_alloc(h, off);
  p->scratch2_bytes = off;
  if (!p->scratch2) return fail(h, SPGEMM_ALLOC_FAILED, "device allocation of the dense workspace lists failed");
  unsigned char* base = static_cast<unsigned char*>(p->scratch2);
  p->tiles = reinterpret_cast<TileRec*>(base + o_tiles);
  p->runs = reinterpret_cast<RunRec*>(base + o_runs);
  p->blk_ptr = with_bp ? reinterpret_cast<int*>(base + o_bp) : nullptr;
  // Column list: the dense symbolic kernel leaves the columns of its ranked tiles there, which saves
  // the numeric kernel one pass over those tiles' products.  At most `entries` are needed; take no
  // more than a third of what the device has free, and do without if the allocation fails.
  size_t free_b = 0, total_b = 0;
  if (h->col_list && hipMemGetInfo(&free_b, &total_b) == hipSuccess) {
    double want = (entries + 4.0 * rows_d * spans) * 4.0;   // (every row's share is rounded up to 16 bytes)
    if (want > (double)free_b / 3.0) want = (double)free_b / 3.0;
    if (h->col_list > 1 && want > (double)h->col_list) want = (double)h->col_list;
    const size_t bytes = ((size_t)want) & ~(size_t)255;
    if (bytes >= 4096) {
      p->scratch3 = dev_alloc(h, bytes);
      if (p->scratch3) {
        p->scratch3_bytes = bytes;
        p->col_list = static_cast<int32_t*>(p->scratch3);
        p->col_list_cap = bytes / 4;
      }
    }
  }
  return SPGEMM_OK;
}

__global__ void k_set_caps(Control* ctl, unsigned tile_cap, unsigned run_cap, unsigned long long list_cap) {
  if (threadIdx.x == 0) { ctl->tile_cap = tile_cap; ctl->run_cap = run_cap; ctl->list_cap = list_cap; }
}

template <typename T>
int run_symbolic(spgemm_context* h, spgemm_plan_s* p, const spgemm_csr* A, const spgemm_csr* B, int64_t* c_rowptr,
                 const Control& host) {
  hipStream_t s = h->stream;
  const int64_t m = p->m;
  const int64_t cap_small = (int64_t)h->num_cus * 32;
  // sorted-list keys can carry their list position when every column, shifted by the list's log2 capacity, stays below the padding key
  const int pack32 = B->cols <= (int64_t(1) << 25) ? 1 : 0, pack128 = B->cols <= (int64_t(1) << 23) ? 1 : 0;
  const size_t lds_hash_small = hash_lds_bytes<64, 10, false>();
  const size_t lds_hash_large = hash_lds_bytes<256, 12, false>();
  const unsigned* hist = host.hist[0];
  const int64_t rows_dense = (int64_t)hist[4] + hist[5] + hist[6];
  // rows of at most this many products never reach the dense numeric kernel (0: class unavailable)
  // (the staged class is taken only on request: short rows whose columns are in the plan's list
  // become searched tiles of the dense kernel, which costs them one global round trip less)
  const int staged = (h->force == 4 && ceil_div(B->cols, kStWinCols) <= kStMaxWindows) ? staged_cap<T>() : 0;
  unsigned tile_cap = 0, run_cap = 0;
  int rc = alloc_dense_lists(h, p, B, host, &tile_cap, &run_cap);
  if (rc) return rc;
  if (rows_dense > 0) {
    hipLaunchKernelGGL(k_set_caps, dim3(1), dim3(64), 0, s, p->ctl, tile_cap, run_cap, p->col_list_cap);
    if (p->blk_ptr) {
      Timer t(h, SPGEMM_K_BLOCK_PTR);
      const int64_t items = B->rows * (int64_t)p->blk_ptr_cols;
      hipLaunchKernelGGL(k_block_ptrs, dim3(grid_for(items, 256, (int64_t)h->num_cus * 64)), dim3(256), 0, s, B->rows,
                         p->blk_ptr_cols, B->rowptr, B->colidx, p->ctl, p->blk_ptr);
    }
  }
  if (m > 0) {
    {
      Timer t(h, SPGEMM_K_SYM_ESC);
      if (hist[0])
        hipLaunchKernelGGL((k_esc<16, 32, T, false>), dim3(grid_for(hist[0], 16, cap_small)), dim3(256), 0, s, p->perm_sym, p->ctl, 0, 0,
                           A->rowptr, A->colidx, (const T*)nullptr, B->rowptr, B->colidx, (const T*)nullptr, p->cnt,
                           (const int64_t*)nullptr, (int32_t*)nullptr, (T*)nullptr, pack32, B->nnz);
      if (hist[1])
        hipLaunchKernelGGL((k_esc<64, 128, T, false>), dim3(grid_for(hist[1], 4, cap_small)), dim3(256), 0, s, p->perm_sym, p->ctl, 0, 1,
                           A->rowptr, A->colidx, (const T*)nullptr, B->rowptr, B->colidx, (const T*)nullptr, p->cnt,
                           (const int64_t*)nullptr, (int32_t*)nullptr, (T*)nullptr, pack128, B->nnz);
    }
    {
      Timer t(h, SPGEMM_K_SYM_HASH);
      if (hist[2])
        hipLaunchKernelGGL((k_hash<64, 10, T, false>), dim3(grid_for(hist[2], 4, cap_small)), dim3(256), lds_hash_small, s,
                           p->perm_sym, p->ctl, 0, 2, p->ip, A->rowptr, A->colidx, (const T*)nullptr, B->rowptr, B->colidx,
                           (const T*)nullptr, p->cnt, (const int64_t*)nullptr, (int32_t*)nullptr, (T*)nullptr, B->cols);
      if (hist[3])
        hipLaunchKernelGGL((k_hash<256, 12, T, false>), dim3(grid_for(hist[3], 1, (int64_t)h->num_cus * 8)), dim3(256),
                           lds_hash_large, s, p->perm_sym, p->ctl, 0, 3, p->ip, A->rowptr, A->colidx,
                           (const T*)nullptr, B->rowptr, B->colidx, (const T*)nullptr, p->cnt, (const int64_t*)nullptr,
                           (int32_t*)nullptr, (T*)nullptr, B->cols);
    }
    if (rows_dense > 0) {
      Timer t(h, SPGEMM_K_SYM_DENSE);
      hipLaunchKernelGGL(k_sym_dense, dim3(grid_for(rows_dense, 1, h->num_cus)), dim3(kDenseThreads), kSymDenseLds, s, p->perm_sym,
                         p->ctl, A->rowptr, A->colidx, B->rowptr, B->colidx, B->cols, p->ip, p->cnt, p->tiles, p->runs, p->col_list, h->direct_min,
                         staged, h->search_ratio, p->blk_ptr, p->blk_ptr_cols);
    }
    {
      Timer t(h, SPGEMM_K_BIN);
      hipLaunchKernelGGL(k_classify_numeric, dim3(grid_for(m, 256, (int64_t)h->num_cus * 8)), dim3(256), 0, s, m, p->ip, p->cnt,
                         p->bin, p->ctl, h->force, staged);
      hipLaunchKernelGGL(k_bin_offsets, dim3(1), dim3(64), 0, s, p->ctl, 1);
      hipLaunchKernelGGL(k_bin_scatter, dim3((unsigned)ceil_div(m, kScatterThreads)), dim3(kScatterThreads), 0, s, m, p->bin, p->perm_num, p->ctl, 1);
    }
  }
  {
    Timer t(h, SPGEMM_K_SCAN);
    if (p->scan_blocks > 0)
      hipLaunchKernelGGL(k_scan_partials, dim3((unsigned)p->scan_blocks), dim3(kScanThreads), 0, s, m, p->cnt, p->partial);
    hipLaunchKernelGGL(k_scan_blocks, dim3(1), dim3(kScanThreads), 0, s, p->scan_blocks, p->partial, m, c_rowptr, p->ctl);
    if (p->scan_blocks > 0)
      hipLaunchKernelGGL(k_scan_final, dim3((unsigned)p->scan_blocks), dim3(kScanThreads), 0, s, m, p->cnt, p->partial, c_rowptr);
  }
  HIP_TRY(h, hipGetLastError());
  return SPGEMM_OK;
}

__global__ void k_reset_numeric_work(Control* ctl) {
  if (threadIdx.x == 0) { ctl->work[1] = 0; ctl->work[2] = 0; }
  SPG_CLK(if (threadIdx.x < kClkSlots) ctl->clk[1][threadIdx.x] = 0;)
}

template <typename T>
int run_numeric(spgemm_context* h, spgemm_plan_s* p, const spgemm_csr* A, const spgemm_csr* B, const int64_t* c_rp,
                int32_t* c_col, void* c_val_v) {
  hipStream_t s = h->stream;
  const int64_t m = p->m;
  if (m == 0) return SPGEMM_OK;
  const int64_t cap_small = (int64_t)h->num_cus * 32;
  // sorted-list keys can carry their list position when every column, shifted by the list's log2 capacity, stays below the padding key
  const int pack32 = B->cols <= (int64_t(1) << 25) ? 1 : 0, pack128 = B->cols <= (int64_t(1) << 23) ? 1 : 0;
  const T* a_val = static_cast<const T*>(A->values);
  const T* b_val = static_cast<const T*>(B->values);
  T* c_val = static_cast<T*>(c_val_v);
  const size_t lds_hash_small = hash_lds_bytes<64, 8, true>();
  const size_t lds_hash_large = hash_lds_bytes<256, 11, true>();
  const int64_t* hist = p->stats.num_bin_rows;
  hipLaunchKernelGGL(k_reset_numeric_work, dim3(1), dim3(64), 0, s, p->ctl);
  {
    Timer t(h, SPGEMM_K_NUM_ESC);
    if (hist[0])
      hipLaunchKernelGGL((k_esc<16, 32, T, true>), dim3(grid_for(hist[0], 16, cap_small)), dim3(256), 0, s, p->perm_num, p->ctl, 1, 0,
                         A->rowptr, A->colidx, a_val, B->rowptr, B->colidx, b_val, (int*)nullptr, c_rp, c_col, c_val, pack32, B->nnz);
    if (hist[1])
      hipLaunchKernelGGL((k_esc<64, 128, T, true>), dim3(grid_for(hist[1], 4, cap_small)), dim3(256), 0, s, p->perm_num, p->ctl, 1, 1,
                         A->rowptr, A->colidx, a_val, B->rowptr, B->colidx, b_val, (int*)nullptr, c_rp, c_col, c_val, pack128, B->nnz);
  }
  {
    Timer t(h, SPGEMM_K_NUM_HASH);
    if (hist[2])
      hipLaunchKernelGGL((k_hash<64, 8, T, true>), dim3(grid_for(hist[2], 4, cap_small)), dim3(256), lds_hash_small, s,
                         p->perm_num, p->ctl, 1, 2, p->ip, A->rowptr, A->colidx, a_val, B->rowptr, B->colidx, b_val, (int*)nullptr,
                         c_rp, c_col, c_val, B->cols);
    if (hist[3])
      hipLaunchKernelGGL((k_hash<256, 11, T, true>), dim3(grid_for(hist[3], 1, (int64_t)h->num_cus * 8)), dim3(256),
                         lds_hash_large, s, p->perm_num, p->ctl, 1, 3, p->ip, A->rowptr, A->colidx, a_val, B->rowptr,
                         B->colidx, b_val, (int*)nullptr, c_rp, c_col, c_val, B->cols);
  }
  if (hist[4]) {
    Timer t(h, SPGEMM_K_NUM_STAGED);
    hipLaunchKernelGGL(k_num_staged<T>, dim3(grid_for(hist[4], 1, h->num_cus)), dim3(kDenseThreads), staged_lds<T>(), s, p->perm_num,
                       p->ctl, A->rowptr, A->colidx, a_val, B->rowptr, B->colidx, b_val, B->cols, c_rp, c_col, c_val);
  }
  const int64_t rows_dense = hist[5] + hist[6];
  if (rows_dense > 0) {
    Timer t(h, SPGEMM_K_NUM_DENSE);
    hipLaunchKernelGGL(k_num_dense<T>, dim3(grid_for(rows_dense, 1, h->num_cus)), dim3(kDenseThreads), num_dense_lds<T>(), s, p->ctl,
                       p->bin, p->tiles, p->runs, A->colidx, a_val, B->rowptr, B->colidx, b_val, B->cols, p->blk_ptr,
                       p->blk_ptr_cols, p->col_list, c_rp, c_col, c_val);
  }
  HIP_TRY(h, hipGetLastError());
  return SPGEMM_OK;
}

}  // namespace

extern "C" {

int spgemm_version(void) { return 100; }

int spgemm_create(spgemm_handle* out, void* hip_stream, const spgemm_allocator* alloc) {
  if (!out) return SPGEMM_INVALID_ARG;
  if (alloc && (!alloc->alloc || !alloc->free)) return SPGEMM_INVALID_ARG;
  spgemm_context* h = new (std::nothrow) spgemm_context();
  if (!h) return SPGEMM_ALLOC_FAILED;
  h->stream = static_cast<hipStream_t>(hip_stream);
  if (alloc) {
    h->alloc = *alloc;
    h->has_alloc = true;
  }
  *out = h;
  return SPGEMM_OK;
}

int spgemm_destroy(spgemm_handle h) {
  if (!h) return SPGEMM_INVALID_ARG;
  for (auto e : h->event_pool) (void)hipEventDestroy(e);
  for (auto& t : h->timed) { (void)hipEventDestroy(t.start); (void)hipEventDestroy(t.stop); }
  delete h;
  return SPGEMM_OK;
}

int spgemm_set_option(spgemm_handle h, int option, int64_t value) {
  if (!h) return SPGEMM_INVALID_ARG;
  switch (option) {
    case SPGEMM_OPT_TIMING:
      if (value != 0 && value != 1) return fail(h, SPGEMM_INVALID_ARG, "timing option takes 0 or 1");
      h->timing = (int)value;
      return SPGEMM_OK;
    case SPGEMM_OPT_FORCE_WORKSPACE:
      if (value < 0 || value > 4) return fail(h, SPGEMM_INVALID_ARG, "workspace option takes 0..4");
      h->force = (int)value;
      return SPGEMM_OK;
    case SPGEMM_OPT_DIRECT_MIN:
      // a direct block keeps its 256 flag words in the list space of its entries
      if (value < kBlkWords || value > 0x3fffffff) return fail(h, SPGEMM_INVALID_ARG, "direct-tile threshold takes 256..2^30-1");
      h->direct_min = (int)value;
      return SPGEMM_OK;
    case SPGEMM_OPT_SEARCH_RATIO:
      if (value < 0 || value > 1000000) return fail(h, SPGEMM_INVALID_ARG, "search-ratio option takes 0..1000000");
      h->search_ratio = (int)value;
      return SPGEMM_OK;
    case SPGEMM_OPT_BLOCK_TABLE:
      if (value != 0 && value != 1) return fail(h, SPGEMM_INVALID_ARG, "block-table option takes 0 or 1");
      h->block_table = (int)value;
      return SPGEMM_OK;
    case SPGEMM_OPT_COLUMN_LIST:
      if (value < 0 || (value > 1 && value < 4096)) return fail(h, SPGEMM_INVALID_ARG, "column-list option takes 0, 1 or a byte limit of 4096 or more");
      h->col_list = value;
      return SPGEMM_OK;
    default:
      return fail(h, SPGEMM_INVALID_ARG, "unknown option");
  }
}

const char* spgemm_last_error(spgemm_handle h) { return h ? h->err.c_str() : "null handle"; }

int spgemm_plan_destroy(spgemm_plan p) {
  if (!p) return SPGEMM_INVALID_ARG;
  // the numeric kernels read the plan's scratch: they must have finished before it is released
  if (p->numeric_in_flight) (void)hipStreamSynchronize(p->h->stream);
  dev_free(p->h, p->scratch);
  dev_free(p->h, p->scratch2);
  dev_free(p->h, p->scratch3);
  delete p;
  return SPGEMM_OK;
}

int spgemm_get_stats(spgemm_plan p, spgemm_stats* out) {
  if (!p || !out) return SPGEMM_INVALID_ARG;
  if (!p->symbolic_done) return fail(p->h, SPGEMM_BAD_STATE, "plan has no symbolic result");
  if (p->numeric_pending) {
    spgemm_context* h = p->h;
    if (!h->timed.empty()) HIP_TRY(h, hipEventSynchronize(h->timed.back().stop));
    p->numeric_in_flight = false;
    for (int c = SPGEMM_K_NUM_ESC; c <= SPGEMM_K_NUM_STAGED; ++c) { p->stats.kernel_ms[c] = 0; p->stats.kernel_launches[c] = 0; }
    collect_times(h, &p->stats);
    p->numeric_pending = false;
  }
  *out = p->stats;
  return SPGEMM_OK;
}

int spgemm_symbolic(spgemm_handle h, const spgemm_csr* A, const spgemm_csr* B, int64_t* c_rowptr, int64_t* nnz_c,
                    spgemm_plan* plan) {
  if (!h) return SPGEMM_INVALID_ARG;
  int rc = check_pair(h, A, B);
  if (rc) return rc;
  if (!c_rowptr || !nnz_c || !plan) return fail(h, SPGEMM_INVALID_ARG, "c_rowptr, nnz_c and plan must not be null");
  *plan = nullptr;
  if ((rc = ensure_device(h))) return rc;
  drop_timed(h);   // (timed launches of an earlier plan that nobody asked about)

  spgemm_plan_s* p = new (std::nothrow) spgemm_plan_s();
  if (!p) return fail(h, SPGEMM_ALLOC_FAILED, "host allocation failed");
  p->h = h;
  p->m = A->rows; p->k = A->cols; p->n = B->cols; p->nnz_a = A->nnz; p->nnz_b = B->nnz; p->dtype = A->dtype;
  const int64_t m = p->m;
  p->scan_blocks = m > 0 ? ceil_div(m, kScanTile) : 0;
  size_t off = 0;
  const size_t o_ctl = off; off = align_up(off + sizeof(Control));
  const size_t o_ip = off; off = align_up(off + (size_t)m * 4);
  const size_t o_cnt = off; off = align_up(off + (size_t)m * 4);
  const size_t o_ps = off; off = align_up(off + (size_t)m * 4);
  const size_t o_pn = off; off = align_up(off + (size_t)m * 4);
  const size_t o_bin = off; off = align_up(off + (size_t)m);
  const size_t o_part = off; off = align_up(off + (size_t)(p->scan_blocks + 1) * 8);
  p->scratch = dev_alloc(h, off);
  p->scratch_bytes = off;
  if (!p->scratch) {
    delete p;
    return fail(h, SPGEMM_ALLOC_FAILED, "device allocation of plan scratch failed");
  }
  unsigned char* base = static_cast<unsigned char*>(p->scratch);
  p->ctl = reinterpret_cast<Control*>(base + o_ctl);
  p->ip = reinterpret_cast<int*>(base + o_ip);
  p->cnt = reinterpret_cast<int*>(base + o_cnt);
  p->perm_sym = reinterpret_cast<int*>(base + o_ps);
  p->perm_num = reinterpret_cast<int*>(base + o_pn);
  p->bin = base + o_bin;
  p->partial = reinterpret_cast<long long*>(base + o_part);

  Control host{};
  rc = run_setup(h, p, A, B, &host);
  if (rc == SPGEMM_OK && !host.error)
    rc = (A->dtype == SPGEMM_F32) ? run_symbolic<float>(h, p, A, B, c_rowptr, host) : run_symbolic<double>(h, p, A, B, c_rowptr, host);
  if (rc == SPGEMM_OK && !host.error) {
    hipError_t e = hipMemcpyAsync(&host, p->ctl, sizeof(Control), hipMemcpyDeviceToHost, h->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(h->stream);
    if (e != hipSuccess) rc = fail(h, SPGEMM_HIP_ERROR, std::string("symbolic phase: ") + hipGetErrorString(e));
  }
  if (rc != SPGEMM_OK) {
    (void)hipStreamSynchronize(h->stream);
    drop_timed(h);
    spgemm_plan_destroy(p);
    return rc;
  }
  std::memset(&p->stats, 0, sizeof(p->stats));
  collect_times(h, &p->stats);
  if (host.error == 2 || host.error == 3) {
    spgemm_plan_destroy(p);
    return host.error == 2 ? fail(h, SPGEMM_UNSUPPORTED, "unsorted B with a row of 2^21 or more entries")
                           : fail(h, SPGEMM_HIP_ERROR, "internal: tile list overflow in the dense symbolic kernel");
  }
  if (host.error) {
    spgemm_plan_destroy(p);
    return fail(h, SPGEMM_INVALID_INPUT, "device-side input check failed (column out of range or rowptr not monotone)");
  }
  p->stats.ip_total = (int64_t)host.ip_total;
  p->stats.nnz_c = host.nnz_c;
  for (int b = 0; b < kNumBins; ++b) {
    p->stats.sym_bin_rows[b] = host.hist[0][b];
    p->stats.num_bin_rows[b] = host.hist[1][b];
    p->stats.sym_bin_ip[b] = (int64_t)host.bin_ip[0][b];
    p->stats.num_bin_ip[b] = (int64_t)host.bin_ip[1][b];
    p->stats.num_bin_nnz[b] = (int64_t)host.bin_nnz[b];
  }
  p->stats.dense_tiles = host.tiles_used;
  p->stats.dense_direct_tiles = host.direct_tiles;
  p->stats.dense_runs = host.runs_used;
  p->stats.dense_search_tiles = host.search_tiles;
  p->stats.plan_bytes = (int64_t)(p->scratch_bytes + p->scratch2_bytes + p->scratch3_bytes);
  p->stats.plan_list_bytes = (int64_t)p->scratch3_bytes;
  p->stats.plan_list_used = (int64_t)((host.list_cursor < host.list_cap ? host.list_cursor : host.list_cap) * 4ULL);
  p->symbolic_done = true;
  *nnz_c = host.nnz_c;
  *plan = p;
  return SPGEMM_OK;
}

int spgemm_numeric(spgemm_handle h, spgemm_plan p, const spgemm_csr* A, const spgemm_csr* B, const int64_t* c_rowptr,
                   int32_t* c_colidx, void* c_values) {
  if (!h) return SPGEMM_INVALID_ARG;
  if (!p) return fail(h, SPGEMM_INVALID_ARG, "plan is null");
  int rc = check_pair(h, A, B);
  if (rc) return rc;
  if (p->h != h || !p->symbolic_done) return fail(h, SPGEMM_BAD_STATE, "plan does not belong to this handle or has no symbolic result");
  if (A->rows != p->m || A->cols != p->k || B->cols != p->n || A->nnz != p->nnz_a || B->nnz != p->nnz_b)
    return fail(h, SPGEMM_DIM_MISMATCH, "operands differ from the ones the plan was built for");
  if (A->dtype != p->dtype) return fail(h, SPGEMM_DTYPE_MISMATCH, "value type differs from the plan's");
  if (!c_rowptr) return fail(h, SPGEMM_INVALID_ARG, "c_rowptr is null");
  if (p->stats.nnz_c > 0 && (!c_colidx || !c_values)) return fail(h, SPGEMM_INVALID_ARG, "c_colidx/c_values null with nnz_c > 0");
  if (p->stats.nnz_c == 0) return SPGEMM_OK;
  rc = (A->dtype == SPGEMM_F32) ? run_numeric<float>(h, p, A, B, c_rowptr, c_colidx, c_values)
                                : run_numeric<double>(h, p, A, B, c_rowptr, c_colidx, c_values);
  if (rc != SPGEMM_OK) return rc;
  p->numeric_pending = h->timing != 0;
  p->numeric_in_flight = true;
  return SPGEMM_OK;
}

#ifdef SPG_PHASE_CLOCKS
// Profiling builds only: shader clocks per phase of the dense kernels (2 x 32 values, host), summed
// over workgroups, of the plan's last symbolic and numeric runs.  Waits for the stream.
int spgemm_debug_phase_clocks(spgemm_plan p, unsigned long long* out) {
  if (!p || !out) return SPGEMM_INVALID_ARG;
  spgemm_context* h = p->h;
  HIP_TRY(h, hipStreamSynchronize(h->stream));
  HIP_TRY(h, hipMemcpy(out, reinterpret_cast<unsigned char*>(p->ctl) + offsetof(Control, clk), sizeof(unsigned long long) * 2 * kClkSlots,
                       hipMemcpyDeviceToHost));
  return SPGEMM_OK;
}
#endif

int spgemm_free_device(spgemm_handle h, void* ptr) {
  if (!h) return SPGEMM_INVALID_ARG;
  dev_free(h, ptr);
  return SPGEMM_OK;
}

int spgemm(spgemm_handle h, const spgemm_csr* A, const spgemm_csr* B, spgemm_csr* C) {
  if (!h) return SPGEMM_INVALID_ARG;
  int rc = check_pair(h, A, B);
  if (rc) return rc;
  if (!C) return fail(h, SPGEMM_INVALID_ARG, "C is null");
  std::memset(C, 0, sizeof(*C));
  int64_t* rp = static_cast<int64_t*>(dev_alloc(h, (size_t)(A->rows + 1) * sizeof(int64_t)));
  if (!rp) return fail(h, SPGEMM_ALLOC_FAILED, "allocation of C.rowptr failed");
  spgemm_plan plan = nullptr;
  int64_t nnz = 0;
  rc = spgemm_symbolic(h, A, B, rp, &nnz, &plan);
  if (rc != SPGEMM_OK) {
    dev_free(h, rp);
    return rc;
  }
  const size_t vsz = A->dtype == SPGEMM_F32 ? 4 : 8;
  int32_t* col = nullptr;
  void* val = nullptr;
  if (nnz > 0) {
    col = static_cast<int32_t*>(dev_alloc(h, (size_t)nnz * 4));
    val = dev_alloc(h, (size_t)nnz * vsz);
    if ((!col || !val) && plan->scratch3 && h->col_list) {
      // the plan's optional structure list may be what stands in the way: plan again without it
      dev_free(h, col); dev_free(h, val);
      spgemm_plan_destroy(plan);
      plan = nullptr;
      const int64_t keep = h->col_list;
      h->col_list = 0;
      rc = spgemm_symbolic(h, A, B, rp, &nnz, &plan);
      h->col_list = keep;
      if (rc != SPGEMM_OK) { dev_free(h, rp); return rc; }
      col = static_cast<int32_t*>(dev_alloc(h, (size_t)nnz * 4));
      val = dev_alloc(h, (size_t)nnz * vsz);
    }
    if (!col || !val) {
      dev_free(h, col); dev_free(h, val); dev_free(h, rp);
      spgemm_plan_destroy(plan);
      return fail(h, SPGEMM_ALLOC_FAILED, "allocation of C.colidx/C.values failed");
    }
    rc = spgemm_numeric(h, plan, A, B, rp, col, val);
  }
  // the plan's scratch may be released only after the numeric kernels that read it finish
  if (hipStreamSynchronize(h->stream) != hipSuccess && rc == SPGEMM_OK) rc = fail(h, SPGEMM_HIP_ERROR, "numeric phase failed");
  spgemm_plan_destroy(plan);
  if (rc != SPGEMM_OK) {
    dev_free(h, col); dev_free(h, val); dev_free(h, rp);
    return rc;
  }
  C->rows = A->rows; C->cols = B->cols; C->nnz = nnz; C->dtype = A->dtype;
  C->rowptr = rp; C->colidx = col; C->values = val;
  return SPGEMM_OK;
}


// ---- sparse tensor entry points ------------------------------------------------------------

namespace {

// The unfolding over `mode`: which coordinate arrays and extents play row-major, row-minor, column.
struct ModeView {
  const int32_t *xa, *xb, *xc;
  int64_t A, B, C;
};

bool mode_view(int mode, int64_t I, int64_t J, int64_t K, const int32_t* xi, const int32_t* xj, const int32_t* xk, ModeView* v) {
  switch (mode) {
    case 1: *v = ModeView{xj, xk, xi, J, K, I}; return true;
    case 2: *v = ModeView{xi, xk, xj, I, K, J}; return true;
    case 3: *v = ModeView{xi, xj, xk, I, J, K}; return true;
    default: return false;
  }
}

int check_tensor(spgemm_context* h, int mode, int64_t I, int64_t J, int64_t K, int64_t nnz, const int32_t* xi, const int32_t* xj,
                 const int32_t* xk, const void* xval, int32_t dtype, ModeView* v) {
  if (!mode_view(mode, I, J, K, xi, xj, xk, v)) return fail(h, SPGEMM_INVALID_ARG, "mode must be 1, 2 or 3");
  if (I < 0 || J < 0 || K < 0 || nnz < 0) return fail(h, SPGEMM_INVALID_ARG, "negative size");
  if (dtype != SPGEMM_F32 && dtype != SPGEMM_F64) return fail(h, SPGEMM_INVALID_ARG, "unknown dtype");
  if (nnz > 0 && (!xi || !xj || !xk || !xval)) return fail(h, SPGEMM_INVALID_ARG, "coordinate or value array null with nnz > 0");
  if (v->C >= 0x7fffffffLL || (v->B > 0 && v->A > 0x7ffffffeLL / v->B) || nnz >= 0xffffffffLL)
    return fail(h, SPGEMM_UNSUPPORTED, "the folded row extent and the column extent must be below 2^31 - 1, nnz below 2^32 - 1");
  return SPGEMM_OK;
}

// Temporary memory of one unfolding: two key buffers, two index buffers, the tile histograms, one flag.
struct UnfoldTmp {
  size_t o_k0, o_k1, o_i0, o_i1, o_h, o_bad, bytes;
  int64_t ntiles;
};

UnfoldTmp unfold_tmp_layout(int64_t nnz) {
  UnfoldTmp t{};
  t.ntiles = ceil_div(nnz > 0 ? nnz : 1, kSortTile);
  size_t off = 0;
  t.o_k0 = off; off = align_up(off + (size_t)nnz * 8);
  t.o_k1 = off; off = align_up(off + (size_t)nnz * 8);
  t.o_i0 = off; off = align_up(off + (size_t)nnz * 4);
  t.o_i1 = off; off = align_up(off + (size_t)nnz * 4);
  t.o_h = off; off = align_up(off + (size_t)t.ntiles * 256 * 4);
  t.o_bad = off; off = align_up(off + 4);
  t.bytes = off;
  return t;
}

__global__ void k_clear_int(int* p) {
  if (threadIdx.x == 0 && blockIdx.x == 0) *p = 0;
}

int bits_of(int64_t n) {   // bits that hold 0 .. n-1
  int b = 0;
  while (n > 1 && (1LL << b) < n) ++b;
  return b;
}

// Stable least-significant-digit radix sort of (key, index) pairs, 8 bits a pass, over the low bits_lo bits
// and the bits_hi bits from bit 32 up.  Returns which of the two buffers holds the result.
int sort_pairs(spgemm_context* h, int64_t n, int64_t ntiles, int bits_lo, int bits_hi, unsigned long long* const keys[2],
               unsigned* const idx[2], unsigned* hist) {
  hipStream_t s = h->stream;
  int cur = 0;
  const unsigned gt = (unsigned)ceil_div(ntiles, kSortWgWaves);
  for (int part = 0; part < 2; ++part) {
    const int base = part == 0 ? 0 : 32, nbits = part == 0 ? bits_lo : bits_hi;
    for (int shift = base; shift < base + nbits; shift += 8) {
      hipLaunchKernelGGL(k_radix_hist, dim3(gt), dim3(256), 0, s, n, ntiles, shift, keys[cur], hist);
      hipLaunchKernelGGL(k_scan_u32, dim3(1), dim3(1024), 0, s, ntiles * 256, hist);
      hipLaunchKernelGGL(k_radix_scatter, dim3(gt), dim3(256), 0, s, n, ntiles, shift, keys[cur], idx[cur], hist, keys[1 - cur], idx[1 - cur]);
      cur = 1 - cur;
    }
  }
  return cur;
}

// Keys, stable radix sort, compress, row pointer; everything it touches is given by the caller.
// Ends with one stream synchronisation (the out-of-range flag comes to the host).
int unfold_run(spgemm_context* h, const ModeView& v, int64_t nnz, const void* xval, int32_t dtype, unsigned char* tmp, const UnfoldTmp& lay,
               int64_t* rp, int32_t* col, void* val) {
  hipStream_t s = h->stream;
  const int64_t rows = v.A * v.B;
  unsigned long long* keys[2] = {reinterpret_cast<unsigned long long*>(tmp + lay.o_k0), reinterpret_cast<unsigned long long*>(tmp + lay.o_k1)};
  unsigned* idx[2] = {reinterpret_cast<unsigned*>(tmp + lay.o_i0), reinterpret_cast<unsigned*>(tmp + lay.o_i1)};
  unsigned* hist = reinterpret_cast<unsigned*>(tmp + lay.o_h);
  int* bad = reinterpret_cast<int*>(tmp + lay.o_bad);
  int host_bad = 0;
  const int64_t ntiles = lay.ntiles;
  hipLaunchKernelGGL(k_clear_int, dim3(1), dim3(64), 0, s, bad);
  int cur = 0;
  if (nnz > 0) {
    const unsigned g = grid_for(nnz, 256 * 4, (int64_t)h->num_cus * 32);
    hipLaunchKernelGGL(k_tensor_keys, dim3(g), dim3(256), 0, s, nnz, v.A, v.B, v.C, v.xa, v.xb, v.xc, keys[0], idx[0], bad);
    cur = sort_pairs(h, nnz, ntiles, bits_of(v.C), bits_of(rows), keys, idx, hist);
    if (dtype == SPGEMM_F32)
      hipLaunchKernelGGL(k_tensor_compress<float>, dim3(g), dim3(256), 0, s, nnz, keys[cur], idx[cur], static_cast<const float*>(xval), col,
                         static_cast<float*>(val));
    else
      hipLaunchKernelGGL(k_tensor_compress<double>, dim3(g), dim3(256), 0, s, nnz, keys[cur], idx[cur], static_cast<const double*>(xval), col,
                         static_cast<double*>(val));
  }
  hipLaunchKernelGGL(k_tensor_rowptr, dim3(grid_for(rows + 1, 256, (int64_t)h->num_cus * 32)), dim3(256), 0, s, nnz, rows, keys[cur], rp);
  hipError_t e = hipGetLastError();
  if (e == hipSuccess) e = hipMemcpyAsync(&host_bad, bad, 4, hipMemcpyDeviceToHost, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (e != hipSuccess) return fail(h, SPGEMM_HIP_ERROR, std::string("unfolding: ") + hipGetErrorString(e));
  if (host_bad) return fail(h, SPGEMM_INVALID_INPUT, "a tensor coordinate is outside its mode's range");
  return SPGEMM_OK;
}

// Scratch of the entry point that allocates nothing: one array per device, held until the process ends.
constexpr int64_t kNoAllocMaxNnz = SPTENSOR_NOALLOC_MAX_NNZ;
constexpr size_t kNoAllocScratchBytes = (size_t)kNoAllocMaxNnz * 24 + ((size_t)kNoAllocMaxNnz / kSortTile + 1) * 1024 + 8 * 256;
static __device__ __align__(256) unsigned char scratch[kNoAllocScratchBytes];
constexpr int kMaxDevices = 64;
unsigned char* g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch` on each device, from hipGetSymbolAddress

}  // namespace

int sptensor_unfold(spgemm_handle h, int mode, int64_t I, int64_t J, int64_t K, int64_t nnz, const int32_t* xi, const int32_t* xj,
                    const int32_t* xk, const void* xval, int32_t dtype, spgemm_csr* out) {
  if (!h) return SPGEMM_INVALID_ARG;
  if (!out) return fail(h, SPGEMM_INVALID_ARG, "out is null");
  ModeView v{};
  int rc = check_tensor(h, mode, I, J, K, nnz, xi, xj, xk, xval, dtype, &v);
  if (rc) return rc;
  std::memset(out, 0, sizeof(*out));
  if ((rc = ensure_device(h))) return rc;
  const int64_t rows = v.A * v.B;
  const size_t vsz = dtype == SPGEMM_F32 ? 4 : 8;
  const UnfoldTmp lay = unfold_tmp_layout(nnz);
  int64_t* rp = static_cast<int64_t*>(dev_alloc(h, (size_t)(rows + 1) * 8));
  int32_t* col = nnz ? static_cast<int32_t*>(dev_alloc(h, (size_t)nnz * 4)) : nullptr;
  void* val = nnz ? dev_alloc(h, (size_t)nnz * vsz) : nullptr;
  unsigned char* tmp = static_cast<unsigned char*>(dev_alloc(h, lay.bytes));
  if (!rp || !tmp || (nnz && (!col || !val))) rc = fail(h, SPGEMM_ALLOC_FAILED, "allocation for the unfolding failed");
  if (rc == SPGEMM_OK) rc = unfold_run(h, v, nnz, xval, dtype, tmp, lay, rp, col, val);
  dev_free(h, tmp);
  if (rc != SPGEMM_OK) {
    dev_free(h, rp); dev_free(h, col); dev_free(h, val);
    return rc;
  }
  out->rows = rows; out->cols = v.C; out->nnz = nnz; out->dtype = dtype;
  out->rowptr = rp; out->colidx = col; out->values = val;
  return SPGEMM_OK;
}

int sptensor_unfold_noalloc(spgemm_handle h, int mode, int64_t I, int64_t J, int64_t K, int64_t nnz, const int32_t* xi, const int32_t* xj,
                            const int32_t* xk, const void* xval, int32_t dtype, int64_t* out_rowptr, int32_t* out_colidx,
                            void* out_values) {
  if (!h) return SPGEMM_INVALID_ARG;
  ModeView v{};
  int rc = check_tensor(h, mode, I, J, K, nnz, xi, xj, xk, xval, dtype, &v);
  if (rc) return rc;
  if (!out_rowptr || (nnz > 0 && (!out_colidx || !out_values))) return fail(h, SPGEMM_INVALID_ARG, "output array null");
  if (nnz > kNoAllocMaxNnz)
    return fail(h, SPGEMM_UNSUPPORTED, "sptensor_unfold_noalloc takes at most " + std::to_string(kNoAllocMaxNnz) + " entries (fixed scratch)");
  if ((rc = ensure_device(h))) return rc;
  int dev = 0;
  HIP_TRY(h, hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(h, SPGEMM_UNSUPPORTED, "device ordinal beyond the scratch table");
  if (!g_scratch_ptr[dev]) {   // once per device, with that device current
    void* ptr = nullptr;
    HIP_TRY(h, hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    g_scratch_ptr[dev] = static_cast<unsigned char*>(ptr);
  }
  const UnfoldTmp lay = unfold_tmp_layout(nnz);
  if (lay.bytes > kNoAllocScratchBytes) return fail(h, SPGEMM_UNSUPPORTED, "internal: scratch layout exceeds the fixed scratch");
  // (every buffer inside the scratch is written before it is read, the flag is cleared by a kernel:
  // what the previous call left behind does not matter)
  return unfold_run(h, v, nnz, xval, dtype, g_scratch_ptr[dev], lay, out_rowptr, out_colidx, out_values);
}

int sptensor_unfold_mode3(spgemm_handle h, int64_t I, int64_t J, int64_t K, int64_t nnz, const int32_t* xi, const int32_t* xj,
                          const int32_t* xk, const void* xval, int32_t dtype, spgemm_csr* out) {
  return sptensor_unfold(h, 3, I, J, K, nnz, xi, xj, xk, xval, dtype, out);
}

int spttm(spgemm_handle h, int mode, int64_t I, int64_t J, int64_t K, int64_t nnz, const int32_t* xi, const int32_t* xj, const int32_t* xk,
          const void* xval, int32_t dtype, const spgemm_csr* M, spgemm_csr* Y) {
  if (!h) return SPGEMM_INVALID_ARG;
  if (!Y) return fail(h, SPGEMM_INVALID_ARG, "Y is null");
  int rc = check_csr(h, M, "M");
  if (rc) return rc;
  ModeView v{};
  if (!mode_view(mode, I, J, K, xi, xj, xk, &v)) return fail(h, SPGEMM_INVALID_ARG, "mode must be 1, 2 or 3");
  if (M->rows != v.C) return fail(h, SPGEMM_DIM_MISMATCH, "M.rows differs from the extent of the contracted mode");
  if (M->dtype != dtype) return fail(h, SPGEMM_DTYPE_MISMATCH, "tensor and matrix value types differ");
  spgemm_csr X{};
  rc = sptensor_unfold(h, mode, I, J, K, nnz, xi, xj, xk, xval, dtype, &X);
  if (rc) return rc;
  rc = spgemm(h, &X, M, Y);
  dev_free(h, const_cast<int64_t*>(X.rowptr));
  dev_free(h, const_cast<int32_t*>(X.colidx));
  dev_free(h, const_cast<void*>(X.values));
  return rc;
}

int spttm_mode3(spgemm_handle h, int64_t I, int64_t J, int64_t K, int64_t nnz, const int32_t* xi, const int32_t* xj, const int32_t* xk,
                const void* xval, int32_t dtype, const spgemm_csr* M, spgemm_csr* Y) {
  return spttm(h, 3, I, J, K, nnz, xi, xj, xk, xval, dtype, M, Y);
}

int sptensor_fold(spgemm_handle h, int mode, int64_t I, int64_t J, int64_t K, const spgemm_csr* Y, int32_t* yi, int32_t* yj, int32_t* yk) {
  if (!h) return SPGEMM_INVALID_ARG;
  int rc = check_csr(h, Y, "Y");
  if (rc) return rc;
  ModeView v{};
  if (!mode_view(mode, I, J, K, yi, yj, yk, &v)) return fail(h, SPGEMM_INVALID_ARG, "mode must be 1, 2 or 3");
  if (I < 0 || J < 0 || K < 0) return fail(h, SPGEMM_INVALID_ARG, "negative size");
  if (v.B <= 0 || Y->rows != v.A * v.B || Y->cols != v.C)
    return fail(h, SPGEMM_DIM_MISMATCH, "Y is not the unfolding of a tensor of these extents over this mode");
  if (Y->nnz > 0 && (!yi || !yj || !yk)) return fail(h, SPGEMM_INVALID_ARG, "coordinate arrays null with nnz > 0");
  if (Y->nnz == 0 || Y->rows == 0) return SPGEMM_OK;
  if ((rc = ensure_device(h))) return rc;
  // (the view was built over the output arrays: xa / xb take the row's two coordinates, xc the column)
  hipLaunchKernelGGL(k_tensor_fold, dim3(grid_for(Y->rows, 4, (int64_t)h->num_cus * 32)), dim3(256), 0, h->stream, Y->rows, v.B, Y->rowptr,
                     Y->colidx, const_cast<int32_t*>(v.xa), const_cast<int32_t*>(v.xb), const_cast<int32_t*>(v.xc));
  HIP_TRY(h, hipGetLastError());
  return SPGEMM_OK;
}

int sptensor_fold_mode3(spgemm_handle h, int64_t J, const spgemm_csr* Y, int32_t* yi, int32_t* yj) {
  if (!h) return SPGEMM_INVALID_ARG;
  int rc = check_csr(h, Y, "Y");
  if (rc) return rc;
  if (J <= 0 || Y->rows % J != 0) return fail(h, SPGEMM_INVALID_ARG, "Y.rows is not a multiple of J");
  if (Y->nnz > 0 && (!yi || !yj)) return fail(h, SPGEMM_INVALID_ARG, "coordinate arrays null with nnz > 0");
  if (Y->nnz == 0 || Y->rows == 0) return SPGEMM_OK;
  if ((rc = ensure_device(h))) return rc;
  hipLaunchKernelGGL(k_tensor_fold, dim3(grid_for(Y->rows, 4, (int64_t)h->num_cus * 32)), dim3(256), 0, h->stream, Y->rows, J, Y->rowptr,
                     (const int32_t*)nullptr, yi, yj, (int32_t*)nullptr);
  HIP_TRY(h, hipGetLastError());
  return SPGEMM_OK;
}

// ---- row blocks in a pipeline ------------------------------------------------------------------

int spgemm_pipelined(spgemm_handle h, const spgemm_csr* A, const spgemm_csr* B, int nblocks, spgemm_csr* C_blocks, int64_t* block_rows) {
  if (!h) return SPGEMM_INVALID_ARG;
  int rc = check_pair(h, A, B);
  if (rc) return rc;
  if (!C_blocks || !block_rows) return fail(h, SPGEMM_INVALID_ARG, "C_blocks and block_rows must not be null");
  if (nblocks < 1 || nblocks > 4096) return fail(h, SPGEMM_INVALID_ARG, "nblocks takes 1..4096");
  if ((rc = ensure_device(h))) return rc;
  const int64_t m = A->rows;
  for (int t = 0; t < nblocks; ++t) std::memset(&C_blocks[t], 0, sizeof(spgemm_csr));
  // 1. products per row of the whole A (the count kernel), their prefix on the host, block boundaries of equal work
  std::vector<int> ip_host((size_t)m);
  {
    size_t off = 0;
    const size_t o_ctl = off; off = align_up(off + sizeof(Control));
    const size_t o_ip = off; off = align_up(off + (size_t)m * 4);
    const size_t o_cnt = off; off = align_up(off + (size_t)m * 4);
    const size_t o_bin = off; off = align_up(off + (size_t)m);
    unsigned char* tmp = static_cast<unsigned char*>(dev_alloc(h, off));
    if (!tmp) return fail(h, SPGEMM_ALLOC_FAILED, "allocation for the row-block planning failed");
    Control* ctl = reinterpret_cast<Control*>(tmp + o_ctl);
    Control host{};
    hipLaunchKernelGGL(k_init_control, dim3(1), dim3(64), 0, h->stream, ctl);
    if (m > 0)
      hipLaunchKernelGGL(k_count_rows, dim3(grid_for(m, 256, (int64_t)h->num_cus * 8)), dim3(kCountThreads), 0, h->stream, m, A->nnz, B->rows, A->rowptr, A->colidx,
                         B->rowptr, reinterpret_cast<int*>(tmp + o_ip), tmp + o_bin, reinterpret_cast<int*>(tmp + o_cnt), ctl, 0, 0);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && m > 0) e = hipMemcpyAsync(ip_host.data(), tmp + o_ip, (size_t)m * 4, hipMemcpyDeviceToHost, h->stream);
    if (e == hipSuccess) e = hipMemcpyAsync(&host, ctl, sizeof(Control), hipMemcpyDeviceToHost, h->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(h->stream);
    dev_free(h, tmp);
    if (e != hipSuccess) return fail(h, SPGEMM_HIP_ERROR, std::string("row-block planning: ") + hipGetErrorString(e));
    if (host.error) return fail(h, SPGEMM_INVALID_INPUT, "device-side input check failed (column out of range or rowptr not monotone)");
  }
  {
    double total = 0;
    for (int64_t i = 0; i < m; ++i) total += ip_host[(size_t)i] + 1.0;   // (+1: rows without products still cost a little)
    double run = 0;
    int t = 1;
    block_rows[0] = 0;
    for (int64_t i = 0; i < m && t < nblocks; ++i) {
      run += ip_host[(size_t)i] + 1.0;
      while (t < nblocks && run >= total * t / nblocks) block_rows[t++] = i + 1;
    }
    while (t <= nblocks) block_rows[t++] = m;
    block_rows[nblocks] = m;
  }
  // 2. a second context on a stream of its own (same priority) for the symbolic phases
  hipStream_t s2 = nullptr;
  HIP_TRY(h, hipStreamCreateWithFlags(&s2, hipStreamNonBlocking));
  spgemm_context h2 = *h;
  h2.stream = s2;
  h2.row_block = 1;
  h2.timing = 0;
  h2.timed.clear();
  h2.event_pool.clear();
  h2.err.clear();
  struct Block { spgemm_plan plan = nullptr; int64_t* rp = nullptr; int32_t* col = nullptr; void* val = nullptr; int64_t nnz = 0; hipEvent_t done = nullptr; };
  std::vector<Block> blk((size_t)nblocks);
  const size_t vsz = A->dtype == SPGEMM_F32 ? 4 : 8;
  auto block_of_a = [&](int t) {
    spgemm_csr a = *A;
    a.rows = block_rows[t + 1] - block_rows[t];
    a.rowptr = A->rowptr + block_rows[t];
    return a;
  };
  auto symbolic_of = [&](int t) -> int {
    const spgemm_csr a = block_of_a(t);
    blk[(size_t)t].rp = static_cast<int64_t*>(dev_alloc(h, (size_t)(a.rows + 1) * 8));
    if (!blk[(size_t)t].rp) return fail(h, SPGEMM_ALLOC_FAILED, "allocation of a block's row pointer failed");
    const int r = spgemm_symbolic(&h2, &a, B, blk[(size_t)t].rp, &blk[(size_t)t].nnz, &blk[(size_t)t].plan);
    if (r != SPGEMM_OK) h->err = h2.err;
    return r;
  };
  auto release_plan = [&](int t) {
    Block& b = blk[(size_t)t];
    if (b.done) { (void)hipEventSynchronize(b.done); (void)hipEventDestroy(b.done); b.done = nullptr; }
    if (b.plan) { spgemm_plan_destroy(b.plan); b.plan = nullptr; }
  };
  rc = symbolic_of(0);
  for (int t = 0; t < nblocks && rc == SPGEMM_OK; ++t) {
    Block& b = blk[(size_t)t];
    const spgemm_csr a = block_of_a(t);
    // numeric of block t on the handle's stream (enqueued only) ...
    if (b.nnz > 0) {
      b.col = static_cast<int32_t*>(dev_alloc(h, (size_t)b.nnz * 4));
      b.val = dev_alloc(h, (size_t)b.nnz * vsz);
      if (!b.col || !b.val) { rc = fail(h, SPGEMM_ALLOC_FAILED, "allocation of a block of C failed"); break; }
      rc = A->dtype == SPGEMM_F32 ? run_numeric<float>(h, b.plan, &a, B, b.rp, b.col, b.val) : run_numeric<double>(h, b.plan, &a, B, b.rp, b.col, b.val);
      if (rc != SPGEMM_OK) break;
    }
    if (hipEventCreateWithFlags(&b.done, hipEventDisableTiming) != hipSuccess || hipEventRecord(b.done, h->stream) != hipSuccess) {
      rc = fail(h, SPGEMM_HIP_ERROR, "event for a block's numeric phase failed");
      break;
    }
    // ... while the symbolic phase of block t + 1 runs on the other stream (this call returns when it is done)
    if (t + 1 < nblocks) rc = symbolic_of(t + 1);
    if (t >= 1) release_plan(t - 1);   // (its numeric phase has been running for a whole symbolic phase: wait and release)
  }
  if (hipStreamSynchronize(h->stream) != hipSuccess && rc == SPGEMM_OK) rc = fail(h, SPGEMM_HIP_ERROR, "numeric phase failed");
  (void)hipStreamSynchronize(s2);
  for (int t = 0; t < nblocks; ++t) release_plan(t);
  for (auto e : h2.event_pool) (void)hipEventDestroy(e);
  (void)hipStreamDestroy(s2);
  drop_timed(h);   // (per-block times are not reported)
  if (rc != SPGEMM_OK) {
    for (auto& b : blk) { dev_free(h, b.rp); dev_free(h, b.col); dev_free(h, b.val); }
    return rc;
  }
  for (int t = 0; t < nblocks; ++t) {
    const Block& b = blk[(size_t)t];
    C_blocks[t].rows = block_rows[t + 1] - block_rows[t];
    C_blocks[t].cols = B->cols;
    C_blocks[t].nnz = b.nnz;
    C_blocks[t].dtype = A->dtype;
    C_blocks[t].rowptr = b.rp; C_blocks[t].colidx = b.col; C_blocks[t].values = b.val;
  }
  return SPGEMM_OK;
}

}  // extern "C"

// ---- outer-product route -------------------------------------------------------------------

namespace {

__global__ void k_pair_keys(int64_t n, const int32_t* __restrict__ hi, const int32_t* __restrict__ lo, unsigned long long* __restrict__ keys,
                            unsigned* __restrict__ idx) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < n; p += stride) {
    keys[p] = ((unsigned long long)(unsigned)hi[p] << 32) | (unsigned)lo[p];
    idx[p] = (unsigned)p;
  }
}

// In-place exclusive scan of n counters (n may be hundreds of millions); sums: ceil(n / kScanTileU32) + 1 slots of scratch.
void scan_u32_large(spgemm_context* h, int64_t n, unsigned* v, unsigned* sums) {
  const int64_t tiles = ceil_div(n > 0 ? n : 1, kScanTileU32);
  hipLaunchKernelGGL(k_scan_tile_sums, dim3((unsigned)tiles), dim3(256), 0, h->stream, n, v, sums);
  hipLaunchKernelGGL(k_scan_u32, dim3(1), dim3(1024), 0, h->stream, tiles, sums);
  hipLaunchKernelGGL(k_scan_tile_final, dim3((unsigned)tiles), dim3(256), 0, h->stream, n, v, sums);
}

struct DevBufs {   // device buffers released together
  spgemm_context* h;
  std::vector<void*> v;
  explicit DevBufs(spgemm_context* h_) : h(h_) {}
  ~DevBufs() { for (void* p : v) dev_free(h, p); }
  template <typename P>
  P* get(size_t count) {
    void* p = dev_alloc(h, count * sizeof(P));
    if (p) v.push_back(p);
    return static_cast<P*>(p);
  }
  void release(void* p) {
    for (auto& q : v) if (q == p) { dev_free(h, q); q = nullptr; }
  }
  void keep(void* p) {   // ownership leaves
    for (auto& q : v) if (q == p) q = nullptr;
  }
};

// Keeps the non-empty vectors of a compressed matrix (ptr over n vectors): vec / out_ptr are allocated here.
int dcs_compress(spgemm_context* h, int64_t n, int64_t nnz, const int64_t* ptr, DevBufs& bufs, int32_t** vec, int64_t** out_ptr, int64_t* nvec) {
  hipStream_t s = h->stream;
  unsigned* pos = bufs.get<unsigned>((size_t)n + 1);
  if (!pos) return fail(h, SPGEMM_ALLOC_FAILED, "allocation for the doubly compressed format failed");
  const unsigned g = grid_for(n, 256, (int64_t)h->num_cus * 32);
  hipLaunchKernelGGL(k_dcs_flags, dim3(g), dim3(256), 0, s, n, ptr, pos);
  hipLaunchKernelGGL(k_clear_int, dim3(1), dim3(64), 0, s, reinterpret_cast<int*>(pos + n));
  unsigned* sums = bufs.get<unsigned>((size_t)ceil_div(n + 1, kScanTileU32) + 1);
  if (!sums) return fail(h, SPGEMM_ALLOC_FAILED, "allocation for the doubly compressed format failed");
  scan_u32_large(h, n + 1, pos, sums);
  unsigned total = 0;
  HIP_TRY(h, hipMemcpyAsync(&total, pos + n, 4, hipMemcpyDeviceToHost, s));
  HIP_TRY(h, hipStreamSynchronize(s));
  *nvec = total;
  *vec = bufs.get<int32_t>((size_t)total + 1);
  *out_ptr = bufs.get<int64_t>((size_t)total + 1);
  if (!*vec || !*out_ptr) return fail(h, SPGEMM_ALLOC_FAILED, "allocation for the doubly compressed format failed");
  hipLaunchKernelGGL(k_dcs_fill, dim3(g), dim3(256), 0, s, n, ptr, pos, *vec, *out_ptr, nnz, (int64_t)total);
  HIP_TRY(h, hipGetLastError());
  return SPGEMM_OK;
}

template <typename T>
int outer_run(spgemm_context* h, const spgemm_dcs* A, const spgemm_dcs* B, int64_t cap, spgemm_csr* C) {
  hipStream_t s = h->stream;
  const int64_t m = A->minor_dim, n = B->minor_dim, na = A->nvec, nb = B->nvec;
  DevBufs bufs(h);
  int64_t* rp = bufs.get<int64_t>((size_t)m + 1);
  long long* off = bufs.get<long long>((size_t)na + 1);
  int32_t* match = bufs.get<int32_t>((size_t)na + 1);
  if (!rp || !off || !match) return fail(h, SPGEMM_ALLOC_FAILED, "allocation for the outer product failed");
  long long total = 0;
  if (na > 0) {
    hipLaunchKernelGGL(k_outer_count, dim3(grid_for(na, 256, (int64_t)h->num_cus * 32)), dim3(256), 0, s, na, A->vec, A->ptr, nb, B->vec, B->ptr,
                       off, match);
    hipLaunchKernelGGL(k_scan_i64, dim3(1), dim3(1024), 0, s, na, off);
    HIP_TRY(h, hipMemcpyAsync(&total, off + na, 8, hipMemcpyDeviceToHost, s));
    HIP_TRY(h, hipStreamSynchronize(s));
  }
  if (cap <= 0) cap = (int64_t)1 << 24;
  if (cap > ((int64_t)1 << 30)) cap = (int64_t)1 << 30;
  if (cap > total) cap = total > 0 ? total : 1;
  const int64_t ntiles = ceil_div(cap, kSortTile);
  // accumulation array: coordinates and insertion numbers twice (the sort's two buffers), values once
  unsigned long long* keys[2] = {bufs.get<unsigned long long>((size_t)cap), bufs.get<unsigned long long>((size_t)cap)};
  unsigned* seq[2] = {bufs.get<unsigned>((size_t)cap), bufs.get<unsigned>((size_t)cap)};
  double* vals = bufs.get<double>((size_t)cap);
  unsigned* hist = bufs.get<unsigned>((size_t)ntiles * 256);
  if (!keys[0] || !keys[1] || !seq[0] || !seq[1] || !vals || !hist) return fail(h, SPGEMM_ALLOC_FAILED, "allocation of the accumulation array failed");
  const int64_t cap_grid = (int64_t)h->num_cus * 32;
  // all array: sorted, unique coordinates with their sums
  unsigned long long* all_k = nullptr;
  double* all_v = nullptr;
  int64_t all_n = 0;
  // sorted array with repeats -> unique array: head flags, their scan, one walk per run
  auto reduce = [&](int64_t cnt, const unsigned long long* k, const unsigned* sq, const double* v, unsigned long long** ok, double** ov,
                    int64_t* on) -> int {
    unsigned* pos = bufs.get<unsigned>((size_t)cnt + 1);
    unsigned* sums = bufs.get<unsigned>((size_t)ceil_div(cnt + 1, kScanTileU32) + 1);
    if (!pos || !sums) return fail(h, SPGEMM_ALLOC_FAILED, "allocation for the merge stage failed");
    hipLaunchKernelGGL(k_outer_heads, dim3(grid_for(cnt, 256, cap_grid)), dim3(256), 0, s, cnt, k, pos);
    hipLaunchKernelGGL(k_clear_int, dim3(1), dim3(64), 0, s, reinterpret_cast<int*>(pos + cnt));
    scan_u32_large(h, cnt + 1, pos, sums);
    unsigned uniq = 0;
    HIP_TRY(h, hipMemcpyAsync(&uniq, pos + cnt, 4, hipMemcpyDeviceToHost, s));
    HIP_TRY(h, hipStreamSynchronize(s));
    *ok = bufs.get<unsigned long long>((size_t)uniq);
    *ov = bufs.get<double>((size_t)uniq);
    if (!*ok || !*ov) return fail(h, SPGEMM_ALLOC_FAILED, "allocation of the all array failed");
    hipLaunchKernelGGL(k_outer_reduce, dim3(grid_for(cnt, 256, cap_grid)), dim3(256), 0, s, cnt, k, sq, v, pos, *ok, *ov);
    HIP_TRY(h, hipGetLastError());
    *on = uniq;
    bufs.release(pos);
    bufs.release(sums);
    return SPGEMM_OK;
  };
  const int bits_lo = bits_of(n), bits_hi = bits_of(m);
  for (long long t0 = 0; t0 < total; t0 += cap) {
    const int64_t cnt = total - t0 < cap ? total - t0 : cap;
    // insert
    hipLaunchKernelGGL(k_outer_insert<T>, dim3(grid_for(cnt, 256, cap_grid)), dim3(256), 0, s, (int64_t)t0, cnt, na, off, match, A->ptr, A->idx,
                       static_cast<const T*>(A->values), B->ptr, B->idx, static_cast<const T*>(B->values), keys[0], seq[0], vals);
    // sort
    const int cur = sort_pairs(h, cnt, ceil_div(cnt, kSortTile), bits_lo, bits_hi, keys, seq, hist);
    // merge: equal coordinates of the batch, then the batch into the all array
    unsigned long long* uk = nullptr;
    double* uv = nullptr;
    int64_t un = 0;
    int rc = reduce(cnt, keys[cur], seq[cur], vals, &uk, &uv, &un);
    if (rc) return rc;
    if (all_n == 0) {
      all_k = uk; all_v = uv; all_n = un;
      continue;
    }
    if (all_n + un >= 0xffffffffLL) return fail(h, SPGEMM_UNSUPPORTED, "the all array of the outer product would exceed 2^32 - 1 components");
    unsigned long long* mk = bufs.get<unsigned long long>((size_t)(all_n + un));
    double* mv = bufs.get<double>((size_t)(all_n + un));
    if (!mk || !mv) return fail(h, SPGEMM_ALLOC_FAILED, "allocation for the merge stage failed");
    hipLaunchKernelGGL(k_outer_merge, dim3(grid_for(all_n + un, 256, cap_grid)), dim3(256), 0, s, all_n, all_k, all_v, un, uk, uv, mk, mv);
    unsigned long long* nk = nullptr;
    double* nv = nullptr;
    int64_t nn = 0;
    rc = reduce(all_n + un, mk, nullptr, mv, &nk, &nv, &nn);
    if (rc) return rc;
    bufs.release(all_k); bufs.release(all_v); bufs.release(uk); bufs.release(uv); bufs.release(mk); bufs.release(mv);
    all_k = nk; all_v = nv; all_n = nn;
  }
  // compress
  int32_t* col = all_n ? bufs.get<int32_t>((size_t)all_n) : nullptr;
  T* val = all_n ? bufs.get<T>((size_t)all_n) : nullptr;
  if (all_n && (!col || !val)) return fail(h, SPGEMM_ALLOC_FAILED, "allocation of C failed");
  hipLaunchKernelGGL(k_tensor_rowptr, dim3(grid_for(m + 1, 256, cap_grid)), dim3(256), 0, s, all_n, m, all_k ? all_k : keys[0], rp);
  if (all_n)
    hipLaunchKernelGGL(k_outer_emit<T>, dim3(grid_for(all_n, 256, cap_grid)), dim3(256), 0, s, all_n, all_k, all_v, col, val);
  HIP_TRY(h, hipGetLastError());
  HIP_TRY(h, hipStreamSynchronize(s));
  bufs.keep(rp); bufs.keep(col); bufs.keep(val);
  C->rows = m; C->cols = n; C->nnz = all_n; C->dtype = A->dtype;
  C->rowptr = rp; C->colidx = col; C->values = val;
  return SPGEMM_OK;
}

int check_dcs(spgemm_context* h, const spgemm_dcs* M, const char* name) {
  if (!M) return fail(h, SPGEMM_INVALID_ARG, std::string(name) + " is null");
  if (M->major_dim < 0 || M->minor_dim < 0 || M->nvec < 0 || M->nnz < 0 || M->nvec > M->major_dim)
    return fail(h, SPGEMM_INVALID_ARG, std::string(name) + ": bad size");
  if (M->dtype != SPGEMM_F32 && M->dtype != SPGEMM_F64) return fail(h, SPGEMM_INVALID_ARG, std::string(name) + ": unknown dtype");
  if (!M->ptr || (M->nvec > 0 && !M->vec) || (M->nnz > 0 && (!M->idx || !M->values)))
    return fail(h, SPGEMM_INVALID_ARG, std::string(name) + ": array null");
  if (M->major_dim >= 0x7fffffffLL || M->minor_dim >= 0x7fffffffLL || M->nnz >= 0xffffffffLL)
    return fail(h, SPGEMM_UNSUPPORTED, std::string(name) + ": extents must be below 2^31 - 1, nnz below 2^32 - 1");
  return SPGEMM_OK;
}

}  // namespace

extern "C" {

int spgemm_dcs_free(spgemm_handle h, spgemm_dcs* M) {
  if (!h || !M) return SPGEMM_INVALID_ARG;
  dev_free(h, const_cast<int32_t*>(M->vec));
  dev_free(h, const_cast<int64_t*>(M->ptr));
  dev_free(h, const_cast<int32_t*>(M->idx));
  dev_free(h, const_cast<void*>(M->values));
  std::memset(M, 0, sizeof(*M));
  return SPGEMM_OK;
}

int spgemm_dcsr_from_csr(spgemm_handle h, const spgemm_csr* M, spgemm_dcs* out) {
  if (!h) return SPGEMM_INVALID_ARG;
  int rc = check_csr(h, M, "M");
  if (rc) return rc;
  if (!out) return fail(h, SPGEMM_INVALID_ARG, "out is null");
  if (M->nnz >= 0xffffffffLL) return fail(h, SPGEMM_UNSUPPORTED, "nnz must be below 2^32 - 1");
  std::memset(out, 0, sizeof(*out));
  if ((rc = ensure_device(h))) return rc;
  DevBufs bufs(h);
  const size_t vsz = M->dtype == SPGEMM_F32 ? 4 : 8;
  int32_t* vec = nullptr;
  int64_t* ptr = nullptr;
  int64_t nvec = 0;
  if ((rc = dcs_compress(h, M->rows, M->nnz, M->rowptr, bufs, &vec, &ptr, &nvec))) return rc;
  int32_t* idx = bufs.get<int32_t>((size_t)M->nnz);
  void* val = bufs.get<unsigned char>((size_t)M->nnz * vsz);
  if (!idx || !val) return fail(h, SPGEMM_ALLOC_FAILED, "allocation for the doubly compressed format failed");
  if (M->nnz > 0) {
    HIP_TRY(h, hipMemcpyAsync(idx, M->colidx, (size_t)M->nnz * 4, hipMemcpyDeviceToDevice, h->stream));
    HIP_TRY(h, hipMemcpyAsync(val, M->values, (size_t)M->nnz * vsz, hipMemcpyDeviceToDevice, h->stream));
  }
  HIP_TRY(h, hipStreamSynchronize(h->stream));
  bufs.keep(vec); bufs.keep(ptr); bufs.keep(idx); bufs.keep(val);
  *out = spgemm_dcs{M->rows, M->cols, nvec, M->nnz, vec, ptr, idx, val, M->dtype};
  return SPGEMM_OK;
}

int spgemm_dcsc_from_csr(spgemm_handle h, const spgemm_csr* M, spgemm_dcs* out) {
  if (!h) return SPGEMM_INVALID_ARG;
  int rc = check_csr(h, M, "M");
  if (rc) return rc;
  if (!out) return fail(h, SPGEMM_INVALID_ARG, "out is null");
  if (M->nnz >= 0xffffffffLL) return fail(h, SPGEMM_UNSUPPORTED, "nnz must be below 2^32 - 1");
  std::memset(out, 0, sizeof(*out));
  if ((rc = ensure_device(h))) return rc;
  hipStream_t s = h->stream;
  DevBufs bufs(h);
  const int64_t nnz = M->nnz;
  const size_t vsz = M->dtype == SPGEMM_F32 ? 4 : 8;
  const int64_t ntiles = ceil_div(nnz > 0 ? nnz : 1, kSortTile);
  // compressed sparse columns first: sort the entries by (column, row), stable
  int32_t* rowid = bufs.get<int32_t>((size_t)nnz);
  unsigned long long* keys[2] = {bufs.get<unsigned long long>((size_t)nnz), bufs.get<unsigned long long>((size_t)nnz)};
  unsigned* seq[2] = {bufs.get<unsigned>((size_t)nnz), bufs.get<unsigned>((size_t)nnz)};
  unsigned* hist = bufs.get<unsigned>((size_t)ntiles * 256);
  int64_t* colptr = bufs.get<int64_t>((size_t)M->cols + 1);
  int32_t* idx = bufs.get<int32_t>((size_t)nnz);
  void* val = bufs.get<unsigned char>((size_t)nnz * vsz);
  if (!rowid || !keys[0] || !keys[1] || !seq[0] || !seq[1] || !hist || !colptr || !idx || !val)
    return fail(h, SPGEMM_ALLOC_FAILED, "allocation for the doubly compressed format failed");
  int cur = 0;
  const int64_t cap_grid = (int64_t)h->num_cus * 32;
  if (nnz > 0) {
    hipLaunchKernelGGL(k_expand_rows, dim3(grid_for(M->rows, 4, cap_grid)), dim3(256), 0, s, M->rows, M->rowptr, rowid);
    hipLaunchKernelGGL(k_pair_keys, dim3(grid_for(nnz, 256 * 4, cap_grid)), dim3(256), 0, s, nnz, M->colidx, rowid, keys[0], seq[0]);
    cur = sort_pairs(h, nnz, ntiles, bits_of(M->rows), bits_of(M->cols), keys, seq, hist);
    const unsigned g = grid_for(nnz, 256 * 4, cap_grid);
    if (M->dtype == SPGEMM_F32)
      hipLaunchKernelGGL(k_tensor_compress<float>, dim3(g), dim3(256), 0, s, nnz, keys[cur], seq[cur], static_cast<const float*>(M->values), idx,
                         static_cast<float*>(val));
    else
      hipLaunchKernelGGL(k_tensor_compress<double>, dim3(g), dim3(256), 0, s, nnz, keys[cur], seq[cur], static_cast<const double*>(M->values), idx,
                         static_cast<double*>(val));
  }
  hipLaunchKernelGGL(k_tensor_rowptr, dim3(grid_for(M->cols + 1, 256, cap_grid)), dim3(256), 0, s, nnz, M->cols, keys[cur], colptr);
  HIP_TRY(h, hipGetLastError());
  int32_t* vec = nullptr;
  int64_t* ptr = nullptr;
  int64_t nvec = 0;
  if ((rc = dcs_compress(h, M->cols, nnz, colptr, bufs, &vec, &ptr, &nvec))) return rc;
  HIP_TRY(h, hipStreamSynchronize(s));
  bufs.keep(vec); bufs.keep(ptr); bufs.keep(idx); bufs.keep(val);
  *out = spgemm_dcs{M->cols, M->rows, nvec, nnz, vec, ptr, idx, val, M->dtype};
  return SPGEMM_OK;
}

int spgemm_outer(spgemm_handle h, const spgemm_dcs* A, const spgemm_dcs* B, int64_t acc_capacity, spgemm_csr* C) {
  if (!h) return SPGEMM_INVALID_ARG;
  int rc = check_dcs(h, A, "A");
  if (rc) return rc;
  if ((rc = check_dcs(h, B, "B"))) return rc;
  if (!C) return fail(h, SPGEMM_INVALID_ARG, "C is null");
  if (acc_capacity < 0) return fail(h, SPGEMM_INVALID_ARG, "negative accumulation capacity");
  if (A->major_dim != B->major_dim) return fail(h, SPGEMM_DIM_MISMATCH, "A's columns and B's rows differ in extent");
  if (A->dtype != B->dtype) return fail(h, SPGEMM_DTYPE_MISMATCH, "A and B value types differ");
  std::memset(C, 0, sizeof(*C));
  if ((rc = ensure_device(h))) return rc;
  return A->dtype == SPGEMM_F32 ? outer_run<float>(h, A, B, acc_capacity, C) : outer_run<double>(h, A, B, acc_capacity, C);
}

}  // extern "C"
