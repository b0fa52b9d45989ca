// Dense LDS workspaces for long rows (Gustavson's flag list / coordinate list of the
// paper's section 4.4, and the dense first-order workspace of section 7.2), one workgroup
// of 1024 threads per row, rows handed out heaviest class first through a device counter.
//
// Symbolic: a flag list with one bit per column (up to 2^20 columns per pass in 128 KB of
//   LDS); products set bits, the row's size is the population count.
// Numeric : the column space is cut into windows of kWinCols columns.  Per window the flag
//   bits are rebuilt, an exclusive prefix over the flag words gives every present column its
//   rank, and the window's columns are cut (at flag-word granularity) into tiles of at most
//   kTileSlots present columns.  A tile's sums live in a dense array of doubles indexed by
//   rank - so LDS holds only columns that exist in C, and the finished tile is already in
//   ascending column order: values stream out as one contiguous run and the column
//   indices are decoded from the flag words (boolean indexing in the paper's words).
#pragma once
#include "common.cuh"

namespace spg {

constexpr int kDenseThreads = 1024;
constexpr int kDenseWaves = kDenseThreads / kWave;
constexpr int kShortLen = 32;           // B-row pieces shorter than this are packed across lanes
constexpr int kSymFlagWords = 32768;    // 2^20 columns per symbolic pass (128 KB)
constexpr int kWinCols = 131072;        // numeric window (16 KB flags + 16 KB prefix)
constexpr int kWinWords = kWinCols / 32;
constexpr int kTileSlots = 12288;       // doubles per numeric tile (96 KB)
constexpr int kTileCut = kTileSlots - 32;

struct WaveScratch {
  long long start[kWave];
  int pre[kWave];
};

// Calls f(q, p) for every pair (A entry p of the row, B entry q of row a_col[p]).  When
// prune is set (B rows ascending) the B rows are first narrowed to columns in
// [c_lo, c_hi) by binary search; f must still test the column range itself otherwise.
// Each wave takes 64 A entries at a time: pieces of kShortLen or more are walked by the
// whole wave one after another (coalesced), the shorter ones are concatenated and
// walked together, a lane finding its piece by a search over the 64 offsets.
template <class F>
__device__ __forceinline__ void stream_products(int64_t a0, int d, const int32_t* __restrict__ a_col,
                                                const int64_t* __restrict__ b_rp, const int32_t* __restrict__ b_col,
                                                bool prune, int c_lo, int c_hi, WaveScratch* ws, F f) {
  const int wave = threadIdx.x >> 6;
  const int lane = lane_id();
  for (int base = wave * kWave; base < d; base += kDenseWaves * kWave) {
    const int e = base + lane;
    int64_t s = 0;
    int len = 0;
    if (e < d) {
      const int k = a_col[a0 + e];
      s = b_rp[k];
      int64_t en = b_rp[k + 1];
      if (prune && en > s) {
        s = lower_bound_i32(b_col, s, en, c_lo);
        en = lower_bound_i32(b_col, s, en, c_hi);
      }
      len = (int)(en - s);
    }
    unsigned long long longs = __ballot(len >= kShortLen);
    while (longs) {
      const int j = __ffsll((long long)longs) - 1;
      longs &= longs - 1;
      const int64_t sj = __shfl(s, j, kWave);
      const int lj = __shfl(len, j, kWave);
      const int64_t pj = a0 + base + j;
      for (int t = lane; t < lj; t += kWave) f(sj + t, pj);
    }
    const int sl = len < kShortLen ? len : 0;
    const int incl = wave_incl_scan(sl);
    const int total = __shfl(incl, kWave - 1, kWave);
    if (total > 0) {
      ws->pre[lane] = incl - sl;
      ws->start[lane] = s;
      wave_sync();
      for (int t = lane; t < total; t += kWave) {
        int lo = 0, hi = kWave;
        while (hi - lo > 1) {
          const int mid = (lo + hi) >> 1;
          if (ws->pre[mid] <= t) lo = mid; else hi = mid;
        }
        f(ws->start[lo] + (t - ws->pre[lo]), a0 + base + lo);
      }
      wave_sync();
    }
  }
}

// Sum over the workgroup; every thread gets the result.  red: kDenseWaves + 1 ints of LDS.
__device__ __forceinline__ int block_sum(int v, int* red) {
  v = wave_sum(v);
  __syncthreads();
  if (lane_id() == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  int s = 0;
#pragma unroll
  for (int w = 0; w < kDenseWaves; ++w) s += red[w];
  return s;
}

// Fetch the next row of the dense bins (4..6), heaviest class first; -1 when none is left.
__device__ __forceinline__ int next_dense_row(const int* __restrict__ perm, Control* ctl, int phase, int* s_row) {
  __syncthreads();
  if (threadIdx.x == 0) {
    const unsigned lo = ctl->offset[phase][4], hi = ctl->offset[phase][7];
    const unsigned idx = atomicAdd(&ctl->work[phase], 1u);
    *s_row = idx < hi - lo ? perm[hi - 1 - idx] : -1;
  }
  __syncthreads();
  return *s_row;
}

__global__ __launch_bounds__(kDenseThreads) void k_sym_dense(const int* __restrict__ perm, Control* ctl,
                                                             const int64_t* __restrict__ a_rp, const int32_t* __restrict__ a_col,
                                                             const int64_t* __restrict__ b_rp, const int32_t* __restrict__ b_col,
                                                             int64_t n_cols, int* __restrict__ cnt) {
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned* flags = reinterpret_cast<unsigned*>(smem);                               // kSymFlagWords
  WaveScratch* ws = reinterpret_cast<WaveScratch*>(smem + kSymFlagWords * 4) + (threadIdx.x >> 6);
  int* red = reinterpret_cast<int*>(smem + kSymFlagWords * 4 + sizeof(WaveScratch) * kDenseWaves);
  int* s_row = red + kDenseWaves + 1;
  if (ctl->error) return;
  const bool sorted = ctl->b_sorted != 0;
  const int64_t span = (int64_t)kSymFlagWords * 32;
  while (true) {
    const int row = next_dense_row(perm, ctl, 0, s_row);
    if (row < 0) break;
    const int64_t a0 = a_rp[row];
    const int d = (int)(a_rp[row + 1] - a0);
    int total = 0;
    for (int64_t c0 = 0; c0 < n_cols; c0 += span) {
      const int64_t c1 = (c0 + span < n_cols) ? c0 + span : n_cols;
      const int words = (int)((c1 - c0 + 31) >> 5);
      for (int w = threadIdx.x; w < words; w += kDenseThreads) flags[w] = 0;
      __syncthreads();
      const int lo = (int)c0, hi = (int)c1;
      stream_products(a0, d, a_col, b_rp, b_col, sorted && n_cols > span, lo, hi, ws,
                      [&](int64_t q, int64_t) {
                        const int c = b_col[q];
                        if (c >= lo && c < hi) atomicOr(&flags[(c - lo) >> 5], 1u << ((c - lo) & 31));
                      });
      __syncthreads();
      int local = 0;
      for (int w = threadIdx.x; w < words; w += kDenseThreads) local += __popc(flags[w]);
      total += block_sum(local, red);
    }
    if (threadIdx.x == 0) cnt[row] = total;
  }
}

constexpr size_t kSymDenseLds = (size_t)kSymFlagWords * 4 + sizeof(WaveScratch) * kDenseWaves + (kDenseWaves + 4) * sizeof(int);

template <typename T>
__global__ __launch_bounds__(kDenseThreads) void k_num_dense(const int* __restrict__ perm, Control* ctl,
                                                             const int64_t* __restrict__ a_rp, const int32_t* __restrict__ a_col,
                                                             const T* __restrict__ a_val, const int64_t* __restrict__ b_rp,
                                                             const int32_t* __restrict__ b_col, const T* __restrict__ b_val,
                                                             int64_t n_cols, const int64_t* __restrict__ c_rp,
                                                             int32_t* __restrict__ c_col, T* __restrict__ c_val) {
  extern __shared__ __align__(16) unsigned char smem[];
  double* acc = reinterpret_cast<double*>(smem);                                     // kTileSlots
  unsigned* flags = reinterpret_cast<unsigned*>(smem + (size_t)kTileSlots * 8);      // kWinWords
  unsigned* cum = flags + kWinWords;                                                 // kWinWords + 1
  unsigned char* tail = reinterpret_cast<unsigned char*>(cum + kWinWords + 4);
  WaveScratch* ws = reinterpret_cast<WaveScratch*>(tail) + (threadIdx.x >> 6);
  int* red = reinterpret_cast<int*>(tail + sizeof(WaveScratch) * kDenseWaves);
  int* s_row = red + kDenseWaves + 1;
  if (ctl->error) return;
  const bool sorted = ctl->b_sorted != 0;
  const int tid = threadIdx.x;
  while (true) {
    const int row = next_dense_row(perm, ctl, 1, s_row);
    if (row < 0) break;
    const int64_t a0 = a_rp[row];
    const int d = (int)(a_rp[row + 1] - a0);
    int64_t out = c_rp[row];
    for (int64_t c0 = 0; c0 < n_cols; c0 += kWinCols) {
      const int64_t c1 = (c0 + kWinCols < n_cols) ? c0 + kWinCols : n_cols;
      const int words = (int)((c1 - c0 + 31) >> 5);
      const int wlo_col = (int)c0, whi_col = (int)c1;
      for (int w = tid; w < kWinWords; w += kDenseThreads) flags[w] = 0;
      __syncthreads();
      // pass 1: which columns of this window exist in the row
      stream_products(a0, d, a_col, b_rp, b_col, sorted, wlo_col, whi_col, ws,
                      [&](int64_t q, int64_t) {
                        const int c = b_col[q];
                        if (c >= wlo_col && c < whi_col) atomicOr(&flags[(c - wlo_col) >> 5], 1u << ((c - wlo_col) & 31));
                      });
      __syncthreads();
      // exclusive prefix of the flag-word populations (4 consecutive words per thread)
      constexpr int kPer = kWinWords / kDenseThreads;
      int pc[kPer], mine = 0;
#pragma unroll
      for (int t = 0; t < kPer; ++t) { pc[t] = __popc(flags[tid * kPer + t]); mine += pc[t]; }
      const int incl = wave_incl_scan(mine);
      if (lane_id() == kWave - 1) red[tid >> 6] = incl;
      __syncthreads();
      int before = 0, win_total = 0;
#pragma unroll
      for (int w = 0; w < kDenseWaves; ++w) {
        const int v = red[w];
        if (w < (tid >> 6)) before += v;
        win_total += v;
      }
      int run = before + incl - mine;
#pragma unroll
      for (int t = 0; t < kPer; ++t) { cum[tid * kPer + t] = (unsigned)run; run += pc[t]; }
      if (tid == kDenseThreads - 1) cum[kWinWords] = (unsigned)run;
      __syncthreads();
      if (win_total == 0) continue;
      // tiles: flag words whose prefix lies in [t*kTileCut, (t+1)*kTileCut)
      for (int tile_lo = 0; tile_lo < win_total; tile_lo += kTileCut) {
        int wa, wb;
        {
          int lo = 0, hi = kWinWords;   // first word with cum >= tile_lo
          while (lo < hi) { const int mid = (lo + hi) >> 1; if ((int)cum[mid] < tile_lo) lo = mid + 1; else hi = mid; }
          wa = lo;
          lo = wa; hi = kWinWords;      // first word with cum >= tile_lo + kTileCut
          while (lo < hi) { const int mid = (lo + hi) >> 1; if ((int)cum[mid] < tile_lo + kTileCut) lo = mid + 1; else hi = mid; }
          wb = lo;
        }
        if (wb > words) wb = words;
        const int base = (int)cum[wa];
        const int count = (int)cum[wb] - base;
        if (count <= 0) continue;
        for (int r = tid; r < count; r += kDenseThreads) acc[r] = 0.0;
        __syncthreads();
        const int t_lo = wlo_col + wa * 32;
        int t_hi = wlo_col + wb * 32;
        if (t_hi > whi_col) t_hi = whi_col;
        // pass 2: accumulate a_ik * b_kj at the rank of column j
        stream_products(a0, d, a_col, b_rp, b_col, sorted, t_lo, t_hi, ws,
                        [&](int64_t q, int64_t p) {
                          const int c = b_col[q];
                          if (c >= t_lo && c < t_hi) {
                            const int rel = c - wlo_col;
                            const int w = rel >> 5;
                            const int rank = (int)cum[w] - base + __popc(flags[w] & ((1u << (rel & 31)) - 1u));
                            __hip_atomic_fetch_add(&acc[rank], (double)a_val[p] * (double)b_val[q], __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_WORKGROUP);
                          }
                        });
        __syncthreads();
        // compress: values are already in column order; columns are decoded from the flags
        for (int r = tid; r < count; r += kDenseThreads) c_val[out + r] = (T)acc[r];
        for (int w = wa + tid; w < wb; w += kDenseThreads) {
          unsigned bits = flags[w];
          int64_t pos = out + ((int)cum[w] - base);
          while (bits) {
            const int b = __ffs((int)bits) - 1;
            bits &= bits - 1;
            c_col[pos++] = wlo_col + w * 32 + b;
          }
        }
        out += count;
        __syncthreads();
      }
    }
  }
}

constexpr size_t kNumDenseLds = (size_t)kTileSlots * 8 + (size_t)(2 * kWinWords + 4) * 4 + sizeof(WaveScratch) * kDenseWaves +
                                (kDenseWaves + 4) * sizeof(int);

}  // namespace spg
