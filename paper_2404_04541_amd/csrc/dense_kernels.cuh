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
constexpr int kUnroll = 4;              // loads in flight per lane while walking a long piece
constexpr int kChunk = kWave * kUnroll; // elements of a piece that one wave takes at a time
constexpr int kSymFlagWords = 32768;    // 2^20 columns per symbolic pass (128 KB)
constexpr int kWinCols = 131072;        // numeric window (16 KB flags + 16 KB prefix)
constexpr int kWinWords = kWinCols / 32;
constexpr int kTileSlots = 12288;       // doubles per numeric tile (96 KB)
constexpr int kTileCut = kTileSlots - 32;

// Per-workgroup bookkeeping of the piece walker below.
struct RowScratch {
  long long start[kDenseThreads];   // first B entry of each A entry's piece
  int plen[kDenseThreads];          // piece length
  int cpre[kDenseThreads + 1];      // exclusive prefix of chunk counts (long pieces)
  int spre[kDenseThreads + 1];      // exclusive prefix of lengths (short pieces)
  int red[2 * kDenseWaves];
  int s_row;
  int pad;
};

// Exclusive scans of two ints over the workgroup, with totals.  Contains barriers.
__device__ __forceinline__ void block_excl_scan2(int a, int b, int& ea, int& eb, int& ta, int& tb, int* red) {
  const int wave = threadIdx.x >> 6;
  const int ia = wave_incl_scan(a), ib = wave_incl_scan(b);
  __syncthreads();
  if (lane_id() == kWave - 1) { red[wave] = ia; red[kDenseWaves + wave] = ib; }
  __syncthreads();
  int pa = 0, pb = 0;
  ta = 0; tb = 0;
#pragma unroll
  for (int w = 0; w < kDenseWaves; ++w) {
    const int va = red[w], vb = red[kDenseWaves + w];
    if (w < wave) { pa += va; pb += vb; }
    ta += va; tb += vb;
  }
  ea = pa + ia - a;
  eb = pb + ib - b;
}

// Walks every pair (A entry p of the row, B entry q of row a_col[p]) and calls
// f(column, product).  range(k, s, en) may narrow the piece [s, en) of B row k first
// (f must test the column range itself when it matters).  Up to 1024 A entries are
// described at once (one per thread); pieces of kShortLen or more are cut into chunks of
// kChunk elements and the chunks are dealt to the 16 waves in contiguous shares, each wave
// reading a chunk coalesced with kUnroll loads in flight per lane; the shorter pieces are
// concatenated and walked by all threads, a thread finding its piece by a search over the
// prefix of lengths.  Returns the number of B entries visited.  Contains barriers: every
// thread of the workgroup must call it.
template <bool WITH_VALUES, typename T, class Range, class F>
__device__ __forceinline__ int stream_products(int64_t a0, int d, const int32_t* __restrict__ a_col, const T* __restrict__ a_val,
                                               const int64_t* __restrict__ b_rp, const int32_t* __restrict__ b_col,
                                               const T* __restrict__ b_val, RowScratch* rs, Range range, F f) {
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  int visited = 0;
  for (int base = 0; base < d; base += kDenseThreads) {
    const int e = base + tid;
    int64_t s = 0;
    int len = 0;
    if (e < d) {
      const int k = a_col[a0 + e];
      s = b_rp[k];
      int64_t en = b_rp[k + 1];
      range(k, s, en);
      len = (int)(en - s);
    }
    const int nch = len >= kShortLen ? (len + kChunk - 1) / kChunk : 0;
    const int sl = len < kShortLen ? len : 0;
    int ec, es, tc, ts;
    block_excl_scan2(nch, sl, ec, es, tc, ts, rs->red);
    rs->start[tid] = s;
    rs->plen[tid] = len;
    rs->cpre[tid] = ec;
    rs->spre[tid] = es;
    if (tid == 0) { rs->cpre[kDenseThreads] = tc; rs->spre[kDenseThreads] = ts; }
    __syncthreads();
    visited += tc + ts;
    if (tc > 0) {
      const int per = (tc + kDenseWaves - 1) / kDenseWaves;
      int c = wave * per;
      const int cend = (c + per < tc) ? c + per : tc;
      if (c < cend) {
        int lo = 0, hi = kDenseThreads;   // last entry whose first chunk is <= c
        while (hi - lo > 1) {
          const int mid = (lo + hi) >> 1;
          if (rs->cpre[mid] <= c) lo = mid; else hi = mid;
        }
        int ent = lo;
        while (c < cend) {
          const int cnext = rs->cpre[ent + 1];
          if (c >= cnext) { ++ent; continue; }
          const int64_t s_e = rs->start[ent];
          const int len_e = rs->plen[ent];
          const int cfirst = rs->cpre[ent];
          double av = 0.0;
          if (WITH_VALUES) av = (double)a_val[a0 + base + ent];
          const int cstop = cnext < cend ? cnext : cend;
          for (; c < cstop; ++c) {
            const int off = (c - cfirst) * kChunk + lane;
            int col[kUnroll];
            T bv[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
              const int idx = off + u * kWave;
              const bool ok = idx < len_e;
              col[u] = ok ? b_col[s_e + idx] : -1;
              if (WITH_VALUES) bv[u] = ok ? b_val[s_e + idx] : T(0);
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u)
              if (col[u] >= 0) f(col[u], WITH_VALUES ? av * (double)bv[u] : 0.0);
          }
        }
      }
    }
    for (int t = tid; t < ts; t += kDenseThreads) {
      int lo = 0, hi = kDenseThreads;
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (rs->spre[mid] <= t) lo = mid; else hi = mid;
      }
      const int64_t q = rs->start[lo] + (t - rs->spre[lo]);
      double prod = 0.0;
      if (WITH_VALUES) prod = (double)a_val[a0 + base + lo] * (double)b_val[q];
      f(b_col[q], prod);
    }
    __syncthreads();
  }
  return visited;
}

// Sum over the workgroup; every thread gets the result.  red: kDenseWaves ints of LDS.
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

// For ascending B rows: wp[k * (nw + 1) + w] = offset inside row k of the first column that
// is >= w * kWinCols (w = nw gives the row length).  Lets the numeric kernel cut a B row to
// a window with two loads instead of two binary searches.
__global__ __launch_bounds__(256) void k_window_ptrs(int64_t rows, int nw, const int64_t* __restrict__ b_rp,
                                                     const int32_t* __restrict__ b_col, const Control* __restrict__ ctl,
                                                     int* __restrict__ wp) {
  if (ctl->error || !ctl->b_sorted) return;
  const int64_t total = rows * (nw + 1);
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
    const int64_t k = i / (nw + 1);
    const int w = (int)(i - k * (nw + 1));
    const int64_t s = b_rp[k], en = b_rp[k + 1];
    int off;
    if (w == 0) off = 0;
    else if (w == nw) off = (int)(en - s);
    else off = (int)(lower_bound_i32(b_col, s, en, w * kWinCols) - s);
    wp[i] = off;
  }
}

struct NoRange {
  __device__ __forceinline__ void operator()(int, int64_t&, int64_t&) const {}
};

struct SearchRange {   // binary search in an ascending row
  const int32_t* b_col; int lo, hi;
  __device__ __forceinline__ void operator()(int, int64_t& s, int64_t& en) const {
    if (en > s) {
      s = lower_bound_i32(b_col, s, en, lo);
      en = lower_bound_i32(b_col, s, en, hi);
    }
  }
};

struct WindowRange {   // window pointers, then (optionally) a search inside the window
  const int* wp; const int32_t* b_col; int nw1, w, lo, hi; bool narrow;
  __device__ __forceinline__ void operator()(int k, int64_t& s, int64_t& en) const {
    const int* row = wp + (int64_t)k * nw1;
    en = s + row[w + 1];
    s = s + row[w];
    if (narrow && en > s) {
      s = lower_bound_i32(b_col, s, en, lo);
      en = lower_bound_i32(b_col, s, en, hi);
    }
  }
};

__global__ __launch_bounds__(kDenseThreads) void k_sym_dense(const int* __restrict__ perm, Control* ctl,
                                                             const int64_t* __restrict__ a_rp, const int32_t* __restrict__ a_col,
                                                             const int64_t* __restrict__ b_rp, const int32_t* __restrict__ b_col,
                                                             int64_t n_cols, int* __restrict__ cnt) {
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned* flags = reinterpret_cast<unsigned*>(smem);                               // kSymFlagWords
  RowScratch* rs = reinterpret_cast<RowScratch*>(smem + (size_t)kSymFlagWords * 4);
  if (ctl->error) return;
  const bool sorted = ctl->b_sorted != 0;
  const int64_t span = (int64_t)kSymFlagWords * 32;
  while (true) {
    const int row = next_dense_row(perm, ctl, 0, &rs->s_row);
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
      auto mark = [&](int c, double) {
        if (c >= lo && c < hi) atomicOr(&flags[(c - lo) >> 5], 1u << ((c - lo) & 31));
      };
      if (n_cols > span && sorted)
        stream_products<false, float>(a0, d, a_col, nullptr, b_rp, b_col, nullptr, rs, SearchRange{b_col, lo, hi}, mark);
      else
        stream_products<false, float>(a0, d, a_col, nullptr, b_rp, b_col, nullptr, rs, NoRange{}, mark);
      int local = 0;
      for (int w = threadIdx.x; w < words; w += kDenseThreads) local += __popc(flags[w]);
      total += block_sum(local, rs->red);
    }
    if (threadIdx.x == 0) cnt[row] = total;
  }
}

constexpr size_t kSymDenseLds = (size_t)kSymFlagWords * 4 + sizeof(RowScratch);

template <typename T>
__global__ __launch_bounds__(kDenseThreads) void k_num_dense(const int* __restrict__ perm, Control* ctl,
                                                             const int64_t* __restrict__ a_rp, const int32_t* __restrict__ a_col,
                                                             const T* __restrict__ a_val, const int64_t* __restrict__ b_rp,
                                                             const int32_t* __restrict__ b_col, const T* __restrict__ b_val,
                                                             int64_t n_cols, const int* __restrict__ wp, int nw,
                                                             const int64_t* __restrict__ c_rp,
                                                             int32_t* __restrict__ c_col, T* __restrict__ c_val) {
  extern __shared__ __align__(16) unsigned char smem[];
  double* acc = reinterpret_cast<double*>(smem);                                     // kTileSlots
  unsigned* flags = reinterpret_cast<unsigned*>(smem + (size_t)kTileSlots * 8);      // kWinWords
  unsigned* cum = flags + kWinWords;                                                 // kWinWords + 1 (+3 pad)
  RowScratch* rs = reinterpret_cast<RowScratch*>(cum + kWinWords + 4);
  if (ctl->error) return;
  const bool sorted = ctl->b_sorted != 0;
  const bool use_wp = sorted && wp != nullptr;
  const int tid = threadIdx.x;
  bool flags_clean = false;
  while (true) {
    const int row = next_dense_row(perm, ctl, 1, &rs->s_row);
    if (row < 0) break;
    const int64_t a0 = a_rp[row];
    const int d = (int)(a_rp[row + 1] - a0);
    int64_t out = c_rp[row];
    for (int w_id = 0; w_id < nw; ++w_id) {
      const int64_t c0 = (int64_t)w_id * kWinCols;
      const int64_t c1 = (c0 + kWinCols < n_cols) ? c0 + kWinCols : n_cols;
      const int words = (int)((c1 - c0 + 31) >> 5);
      const int wlo_col = (int)c0, whi_col = (int)c1;
      if (!flags_clean) {
        for (int w = tid; w < kWinWords; w += kDenseThreads) flags[w] = 0;
        flags_clean = true;
      }
      // (the barriers inside stream_products order the clearing before the first mark)
      // pass 1: which columns of this window exist in the row
      auto mark = [&](int c, double) {
        if (c >= wlo_col && c < whi_col) atomicOr(&flags[(c - wlo_col) >> 5], 1u << ((c - wlo_col) & 31));
      };
      int visited;
      if (use_wp)
        visited = stream_products<false, T>(a0, d, a_col, a_val, b_rp, b_col, b_val, rs,
                                            WindowRange{wp, b_col, nw + 1, w_id, wlo_col, whi_col, false}, mark);
      else if (sorted)
        visited = stream_products<false, T>(a0, d, a_col, a_val, b_rp, b_col, b_val, rs, SearchRange{b_col, wlo_col, whi_col}, mark);
      else
        visited = stream_products<false, T>(a0, d, a_col, a_val, b_rp, b_col, b_val, rs, NoRange{}, mark);
      if (visited == 0) continue;   // nothing of this row falls into the window: flags still clear
      flags_clean = false;
      // exclusive prefix of the flag-word populations (consecutive words per thread)
      constexpr int kPer = kWinWords / kDenseThreads;
      int pc[kPer], mine = 0;
#pragma unroll
      for (int t = 0; t < kPer; ++t) { pc[t] = __popc(flags[tid * kPer + t]); mine += pc[t]; }
      int excl, dummy_e, win_total, dummy_t;
      block_excl_scan2(mine, 0, excl, dummy_e, win_total, dummy_t, rs->red);
      int run = excl;
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
          hi = kWinWords;               // first word with cum >= tile_lo + kTileCut
          while (lo < hi) { const int mid = (lo + hi) >> 1; if ((int)cum[mid] < tile_lo + kTileCut) lo = mid + 1; else hi = mid; }
          wb = lo;
        }
        if (wb > words) wb = words;
        const int base = (int)cum[wa];
        const int count = (int)cum[wb] - base;
        if (count <= 0) continue;
        for (int r = tid; r < count; r += kDenseThreads) acc[r] = 0.0;
        const int t_lo = wlo_col + wa * 32;
        int t_hi = wlo_col + wb * 32;
        if (t_hi > whi_col) t_hi = whi_col;
        const bool whole = (wa == 0 && wb == words);
        // pass 2: accumulate a_ik * b_kj at the rank of column j
        auto add = [&](int c, double prod) {
          if (c >= t_lo && c < t_hi) {
            const int rel = c - wlo_col;
            const int w = rel >> 5;
            const int rank = (int)cum[w] - base + __popc(flags[w] & ((1u << (rel & 31)) - 1u));
            __hip_atomic_fetch_add(&acc[rank], prod, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
          }
        };
        if (use_wp)
          stream_products<true, T>(a0, d, a_col, a_val, b_rp, b_col, b_val, rs,
                                   WindowRange{wp, b_col, nw + 1, w_id, t_lo, t_hi, !whole}, add);
        else if (sorted)
          stream_products<true, T>(a0, d, a_col, a_val, b_rp, b_col, b_val, rs, SearchRange{b_col, t_lo, t_hi}, add);
        else
          stream_products<true, T>(a0, d, a_col, a_val, b_rp, b_col, b_val, rs, NoRange{}, add);
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

constexpr size_t kNumDenseLds = (size_t)kTileSlots * 8 + (size_t)(2 * kWinWords + 4) * 4 + sizeof(RowScratch);

}  // namespace spg
