// Dense LDS workspaces for long rows (Gustavson's flag list / coordinate list of the
// paper's section 4.4, and the dense first-order workspace of section 7.2), one workgroup
// of 1024 threads per row.
//
// Symbolic (k_sym_dense): a flag list with one bit per column (2^20 columns per span in
//   128 KB of LDS); products set bits, the row's size is the population count.  From the
//   finished flag list the kernel also plans the row's numeric work: the column space is cut
//   at multiples of kBlkCols columns into tiles, each small enough for the numeric workspace,
//   and the row's column structure goes to the plan (decoded columns, or the flag words of
//   direct blocks), so that the numeric phase need not find it again.
// Numeric (k_num_dense), one tile at a time, one pass over the tile's products:
//   direct tile (one block of kBlkCols columns in which the row is dense): sums live in a
//     dense array indexed by column; the flags say which exist; flags and sums are compressed
//     at the end ("boolean indexing" in the paper's words).
//   ranked tile (a run of blocks in which the row is sparse): an exclusive prefix over the flag
//     words gives every present column its rank; a product adds a_ik * b_kj at the rank of
//     column j - LDS holds only columns that exist in C and the finished tile is already in
//     ascending column order.  Flags and ranks come from the plan's column list; without one,
//     a first pass over the products rebuilds them.
//   searched tile (a whole short row): the row's columns sit in LDS and a product finds its
//     rank by bisection, so the tile's width does not matter.
//   The piece of B row k that falls into a tile is found with two loads from a table of
//   per-row block offsets (ascending B rows), so a pass touches only its own products.
#pragma once
#include "common.hpp"

namespace spg {

constexpr int kDenseThreads = 1024;
constexpr int kDenseWaves = kDenseThreads / kWave;
constexpr int kShortLen = 32;           // B-row pieces shorter than this are packed across lanes
constexpr int kUnroll = 4;              // loads in flight per lane while walking a long piece
constexpr int kChunk = kWave * kUnroll; // elements of a piece that one wave takes at a time
constexpr int kSymFlagWords = 32768;    // 2^20 columns per symbolic span (128 KB)
constexpr int kBlkCols = 8192;          // tile boundaries are multiples of this many columns
constexpr int kBlkShift = 13;
constexpr int kSpanBlocks = kSymFlagWords * 32 / kBlkCols;   // 128 blocks per symbolic span
constexpr int kTileBudget = 135 * 1024; // LDS bytes of one numeric tile (flags + ranks + sums)
constexpr int kRankBlkBytes = kBlkCols / 32 * 8;   // flag word + rank per 32 columns of a ranked tile
constexpr int kRankEntryBytes = 8;                // sum per entry of a ranked tile (its column goes straight to C)
constexpr int kDirectMinDefault = 6144; // a block with at least this many entries becomes a direct tile
constexpr int kRunTiles = 16;           // tiles handed to a workgroup at a time
constexpr int kListSlab = 1 << 20;      // list entries, tile and run records that a symbolic workgroup draws at a time
constexpr int kTileSlab = 2048;
constexpr int kRunSlab = 256;
constexpr int kDirectBit = 1 << 30;     // in TileRec::cnt
constexpr int kSearchBit = 1 << 29;     // in TileRec::cnt: a searched tile (ranks by bisection of the column list)
constexpr int kCountMask = kSearchBit - 1;
constexpr int kSearchCap = 11264;       // entries of a searched tile (column 4 B + sum 8 B each)
constexpr int kSegCap = 1024;           // A entries described in LDS at a time (numeric)
constexpr int kBlkWords = kBlkCols / 32;
constexpr int kSymPieces = 1024;         // A entries that the symbolic kernel describes in LDS at a time
constexpr int kListStage = kSymPieces * 5 / kDenseWaves;   // entries that a wave gathers in LDS (the piece walker's, free by then) before writing them to the column list
constexpr int kListBatch = 4;           // column-list loads in flight per thread
// every tile kind must fit the tile area of the numeric kernel
static_assert((long long)kSearchCap * 12 <= kTileBudget, "searched tile: 4 B column + 8 B sum per entry");
static_assert((long long)kBlkCols * 12 + kBlkCols / 8 <= kTileBudget, "direct tile: sums, columns by rank, flag words");
static_assert(kRankBlkBytes + 8LL * kBlkCols <= kTileBudget, "ranked tile: one block must fit even when it is full");
constexpr int kRegSegs = 2;             // segments of A entries that the numeric kernel keeps in registers
constexpr long long kListBias = 1LL << 40;   // RunRec::list holds position + bias (so that -1 can mean "none")
constexpr long long kListFlagWords = 1LL << 60;   // RunRec::list: the row's structure is kept as flag words, not as columns
constexpr int kFlagWordsNum = 1, kFlagWordsDen = 1;   // flag words are kept when words * Num <= entries * Den (measured: best near one entry per word)
constexpr int kGrpWords = 64;                // flag words per group: the plan keeps the rank of every group's first entry
constexpr int kSpanGroups = kSymFlagWords / kGrpWords;

// Layout of a span's structure kept as flag words: first the group ranks (row-relative rank of the first
// entry of every group of kGrpWords words, padded to 16 bytes), then the flag words themselves.
__host__ __device__ __forceinline__ int span_flag_words(int64_t n_cols, int64_t c0) {
  const int64_t left = n_cols - c0, span = (int64_t)kSymFlagWords * 32;
  return (int)(((left < span ? left : span) + 31) >> 5);
}
__host__ __device__ __forceinline__ int span_rank_slots(int words) { return (((words + kGrpWords - 1) / kGrpWords) + 3) & ~3; }

// Stores and loads of data that passes through the numeric kernel once (the result, the plan's
// column list): the non-temporal hint keeps it from displacing B, which is re-read all the time,
// from the caches.  (Not for the symbolic kernel's list writes: partial lines written with the
// hint are not combined, which costs more than it saves.)
template <typename V>
__device__ __forceinline__ void stream_store(V* p, V v) { __builtin_nontemporal_store(v, p); }
template <typename V>
__device__ __forceinline__ V stream_load(const V* p) { return __builtin_nontemporal_load(p); }

struct TileRec { int b0, b1, cnt, out; };     // blocks [b0, b1), entries (| kDirectBit), offset inside the row of C
// tiles [first, first + count) of one row; its A entries [a0, a0 + d); list (-1: the row has no list):
// where entry 0 of the row sits in the plan's list, plus kListBias - or, with kListFlagWords set,
// where the flag word of column 0 sits (the row's structure is kept as one bit per column)
struct RunRec { int row; unsigned first; int count, d; long long a0, list; };

// Per-workgroup bookkeeping of the piece walker below.
struct RowScratch {
  long long start[kSymPieces];   // first B entry of each A entry's piece
  int plen[kSymPieces];          // piece length
  int cpre[kSymPieces + 1];      // exclusive prefix of chunk counts (long pieces)
  int spre[kSymPieces + 1];      // exclusive prefix of lengths (short pieces)
  int red[2 * kDenseWaves];
  int s_row;
  int pad;
  unsigned long long span_ip;       // products streamed since the owner last cleared it
  SPG_CLK(ClkLds clk;)
};

// Exclusive scans of two ints over the workgroup, with totals.  Contains barriers.
// The 16 wave totals are scanned by every wave itself: lane w reads the total of wave w, a DPP row
// scan adds them up, and the wave takes its own prefix and the grand total with readlane.
__device__ __forceinline__ void block_excl_scan2(int a, int b, int& ea, int& eb, int& ta, int& tb, int* red) {
  static_assert(kDenseWaves == 16, "one DPP row of wave totals");
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int ia = wave_incl_scan(a), ib = wave_incl_scan(b);
  __syncthreads();
  if (lane_id() == kWave - 1) { red[wave] = ia; red[kDenseWaves + wave] = ib; }
  __syncthreads();
  const int l = lane_id() & (kDenseWaves - 1);
  const int sa = group_incl_scan<16>(red[l]), sb = group_incl_scan<16>(red[kDenseWaves + l]);
  ta = __builtin_amdgcn_readlane(sa, kDenseWaves - 1);
  tb = __builtin_amdgcn_readlane(sb, kDenseWaves - 1);
  const int pa = wave ? __builtin_amdgcn_readlane(sa, wave - 1) : 0;
  const int pb = wave ? __builtin_amdgcn_readlane(sb, wave - 1) : 0;
  ea = pa + ia - a;
  eb = pb + ib - b;
}

constexpr int kChunkUnroll = 8;

// The non-empty pieces that a pass walks, in LDS: first B entry, exclusive prefix of the chunk counts (np + 1
// values), length and (numeric) a_ik of every piece.
template <typename T>
struct PieceList {
  const long long* s;
  const int* cpre;
  const int* len;
  const T* av;
};

__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ long long uni64(long long v) {
  const unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(unsigned long long)v);
  const unsigned hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)((unsigned long long)v >> 32));
  return (long long)(((unsigned long long)hi << 32) | lo);
}

__device__ __forceinline__ int lane_get(int v, int lane) { return __builtin_amdgcn_readlane(v, lane); }
__device__ __forceinline__ long long lane_get(long long v, int lane) {
  const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(unsigned long long)v, lane);
  const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)((unsigned long long)v >> 32), lane);
  return (long long)(((unsigned long long)hi << 32) | lo);
}
__device__ __forceinline__ float lane_get(float v, int lane) { return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane)); }
__device__ __forceinline__ double lane_get(double v, int lane) { return __longlong_as_double(lane_get(__double_as_longlong(v), lane)); }

// Visits every element of the pieces once.  A piece is cut into chunks of 64 elements; the
// chunks of all pieces are dealt to the waves in contiguous shares; a wave reads a chunk
// coalesced (one element per lane) with kChunkUnroll chunks in flight.  Everything that
// describes a chunk is wave-uniform: the descriptors of the pieces that a batch of chunks can
// touch are fetched from LDS by one lane each and handed out with readlane, so a batch costs
// one LDS round trip before its loads are issued.  f(column, a, b) is called per element
// (a, b only meaningful when WITH_VALUES); g(columns, a's, b's) gets a whole batch of
// kChunkUnroll elements per lane (column -1: no element).
template <bool WITH_VALUES, typename T, class G>
__device__ __forceinline__ void chunk_pass_batches(int np, int nchunks, const PieceList<T> pl, const int32_t* __restrict__ b_col,
                                                   const T* __restrict__ b_val, G g) {
  const int wave = uni(threadIdx.x >> 6), lane = threadIdx.x & 63;
  np = uni(np);
  nchunks = uni(nchunks);
  const int per = (nchunks + kDenseWaves - 1) / kDenseWaves;
  int c = wave * per;
  const int cend = c + per < nchunks ? c + per : nchunks;
  if (c >= cend) return;
  int p;
  {
    int lo = 0, hi = np;   // last piece whose first chunk is <= c
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (uni(pl.cpre[mid]) <= c) lo = mid; else hi = mid;
    }
    p = lo;
  }
  for (; c < cend; c += kChunkUnroll) {
    // lane i describes piece p + i (a batch of kChunkUnroll chunks touches at most that many pieces)
    const int pi = p + lane < np ? p + lane : np;
    const int pj = p + lane < np ? p + lane : np - 1;
    const int d_first = pl.cpre[pi];
    const int d_len = pl.len[pj];
    const long long d_s = pl.s[pj];
    const T d_av = WITH_VALUES ? pl.av[pj] : T(0);
    int q = 0;
    // the piece in hand (wave-uniform; re-read from the lanes only when the piece changes)
    int q_first = lane_get(d_first, 0), q_next = lane_get(d_first, 1), q_len = lane_get(d_len, 0);
    const int32_t* pc = b_col + lane_get(d_s, 0);
    const T* pv = b_val + lane_get(d_s, 0);
    T q_av = WITH_VALUES ? lane_get(d_av, 0) : T(0);
    int col[kChunkUnroll];
    T bv[kChunkUnroll], au[kChunkUnroll];
#pragma unroll
    for (int u = 0; u < kChunkUnroll; ++u) {
      const int cu = c + u;
      col[u] = -1;
      bv[u] = T(0);
      au[u] = T(0);
      if (cu < cend) {
        if (cu >= q_next) {   // every piece has at least one chunk: one step suffices
          ++q;
          q_first = q_next;
          q_next = lane_get(d_first, q + 1);
          q_len = lane_get(d_len, q);
          pc = b_col + lane_get(d_s, q);
          pv = b_val + lane_get(d_s, q);
          if (WITH_VALUES) q_av = lane_get(d_av, q);
        }
        const int off = (cu - q_first) * kWave + lane;
        // (wave-uniform piece start + 32-bit lane offset: scalar base, one vector offset)
        if (off < q_len) {
          // (a piece is far shorter than 2^30 elements: the byte offset fits 32 bits, which lets the
          // load take the scalar base plus one vector offset)
          const unsigned byte_off = (unsigned)off * (unsigned)sizeof(int32_t);
          col[u] = *reinterpret_cast<const int32_t*>(reinterpret_cast<const char*>(pc) + byte_off);
          if (WITH_VALUES) bv[u] = *reinterpret_cast<const T*>(reinterpret_cast<const char*>(pv) + (unsigned)off * (unsigned)sizeof(T));
        }
        au[u] = q_av;
      }
    }
    p += q;
    g(col, au, bv);
  }
}

// chunk_pass with a functor f(column, a, b) per element.
template <bool WITH_VALUES, typename T, class F>
__device__ __forceinline__ void chunk_pass(int np, int nchunks, const PieceList<T> pl, const int32_t* __restrict__ b_col,
                                           const T* __restrict__ b_val, F f) {
  chunk_pass_batches<WITH_VALUES, T>(np, nchunks, pl, b_col, b_val,
                                     [&](const int (&col)[kChunkUnroll], const T (&au)[kChunkUnroll], const T (&bv)[kChunkUnroll]) {
#pragma unroll
                                       for (int u = 0; u < kChunkUnroll; ++u)
                                         if (col[u] >= 0) f(col[u], au[u], bv[u]);
                                     });
}

// Walks every pair (A entry p of the row, B entry q of row a_col[p]) and calls
// f(column).  range(k, s, en) may narrow the piece [s, en) of B row k first.  Up to kSymPieces A
// entries are described at once (one per thread).  Pieces of kShortLen or more are compacted to the
// front of the scratch arrays and walked like the numeric kernel's pieces: in chunks of 64 elements,
// dealt to the 16 waves in contiguous shares, kChunkUnroll chunks of whatever pieces in flight per
// wave.  The shorter pieces are compacted to the back and walked by all threads as one index space,
// a thread finding its piece by a search over the prefix of their lengths.
// Contains barriers: every thread of the workgroup must call it.
template <class Range, class F, class FB>
__device__ __forceinline__ void stream_columns(int64_t a0, int d, const int32_t* __restrict__ a_col,
                                               const int64_t* __restrict__ b_rp, const int32_t* __restrict__ b_col,
                                               RowScratch* rs, Range range, F f, FB fb) {
  const int tid = threadIdx.x, lane = tid & 63;
  static_assert(kSymPieces <= kDenseThreads, "a thread per described entry");
  for (int base = 0; base < d; base += kSymPieces) {
    const int e = base + tid;
    int64_t s = 0;
    int len = 0;
    if (e < d && tid < kSymPieces) {
      const int k = a_col[a0 + e];
      const Run<int64_t, 2> bounds = load_run<int64_t, 2>(b_rp + k);
      s = bounds.v[0];
      int64_t en = bounds.v[1];
      range(k, s, en);
      len = (int)(en - s);
    }
    const bool is_long = len >= kShortLen;
    const int nch = is_long ? (len + kWave - 1) >> 6 : 0;
    const int sl = is_long ? 0 : len;
    if (Range::kNarrows) {   // (a narrowed walk covers a part of the row: its products are counted for the caller)
      unsigned long long wl = (unsigned long long)len;
#pragma unroll
      for (int sh = 1; sh < kWave; sh <<= 1) wl += __shfl_xor(wl, sh, kWave);
      if (lane == 0 && wl) atomicAdd(&rs->span_ip, wl);
    }
    int li, ec, nl, tc, sj, es, nshort, ts;
    block_excl_scan2(is_long ? 1 : 0, nch, li, ec, nl, tc, rs->red);
    block_excl_scan2(sl > 0 ? 1 : 0, sl, sj, es, nshort, ts, rs->red);
    if (is_long) {
      rs->start[li] = s;
      rs->plen[li] = len;
      rs->cpre[li] = ec;
    } else if (sl > 0) {   // (long pieces fill the start array from the front, short ones from the back)
      rs->start[kSymPieces - 1 - sj] = s;
      rs->spre[sj] = es;
    }
    if (tid == 0) { rs->cpre[nl] = tc; rs->spre[nshort] = ts; }
    __syncthreads();
    SPG_CLK(clk_mark(&rs->clk, 2); clk_add(&rs->clk, 18, 1); clk_add(&rs->clk, 19, (unsigned long long)tc);)
    if (tc > 0)
      chunk_pass_batches<false, int>(nl, tc, PieceList<int>{rs->start, rs->cpre, rs->plen, nullptr}, b_col, static_cast<const int*>(nullptr),
                                     [&](const int (&c)[kChunkUnroll], const int (&)[kChunkUnroll], const int (&)[kChunkUnroll]) { fb(c); });
    SPG_CLK(clk_mark(&rs->clk, 3);)
    for (int t = tid; t < ts; t += kDenseThreads) {
      int lo = 0, hi = nshort;   // last short piece whose first element is <= t
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (rs->spre[mid] <= t) lo = mid; else hi = mid;
      }
      f(b_col[rs->start[kSymPieces - 1 - lo] + (t - rs->spre[lo])]);
    }
    __syncthreads();
    SPG_CLK(clk_mark(&rs->clk, 4);)
  }
}

// For ascending B rows: bp[k * nb1 + b] = number of entries of row k with a column below
// b * kBlkCols (b = nb1 - 1 gives the row length).  One thread per table slot, each bisecting its
// row (the threads of a row read the same few lines, and the table leaves in coalesced stores).
__global__ __launch_bounds__(256) void k_block_ptrs(int64_t rows, int nb1, const int64_t* __restrict__ b_rp,
                                                    const int32_t* __restrict__ b_col, const Control* __restrict__ ctl,
                                                    int* __restrict__ bp) {
  if (ctl->error || !ctl->b_sorted) return;
  const int64_t total = rows * nb1;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
    const int64_t k = i / nb1;
    const int b = (int)(i - k * nb1);
    const Run<int64_t, 2> bounds = load_run<int64_t, 2>(b_rp + k);
    const int64_t s = bounds.v[0], en = bounds.v[1];
    int off;
    if (b == 0 || en == s) off = 0;
    else if (b == nb1 - 1) off = (int)(en - s);
    else off = (int)(lower_bound_i32(b_col, s, en, b << kBlkShift) - s);
    bp[i] = off;
  }
}

struct NoRange {
  static constexpr bool kNarrows = false;
  __device__ __forceinline__ void operator()(int, int64_t&, int64_t&) const {}
};

struct TableRange {   // ascending rows with the block-offset table: the entries in blocks [b0, b1)
  static constexpr bool kNarrows = true;
  const int* bp; int nb1; int b0, b1;
  __device__ __forceinline__ void operator()(int k, int64_t& s, int64_t& en) const {
    const int* row = bp + (int64_t)k * nb1;
    en = s + row[b1];
    s += row[b0];
  }
};

struct SearchRange {   // binary search in an ascending row
  static constexpr bool kNarrows = true;
  const int32_t* b_col; int lo; int64_t hi;
  __device__ __forceinline__ void operator()(int, int64_t& s, int64_t& en) const {
    if (en > s) {
      s = lower_bound_i32(b_col, s, en, lo);
      if (hi <= 0x7fffffff) en = lower_bound_i32(b_col, s, en, (int)hi);
    }
  }
};

// LDS of the tile planner.
struct TilePlan {
  int blk_cnt[kSpanBlocks];
  int cum[kSpanBlocks + 1];
  int nxt[kSpanBlocks];
  TileRec rec[kSpanBlocks];
  int ntiles, ndirect, nruns;
  int next_block;         // list decode: the next block to hand to a wave
  unsigned tile_base, run_base;
  int row_out;
  int span_out0;          // row_out when the span began
  long long list_base;    // position of the span's first entry (or first flag word) in the plan's list, -1 = none
  int list_words;         // > 0: the span's structure goes to the list as that many flag words instead of columns
  int grp[kSpanGroups];   // entries per group of kGrpWords flag words
};

// index of the lowest set bit at or above position b in the 128-bit mask (hi:lo); 128 when none
__device__ __forceinline__ int next_bit128(unsigned long long lo, unsigned long long hi, int b) {
  if (b < 64) {
    const unsigned long long m = lo >> b;
    if (m) return b + __ffsll((long long)m) - 1;
    if (hi) return 64 + __ffsll((long long)hi) - 1;
    return 128;
  }
  if (b >= 128) return 128;
  const unsigned long long m = hi >> (b - 64);
  return m ? b + __ffsll((long long)m) - 1 : 128;
}

// index of the highest set bit below position e; -1 when none
__device__ __forceinline__ int prev_bit128(unsigned long long lo, unsigned long long hi, int e) {
  if (e > 64) {
    const unsigned long long m = e >= 128 ? hi : (hi & ((1ULL << (e - 64)) - 1ULL));
    if (m) return 127 - __clzll((long long)m);
    e = 64;
  }
  if (e <= 0) return -1;
  const unsigned long long m = e >= 64 ? lo : (lo & ((1ULL << e) - 1ULL));
  return m ? 63 - __clzll((long long)m) : -1;
}

// Cuts the nb blocks of one span (counts in tp->blk_cnt) into tiles; run by wave 0.
// A block with at least direct_min entries is a direct tile of its own; the blocks between
// are grouped greedily into ranked tiles of at most kTileBudget bytes
// (kRankBlkBytes per block + kRankEntryBytes per entry).  Records land in tp->rec, their number in tp->ntiles.
// First part (wave 0): entry prefix over the blocks and the span's total.
constexpr bool kSpanTwoHalves = kSpanBlocks > kWave;   // a lane plans one block, or two
static_assert(kSpanBlocks == kWave || kSpanBlocks == 2 * kWave, "a span of 64 or 128 blocks");
__device__ __forceinline__ void plan_head(TilePlan* tp, int nb, bool count_only) {
  const int l = lane_id();
  const int c0 = l < nb ? tp->blk_cnt[l] : 0;
  const int c1 = (kSpanTwoHalves && l + 64 < nb) ? tp->blk_cnt[l + 64] : 0;
  const int i0 = wave_incl_scan(c0);
  const int t0 = __builtin_amdgcn_readlane(i0, 63);
  const int i1 = kSpanTwoHalves ? wave_incl_scan(c1) : 0;
  tp->cum[l] = i0 - c0;
  if (kSpanTwoHalves) tp->cum[l + 64] = t0 + i1 - c1;
  if (l == 63) {
    const int total = t0 + i1;
    tp->cum[kSpanBlocks] = total;
    tp->ntiles = 0;
    tp->ndirect = 0;
    if (count_only) tp->row_out += total;   // the row's numeric class needs no tiles
  }
}

// Second part (wave 0): the tile records (direct and ranked tiles).
__device__ __forceinline__ void plan_tail(TilePlan* tp, int nb, int block0, int direct_min) {
  const int l = lane_id();
  const int c0 = l < nb ? tp->blk_cnt[l] : 0;
  const int c1 = (kSpanTwoHalves && l + 64 < nb) ? tp->blk_cnt[l + 64] : 0;
  const unsigned long long dm0 = __ballot(c0 >= direct_min), dm1 = __ballot(c1 >= direct_min);
  const unsigned long long nm0 = __ballot(c0 > 0), nm1 = __ballot(c1 > 0);
#pragma unroll
  for (int half = 0; half < (kSpanTwoHalves ? 2 : 1); ++half) {
    const int b = l + 64 * half;
    if (b < nb) {
      int lim = next_bit128(dm0, dm1, b);   // first direct block at or behind b
      if (lim > nb) lim = nb;
      const int base = tp->cum[b];
      int lo = b + 1, hi = lim;             // largest e in [b+1, lim] that fits
      while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if ((long long)(mid - b) * kRankBlkBytes + (long long)kRankEntryBytes * (tp->cum[mid] - base) <= kTileBudget) lo = mid; else hi = mid - 1;
      }
      tp->nxt[b] = lo;
    }
  }
  wave_sync();
  if (l == 0) {
    int n = 0, nd = 0, out = tp->row_out;
    int b = next_bit128(nm0, nm1, 0);
    while (b < nb) {
      const int cb = tp->blk_cnt[b];
      if (cb >= direct_min) {
        tp->rec[n++] = TileRec{block0 + b, block0 + b + 1, cb | kDirectBit, out};
        ++nd;
        out += cb;
        b = b + 1;
      } else {
        const int e = tp->nxt[b];
        const int c = tp->cum[e] - tp->cum[b];
        const int et = prev_bit128(nm0, nm1, e) + 1;   // drop empty blocks at the end
        tp->rec[n++] = TileRec{block0 + b, block0 + et, c, out};
        out += c;
        b = e;
      }
      b = next_bit128(nm0, nm1, b);
    }
    tp->ntiles = n;
    tp->ndirect = nd;
    tp->row_out = out;
  }
}

// Takes `amount` from a shared cursor if that stays within `cap` (compare and advance: the cursor never
// passes the capacity, so a request that does not fit costs later, smaller requests nothing).
__device__ __forceinline__ bool reserve_below(unsigned long long* cursor, unsigned long long amount, unsigned long long cap,
                                              unsigned long long& base) {
  unsigned long long cur = __hip_atomic_load(cursor, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  while (cur + amount <= cap) {
    const unsigned long long seen = atomicCAS(cursor, cur, cur + amount);
    if (seen == cur) { base = cur; return true; }
    cur = seen;
  }
  return false;
}

// Fetch the next row of the dense symbolic bins (4..6), heaviest class first; -1 when none is left.
__device__ __forceinline__ int next_dense_row(const int* __restrict__ perm, Control* ctl, int* s_row) {
  __syncthreads();
  if (threadIdx.x == 0) {
    const unsigned lo = ctl->offset[0][4], hi = ctl->offset[0][7];
    const unsigned idx = atomicAdd(&ctl->work[0], 1u);
    *s_row = idx < hi - lo ? perm[hi - 1 - idx] : -1;
  }
  __syncthreads();
  return *s_row;
}

__global__ __launch_bounds__(kDenseThreads) void k_sym_dense(const int* __restrict__ perm, Control* ctl,
                                                             const int64_t* __restrict__ a_rp, const int32_t* __restrict__ a_col,
                                                             const int64_t* __restrict__ b_rp, const int32_t* __restrict__ b_col,
                                                             int64_t n_cols, const int* __restrict__ ip, int* __restrict__ cnt,
                                                             TileRec* __restrict__ tiles, RunRec* __restrict__ runs,
                                                             int32_t* __restrict__ col_list, int direct_min, int no_tiles_ip,
                                                             int search_ratio, const int* __restrict__ bp, int nb1) {
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned* flags = reinterpret_cast<unsigned*>(smem);                               // kSymFlagWords
  RowScratch* rs = reinterpret_cast<RowScratch*>(smem + (size_t)kSymFlagWords * 4);
  TilePlan* tp = reinterpret_cast<TilePlan*>(smem + (size_t)kSymFlagWords * 4 + sizeof(RowScratch));
  if (ctl->error) return;
  const bool sorted = ctl->b_sorted != 0;
  const int64_t span = (int64_t)kSymFlagWords * 32;
  const int tid = threadIdx.x;
  const unsigned row_lo = ctl->offset[0][4], row_hi = ctl->offset[0][7];   // the dense bins, heaviest class last
  const unsigned tile_cap = ctl->tile_cap, run_cap = ctl->run_cap;
  const unsigned long long list_cap = ctl->list_cap;
  SPG_CLK(clk_begin(&rs->clk);)
  int row = next_dense_row(perm, ctl, &rs->s_row);
  int next_row = -1;   // (thread 0) the row after this one, fetched while this one is in the works
  // (thread 0) what is left of the slabs drawn from the plan's lists, and what this workgroup used
  unsigned long long sl_pos = 0, sl_left = 0;
  // (slabs of the list: together at most a quarter of it, so that a short list is not spent on slack)
  const unsigned long long list_slab = list_cap / (4ULL * gridDim.x) < (unsigned long long)kListSlab ? (list_cap / (4ULL * gridDim.x)) & ~3ULL : (unsigned long long)kListSlab;
  unsigned st_pos = 0, st_left = 0, sr_pos = 0, sr_left = 0, used_tiles = 0, used_runs = 0;
  while (row >= 0) {
    unsigned nx = 0;   // (thread 0) the draw for the row after this one: on its way while this row is in the works
    if (tid == 0) nx = atomicAdd(&ctl->work[0], 1u);
    const int64_t a0 = a_rp[row];
    const int d = (int)(a_rp[row + 1] - a0);
    if (tid == 0) tp->row_out = 0;
    SPG_CLK(clk_mark(&rs->clk, 0); clk_add(&rs->clk, 16, 1);)
    for (int64_t c0 = 0; c0 < n_cols; c0 += span) {
      const int64_t c1 = (c0 + span < n_cols) ? c0 + span : n_cols;
      const int words = (int)((c1 - c0 + 31) >> 5);
      const int nb = (int)((c1 - c0 + kBlkCols - 1) >> kBlkShift);
      {
        uint4* f4 = reinterpret_cast<uint4*>(flags);
        for (int w = tid; w < kSymFlagWords / 4; w += kDenseThreads) f4[w] = make_uint4(0, 0, 0, 0);
      }
      if (tid < kSpanBlocks) tp->blk_cnt[tid] = 0;
      if (tid == 0) { tp->span_out0 = tp->row_out; tp->list_base = -1; rs->span_ip = 0; }
      __syncthreads();
      SPG_CLK(clk_mark(&rs->clk, 1); clk_add(&rs->clk, 17, 1);)
      const int lo = (int)c0;
      const int64_t hi = c1;
      auto mark = [&](int c) {
        if (c >= lo && (int64_t)c < hi) atomicOr(&flags[(c - lo) >> 5], 1u << ((c - lo) & 31));
      };
      // a batch of columns: the flag words are read first (reads of one address are broadcast), and only bits
      // that are not set yet go through the atomic (hub columns are set early and hit by most pieces)
      auto mark_batch = [&](const int (&c)[kChunkUnroll]) {
        unsigned w[kChunkUnroll];
#pragma unroll
        for (int u = 0; u < kChunkUnroll; ++u) {
          const bool ok = c[u] >= lo && (int64_t)c[u] < hi;
          w[u] = flags[ok ? (c[u] - lo) >> 5 : 0];
        }
#pragma unroll
        for (int u = 0; u < kChunkUnroll; ++u) {
          const bool ok = c[u] >= lo && (int64_t)c[u] < hi;
          const unsigned bit = 1u << ((c[u] - lo) & 31);
          if (ok && !(w[u] & bit)) atomicOr(&flags[(c[u] - lo) >> 5], bit);
        }
      };
      if (n_cols > span && sorted && bp)
        stream_columns(a0, d, a_col, b_rp, b_col, rs, TableRange{bp, nb1, (int)(c0 >> kBlkShift), (int)((c1 + kBlkCols - 1) >> kBlkShift)}, mark, mark_batch);
      else if (n_cols > span && sorted)
        stream_columns(a0, d, a_col, b_rp, b_col, rs, SearchRange{b_col, lo, hi}, mark, mark_batch);
      else
        stream_columns(a0, d, a_col, b_rp, b_col, rs, NoRange{}, mark, mark_batch);
      // entries per block and per group: thread t owns kWordsPerThread consecutive flag words
      {
        constexpr int kWordsPerThread = kSymFlagWords / kDenseThreads;
        static_assert(kWordsPerThread % 4 == 0 && kGrpWords % kWordsPerThread == 0 && kBlkWords % kWordsPerThread == 0, "whole threads per group and block");
        constexpr int kThreadsPerGroup = kGrpWords / kWordsPerThread, kThreadsPerBlock = kBlkWords / kWordsPerThread;
        static_assert(kThreadsPerBlock <= kWave, "a block's threads sit in one wave");
        const uint4* f4 = reinterpret_cast<const uint4*>(flags) + tid * (kWordsPerThread / 4);
        int local = 0;
#pragma unroll
        for (int q = 0; q < kWordsPerThread / 4; ++q) {
          const uint4 v = f4[q];
          local += __popc(v.x) + __popc(v.y) + __popc(v.z) + __popc(v.w);
        }
#pragma unroll
        for (int sh = 1; sh < kThreadsPerGroup; sh <<= 1) local += __shfl_xor(local, sh, kWave);
        if (tid % kThreadsPerGroup == 0) tp->grp[tid / kThreadsPerGroup] = local;
#pragma unroll
        for (int sh = kThreadsPerGroup; sh < kThreadsPerBlock; sh <<= 1) local += __shfl_xor(local, sh, kWave);
        if (tid % kThreadsPerBlock == 0) tp->blk_cnt[tid / kThreadsPerBlock] = local;
      }
      __syncthreads();
      SPG_CLK(clk_mark(&rs->clk, 5);)
      const bool count_only = ip[row] <= no_tiles_ip;
      const bool last_span = c1 >= n_cols;
      const int block0 = (int)(c0 >> kBlkShift);
      if (tid < kWave) {
        plan_head(tp, nb, count_only);
        if (!count_only) plan_tail(tp, nb, block0, direct_min);
      }
      __syncthreads();
      SPG_CLK(clk_mark(&rs->clk, 6);)
      if (tid == 0) {
        // Everything this span needs from the plan's shared lists, and the next row, in one round trip:
        // room for the entries in the column list (without it the numeric kernel rebuilds the flags
        // itself), tile and run records.  A span that got room in the list and has at
        // most kSearchCap entries and at most search_ratio products per entry becomes one searched tile
        // (the records planned above stay unused).
        const int total = tp->cum[kSpanBlocks];
        const int nt = tp->ntiles;
        const int nr = (nt + kRunTiles - 1) / kRunTiles;
        const bool want_list = !count_only && total > 0 && list_cap > 0;
        // a short row with little deduplication becomes one searched tile and needs its columns; every
        // other row keeps its flag words as they are (no decoding here, and far less memory for rows
        // with many entries) unless they would take much more room than the columns
        // (products of the span: counted by the walk when it covered a part of the row)
        const long long span_products = (n_cols > span && sorted) ? (long long)rs->span_ip : (long long)ip[row];
        // (a searched tile takes every product of its pieces: with unordered B rows the pieces are whole rows,
        // so the tile must be the whole row)
        const bool search_row = (sorted || n_cols <= span) && total <= kSearchCap && nt > 1 && span_products <= (long long)search_ratio * total;
        const int fwords = (words + 3) & ~3;
        const bool as_words = !search_row && (long long)fwords * kFlagWordsNum <= (long long)kFlagWordsDen * total;
        const unsigned long long need = as_words ? (unsigned long long)(span_rank_slots(words) + fwords)
                                                 : (unsigned long long)((total + 3) & ~3);   // (16-byte granules)
        // The shares come out of slabs that the workgroup draws from the shared cursors now and then: a round
        // trip to a counter that every workgroup hits costs microseconds, a row needs its answer at once.
        unsigned long long at = 0;
        unsigned tb = 0, rb = 0;
        bool listed = false;
        if (want_list) {
          if (need <= sl_left) {
            at = sl_pos; sl_pos += need; sl_left -= need; listed = true;
          } else {   // (what is left of the old slab stays unused)
            const unsigned long long grab = need > list_slab ? need : list_slab;
            unsigned long long base;
            if (reserve_below(&ctl->list_cursor, grab, list_cap, base)) {
              at = base; sl_pos = base + need; sl_left = grab - need; listed = true;
            } else if (grab != need && reserve_below(&ctl->list_cursor, need, list_cap, base)) {
              at = base; listed = true;   // (no room for a slab, but for the row alone)
            }
          }
        }
        bool room = true;
        if (nt > 0) {
          if ((unsigned)nt > st_left) {
            st_pos = atomicAdd(&ctl->tile_cursor, (unsigned)kTileSlab);
            room = st_pos + (unsigned)kTileSlab <= tile_cap;
            st_left = room ? (unsigned)kTileSlab : 0u;
          }
          if (room && (unsigned)nr > sr_left) {
            for (unsigned i = 0; i < sr_left; ++i) runs[sr_pos + i].count = 0;   // (slots left behind: empty records)
            sr_pos = atomicAdd(&ctl->run_cursor, (unsigned)kRunSlab);
            room = sr_pos + (unsigned)kRunSlab <= run_cap;
            sr_left = room ? (unsigned)kRunSlab : 0u;
          }
          if (room) {
            tb = st_pos; st_pos += (unsigned)nt; st_left -= (unsigned)nt;
            rb = sr_pos; sr_pos += (unsigned)nr; sr_left -= (unsigned)nr;
          }
        }
        tp->list_base = listed ? (long long)at : -1;
        tp->list_words = listed && as_words ? fwords : 0;
        tp->tile_base = tb;
        tp->run_base = rb;
        tp->next_block = 0;
        tp->nruns = nr;
        if (nt > 0 && !room) {
          ctl->error = 3;   // cannot happen when the host sized the lists from the bound
          tp->ntiles = 0;
          tp->nruns = 0;
        } else if (listed && search_row) {
          // (a searched tile pays a bisection per product: only for rows with little deduplication, and
          // only where it saves tiles - a row that is one ranked or direct tile anyway stays that)
          tp->rec[0] = TileRec{block0, block0 + nb, total | kSearchBit, tp->span_out0};
          tp->ntiles = 1;
          atomicAdd(&ctl->search_tiles, 1u);
        } else if (tp->ndirect > 0) {
          atomicAdd(&ctl->direct_tiles, (unsigned)tp->ndirect);
        }
        used_tiles += (unsigned)tp->ntiles;
        used_runs += (unsigned)tp->nruns;
        if (last_span) next_row = nx < row_hi - row_lo ? perm[row_hi - 1 - nx] : -1;
      }
      __syncthreads();
      SPG_CLK(clk_mark(&rs->clk, 7);)
      const long long lb = tp->list_base;
      const int nt = tp->ntiles;
      if (nt > 0 || tp->nruns > 0) {
        if (tid < nt) tiles[tp->tile_base + tid] = tp->rec[tid];
        if (tid < tp->nruns) {   // (runs behind the tiles in use stay empty: count 0)
          const int left = nt - tid * kRunTiles;
          // (flag words: the position of the word of column 0, which may lie before the span's words)
          const long long lpos = lb < 0 ? -1LL : (tp->list_words ? (lb + kListBias) | kListFlagWords : lb - tp->span_out0 + kListBias);
          runs[tp->run_base + tid] = RunRec{row, tp->tile_base + (unsigned)(tid * kRunTiles), left < 0 ? 0 : (left < kRunTiles ? left : kRunTiles), d, a0, lpos};
        }
      }
      if (lb >= 0 && tp->list_words) {
        // the flag list leaves as it is (one coalesced copy), behind the rank of every group's first entry
        static_assert(kGrpWords * 4 == kBlkWords && kSpanGroups <= kDenseThreads, "four groups per block, a thread per group");
        const int nslots = span_rank_slots(words);
        if (tid < nslots) {
          int r = tp->span_out0 + tp->cum[(tid >> 2) < kSpanBlocks ? (tid >> 2) : kSpanBlocks];
          for (int g = tid & ~3; g < tid; ++g) r += tp->grp[g];
          col_list[lb + tid] = r;
        }
        const uint4* f4 = reinterpret_cast<const uint4*>(flags);
        uint4* o4 = reinterpret_cast<uint4*>(col_list + lb + nslots);
        const int n4 = tp->list_words >> 2;
        for (int w = tid; w < n4; w += kDenseThreads) o4[w] = f4[w];
      } else if (lb >= 0) {
        // The list position of a block's first entry is its entry prefix.  Sparse blocks: the columns are decoded, a round
        // with few entries is gathered in LDS first and leaves as one coalesced run.
        // Direct blocks: the numeric kernel wants the flag words themselves (their 256 words fit
        // in the space of the block's entries).
        const int wave = tid >> 6, lane = tid & 63;
        const bool searched = nt == 1 && (tp->rec[0].cnt & kSearchBit) != 0;
        int* wst = reinterpret_cast<int*>(rs) + wave * kListStage;   // the piece walker's scratch is free now
        // (blocks are handed out one at a time: their entry counts differ by orders of magnitude,
        // so a fixed share per wave would leave most waves waiting for the one with the dense blocks)
        while (true) {
          int blk = 0;
          if (lane == 0) blk = atomicAdd(&tp->next_block, 1);
          blk = __builtin_amdgcn_readfirstlane(blk);
          if (blk >= nb) break;
          const int cb = tp->blk_cnt[blk];
          if (cb == 0) continue;
          int running = tp->cum[blk];
          if (cb >= direct_min && !searched) {
#pragma unroll
            for (int q = 0; q < kBlkWords; q += kWave) col_list[lb + running + q + lane] = (int)flags[blk * kBlkWords + q + lane];
            continue;
          }
          if (cb <= kListStage) {
            // a sparse block in one round: lane l decodes words 4 l .. 4 l + 3
            const uint4 v = reinterpret_cast<const uint4*>(flags)[blk * (kBlkWords / 4) + lane];
            const int c = __popc(v.x) + __popc(v.y) + __popc(v.z) + __popc(v.w);
            int excl = wave_incl_scan(c) - c;
            const int cbase = lo + (blk * kBlkWords + lane * 4) * 32;
            if (c) {
              unsigned wd[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
              for (int k = 0; k < 4; ++k) {
                unsigned bits = wd[k];
                while (bits) {
                  const int b = __ffs((int)bits) - 1;
                  bits &= bits - 1;
                  wst[excl++] = cbase + k * 32 + b;
                }
              }
            }
            wave_sync_lds();
            for (int j = lane; j < cb; j += kWave) col_list[lb + running + j] = wst[j];
            wave_sync_lds();
            continue;
          }
          for (int q = 0; q < kBlkWords; q += kWave) {
            const int w = blk * kBlkWords + q + lane;
            unsigned bits = flags[w];
            const int c = __popc(bits);
            const int incl = wave_incl_scan(c);
            const int tot = __builtin_amdgcn_readlane(incl, kWave - 1);
            if (tot == 0) continue;
            int excl = incl - c;
            const int cbase = lo + w * 32;
            if (tot <= kListStage) {
              while (bits) {
                const int b = __ffs((int)bits) - 1;
                bits &= bits - 1;
                wst[excl++] = cbase + b;
              }
              wave_sync_lds();
              for (int j = lane; j < tot; j += kWave) col_list[lb + running + j] = wst[j];
              wave_sync_lds();   // (the stores themselves need not have left before the next round)
            } else {
              while (bits) {
                const int b = __ffs((int)bits) - 1;
                bits &= bits - 1;
                col_list[lb + running + excl++] = cbase + b;
              }
            }
            running += tot;
          }
        }
      }
      __syncthreads();
      SPG_CLK(clk_mark(&rs->clk, 8);)
    }
    if (tid == 0) {
      cnt[row] = tp->row_out;
      rs->s_row = next_row;
    }
    __syncthreads();
    row = rs->s_row;
  }
  if (tid == 0) {
    for (unsigned i = 0; i < sr_left; ++i) runs[sr_pos + i].count = 0;
    if (used_tiles) atomicAdd(&ctl->tiles_used, used_tiles);
    if (used_runs) atomicAdd(&ctl->runs_used, used_runs);
  }
  SPG_CLK(clk_mark(&rs->clk, 9); clk_flush(&rs->clk, ctl->clk[0]);)
}

constexpr size_t kSymDenseLds = (size_t)kSymFlagWords * 4 + sizeof(RowScratch) + sizeof(TilePlan);

// ---- numeric --------------------------------------------------------------------------

// LDS behind the tile area of the numeric kernel.
template <typename T>
struct NumScratch {
  long long c_s[kSegCap];      // first B entry of every non-empty piece of the tile
  int c_cpre[kSegCap + 1];     // exclusive prefix of the pieces' chunk counts
  int c_len[kSegCap];          // piece length
  T c_av[kSegCap];             // a_ik of the piece
  TileRec rec[kRunTiles];
  RunRec rr;                   // the run in the works
  int red[2 * kDenseWaves];
  int s_run;
  int pad;
  SPG_CLK(ClkLds clk;)
};

// The piece [s, s + len) of B row k that falls into the tile (blocks [b0, b1), columns [t_lo, t_hi)).
__device__ __forceinline__ void piece_range(int k, long long rs, long long re, int b0, int b1, int t_lo, int64_t t_hi, bool sorted,
                                            const int* __restrict__ bp, int nb1, const int32_t* __restrict__ b_col,
                                            long long& s, int& len) {
  if (sorted && bp) {
    const int* row = bp + (int64_t)k * nb1;
    const int o0 = row[b0], o1 = row[b1];
    s = rs + o0;
    len = o1 - o0;
  } else {
    int64_t st = rs, en = re;
    if (sorted) SearchRange{b_col, t_lo, t_hi}(k, st, en);
    s = st;
    len = (int)(en - st);
  }
}

// Compacts the non-empty pieces of the workgroup's threads into c_s / c_cpre / c_len / c_av.
// Returns their number and the chunk total.  Contains barriers.
template <typename T>
__device__ __forceinline__ void tile_pieces(NumScratch<T>* ns, long long s, int len, T av, int& np, int& nchunks) {
  int idx, cpre;
  block_excl_scan2(len > 0 ? 1 : 0, (len + kWave - 1) >> 6, idx, cpre, np, nchunks, ns->red);
  if (len > 0) {
    ns->c_s[idx] = s;
    ns->c_cpre[idx] = cpre;
    ns->c_len[idx] = len;
    ns->c_av[idx] = av;
  }
  if (threadIdx.x == 0) ns->c_cpre[np] = nchunks;
  __syncthreads();
  SPG_CLK(clk_add(&ns->clk, 20, (unsigned long long)nchunks); clk_add(&ns->clk, 21, (unsigned long long)np);)
}

template <typename T, bool CHECK>
__device__ __forceinline__ void num_dense_run(const RunRec rr, NumScratch<T>* ns, unsigned char* tile, bool sorted,
                                              const int32_t* __restrict__ a_col, const T* __restrict__ a_val,
                                              const int64_t* __restrict__ b_rp, const int32_t* __restrict__ b_col,
                                              const T* __restrict__ b_val, int64_t n_cols, const int* __restrict__ bp, int nb1,
                                              const int32_t* __restrict__ col_list,
                                              int64_t out_row, int32_t* __restrict__ c_col, T* __restrict__ c_val,
                                              const int (&pre_k)[kRegSegs], const T (&pre_av)[kRegSegs]) {
  const int tid = threadIdx.x;
  // the row's structure in the plan: none, its columns, or its flag words
  const bool have_words = rr.list >= 0 && (rr.list & kListFlagWords) != 0;
  const bool have_list = rr.list >= 0 && !have_words;
  const long long list_at = (rr.list & (kListFlagWords - 1)) - kListBias;   // entry 0 of the row, or the span's kept structure
  const int64_t a0 = rr.a0;
  const int d = rr.d;
  const int nseg = (d + kSegCap - 1) / kSegCap;
  // with few segments, thread e keeps its A entry of every segment in registers for the whole
  // run, together with the block offsets of the coming tile inside the entry's B row (fetched
  // while the current tile is in the works)
  const bool use_table = sorted && bp != nullptr;
  const bool cached = nseg == 1 || (use_table && nseg <= kRegSegs);
  int ck[kRegSegs], pf0[kRegSegs], pf1[kRegSegs];
  long long crs[kRegSegs];
  T cav[kRegSegs];
  long long my_re = 0;
#pragma unroll
  for (int g = 0; g < kRegSegs; ++g) {
    ck[g] = 0; pf0[g] = 0; pf1[g] = 0; crs[g] = 0; cav[g] = T(0);
    const int e = g * kSegCap + tid;
    if (cached && e < d) {
      ck[g] = pre_k[g];     // (fetched by the caller together with the run's tile records)
      cav[g] = pre_av[g];
      crs[g] = b_rp[ck[g]];
      if (!use_table) my_re = b_rp[ck[g] + 1];
      if (use_table) {
        const TileRec nx = ns->rec[0];
        const int* row = bp + (int64_t)ck[g] * nb1;
        pf0[g] = row[nx.b0];
        pf1[g] = row[nx.b1];
      }
    }
  }
  SPG_CLK(clk_mark(&ns->clk, 1);)
  for (int t = 0; t < rr.count; ++t) {
    const TileRec tr = ns->rec[t];
    const bool direct = (tr.cnt & kDirectBit) != 0;
    const bool searched = (tr.cnt & kSearchBit) != 0;
    const int count = tr.cnt & kCountMask;
    const int t_lo = tr.b0 << kBlkShift;
    int64_t t_hi = (int64_t)tr.b1 << kBlkShift;
    if (t_hi > n_cols) t_hi = n_cols;
    const int64_t out = out_row + tr.out;
    // kept flag words of the tile's span: group ranks first, then the words (indexed here by absolute word)
    const int64_t span_c0 = (int64_t)(tr.b0 / kSpanBlocks) * kSpanBlocks * kBlkCols;
    const int32_t* kept_ranks = col_list + list_at;
    const int32_t* kept_words = col_list + list_at + span_rank_slots(span_flag_words(n_cols, span_c0)) - (span_c0 >> 5);
    // this thread's pieces of the tile, one per cached segment
    int off_c[kRegSegs], len_c[kRegSegs];
#pragma unroll
    for (int g = 0; g < kRegSegs; ++g) {
      off_c[g] = 0; len_c[g] = 0;
      const int e = g * kSegCap + tid;
      if (cached && e < d) {
        if (use_table) {
          off_c[g] = pf0[g];
          len_c[g] = pf1[g] - pf0[g];
          if (t + 1 < rr.count) {
            const TileRec nx = ns->rec[t + 1];
            const int* row = bp + (int64_t)ck[g] * nb1;
            pf0[g] = nx.b0 == tr.b1 ? pf1[g] : row[nx.b0];
            pf1[g] = row[nx.b1];
          }
        } else {   // one segment, no table
          long long ps;
          piece_range(ck[g], crs[g], my_re, tr.b0, tr.b1, t_lo, t_hi, sorted, bp, nb1, b_col, ps, len_c[g]);
          off_c[g] = (int)(ps - crs[g]);
        }
      }
    }
    // piece of segment sg for this thread
    auto seg_piece = [&](int sg, long long& ps, int& plen, T& pav) {
      if (cached) {
        static_assert(kRegSegs == 2, "the selects below cover two segments");
        const int o = sg == 0 ? off_c[0] : off_c[1];
        plen = sg == 0 ? len_c[0] : len_c[1];
        ps = (sg == 0 ? crs[0] : crs[1]) + o;
        pav = sg == 0 ? cav[0] : cav[1];
        return;
      }
      ps = 0; plen = 0; pav = T(0);
      const int e = sg * kSegCap + tid;
      if (e < d && e < (sg + 1) * kSegCap) {
        const int k = a_col[a0 + e];
        pav = a_val[a0 + e];
        piece_range(k, b_rp[k], b_rp[k + 1], tr.b0, tr.b1, t_lo, t_hi, sorted, bp, nb1, b_col, ps, plen);
      }
    };
    long long s = 0;
    int len = 0;
    T my_av = T(0);
    if (nseg == 1) seg_piece(0, s, len, my_av);
    __syncthreads();   // the previous tile's output has left the tile area
    SPG_CLK(clk_mark(&ns->clk, 2); clk_add(&ns->clk, 22, (unsigned long long)count);)
    if (searched) {
      // the tile's columns (from the plan's list) and their sums, by rank; a product finds the rank of
      // its column by bisection, so the tile may be as wide as the matrix
      int* cols = reinterpret_cast<int*>(tile);
      double* acc = reinterpret_cast<double*>(tile + (((size_t)count * 4 + 7) & ~(size_t)7));
      const int32_t* lst = col_list + list_at + tr.out;
      for (int j0 = 0; j0 < count; j0 += kListBatch * kDenseThreads) {
        int lc[kListBatch];
#pragma unroll
        for (int i = 0; i < kListBatch; ++i) {
          const int j = j0 + i * kDenseThreads + tid;
          lc[i] = j < count ? stream_load(&lst[j]) : -1;
        }
#pragma unroll
        for (int i = 0; i < kListBatch; ++i) {
          const int j = j0 + i * kDenseThreads + tid;
          if (j < count) {
            cols[j] = lc[i];
            acc[j] = 0.0;
            stream_store(&c_col[out + j], lc[i]);
          }
        }
      }
      SPG_CLK(clk_mark(&ns->clk, 10); clk_add(&ns->clk, 19, 1);)
      int top = 1;   // largest power of two below count
      while (top * 2 < count) top *= 2;
      for (int sg = 0; sg < nseg; ++sg) {
        T av = my_av;
        if (nseg > 1) seg_piece(sg, s, len, av);
        int np, nchunks;
        tile_pieces(ns, s, len, av, np, nchunks);   // (its barriers also publish cols and the cleared sums)
        chunk_pass_batches<true, T>(np, nchunks, PieceList<T>{ns->c_s, ns->c_cpre, ns->c_len, ns->c_av}, b_col, b_val,
                                    [&](const int (&c)[kChunkUnroll], const T (&a)[kChunkUnroll], const T (&b)[kChunkUnroll]) {
          // last position whose column is <= c (the column is in the list); four bisections
          // advance in lockstep so that their LDS reads overlap
#pragma unroll
          for (int u0 = 0; u0 < kChunkUnroll; u0 += 4) {
            int lo[4] = {0, 0, 0, 0};
            for (int step = top; step > 0; step >>= 1) {
#pragma unroll
              for (int u = 0; u < 4; ++u) {
                const int mid = lo[u] + step;
                if (mid < count && cols[mid < count ? mid : 0] <= c[u0 + u]) lo[u] = mid;
              }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
              if (c[u0 + u] >= 0)
                __hip_atomic_fetch_add(&acc[lo[u]], (double)a[u0 + u] * (double)b[u0 + u], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
          }
        });
        if (nseg > 1) __syncthreads();
      }
      __syncthreads();
      SPG_CLK(clk_mark(&ns->clk, 11);)
      for (int r = tid; r < count; r += kDenseThreads) stream_store(&c_val[out + r], (T)acc[r]);
      SPG_CLK(clk_mark(&ns->clk, 12);)
    } else if (direct) {
      double* acc = reinterpret_cast<double*>(tile);                      // kBlkCols sums, indexed by column
      int* stage = reinterpret_cast<int*>(tile + (size_t)kBlkCols * 8);   // kBlkCols columns, by rank
      unsigned* flags = reinterpret_cast<unsigned*>(tile + (size_t)kBlkCols * 12);   // kBlkCols / 32
      {
        double2* a2 = reinterpret_cast<double2*>(acc);
        for (int r = tid; r < kBlkCols / 2; r += kDenseThreads) a2[r] = make_double2(0.0, 0.0);
      }
      // which columns exist: the flag words are in the plan's list, or are rebuilt by the pass
      if (tid < kBlkCols / 32)   // (the last block of the matrix may be cut short: no flag words are kept behind its end)
        flags[tid] = have_words ? (tid < (int)((t_hi - t_lo + 31) >> 5) ? (unsigned)kept_words[(long long)tr.b0 * kBlkWords + tid] : 0u)
                                : (have_list ? (unsigned)col_list[list_at + tr.out + tid] : 0u);
      SPG_CLK(clk_add(&ns->clk, 18, 1);)
      for (int sg = 0; sg < nseg; ++sg) {
        T av = my_av;
        if (nseg > 1) seg_piece(sg, s, len, av);
        int np, nchunks;
        tile_pieces(ns, s, len, av, np, nchunks);
        SPG_CLK(clk_mark(&ns->clk, 7);)
        chunk_pass<true, T>(np, nchunks, PieceList<T>{ns->c_s, ns->c_cpre, ns->c_len, ns->c_av}, b_col, b_val, [&](int c, T a, T b) {
          if (!CHECK || (c >= t_lo && (int64_t)c < t_hi)) {
            const int rel = c - t_lo;
            if (!have_list && !have_words) atomicOr(&flags[rel >> 5], 1u << (rel & 31));
            __hip_atomic_fetch_add(&acc[rel], (double)a * (double)b, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
          }
        });
        if (nseg > 1) __syncthreads();
      }
      __syncthreads();
      SPG_CLK(clk_mark(&ns->clk, 8);)
      // compress: thread t owns columns [8 t, 8 t + 8)
      const unsigned byte = (flags[tid >> 2] >> ((tid & 3) * 8)) & 255u;
      double v[8];
      {
        const double2* a2 = reinterpret_cast<const double2*>(acc) + tid * 4;
#pragma unroll
        for (int i = 0; i < 4; ++i) { const double2 x = a2[i]; v[2 * i] = x.x; v[2 * i + 1] = x.y; }
      }
      int base, dummy_e, tot, dummy_t;
      block_excl_scan2(__popc(byte), 0, base, dummy_e, tot, dummy_t, ns->red);   // barriers: every sum has been read
      (void)tot;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        if (byte & (1u << i)) {
          acc[base] = v[i];
          stage[base] = t_lo + tid * 8 + i;
          ++base;
        }
      }
      __syncthreads();
      for (int r = tid; r < count; r += kDenseThreads) {
        stream_store(&c_val[out + r], (T)acc[r]);
        stream_store(&c_col[out + r], stage[r]);
      }
      SPG_CLK(clk_mark(&ns->clk, 9);)
    } else {
      const int nw = (tr.b1 - tr.b0) * (kBlkCols / 32);                   // 32-bit flag words
      uint2* fc = reinterpret_cast<uint2*>(tile);                         // per word: .x flag bits, .y rank of its first column
      double* acc = reinterpret_cast<double*>(tile + (size_t)nw * 8);     // count sums, by rank
      // with a column list: the first batch of its entries is on its way while the workspace is set up
      const int32_t* lst = col_list + (have_list ? list_at + tr.out : 0);
      int lc[kListBatch], lp[kListBatch];   // kListBatch loads in flight per thread
      auto fetch_list = [&](int j0) {
#pragma unroll
        for (int i = 0; i < kListBatch; ++i) {
          const int j = j0 + i * kDenseThreads + tid;
          lc[i] = j < count ? stream_load(&lst[j]) : -1;
          lp[i] = ((tid & 63) == 0 && j > 0 && j < count) ? lst[j - 1] : -1;   // left neighbour of the wave's first entry
        }
      };
      if (have_list) fetch_list(0);
      int np = 0, nchunks = 0;
      int* stage = reinterpret_cast<int*>(acc);   // columns by rank, in the space of the sums, on their way to C
      if (!have_words)
        for (int w = tid; w < nw; w += kDenseThreads) fc[w] = make_uint2(0u, 0u);
      if (have_list) {
        // the symbolic phase left the tile's columns (ascending) in the plan: flag bits and ranks
        // come from that list, and the list is this tile's run of C's column indices
        for (int r = tid; r < count; r += kDenseThreads) acc[r] = 0.0;
        if (nseg == 1) tile_pieces(ns, s, len, my_av, np, nchunks); else __syncthreads();
        SPG_CLK(clk_mark(&ns->clk, 3); clk_add(&ns->clk, 17, 1);)
        for (int j0 = 0; j0 < count; j0 += kListBatch * kDenseThreads) {
          if (j0 > 0) fetch_list(j0);
#pragma unroll
          for (int i = 0; i < kListBatch; ++i) {
            const int j = j0 + i * kDenseThreads + tid;
            const int c = lc[i];
            int prev = __shfl_up(c, 1, kWave);
            if ((tid & 63) == 0) prev = lp[i];
            if (c >= 0) {
              const int rel = c - t_lo;
              flags_or_combined(rel >> 5, 1u << (rel & 31), [&](int w) { return &fc[w].x; });
              if (prev < 0 || ((prev - t_lo) >> 5) != (rel >> 5)) fc[rel >> 5].y = (unsigned)j;
              stream_store(&c_col[out + j], c);
            }
          }
        }
        __syncthreads();
        SPG_CLK(clk_mark(&ns->clk, 4);)
      } else if (have_words) {
        // the symbolic phase left the span's flag words in the plan, with the rank of the first entry of
        // every group of kGrpWords words: groups are dealt to the waves in turn (entries thin out with the
        // column, so neighbouring groups cost about the same), a lane takes a word, ranks follow from one
        // scan over the wave, and the columns are decoded ("boolean indexing") by rank into LDS
        const int wave = tid >> 6, lane = tid & 63;
        const int ngrp = nw / kGrpWords;
        const int nw_kept = (int)((t_hi - t_lo + 31) >> 5);   // (the last block of the matrix may be cut short)
        const int32_t* tw = kept_words + (long long)tr.b0 * kBlkWords;
        const int32_t* tr_ranks = kept_ranks + (int)((t_lo - span_c0) >> 5) / kGrpWords;
        constexpr int kGrpBatch = 4;
        int wd[kGrpBatch], rk[kGrpBatch];
        auto fetch_groups = [&](int g0) {
#pragma unroll
          for (int i = 0; i < kGrpBatch; ++i) {
            const int g = g0 + i * kDenseWaves;
            const int w = g * kGrpWords + lane;
            wd[i] = (g < ngrp && w < nw_kept) ? stream_load(&tw[w]) : 0;
            rk[i] = g < ngrp ? tr_ranks[g] : 0;
          }
        };
        fetch_groups(wave);
        for (int g0 = wave; g0 < ngrp; g0 += kDenseWaves * kGrpBatch) {
          int cw[kGrpBatch], cr[kGrpBatch];
#pragma unroll
          for (int i = 0; i < kGrpBatch; ++i) { cw[i] = wd[i]; cr[i] = rk[i]; }
          if (g0 + kDenseWaves * kGrpBatch < ngrp) fetch_groups(g0 + kDenseWaves * kGrpBatch);   // the next batch, while this one is decoded
#pragma unroll
          for (int i = 0; i < kGrpBatch; ++i) {
            const int g = g0 + i * kDenseWaves;
            if (g < ngrp) {
              const int w = g * kGrpWords + lane;
              unsigned bits = (unsigned)cw[i];
              const int c = __popc(bits);
              int excl = cr[i] - tr.out + wave_incl_scan(c) - c;   // rank inside the tile
              fc[w] = make_uint2(bits, (unsigned)excl);
              const int cbase = t_lo + w * 32;
              while (bits) {
                const int b = __ffs((int)bits) - 1;
                bits &= bits - 1;
                stage[excl++] = cbase + b;
              }
            }
          }
        }
        __syncthreads();
        for (int r = tid; r < count; r += kDenseThreads) stream_store(&c_col[out + r], stage[r]);
        __syncthreads();
        for (int r = tid; r < count; r += kDenseThreads) acc[r] = 0.0;
        if (nseg == 1) tile_pieces(ns, s, len, my_av, np, nchunks); else __syncthreads();
        SPG_CLK(clk_mark(&ns->clk, 15); clk_add(&ns->clk, 17, 1);)
      } else {
      // pass 1: which columns of the tile exist in the row
      for (int sg = 0; sg < nseg; ++sg) {
        T av = my_av;
        if (nseg > 1) seg_piece(sg, s, len, av);
        tile_pieces(ns, s, len, av, np, nchunks);
        chunk_pass<false, T>(np, nchunks, PieceList<T>{ns->c_s, ns->c_cpre, ns->c_len, ns->c_av}, b_col, b_val, [&](int c, T, T) {
          if (!CHECK || (c >= t_lo && (int64_t)c < t_hi)) {
            const int rel = c - t_lo;
            atomicOr(&fc[rel >> 5].x, 1u << (rel & 31));
          }
        });
        if (nseg > 1) __syncthreads();
      }
      // exclusive prefix of the flag-word populations: every wave owns a contiguous share of
      // the words and walks it 64 words at a time (lane = word, so LDS reads do not collide);
      // the columns are decoded from the flag words into the space of the sums, by rank, and
      // leave from there as one coalesced run of C's column indices
      const int wave = tid >> 6, lane = tid & 63;
      const int wper = ((nw + kDenseThreads - 1) / kDenseThreads) * kWave;
      const int wbase = wave * wper;
      __syncthreads();
      int mine = 0;
      for (int i = lane; i < wper; i += kWave) {
        const int w = wbase + i;
        if (w < nw) mine += __popc(fc[w].x);
      }
      mine = wave_sum(mine);
      if (lane == 0) ns->red[wave] = mine;
      __syncthreads();
      int running = 0;
#pragma unroll
      for (int w = 0; w < kDenseWaves; ++w) running += w < wave ? ns->red[w] : 0;
      for (int i0 = 0; i0 < wper; i0 += kWave) {
        const int w = wbase + i0 + lane;
        unsigned bits = w < nw ? fc[w].x : 0u;
        const int c = __popc(bits);
        const int incl = wave_incl_scan(c);
        int excl = running + incl - c;
        running += __builtin_amdgcn_readlane(incl, kWave - 1);
        if (w < nw) fc[w].y = (unsigned)excl;
        const int cbase = t_lo + w * 32;
        while (bits) {
          const int b = __ffs((int)bits) - 1;
          bits &= bits - 1;
          stage[excl++] = cbase + b;
        }
      }
      __syncthreads();
      for (int r = tid; r < count; r += kDenseThreads) stream_store(&c_col[out + r], stage[r]);
      __syncthreads();
      for (int r = tid; r < count; r += kDenseThreads) acc[r] = 0.0;
      __syncthreads();
      SPG_CLK(clk_mark(&ns->clk, 13);)
      }
      // pass 2: accumulate a_ik * b_kj at the rank of column j
      for (int sg = 0; sg < nseg; ++sg) {
        if (nseg > 1) {
          T av;
          seg_piece(sg, s, len, av);
          tile_pieces(ns, s, len, av, np, nchunks);
        }
        auto add = [&](int c, T a, T b) {
          if (!CHECK || (c >= t_lo && (int64_t)c < t_hi)) {
            const int rel = c - t_lo;
            const uint2 w = fc[rel >> 5];
            const int rank = (int)w.y + __popc(w.x & ((1u << (rel & 31)) - 1u));
            __hip_atomic_fetch_add(&acc[rank], (double)a * (double)b, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
          }
        };
        chunk_pass<true, T>(np, nchunks, PieceList<T>{ns->c_s, ns->c_cpre, ns->c_len, ns->c_av}, b_col, b_val, add);
        if (nseg > 1) __syncthreads();
      }
      __syncthreads();
      SPG_CLK(clk_mark(&ns->clk, 5);)
      // compress: sums and columns are already in ascending column order
      for (int r = tid; r < count; r += kDenseThreads) stream_store(&c_val[out + r], (T)acc[r]);
      SPG_CLK(clk_mark(&ns->clk, 6);)
    }
  }
}

template <typename T>
__global__ __launch_bounds__(kDenseThreads) void k_num_dense(Control* ctl, const unsigned char* __restrict__ numbin,
                                                             const TileRec* __restrict__ tiles, const RunRec* __restrict__ runs,
                                                             const int32_t* __restrict__ a_col,
                                                             const T* __restrict__ a_val, const int64_t* __restrict__ b_rp,
                                                             const int32_t* __restrict__ b_col, const T* __restrict__ b_val,
                                                             int64_t n_cols, const int* __restrict__ bp, int nb1,
                                                             const int32_t* __restrict__ col_list,
                                                             const int64_t* __restrict__ c_rp,
                                                             int32_t* __restrict__ c_col, T* __restrict__ c_val) {
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* tile = smem;                                                         // kTileBudget bytes
  NumScratch<T>* ns = reinterpret_cast<NumScratch<T>*>(smem + kTileBudget);
  if (ctl->error) return;
  const bool sorted = ctl->b_sorted != 0;
  const int tid = threadIdx.x;
  const unsigned nruns = ctl->run_cursor;
  // Thread 0 draws runs ahead of their use: the counter value for the run after next and the record
  // of the next run are on their way while the current run is in the works.
  unsigned drawn = 0;
  RunRec coming{};
  bool have_coming = false;
  SPG_CLK(clk_begin(&ns->clk);)
  if (tid == 0) {
    const unsigned first = atomicAdd(&ctl->work[1], 1u);
    drawn = atomicAdd(&ctl->work[1], 1u);
    have_coming = first < nruns;
    if (have_coming) coming = runs[first];
  }
  while (true) {
    __syncthreads();
    if (tid == 0) {
      ns->s_run = have_coming ? 1 : -1;
      if (have_coming) ns->rr = coming;
      have_coming = drawn < nruns;
      if (have_coming) {
        coming = runs[drawn];
        drawn = atomicAdd(&ctl->work[1], 1u);
      }
    }
    __syncthreads();
    if (ns->s_run < 0) break;
    const RunRec rr = ns->rr;
    if (rr.count == 0) continue;   // a record that its row did not need
    // one round trip: the row's class and position in C, the run's tile records, its A entries
    const int cls = numbin[rr.row];
    const int64_t out_row = c_rp[rr.row];
    if (tid < rr.count) ns->rec[tid] = tiles[rr.first + tid];
    int pre_k[kRegSegs];
    T pre_av[kRegSegs];
#pragma unroll
    for (int g = 0; g < kRegSegs; ++g) {
      pre_k[g] = 0; pre_av[g] = T(0);
      const int e = g * kSegCap + tid;
      if (e < rr.d && rr.d <= kRegSegs * kSegCap) {
        pre_k[g] = a_col[rr.a0 + e];
        pre_av[g] = a_val[rr.a0 + e];
      }
    }
    if (cls < 5 || cls > 6) continue;   // the row's numeric class is not this kernel's
    __syncthreads();
    SPG_CLK(clk_mark(&ns->clk, 0); clk_add(&ns->clk, 16, 1);)
    if (sorted)
      num_dense_run<T, false>(rr, ns, tile, true, a_col, a_val, b_rp, b_col, b_val, n_cols, bp, nb1, col_list, out_row, c_col, c_val, pre_k, pre_av);
    else
      num_dense_run<T, true>(rr, ns, tile, false, a_col, a_val, b_rp, b_col, b_val, n_cols, bp, nb1, col_list, out_row, c_col, c_val, pre_k, pre_av);
  }
  SPG_CLK(clk_mark(&ns->clk, 14); clk_flush(&ns->clk, ctl->clk[1]);)
}

template <typename T>
constexpr size_t num_dense_lds() { return (size_t)kTileBudget + sizeof(NumScratch<T>); }

}  // namespace spg
