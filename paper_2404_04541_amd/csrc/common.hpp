// Shared device helpers for the gfx950 SpGEMM kernels (wave64 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace spg {

constexpr int kWave = 64;
constexpr int kNumBins = 8;       // bins 0..6 hold work, bin 7 = rows with nothing to do
constexpr int kEmptyBin = 7;
constexpr int kEmptyKey = -1;     // hash-slot sentinel (column indices are >= 0)
constexpr int kPadKey = 0x7fffffff;  // sorts behind every real column

// Row classes.  Symbolic classes depend on the row's intermediate-product count ip
// (an upper bound of its output size); numeric classes on ip and the exact output size.
constexpr int kEscSmallCap = 32;     // bin 0: sorted-list workspace, 16 lanes per row
constexpr int kEscLargeCap = 128;    // bin 1: sorted-list workspace, one wave per row
constexpr int kSymHashSmall = 768;   // bin 2: hash set with 1024 slots, one wave per row
constexpr int kSymHashLarge = 1536;  // bin 3: hash set with 4096 slots, 256 threads per row
constexpr int kNumHashSmall = 192;   // bin 2: hash table with 256 slots, one wave per row
constexpr int kNumHashLarge = 1536;  // bin 3: hash table with 2048 slots, 256 threads per row
constexpr int64_t kDenseMid = 65536;     // bins 4/5/6: dense workspace, split by ip so that
constexpr int64_t kDenseBig = 1048576;   // the heaviest rows are scheduled first
// A row is in a dense numeric bin only if it was in a dense symbolic bin (cnt <= ip), so the
// tile list that the dense symbolic kernel plans exists for every row the dense numeric kernel sees.
static_assert(kSymHashLarge <= kNumHashLarge, "dense numeric rows need a dense symbolic pass");

// Control block shared by host and device (one small device allocation per plan).
struct Control {
  unsigned hist[2][kNumBins];     // [0] symbolic, [1] numeric: rows per bin
  unsigned offset[2][kNumBins + 1];
  unsigned cursor[2][kNumBins];
  unsigned work[4];               // dynamic work counters: [0] dense symbolic rows, [1] dense numeric runs, [2] staged rows, [3] chunks of the row count
  unsigned tile_cursor, run_cursor;   // tile / run records written by the dense symbolic kernel
  unsigned tile_cap, run_cap;         // capacity of the two lists (set by the host)
  unsigned tiles_used, runs_used;     // records in use (the cursors also count what is left of the workgroups' slabs)
  unsigned direct_tiles;              // how many of the tiles are direct
  unsigned search_tiles;              // how many are searched tiles
  unsigned long long list_cursor, list_cap;   // entries used / available in the plan's column list
  int error;                      // nonzero: a device-side input check failed
  int b_sorted;                   // 1 when every B row is strictly ascending
  int long_b_row;                 // 1 when some B row has 2^21 or more entries
  unsigned long long desc_flat, desc_bnd;  // descent counts behind b_sorted
  unsigned long long ip_total;
  unsigned long long bin_ip[2][kNumBins];   // intermediate products per bin
  unsigned long long bin_nnz[kNumBins];     // output entries per numeric bin
  long long nnz_c;
  long long scan_blocks;
#ifdef SPG_PHASE_CLOCKS
  unsigned long long clk[2][32];   // [0] dense symbolic, [1] dense numeric: shader clocks per phase, summed over workgroups
#endif
};

// Optional phase clocks of the two dense kernels (a build with -DSPG_PHASE_CLOCKS; the product is
// built without): thread 0 of a workgroup reads the shader clock at phase boundaries and adds the
// differences up in LDS; at the end of the kernel the sums go to the control block.  Nothing is
// skipped or reordered, the marks only add a scalar clock read and one LDS update each.
#ifdef SPG_PHASE_CLOCKS
constexpr int kClkSlots = 32;
struct ClkLds { unsigned long long t, acc[kClkSlots]; };
__device__ __forceinline__ void clk_begin(ClkLds* c) {
  if (threadIdx.x == 0) { for (int i = 0; i < kClkSlots; ++i) c->acc[i] = 0; c->t = __builtin_readcyclecounter(); }
}
__device__ __forceinline__ void clk_mark(ClkLds* c, int slot) {
  if (threadIdx.x == 0) { const unsigned long long n = __builtin_readcyclecounter(); c->acc[slot] += n - c->t; c->t = n; }
}
__device__ __forceinline__ void clk_add(ClkLds* c, int slot, unsigned long long v) { if (threadIdx.x == 0) c->acc[slot] += v; }
__device__ __forceinline__ void clk_flush(ClkLds* c, unsigned long long* out) {
  if (threadIdx.x == 0) for (int i = 0; i < kClkSlots; ++i) if (c->acc[i]) atomicAdd(&out[i], c->acc[i]);
}
#define SPG_CLK(...) __VA_ARGS__
#else
#define SPG_CLK(...)
#endif

// A few consecutive elements behind a pointer that is only element-aligned, fetched by one load
// instruction: a gather costs the memory pipeline one pass per cache line and instruction, so a lane
// that wants neighbouring elements should ask for them together.
template <typename E, int N>
struct __attribute__((packed, aligned(sizeof(E)))) Run { E v[N]; };

template <typename E, int N>
__device__ __forceinline__ Run<E, N> load_run(const E* p) { return *reinterpret_cast<const Run<E, N>*>(p); }

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// The same for LDS traffic only: global loads and stores of the wave stay in flight.
__device__ __forceinline__ void wave_sync_lds() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
}

template <int GROUP>
__device__ __forceinline__ void group_sync() {
  if constexpr (GROUP <= kWave) wave_sync_lds(); else __syncthreads();
}

// Inclusive scan over the wave (all 64 lanes must call), on the DPP data path: four
// shifted adds inside each row of 16 lanes, then the row totals are broadcast into the
// following rows (row_bcast 15 and 31).
__device__ __forceinline__ int wave_incl_scan(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);   // row_shr:1
  v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);   // row_shr:2
  v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true);   // row_shr:4
  v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, true);   // row_shr:8
  v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);  // row_bcast:15 into rows 1 and 3
  v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);  // row_bcast:31 into rows 2 and 3
  return v;
}

// Inclusive scan inside aligned groups of WIDTH lanes (16: a DPP row, or the whole wave).
template <int WIDTH>
__device__ __forceinline__ int group_incl_scan(int v) {
  static_assert(WIDTH == 16 || WIDTH == kWave, "a DPP row or the wave");
  if constexpr (WIDTH == kWave) {
    return wave_incl_scan(v);
  } else {
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, true);   // row_shr:8
    return v;
  }
}

// Sets `bits` in the flag word *word(w) for every calling lane, combining lanes first.  Lanes that
// hold consecutive entries of an ascending column list hold runs of equal words, and LDS atomics on
// one address are executed one lane after the other; so inside each DPP row of 16 lanes a lane ORs
// in the bits of the lanes below it that hold the same word (four shifted steps), and only the last
// lane of a run issues the atomic.  Any set of lanes may call (lanes that are off count as "another
// word"); without runs it degenerates to one atomic per lane.
template <int D>
__device__ __forceinline__ void or_from_below(int w, unsigned& bits) {
  const int wl = __builtin_amdgcn_update_dpp(-2, w, 0x110 + D, 0xf, 0xf, false);              // row_shr:D
  const unsigned bl = (unsigned)__builtin_amdgcn_update_dpp(0, (int)bits, 0x110 + D, 0xf, 0xf, false);
  if (wl == w) bits |= bl;
}

template <class WordOf>
__device__ __forceinline__ void flags_or_combined(int w, unsigned bits, WordOf word) {
  or_from_below<1>(w, bits);
  or_from_below<2>(w, bits);
  or_from_below<4>(w, bits);
  or_from_below<8>(w, bits);
  const int wr = __builtin_amdgcn_update_dpp(-2, w, 0x101, 0xf, 0xf, false);                   // row_shl:1
  if (wr != w) atomicOr(word(w), bits);
}

__device__ __forceinline__ int wave_sum(int v) {
#pragma unroll
  for (int d = kWave / 2; d > 0; d >>= 1) v += __shfl_xor(v, d, kWave);
  return v;
}

__device__ __forceinline__ unsigned hash_col(int key) { return (unsigned)key * 0x9E3779B1u; }

// First position in [lo, hi) of an ascending int32 array whose value is >= target.
__device__ __forceinline__ int64_t lower_bound_i32(const int32_t* __restrict__ a, int64_t lo, int64_t hi, int target) {
  while (lo < hi) {
    int64_t mid = lo + ((hi - lo) >> 1);
    if (a[mid] < target) lo = mid + 1; else hi = mid;
  }
  return lo;
}

__device__ __forceinline__ int classify_symbolic(long long ip, int force) {
  if (ip <= 0) return kEmptyBin;
  const int dense = ip <= kDenseMid ? 4 : (ip <= kDenseBig ? 5 : 6);
  if (force == 3) return dense;
  if (force != 2) {
    if (ip <= kEscSmallCap) return 0;
    if (ip <= kEscLargeCap) return 1;
  }
  if (ip <= kSymHashSmall) return 2;
  if (ip <= kSymHashLarge) return 3;
  return dense;
}

// Numeric classes: 0/1 sorted list, 2/3 hash, 4 staged products (at most staged_cap of them,
// 0 = class not available), 5/6 dense tiles.
__device__ __forceinline__ int classify_numeric(long long ip, int cnt, int force, int staged_cap) {
  if (cnt <= 0) return kEmptyBin;
  const int dense = ip <= kDenseBig ? 5 : 6;
  const bool staged_ok = ip <= staged_cap;
  if (force == 3) return dense;
  if (force == 4 && staged_ok) return 4;
  if (force != 2) {
    if (ip <= kEscSmallCap) return 0;
    if (ip <= kEscLargeCap) return 1;
  }
  if (cnt <= kNumHashSmall) return 2;
  if (cnt <= kNumHashLarge) return 3;
  return staged_ok ? 4 : dense;
}

// Bitonic sort of the first n keys (a power of two, at most NMAX) held in LDS by G cooperating
// threads (thread index gl in [0, G)).  When vals is non-null the values move with their keys.
// A thread loads all the pairs it compares in a stage before it writes any back, so that a
// stage costs one LDS round trip instead of one per pair.
template <int G, int NMAX, typename V>
__device__ __forceinline__ void bitonic_sort_lds(int* keys, V* vals, int n, int gl) {
  constexpr int kPairs = (NMAX / 2 + G - 1) / G;
  const int half = n >> 1;
  for (int k = 2; k <= n; k <<= 1) {
    for (int j = k >> 1; j > 0; j >>= 1) {
      int ka[kPairs], kb[kPairs];
#pragma unroll
      for (int q = 0; q < kPairs; ++q) {
        const int t = gl + q * G;
        if (t < half) {
          const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1));
          ka[q] = keys[i];
          kb[q] = keys[i | j];
        }
      }
#pragma unroll
      for (int q = 0; q < kPairs; ++q) {
        const int t = gl + q * G;
        if (t < half) {
          const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1));
          const int p = i | j;
          const bool up = (i & k) == 0;
          if ((ka[q] > kb[q]) == up) {
            keys[i] = kb[q]; keys[p] = ka[q];
            if (vals) { const V a = vals[i]; vals[i] = vals[p]; vals[p] = a; }
          }
        }
      }
      group_sync<G>();
    }
  }
}

}  // namespace spg
