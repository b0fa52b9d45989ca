// Per-row intermediate-product count, input checks, binning and the row-count scan.
#pragma once
#include "common.hpp"

namespace spg {

__global__ void k_init_control(Control* ctl) {
  unsigned* w = reinterpret_cast<unsigned*>(ctl);
  for (int i = threadIdx.x; i < (int)(sizeof(Control) / sizeof(unsigned)); i += blockDim.x) w[i] = 0;
}

// Checks B: rowptr starts at 0, is non-decreasing, ends at nnz, no row of 2^31 or more
// entries; every column inside [0, cols).  Also counts descents (col[p] <= col[p-1]) over
// the flat column array and descents that straddle a row boundary: every row is strictly
// ascending exactly when the two counts agree (k_bin_offsets turns them into b_sorted).
__global__ __launch_bounds__(256) void k_validate_b(int64_t rows, int64_t cols, int64_t nnz,
                                                    const int64_t* __restrict__ rp, const int32_t* __restrict__ col,
                                                    Control* ctl) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  const int64_t t0 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  bool bad = false;
  int flat = 0, bnd = 0;
  if (t0 == 0 && (rp[0] != 0 || rp[rows] != nnz)) bad = true;
  for (int64_t i = t0; i < rows; i += stride) {
    const int64_t a = rp[i], b = rp[i + 1];
    if (b < a || a < 0 || b > nnz || b - a > 0x7fffffff) { bad = true; continue; }
    if (b - a >= (1 << 21)) ctl->long_b_row = 1;
    if (b > a && a > 0 && col[a] <= col[a - 1]) ++bnd;
  }
  for (int64_t p = t0; p < nnz; p += stride) {
    const int c = col[p];
    if (c < 0 || c >= cols) bad = true;
    if (p > 0 && c <= col[p - 1]) ++flat;
  }
  if (bad) ctl->error = 1;
  // one pair of atomics per workgroup: nearly every wave has descents to report (the row boundaries)
  __shared__ int part[2][4];
  flat = wave_sum(flat);
  bnd = wave_sum(bnd);
  if (lane_id() == 0) { part[0][threadIdx.x >> 6] = flat; part[1][threadIdx.x >> 6] = bnd; }
  __syncthreads();
  if (threadIdx.x == 0) {
    const int f4 = part[0][0] + part[0][1] + part[0][2] + part[0][3], b4 = part[1][0] + part[1][1] + part[1][2] + part[1][3];
    if (f4) atomicAdd(&ctl->desc_flat, (unsigned long long)f4);
    if (b4) atomicAdd(&ctl->desc_bnd, (unsigned long long)b4);
  }
}

// One workgroup of 1024 threads per 256 consecutive rows of A (a chunk of hub rows holds a large
// share of all entries, so the chunk gets the widest workgroup): the chunk's A entries are read
// coalesced, each entry adds the length of its B row to its row's counter in LDS.
// Writes ip (saturated to int32), the symbolic bin, zero counts for rows without products.
constexpr int kCountThreads = 1024;
__global__ __launch_bounds__(kCountThreads) void k_count_rows(int64_t m, int64_t nnz_a, int64_t b_rows,
                                                    const int64_t* __restrict__ a_rp, const int32_t* __restrict__ a_col,
                                                    const int64_t* __restrict__ b_rp, int* __restrict__ ip_out,
                                                    unsigned char* __restrict__ bin_out, int* __restrict__ cnt_out,
                                                    Control* ctl, int force, int row_block) {
  __shared__ long long rp[257];
  __shared__ unsigned long long ipl[256];
  __shared__ unsigned hist[kNumBins];
  __shared__ unsigned long long hip[kNumBins];
  __shared__ int bad;
  const int tid = threadIdx.x;
  if (tid < kNumBins) { hist[tid] = 0; hip[tid] = 0; }
  // a workgroup takes several chunks and reports its bin populations once (thousands of workgroups adding to
  // the same few counters cost more than the counting)
  __shared__ long long next_chunk;
  int64_t chunk = blockIdx.x;
  while (chunk * 256 < m) {
    // (the chunk after this one is drawn now and looked at when this one is done: chunks differ by orders of
    // magnitude in their entries, so they are handed out rather than dealt)
    long long drawn = 0;
    if (tid == 0) drawn = (long long)gridDim.x + atomicAdd(&ctl->work[3], 1u);
    const int64_t r0 = chunk * 256;
    const int nr = (int)((m - r0) < 256 ? (m - r0) : 256);
    __syncthreads();   // (the bin counters are initialised; the chunk before has left rp and ipl)
    if (tid == 0) bad = 0;
    for (int t = tid; t <= nr; t += kCountThreads) rp[t] = a_rp[r0 + t];
    if (tid < 256) ipl[tid] = 0;
    __syncthreads();
    if (tid < nr && rp[tid + 1] < rp[tid]) bad = 1;
    if (tid == 0) {
      if (rp[0] < 0 || rp[nr] > nnz_a) bad = 1;
      // (a block of rows of a larger matrix keeps that matrix's positions: it neither starts at 0 nor ends at nnz)
      if (!row_block && r0 == 0 && rp[0] != 0) bad = 1;
      if (!row_block && r0 + nr == m && rp[nr] != nnz_a) bad = 1;
    }
    __syncthreads();
    if (bad) {
      if (tid == 0) ctl->error = 1;
      return;
    }
    const long long lo = rp[0], hi = rp[nr];
    bool badcol = false;
    // four entries per thread and round, so that their (dependent) loads overlap
    for (long long p0 = lo + tid; p0 < hi; p0 += kCountThreads * 4) {
      int k[4];
      long long len[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const long long p = p0 + u * kCountThreads;
        k[u] = p < hi ? a_col[p] : -1;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const long long p = p0 + u * kCountThreads;
        len[u] = 0;
        if (p < hi) {
          if (k[u] < 0 || k[u] >= b_rows) { badcol = true; continue; }
          const Run<int64_t, 2> bounds = load_run<int64_t, 2>(b_rp + k[u]);   // (both ends of the row in one load)
          len[u] = bounds.v[1] - bounds.v[0];
          if (len[u] < 0) { badcol = true; len[u] = 0; }
        }
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const long long p = p0 + u * kCountThreads;
        if (len[u] > 0) {
          // row of entry p: last t with rp[t] <= p
          int a = 0, b = nr;
          while (b - a > 1) {
            const int mid = (a + b) >> 1;
            if (rp[mid] <= p) a = mid; else b = mid;
          }
          atomicAdd(&ipl[a], (unsigned long long)len[u]);
        }
      }
    }
    if (badcol) ctl->error = 1;
    __syncthreads();
    if (tid < nr) {
      const unsigned long long mine = ipl[tid];
      const int bin = classify_symbolic((long long)mine, force);
      ip_out[r0 + tid] = mine > 0x7fffffffULL ? 0x7fffffff : (int)mine;
      bin_out[r0 + tid] = (unsigned char)bin;
      if (bin == kEmptyBin) cnt_out[r0 + tid] = 0;
      atomicAdd(&hist[bin], 1u);
      if (mine) atomicAdd(&hip[bin], mine);
    }
    if (tid == 0) next_chunk = drawn;
    __syncthreads();
    chunk = next_chunk;
  }
  __syncthreads();
  if (tid < kNumBins && hist[tid]) {
    atomicAdd(&ctl->hist[0][tid], hist[tid]);
    if (hip[tid]) atomicAdd(&ctl->bin_ip[0][tid], hip[tid]);
  }
  if (tid == 0) {   // the products of all rows = the products of all bins
    unsigned long long tot = 0;
    for (int b = 0; b < kNumBins; ++b) tot += hip[b];
    if (tot) atomicAdd(&ctl->ip_total, tot);
  }
}

// Numeric classes from ip and the symbolic counts.
__global__ void k_classify_numeric(int64_t m, const int* __restrict__ ip, const int* __restrict__ cnt,
                                   unsigned char* __restrict__ bin_out, Control* ctl, int force, int staged_cap) {
  __shared__ unsigned hist[kNumBins];
  __shared__ unsigned long long hip[kNumBins], hnz[kNumBins];
  if (threadIdx.x < kNumBins) { hist[threadIdx.x] = 0; hip[threadIdx.x] = 0; hnz[threadIdx.x] = 0; }
  __syncthreads();
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < m; i += stride) {
    const int bin = classify_numeric(ip[i], cnt[i], force, staged_cap);
    bin_out[i] = (unsigned char)bin;
    atomicAdd(&hist[bin], 1u);
    if (bin != kEmptyBin) {
      atomicAdd(&hip[bin], (unsigned long long)ip[i]);
      atomicAdd(&hnz[bin], (unsigned long long)cnt[i]);
    }
  }
  __syncthreads();
  if (threadIdx.x < kNumBins && hist[threadIdx.x]) {
    atomicAdd(&ctl->hist[1][threadIdx.x], hist[threadIdx.x]);
    atomicAdd(&ctl->bin_ip[1][threadIdx.x], hip[threadIdx.x]);
    atomicAdd(&ctl->bin_nnz[threadIdx.x], hnz[threadIdx.x]);
  }
}

__global__ void k_bin_offsets(Control* ctl, int phase) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    unsigned s = 0;
    for (int b = 0; b < kNumBins; ++b) {
      ctl->offset[phase][b] = s;
      s += ctl->hist[phase][b];
      ctl->cursor[phase][b] = 0;
    }
    ctl->offset[phase][kNumBins] = s;
    if (phase == 0) {
      ctl->b_sorted = (ctl->desc_flat == ctl->desc_bnd) ? 1 : 0;
      // the dense workspaces walk whole rows of an unsorted B per tile: 32-bit piece prefixes
      if (!ctl->b_sorted && ctl->long_b_row && !ctl->error) ctl->error = 2;
    }
  }
}

// Scatter row ids into their bins.  Each wave ballots per bin and ranks its lanes inside the
// ballot mask (a wavefront-level prefix count); the waves of a workgroup add their counts up in
// LDS, so that a bin costs one global atomic per workgroup of 1024 rows.
constexpr int kScatterThreads = 1024;
__global__ __launch_bounds__(kScatterThreads) void k_bin_scatter(int64_t m, const unsigned char* __restrict__ bin, int* __restrict__ perm,
                                                                 Control* ctl, int phase) {
  constexpr int kWaves = kScatterThreads / kWave;
  __shared__ unsigned wcount[kNumBins][kWaves];   // per bin: rows of each wave, then their prefix
  __shared__ unsigned base[kNumBins];
  if (ctl->error) return;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int b = i < m ? bin[i] : -1;
  const int lane = lane_id(), wave = threadIdx.x >> 6;
  const unsigned long long below = lane == 0 ? 0ULL : (~0ULL >> (64 - lane));
  int rank = 0;
  for (int v = 0; v < kNumBins - 1; ++v) {   // bin 7 holds rows with no work: not listed
    const unsigned long long mask = __ballot(b == v);
    if (lane == 0) wcount[v][wave] = (unsigned)__popcll(mask);
    if (b == v) rank = __popcll(mask & below);
  }
  __syncthreads();
  if (threadIdx.x < kNumBins - 1) {
    const int v = threadIdx.x;
    unsigned run = 0;
    for (int w = 0; w < kWaves; ++w) { const unsigned c = wcount[v][w]; wcount[v][w] = run; run += c; }
    base[v] = run ? atomicAdd(&ctl->cursor[phase][v], run) : 0u;
  }
  __syncthreads();
  if (b >= 0 && b < kNumBins - 1) perm[ctl->offset[phase][b] + base[b] + wcount[b][wave] + rank] = (int)i;
}

// ---- exclusive scan of int32 row counts into the int64 row pointer -------------------
constexpr int kScanThreads = 256;
constexpr int kScanItems = 16;
constexpr int kScanTile = kScanThreads * kScanItems;

__global__ __launch_bounds__(kScanThreads) void k_scan_partials(int64_t m, const int* __restrict__ cnt,
                                                                long long* __restrict__ partial) {
  const int64_t base = (int64_t)blockIdx.x * kScanTile;
  long long s = 0;
  for (int t = 0; t < kScanItems; ++t) {
    const int64_t i = base + (int64_t)t * kScanThreads + threadIdx.x;
    if (i < m) s += cnt[i];
  }
  for (int d = 32; d > 0; d >>= 1) s += __shfl_xor(s, d, kWave);
  __shared__ long long ws[kScanThreads / kWave];
  if ((threadIdx.x & 63) == 0) ws[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    long long t = 0;
    for (int w = 0; w < kScanThreads / kWave; ++w) t += ws[w];
    partial[blockIdx.x] = t;
  }
}

__global__ __launch_bounds__(kScanThreads) void k_scan_blocks(int64_t nblocks, long long* __restrict__ partial,
                                                              int64_t m, int64_t* __restrict__ rowptr, Control* ctl) {
  // single workgroup: exclusive scan of the per-tile sums, in place
  __shared__ long long tile[kScanThreads];
  __shared__ long long carry;
  if (threadIdx.x == 0) carry = 0;
  __syncthreads();
  for (int64_t b0 = 0; b0 < nblocks; b0 += kScanThreads) {
    const int64_t i = b0 + threadIdx.x;
    const long long v = i < nblocks ? partial[i] : 0;
    tile[threadIdx.x] = v;
    __syncthreads();
    for (int d = 1; d < kScanThreads; d <<= 1) {
      long long t = threadIdx.x >= d ? tile[threadIdx.x - d] : 0;
      __syncthreads();
      tile[threadIdx.x] += t;
      __syncthreads();
    }
    if (i < nblocks) partial[i] = carry + tile[threadIdx.x] - v;
    __syncthreads();
    if (threadIdx.x == 0) carry += tile[kScanThreads - 1];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    rowptr[m] = carry;
    ctl->nnz_c = carry;
  }
}

__global__ __launch_bounds__(kScanThreads) void k_scan_final(int64_t m, const int* __restrict__ cnt,
                                                             const long long* __restrict__ partial,
                                                             int64_t* __restrict__ rowptr) {
  // thread t owns kScanItems consecutive rows of the tile
  __shared__ long long tsum[kScanThreads];
  const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
  int v[kScanItems];
  long long s = 0;
#pragma unroll
  for (int t = 0; t < kScanItems; ++t) {
    v[t] = (base + t < m) ? cnt[base + t] : 0;
    s += v[t];
  }
  tsum[threadIdx.x] = s;
  __syncthreads();
  for (int d = 1; d < kScanThreads; d <<= 1) {
    long long t = threadIdx.x >= d ? tsum[threadIdx.x - d] : 0;
    __syncthreads();
    tsum[threadIdx.x] += t;
    __syncthreads();
  }
  long long run = partial[blockIdx.x] + tsum[threadIdx.x] - s;
#pragma unroll
  for (int t = 0; t < kScanItems; ++t) {
    if (base + t < m) rowptr[base + t] = run;
    run += v[t];
  }
}

}  // namespace spg
