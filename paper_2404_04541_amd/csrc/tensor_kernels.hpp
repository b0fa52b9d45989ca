// Mode-3 unfolding of a sparse 3-tensor given as coordinates (the "index folding" route to a
// sparse tensor-times-matrix product, paper section 7.4): X(i,j,k) becomes row i*J + j, column k
// of a CSR matrix, so that Y(i,j,l) = sum_k X(i,j,k) M(k,l) is one row-wise product whose CSR
// result is the unfolding of Y.  Coordinates may come in any order; repeated coordinates stay
// separate entries (the product adds them).
//   keys     row << 32 | k per entry
//   sort     least-significant-digit radix sort, 8 bits per pass, over the bits that k and the
//            row can occupy; a wave owns a tile of kSortTile consecutive entries and ranks its
//            lanes per digit with ballots, which keeps the pass stable
//   compress row pointer from the sorted keys, columns and permuted values
#pragma once
#include "common.hpp"

namespace spg {

constexpr int kSortTile = 4096;     // entries per wave and pass
constexpr int kSortWgWaves = 4;

__global__ __launch_bounds__(256) void k_tensor_keys(int64_t nnz, int64_t I, int64_t J, int64_t K, const int32_t* __restrict__ xi,
                                                     const int32_t* __restrict__ xj, const int32_t* __restrict__ xk,
                                                     unsigned long long* __restrict__ keys, unsigned* __restrict__ idx, int* __restrict__ bad) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < nnz; p += stride) {
    const int i = xi[p], j = xj[p], k = xk[p];
    if (i < 0 || i >= I || j < 0 || j >= J || k < 0 || k >= K) { *bad = 1; keys[p] = 0; idx[p] = (unsigned)p; continue; }
    keys[p] = ((unsigned long long)((long long)i * J + j) << 32) | (unsigned)k;
    idx[p] = (unsigned)p;
  }
}

// hist[digit * ntiles + tile] = entries of the tile whose digit (bits [shift, shift+8) of the key) is `digit`
__global__ __launch_bounds__(256) void k_radix_hist(int64_t n, int64_t ntiles, int shift, const unsigned long long* __restrict__ keys,
                                                    unsigned* __restrict__ hist) {
  __shared__ unsigned cnt[kSortWgWaves][256];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int64_t tile = (int64_t)blockIdx.x * kSortWgWaves + wave;
  for (int d = lane; d < 256; d += kWave) cnt[wave][d] = 0;
  wave_sync_lds();
  if (tile < ntiles) {
    const int64_t lo = tile * kSortTile;
    const int64_t hi = lo + kSortTile < n ? lo + kSortTile : n;
    for (int64_t p = lo + lane; p < hi; p += kWave) atomicAdd(&cnt[wave][(unsigned)(keys[p] >> shift) & 255u], 1u);
    wave_sync_lds();
    for (int d = lane; d < 256; d += kWave) hist[(int64_t)d * ntiles + tile] = cnt[wave][d];
  }
}

// In-place exclusive scan of `n` counters by one workgroup (n is a few hundred thousand at most).
__global__ __launch_bounds__(1024) void k_scan_u32(int64_t n, unsigned* __restrict__ v) {
  __shared__ unsigned long long part[1024];
  const int tid = threadIdx.x;
  const int64_t per = (n + 1023) / 1024;
  const int64_t lo = tid * per, hi = lo + per < n ? lo + per : n;
  unsigned long long s = 0;
  for (int64_t i = lo; i < hi; ++i) s += v[i];
  part[tid] = s;
  __syncthreads();
  for (int dd = 1; dd < 1024; dd <<= 1) {
    const unsigned long long t = tid >= dd ? part[tid - dd] : 0;
    __syncthreads();
    part[tid] += t;
    __syncthreads();
  }
  unsigned run = (unsigned)(part[tid] - s);
  for (int64_t i = lo; i < hi; ++i) { const unsigned c = v[i]; v[i] = run; run += c; }
}

// Stable scatter of one pass: the wave walks its tile 64 entries at a time; lanes with the same
// digit find each other with 8 ballots, rank themselves inside that set, and the set's first lane
// advances the digit's position.
__global__ __launch_bounds__(256) void k_radix_scatter(int64_t n, int64_t ntiles, int shift, const unsigned long long* __restrict__ keys,
                                                       const unsigned* __restrict__ idx, const unsigned* __restrict__ hist,
                                                       unsigned long long* __restrict__ keys_out, unsigned* __restrict__ idx_out) {
  __shared__ unsigned pos[kSortWgWaves][256];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int64_t tile = (int64_t)blockIdx.x * kSortWgWaves + wave;
  if (tile >= ntiles) return;
  for (int d = lane; d < 256; d += kWave) pos[wave][d] = hist[(int64_t)d * ntiles + tile];
  wave_sync_lds();
  const int64_t lo = tile * kSortTile;
  const int64_t hi = lo + kSortTile < n ? lo + kSortTile : n;
  const unsigned long long below = lane == 0 ? 0ULL : (~0ULL >> (64 - lane));
  for (int64_t p0 = lo; p0 < hi; p0 += kWave) {
    const int64_t p = p0 + lane;
    const bool live = p < hi;
    const unsigned long long key = live ? keys[p] : 0ULL;
    const unsigned id = live ? idx[p] : 0u;
    const unsigned d = (unsigned)(key >> shift) & 255u;
    unsigned long long peers = __ballot(live);
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      const unsigned long long m = __ballot((d >> b) & 1u);
      peers &= ((d >> b) & 1u) ? m : ~m;
    }
    if (live) {
      const unsigned at = pos[wave][d] + (unsigned)__popcll(peers & below);
      keys_out[at] = key;
      idx_out[at] = id;
    }
    wave_sync_lds();
    if (live && (peers & below) == 0) pos[wave][d] += (unsigned)__popcll(peers);
    wave_sync_lds();
  }
}

// From the sorted keys: columns, and values gathered through the permutation.
template <typename T>
__global__ __launch_bounds__(256) void k_tensor_compress(int64_t nnz, const unsigned long long* __restrict__ keys,
                                                         const unsigned* __restrict__ idx, const T* __restrict__ xval,
                                                         int32_t* __restrict__ colidx, T* __restrict__ values) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < nnz; p += stride) {
    colidx[p] = (int32_t)(unsigned)keys[p];
    values[p] = xval[idx[p]];
  }
}

// rowptr[r] = first position of the sorted keys whose row is r or more (r = 0 .. rows).
__global__ __launch_bounds__(256) void k_tensor_rowptr(int64_t nnz, int64_t rows, const unsigned long long* __restrict__ keys,
                                                       int64_t* __restrict__ rowptr) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; r <= rows; r += stride) {
    int64_t lo = 0, hi = nnz;
    while (lo < hi) {
      const int64_t mid = lo + ((hi - lo) >> 1);
      if ((int64_t)(keys[mid] >> 32) < r) lo = mid + 1; else hi = mid;
    }
    rowptr[r] = lo;
  }
}

// A row of an unfolded result back to coordinates: per entry the row's two folded coordinates
// (row / B, row % B) and, when asked for, the column as the third.
__global__ __launch_bounds__(256) void k_tensor_fold(int64_t rows, int64_t B, const int64_t* __restrict__ rowptr,
                                                     const int32_t* __restrict__ colidx, int32_t* __restrict__ ya,
                                                     int32_t* __restrict__ yb, int32_t* __restrict__ yc) {
  const int64_t stride = (int64_t)gridDim.x * (blockDim.x / kWave);
  const int lane = threadIdx.x & 63;
  for (int64_t r = (int64_t)blockIdx.x * (blockDim.x / kWave) + (threadIdx.x >> 6); r < rows; r += stride) {
    const int64_t lo = rowptr[r], hi = rowptr[r + 1];
    const int32_t a = (int32_t)(r / B), b = (int32_t)(r % B);
    for (int64_t p = lo + lane; p < hi; p += kWave) {
      ya[p] = a;
      yb[p] = b;
      if (yc) yc[p] = colidx[p];
    }
  }
}

}  // namespace spg
