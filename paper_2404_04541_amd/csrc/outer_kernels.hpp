// Outer-product sparse x sparse product with a second-order (coordinate) sparse workspace: the
// paper's leading example (sections 1 and 4.1, the algorithm template of section 4.3, evaluated
// in section 7.3).  Loop order k -> i -> j over A in doubly compressed sparse columns and B in
// doubly compressed sparse rows; consecutive products land on unrelated coordinates (i, j), so
// they pass through a workspace of whole components:
//   insert   a batch of products (i << 32 | j, a_ik * b_kj) fills the accumulation array
//   sort     the accumulation array goes into result order (stable radix sort by coordinate)
//   merge    equal coordinates are added up; the sorted batch is merged into the all array
//            (sorted, unique), again adding equal coordinates
//   compress the all array becomes the row pointer / column / value arrays of C
// On the GPU a batch is inserted by one launch (a thread per product), not by one append at a
// time, and the merge is a rank computation on both sides followed by one reduction of equal
// neighbours; the stages and the two arrays are the paper's.
#pragma once
#include "common.hpp"

namespace spg {

// In-place exclusive scan of n int64 counters by one workgroup; v[n] receives the total.
__global__ __launch_bounds__(1024) void k_scan_i64(int64_t n, long long* __restrict__ v) {
  __shared__ long long part[1024];
  const int tid = threadIdx.x;
  const int64_t per = (n + 1023) / 1024;
  const int64_t lo = tid * per, hi = lo + per < n ? lo + per : n;
  long long s = 0;
  for (int64_t i = lo; i < hi; ++i) s += v[i];
  part[tid] = s;
  __syncthreads();
  for (int dd = 1; dd < 1024; dd <<= 1) {
    const long long t = tid >= dd ? part[tid - dd] : 0;
    __syncthreads();
    part[tid] += t;
    __syncthreads();
  }
  long long run = part[tid] - s;
  for (int64_t i = lo; i < hi; ++i) { const long long c = v[i]; v[i] = run; run += c; }
  if (tid == 1023) v[n] = part[1023];
}

// Exclusive scan of n 32-bit counters in place, in three steps: sums of tiles of kScanTileU32 counters,
// a scan of those sums (one workgroup: k_scan_u32), and the scan inside every tile on top of its sum.
constexpr int kScanTileU32 = 4096;   // 256 threads x 16 counters
__global__ __launch_bounds__(256) void k_scan_tile_sums(int64_t n, const unsigned* __restrict__ v, unsigned* __restrict__ sums) {
  __shared__ unsigned ws[4];
  const int64_t base = (int64_t)blockIdx.x * kScanTileU32;
  unsigned s = 0;
  for (int t = 0; t < 16; ++t) {
    const int64_t i = base + (int64_t)t * 256 + threadIdx.x;
    if (i < n) s += v[i];
  }
  s = (unsigned)wave_sum((int)s);
  if ((threadIdx.x & 63) == 0) ws[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) sums[blockIdx.x] = ws[0] + ws[1] + ws[2] + ws[3];
}

__global__ __launch_bounds__(256) void k_scan_tile_final(int64_t n, unsigned* __restrict__ v, const unsigned* __restrict__ sums) {
  __shared__ unsigned ws[4];
  const int64_t base = (int64_t)blockIdx.x * kScanTileU32 + (int64_t)threadIdx.x * 16;   // a thread owns 16 consecutive counters
  unsigned x[16], s = 0;
#pragma unroll
  for (int t = 0; t < 16; ++t) { x[t] = base + t < n ? v[base + t] : 0u; s += x[t]; }
  const unsigned incl = (unsigned)wave_incl_scan((int)s);
  if ((threadIdx.x & 63) == 63) ws[threadIdx.x >> 6] = incl;
  __syncthreads();
  unsigned run = sums[blockIdx.x] + incl - s;
  for (int w = 0; w < (int)(threadIdx.x >> 6); ++w) run += ws[w];
#pragma unroll
  for (int t = 0; t < 16; ++t) { if (base + t < n) v[base + t] = run; run += x[t]; }
}

// Row index of every entry of a CSR matrix (a wave per row).
__global__ __launch_bounds__(256) void k_expand_rows(int64_t rows, const int64_t* __restrict__ rowptr, int32_t* __restrict__ out) {
  const int64_t stride = (int64_t)gridDim.x * (blockDim.x / kWave);
  const int lane = threadIdx.x & 63;
  for (int64_t r = (int64_t)blockIdx.x * (blockDim.x / kWave) + (threadIdx.x >> 6); r < rows; r += stride)
    for (int64_t p = rowptr[r] + lane; p < rowptr[r + 1]; p += kWave) out[p] = (int32_t)r;
}

// flag[v] = 1 when vector v (a row, or a column) has entries.
__global__ __launch_bounds__(256) void k_dcs_flags(int64_t n, const int64_t* __restrict__ ptr, unsigned* __restrict__ flag) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v < n; v += stride) flag[v] = ptr[v + 1] > ptr[v] ? 1u : 0u;
}

// pos = exclusive scan of the flags: the non-empty vectors move up, in order.
__global__ __launch_bounds__(256) void k_dcs_fill(int64_t n, const int64_t* __restrict__ ptr, const unsigned* __restrict__ pos,
                                                  int32_t* __restrict__ vec, int64_t* __restrict__ out_ptr, int64_t nnz, int64_t nvec) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v < n; v += stride)
    if (ptr[v + 1] > ptr[v]) { vec[pos[v]] = (int32_t)v; out_ptr[pos[v]] = ptr[v]; }
  if (blockIdx.x == 0 && threadIdx.x == 0) out_ptr[nvec] = nnz;
}

// cnt[p] = products of A's p-th kept column: its length times the length of the B row of the same
// index k (0 when B has no such row); match[p] = that row's position in B's list, or -1.
__global__ __launch_bounds__(256) void k_outer_count(int64_t na, const int32_t* __restrict__ a_vec, const int64_t* __restrict__ a_ptr,
                                                     int64_t nb, const int32_t* __restrict__ b_vec, const int64_t* __restrict__ b_ptr,
                                                     long long* __restrict__ cnt, int32_t* __restrict__ match) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < na; p += stride) {
    const int k = a_vec[p];
    const int64_t q = lower_bound_i32(b_vec, 0, nb, k);
    const bool hit = q < nb && b_vec[q] == k;
    match[p] = hit ? (int32_t)q : -1;
    cnt[p] = hit ? (a_ptr[p + 1] - a_ptr[p]) * (b_ptr[q + 1] - b_ptr[q]) : 0;
  }
}

// Insert stage: products [t0, t0 + n) of the k -> i -> j order fill the accumulation array.
template <typename T>
__global__ __launch_bounds__(256) void k_outer_insert(int64_t t0, int64_t n, int64_t na, const long long* __restrict__ off,
                                                      const int32_t* __restrict__ match, const int64_t* __restrict__ a_ptr,
                                                      const int32_t* __restrict__ a_idx, const T* __restrict__ a_val,
                                                      const int64_t* __restrict__ b_ptr, const int32_t* __restrict__ b_idx,
                                                      const T* __restrict__ b_val, unsigned long long* __restrict__ keys,
                                                      unsigned* __restrict__ seq, double* __restrict__ vals) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t x = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; x < n; x += stride) {
    const int64_t t = t0 + x;
    int64_t lo = 0, hi = na;   // last column whose first product is <= t
    while (hi - lo > 1) {
      const int64_t mid = lo + ((hi - lo) >> 1);
      if (off[mid] <= t) lo = mid; else hi = mid;
    }
    const int64_t q = match[lo];
    const int64_t lb = b_ptr[q + 1] - b_ptr[q];
    const int64_t local = t - off[lo];
    const int64_t pa = a_ptr[lo] + local / lb, pb = b_ptr[q] + local % lb;
    keys[x] = ((unsigned long long)(unsigned)a_idx[pa] << 32) | (unsigned)b_idx[pb];
    seq[x] = (unsigned)x;
    vals[x] = (double)a_val[pa] * (double)b_val[pb];
  }
}

// head[x] = 1 when component x starts a new coordinate in a sorted array.
__global__ __launch_bounds__(256) void k_outer_heads(int64_t n, const unsigned long long* __restrict__ keys, unsigned* __restrict__ head) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t x = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; x < n; x += stride) head[x] = (x == 0 || keys[x] != keys[x - 1]) ? 1u : 0u;
}

// Adds up equal coordinates of a sorted array: the thread of a run's first component walks the run in
// order (seq, when given, leads to the value of a component through the sort's permutation).
// pos = exclusive scan of the head flags = where the run's sum goes.
__global__ __launch_bounds__(256) void k_outer_reduce(int64_t n, const unsigned long long* __restrict__ keys, const unsigned* __restrict__ seq,
                                                      const double* __restrict__ vals, const unsigned* __restrict__ pos,
                                                      unsigned long long* __restrict__ out_keys, double* __restrict__ out_vals) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t x = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; x < n; x += stride) {
    const unsigned long long key = keys[x];
    if (x > 0 && keys[x - 1] == key) continue;
    double s = vals[seq ? seq[x] : x];
    for (int64_t y = x + 1; y < n && keys[y] == key; ++y) s += vals[seq ? seq[y] : y];
    out_keys[pos[x]] = key;
    out_vals[pos[x]] = s;
  }
}

// Merge stage, first half: two sorted arrays of unique coordinates into one sorted array (the all array's
// component first where both hold a coordinate): a component's place is its own index plus its rank in
// the other array.
__global__ __launch_bounds__(256) void k_outer_merge(int64_t na, const unsigned long long* __restrict__ ka, const double* __restrict__ va,
                                                     int64_t nb, const unsigned long long* __restrict__ kb, const double* __restrict__ vb,
                                                     unsigned long long* __restrict__ out_keys, double* __restrict__ out_vals) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t x = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; x < na + nb; x += stride) {
    const bool first = x < na;
    const int64_t i = first ? x : x - na;
    const unsigned long long key = first ? ka[i] : kb[i];
    const unsigned long long* other = first ? kb : ka;
    int64_t lo = 0, hi = first ? nb : na;
    while (lo < hi) {   // first: components of b below key; second: components of a up to and including key
      const int64_t mid = lo + ((hi - lo) >> 1);
      const bool below = first ? other[mid] < key : other[mid] <= key;
      if (below) lo = mid + 1; else hi = mid;
    }
    out_keys[i + lo] = key;
    out_vals[i + lo] = first ? va[i] : vb[i];
  }
}

// Compress stage: columns and values of C from the all array (the row pointer comes from the coordinates' high halves).
template <typename T>
__global__ __launch_bounds__(256) void k_outer_emit(int64_t n, const unsigned long long* __restrict__ keys, const double* __restrict__ vals,
                                                    int32_t* __restrict__ colidx, T* __restrict__ values) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t x = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; x < n; x += stride) {
    colidx[x] = (int32_t)(unsigned)keys[x];
    values[x] = (T)vals[x];
  }
}

}  // namespace spg
