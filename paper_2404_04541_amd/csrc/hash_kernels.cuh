// LDS hash workspace for mid-sized rows: a 1-D open-addressing table along the column
// index with deduplication on collision (the hash policy of the paper's sections 4.4 and
// 5.2; the paper's bucket function "label mod L, L a power of two" becomes a
// multiplicative hash here because power-law and banded columns cluster in the low bits).
// Symbolic: a key-only set, the answer is the number of occupied slots.
// Numeric : keys plus double sums; afterwards the whole table is sorted by key so that
//           the occupied slots come first in ascending column order (hash retrieval),
//           and that prefix is copied to the row of C.
#pragma once
#include "common.cuh"

namespace spg {

template <int LOGH>
__device__ __forceinline__ int hash_find_or_insert(int* keys, int key, int& is_new) {
  constexpr unsigned mask = (1u << LOGH) - 1;
  unsigned h = hash_col(key) >> (32 - LOGH);
  is_new = 0;
  while (true) {
    const int old = atomicCAS(&keys[h], kEmptyKey, key);
    if (old == kEmptyKey) { is_new = 1; return (int)h; }
    if (old == key) return (int)h;
    h = (h + 1) & mask;
  }
}

// Lanes of a group are laid out as LA x LB: LB lanes walk one B row together, LA rows of B
// are in flight at once; LB is the power of two nearest above the row's mean B-row length.
__device__ __forceinline__ int pick_lb(int ip, int d, int group) {
  int avg = d > 0 ? (ip + d - 1) / d : 1;
  int lb = 1;
  while (lb < avg && lb < group && lb < kWave) lb <<= 1;
  return lb;
}

// GROUP threads per row (64: one wave, several rows per workgroup; 256: the workgroup).
template <int GROUP, int LOGH, typename T, bool NUMERIC>
__global__ __launch_bounds__(256) void k_hash(const int* __restrict__ perm, const Control* __restrict__ ctl, int phase, int bin,
                                               const int* __restrict__ ip_row,
                                               const int64_t* __restrict__ a_rp, const int32_t* __restrict__ a_col,
                                               const T* __restrict__ a_val, const int64_t* __restrict__ b_rp,
                                               const int32_t* __restrict__ b_col, const T* __restrict__ b_val,
                                               int* __restrict__ cnt, const int64_t* __restrict__ c_rp,
                                               int32_t* __restrict__ c_col, T* __restrict__ c_val) {
  constexpr int H = 1 << LOGH;
  constexpr int kGroups = 256 / GROUP;
  extern __shared__ __align__(16) unsigned char smem[];
  // layout: per group H keys, then (numeric) H doubles; one int counter per group at the end
  double* all_vals = reinterpret_cast<double*>(smem);
  int* all_keys = reinterpret_cast<int*>(smem + (NUMERIC ? (size_t)kGroups * H * sizeof(double) : 0));
  int* counters = all_keys + kGroups * H;
  if (ctl->error) return;
  const unsigned first = ctl->offset[phase][bin];
  const unsigned nrows = ctl->offset[phase][bin + 1] - first;
  const int g = threadIdx.x / GROUP;
  const int gl = threadIdx.x % GROUP;
  int* keys = all_keys + g * H;
  double* vals = NUMERIC ? all_vals + g * H : nullptr;
  const unsigned ngroups = gridDim.x * kGroups;
  const unsigned rounds = (nrows + ngroups - 1) / ngroups;
  for (unsigned r = 0; r < rounds; ++r) {
    const unsigned slot = r * ngroups + blockIdx.x * kGroups + g;
    const bool live = slot < nrows;
    const int row = live ? perm[first + slot] : 0;
    for (int t = gl; t < H; t += GROUP) {
      keys[t] = kEmptyKey;
      if (NUMERIC) vals[t] = 0.0;
    }
    if (gl == 0) counters[g] = 0;
    group_sync<GROUP>();
    if (live) {
      const int64_t a0 = a_rp[row];
      const int d = (int)(a_rp[row + 1] - a0);
      const int lb = pick_lb(ip_row[row], d, GROUP);
      const int la = GROUP / lb;
      const int ai = gl / lb, bo = gl % lb;
      int fresh = 0;
      for (int e = ai; e < d; e += la) {
        const int k = a_col[a0 + e];
        const int64_t bs = b_rp[k], be = b_rp[k + 1];
        double av = 0.0;
        if (NUMERIC) av = (double)a_val[a0 + e];
        for (int64_t q = bs + bo; q < be; q += lb) {
          int is_new;
          const int h = hash_find_or_insert<LOGH>(keys, b_col[q], is_new);
          fresh += is_new;
          if (NUMERIC)
            __hip_atomic_fetch_add(&vals[h], av * (double)b_val[q], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
      }
      if (!NUMERIC && fresh) atomicAdd(&counters[g], fresh);
    }
    group_sync<GROUP>();
    if (!NUMERIC) {
      if (live && gl == 0) cnt[row] = counters[g];
    } else {
      // empty slots hold kEmptyKey = -1: turn them into the pad key so they sort last
      for (int t = gl; t < H; t += GROUP) if (keys[t] == kEmptyKey) keys[t] = kPadKey;
      group_sync<GROUP>();
      bitonic_sort_lds<GROUP, H, double>(keys, vals, gl);
      if (live) {
        const int64_t out = c_rp[row];
        const int n = (int)(c_rp[row + 1] - out);
        for (int t = gl; t < n; t += GROUP) {
          c_col[out + t] = keys[t];
          c_val[out + t] = (T)vals[t];
        }
      }
    }
    group_sync<GROUP>();
  }
}

template <int GROUP, int LOGH, bool NUMERIC>
constexpr size_t hash_lds_bytes() {
  return (size_t)(256 / GROUP) * (1u << LOGH) * (sizeof(int) + (NUMERIC ? sizeof(double) : 0)) + (256 / GROUP) * sizeof(int);
}

}  // namespace spg
