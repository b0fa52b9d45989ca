// LDS hash workspace for mid-sized rows: a 1-D open-addressing table along the column
// index with deduplication on collision (the hash policy of the paper's sections 4.4 and
// 5.2; the paper's bucket function "label mod L, L a power of two" becomes a
// multiplicative hash here because power-law and banded columns cluster in the low bits).
// Symbolic: a key-only set, the answer is the number of occupied slots.
// Numeric : keys plus double sums; afterwards the whole table is sorted by key so that
//           the occupied slots come first in ascending column order (hash retrieval),
//           and that prefix is copied to the row of C.
#pragma once
#include "common.hpp"

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

constexpr int kHashUnroll = 4;

// An A entry of the row being inserted: its products are [first, next) of the row's product index space,
// its B row starts at bs.
struct __align__(16) HashEntry { int first, next; int64_t bs; };

// Exclusive scan over a group of GROUP threads (a wave, or the workgroup of 256), with the total.
// part: GROUP / 64 + 1 ints of LDS of the group.  Contains the group's synchronisation when GROUP > 64.
template <int GROUP>
__device__ __forceinline__ int group_excl_scan(int v, int& total, int* part) {
  const int incl = wave_incl_scan(v);
  if constexpr (GROUP <= kWave) {
    total = __builtin_amdgcn_readlane(incl, kWave - 1);
    return incl - v;
  } else {
    constexpr int kW = GROUP / kWave;
    const int wave = threadIdx.x >> 6;
    __syncthreads();
    if (lane_id() == kWave - 1) part[wave] = incl;
    __syncthreads();
    int before = 0;
    total = 0;
#pragma unroll
    for (int w = 0; w < kW; ++w) { const int x = part[w]; if (w < wave) before += x; total += x; }
    return before + incl - v;
  }
}

// GROUP threads per row (64: one wave, several rows per workgroup; 256: the workgroup).
template <int GROUP, int LOGH, typename T, bool NUMERIC>
__global__ __launch_bounds__(256) void k_hash(const int* __restrict__ perm, const Control* __restrict__ ctl, int phase, int bin,
                                               const int* __restrict__ ip_row,
                                               const int64_t* __restrict__ a_rp, const int32_t* __restrict__ a_col,
                                               const T* __restrict__ a_val, const int64_t* __restrict__ b_rp,
                                               const int32_t* __restrict__ b_col, const T* __restrict__ b_val,
                                               int* __restrict__ cnt, const int64_t* __restrict__ c_rp,
                                               int32_t* __restrict__ c_col, T* __restrict__ c_val, int64_t n_cols) {
  constexpr int H = 1 << LOGH;
  const bool packable = n_cols <= (int64_t(1) << (31 - LOGH));   // column << LOGH stays below the pad key
  constexpr int kGroups = 256 / GROUP;
  extern __shared__ __align__(16) unsigned char smem[];
  // layout: per group H keys, then (numeric) H doubles; one int counter per group at the end
  double* all_vals = reinterpret_cast<double*>(smem);
  int* all_keys = reinterpret_cast<int*>(smem + (NUMERIC ? (size_t)kGroups * H * sizeof(double) : 0));
  int* counters = all_keys + kGroups * H;
  // per group: the entries being inserted (length prefix, B row start, a_ik) and scan partials
  unsigned char* extra = reinterpret_cast<unsigned char*>(counters + kGroups);
  extra += (8 - (reinterpret_cast<size_t>(extra) & 7)) & 7;
  extra += (16 - (reinterpret_cast<size_t>(extra) & 15)) & 15;
  HashEntry* all_ent = reinterpret_cast<HashEntry*>(extra);
  double* all_pav = reinterpret_cast<double*>(all_ent + kGroups * GROUP);
  int* part = reinterpret_cast<int*>(all_pav + kGroups * GROUP);
  if (ctl->error) return;
  const unsigned first = ctl->offset[phase][bin];
  const unsigned nrows = ctl->offset[phase][bin + 1] - first;
  const int g = threadIdx.x / GROUP;
  const int gl = threadIdx.x % GROUP;
  int* keys = all_keys + g * H;
  double* vals = NUMERIC ? all_vals + g * H : nullptr;
  HashEntry* ent = all_ent + g * GROUP;
  double* pav = all_pav + g * GROUP;
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
    // insert: GROUP entries of the A row are described at a time (B row start, length, a_ik); their
    // products form one index space that the group's threads walk with kHashUnroll loads in flight,
    // a thread finding the entry of a product by bisection of the length prefix
    {
      const int64_t a0 = live ? a_rp[row] : 0;
      const int d = live ? (int)(a_rp[row + 1] - a0) : 0;
      int dmax = d;   // all groups of the workgroup walk in step (the barriers below are shared when GROUP > 64)
      if constexpr (GROUP > kWave) dmax = d; else {
#pragma unroll
        for (int sh = GROUP; sh < kWave; sh <<= 1) { const int o = __shfl_xor(dmax, sh, kWave); dmax = o > dmax ? o : dmax; }
      }
      int fresh = 0;
      for (int base = 0; base < dmax; base += GROUP) {
        const int e = base + gl;
        int64_t bs = 0;
        int len = 0;
        double av = 0.0;
        if (e < d) {
          const int k = a_col[a0 + e];
          const Run<int64_t, 2> bounds = load_run<int64_t, 2>(b_rp + k);
          bs = bounds.v[0];
          len = (int)(bounds.v[1] - bs);
          if (NUMERIC) av = (double)a_val[a0 + e];
        }
        int total;
        const int excl = group_excl_scan<GROUP>(len, total, part + g * (GROUP / kWave + 1));
        ent[gl] = HashEntry{excl, excl + len, bs};
        if (NUMERIC) pav[gl] = av;
        group_sync<GROUP>();
        const int nent = d - base < GROUP ? d - base : GROUP;
        const float per_product = total > 0 ? (float)nent / (float)total : 0.0f;   // entries per product
        for (int f0 = gl; f0 < total; f0 += GROUP * kHashUnroll) {
          int col[kHashUnroll];
          double prod[kHashUnroll];
#pragma unroll
          for (int u = 0; u < kHashUnroll; ++u) {
            const int f = f0 + u * GROUP;
            col[u] = -1;
            prod[u] = 0.0;
            if (f < total) {
              // entry of product f: the last one whose first product is <= f.  With B rows of similar length it
              // sits where the product's share of the total points, or next to it; otherwise it is bisected
              int lo = (int)((float)f * per_product);
              lo = lo < GROUP - 1 ? lo : GROUP - 1;
              HashEntry en = ent[lo];   // (one 16-byte read: first product, end, start in B)
              if (en.first > f) en = ent[--lo];
              else if (en.next <= f) en = ent[++lo];   // (f < total: an entry with products follows)
              if (en.first > f || en.next <= f) {
                int hi = GROUP;
                lo = 0;
                while (hi - lo > 1) {
                  const int mid = (lo + hi) >> 1;
                  if (ent[mid].first <= f) lo = mid; else hi = mid;
                }
                en = ent[lo];
              }
              const int64_t q = en.bs + (f - en.first);
              col[u] = b_col[q];
              if (NUMERIC) prod[u] = pav[lo] * (double)b_val[q];
            }
          }
#pragma unroll
          for (int u = 0; u < kHashUnroll; ++u) {
            if (col[u] >= 0) {
              int is_new;
              const int h = hash_find_or_insert<LOGH>(keys, col[u], is_new);
              fresh += is_new;
              if (NUMERIC) __hip_atomic_fetch_add(&vals[h], prod[u], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            }
          }
        }
        group_sync<GROUP>();
      }
      if (!NUMERIC && fresh) atomicAdd(&counters[g], fresh);
    }
    group_sync<GROUP>();
    if (!NUMERIC) {
      if (live && gl == 0) cnt[row] = counters[g];
    } else {
      // retrieve: the occupied slots move to the front of the table (through registers: a thread
      // reads its share of slots before anything is written back), the rest up to the next power of
      // two is padded, and only that many entries are sorted
      constexpr int kSlots = H / GROUP;
      int sk[kSlots];
      double sv[kSlots];
      int mine = 0;
#pragma unroll
      for (int q = 0; q < kSlots; ++q) {
        sk[q] = keys[gl * kSlots + q];
        sv[q] = vals[gl * kSlots + q];
        mine += sk[q] != kEmptyKey ? 1 : 0;
      }
      int filled;
      int at = group_excl_scan<GROUP>(mine, filled, part + g * (GROUP / kWave + 1));
      group_sync<GROUP>();
      // When column and slot number fit one 32-bit word together, only those words are sorted and a
      // sum is fetched through its slot number afterwards: a third of the LDS traffic of moving
      // (column, double) pairs through the network.
#pragma unroll
      for (int q = 0; q < kSlots; ++q)
        if (sk[q] != kEmptyKey) { keys[at] = packable ? (sk[q] << LOGH) | at : sk[q]; vals[at] = sv[q]; ++at; }
      int nsort = 2;
      while (nsort < filled) nsort <<= 1;
      for (int t = filled + gl; t < nsort; t += GROUP) keys[t] = kPadKey;
      group_sync<GROUP>();
      // (the usual sizes as compile-time constants, so that the network's stages unroll)
      if (packable) {
        if (nsort == H) bitonic_sort_lds<GROUP, H, double>(keys, nullptr, H, gl);
        else if (nsort == H / 2) bitonic_sort_lds<GROUP, H, double>(keys, nullptr, H / 2, gl);
        else if (nsort == H / 4) bitonic_sort_lds<GROUP, H, double>(keys, nullptr, H / 4, gl);
        else if (nsort == H / 8) bitonic_sort_lds<GROUP, H, double>(keys, nullptr, H / 8, gl);
        else bitonic_sort_lds<GROUP, H, double>(keys, nullptr, nsort, gl);
      } else {
        bitonic_sort_lds<GROUP, H, double>(keys, vals, nsort, gl);
      }
      if (live) {
        const int64_t out = c_rp[row];
        const int n = (int)(c_rp[row + 1] - out);
        for (int t = gl; t < n; t += GROUP) {
          const int kv = keys[t];
          c_col[out + t] = packable ? kv >> LOGH : kv;
          c_val[out + t] = (T)vals[packable ? kv & (H - 1) : t];
        }
      }
    }
    group_sync<GROUP>();
  }
}

template <int GROUP, int LOGH, bool NUMERIC>
constexpr size_t hash_lds_bytes() {
  return (size_t)(256 / GROUP) * (1u << LOGH) * (sizeof(int) + (NUMERIC ? sizeof(double) : 0)) + (256 / GROUP) * sizeof(int) + 8 +
         16 + (size_t)256 * (sizeof(HashEntry) + 8) + (size_t)(256 / GROUP) * (GROUP / kWave + 1) * 4;
}

}  // namespace spg
