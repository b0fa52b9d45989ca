// Sorted-list (sparse) workspace for short rows: every intermediate product of a row is
// appended to a small coordinate list in LDS (insert), the list is put in column order (sort:
// a bitonic network for columns alone, a count of the entries before each entry when values
// travel along) and runs of equal columns are summed (merge).  This is the expand / sort /
// reduce-by-key policy of the paper's table of library algorithms (section 4.4) run at
// wavefront level, one row per GROUP lanes.
#pragma once
#include "common.hpp"

namespace spg {

// Number of list entries before entry e with key k: those with a smaller key, and with TIE also those
// with the same key at an earlier position (without TIE the keys are distinct).  The lanes of a group
// read the list together, four keys at a time (one address for the group: no bank conflicts).
template <bool TIE>
__device__ __forceinline__ int count_before(const int* keys, int nscan, unsigned k, int e) {
  int r = 0;
#pragma unroll 2
  for (int j = 0; j < nscan; j += 4) {
    const int4 q = *reinterpret_cast<const int4*>(&keys[j]);
    r += (unsigned)q.x < k + ((TIE && j + 0 < e) ? 1u : 0u) ? 1 : 0;
    r += (unsigned)q.y < k + ((TIE && j + 1 < e) ? 1u : 0u) ? 1 : 0;
    r += (unsigned)q.z < k + ((TIE && j + 2 < e) ? 1u : 0u) ? 1 : 0;
    r += (unsigned)q.w < k + ((TIE && j + 3 < e) ? 1u : 0u) ? 1 : 0;
  }
  return r;
}

// GROUP lanes per row (16 or 64), list capacity CAP = 2 * GROUP products.
// NUMERIC = false: writes the number of distinct columns to cnt[row].
// NUMERIC = true : writes the merged (column, value) run at c_rp[row]; pack != 0: every column shifted
//                  left by log2(CAP) stays below the padding key, so a key can carry its list position.
template <int GROUP, int CAP, typename T, bool NUMERIC>
__global__ __launch_bounds__(256) void k_esc(const int* __restrict__ perm, const Control* __restrict__ ctl, int phase, int bin,
                                              const int64_t* __restrict__ a_rp, const int32_t* __restrict__ a_col,
                                              const T* __restrict__ a_val, const int64_t* __restrict__ b_rp,
                                              const int32_t* __restrict__ b_col, const T* __restrict__ b_val,
                                              int* __restrict__ cnt, const int64_t* __restrict__ c_rp,
                                              int32_t* __restrict__ c_col, T* __restrict__ c_val, int pack, int64_t b_nnz) {
  static_assert(CAP == 2 * GROUP, "each lane owns two list positions");
  constexpr int kGroups = 256 / GROUP;
  constexpr int kLogCap = CAP == 32 ? 5 : 7;
  static_assert((1 << kLogCap) == CAP, "list capacities 32 and 128");
  const int shift = (NUMERIC && pack) ? kLogCap : 0;   // a numeric key: (column << shift) | position
  const int pmask = (NUMERIC && pack) ? CAP - 1 : 0;
  constexpr int kSpreadMax = 16;   // A entries up to which a wave deals a row's products, not its entries, to its lanes
  __shared__ __align__(16) int s_keys[kGroups][CAP];
  __shared__ double s_vals[NUMERIC ? kGroups : 1][NUMERIC ? CAP : 1];
  if (ctl->error) return;
  const unsigned first = ctl->offset[phase][bin];
  const unsigned nrows = ctl->offset[phase][bin + 1] - first;
  const int g = threadIdx.x / GROUP;   // group inside the workgroup
  const int gl = threadIdx.x % GROUP;  // lane inside the group
  int* keys = s_keys[g];
  double* vals = NUMERIC ? s_vals[g] : nullptr;
  const unsigned ngroups = gridDim.x * kGroups;
  // every wave iterates the same number of times so that the shuffles below always see
  // all 64 lanes; groups past the end of the bin run on an empty row
  const unsigned rounds = (nrows + ngroups - 1) / ngroups;
  for (unsigned r = 0; r < rounds; ++r) {
    const unsigned slot = r * ngroups + blockIdx.x * kGroups + g;
    const bool live = slot < nrows;
    const int row = live ? perm[first + slot] : 0;
    const int64_t a0 = live ? a_rp[row] : 0;
    const int d = live ? (int)(a_rp[row + 1] - a0) : 0;
    // ---- insert: lane-per-A-entry, positions from a running prefix of B row lengths
    int filled = 0;
    int dmax = d;
#pragma unroll
    for (int s = GROUP; s < kWave; s <<= 1) { int o = __shfl_xor(dmax, s, kWave); dmax = o > dmax ? o : dmax; }
    for (int c = 0; c < dmax; c += GROUP) {
      const int e = c + gl;
      int64_t bs = 0; int len = 0; double av = 0.0;
      if (e < d) {
        const int k = a_col[a0 + e];
        const Run<int64_t, 2> bounds = load_run<int64_t, 2>(b_rp + k);
        bs = bounds.v[0];
        len = (int)(bounds.v[1] - bs);
        if (NUMERIC) av = (double)a_val[a0 + e];
      }
      const int incl = group_incl_scan<GROUP>(len);
      if constexpr (GROUP == kWave) {
        // one row per wave: with few A entries most lanes would idle while a few walk their B rows, so
        // the products themselves are dealt to the lanes (at most two each); a lane finds the entry of
        // its product by counting the entries that end at or before it
        const int nent = __builtin_amdgcn_readfirstlane(d - c);
        if (nent <= kSpreadMax) {
          const int batch = __builtin_amdgcn_readlane(incl, kWave - 1);
          int cc[2];
          T vv[2];
          double aa[2];
#pragma unroll
          for (int u = 0; u < 2; ++u) {
            const int t = gl + u * kWave;
            const bool ok = t < batch;
            int ent = 0;
            for (int x = 0; x < nent; ++x) ent += __builtin_amdgcn_readlane(incl, x) <= t ? 1 : 0;
            if (!ok) ent = 0;
            const int ent_first = __shfl(incl - len, ent, kWave);
            const long long ent_bs = __shfl((long long)bs, ent, kWave);
            aa[u] = NUMERIC ? __shfl(av, ent, kWave) : 0.0;
            const long long q = ent_bs + (t - ent_first);
            cc[u] = ok ? b_col[q] : 0;
            vv[u] = (NUMERIC && ok) ? b_val[q] : T(0);
          }
#pragma unroll
          for (int u = 0; u < 2; ++u) {
            const int t = gl + u * kWave;
            if (t < batch) {
              keys[filled + t] = (cc[u] << shift) | ((filled + t) & pmask);
              if (NUMERIC) vals[filled + t] = aa[u] * (double)vv[u];
            }
          }
          filled += batch;
          continue;
        }
      }
      int pos = filled + incl - len;
      for (int t0 = 0; t0 < len; t0 += 4) {   // four loads in flight per lane
        int cc[4];
        T vv[4];
        if (bs + t0 + 4 <= b_nnz) {   // four elements exist behind the position, whatever the row's length
          const Run<int32_t, 4> qc = load_run<int32_t, 4>(b_col + bs + t0);
#pragma unroll
          for (int u = 0; u < 4; ++u) cc[u] = qc.v[u];
          if (NUMERIC) {
            const Run<T, 4> qv = load_run<T, 4>(b_val + bs + t0);
#pragma unroll
            for (int u = 0; u < 4; ++u) vv[u] = qv.v[u];
          }
        } else {
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const bool ok = t0 + u < len;
            cc[u] = ok ? b_col[bs + t0 + u] : 0;
            if (NUMERIC) vv[u] = ok ? b_val[bs + t0 + u] : T(0);
          }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          if (t0 + u < len) {
            keys[pos + t0 + u] = (cc[u] << shift) | ((pos + t0 + u) & pmask);
            if (NUMERIC) vals[pos + t0 + u] = av * (double)vv[u];
          }
        }
      }
      filled += __shfl(incl, GROUP - 1, GROUP);
    }
    // pad the tail so that it sorts behind every real column
    for (int t = filled + gl; t < CAP; t += GROUP) keys[t] = kPadKey;
    group_sync<GROUP>();
    // ---- sort and merge.  With values, an exchange in a sorting network would carry 12 bytes through
    // LDS per entry and stage; instead every lane looks at its two entries (positions gl and gl + GROUP;
    // the second only when some row of the wave has that many) against the whole list.
    const int e0 = gl, e1 = gl + GROUP;
    const bool two = __any(filled > GROUP);
    int nscan = CAP;
    if constexpr (GROUP == kWave) nscan = __builtin_amdgcn_readfirstlane((filled + 3) & ~3);
    if constexpr (!NUMERIC) {
      // symbolic: the columns alone go through the bitonic network (4 bytes per entry and stage); a
      // position is a head when its column differs from its left neighbour
      // (half the network when no row of the wave reaches into its second half; both sizes are compile-time
      // constants so that the stages unroll)
      if (two) bitonic_sort_lds<GROUP, CAP, double>(keys, static_cast<double*>(nullptr), CAP, gl);
      else bitonic_sort_lds<GROUP, CAP, double>(keys, static_cast<double*>(nullptr), GROUP, gl);
      const int i0 = 2 * gl, i1 = 2 * gl + 1;
      const int k0 = keys[i0], k1 = keys[i1];
      const int kprev = i0 > 0 ? keys[i0 - 1] : -1;
      const int heads = ((i0 < filled && k0 != kprev) ? 1 : 0) + ((i1 < filled && k1 != k0) ? 1 : 0);
      const int total = __shfl(group_incl_scan<GROUP>(heads), GROUP - 1, GROUP);
      if (live && gl == 0) cnt[row] = total;
    } else {
      // numeric: an entry's place in column order is the number of entries before it (smaller column,
      // or the same column and an earlier position); entries go there, then runs of equal columns are summed
      const unsigned ka = (unsigned)keys[e0], kb = (unsigned)keys[e1];
      const double va = vals[e0], vb = vals[e1];
      int ra = 0, rb = 0;
      if (pack) {
        ra = count_before<false>(keys, nscan, ka, e0);
        if (two) rb = count_before<false>(keys, nscan, kb, e1);
      } else {
        ra = count_before<true>(keys, nscan, ka, e0);
        if (two) rb = count_before<true>(keys, nscan, kb, e1);
      }
      group_sync<GROUP>();
      // (positions from `filled` on hold padding and stay as they are)
      if (e0 < filled) { keys[ra] = (int)(ka >> shift); vals[ra] = va; }
      if (e1 < filled) { keys[rb] = (int)(kb >> shift); vals[rb] = vb; }
      group_sync<GROUP>();
      // a list position is a head when its column differs from its left neighbour
      const int i0 = 2 * gl, i1 = 2 * gl + 1;
      const int k0 = keys[i0], k1 = keys[i1];
      const int kprev = i0 > 0 ? keys[i0 - 1] : -1;
      const int h0 = (i0 < filled && k0 != kprev) ? 1 : 0;
      const int h1 = (i1 < filled && k1 != k0) ? 1 : 0;
      const int incl = group_incl_scan<GROUP>(h0 + h1);
      if (live) {
        const int64_t out = c_rp[row];
        int rank = incl - (h0 + h1);
        if (h0) {
          double s = vals[i0];
          for (int t = i0 + 1; t < filled && keys[t] == k0; ++t) s += vals[t];
          c_col[out + rank] = k0;
          c_val[out + rank] = (T)s;
          ++rank;
        }
        if (h1) {
          double s = vals[i1];
          for (int t = i1 + 1; t < filled && keys[t] == k1; ++t) s += vals[t];
          c_col[out + rank] = k1;
          c_val[out + rank] = (T)s;
        }
      }
    }
    group_sync<GROUP>();
  }
}

}  // namespace spg
