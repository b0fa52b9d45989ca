// Sorted-list (sparse) workspace for short rows: every intermediate product of a row is
// appended to a small coordinate list in LDS (insert), the list is sorted by column with
// a bitonic network (sort) and runs of equal columns are summed (merge).  This is the
// expand / sort / reduce-by-key policy of the paper's table of library algorithms
// (section 4.4) run at wavefront level, one row per GROUP lanes.
#pragma once
#include "common.hpp"

namespace spg {

// GROUP lanes per row (16 or 64), list capacity CAP = 2 * GROUP products.
// NUMERIC = false: writes the number of distinct columns to cnt[row].
// NUMERIC = true : writes the merged (column, value) run at c_rp[row].
template <int GROUP, int CAP, typename T, bool NUMERIC>
__global__ __launch_bounds__(256) void k_esc(const int* __restrict__ perm, const Control* __restrict__ ctl, int phase, int bin,
                                              const int64_t* __restrict__ a_rp, const int32_t* __restrict__ a_col,
                                              const T* __restrict__ a_val, const int64_t* __restrict__ b_rp,
                                              const int32_t* __restrict__ b_col, const T* __restrict__ b_val,
                                              int* __restrict__ cnt, const int64_t* __restrict__ c_rp,
                                              int32_t* __restrict__ c_col, T* __restrict__ c_val) {
  static_assert(CAP == 2 * GROUP, "each lane owns two list positions");
  constexpr int kGroups = 256 / GROUP;
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
        bs = b_rp[k];
        len = (int)(b_rp[k + 1] - bs);
        if (NUMERIC) av = (double)a_val[a0 + e];
      }
      const int incl = group_incl_scan<GROUP>(len);
      int pos = filled + incl - len;
      for (int t0 = 0; t0 < len; t0 += 4) {   // four loads in flight per lane
        int cc[4];
        T vv[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const bool ok = t0 + u < len;
          cc[u] = ok ? b_col[bs + t0 + u] : 0;
          if (NUMERIC) vv[u] = ok ? b_val[bs + t0 + u] : T(0);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          if (t0 + u < len) {
            keys[pos + t0 + u] = cc[u];
            if (NUMERIC) vals[pos + t0 + u] = av * (double)vv[u];
          }
        }
      }
      filled += __shfl(incl, GROUP - 1, GROUP);
    }
    // pad the tail so that it sorts behind every real column
    for (int t = filled + gl; t < CAP; t += GROUP) keys[t] = kPadKey;
    group_sync<GROUP>();
    // ---- sort.  Columns alone go through the bitonic network.  With values, an exchange in the network
    // would move 12 bytes through LDS per entry and stage; there an entry's place is counted instead:
    // the number of entries before it (smaller column, or the same column and an earlier position);
    // every lane counts for its two entries while the group reads the list four keys at a time (one
    // address for the whole group: no bank conflicts)
    if constexpr (!NUMERIC) {
      bitonic_sort_lds<GROUP, CAP, double>(keys, vals, CAP, gl);
    } else {
      const int e0 = gl, e1 = gl + GROUP;
      const unsigned ka = (unsigned)keys[e0], kb = (unsigned)keys[e1];
      const double va = vals[e0], vb = vals[e1];
      int nscan = CAP;
      if constexpr (GROUP == kWave) nscan = __builtin_amdgcn_readfirstlane((filled + 3) & ~3);
      int ra = 0, rb = 0;
#pragma unroll 2
      for (int j = 0; j < nscan; j += 4) {
        const int4 q4 = *reinterpret_cast<const int4*>(&keys[j]);
        const unsigned q[4] = {(unsigned)q4.x, (unsigned)q4.y, (unsigned)q4.z, (unsigned)q4.w};
#pragma unroll
        for (int x = 0; x < 4; ++x) {
          ra += q[x] < ka + (j + x < e0 ? 1u : 0u) ? 1 : 0;
          rb += q[x] < kb + (j + x < e1 ? 1u : 0u) ? 1 : 0;
        }
      }
      group_sync<GROUP>();
      // (positions from `filled` on hold padding and stay as they are)
      if (e0 < filled) { keys[ra] = (int)ka; vals[ra] = va; }
      if (e1 < filled) { keys[rb] = (int)kb; vals[rb] = vb; }
      group_sync<GROUP>();
    }
    // ---- merge: a list position is a head when its column differs from its left neighbour
    const int i0 = 2 * gl, i1 = 2 * gl + 1;
    const int k0 = keys[i0], k1 = keys[i1];
    const int kprev = i0 > 0 ? keys[i0 - 1] : -1;
    const int h0 = (i0 < filled && k0 != kprev) ? 1 : 0;
    const int h1 = (i1 < filled && k1 != k0) ? 1 : 0;
    const int incl = group_incl_scan<GROUP>(h0 + h1);
    const int total = __shfl(incl, GROUP - 1, GROUP);
    if (!NUMERIC) {
      if (live && gl == 0) cnt[row] = total;
    } else if (live) {
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
    group_sync<GROUP>();
  }
}

}  // namespace spg
