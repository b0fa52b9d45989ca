// Staged-product workspace for rows with few intermediate products but an output too long
// for the hash workspace (at most staged_cap<T>() products, any number of columns).
// It is the coordinate-list workspace of the paper's section 5.2 kept entirely on chip:
//   insert : every product a_ik * b_kj of the row is appended to a coordinate list in LDS
//            with one coalesced pass over the B rows (no atomics: positions come from a
//            prefix over the piece lengths);
//   sort   : the column space is walked in windows of kStWinCols columns; the list entries
//            of a window set bits in a flag list, an exclusive prefix over the flag words
//            gives every present column its rank (a counting sort with boolean indexing);
//   merge  : the list entries add their values at the rank of their column;
//   compress: sums and decoded columns leave as contiguous runs of the row of C.
// After the single pass over global memory all work is LDS-only, so a row costs one global
// round trip however wide its columns are spread.  B rows need not be sorted.
#pragma once
#include "common.hpp"
#include "dense_kernels.hpp"

namespace spg {

constexpr int kStWinCols = 131072;
constexpr int kStWinShift = 17;
constexpr int kStWinWords = kStWinCols / 32;
constexpr int kStMaxWindows = 64;   // occupancy mask of the windows: rows of wider matrices take the tile route

template <typename T>
constexpr int staged_cap() { return sizeof(T) == 4 ? 6144 : 5120; }

// Pieces of the segment being staged (aliases the window area).
struct StagePieces {
  long long s[kDenseThreads];     // first B entry of the piece
  int cpre[kDenseThreads + 1];    // exclusive prefix of chunk counts
  int epre[kDenseThreads];        // exclusive prefix of lengths
  int len[kDenseThreads];
};

template <typename T>
constexpr size_t staged_lds() {
  const size_t list = (size_t)staged_cap<T>() * (4 + sizeof(T));
  const size_t window = (size_t)kStWinWords * 8 + (size_t)staged_cap<T>() * 12;
  return list + (window > sizeof(StagePieces) + kDenseThreads * sizeof(T) ? window : sizeof(StagePieces) + kDenseThreads * sizeof(T)) + 256;
}

// Exclusive scans of three ints over the workgroup, with totals.  Contains barriers.
__device__ __forceinline__ void block_excl_scan3(int a, int b, int c, int& ea, int& eb, int& ec, int& ta, int& tb, int& tc, int* red) {
  const int wave = threadIdx.x >> 6;
  const int ia = wave_incl_scan(a), ib = wave_incl_scan(b), ic = wave_incl_scan(c);
  __syncthreads();
  if (lane_id() == kWave - 1) { red[wave] = ia; red[kDenseWaves + wave] = ib; red[2 * kDenseWaves + wave] = ic; }
  __syncthreads();
  int pa = 0, pb = 0, pc = 0;
  ta = 0; tb = 0; tc = 0;
#pragma unroll
  for (int w = 0; w < kDenseWaves; ++w) {
    const int va = red[w], vb = red[kDenseWaves + w], vc = red[2 * kDenseWaves + w];
    if (w < wave) { pa += va; pb += vb; pc += vc; }
    ta += va; tb += vb; tc += vc;
  }
  ea = pa + ia - a;
  eb = pb + ib - b;
  ec = pc + ic - c;
}

template <typename T>
__global__ __launch_bounds__(kDenseThreads) void k_num_staged(const int* __restrict__ perm, Control* ctl,
                                                              const int64_t* __restrict__ a_rp, const int32_t* __restrict__ a_col,
                                                              const T* __restrict__ a_val, const int64_t* __restrict__ b_rp,
                                                              const int32_t* __restrict__ b_col, const T* __restrict__ b_val,
                                                              int64_t n_cols, const int64_t* __restrict__ c_rp,
                                                              int32_t* __restrict__ c_col, T* __restrict__ c_val) {
  constexpr int CAP = staged_cap<T>();
  extern __shared__ __align__(16) unsigned char smem[];
  int* st_col = reinterpret_cast<int*>(smem);                               // CAP columns of the products
  T* st_val = reinterpret_cast<T*>(smem + (size_t)CAP * 4);                 // CAP products
  unsigned char* area = smem + (size_t)CAP * (4 + sizeof(T));
  // while staging
  StagePieces* sp = reinterpret_cast<StagePieces*>(area);
  T* p_av = reinterpret_cast<T*>(area + sizeof(StagePieces));
  // while sorting / merging
  uint2* fc = reinterpret_cast<uint2*>(area);                               // per flag word: bits, rank of its first column
  double* acc = reinterpret_cast<double*>(area + (size_t)kStWinWords * 8);  // CAP sums, by rank
  int* stage = reinterpret_cast<int*>(area + (size_t)kStWinWords * 8 + (size_t)CAP * 8);   // CAP columns, by rank
  int* misc = reinterpret_cast<int*>(smem + staged_lds<T>() - 256);         // 3 * 16 scan partials, row, window mask (2 words)
  int* red = misc;
  int* s_row = misc + 48;
  unsigned* s_mask = reinterpret_cast<unsigned*>(misc + 50);
  if (ctl->error) return;
  const int tid = threadIdx.x, wave = uni(tid >> 6), lane = tid & 63;
  const unsigned first = ctl->offset[1][4];
  const unsigned nrows = ctl->offset[1][5] - first;
  const int nwin = (int)((n_cols + kStWinCols - 1) >> kStWinShift);
  while (true) {
    __syncthreads();
    if (tid == 0) {
      const unsigned idx = atomicAdd(&ctl->work[2], 1u);
      *s_row = idx < nrows ? perm[first + idx] : -1;
      s_mask[0] = 0; s_mask[1] = 0;
    }
    __syncthreads();
    const int row = *s_row;
    if (row < 0) break;
    const int64_t a0 = a_rp[row];
    const int d = (int)(a_rp[row + 1] - a0);
    int64_t out = c_rp[row];
    // ---- insert: stage every product of the row
    int total = 0;
    unsigned m0 = 0, m1 = 0;   // windows that this thread's products fall into
    for (int base = 0; base < d; base += kDenseThreads) {
      const int e = base + tid;
      long long s = 0;
      int len = 0;
      T av = T(0);
      if (e < d) {
        const int k = a_col[a0 + e];
        av = a_val[a0 + e];
        const Run<int64_t, 2> bounds = load_run<int64_t, 2>(b_rp + k);
        s = bounds.v[0];
        len = (int)(bounds.v[1] - s);
      }
      int idx, cpre, epre, np, nchunks, nel;
      block_excl_scan3(len > 0 ? 1 : 0, (len + kWave - 1) >> 6, len, idx, cpre, epre, np, nchunks, nel, red);
      if (len > 0) {
        sp->s[idx] = s;
        sp->cpre[idx] = cpre;
        sp->epre[idx] = total + epre;
        sp->len[idx] = len;
        p_av[idx] = av;
      }
      if (tid == 0) sp->cpre[np] = nchunks;
      __syncthreads();
      np = uni(np);
      nchunks = uni(nchunks);
      // chunks of 64 elements are dealt to the waves in contiguous shares
      const int per = (nchunks + kDenseWaves - 1) / kDenseWaves;
      int c = wave * per;
      const int cend = c + per < nchunks ? c + per : nchunks;
      if (c < cend) {
        int p;
        {
          int lo = 0, hi = np;   // last piece whose first chunk is <= c
          while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (uni(sp->cpre[mid]) <= c) lo = mid; else hi = mid;
          }
          p = lo;
        }
        int cfirst = uni(sp->cpre[p]), cnext = uni(sp->cpre[p + 1]);
        int plen = uni(sp->len[p]), pbase = uni(sp->epre[p]);
        long long ps = uni64(sp->s[p]);
        T pav = p_av[p];
        for (; c < cend; c += kChunkUnroll) {
          int col[kChunkUnroll], pos[kChunkUnroll];
          T bv[kChunkUnroll], au[kChunkUnroll];
#pragma unroll
          for (int u = 0; u < kChunkUnroll; ++u) {
            const int cu = c + u;
            col[u] = -1;
            pos[u] = 0;
            bv[u] = T(0);
            au[u] = pav;
            if (cu < cend) {
              if (cu >= cnext) {
                ++p;
                cfirst = cnext;
                cnext = uni(sp->cpre[p + 1]);
                plen = uni(sp->len[p]);
                pbase = uni(sp->epre[p]);
                ps = uni64(sp->s[p]);
                pav = p_av[p];
              }
              const int off = (cu - cfirst) * kWave + lane;
              if (off < plen) {
                col[u] = b_col[ps + off];
                bv[u] = b_val[ps + off];
                pos[u] = pbase + off;
              }
              au[u] = pav;
            }
          }
#pragma unroll
          for (int u = 0; u < kChunkUnroll; ++u) {
            if (col[u] >= 0) {
              st_col[pos[u]] = col[u];
              st_val[pos[u]] = au[u] * bv[u];
              const int w = col[u] >> kStWinShift;
              if (w < 32) m0 |= 1u << w; else m1 |= 1u << (w & 31);
            }
          }
        }
      }
      total += uni(nel);
      __syncthreads();
    }
    // windows that hold products
#pragma unroll
    for (int sh = 1; sh < kWave; sh <<= 1) { m0 |= __shfl_xor(m0, sh, kWave); m1 |= __shfl_xor(m1, sh, kWave); }
    if (lane == 0) { if (m0) atomicOr(&s_mask[0], m0); if (m1) atomicOr(&s_mask[1], m1); }
    __syncthreads();
    unsigned long long wmask = ((unsigned long long)s_mask[1] << 32) | s_mask[0];
    // ---- sort / merge / compress, one window at a time
    while (wmask) {
      const int w = __ffsll((long long)wmask) - 1;
      wmask &= wmask - 1;
      (void)nwin;
      const int w_lo = w << kStWinShift;
      for (int i = tid; i < kStWinWords; i += kDenseThreads) fc[i] = make_uint2(0u, 0u);
      __syncthreads();
      for (int j = tid; j < total; j += kDenseThreads) {
        const int c = st_col[j];
        if ((c >> kStWinShift) == w) {
          const int rel = c - w_lo;
          atomicOr(&fc[rel >> 5].x, 1u << (rel & 31));
        }
      }
      __syncthreads();
      // exclusive prefix of the flag-word populations: wave v owns words [256 v, 256 v + 256)
      constexpr int kPerWave = kStWinWords / kDenseWaves;
      const int wbase = wave * kPerWave;
      int mine = 0;
#pragma unroll
      for (int i = 0; i < kPerWave; i += kWave) mine += __popc(fc[wbase + i + lane].x);
      mine = wave_sum(mine);
      if (lane == 0) red[wave] = mine;
      __syncthreads();
      int running = 0, count = 0;
#pragma unroll
      for (int v = 0; v < kDenseWaves; ++v) { const int r = red[v]; running += v < wave ? r : 0; count += r; }
#pragma unroll
      for (int i = 0; i < kPerWave; i += kWave) {
        const int wi = wbase + i + lane;
        unsigned bits = fc[wi].x;
        const int c = __popc(bits);
        const int incl = wave_incl_scan(c);
        int excl = running + incl - c;
        running += __builtin_amdgcn_readlane(incl, kWave - 1);
        fc[wi].y = (unsigned)excl;
        const int cbase = w_lo + wi * 32;
        while (bits) {
          const int b = __ffs((int)bits) - 1;
          bits &= bits - 1;
          stage[excl++] = cbase + b;
        }
      }
      for (int r = tid; r < count; r += kDenseThreads) acc[r] = 0.0;
      __syncthreads();
      for (int j = tid; j < total; j += kDenseThreads) {
        const int c = st_col[j];
        if ((c >> kStWinShift) == w) {
          const int rel = c - w_lo;
          const uint2 f = fc[rel >> 5];
          const int rank = (int)f.y + __popc(f.x & ((1u << (rel & 31)) - 1u));
          __hip_atomic_fetch_add(&acc[rank], (double)st_val[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
      }
      __syncthreads();
      for (int r = tid; r < count; r += kDenseThreads) {
        c_val[out + r] = (T)acc[r];
        c_col[out + r] = stage[r];
      }
      out += count;
      __syncthreads();
    }
  }
}

}  // namespace spg
