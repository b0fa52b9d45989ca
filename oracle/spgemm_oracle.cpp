// CPU checker for row-wise sparse x sparse products.  TEST INFRASTRUCTURE ONLY:
// nothing on the product path may link, load or call this file; it shares no
// code with the GPU library.
//
// What it computes is the plain definition of the product the paper states in
// section 2.1 (A_ij = sum_k B_ik C_kj; here named C = A * B), traversed in the
// row-wise loop order i -> k -> j of section 2.2 (Gustavson).  The workspace is
// one ordered map per output row: every intermediate product is inserted, equal
// coordinates are summed (the "deduplication" behaviour of section 4.3), and an
// in-order walk of the map emits the row in ascending column order.  A map is
// the one-array "sort on every insert" workspace of section 7.5.  Output
// conventions follow the compress stage of the outer-product listing
// (section 4.3): 0-based, rowptr[0] = 0, an empty row repeats its neighbour's
// offset, every inserted coordinate is kept even if its sum is exactly zero.
//
// Arithmetic: products and sums are carried in double for both input types
// (a product of two floats is exact in double); k runs in A's stored order,
// j in B's stored order.  Beside each sum the map carries S_ij = sum |a*b|,
// the scale against which callers test a relative tolerance.
//
// Pinned by tests/test_oracle_pins.py: dense triple-loop brute force on tiny
// operands (unsorted and duplicated inputs included), identity / permutation /
// diagonal products that must be bit-identical, the 27-point stencil closed
// forms, the count invariants, and the paper's (2,2,3)+(2,2,8) example.
// The paper's own worked figure example is not reproducible from its text:
// parity unpinned for that one example.
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <map>
#include <vector>
#include <utility>
#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

struct Slot { double sum; double absum; };

inline double load_val(const void* v, int is_f32, int64_t p) {
  return is_f32 ? (double)((const float*)v)[p] : ((const double*)v)[p];
}

}  // namespace

extern "C" {

// nr rows of C = A*B: row r of the output is row row_ids[r] of the product, or row
// row_lo + r when row_ids is null.  On return *out_col / *out_val / *out_abs are
// malloc'ed arrays of length sum(out_cnt) (release with oracle_free), row after row.
// out_cnt[r] = number of entries of output row r, out_ip[r] = its intermediate products.
// Returns 0, or -1 on allocation failure / bad arguments.
int oracle_spgemm_rows(int64_t nr, int64_t row_lo, const int64_t* row_ids,
                       const int64_t* a_rowptr, const int32_t* a_col, const void* a_val,
                       const int64_t* b_rowptr, const int32_t* b_col, const void* b_val,
                       int is_f32, int nthreads,
                       int64_t* out_cnt, int64_t* out_ip,
                       int32_t** out_col, double** out_val, double** out_abs) {
  if (nr < 0 || !a_rowptr || !b_rowptr || !out_cnt || !out_ip) return -1;
  std::vector<std::vector<std::pair<int32_t, Slot>>> rows((size_t)nr);
#ifdef _OPENMP
  if (nthreads > 0) omp_set_num_threads(nthreads);
#endif
#pragma omp parallel for schedule(dynamic, 16)
  for (int64_t r = 0; r < nr; ++r) {
    const int64_t i = row_ids ? row_ids[r] : row_lo + r;
    std::map<int32_t, Slot> acc;
    int64_t ip = 0;
    for (int64_t p = a_rowptr[i]; p < a_rowptr[i + 1]; ++p) {
      const int32_t k = a_col[p];
      const double a = a_val ? load_val(a_val, is_f32, p) : 1.0;
      for (int64_t q = b_rowptr[k]; q < b_rowptr[k + 1]; ++q) {
        const int32_t j = b_col[q];
        const double prod = a * (b_val ? load_val(b_val, is_f32, q) : 1.0);
        auto it = acc.find(j);
        if (it == acc.end()) {
          acc.emplace(j, Slot{prod, prod < 0 ? -prod : prod});
        } else {
          it->second.sum += prod;
          it->second.absum += (prod < 0 ? -prod : prod);
        }
        ++ip;
      }
    }
    out_ip[r] = ip;
    out_cnt[r] = (int64_t)acc.size();
    rows[(size_t)r].assign(acc.begin(), acc.end());
  }
  int64_t total = 0;
  for (int64_t r = 0; r < nr; ++r) total += out_cnt[r];
  int32_t* c = (int32_t*)malloc((size_t)(total > 0 ? total : 1) * sizeof(int32_t));
  double* v = (double*)malloc((size_t)(total > 0 ? total : 1) * sizeof(double));
  double* s = (double*)malloc((size_t)(total > 0 ? total : 1) * sizeof(double));
  if (!c || !v || !s) { free(c); free(v); free(s); return -1; }
  int64_t o = 0;
  for (int64_t r = 0; r < nr; ++r) {
    for (const auto& e : rows[(size_t)r]) {
      c[o] = e.first; v[o] = e.second.sum; s[o] = e.second.absum; ++o;
    }
    std::vector<std::pair<int32_t, Slot>>().swap(rows[(size_t)r]);
  }
  *out_col = c; *out_val = v; *out_abs = s;
  return 0;
}

void oracle_free(void* p) { free(p); }

int oracle_max_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

}  // extern "C"
