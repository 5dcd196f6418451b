// Host-side construction of a partition's local view (Eq. 2; appendix
// P = P_in + P_out): halo list, relabelled CSR [P_in | P_out] with A_hat
// values from global degrees, per-row split, transposed halo block.
//
// Because a row of the global CSR is ascending in global id and relabelling is
// monotone inside the local class and inside the halo class, the canonical row
// (ascending relabelled id) is: local neighbours in input order with the
// self-loop merged in at its rank, followed by halo neighbours in input order.
// No sort is needed anywhere; everything is counting passes.
#include <cmath>
#include <cstdint>
#include <vector>

#include "../../include/sat.h"

namespace {

struct Scan {
  int64_t n_local = 0, n_halo = 0, nnz = 0, nnz_halo = 0;
  std::vector<uint8_t> halo_mark;  // [N] 1 if the node is in the halo of m
};

sat_status scan(int64_t N, const int64_t* g_rowptr, const int32_t* g_col, const int32_t* part,
                int32_t m, Scan* out) {
  if (N < 0 || N > INT32_MAX || !g_rowptr || !part || (!g_col && N > 0 && g_rowptr[N] > 0))
    return SAT_EINVAL;
  out->halo_mark.assign(static_cast<size_t>(N), 0);
  for (int64_t g = 0; g < N; ++g) {
    if (part[g] != m) continue;
    const int64_t s = g_rowptr[g], e = g_rowptr[g + 1];
    if (s < 0 || e < s) return SAT_EINVAL;
    out->n_local += 1;
    out->nnz += (e - s) + 1;
    int64_t prev = -1;
    for (int64_t k = s; k < e; ++k) {
      const int64_t c = g_col[k];
      if (c < 0 || c >= N || c == g || c <= prev) return SAT_EINVAL;
      prev = c;
      if (part[c] != m) {
        out->nnz_halo += 1;
        if (!out->halo_mark[c]) {
          out->halo_mark[c] = 1;
          out->n_halo += 1;
        }
      }
    }
  }
  return SAT_OK;
}

inline float inv_sqrt_deg(int64_t deg) {
  return static_cast<float>(1.0 / std::sqrt(1.0 + static_cast<double>(deg)));
}

}  // namespace

extern "C" sat_status sat_partition_view_sizes(int64_t N, const int64_t* g_rowptr,
                                               const int32_t* g_col, const int32_t* part,
                                               int32_t m, int64_t* n_local, int64_t* n_halo,
                                               int64_t* nnz, int64_t* nnz_halo) {
  if (!n_local || !n_halo || !nnz || !nnz_halo) return SAT_EINVAL;
  Scan sc;
  sat_status st = scan(N, g_rowptr, g_col, part, m, &sc);
  if (st != SAT_OK) return st;
  *n_local = sc.n_local;
  *n_halo = sc.n_halo;
  *nnz = sc.nnz;
  *nnz_halo = sc.nnz_halo;
  return SAT_OK;
}

extern "C" sat_status sat_partition_view_build(int64_t N, const int64_t* g_rowptr,
                                               const int32_t* g_col, const int32_t* g_deg,
                                               const int32_t* part, int32_t m,
                                               int32_t* local_ids, int32_t* halo_ids,
                                               int64_t* rowptr, int64_t* split, int32_t* col,
                                               float* val, int64_t* h_colptr, int32_t* h_row,
                                               float* h_val, float* h_self) {
  Scan sc;
  sat_status st = scan(N, g_rowptr, g_col, part, m, &sc);
  if (st != SAT_OK) return st;
  if (!rowptr || !h_colptr) return SAT_EINVAL;
  if (sc.n_local > 0 && (!local_ids || !split || !col || !val)) return SAT_EINVAL;
  if (sc.n_halo > 0 && (!halo_ids || !h_row || !h_val || !h_self)) return SAT_EINVAL;
  if (g_deg)
    for (int64_t g = 0; g < N; ++g)
      if (g_deg[g] < 0) return SAT_EINVAL;

  // relabel: local rank / n_local + halo rank, both in ascending global id
  std::vector<int32_t> relabel(static_cast<size_t>(N), -1);
  {
    int32_t nl = 0, nh = 0;
    for (int64_t g = 0; g < N; ++g) {
      if (part[g] == m) {
        local_ids[nl] = static_cast<int32_t>(g);
        relabel[g] = nl++;
      } else if (sc.halo_mark[g]) {
        halo_ids[nh] = static_cast<int32_t>(g);
        relabel[g] = static_cast<int32_t>(sc.n_local) + nh++;
      }
    }
  }
  auto isd = [&](int64_t g) {
    return inv_sqrt_deg(g_deg ? static_cast<int64_t>(g_deg[g]) : g_rowptr[g + 1] - g_rowptr[g]);
  };

  for (int64_t u = 0; u <= sc.n_halo; ++u) h_colptr[u] = 0;
  int64_t w = 0;
  rowptr[0] = 0;
  for (int64_t i = 0; i < sc.n_local; ++i) {
    const int64_t g = local_ids[i];
    const float isd_g = isd(g);
    const int64_t s = g_rowptr[g], e = g_rowptr[g + 1];
    bool self_done = false;
    for (int64_t k = s; k < e; ++k) {       // local columns, self-loop merged in
      const int64_t c = g_col[k];
      if (part[c] != m) continue;
      if (!self_done && c > g) {
        col[w] = static_cast<int32_t>(i);
        val[w++] = isd_g * isd_g;
        self_done = true;
      }
      col[w] = relabel[c];
      val[w++] = isd_g * isd(c);
    }
    if (!self_done) {
      col[w] = static_cast<int32_t>(i);
      val[w++] = isd_g * isd_g;
    }
    split[i] = w;
    for (int64_t k = s; k < e; ++k) {       // halo columns
      const int64_t c = g_col[k];
      if (part[c] == m) continue;
      col[w] = relabel[c];
      val[w++] = isd_g * isd(c);
      h_colptr[relabel[c] - sc.n_local + 1] += 1;
    }
    rowptr[i + 1] = w;
  }

  // transposed halo block: counting sort by halo column; rows come out ascending
  for (int64_t u = 0; u < sc.n_halo; ++u) h_colptr[u + 1] += h_colptr[u];
  std::vector<int64_t> cursor(h_colptr, h_colptr + sc.n_halo);
  for (int64_t i = 0; i < sc.n_local; ++i) {
    for (int64_t k = split[i]; k < rowptr[i + 1]; ++k) {
      const int64_t u = col[k] - sc.n_local;
      const int64_t p = cursor[u]++;
      h_row[p] = static_cast<int32_t>(i);
      h_val[p] = val[k];
    }
  }
  for (int64_t u = 0; u < sc.n_halo; ++u) {
    const float x = isd(halo_ids[u]);
    h_self[u] = x * x;
  }
  return SAT_OK;
}
