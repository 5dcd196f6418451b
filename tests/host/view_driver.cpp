// Stand-alone driver of the library's host entry points (the partition view), built by
// tests/test_host_sanitize.py together with csrc/partition_view.cpp under
// -fsanitize=address,undefined. Reads one graph from a binary file, runs
// sat_partition_view_sizes / _build and writes every output array to a second file, so the
// test can compare them with the oracle while the sanitizers watch the library's accesses.
//
// Input  (little endian): int64 N, int64 nnz, int32 m, int32 has_deg, int64 rowptr[N+1],
//                         int32 col[nnz], int32 part[N], int32 deg[N] if has_deg.
// Output: int32 status_sizes, int32 status_build, int64 n_local, n_halo, nnz, nnz_halo, then
//         (status_build == 0 only) local_ids, halo_ids, rowptr, split, col, val, h_colptr,
//         h_row, h_val, h_self in that order, raw.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../../include/sat.h"

namespace {
template <typename T>
bool read_vec(FILE* f, std::vector<T>* v, size_t n) {
  v->reserve(n + 1);      // an empty array still has a non-null address (null means "missing" to the library)
  v->resize(n);
  return n == 0 || fread(v->data(), sizeof(T), n, f) == n;
}
template <typename T>
void write_vec(FILE* f, const std::vector<T>& v) {
  if (!v.empty()) fwrite(v.data(), sizeof(T), v.size(), f);
}
}  // namespace

int main(int argc, char** argv) {
  if (argc != 3) return 2;
  FILE* in = fopen(argv[1], "rb");
  if (!in) return 2;
  int64_t N = 0, nnz_g = 0;
  int32_t m = 0, has_deg = 0;
  if (fread(&N, 8, 1, in) != 1 || fread(&nnz_g, 8, 1, in) != 1 || fread(&m, 4, 1, in) != 1 ||
      fread(&has_deg, 4, 1, in) != 1)
    return 2;
  std::vector<int64_t> g_rowptr;
  std::vector<int32_t> g_col, part, deg;
  if (!read_vec(in, &g_rowptr, static_cast<size_t>(N + 1)) || !read_vec(in, &g_col, static_cast<size_t>(nnz_g)) ||
      !read_vec(in, &part, static_cast<size_t>(N)) || (has_deg && !read_vec(in, &deg, static_cast<size_t>(N))))
    return 2;
  fclose(in);

  int64_t n_local = 0, n_halo = 0, nnz = 0, nnz_halo = 0;
  // exactly-sized heap copies of the inputs: an access one element past any of them is caught
  const int32_t st_sizes = sat_partition_view_sizes(N, g_rowptr.data(), g_col.data(), part.data(), m,
                                                    &n_local, &n_halo, &nnz, &nnz_halo);
  FILE* out = fopen(argv[2], "wb");
  if (!out) return 2;
  int32_t st_build = st_sizes;
  std::vector<int32_t> local_ids, halo_ids, col, h_row;
  std::vector<int64_t> rowptr, split, h_colptr;
  std::vector<float> val, h_val, h_self;
  if (st_sizes == SAT_OK) {
    local_ids.resize(n_local);
    halo_ids.resize(n_halo);
    rowptr.resize(n_local + 1);
    split.resize(n_local);
    col.resize(nnz);
    val.resize(nnz);
    h_colptr.resize(n_halo + 1);
    h_row.resize(nnz_halo);
    h_val.resize(nnz_halo);
    h_self.resize(n_halo);
    st_build = sat_partition_view_build(N, g_rowptr.data(), g_col.data(), has_deg ? deg.data() : nullptr,
                                        part.data(), m, local_ids.data(), halo_ids.data(), rowptr.data(),
                                        split.data(), col.data(), val.data(), h_colptr.data(),
                                        h_row.data(), h_val.data(), h_self.data());
  }
  fwrite(&st_sizes, 4, 1, out);
  fwrite(&st_build, 4, 1, out);
  const int64_t counts[4] = {n_local, n_halo, nnz, nnz_halo};
  fwrite(counts, 8, 4, out);
  if (st_build == SAT_OK) {
    write_vec(out, local_ids);
    write_vec(out, halo_ids);
    write_vec(out, rowptr);
    write_vec(out, split);
    write_vec(out, col);
    write_vec(out, val);
    write_vec(out, h_colptr);
    write_vec(out, h_row);
    write_vec(out, h_val);
    write_vec(out, h_self);
  }
  fclose(out);
  return 0;
}
