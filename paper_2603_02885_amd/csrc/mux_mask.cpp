// Host-side layout of the two listings of a Diff-Pruning mask (index work only).
#include <string>
#include <vector>

#include "mux_internal.h"

using namespace mux;

extern "C" mux_status mux_sparse_mask_layout(const int32_t* k, const int32_t* n, int32_t nnz, int32_t K, int32_t N,
                                             int32_t* row_ptr, int32_t* col_idx, int32_t* col_ptr, int32_t* col_ent) {
  static const char* fn = "mux_sparse_mask_layout";
  if (nnz < 0 || K <= 0 || N <= 0) return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": nnz must be >= 0, K and N positive");
  if (!row_ptr || !col_ptr || (nnz > 0 && (!k || !n || !col_idx || !col_ent)))
    return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": null array");
  for (int32_t e = 0; e < nnz; ++e) {
    if (k[e] < 0 || k[e] >= K || n[e] < 0 || n[e] >= N) return fail(MUX_ERR_SHAPE, std::string(fn) + ": entry outside W");
    if (e > 0 && (k[e] < k[e - 1] || (k[e] == k[e - 1] && n[e] <= n[e - 1])))
      return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": entries must be sorted by (k, n) without duplicates");
  }
  // by row: the entries are already in this order
  for (int32_t r = 0; r <= K; ++r) row_ptr[r] = 0;
  for (int32_t c = 0; c <= N; ++c) col_ptr[c] = 0;
  for (int32_t e = 0; e < nnz; ++e) { row_ptr[k[e] + 1]++; col_ptr[n[e] + 1]++; col_idx[e] = n[e]; }
  for (int32_t r = 0; r < K; ++r) row_ptr[r + 1] += row_ptr[r];
  for (int32_t c = 0; c < N; ++c) col_ptr[c + 1] += col_ptr[c];
  // by column: a counting sort keeps k ascending inside a column
  try {
    std::vector<int32_t> next(col_ptr, col_ptr + N);
    for (int32_t e = 0; e < nnz; ++e) {
      const int32_t i = next[n[e]]++;
      col_ent[2 * i] = k[e];
      col_ent[2 * i + 1] = e;
    }
  } catch (const std::bad_alloc&) {
    return fail(MUX_ERR_HOST_NOMEM, std::string(fn) + ": out of host memory");
  }
  return MUX_OK;
}

extern "C" mux_status mux_sparse_mask_tile_layout(const int32_t* k, const int32_t* n, int32_t nnz, int32_t K, int32_t N,
                                                  int32_t* fwd_ptr, int32_t* fwd_ent, int32_t* bwd_ptr, int32_t* bwd_ent) {
  static const char* fn = "mux_sparse_mask_tile_layout";
  if (nnz < 0 || K <= 0 || N <= 0) return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": nnz must be >= 0, K and N positive");
  if (!fwd_ptr || !bwd_ptr || (nnz > 0 && (!k || !n || !fwd_ent || !bwd_ent)))
    return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": null array");
  for (int32_t e = 0; e < nnz; ++e) {
    if (k[e] < 0 || k[e] >= K || n[e] < 0 || n[e] >= N) return fail(MUX_ERR_SHAPE, std::string(fn) + ": entry outside W");
    if (e > 0 && (k[e] < k[e - 1] || (k[e] == k[e - 1] && n[e] <= n[e - 1])))
      return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": entries must be sorted by (k, n) without duplicates");
  }
  const int64_t nbn = (N + 127) / 128, nbk = (K + 127) / 128;
  const int64_t n_fwd = (int64_t)((K + 63) / 64) * nbn, n_bwd = (int64_t)((N + 63) / 64) * nbk;
  try {
    // counting sorts: the entries come in (k, n) order and keep it inside a bucket
    std::vector<int32_t> next_f((size_t)n_fwd + 1, 0), next_b((size_t)n_bwd + 1, 0);
    for (int32_t e = 0; e < nnz; ++e) {
      next_f[(size_t)((int64_t)(k[e] / 64) * nbn + n[e] / 128) + 1]++;
      next_b[(size_t)((int64_t)(n[e] / 64) * nbk + k[e] / 128) + 1]++;
    }
    for (int64_t b = 0; b < n_fwd; ++b) next_f[(size_t)b + 1] += next_f[(size_t)b];
    for (int64_t b = 0; b < n_bwd; ++b) next_b[(size_t)b + 1] += next_b[(size_t)b];
    for (int64_t b = 0; b <= n_fwd; ++b) fwd_ptr[b] = next_f[(size_t)b];
    for (int64_t b = 0; b <= n_bwd; ++b) bwd_ptr[b] = next_b[(size_t)b];
    for (int32_t e = 0; e < nnz; ++e) {
      const int32_t i = next_f[(size_t)((int64_t)(k[e] / 64) * nbn + n[e] / 128)]++;
      fwd_ent[2 * i] = e;
      fwd_ent[2 * i + 1] = (k[e] % 64) << 7 | (n[e] % 128);
      const int32_t j = next_b[(size_t)((int64_t)(n[e] / 64) * nbk + k[e] / 128)]++;
      bwd_ent[2 * j] = e;
      bwd_ent[2 * j + 1] = (n[e] % 64) << 7 | (k[e] % 128);
    }
  } catch (const std::bad_alloc&) {
    return fail(MUX_ERR_HOST_NOMEM, std::string(fn) + ": out of host memory");
  }
  return MUX_OK;
}
