// CSR of the transposed graph plus the edge-id map, for the backward SpMM dX <- A_w^T dY
// (paper section 2.1.2), and CSR from a COO edge list (section 2.1.1).  One-off set-up: a stable radix sort of
// the non-zeros by column id, or by (row id, column id) (rocPRIM's device radix sort is the library step), then
// offsets by binary search.
#include <string.h>

#include <rocprim/device/device_radix_sort.hpp>

#include "common.h"

namespace hgnn {

__global__ void iota_kernel(int* __restrict__ v, int64_t n) {
  int64_t k = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
  if (k < n) v[k] = int(k);
}

// rowptr_T[j] = number of non-zeros whose column is < j = lower bound of j in the sorted column keys
__global__ void offsets_kernel(const int* __restrict__ sorted_col, int64_t nnz, int ncols, int* __restrict__ rowptr_T) {
  int64_t j = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
  if (j > ncols) return;
  int64_t lo = 0, hi = nnz;
  while (lo < hi) {
    int64_t mid = (lo + hi) >> 1;
    if (sorted_col[mid] < j) lo = mid + 1;
    else hi = mid;
  }
  rowptr_T[j] = int(lo);
}

// COO -> CSR: key = (row, col) in one 64-bit word, so that one stable sort orders the edges by row, then column,
// then position in the list; bad receives 1 when an id is out of range (such an edge gets key 0)
__global__ void coo_keys_kernel(const int* __restrict__ row, const int* __restrict__ col, int64_t nnz, int nrows, int ncols,
                                uint64_t* __restrict__ keys, int* __restrict__ ids, int* __restrict__ bad) {
  int64_t k = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
  if (k >= nnz) return;
  const int r = row[k], c = col[k];
  const bool ok = r >= 0 && r < nrows && c >= 0 && c < ncols;
  if (!ok) atomicOr(bad, 1);
  keys[k] = ok ? (uint64_t(uint32_t(r)) << 32) | uint64_t(uint32_t(c)) : 0;
  ids[k] = int(k);
}

__global__ void coo_split_kernel(const uint64_t* __restrict__ keys, int64_t nnz, int* __restrict__ row_sorted,
                                 int* __restrict__ col_out) {
  int64_t k = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
  if (k >= nnz) return;
  row_sorted[k] = int(keys[k] >> 32);
  col_out[k] = int(uint32_t(keys[k]));
}

// col_T[k'] = row of the non-zero eid_T[k'] of A (upper bound over rowptr, minus one)
__global__ void source_rows_kernel(const int* __restrict__ rowptr, int nrows, const int* __restrict__ eid_T, int64_t nnz,
                                   int* __restrict__ col_T) {
  int64_t k = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
  if (k >= nnz) return;
  col_T[k] = row_of_edge(rowptr, nrows, eid_T[k]);
}

// out[i, f] = fp16(scale[i] * X[i, f]), 8 halves per thread
__global__ void scale_rows_kernel(int64_t n, int F8, const half_t* __restrict__ X, int64_t ldx, const float* __restrict__ scale,
                                  half_t* __restrict__ out, int64_t ldo) {
  const int64_t j = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
  if (j >= n * F8) return;
  const int64_t i = j / F8;
  const int f0 = int(j - i * F8) * 8;
  const float sc = scale[i];
  const half8_t x = *reinterpret_cast<const half8_t*>(X + i * ldx + f0);
  half8_t y;
#pragma unroll
  for (int q = 0; q < 8; ++q) y[q] = half_t(sc * float(x[q]));
  *reinterpret_cast<half8_t*>(out + i * ldo + f0) = y;
}

// out[k*H + h] = in[eid[k]*H + h]: an edge tensor brought into the edge order of the transposed graph
__global__ void edge_gather_kernel(const int* __restrict__ eid, int64_t total, int H, const half_t* __restrict__ in,
                                   half_t* __restrict__ out) {
  const int64_t j = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
  if (j >= total) return;
  const int64_t k = j / H;
  out[j] = in[int64_t(eid[k]) * H + (j - k * H)];
}

}  // namespace hgnn

using namespace hgnn;

extern "C" hgnn_status hgnn_transpose(const hgnn_csr* g, int32_t* rowptr_T, int32_t* col_T, int32_t* eid_T,
                                      void* stream) {
  clear_error();
  hgnn_status st = check_csr_args(g, "hgnn_transpose");
  if (st != HGNN_OK) return st;
  HGNN_REQUIRE(g->eid == nullptr, HGNN_EINVAL, "hgnn_transpose: the input graph must not carry an edge-id map");
  HGNN_REQUIRE(rowptr_T != nullptr, HGNN_EINVAL, "hgnn_transpose: rowptr_T is NULL");
  HGNN_REQUIRE(g->nnz == 0 || (col_T && eid_T), HGNN_EINVAL, "hgnn_transpose: col_T or eid_T is NULL");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int64_t E = g->nnz;
  if (E == 0) {
    HGNN_HIP(hipMemsetAsync(rowptr_T, 0, sizeof(int) * (size_t(g->ncols) + 1), s));
    HGNN_HIP(hipStreamSynchronize(s));
    return HGNN_OK;
  }
  int bits = 1;
  while ((int64_t(1) << bits) < int64_t(g->ncols)) ++bits;
  int *ids = nullptr, *keys_out = nullptr;
  void* tmp = nullptr;
  size_t tmp_bytes = 0;
  hgnn_status rc = HGNN_OK;
  hipError_t e = hipMalloc(&ids, sizeof(int) * size_t(E));
  if (e == hipSuccess) e = hipMalloc(&keys_out, sizeof(int) * size_t(E));
  if (e == hipSuccess) {
    iota_kernel<<<dim3(unsigned(ceil_div(E, kBlock))), kBlock, 0, s>>>(ids, E);
    e = rocprim::radix_sort_pairs(nullptr, tmp_bytes, g->col, keys_out, ids, eid_T, size_t(E), 0u, unsigned(bits), s);
  }
  if (e == hipSuccess) e = hipMalloc(&tmp, tmp_bytes > 0 ? tmp_bytes : 16);
  if (e == hipSuccess)
    e = rocprim::radix_sort_pairs(tmp, tmp_bytes, g->col, keys_out, ids, eid_T, size_t(E), 0u, unsigned(bits), s);
  if (e == hipSuccess) {
    offsets_kernel<<<dim3(unsigned(ceil_div(int64_t(g->ncols) + 1, kBlock))), kBlock, 0, s>>>(keys_out, E, g->ncols,
                                                                                               rowptr_T);
    source_rows_kernel<<<dim3(unsigned(ceil_div(E, kBlock))), kBlock, 0, s>>>(g->rowptr, g->nrows, eid_T, E, col_T);
    e = hipGetLastError();
  }
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (e != hipSuccess)
    rc = fail(e == hipErrorOutOfMemory ? HGNN_ENOMEM : HGNN_EHIP, "hgnn_transpose: %s", hipGetErrorString(e));
  (void)hipFree(ids);
  (void)hipFree(keys_out);
  (void)hipFree(tmp);
  return rc;
}

extern "C" hgnn_status hgnn_coo_to_csr(int32_t nrows, int32_t ncols, int64_t nnz, const int32_t* row, const int32_t* col,
                                       int32_t* rowptr, int32_t* col_out, int32_t* eid, void* stream) {
  clear_error();
  const char* who = "hgnn_coo_to_csr";
  HGNN_REQUIRE(nrows >= 0 && ncols >= 0 && nnz >= 0, HGNN_EINVAL, "%s: negative size", who);
  HGNN_REQUIRE(nnz < (int64_t(1) << 31), HGNN_EINVAL, "%s: nnz = %lld does not fit int32", who, (long long)nnz);
  HGNN_REQUIRE(rowptr != nullptr, HGNN_EINVAL, "%s: rowptr is NULL", who);
  HGNN_REQUIRE(nnz == 0 || (row && col && col_out), HGNN_EINVAL, "%s: row, col or col_out is NULL", who);
  HGNN_REQUIRE(nnz == 0 || (nrows > 0 && ncols > 0), HGNN_EINVAL, "%s: edges in a graph without rows or columns", who);
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (nnz == 0) {
    HGNN_HIP(hipMemsetAsync(rowptr, 0, sizeof(int) * (size_t(nrows) + 1), s));
    HGNN_HIP(hipStreamSynchronize(s));
    return HGNN_OK;
  }
  int row_bits = 1, col_bits = 1;
  while ((int64_t(1) << row_bits) < int64_t(nrows)) ++row_bits;
  while ((int64_t(1) << col_bits) < int64_t(ncols)) ++col_bits;
  const size_t E = size_t(nnz);
  uint64_t *keys = nullptr, *keys_out = nullptr;
  int *ids = nullptr, *ids_out = nullptr, *row_sorted = nullptr, *bad = nullptr;
  void* tmp = nullptr;
  size_t tmp_bytes = 0;
  int hbad = 0;
  hgnn_status rc = HGNN_OK;
  hipError_t e = hipMalloc(&keys, 8 * E);
  if (e == hipSuccess) e = hipMalloc(&keys_out, 8 * E);
  if (e == hipSuccess) e = hipMalloc(&ids, 4 * E);
  if (e == hipSuccess) e = hipMalloc(&row_sorted, 4 * E);
  if (e == hipSuccess) e = hipMalloc(&bad, 4);
  if (e == hipSuccess && !eid) e = hipMalloc(&ids_out, 4 * E);
  int* order = eid ? eid : ids_out;
  if (e == hipSuccess) e = hipMemsetAsync(bad, 0, 4, s);
  if (e == hipSuccess) {
    coo_keys_kernel<<<dim3(unsigned(ceil_div(nnz, kBlock))), kBlock, 0, s>>>(row, col, nnz, nrows, ncols, keys, ids, bad);
    // the columns occupy the low word: the bits between col_bits and 32 are zero in every key and are skipped by
    // sorting the two fields one after the other (least significant field first; the sort is stable)
    e = rocprim::radix_sort_pairs(nullptr, tmp_bytes, keys, keys_out, ids, order, E, 0u, unsigned(col_bits), s);
  }
  if (e == hipSuccess) e = hipMalloc(&tmp, tmp_bytes > 0 ? tmp_bytes : 16);
  if (e == hipSuccess) e = rocprim::radix_sort_pairs(tmp, tmp_bytes, keys, keys_out, ids, order, E, 0u, unsigned(col_bits), s);
  if (e == hipSuccess) {
    size_t need = 0;
    e = rocprim::radix_sort_pairs(nullptr, need, keys_out, keys, order, ids, E, 32u, unsigned(32 + row_bits), s);
    if (e == hipSuccess && need > tmp_bytes) {
      (void)hipStreamSynchronize(s);
      (void)hipFree(tmp);
      tmp = nullptr;
      tmp_bytes = need;
      e = hipMalloc(&tmp, tmp_bytes);
    }
  }
  if (e == hipSuccess)
    e = rocprim::radix_sort_pairs(tmp, tmp_bytes, keys_out, keys, order, ids, E, 32u, unsigned(32 + row_bits), s);
  if (e == hipSuccess) {  // sorted keys are back in `keys`, the order in `ids`
    coo_split_kernel<<<dim3(unsigned(ceil_div(nnz, kBlock))), kBlock, 0, s>>>(keys, nnz, row_sorted, col_out);
    offsets_kernel<<<dim3(unsigned(ceil_div(int64_t(nrows) + 1, kBlock))), kBlock, 0, s>>>(row_sorted, nnz, nrows, rowptr);
    e = hipGetLastError();
  }
  if (e == hipSuccess && eid) e = hipMemcpyAsync(eid, ids, 4 * E, hipMemcpyDeviceToDevice, s);
  if (e == hipSuccess) e = hipMemcpyAsync(&hbad, bad, 4, hipMemcpyDeviceToHost, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (e != hipSuccess)
    rc = fail(e == hipErrorOutOfMemory ? HGNN_ENOMEM : HGNN_EHIP, "%s: %s", who, hipGetErrorString(e));
  else if (hbad)
    rc = fail(HGNN_EINVAL, "%s: a row id outside [0, nrows) or a column id outside [0, ncols)", who);
  (void)hipFree(keys);
  (void)hipFree(keys_out);
  (void)hipFree(ids);
  (void)hipFree(ids_out);
  (void)hipFree(row_sorted);
  (void)hipFree(bad);
  (void)hipFree(tmp);
  return rc;
}

extern "C" hgnn_status hgnn_edge_to_transposed(const hgnn_csr* gt, int32_t H, const hgnn_half* t, hgnn_half* t_T,
                                               void* stream) {
  clear_error();
  const char* who = "hgnn_edge_to_transposed";
  hgnn_status st = check_csr_args(gt, who);
  if (st != HGNN_OK) return st;
  HGNN_REQUIRE(gt->eid != nullptr, HGNN_EINVAL, "%s: the graph carries no edge-id map", who);
  HGNN_REQUIRE(H >= 1, HGNN_EINVAL, "%s: H = %d must be positive", who, H);
  if (gt->nnz == 0) return HGNN_OK;
  HGNN_REQUIRE(t != nullptr && t_T != nullptr, HGNN_EINVAL, "%s: t or t_T is NULL", who);
  HGNN_REQUIRE(t != t_T, HGNN_EINVAL, "%s: the permutation cannot run in place", who);
  const int64_t total = gt->nnz * H;
  edge_gather_kernel<<<dim3(unsigned(ceil_div(total, kBlock))), kBlock, 0, static_cast<hipStream_t>(stream)>>>(
      gt->eid, total, H, reinterpret_cast<const half_t*>(t), reinterpret_cast<half_t*>(t_T));
  HGNN_LAUNCH_CHECK("edge_gather_kernel");
  return HGNN_OK;
}

extern "C" hgnn_status hgnn_scale_rows(int64_t n, int32_t F, const hgnn_half* X, int64_t ldx, const float* scale,
                                       hgnn_half* out, int64_t ldo, void* stream) {
  clear_error();
  const char* who = "hgnn_scale_rows";
  HGNN_REQUIRE(n >= 0 && F > 0, HGNN_EINVAL, "%s: n = %lld, F = %d", who, static_cast<long long>(n), F);
  HGNN_REQUIRE(ldx >= F && ldo >= F, HGNN_EINVAL, "%s: leading dimension smaller than F", who);
  if (n == 0) return HGNN_OK;
  HGNN_REQUIRE(X && scale && out, HGNN_EINVAL, "%s: NULL argument", who);
  HGNN_REQUIRE(ldx % 8 == 0 && ldo % 8 == 0 && aligned16(X) && aligned16(out), HGNN_EUNSUPPORTED,
               "%s: needs ld %% 8 == 0 and 16-byte aligned X, out (rows are moved in 16-byte pieces up to the pitch)", who);
  const int F8 = (F + 7) / 8;
  scale_rows_kernel<<<dim3(unsigned(ceil_div(n * F8, kBlock))), kBlock, 0, static_cast<hipStream_t>(stream)>>>(
      n, F8, reinterpret_cast<const half_t*>(X), ldx, scale, reinterpret_cast<half_t*>(out), ldo);
  HGNN_LAUNCH_CHECK("scale_rows_kernel");
  return HGNN_OK;
}
