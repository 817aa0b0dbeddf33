// CSR of the transposed graph plus the edge-id map, for the backward SpMM dX <- A_w^T dY
// (paper section 2.1.2).  One-off set-up: a stable radix sort of the non-zeros by column id
// (rocPRIM's device radix sort is the library step), then offsets by binary search.
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
