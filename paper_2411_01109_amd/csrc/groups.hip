// Neighbour groups for the vertex-parallel variant of the discretized SpMM (paper section 5.4).
//
// A vertex-parallel kernel never lets a batch hold non-zeros of two rows: every row is cut, from its
// own first non-zero on, into groups of at most ng neighbours, and a wave reduces one group.  Rows
// with more than one group meet the same write conflict as the edge-parallel form, between waves
// instead of inside one, and are resolved the same way: a staging slot per group and a follow-up
// kernel, no atomics.  This file builds the lists inside an existing plan; one-off set-up code,
// rocPRIM's device scan is the library step.
#include <string.h>

#include <rocprim/device/device_scan.hpp>

#include "common.h"

namespace hgnn {

// cnt[r] = groups of row r; mcnt[r] = the same when the row has more than one group, else 0; entry nrows = 0
__global__ void group_counts_kernel(const int* __restrict__ rowptr, int nrows, int ng, int* __restrict__ cnt,
                                    int* __restrict__ mcnt) {
  const int64_t r = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
  if (r > nrows) return;
  int c = 0;
  if (r < nrows) c = (rowptr[r + 1] - rowptr[r] + ng - 1) / ng;
  cnt[r] = c;
  mcnt[r] = c > 1 ? c : 0;
}

// grp_row[j] = the row r with goff[r] <= j < goff[r+1]
__global__ void group_rows_kernel(const int* __restrict__ goff, int nrows, int64_t n_groups, int* __restrict__ grp_row) {
  const int64_t j = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
  if (j >= n_groups) return;
  int lo = 0, hi = nrows;  // first index in [0, nrows] whose offset exceeds j
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (goff[mid] <= j) lo = mid + 1;
    else hi = mid;
  }
  grp_row[j] = lo - 1;
}

__global__ void group_first_kernel(const int* __restrict__ rowptr, const int* __restrict__ goff,
                                   const int* __restrict__ grp_row, int64_t n_groups, int ng, int* __restrict__ first) {
  const int64_t j = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
  if (j >= n_groups) return;
  const int r = grp_row[j];
  first[j] = rowptr[r] + int(j - goff[r]) * ng;
}

static void free_groups(hgnn_plan* p) {
  (void)hipFree(p->goff);
  (void)hipFree(p->moff);
  (void)hipFree(p->grp_row);
  (void)hipFree(p->gstage);
  p->goff = p->moff = p->grp_row = nullptr;
  p->gstage = nullptr;
  p->ng = 0;
  p->n_groups = p->n_gslots = 0;
}

}  // namespace hgnn

using namespace hgnn;

extern "C" {

hgnn_status hgnn_plan_add_groups(hgnn_plan* p, const hgnn_csr* g, int32_t group_edges, void* stream) {
  clear_error();
  const char* who = "hgnn_plan_add_groups";
  hgnn_status st = check_csr_args(g, who);
  if (st != HGNN_OK) return st;
  HGNN_REQUIRE(p != nullptr, HGNN_EINVAL, "%s: plan is NULL", who);
  HGNN_REQUIRE(p->nrows == g->nrows && p->ncols == g->ncols && p->nnz == g->nnz, HGNN_EINVAL,
               "%s: the plan was built for another graph", who);
  HGNN_REQUIRE(group_edges >= 1 && group_edges <= 1024, HGNN_EINVAL, "%s: group_edges = %d outside [1, 1024]", who,
               group_edges);
  hipStream_t s = static_cast<hipStream_t>(stream);
  free_groups(p);
  const int V = g->nrows;
  int *cnt = nullptr, *mcnt = nullptr;
  void* tmp = nullptr;
  size_t tmp_bytes = 0;
  const size_t n1 = size_t(V) + 1;
  hipError_t e = hipMalloc(&cnt, sizeof(int) * n1);
  if (e == hipSuccess) e = hipMalloc(&mcnt, sizeof(int) * n1);
  if (e == hipSuccess) e = hipMalloc(&p->goff, sizeof(int) * n1);
  if (e == hipSuccess) e = hipMalloc(&p->moff, sizeof(int) * n1);
  if (e == hipSuccess) {
    group_counts_kernel<<<dim3(unsigned(ceil_div(int64_t(n1), kBlock))), kBlock, 0, s>>>(g->rowptr, V, group_edges, cnt, mcnt);
    e = rocprim::exclusive_scan(nullptr, tmp_bytes, cnt, p->goff, 0, n1, rocprim::plus<int>(), s);
  }
  if (e == hipSuccess) e = hipMalloc(&tmp, tmp_bytes > 0 ? tmp_bytes : 16);
  if (e == hipSuccess) e = rocprim::exclusive_scan(tmp, tmp_bytes, cnt, p->goff, 0, n1, rocprim::plus<int>(), s);
  if (e == hipSuccess) e = rocprim::exclusive_scan(tmp, tmp_bytes, mcnt, p->moff, 0, n1, rocprim::plus<int>(), s);
  int totals[2] = {0, 0};
  if (e == hipSuccess) e = hipMemcpyAsync(&totals[0], p->goff + V, sizeof(int), hipMemcpyDeviceToHost, s);
  if (e == hipSuccess) e = hipMemcpyAsync(&totals[1], p->moff + V, sizeof(int), hipMemcpyDeviceToHost, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (e == hipSuccess && totals[0] > 0) e = hipMalloc(&p->grp_row, sizeof(int) * size_t(totals[0]));
  if (e == hipSuccess && totals[1] > 0)
    e = hipMalloc(&p->gstage, sizeof(hgnn_half) * size_t(totals[1]) * size_t(p->max_F));
  if (e == hipSuccess && totals[0] > 0) {
    group_rows_kernel<<<dim3(unsigned(ceil_div(int64_t(totals[0]), kBlock))), kBlock, 0, s>>>(p->goff, V, totals[0],
                                                                                              p->grp_row);
    e = hipGetLastError();
    if (e == hipSuccess) e = hipStreamSynchronize(s);
  }
  (void)hipFree(cnt);
  (void)hipFree(mcnt);
  (void)hipFree(tmp);
  if (e != hipSuccess) {
    free_groups(p);
    return fail(e == hipErrorOutOfMemory ? HGNN_ENOMEM : HGNN_EHIP, "%s: %s", who, hipGetErrorString(e));
  }
  p->ng = group_edges;
  p->n_groups = totals[0];
  p->n_gslots = totals[1];
  return HGNN_OK;
}

int64_t hgnn_plan_num_groups(const hgnn_plan* p) { return p ? p->n_groups : 0; }
int32_t hgnn_plan_group_edges(const hgnn_plan* p) { return p ? p->ng : 0; }

hgnn_status hgnn_plan_groups_export(const hgnn_plan* p, const hgnn_csr* g, int32_t* group_row, int32_t* group_first) {
  clear_error();
  const char* who = "hgnn_plan_groups_export";
  hgnn_status st = check_csr_args(g, who);
  if (st != HGNN_OK) return st;
  HGNN_REQUIRE(p != nullptr && p->ng > 0, HGNN_EINVAL, "%s: the plan holds no neighbour groups", who);
  HGNN_REQUIRE(p->nrows == g->nrows && p->nnz == g->nnz, HGNN_EINVAL, "%s: the plan was built for another graph", who);
  if (p->n_groups == 0) return HGNN_OK;
  HGNN_REQUIRE(group_row && group_first, HGNN_EINVAL, "%s: output array is NULL", who);
  int* first = nullptr;
  HGNN_HIP(hipMalloc(&first, sizeof(int) * size_t(p->n_groups)));
  group_first_kernel<<<dim3(unsigned(ceil_div(p->n_groups, kBlock))), kBlock, 0, nullptr>>>(g->rowptr, p->goff, p->grp_row,
                                                                                            p->n_groups, p->ng, first);
  hipError_t e = hipGetLastError();
  if (e == hipSuccess) e = hipMemcpy(group_first, first, sizeof(int) * size_t(p->n_groups), hipMemcpyDeviceToHost);
  if (e == hipSuccess) e = hipMemcpy(group_row, p->grp_row, sizeof(int) * size_t(p->n_groups), hipMemcpyDeviceToHost);
  (void)hipFree(first);
  if (e != hipSuccess) return fail(HGNN_EHIP, "%s: %s", who, hipGetErrorString(e));
  return HGNN_OK;
}

}  // extern "C"
