// Column blocking of the SpMM for feature tables that miss an XCD's L2 but fit the Infinity Cache.
//
// The gather of neighbour rows is what bounds the SpMM (paper section 6.2: "not compute-bound");
// on MI355X each XCD has a private 4 MB L2, so a table of tens of MB is re-fetched over the fabric
// for almost every non-zero.  The plan therefore may cut the columns into nb blocks: block b keeps,
// as a CSR of its own, the non-zeros whose column lies in [b*width, (b+1)*width).  Because columns
// ascend inside a row, a block's share of a row is a contiguous piece of that row.  The SpMM then
// runs block after block -- all compute units gather from the same slice of the table at the same
// time, which the L2s can hold -- each block reducing its pieces with the usual segment kernels
// into a per-block partial output, and one pass adds the nb partials of every row (no atomics).
// One-off set-up code; rocPRIM's device scan is the library step.
#include <string.h>

#include <rocprim/device/device_scan.hpp>

#include "common.h"

namespace hgnn {

// cut[r*(nb+1) + b] = first CSR position of row r whose column is >= b*width (b = nb: end of the row)
__global__ void block_cuts_kernel(const int* __restrict__ rowptr, const int* __restrict__ col, int nrows, int nb, int width,
                                  int* __restrict__ cut) {
  const int64_t idx = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
  if (idx >= int64_t(nrows) * (nb + 1)) return;
  const int r = int(idx / (nb + 1)), b = int(idx % (nb + 1));
  int lo = rowptr[r], hi = rowptr[r + 1];
  if (b < nb) {
    const int64_t key = int64_t(b) * width;
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (col[mid] < key) lo = mid + 1;
      else hi = mid;
    }
  } else {
    lo = hi;
  }
  cut[idx] = lo;
}

// cnt[b*nrows + r] = number of non-zeros of row r in block b
__global__ void block_counts_kernel(const int* __restrict__ cut, int nrows, int nb, int* __restrict__ cnt) {
  const int64_t idx = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
  if (idx >= int64_t(nrows) * nb) return;
  const int b = int(idx / nrows), r = int(idx % nrows);
  cnt[idx] = cut[int64_t(r) * (nb + 1) + b + 1] - cut[int64_t(r) * (nb + 1) + b];
}

// goff = exclusive scan of cnt (block-major); brp[b][r] = goff[b*nrows + r] - goff[b*nrows]
__global__ void block_rowptr_kernel(const int* __restrict__ goff, int nrows, int nb, int64_t nnz, int* __restrict__ brp) {
  const int64_t idx = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
  if (idx >= int64_t(nb) * (nrows + 1)) return;
  const int b = int(idx / (nrows + 1)), r = int(idx % (nrows + 1));
  const int64_t base = goff[int64_t(b) * nrows];
  const int64_t here = r < nrows ? goff[int64_t(b) * nrows + r] : (b + 1 < nb ? goff[int64_t(b + 1) * nrows] : nnz);
  brp[idx] = int(here - base);
}

// delta[b*nrows + r] = (first CSR position of row r's piece in block b) - (its position inside block b), so that
// the original position of a blocked non-zero is its block position + delta of its row
__global__ void block_delta_kernel(const int* __restrict__ cut, const int* __restrict__ goff, int nrows, int nb,
                                   int* __restrict__ delta) {
  const int64_t idx = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
  if (idx >= int64_t(nrows) * nb) return;
  const int b = int(idx / nrows), r = int(idx % nrows);
  delta[idx] = cut[int64_t(r) * (nb + 1) + b] - (goff[idx] - goff[int64_t(b) * nrows]);
}

// every non-zero k of the graph goes to its block, keeping its place inside the row piece
__global__ void block_fill_kernel(hgnn_csr g, const int* __restrict__ cut, const int* __restrict__ goff, int nb, int width,
                                  int* __restrict__ bcol, int* __restrict__ beid) {
  const int64_t k = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
  if (k >= g.nnz) return;
  const int r = row_of_edge(g.rowptr, g.nrows, k);
  const int c = g.col[k];
  const int b = c / width;
  const int64_t dest = int64_t(goff[int64_t(b) * g.nrows + r]) + (k - cut[int64_t(r) * (nb + 1) + b]);
  bcol[dest] = c;
  beid[dest] = g.eid ? g.eid[k] : int(k);
}

hgnn_status build_col_blocks(hgnn_plan* p, const hgnn_csr* g, int nb, hipStream_t s) {
  const int V = g->nrows;
  const int64_t E = g->nnz;
  const int width = int(ceil_div(g->ncols, nb));
  p->nb = nb;
  p->block_width = width;
  p->block_eid = g->eid != nullptr;
  int *cut = nullptr, *cnt = nullptr, *goff = nullptr;
  void* tmp = nullptr;
  size_t tmp_bytes = 0;
  const size_t n_flat = size_t(nb) * size_t(V);
  hgnn_status rc = HGNN_OK;
  hipError_t e = hipMalloc(&cut, sizeof(int) * size_t(V) * size_t(nb + 1));
  if (e == hipSuccess) e = hipMalloc(&cnt, sizeof(int) * n_flat);
  if (e == hipSuccess) e = hipMalloc(&goff, sizeof(int) * n_flat);
  if (e == hipSuccess) e = hipMalloc(&p->brp, sizeof(int) * size_t(nb) * (size_t(V) + 1));
  if (e == hipSuccess) e = hipMalloc(&p->bcol, sizeof(int) * size_t(E));
  if (e == hipSuccess) e = hipMalloc(&p->beid, sizeof(int) * size_t(E));
  // partial rows twice over and three scalars per row and head: the fused GAT pass that saves for its backward
  // leaves two vectors and (max, sum, masked sum) per block; row sums of edge tensors use one scalar
  if (e == hipSuccess) e = hipMalloc(&p->bstage, sizeof(hgnn_half) * 2 * n_flat * size_t(p->max_F));
  if (e == hipSuccess) e = hipMalloc(&p->bsum, sizeof(float) * 3 * n_flat * size_t(p->max_H));
  if (e == hipSuccess) e = hipMalloc(&p->bdelta, sizeof(int) * n_flat);
  if (e == hipSuccess) {
    block_cuts_kernel<<<dim3(unsigned(ceil_div(int64_t(V) * (nb + 1), kBlock))), kBlock, 0, s>>>(g->rowptr, g->col, V, nb,
                                                                                                 width, cut);
    block_counts_kernel<<<dim3(unsigned(ceil_div(int64_t(n_flat), kBlock))), kBlock, 0, s>>>(cut, V, nb, cnt);
    e = rocprim::exclusive_scan(nullptr, tmp_bytes, cnt, goff, 0, n_flat, rocprim::plus<int>(), s);
  }
  if (e == hipSuccess) e = hipMalloc(&tmp, tmp_bytes > 0 ? tmp_bytes : 16);
  if (e == hipSuccess) e = rocprim::exclusive_scan(tmp, tmp_bytes, cnt, goff, 0, n_flat, rocprim::plus<int>(), s);
  if (e == hipSuccess) {
    block_rowptr_kernel<<<dim3(unsigned(ceil_div(int64_t(nb) * (V + 1), kBlock))), kBlock, 0, s>>>(goff, V, nb, E, p->brp);
    block_fill_kernel<<<dim3(unsigned(ceil_div(E, kBlock))), kBlock, 0, s>>>(*g, cut, goff, nb, width, p->bcol, p->beid);
    block_delta_kernel<<<dim3(unsigned(ceil_div(int64_t(n_flat), kBlock))), kBlock, 0, s>>>(cut, goff, V, nb, p->bdelta);
    e = hipGetLastError();
  }
  p->boff.assign(size_t(nb) + 1, 0);
  for (int b = 0; b < nb && e == hipSuccess; ++b) {
    int v = 0;
    e = hipMemcpyAsync(&v, goff + size_t(b) * V, sizeof(int), hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    p->boff[size_t(b)] = v;
  }
  p->boff[size_t(nb)] = E;
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (e != hipSuccess)
    rc = fail(e == hipErrorOutOfMemory ? HGNN_ENOMEM : HGNN_EHIP, "build_col_blocks: %s", hipGetErrorString(e));
  (void)hipFree(cut);
  (void)hipFree(cnt);
  (void)hipFree(goff);
  (void)hipFree(tmp);
  if (rc != HGNN_OK) return rc;
  // a segment plan per block, over the block's own CSR
  for (int b = 0; b < nb; ++b) {
    hgnn_plan* q = new (std::nothrow) hgnn_plan();
    if (!q) return fail(HGNN_ENOMEM, "build_col_blocks: host allocation failed");
    p->sub.push_back(q);
    q->nrows = V;
    q->ncols = g->ncols;
    q->nnz = p->boff[size_t(b) + 1] - p->boff[size_t(b)];
    q->S = p->S;
    q->nseg = ceil_div(q->nnz, q->S);
    q->max_F = p->max_F;
    q->max_H = p->max_H;
    hgnn_csr view{V, g->ncols, q->nnz, p->brp + size_t(b) * (size_t(V) + 1), p->bcol + p->boff[size_t(b)], nullptr,
                  p->beid + p->boff[size_t(b)]};
    rc = plan_build_arrays(q, &view, s, true);
    if (rc != HGNN_OK) return rc;
  }
  // the blocks' arrays in one device table
  std::vector<hgnn_seg_block> desc{};
  desc.resize(size_t(nb));
  for (int b = 0; b < nb; ++b) {
    const hgnn_plan* q = p->sub[size_t(b)];
    hgnn_seg_block& d = desc[size_t(b)];
    d.rowptr = p->brp + size_t(b) * (size_t(V) + 1);
    d.col = p->bcol + p->boff[size_t(b)];
    d.eid = p->beid + p->boff[size_t(b)];
    d.delta = p->bdelta + size_t(b) * size_t(V);
    d.seg_lo = q->seg_row_lo;
    d.seg_hi = q->seg_row_hi;
    d.staging = q->staging;
    d.split_row = q->split_row;
    d.split_lo = q->split_seg_lo;
    d.split_hi = q->split_seg_hi;
    d.nnz = q->nnz;
    d.nseg = q->nseg;
    d.n_split = q->n_split;
    d.pad = 0;
    d.stage_mz = q->stage_mz;
  }
  HGNN_HIP(hipMalloc(&p->bdesc, sizeof(hgnn_seg_block) * size_t(nb)));
  HGNN_HIP(hipMemcpyAsync(p->bdesc, desc.data(), sizeof(hgnn_seg_block) * size_t(nb), hipMemcpyHostToDevice, s));
  HGNN_HIP(hipStreamSynchronize(s));
  return HGNN_OK;
}

}  // namespace hgnn
