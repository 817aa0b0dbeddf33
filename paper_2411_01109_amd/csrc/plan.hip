// Status strings, graph validation and the segment plan of the discretized SpMM
// (paper section 5.2.1: edges are dealt out in storage order in fixed-size batches,
// observation rules 1-3).  Integer work only; everything here is one-off set-up.
#include <stdarg.h>
#include <stdio.h>

#include <hsa/hsa.h>

#include <mutex>

#include "common.h"

namespace hgnn {

static thread_local char g_err[512] = "";

// ---- cache sizes of the current device ----------------------------------------------------------------
// L2 (per XCD) from the HIP device attribute; the last-level cache behind the L2s (the Infinity Cache) is not a
// HIP attribute, so it is read from the HSA agent's cache list (level 3).  Either falls back to the MI355X
// figure (4 MB, 256 MB) when the query gives nothing.
struct CacheQuery {
  int want;      // ordinal of the GPU agent looked for
  int seen;      // GPU agents met so far
  int64_t l3;    // largest level-3 cache of that agent
};

static hsa_status_t cache_cb(hsa_cache_t cache, void* data) {
  CacheQuery* q = static_cast<CacheQuery*>(data);
  uint8_t level = 0;
  uint32_t size = 0;
  if (hsa_cache_get_info(cache, HSA_CACHE_INFO_LEVEL, &level) == HSA_STATUS_SUCCESS &&
      hsa_cache_get_info(cache, HSA_CACHE_INFO_SIZE, &size) == HSA_STATUS_SUCCESS && level == 3) {
    // the attribute is specified in bytes; runtimes have been seen to hand through the driver's KiB figure.  No
    // last-level cache is below 1 MiB and none is 2^30 KiB, so the unit can be told from the value
    int64_t bytes = int64_t(size);
    if (bytes < (int64_t(1) << 20)) bytes <<= 10;
    if (bytes > q->l3) q->l3 = bytes;
  }
  return HSA_STATUS_SUCCESS;
}

static hsa_status_t agent_cb(hsa_agent_t agent, void* data) {
  CacheQuery* q = static_cast<CacheQuery*>(data);
  hsa_device_type_t type;
  if (hsa_agent_get_info(agent, HSA_AGENT_INFO_DEVICE, &type) != HSA_STATUS_SUCCESS || type != HSA_DEVICE_TYPE_GPU)
    return HSA_STATUS_SUCCESS;
  if (q->seen++ == q->want) (void)hsa_agent_iterate_caches(agent, cache_cb, q);
  return HSA_STATUS_SUCCESS;
}

void device_cache_bytes(int64_t* l2, int64_t* llc) {
  *l2 = int64_t(4) << 20;
  *llc = int64_t(256) << 20;
  int dev = 0, v = 0;
  if (hipGetDevice(&dev) != hipSuccess) return;
  // asked once per device: compute calls consult the sizes too
  constexpr int kMaxDev = 64;
  static std::mutex mu;
  static bool known[kMaxDev];
  static int64_t kept[kMaxDev][2];
  std::lock_guard<std::mutex> lock(mu);
  if (dev >= 0 && dev < kMaxDev && known[dev]) {
    *l2 = kept[dev][0];
    *llc = kept[dev][1];
    return;
  }
  if (hipDeviceGetAttribute(&v, hipDeviceAttributeL2CacheSize, dev) == hipSuccess && v > 0) *l2 = v;
  if (hsa_init() == HSA_STATUS_SUCCESS) {
    CacheQuery q{dev, 0, 0};
    (void)hsa_iterate_agents(agent_cb, &q);
    (void)hsa_shut_down();
    if (q.l3 > 0) *llc = q.l3;
  }
  if (dev >= 0 && dev < kMaxDev) {
    kept[dev][0] = *l2;
    kept[dev][1] = *llc;
    known[dev] = true;
  }
}

hgnn_status fail(hgnn_status s, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return s;
}
void clear_error() { g_err[0] = 0; }

hgnn_status check_csr_args(const hgnn_csr* g, const char* who) {
  HGNN_REQUIRE(g != nullptr, HGNN_EINVAL, "%s: graph is NULL", who);
  HGNN_REQUIRE(g->nrows >= 0 && g->ncols >= 0 && g->nnz >= 0, HGNN_EINVAL, "%s: negative graph size", who);
  HGNN_REQUIRE(g->nnz < (int64_t(1) << 31), HGNN_EINVAL, "%s: nnz = %lld does not fit int32", who, (long long)g->nnz);
  HGNN_REQUIRE(g->rowptr != nullptr, HGNN_EINVAL, "%s: rowptr is NULL", who);
  HGNN_REQUIRE(g->nnz == 0 || g->col != nullptr, HGNN_EINVAL, "%s: col is NULL", who);
  return HGNN_OK;
}

// ---- validation ---------------------------------------------------------------------------------
// err starts at kNoError and receives the smallest rule number broken.  Two passes: the offset array first
// (rules 1-3); the per-edge rules only run on a graph that passed them, because they index the offset array
// with values that are in range only when it is monotone and has the right end points.
constexpr int kNoError = 0x7f7f7f7f;
__global__ void validate_rowptr_kernel(hgnn_csr g, int* err) {
  const int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
  int bad = 0;
  if (i == 0) {
    if (g.rowptr[0] != 0) bad = 1;
    else if (int64_t(g.rowptr[g.nrows]) != g.nnz) bad = 2;
  }
  if (!bad && i < g.nrows && g.rowptr[i] > g.rowptr[i + 1]) bad = 3;
  if (bad) atomicMin(err, bad);
}

__global__ void validate_edges_kernel(hgnn_csr g, int* err) {
  const int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
  if (i >= g.nnz) return;
  int bad = 0;
  const int c = g.col[i];
  if (c < 0 || c >= g.ncols) bad = 4;
  if (!bad && g.eid) {
    const int e = g.eid[i];
    if (e < 0 || int64_t(e) >= g.nnz) bad = 5;
  }
  if (!bad && g.row) {
    const int r = g.row[i];
    if (r < 0 || r >= g.nrows) bad = 6;
    else if (!(int64_t(g.rowptr[r]) <= i && i < int64_t(g.rowptr[r + 1]))) bad = 6;
  }
  // a column id may only drop where a new row starts (rowptr is monotone from 0 to nnz here, so the row found is
  // in [0, nrows))
  if (!bad && i > 0 && g.col[i - 1] > c && int64_t(g.rowptr[row_of_edge(g.rowptr, g.nrows, i)]) != i) bad = 7;
  if (bad) atomicMin(err, bad);
}

static const char* const kRule[] = {"ok",
                                    "rowptr[0] != 0",
                                    "rowptr[nrows] != nnz",
                                    "rowptr decreases",
                                    "a column id is outside [0, ncols)",
                                    "an edge id is outside [0, nnz)",
                                    "a COO row id disagrees with rowptr",
                                    "column ids are not ascending inside a row"};

// ---- first and last row of every segment: binary searches in the offset array ------------------------
__global__ void seg_rows_kernel(const int* __restrict__ rowptr, int nrows, int64_t nnz, int S, int64_t nseg,
                                int* __restrict__ lo, int* __restrict__ hi) {
  int64_t k = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
  if (k >= nseg) return;
  int64_t e0 = k * S, e1 = e0 + S < nnz ? e0 + S : nnz;
  lo[k] = row_of_edge(rowptr, nrows, e0);
  hi[k] = row_of_edge(rowptr, nrows, e1 - 1);
}

// ---- ordered compaction of the rows that satisfy a predicate -------------------------------------------
struct SplitPred {  // first and last edge of the row fall in different segments
  const int* rowptr;
  int S;
  __device__ bool operator()(int r) const {
    int b = rowptr[r], e = rowptr[r + 1];
    return e > b && (b / S) != ((e - 1) / S);
  }
};
struct MidPred {  // row longer than lo and at most hi
  const int* rowptr;
  int lo, hi;
  __device__ bool operator()(int r) const {
    const int d = rowptr[r + 1] - rowptr[r];
    return d > lo && d <= hi;
  }
};
struct BigPred {  // row longer than a threshold
  const int* rowptr;
  int deg;
  __device__ bool operator()(int r) const { return rowptr[r + 1] - rowptr[r] > deg; }
};

// total[0] += the lengths of the listed rows
__global__ void list_length_sum_kernel(const int* __restrict__ rowptr, const int* __restrict__ list, int n,
                                       unsigned long long* __restrict__ total) {
  __shared__ unsigned long long part[kBlock / kWave];
  const int i = blockIdx.x * kBlock + threadIdx.x;
  unsigned long long v = 0;
  if (i < n) v = (unsigned long long)(rowptr[list[i] + 1] - rowptr[list[i]]);
  for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_down(v, off);
  if ((threadIdx.x & (kWave - 1)) == 0) part[threadIdx.x / kWave] = v;
  __syncthreads();
  if (threadIdx.x == 0) {
    unsigned long long t = 0;
    for (int w = 0; w < kBlock / kWave; ++w) t += part[w];
    if (t) atomicAdd(total, t);
  }
}

constexpr int kRowsPerThread = 4;
constexpr int kRowsPerBlock = kBlock * kRowsPerThread;

__device__ inline int block_exclusive_scan(int v, int* total) {  // blockDim.x == kBlock
  __shared__ int buf[2][kBlock];
  int t = threadIdx.x, cur = 0;
  buf[0][t] = v;
  __syncthreads();
  for (int d = 1; d < kBlock; d <<= 1) {
    int x = buf[cur][t];
    if (t >= d) x += buf[cur][t - d];
    buf[cur ^ 1][t] = x;
    cur ^= 1;
    __syncthreads();
  }
  int incl = buf[cur][t];
  *total = buf[cur][kBlock - 1];
  __syncthreads();
  return incl - v;
}

template <class Pred>
__global__ void compact_count_kernel(Pred pred, int nrows, int* __restrict__ block_count) {
  int base = blockIdx.x * kRowsPerBlock + threadIdx.x * kRowsPerThread;
  int c = 0;
  for (int u = 0; u < kRowsPerThread; ++u)
    if (base + u < nrows && pred(base + u)) ++c;
  int total;
  (void)block_exclusive_scan(c, &total);
  if (threadIdx.x == 0) block_count[blockIdx.x] = total;
}

// one workgroup: exclusive scan of n block counts in place; total[0] = sum
__global__ void scan_counts_kernel(int* __restrict__ counts, int n, int* __restrict__ total) {
  int carry = 0;
  for (int base = 0; base < n; base += kBlock) {
    int i = base + threadIdx.x;
    int v = i < n ? counts[i] : 0;
    int tot;
    int ex = block_exclusive_scan(v, &tot);
    if (i < n) counts[i] = carry + ex;
    carry += tot;
  }
  if (threadIdx.x == 0) total[0] = carry;
}

template <class Pred>
__global__ void compact_write_kernel(Pred pred, int nrows, const int* __restrict__ block_offset, int* __restrict__ out) {
  int base = blockIdx.x * kRowsPerBlock + threadIdx.x * kRowsPerThread;
  bool f[kRowsPerThread];
  int c = 0;
  for (int u = 0; u < kRowsPerThread; ++u) {
    f[u] = base + u < nrows && pred(base + u);
    c += f[u];
  }
  int total;
  int pos = block_offset[blockIdx.x] + block_exclusive_scan(c, &total);
  for (int u = 0; u < kRowsPerThread; ++u)
    if (f[u]) out[pos++] = base + u;
}

template <class Pred>
static hgnn_status compact_rows(Pred pred, int nrows, int** out, int* n_out, hipStream_t s) {
  *out = nullptr;
  *n_out = 0;
  if (nrows == 0) return HGNN_OK;
  int nblk = int(ceil_div(nrows, kRowsPerBlock));
  int* counts = nullptr;
  HGNN_HIP(hipMalloc(&counts, sizeof(int) * (size_t(nblk) + 1)));
  compact_count_kernel<Pred><<<nblk, kBlock, 0, s>>>(pred, nrows, counts);
  scan_counts_kernel<<<1, kBlock, 0, s>>>(counts, nblk, counts + nblk);
  int total = 0;
  hipError_t e = hipMemcpyAsync(&total, counts + nblk, sizeof(int), hipMemcpyDeviceToHost, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (e != hipSuccess) {
    (void)hipFree(counts);
    return fail(HGNN_EHIP, "compact_rows: %s", hipGetErrorString(e));
  }
  if (total > 0) {
    e = hipMalloc(out, sizeof(int) * size_t(total));
    if (e != hipSuccess) {
      (void)hipFree(counts);
      return fail(HGNN_ENOMEM, "compact_rows: %s", hipGetErrorString(e));
    }
    compact_write_kernel<Pred><<<nblk, kBlock, 0, s>>>(pred, nrows, counts, *out);
    e = hipStreamSynchronize(s);
  }
  (void)hipFree(counts);
  if (e != hipSuccess) return fail(HGNN_EHIP, "compact_rows: %s", hipGetErrorString(e));
  *n_out = total;
  return HGNN_OK;
}

__global__ void split_segs_kernel(const int* __restrict__ rowptr, const int* __restrict__ split_row, int n, int S,
                                  int* __restrict__ lo, int* __restrict__ hi) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  int r = split_row[i];
  lo[i] = rowptr[r] / S;
  hi[i] = (rowptr[r + 1] - 1) / S;
}

// Builds the segment arrays, split-row list and staging buffer of p for the graph g (p->S, p->nseg,
// p->max_F set by the caller).  sub = true: p is the sub-plan of one column block.
hgnn_status plan_build_arrays(hgnn_plan* p, const hgnn_csr* g, hipStream_t s, bool sub) {
  const int64_t E = g->nnz;
  if (E > 0) {
    HGNN_HIP(hipMalloc(&p->seg_row_lo, sizeof(int) * size_t(p->nseg)));
    HGNN_HIP(hipMalloc(&p->seg_row_hi, sizeof(int) * size_t(p->nseg)));
    seg_rows_kernel<<<dim3(unsigned(ceil_div(p->nseg, kBlock))), kBlock, 0, s>>>(g->rowptr, g->nrows, E, p->S, p->nseg,
                                                                                  p->seg_row_lo, p->seg_row_hi);
    HGNN_LAUNCH_CHECK("seg_rows_kernel");
    // staging: two partial vectors (entering piece / leaving piece) per segment
    // (twice over, and three scalars per piece and head: the fused GAT pass that saves for its backward stages two
    // vectors and (max, sum, masked sum) per piece)
    HGNN_HIP(hipMalloc(&p->staging, sizeof(hgnn_half) * size_t(4) * size_t(p->nseg) * size_t(p->max_F)));
    HGNN_HIP(hipMemsetAsync(p->staging, 0, sizeof(hgnn_half) * size_t(4) * size_t(p->nseg) * size_t(p->max_F), s));
    HGNN_HIP(hipMalloc(&p->stage_mz, sizeof(float) * size_t(6) * size_t(p->nseg) * size_t(p->max_H)));
  }
  hgnn_status st = compact_rows(SplitPred{g->rowptr, p->S}, g->nrows, &p->split_row, &p->n_split, s);
  if (st != HGNN_OK) return st;
  if (p->n_split > 0) {
    HGNN_HIP(hipMalloc(&p->split_seg_lo, sizeof(int) * size_t(p->n_split)));
    HGNN_HIP(hipMalloc(&p->split_seg_hi, sizeof(int) * size_t(p->n_split)));
    split_segs_kernel<<<dim3(unsigned(ceil_div(p->n_split, kBlock))), kBlock, 0, s>>>(
        g->rowptr, p->split_row, p->n_split, p->S, p->split_seg_lo, p->split_seg_hi);
    HGNN_LAUNCH_CHECK("split_segs_kernel");
  }
  if (!sub) {  // a column block's sub-plan only serves the SpMM kernels
    st = compact_rows(BigPred{g->rowptr, p->big_deg}, g->nrows, &p->big_row, &p->n_big, s);
    if (st != HGNN_OK) return st;
    st = compact_rows(MidPred{g->rowptr, p->mid_deg, p->big_deg}, g->nrows, &p->mid_row, &p->n_mid, s);
    if (st != HGNN_OK) return st;
    if (p->n_big > 0) {  // chunk table of the long rows (a short list: built on the host)
      std::vector<int> rows(size_t(p->n_big)), rp(size_t(g->nrows) + 1);
      HGNN_HIP(hipMemcpyAsync(rows.data(), p->big_row, sizeof(int) * rows.size(), hipMemcpyDeviceToHost, s));
      HGNN_HIP(hipMemcpyAsync(rp.data(), g->rowptr, sizeof(int) * rp.size(), hipMemcpyDeviceToHost, s));
      HGNN_HIP(hipStreamSynchronize(s));
      std::vector<int> c_row, c_first, c_count, first(size_t(p->n_big));
      for (size_t i = 0; i < rows.size(); ++i) {
        const int deg = rp[size_t(rows[i]) + 1] - rp[size_t(rows[i])];
        const int nch = (deg + kHubEdges - 1) / kHubEdges;
        first[i] = int(c_row.size());
        for (int c = 0; c < nch; ++c) {
          c_row.push_back(rows[i]);
          c_first.push_back(first[i]);
          c_count.push_back(nch);
        }
      }
      p->n_hub_chunks = int32_t(c_row.size());
      const size_t nc = c_row.size();
      HGNN_HIP(hipMalloc(&p->hub_chunk_row, sizeof(int) * nc));
      HGNN_HIP(hipMalloc(&p->hub_chunk_first, sizeof(int) * nc));
      HGNN_HIP(hipMalloc(&p->hub_chunk_count, sizeof(int) * nc));
      HGNN_HIP(hipMalloc(&p->big_first, sizeof(int) * first.size()));
      HGNN_HIP(hipMalloc(&p->hub_part, sizeof(float) * 2 * nc * size_t(p->max_H)));
      HGNN_HIP(hipMemcpyAsync(p->hub_chunk_row, c_row.data(), sizeof(int) * nc, hipMemcpyHostToDevice, s));
      HGNN_HIP(hipMemcpyAsync(p->hub_chunk_first, c_first.data(), sizeof(int) * nc, hipMemcpyHostToDevice, s));
      HGNN_HIP(hipMemcpyAsync(p->hub_chunk_count, c_count.data(), sizeof(int) * nc, hipMemcpyHostToDevice, s));
      HGNN_HIP(hipMemcpyAsync(p->big_first, first.data(), sizeof(int) * first.size(), hipMemcpyHostToDevice, s));
      HGNN_HIP(hipStreamSynchronize(s));  // the host vectors go out of scope
    }
    if (p->n_mid + p->n_big > 0) {  // how many non-zeros the two lists hold: the edge-row kernels size their teams by the rest
      unsigned long long* total = nullptr;
      HGNN_HIP(hipMalloc(&total, sizeof(unsigned long long)));
      hipError_t e = hipMemsetAsync(total, 0, sizeof(unsigned long long), s);
      if (e == hipSuccess && p->n_mid > 0)
        list_length_sum_kernel<<<dim3(unsigned(ceil_div(p->n_mid, kBlock))), kBlock, 0, s>>>(g->rowptr, p->mid_row, p->n_mid, total);
      if (e == hipSuccess && p->n_big > 0)
        list_length_sum_kernel<<<dim3(unsigned(ceil_div(p->n_big, kBlock))), kBlock, 0, s>>>(g->rowptr, p->big_row, p->n_big, total);
      unsigned long long h = 0;
      if (e == hipSuccess) e = hipMemcpyAsync(&h, total, sizeof(h), hipMemcpyDeviceToHost, s);
      if (e == hipSuccess) e = hipStreamSynchronize(s);
      (void)hipFree(total);
      if (e != hipSuccess) return fail(HGNN_EHIP, "hgnn_plan_create: %s", hipGetErrorString(e));
      p->listed_nnz = int64_t(h);
    }
    size_t nv = (size_t(g->nrows) + size_t(g->ncols)) * size_t(p->max_H);
    if (nv > 0) HGNN_HIP(hipMalloc(&p->vscratch, sizeof(float) * nv));
    if (g->nrows > 0) HGNN_HIP(hipMalloc(&p->vtab, sizeof(float) * 4 * size_t(g->nrows) * size_t(p->max_H)));
  }
  HGNN_HIP(hipStreamSynchronize(s));
  return HGNN_OK;
}

}  // namespace hgnn

using namespace hgnn;

extern "C" {

const char* hgnn_status_str(hgnn_status s) {
  switch (s) {
    case HGNN_OK: return "HGNN_OK";
    case HGNN_EINVAL: return "HGNN_EINVAL: invalid argument";
    case HGNN_EUNSUPPORTED: return "HGNN_EUNSUPPORTED: shape not supported";
    case HGNN_ENOMEM: return "HGNN_ENOMEM: out of memory";
    case HGNN_EHIP: return "HGNN_EHIP: HIP runtime error";
  }
  return "unknown hgnn_status";
}

const char* hgnn_last_error(void) { return g_err; }

hgnn_status hgnn_plan_set_vector_halves(hgnn_plan* p, int32_t halves) {
  clear_error();
  HGNN_REQUIRE(p != nullptr, HGNN_EINVAL, "hgnn_plan_set_vector_halves: plan is NULL");
  HGNN_REQUIRE(halves == 2 || halves == 4 || halves == 8, HGNN_EINVAL, "hgnn_plan_set_vector_halves: %d is not 2, 4 or 8", halves);
  p->vec_halves = halves;
  if (p->fine) p->fine->vec_halves = halves;
  return HGNN_OK;
}

int32_t hgnn_plan_vector_halves(const hgnn_plan* p) { return p ? p->vec_halves : 0; }

hgnn_status hgnn_csr_validate(const hgnn_csr* g, void* stream) {
  clear_error();
  hgnn_status st = check_csr_args(g, "hgnn_csr_validate");
  if (st != HGNN_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  int* derr = nullptr;
  HGNN_HIP(hipMalloc(&derr, sizeof(int)));
  int herr = 0;
  hipError_t e = hipMemsetAsync(derr, 0x7f, sizeof(int), s);
  if (e == hipSuccess) {
    validate_rowptr_kernel<<<dim3(unsigned(ceil_div(int64_t(g->nrows) + 1, kBlock))), kBlock, 0, s>>>(*g, derr);
    e = hipGetLastError();
  }
  if (e == hipSuccess) e = hipMemcpyAsync(&herr, derr, sizeof(int), hipMemcpyDeviceToHost, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (e == hipSuccess && herr == kNoError && g->nnz > 0) {
    validate_edges_kernel<<<dim3(unsigned(ceil_div(g->nnz, kBlock))), kBlock, 0, s>>>(*g, derr);
    e = hipGetLastError();
    if (e == hipSuccess) e = hipMemcpyAsync(&herr, derr, sizeof(int), hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
  }
  (void)hipFree(derr);
  if (e != hipSuccess) return fail(HGNN_EHIP, "hgnn_csr_validate: %s", hipGetErrorString(e));
  if (herr != kNoError) return fail(HGNN_EINVAL, "hgnn_csr_validate: %s", kRule[herr > 0 && herr < 8 ? herr : 0]);
  return HGNN_OK;
}

int64_t hgnn_plan_num_segments(const hgnn_plan* p) { return p ? p->nseg : 0; }
int32_t hgnn_plan_num_split_rows(const hgnn_plan* p) { return p ? p->n_split : 0; }
int32_t hgnn_plan_seg_edges(const hgnn_plan* p) { return p ? p->S : 0; }

int32_t hgnn_plan_col_blocks(const hgnn_plan* p) { return p ? p->nb : 0; }
int32_t hgnn_plan_col_blocks_fine(const hgnn_plan* p) { return p ? (p->fine ? p->fine->nb : p->nb) : 0; }

void hgnn_plan_cache_bytes(const hgnn_plan* p, int64_t* l2_bytes, int64_t* llc_bytes) {
  if (l2_bytes) *l2_bytes = p ? p->l2_bytes : 0;
  if (llc_bytes) *llc_bytes = p ? p->llc_bytes : 0;
}

void hgnn_plan_destroy(hgnn_plan* p) {
  if (!p) return;
  for (hgnn_plan* q : p->sub) hgnn_plan_destroy(q);
  hgnn_plan_destroy(p->fine);
  (void)hipFree(p->brp);
  (void)hipFree(p->bcol);
  (void)hipFree(p->beid);
  (void)hipFree(p->bdelta);
  (void)hipFree(p->bstage);
  (void)hipFree(p->bsum);
  (void)hipFree(p->bdesc);
  (void)hipFree(p->seg_row_lo);
  (void)hipFree(p->seg_row_hi);
  (void)hipFree(p->split_row);
  (void)hipFree(p->split_seg_lo);
  (void)hipFree(p->split_seg_hi);
  (void)hipFree(p->big_row);
  (void)hipFree(p->hub_chunk_row);
  (void)hipFree(p->hub_chunk_first);
  (void)hipFree(p->hub_chunk_count);
  (void)hipFree(p->big_first);
  (void)hipFree(p->hub_part);
  (void)hipFree(p->mid_row);
  (void)hipFree(p->staging);
  (void)hipFree(p->stage_mz);
  (void)hipFree(p->vscratch);
  (void)hipFree(p->vtab);
  (void)hipFree(p->goff);
  (void)hipFree(p->moff);
  (void)hipFree(p->grp_row);
  (void)hipFree(p->gstage);
  (void)hipFree(p->scut);
  (void)hipFree(p->chunk_row);
  (void)hipFree(p->col_part);
  (void)hipFree(p->col_poison);
  delete p;
}

hgnn_status hgnn_plan_create(const hgnn_csr* g, int32_t seg_edges, int32_t max_F, int32_t max_H, int32_t col_blocks,
                             hgnn_plan** out, void* stream) {
  clear_error();
  HGNN_REQUIRE(out != nullptr, HGNN_EINVAL, "hgnn_plan_create: out is NULL");
  *out = nullptr;
  hgnn_status st = check_csr_args(g, "hgnn_plan_create");
  if (st != HGNN_OK) return st;
  HGNN_REQUIRE(seg_edges >= 1 && seg_edges <= 2048, HGNN_EINVAL, "hgnn_plan_create: seg_edges = %d outside [1, 2048]",
               seg_edges);
  HGNN_REQUIRE(max_F >= 8 && max_F % 8 == 0, HGNN_EINVAL, "hgnn_plan_create: max_F = %d must be a positive multiple of 8",
               max_F);
  HGNN_REQUIRE(max_H >= 1, HGNN_EINVAL, "hgnn_plan_create: max_H = %d must be positive", max_H);
  HGNN_REQUIRE(col_blocks >= 0 && col_blocks <= 64, HGNN_EINVAL, "hgnn_plan_create: col_blocks = %d outside [0, 64]",
               col_blocks);
  st = hgnn_csr_validate(g, stream);
  if (st != HGNN_OK) return st;
  hgnn_plan* p = new (std::nothrow) hgnn_plan();
  HGNN_REQUIRE(p != nullptr, HGNN_ENOMEM, "hgnn_plan_create: host allocation failed");
  p->nrows = g->nrows;
  p->ncols = g->ncols;
  p->nnz = g->nnz;
  p->S = seg_edges;
  p->nseg = ceil_div(g->nnz, seg_edges);
  p->max_F = max_F;
  p->max_H = max_H;
  p->big_deg = 2048;
  p->mid_deg = 32;
  device_cache_bytes(&p->l2_bytes, &p->llc_bytes);
  hipStream_t s = static_cast<hipStream_t>(stream);
  st = plan_build_arrays(p, g, s, false);
  if (st == HGNN_OK) {
    int nb = col_blocks;
    p->auto_blocks = nb == 0;
    if (nb == 0) {
      // automatic: block only when the feature table is too large for an XCD's L2 (beyond three times its size)
      // but fits the last-level cache with room for the streams (three quarters of it), and rows are long enough
      // that a row piece per block still amortises its partial vector; about two L2 sizes of feature rows per block
      const double table = double(g->ncols) * max_F * 2.0;
      const double mean_deg = g->nrows > 0 ? double(g->nnz) / g->nrows : 0.0;
      nb = 1;
      if (table > 3.0 * double(p->l2_bytes) && table < 0.75 * double(p->llc_bytes) && mean_deg >= 128.0) {
        nb = int(table / (2.0 * double(p->l2_bytes)) + 0.5);
        if (nb < 2) nb = 2;
        if (nb > 16) nb = 16;
      }
    }
    if (nb > 1 && g->nnz > 0 && g->ncols >= nb) st = build_col_blocks(p, g, nb, s);
    // A call that reads edge values through the edge-id map gathers from two tables at once: the feature rows of the
    // block's columns and, for each of those columns, the 128-byte line of the edge tensor that the walk is currently
    // passing (the slots of one source row are consecutive).  Both sets grow with the block's width, so such calls get
    // blocks of half the width.  So does the SDDMM, which leaves no partial row per block behind and only gains from
    // the narrower slice.
    if (st == HGNN_OK && p->auto_blocks && p->nb > 1 && g->ncols >= 2 * p->nb) {
      hgnn_plan* f = new (std::nothrow) hgnn_plan();
      if (f == nullptr) {
        st = fail(HGNN_ENOMEM, "hgnn_plan_create: host allocation failed");
      } else {
        p->fine = f;
        f->nrows = p->nrows;
        f->ncols = p->ncols;
        f->nnz = p->nnz;
        f->S = p->S;
        f->nseg = p->nseg;
        f->max_F = p->max_F;
        f->max_H = p->max_H;
        f->big_deg = p->big_deg;
        f->mid_deg = p->mid_deg;
        f->l2_bytes = p->l2_bytes;
        f->llc_bytes = p->llc_bytes;
        f->auto_blocks = true;
        st = build_col_blocks(f, g, 2 * p->nb, s);
      }
    }
    // column slices for the per-edge passes over per-vertex scalars: where a row's share of a slice still is a piece
    // of 16 non-zeros or more on average
    if (st == HGNN_OK && col_blocks == 0 && g->nrows > 0 && g->nnz > 0) {
      const int64_t ns = ceil_div(g->ncols, kSliceMaxCols);
      if (double(g->nnz) / g->nrows >= 16.0 * double(ns)) st = build_col_slices(p, g, kSliceMaxCols, s);
    }
  }
  if (st != HGNN_OK) {
    hgnn_plan_destroy(p);
    return st;
  }
  *out = p;
  return HGNN_OK;
}

hgnn_status hgnn_plan_block_export(const hgnn_plan* p, int32_t b, int64_t* nnz_b, int32_t* rowptr_b, int32_t* col_b,
                                   int32_t* eid_b, int32_t* seg_row_lo, int32_t* seg_row_hi) {
  clear_error();
  HGNN_REQUIRE(p != nullptr, HGNN_EINVAL, "hgnn_plan_block_export: plan is NULL");
  HGNN_REQUIRE(p->nb > 1 && b >= 0 && b < p->nb, HGNN_EINVAL, "hgnn_plan_block_export: block %d of %d", b, p->nb);
  HGNN_HIP(hipDeviceSynchronize());
  const int64_t off = p->boff[size_t(b)], n = p->boff[size_t(b) + 1] - off;
  if (nnz_b) *nnz_b = n;
  if (rowptr_b)
    HGNN_HIP(hipMemcpy(rowptr_b, p->brp + size_t(b) * (size_t(p->nrows) + 1), sizeof(int) * (size_t(p->nrows) + 1),
                       hipMemcpyDeviceToHost));
  if (n > 0) {
    if (col_b) HGNN_HIP(hipMemcpy(col_b, p->bcol + off, sizeof(int) * size_t(n), hipMemcpyDeviceToHost));
    if (eid_b) HGNN_HIP(hipMemcpy(eid_b, p->beid + off, sizeof(int) * size_t(n), hipMemcpyDeviceToHost));
    const hgnn_plan* q = p->sub[size_t(b)];
    if (seg_row_lo) HGNN_HIP(hipMemcpy(seg_row_lo, q->seg_row_lo, sizeof(int) * size_t(q->nseg), hipMemcpyDeviceToHost));
    if (seg_row_hi) HGNN_HIP(hipMemcpy(seg_row_hi, q->seg_row_hi, sizeof(int) * size_t(q->nseg), hipMemcpyDeviceToHost));
  }
  return HGNN_OK;
}

hgnn_status hgnn_plan_export(const hgnn_plan* p, int32_t* seg_row_lo, int32_t* seg_row_hi, int32_t* split_row,
                             int32_t* split_seg_lo, int32_t* split_seg_hi) {
  clear_error();
  HGNN_REQUIRE(p != nullptr, HGNN_EINVAL, "hgnn_plan_export: plan is NULL");
  HGNN_HIP(hipDeviceSynchronize());
  if (p->nseg > 0) {
    if (seg_row_lo) HGNN_HIP(hipMemcpy(seg_row_lo, p->seg_row_lo, sizeof(int) * size_t(p->nseg), hipMemcpyDeviceToHost));
    if (seg_row_hi) HGNN_HIP(hipMemcpy(seg_row_hi, p->seg_row_hi, sizeof(int) * size_t(p->nseg), hipMemcpyDeviceToHost));
  }
  if (p->n_split > 0) {
    size_t b = sizeof(int) * size_t(p->n_split);
    if (split_row) HGNN_HIP(hipMemcpy(split_row, p->split_row, b, hipMemcpyDeviceToHost));
    if (split_seg_lo) HGNN_HIP(hipMemcpy(split_seg_lo, p->split_seg_lo, b, hipMemcpyDeviceToHost));
    if (split_seg_hi) HGNN_HIP(hipMemcpy(split_seg_hi, p->split_seg_hi, b, hipMemcpyDeviceToHost));
  }
  return HGNN_OK;
}

}  // extern "C"
