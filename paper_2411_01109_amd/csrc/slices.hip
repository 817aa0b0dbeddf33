// Column slices: per-edge passes whose only random access is a per-vertex scalar of the column side.
//
// Two steps of the GAT path read or update one scalar per non-zero at the non-zero's column: the factorised
// score e = LeakyReLU(el[row] + er[col]) (paper section 3.1.2, the SDDMM variant of GAT) gathers er[col], and the
// column sums of the score gradient d(e_r)[j] = sum over the non-zeros of column j (section 2.1.2: the backward
// pass needs the transposed direction) scatter into out[col].  Served by the L2s, either costs one cache request
// per non-zero, and the request rate of the L2s then bounds the pass at a fraction of what streaming the edge
// arrays would take.  On gfx950 a workgroup may hold 160 KB of LDS, enough for the scalars of 16 K columns, so
// the plan can cut the columns into slices of that width: a workgroup loads (or zeroes) the table of one slice
// in LDS and walks the pieces of the rows of one row chunk that fall into the slice -- contiguous pieces of the
// column array, because columns ascend inside a row -- gathering from / adding into LDS.  What is left in
// memory traffic is the stream of column ids and edge values.
//
// Column sums are accumulated as 64-bit fixed-point integers (an fp16 value is an integer multiple of 2^-24 below
// 2^16 in magnitude, so the conversion is exact), with LDS atomic adds: integer addition is associative, so the
// result does not depend on the order in which the waves arrive (no run-to-run variation), and it is the exact sum,
// rounded once on output.  Every workgroup leaves its slice's partial sums in the plan; a second kernel adds the
// row chunks' partials per column.  Non-finite inputs (never produced by the path itself) go through a separate
// fp32 side array so that they still poison their column's sum.
#include "common.h"

#include <algorithm>

namespace hgnn {

constexpr int kSliceThreads = 1024;
constexpr int kSliceWaves = kSliceThreads / kWave;
constexpr int kSliceUnroll = 8;  // row pieces whose loads a wave has in flight together

struct SliceArgs {
  const int* scut;       // [ns+1][nrows]: first CSR position of row r whose column is >= s*W (s = ns: end of the row)
  const int* chunk_row;  // [nch+1] row chunks holding about nnz / nch non-zeros each
  const int* col;
  int nrows, ncols, ns, nch, W;
  // score (and alpha from lse)
  const float* el;   // [nrows]
  const float* er;   // [ncols]
  const float* lse;  // [nrows] or nullptr
  half_t* out;       // [nnz]
  float slope;
  // column sums
  const half_t* t;            // [nnz]
  unsigned long long* part;   // [nch][ncols]
  float* poison;              // [ncols]
};

// fp16 bit pattern -> value * 2^24 as a 64-bit integer (exact); finite inputs only
__device__ __forceinline__ long long half_bits_to_fixed(unsigned bits) {
  const unsigned ex = (bits >> 10) & 31u, man = bits & 1023u;
  const unsigned long long m = ex ? (man | 1024u) : man;
  const long long v = (long long)(m << (ex ? ex - 1u : 0u));
  return (bits & 0x8000u) ? -v : v;
}

// LDS of a workgroup: the slice's table (W scalars of 4 or 8 bytes), then per wave the bookkeeping of the 64 rows
// it is working on: exclusive prefix of the pieces' lengths (65 ints), their first positions, and for the score the
// rows' el and lse
__host__ __device__ inline int slice_wave_bytes(bool colsum) { return (66 + 64 + (colsum ? 0 : 128)) * 4; }
__host__ __device__ inline size_t slice_lds_bytes(int W, bool colsum) {
  return size_t(W) * (colsum ? 8 : 4) + size_t(kSliceWaves) * slice_wave_bytes(colsum);
}

template <bool COLSUM>
__global__ __launch_bounds__(kSliceThreads) void edge_slice_kernel(SliceArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  float* s_er = reinterpret_cast<float*>(smem);
  unsigned long long* s_acc = reinterpret_cast<unsigned long long*>(smem);
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  int* s_p = reinterpret_cast<int*>(smem + size_t(a.W) * (COLSUM ? 8 : 4) + size_t(wave) * slice_wave_bytes(COLSUM));
  int* s_d = s_p + 66;
  float* s_el = reinterpret_cast<float*>(s_d + 64);
  float* s_lse = s_el + 64;
  // workgroup id = slice * nch + chunk, nch a multiple of 8: the slices of one row chunk run on one XCD (workgroups
  // are dealt out to the XCDs in turn), so the cache lines that neighbouring pieces of a row share meet in one L2
  const int s = int(blockIdx.x) / a.nch, c = int(blockIdx.x) % a.nch;
  const int col0 = s * a.W;
  const int wcols = a.ncols - col0 < a.W ? a.ncols - col0 : a.W;
  for (int i = tid; i < wcols; i += kSliceThreads) {
    if (COLSUM) s_acc[i] = 0ull;
    else s_er[i] = a.er[col0 + i];
  }
  __syncthreads();
  const int r0 = a.chunk_row[c], r1 = a.chunk_row[c + 1];
  const int* __restrict__ lo = a.scut + size_t(s) * size_t(a.nrows);
  const int* __restrict__ hi = lo + a.nrows;
  const unsigned short* __restrict__ tbits = reinterpret_cast<const unsigned short*>(a.t);

  // A wave takes 64 rows at a time.  The non-zeros of their pieces of this slice are numbered through (slot q belongs
  // to the row j with p[j] <= q < p[j+1]) and dealt out to the lanes in turn, so that every load instruction moves 64
  // non-zeros whatever the lengths of the pieces; a lane's slots ascend, so it finds their rows by walking j forward.
  // The loads run one round ahead of the work: while the non-zeros of a round (8 x 64 slots) are scored or added, the
  // column ids and values of the next round are on their way; the row bounds of the next 64 rows are requested when a
  // batch begins.
  // Slots beyond the batch's total repeat its last slot (a valid position): for the score that stores the same value
  // twice, for the sums the repeated value is replaced by zero.  The row of a slot comes from a branch-free binary
  // search over the 65 prefix values, six LDS reads per slot; the eight searches of a round are independent chains.
  auto plan_round = [&](int q0, int total, int (&kk)[kSliceUnroll], int (&jj)[kSliceUnroll]) {
    int q[kSliceUnroll];
#pragma unroll
    for (int u = 0; u < kSliceUnroll; ++u) {
      q[u] = q0 + u * kWave < total ? q0 + u * kWave : total - 1;
      jj[u] = 0;
    }
#pragma unroll
    for (int step = kWave / 2; step > 0; step >>= 1) {
#pragma unroll
      for (int u = 0; u < kSliceUnroll; ++u)
        if (s_p[jj[u] + step] <= q[u]) jj[u] += step;  // largest j in [0, 63] with p[j] <= q
    }
#pragma unroll
    for (int u = 0; u < kSliceUnroll; ++u) kk[u] = s_d[jj[u]] + q[u];  // position = slot + (first position - first slot) of the row
  };
  auto issue = [&](const int (&kk)[kSliceUnroll], int (&cc)[kSliceUnroll], unsigned (&tt)[kSliceUnroll]) {
#pragma unroll
    for (int u = 0; u < kSliceUnroll; ++u) {
      cc[u] = a.col[kk[u]];  // ordinary loads: the lines that pieces share are met again in the L1 and the L2
      if (COLSUM) tt[u] = tbits[kk[u]];
    }
  };
  auto work = [&](int q0, int total, const int (&kk)[kSliceUnroll], const int (&jj)[kSliceUnroll], const int (&cc)[kSliceUnroll],
                  const unsigned (&tt)[kSliceUnroll]) {
#pragma unroll
    for (int u = 0; u < kSliceUnroll; ++u) {
      const int cidx = cc[u] - col0;
      if (COLSUM) {
        const unsigned tb = q0 + u * kWave < total ? tt[u] : 0u;
        if (((tb >> 10) & 31u) == 31u) {  // inf / nan: through the side array
          atomicAdd(a.poison + col0 + cidx, float(a.t[kk[u]]));
        } else if (tb & 0x7fffu) {
          atomicAdd(s_acc + cidx, (unsigned long long)half_bits_to_fixed(tb));
        }
      } else {
        float v = s_el[jj[u]] + s_er[cidx];
        v = v > 0.f ? v : a.slope * v;
        if (a.lse) v = __expf(v - s_lse[jj[u]]);
        a.out[kk[u]] = half_t(v);
      }
    }
  };
  auto bounds = [&](int base, int& b, int& e, float& elv, float& lsev) {
    const int r = base + lane;
    const bool in = r < r1;
    b = in ? lo[r] : 0;
    e = in ? hi[r] : 0;
    elv = lsev = 0.f;
    if (!COLSUM && in) {
      elv = a.el[r];
      if (a.lse) lsev = a.lse[r];
    }
  };
  int nb_ = 0, ne_ = 0;
  float nel = 0.f, nlse = 0.f;
  const int first = r0 + wave * kWave;
  if (first < r1) bounds(first, nb_, ne_, nel, nlse);
  for (int base = first; base < r1; base += kSliceWaves * kWave) {
    const int b = nb_, e = ne_;
    const float elv = nel, lsev = nlse;
    if (base + kSliceWaves * kWave < r1) bounds(base + kSliceWaves * kWave, nb_, ne_, nel, nlse);  // for the next batch
    int inc = e - b;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
      const int t = __shfl_up(inc, d);
      if (lane >= d) inc += t;
    }
    const int total = __shfl(inc, kWave - 1);
    if (lane == 0) s_p[0] = 0;
    s_p[lane + 1] = inc;
    s_d[lane] = b - (inc - (e - b));  // first position minus first slot
    if (!COLSUM) {
      s_el[lane] = elv;
      s_lse[lane] = lsev;
    }
    wave_sync();
    int kA[kSliceUnroll], jA[kSliceUnroll], cA[kSliceUnroll], kB[kSliceUnroll], jB[kSliceUnroll], cB[kSliceUnroll];
    unsigned tA[kSliceUnroll], tB[kSliceUnroll];
    if (total > 0) {
      plan_round(lane, total, kA, jA);
      issue(kA, cA, tA);
    }
    for (int qb = 0; qb < total; qb += kWave * kSliceUnroll) {
      const bool more = qb + kWave * kSliceUnroll < total;
      if (more) {
        plan_round(lane + qb + kWave * kSliceUnroll, total, kB, jB);
        issue(kB, cB, tB);
      }
      work(lane + qb, total, kA, jA, cA, tA);
      if (more) {
#pragma unroll
        for (int u = 0; u < kSliceUnroll; ++u) {
          kA[u] = kB[u];
          jA[u] = jB[u];
          cA[u] = cB[u];
          tA[u] = tB[u];
        }
      }
    }
    wave_sync();  // the wave's bookkeeping is rewritten for the next 64 rows
  }
  if (COLSUM) {
    __syncthreads();
    unsigned long long* dst = a.part + size_t(c) * size_t(a.ncols) + col0;
    for (int i = tid; i < wcols; i += kSliceThreads) dst[i] = s_acc[i];
  }
}

// out[j] = fp16(sum over the row chunks of their partial sums of column j); the side array of non-finite inputs is
// added and cleared
__global__ __launch_bounds__(kBlock) void colsum_reduce_kernel(const unsigned long long* __restrict__ part, int nch, int ncols,
                                                                float* __restrict__ poison, half_t* __restrict__ out) {
  const int j = blockIdx.x * kBlock + threadIdx.x;
  if (j >= ncols) return;
  long long sum = 0;
  for (int c = 0; c < nch; ++c) sum += (long long)part[size_t(c) * size_t(ncols) + j];
  double v = double(sum) * (1.0 / 16777216.0);
  const float p = poison ? poison[j] : 0.f;
  if (p != 0.f) {  // also true for nan
    v += double(p);
    poison[j] = 0.f;
  }
  out[j] = half_t(float(v));
}

// scut[s*nrows + r] = first CSR position of row r whose column is >= s*W (s = ns: end of the row)
__global__ void slice_cuts_kernel(const int* __restrict__ rowptr, const int* __restrict__ col, int nrows, int ns, int W,
                                  int* __restrict__ scut) {
  const int64_t idx = blockIdx.x * int64_t(blockDim.x) + threadIdx.x;
  if (idx >= int64_t(nrows) * (ns + 1)) return;
  const int s = int(idx / nrows), r = int(idx % nrows);
  int lo = rowptr[r], hi = rowptr[r + 1];
  if (s < ns) {
    const int64_t key = int64_t(s) * W;
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (col[mid] < key) lo = mid + 1;
      else hi = mid;
    }
  } else {
    lo = hi;
  }
  scut[idx] = lo;
}

// chunk_row[c] = first row whose first non-zero is at or beyond c * nnz / nch; chunk_row[nch] = nrows
__global__ void chunk_rows_kernel(const int* __restrict__ rowptr, int nrows, int64_t nnz, int nch, int* __restrict__ chunk_row) {
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c > nch) return;
  if (c == nch) {
    chunk_row[c] = nrows;
    return;
  }
  const int64_t target = nnz * c / nch;
  int lo = 0, hi = nrows;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (int64_t(rowptr[mid]) < target) lo = mid + 1;
    else hi = mid;
  }
  chunk_row[c] = lo;
}

hgnn_status build_col_slices(hgnn_plan* p, const hgnn_csr* g, int W, hipStream_t s) {
  (void)hipFree(p->scut);
  (void)hipFree(p->chunk_row);
  (void)hipFree(p->col_part);
  (void)hipFree(p->col_poison);
  p->scut = p->chunk_row = nullptr;
  p->col_part = nullptr;
  p->col_poison = nullptr;
  p->ns = 0;
  if (g->nrows == 0 || g->ncols == 0) return HGNN_OK;
  int dev = 0, cus = 256;
  HGNN_HIP(hipGetDevice(&dev));
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 8) cus = 256;
  const int ns = int(ceil_div(g->ncols, W));
  W = int(ceil_div(ceil_div(g->ncols, ns), 64) * 64);  // the same number of slices, of equal width (a short last slice would idle its compute units)
  // one workgroup per compute unit at a time (its LDS table fills most of the 160 KB): as many row chunks as give
  // every compute unit one (slice, chunk) pair, a multiple of 8 so that a chunk's slices share an XCD, and not so
  // many that a chunk is shorter than a few hundred rows
  int nch = 8 * std::max(1, (cus / 8) / ns);
  const int by_rows = 8 * int(ceil_div(g->nrows, 8 * 512));
  if (nch > by_rows) nch = by_rows;
  HGNN_HIP(hipMalloc(&p->scut, sizeof(int) * size_t(ns + 1) * size_t(g->nrows)));
  HGNN_HIP(hipMalloc(&p->chunk_row, sizeof(int) * size_t(nch + 1)));
  HGNN_HIP(hipMalloc(&p->col_part, sizeof(unsigned long long) * size_t(nch) * size_t(g->ncols)));
  HGNN_HIP(hipMalloc(&p->col_poison, sizeof(float) * size_t(g->ncols)));
  HGNN_HIP(hipMemsetAsync(p->col_poison, 0, sizeof(float) * size_t(g->ncols), s));
  slice_cuts_kernel<<<dim3(unsigned(ceil_div(int64_t(g->nrows) * (ns + 1), kBlock))), kBlock, 0, s>>>(g->rowptr, g->col, g->nrows,
                                                                                                    ns, W, p->scut);
  chunk_rows_kernel<<<dim3(unsigned(ceil_div(nch + 1, kBlock))), kBlock, 0, s>>>(g->rowptr, g->nrows, g->nnz, nch, p->chunk_row);
  HGNN_LAUNCH_CHECK("slice_cuts_kernel / chunk_rows_kernel");
  HGNN_HIP(hipStreamSynchronize(s));
  p->ns = ns;
  p->slice_w = W;
  p->nch = nch;
  return HGNN_OK;
}

static SliceArgs slice_args(const hgnn_plan* p, const hgnn_csr* g) {
  SliceArgs a{};
  a.scut = p->scut;
  a.chunk_row = p->chunk_row;
  a.col = g->col;
  a.nrows = g->nrows;
  a.ncols = g->ncols;
  a.ns = p->ns;
  a.nch = p->nch;
  a.W = p->slice_w;
  return a;
}

template <bool COLSUM>
static hgnn_status launch_slices(const hgnn_plan* p, const SliceArgs& a, hipStream_t s) {
  const size_t lds = slice_lds_bytes(a.W, COLSUM);
  // beyond 64 KB of dynamic LDS the runtime wants to be told, once per kernel and device
  static bool told[64][2] = {};
  int dev = 0;
  HGNN_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= 64 || !told[dev][COLSUM ? 1 : 0]) {
    HGNN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&edge_slice_kernel<COLSUM>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, int(slice_lds_bytes(kSliceMaxCols, true))));
    if (dev >= 0 && dev < 64) told[dev][COLSUM ? 1 : 0] = true;
  }
  edge_slice_kernel<COLSUM><<<dim3(unsigned(p->ns) * unsigned(p->nch)), kSliceThreads, lds, s>>>(a);
  HGNN_LAUNCH_CHECK("edge_slice_kernel");
  return HGNN_OK;
}

// e[k] = LeakyReLU(el[row k] + er[col k]) (one head), or alpha = exp(e - lse[row]) when lse is given, over the plan's
// column slices
hgnn_status slice_edge_score(const hgnn_plan* p, const hgnn_csr* g, const float* el, const float* er, const float* lse,
                             float slope, hgnn_half* out, hipStream_t s) {
  SliceArgs a = slice_args(p, g);
  a.el = el;
  a.er = er;
  a.lse = lse;
  a.slope = slope;
  a.out = reinterpret_cast<half_t*>(out);
  return launch_slices<false>(p, a, s);
}

}  // namespace hgnn

using namespace hgnn;

extern "C" {

hgnn_status hgnn_plan_add_slices(hgnn_plan* p, const hgnn_csr* g, int32_t slice_cols, void* stream) {
  clear_error();
  const char* who = "hgnn_plan_add_slices";
  HGNN_REQUIRE(p != nullptr, HGNN_EINVAL, "%s: plan is NULL", who);
  hgnn_status st = check_csr_args(g, who);
  if (st != HGNN_OK) return st;
  HGNN_REQUIRE(p->nrows == g->nrows && p->ncols == g->ncols && p->nnz == g->nnz, HGNN_EINVAL,
               "%s: the plan was built for another graph", who);
  HGNN_REQUIRE(slice_cols == 0 || (slice_cols >= 64 && slice_cols <= kSliceMaxCols), HGNN_EINVAL,
               "%s: slice_cols = %d outside [64, %d] (0 = default)", who, slice_cols, kSliceMaxCols);
  return build_col_slices(p, g, slice_cols == 0 ? kSliceMaxCols : slice_cols, static_cast<hipStream_t>(stream));
}

int32_t hgnn_plan_num_slices(const hgnn_plan* p) { return p ? p->ns : 0; }

hgnn_status hgnn_edge_colsum(const hgnn_csr* g, const hgnn_plan* p, int32_t H, const hgnn_half* t, hgnn_half* out,
                             void* stream) {
  clear_error();
  const char* who = "hgnn_edge_colsum";
  hgnn_status st = check_csr_args(g, who);
  if (st != HGNN_OK) return st;
  HGNN_REQUIRE(p != nullptr, HGNN_EINVAL, "%s: plan is NULL", who);
  HGNN_REQUIRE(p->nrows == g->nrows && p->ncols == g->ncols && p->nnz == g->nnz, HGNN_EINVAL,
               "%s: the plan was built for another graph", who);
  HGNN_REQUIRE(H >= 1, HGNN_EINVAL, "%s: H = %d must be positive", who, H);
  HGNN_REQUIRE(g->eid == nullptr, HGNN_EUNSUPPORTED, "%s: an edge-id map is not supported here", who);
  HGNN_REQUIRE(H == 1, HGNN_EUNSUPPORTED, "%s: one head only (use hgnn_edge_rowsum on the transposed graph)", who);
  HGNN_REQUIRE(p->ns > 0 || g->ncols == 0 || g->nrows == 0, HGNN_EINVAL,
               "%s: the plan holds no column slices (hgnn_plan_add_slices)", who);
  if (g->ncols == 0) return HGNN_OK;
  HGNN_REQUIRE(out != nullptr && (g->nnz == 0 || t != nullptr), HGNN_EINVAL, "%s: t or out is NULL", who);
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (g->nrows == 0) {  // no rows, hence no slices: every column sum is zero
    colsum_reduce_kernel<<<dim3(unsigned(ceil_div(g->ncols, kBlock))), kBlock, 0, s>>>(nullptr, 0, g->ncols, nullptr,
                                                                                       reinterpret_cast<half_t*>(out));
    HGNN_LAUNCH_CHECK("colsum_reduce_kernel");
    return HGNN_OK;
  }
  SliceArgs a = slice_args(p, g);
  a.t = reinterpret_cast<const half_t*>(t);
  a.part = p->col_part;
  a.poison = p->col_poison;
  st = launch_slices<true>(p, a, s);
  if (st != HGNN_OK) return st;
  colsum_reduce_kernel<<<dim3(unsigned(ceil_div(g->ncols, kBlock))), kBlock, 0, s>>>(p->col_part, p->nch, g->ncols, p->col_poison,
                                                                                     reinterpret_cast<half_t*>(out));
  HGNN_LAUNCH_CHECK("colsum_reduce_kernel");
  return HGNN_OK;
}

}  // extern "C"
