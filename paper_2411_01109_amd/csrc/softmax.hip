// Edge softmax (paper Eq. 1), its backward, and row sums of edge tensors, for gfx950.
//
// The scores of one row (neighbourhood) are the contiguous slice e[rowptr[i]*H, rowptr[i+1]*H),
// element j of the slice belonging to head j % H.  A wave owns a row: lane t walks the elements
// t, t+64, ... (so its head is fixed when H divides 64), keeps the first few in registers so a
// short row is read once, and the per-head max / sum are finished with xor shuffles over the
// lanes of equal head.  Rows longer than the plan's threshold are left to a kernel that gives
// a whole 1024-thread workgroup to each of them.  exp, sums and the division stay in fp32; the
// exponent is <= 0, so the numerator is in (0,1] (section 3.1.2) and alpha is rounded once.
#include "common.h"

namespace hgnn {

constexpr int kKeep = 4;        // elements per lane held in registers
constexpr int kBigBlock = 1024; // threads given to one long row

struct SoftmaxArgs {
  const int* rowptr;
  const int* big_row;
  const half_t* e;       // scores (forward) or nullptr / scores for the LeakyReLU mask (backward)
  const half_t* alpha;   // backward: alpha
  const half_t* dalpha;  // backward: d alpha
  half_t* out;           // forward: alpha; backward: de
  int nrows, H;
  int skip_above;        // rows longer than this are skipped by the wave kernel (0 = none)
  float slope;
};

// reduce over the lanes of a wave whose lane id is congruent modulo H (H divides 64)
__device__ __forceinline__ float wave_max_heads(float v, int H) {
  for (int off = H; off < kWave; off <<= 1) v = fmaxf(v, __shfl_xor(v, off));
  return v;
}
__device__ __forceinline__ float wave_sum_heads(float v, int H) {
  for (int off = H; off < kWave; off <<= 1) v += __shfl_xor(v, off);
  return v;
}

__global__ __launch_bounds__(kBlock) void softmax_fwd_wave_kernel(SoftmaxArgs a) {
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int64_t row = int64_t(blockIdx.x) * kWavesPerBlock + wave;
  if (row >= a.nrows) return;
  const int beg = a.rowptr[row], deg = a.rowptr[row + 1] - beg;
  if (deg == 0 || (a.skip_above > 0 && deg > a.skip_above)) return;
  const int64_t n = int64_t(deg) * a.H;
  const half_t* x = a.e + int64_t(beg) * a.H;
  half_t* y = a.out + int64_t(beg) * a.H;
  float v[kKeep];
  float m = -INFINITY;
#pragma unroll
  for (int t = 0; t < kKeep; ++t) {
    const int64_t i = lane + int64_t(kWave) * t;
    v[t] = i < n ? float(x[i]) : -INFINITY;
    m = fmaxf(m, v[t]);
  }
  for (int64_t i = lane + int64_t(kWave) * kKeep; i < n; i += kWave) m = fmaxf(m, float(x[i]));
  m = wave_max_heads(m, a.H);
  float z = 0.f;
#pragma unroll
  for (int t = 0; t < kKeep; ++t) {
    v[t] = __expf(v[t] - m);  // exp(-inf) = 0 for the padding
    z += v[t];
  }
  for (int64_t i = lane + int64_t(kWave) * kKeep; i < n; i += kWave) z += __expf(float(x[i]) - m);
  z = wave_sum_heads(z, a.H);
  const float inv = 1.f / z;
#pragma unroll
  for (int t = 0; t < kKeep; ++t) {
    const int64_t i = lane + int64_t(kWave) * t;
    if (i < n) y[i] = half_t(v[t] * inv);
  }
  for (int64_t i = lane + int64_t(kWave) * kKeep; i < n; i += kWave) y[i] = half_t(__expf(float(x[i]) - m) * inv);
}

// combine per-wave partials of a 1024-thread workgroup, per head; every thread gets the result of its head
template <bool IS_MAX>
__device__ __forceinline__ float block_reduce_heads(float v, int H, float* sm /* [16][64] */) {
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  v = IS_MAX ? wave_max_heads(v, H) : wave_sum_heads(v, H);
  __syncthreads();  // protects sm against the previous use
  if (lane < H) sm[wave * kWave + lane] = v;
  __syncthreads();
  const int h = lane % H;
  float r = sm[h];
  for (int w = 1; w < kBigBlock / kWave; ++w) r = IS_MAX ? fmaxf(r, sm[w * kWave + h]) : r + sm[w * kWave + h];
  return r;
}

__global__ __launch_bounds__(kBigBlock) void softmax_fwd_big_kernel(SoftmaxArgs a) {
  __shared__ float sm[(kBigBlock / kWave) * kWave];
  const int row = a.big_row[blockIdx.x];
  const int beg = a.rowptr[row];
  const int64_t n = int64_t(a.rowptr[row + 1] - beg) * a.H;
  const half_t* x = a.e + int64_t(beg) * a.H;
  half_t* y = a.out + int64_t(beg) * a.H;
  float m = -INFINITY;
  for (int64_t i = threadIdx.x; i < n; i += kBigBlock) m = fmaxf(m, float(x[i]));
  m = block_reduce_heads<true>(m, a.H, sm);
  float z = 0.f;
  for (int64_t i = threadIdx.x; i < n; i += kBigBlock) z += __expf(float(x[i]) - m);
  z = block_reduce_heads<false>(z, a.H, sm);
  const float inv = 1.f / z;
  for (int64_t i = threadIdx.x; i < n; i += kBigBlock) y[i] = half_t(__expf(float(x[i]) - m) * inv);
}

// backward: t = sum alpha*dalpha over the row (per head); de = alpha*(dalpha - t) [* LeakyReLU'(e)]
__global__ __launch_bounds__(kBlock) void softmax_bwd_wave_kernel(SoftmaxArgs a) {
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int64_t row = int64_t(blockIdx.x) * kWavesPerBlock + wave;
  if (row >= a.nrows) return;
  const int beg = a.rowptr[row], deg = a.rowptr[row + 1] - beg;
  if (deg == 0 || (a.skip_above > 0 && deg > a.skip_above)) return;
  const int64_t n = int64_t(deg) * a.H, off = int64_t(beg) * a.H;
  const half_t* al = a.alpha + off;
  const half_t* da = a.dalpha + off;
  float va[kKeep], vd[kKeep];
  float t = 0.f;
#pragma unroll
  for (int q = 0; q < kKeep; ++q) {
    const int64_t i = lane + int64_t(kWave) * q;
    va[q] = i < n ? float(al[i]) : 0.f;
    vd[q] = i < n ? float(da[i]) : 0.f;
    t = fmaf(va[q], vd[q], t);
  }
  for (int64_t i = lane + int64_t(kWave) * kKeep; i < n; i += kWave) t = fmaf(float(al[i]), float(da[i]), t);
  t = wave_sum_heads(t, a.H);
#pragma unroll
  for (int q = 0; q < kKeep; ++q) {
    const int64_t i = lane + int64_t(kWave) * q;
    if (i < n) {
      float d = va[q] * (vd[q] - t);
      if (a.e) d *= float(a.e[off + i]) > 0.f ? 1.f : a.slope;
      a.out[off + i] = half_t(d);
    }
  }
  for (int64_t i = lane + int64_t(kWave) * kKeep; i < n; i += kWave) {
    float d = float(al[i]) * (float(da[i]) - t);
    if (a.e) d *= float(a.e[off + i]) > 0.f ? 1.f : a.slope;
    a.out[off + i] = half_t(d);
  }
}

__global__ __launch_bounds__(kBigBlock) void softmax_bwd_big_kernel(SoftmaxArgs a) {
  __shared__ float sm[(kBigBlock / kWave) * kWave];
  const int row = a.big_row[blockIdx.x];
  const int beg = a.rowptr[row];
  const int64_t n = int64_t(a.rowptr[row + 1] - beg) * a.H, off = int64_t(beg) * a.H;
  const half_t* al = a.alpha + off;
  const half_t* da = a.dalpha + off;
  float t = 0.f;
  for (int64_t i = threadIdx.x; i < n; i += kBigBlock) t = fmaf(float(al[i]), float(da[i]), t);
  t = block_reduce_heads<false>(t, a.H, sm);
  for (int64_t i = threadIdx.x; i < n; i += kBigBlock) {
    float d = float(al[i]) * (float(da[i]) - t);
    if (a.e) d *= float(a.e[off + i]) > 0.f ? 1.f : a.slope;
    a.out[off + i] = half_t(d);
  }
}

// Scalar path for head counts that do not divide 64: one thread per (row, head).
__global__ __launch_bounds__(kBlock) void softmax_fwd_scalar_kernel(SoftmaxArgs a) {
  const int64_t idx = int64_t(blockIdx.x) * kBlock + threadIdx.x;
  if (idx >= int64_t(a.nrows) * a.H) return;
  const int row = int(idx / a.H), h = int(idx % a.H);
  const int beg = a.rowptr[row], end = a.rowptr[row + 1];
  if (beg == end) return;
  float m = -INFINITY, z = 0.f;
  for (int k = beg; k < end; ++k) m = fmaxf(m, float(a.e[int64_t(k) * a.H + h]));
  for (int k = beg; k < end; ++k) z += __expf(float(a.e[int64_t(k) * a.H + h]) - m);
  const float inv = 1.f / z;
  for (int k = beg; k < end; ++k) a.out[int64_t(k) * a.H + h] = half_t(__expf(float(a.e[int64_t(k) * a.H + h]) - m) * inv);
}

__global__ __launch_bounds__(kBlock) void softmax_bwd_scalar_kernel(SoftmaxArgs a) {
  const int64_t idx = int64_t(blockIdx.x) * kBlock + threadIdx.x;
  if (idx >= int64_t(a.nrows) * a.H) return;
  const int row = int(idx / a.H), h = int(idx % a.H);
  const int beg = a.rowptr[row], end = a.rowptr[row + 1];
  float t = 0.f;
  for (int k = beg; k < end; ++k) t = fmaf(float(a.alpha[int64_t(k) * a.H + h]), float(a.dalpha[int64_t(k) * a.H + h]), t);
  for (int k = beg; k < end; ++k) {
    const int64_t i = int64_t(k) * a.H + h;
    float d = float(a.alpha[i]) * (float(a.dalpha[i]) - t);
    if (a.e) d *= float(a.e[i]) > 0.f ? 1.f : a.slope;
    a.out[i] = half_t(d);
  }
}

// ---- row sums of an edge tensor ------------------------------------------------------------------------
struct RowsumArgs {
  const int* rowptr;
  const int* eid;
  const half_t* t;
  half_t* out;
  int nrows, H;
};

__global__ __launch_bounds__(kBlock) void edge_rowsum_wave_kernel(RowsumArgs a) {
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int64_t row = int64_t(blockIdx.x) * kWavesPerBlock + wave;
  if (row >= a.nrows) return;
  const int beg = a.rowptr[row], deg = a.rowptr[row + 1] - beg;
  const int64_t n = int64_t(deg) * a.H;
  const int h = lane % a.H;
  float s = 0.f;
  if (a.eid) {
    for (int64_t i = lane; i < n; i += kWave) s += float(a.t[int64_t(a.eid[beg + i / a.H]) * a.H + h]);
  } else {
    const half_t* x = a.t + int64_t(beg) * a.H;
    for (int64_t i = lane; i < n; i += kWave) s += float(x[i]);
  }
  s = wave_sum_heads(s, a.H);
  if (lane < a.H) a.out[row * a.H + lane] = half_t(s);
}

__global__ __launch_bounds__(kBlock) void edge_rowsum_scalar_kernel(RowsumArgs a) {
  const int64_t idx = int64_t(blockIdx.x) * kBlock + threadIdx.x;
  if (idx >= int64_t(a.nrows) * a.H) return;
  const int row = int(idx / a.H), h = int(idx % a.H);
  float s = 0.f;
  for (int k = a.rowptr[row]; k < a.rowptr[row + 1]; ++k) {
    const int64_t slot = a.eid ? a.eid[k] : k;
    s += float(a.t[slot * a.H + h]);
  }
  a.out[idx] = half_t(s);
}

static hgnn_status softmax_common(const char* who, const hgnn_csr* g, const hgnn_plan* p, int H) {
  hgnn_status st = check_csr_args(g, who);
  if (st != HGNN_OK) return st;
  HGNN_REQUIRE(H >= 1, HGNN_EINVAL, "%s: H = %d must be positive", who, H);
  HGNN_REQUIRE(g->eid == nullptr, HGNN_EUNSUPPORTED, "%s: an edge-id map is not supported here", who);
  if (p)
    HGNN_REQUIRE(p->nrows == g->nrows && p->ncols == g->ncols && p->nnz == g->nnz, HGNN_EINVAL,
                 "%s: the plan was built for another graph", who);
  return HGNN_OK;
}

}  // namespace hgnn

using namespace hgnn;

extern "C" {

hgnn_status hgnn_edge_softmax(const hgnn_csr* g, const hgnn_plan* p, int32_t H, const hgnn_half* e, hgnn_half* alpha,
                              void* stream) {
  clear_error();
  hgnn_status st = softmax_common("hgnn_edge_softmax", g, p, H);
  if (st != HGNN_OK) return st;
  if (g->nnz == 0 || g->nrows == 0) return HGNN_OK;
  HGNN_REQUIRE(e && alpha, HGNN_EINVAL, "hgnn_edge_softmax: e or alpha is NULL");
  hipStream_t s = static_cast<hipStream_t>(stream);
  SoftmaxArgs a{};
  a.rowptr = g->rowptr;
  a.e = reinterpret_cast<const half_t*>(e);
  a.out = reinterpret_cast<half_t*>(alpha);
  a.nrows = g->nrows;
  a.H = H;
  if (kWave % H != 0) {
    softmax_fwd_scalar_kernel<<<dim3(unsigned(ceil_div(int64_t(g->nrows) * H, kBlock))), kBlock, 0, s>>>(a);
    HGNN_LAUNCH_CHECK("softmax_fwd_scalar_kernel");
    return HGNN_OK;
  }
  a.skip_above = p ? p->big_deg : 0;
  a.big_row = p ? p->big_row : nullptr;
  softmax_fwd_wave_kernel<<<dim3(unsigned(ceil_div(g->nrows, kWavesPerBlock))), kBlock, 0, s>>>(a);
  HGNN_LAUNCH_CHECK("softmax_fwd_wave_kernel");
  if (p && p->n_big > 0) {
    softmax_fwd_big_kernel<<<dim3(unsigned(p->n_big)), kBigBlock, 0, s>>>(a);
    HGNN_LAUNCH_CHECK("softmax_fwd_big_kernel");
  }
  return HGNN_OK;
}

hgnn_status hgnn_edge_softmax_bwd(const hgnn_csr* g, const hgnn_plan* p, int32_t H, const hgnn_half* alpha,
                                  const hgnn_half* dalpha, const hgnn_half* e, float neg_slope, hgnn_half* de,
                                  void* stream) {
  clear_error();
  hgnn_status st = softmax_common("hgnn_edge_softmax_bwd", g, p, H);
  if (st != HGNN_OK) return st;
  if (g->nnz == 0 || g->nrows == 0) return HGNN_OK;
  HGNN_REQUIRE(alpha && dalpha && de, HGNN_EINVAL, "hgnn_edge_softmax_bwd: alpha, dalpha or de is NULL");
  hipStream_t s = static_cast<hipStream_t>(stream);
  SoftmaxArgs a{};
  a.rowptr = g->rowptr;
  a.e = reinterpret_cast<const half_t*>(e);
  a.alpha = reinterpret_cast<const half_t*>(alpha);
  a.dalpha = reinterpret_cast<const half_t*>(dalpha);
  a.out = reinterpret_cast<half_t*>(de);
  a.nrows = g->nrows;
  a.H = H;
  a.slope = neg_slope;
  if (kWave % H != 0) {
    softmax_bwd_scalar_kernel<<<dim3(unsigned(ceil_div(int64_t(g->nrows) * H, kBlock))), kBlock, 0, s>>>(a);
    HGNN_LAUNCH_CHECK("softmax_bwd_scalar_kernel");
    return HGNN_OK;
  }
  a.skip_above = p ? p->big_deg : 0;
  a.big_row = p ? p->big_row : nullptr;
  softmax_bwd_wave_kernel<<<dim3(unsigned(ceil_div(g->nrows, kWavesPerBlock))), kBlock, 0, s>>>(a);
  HGNN_LAUNCH_CHECK("softmax_bwd_wave_kernel");
  if (p && p->n_big > 0) {
    softmax_bwd_big_kernel<<<dim3(unsigned(p->n_big)), kBigBlock, 0, s>>>(a);
    HGNN_LAUNCH_CHECK("softmax_bwd_big_kernel");
  }
  return HGNN_OK;
}

hgnn_status hgnn_edge_rowsum(const hgnn_csr* g, int32_t H, const hgnn_half* t, hgnn_half* out, void* stream) {
  clear_error();
  hgnn_status st = check_csr_args(g, "hgnn_edge_rowsum");
  if (st != HGNN_OK) return st;
  HGNN_REQUIRE(H >= 1, HGNN_EINVAL, "hgnn_edge_rowsum: H = %d must be positive", H);
  if (g->nrows == 0) return HGNN_OK;
  HGNN_REQUIRE(out != nullptr && (g->nnz == 0 || t != nullptr), HGNN_EINVAL, "hgnn_edge_rowsum: t or out is NULL");
  hipStream_t s = static_cast<hipStream_t>(stream);
  RowsumArgs a{g->rowptr, g->eid, reinterpret_cast<const half_t*>(t), reinterpret_cast<half_t*>(out), g->nrows, H};
  if (kWave % H != 0) {
    edge_rowsum_scalar_kernel<<<dim3(unsigned(ceil_div(int64_t(g->nrows) * H, kBlock))), kBlock, 0, s>>>(a);
    HGNN_LAUNCH_CHECK("edge_rowsum_scalar_kernel");
  } else {
    edge_rowsum_wave_kernel<<<dim3(unsigned(ceil_div(g->nrows, kWavesPerBlock))), kBlock, 0, s>>>(a);
    HGNN_LAUNCH_CHECK("edge_rowsum_wave_kernel");
  }
  return HGNN_OK;
}

}  // extern "C"
