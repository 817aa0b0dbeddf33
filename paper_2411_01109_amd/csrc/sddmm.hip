// fp16 SDDMM for gfx950 (paper sections 2.1.2 and 5.1): per non-zero, a reduction along the
// feature dimension of the row vertex's and the column vertex's vectors.
//
// Edge-parallel: a wave owns a tile of consecutive non-zeros; each group of L lanes takes one
// non-zero at a time and every lane loads 16 bytes (8 halves) of both feature rows -- the wide
// per-lane load of section 5.1.3 -- so only log2(D/8) shuffle rounds are left per head.  Results
// are collected in LDS and written back coalesced.
#include "common.h"

namespace hgnn {

struct SddmmArgs {
  const int* col;
  const int* erow;
  const half_t* U;
  const half_t* Vt;
  const half_t* a_l;
  const half_t* a_r;
  half_t* out;
  float* el;  // [nrows][H] fp32 scratch (factorised GAT score)
  float* er;  // [ncols][H]
  int64_t ldu, ldv, nnz;
  int nrows, ncols;
  int H, D, F;
  float slope;
};

constexpr int kTile = 256;  // non-zeros per wave

__device__ __forceinline__ float dot8(const half8_t& a, const half8_t& b) {
  float p = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) p = fmaf(float(a[i]), float(b[i]), p);
  return p;
}

// SCORE = false: out = <U[i,h], Vt[j,h]>.  SCORE = true: out = LeakyReLU(<a_l[h],U[i,h]> + <a_r[h],Vt[j,h]>).
template <int L, bool SCORE>
__global__ __launch_bounds__(kBlock) void sddmm_edge_kernel(SddmmArgs a) {
  constexpr int G = kWave / L;
  constexpr int C = kTile / G;  // consecutive non-zeros per group
  constexpr int U_ = 4;
  extern __shared__ __align__(16) unsigned char smem[];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int g = lane / L, l = lane % L;
  const int f0 = 8 * l;
  const bool active = f0 < a.F;
  const int LH = a.D / 8;  // lanes per head (power of two)
  const int head = active ? l / LH : 0;
  half_t* s_out = reinterpret_cast<half_t*>(smem) + size_t(wave) * kTile * a.H;
  const int64_t e0 = (int64_t(blockIdx.x) * kWavesPerBlock + wave) * kTile;
  const int n = e0 < a.nnz ? int(a.nnz - e0 < kTile ? a.nnz - e0 : kTile) : 0;
  half8_t al = half8_t(0), ar = half8_t(0);
  if (SCORE && active) {
    al = *reinterpret_cast<const half8_t*>(a.a_l + f0);
    ar = *reinterpret_cast<const half8_t*>(a.a_r + f0);
  }
  const int c0 = g * C < n ? g * C : n;
  const int c1 = c0 + C < n ? c0 + C : n;
  for (int i = c0; i < c1; i += U_) {
    half8_t u[U_], v[U_];
#pragma unroll
    for (int q = 0; q < U_; ++q) {
      u[q] = half8_t(0);
      v[q] = half8_t(0);
      if (i + q < c1 && active) {
        const int64_t k = e0 + i + q;
        u[q] = *reinterpret_cast<const half8_t*>(a.U + int64_t(a.erow[k]) * a.ldu + f0);
        v[q] = *reinterpret_cast<const half8_t*>(a.Vt + int64_t(a.col[k]) * a.ldv + f0);
      }
    }
#pragma unroll
    for (int q = 0; q < U_; ++q) {
      float p = SCORE ? dot8(al, u[q]) + dot8(ar, v[q]) : dot8(u[q], v[q]);
      for (int off = 1; off < LH; off <<= 1) p += __shfl_xor(p, off);
      if (SCORE) p = p > 0.f ? p : a.slope * p;
      if (i + q < c1 && active && (l % LH) == 0) s_out[(i + q) * a.H + head] = half_t(p);
    }
  }
  __syncthreads();
  for (int j = lane; j < n * a.H; j += kWave) a.out[e0 * a.H + j] = s_out[j];
}

// Scalar path: one thread per (non-zero, head).
template <bool SCORE>
__global__ __launch_bounds__(kBlock) void sddmm_scalar_kernel(SddmmArgs a) {
  const int64_t idx = int64_t(blockIdx.x) * kBlock + threadIdx.x;
  if (idx >= a.nnz * a.H) return;
  const int64_t k = idx / a.H;
  const int h = int(idx % a.H);
  const half_t* u = a.U + int64_t(a.erow[k]) * a.ldu + h * a.D;
  const half_t* v = a.Vt + int64_t(a.col[k]) * a.ldv + h * a.D;
  float p = 0.f;
  if (SCORE) {
    for (int d = 0; d < a.D; ++d) p = fmaf(float(a.a_l[h * a.D + d]), float(u[d]), p);
    for (int d = 0; d < a.D; ++d) p = fmaf(float(a.a_r[h * a.D + d]), float(v[d]), p);
    p = p > 0.f ? p : a.slope * p;
  } else {
    for (int d = 0; d < a.D; ++d) p = fmaf(float(u[d]), float(v[d]), p);
  }
  a.out[idx] = half_t(p);
}

// Factorised GAT score, step 1: proj[v,h] = <avec[h], feat[v,h]> for every vertex, fp32.
template <int L>
__global__ __launch_bounds__(kBlock) void vertex_proj_kernel(const half_t* __restrict__ feat, int64_t ld, int nv,
                                                              const half_t* __restrict__ avec, int F, int D,
                                                              float* __restrict__ proj, int H) {
  constexpr int G = kWave / L;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int g = lane / L, l = lane % L;
  const int f0 = 8 * l;
  const bool active = f0 < F;
  const int LH = D / 8;
  const int64_t v = (int64_t(blockIdx.x) * kWavesPerBlock + wave) * G + g;
  float p = 0.f;
  if (active && v < nv)
    p = dot8(*reinterpret_cast<const half8_t*>(avec + f0), *reinterpret_cast<const half8_t*>(feat + v * ld + f0));
  for (int off = 1; off < LH; off <<= 1) p += __shfl_xor(p, off);
  if (active && v < nv && (l % LH) == 0) proj[v * H + l / LH] = p;
}

// step 2: e[k,h] = LeakyReLU(el[row k, h] + er[col k, h])
__global__ __launch_bounds__(kBlock) void edge_score_kernel(SddmmArgs a) {
  const int64_t idx = int64_t(blockIdx.x) * kBlock + threadIdx.x;
  if (idx >= a.nnz * a.H) return;
  const int64_t k = idx / a.H;
  const int h = int(idx % a.H);
  const float s = a.el[int64_t(a.erow[k]) * a.H + h] + a.er[int64_t(a.col[k]) * a.H + h];
  a.out[idx] = half_t(s > 0.f ? s : a.slope * s);
}

template <bool SCORE>
static void launch_edge(int L, dim3 grid, size_t lds, hipStream_t s, const SddmmArgs& a) {
  switch (L) {
    case 1: sddmm_edge_kernel<1, SCORE><<<grid, kBlock, lds, s>>>(a); break;
    case 2: sddmm_edge_kernel<2, SCORE><<<grid, kBlock, lds, s>>>(a); break;
    case 4: sddmm_edge_kernel<4, SCORE><<<grid, kBlock, lds, s>>>(a); break;
    case 8: sddmm_edge_kernel<8, SCORE><<<grid, kBlock, lds, s>>>(a); break;
    case 16: sddmm_edge_kernel<16, SCORE><<<grid, kBlock, lds, s>>>(a); break;
    case 32: sddmm_edge_kernel<32, SCORE><<<grid, kBlock, lds, s>>>(a); break;
    default: sddmm_edge_kernel<64, SCORE><<<grid, kBlock, lds, s>>>(a); break;
  }
}

static void launch_proj(int L, dim3 grid, hipStream_t s, const half_t* feat, int64_t ld, int nv, const half_t* avec, int F,
                        int D, float* proj, int H) {
  switch (L) {
    case 1: vertex_proj_kernel<1><<<grid, kBlock, 0, s>>>(feat, ld, nv, avec, F, D, proj, H); break;
    case 2: vertex_proj_kernel<2><<<grid, kBlock, 0, s>>>(feat, ld, nv, avec, F, D, proj, H); break;
    case 4: vertex_proj_kernel<4><<<grid, kBlock, 0, s>>>(feat, ld, nv, avec, F, D, proj, H); break;
    case 8: vertex_proj_kernel<8><<<grid, kBlock, 0, s>>>(feat, ld, nv, avec, F, D, proj, H); break;
    case 16: vertex_proj_kernel<16><<<grid, kBlock, 0, s>>>(feat, ld, nv, avec, F, D, proj, H); break;
    case 32: vertex_proj_kernel<32><<<grid, kBlock, 0, s>>>(feat, ld, nv, avec, F, D, proj, H); break;
    default: vertex_proj_kernel<64><<<grid, kBlock, 0, s>>>(feat, ld, nv, avec, F, D, proj, H); break;
  }
}

}  // namespace hgnn

using namespace hgnn;

extern "C" hgnn_status hgnn_sddmm(const hgnn_csr* g, const hgnn_plan* p, hgnn_sddmm_op op, int32_t H, int32_t D,
                                  const hgnn_half* U, int64_t ldu, const hgnn_half* Vt, int64_t ldv,
                                  const hgnn_half* a_l, const hgnn_half* a_r, float neg_slope, hgnn_half* out,
                                  void* stream) {
  clear_error();
  hgnn_status st = check_csr_args(g, "hgnn_sddmm");
  if (st != HGNN_OK) return st;
  HGNN_REQUIRE(op == HGNN_SDDMM_DOT || op == HGNN_SDDMM_GAT_SCORE, HGNN_EINVAL, "hgnn_sddmm: unknown op %d", int(op));
  HGNN_REQUIRE(H >= 1 && D >= 1, HGNN_EINVAL, "hgnn_sddmm: H = %d, D = %d must be positive", H, D);
  const int64_t F64 = int64_t(H) * D;
  HGNN_REQUIRE(F64 <= (1 << 20), HGNN_EINVAL, "hgnn_sddmm: H * D too large");
  const int F = int(F64);
  HGNN_REQUIRE(F % 2 == 0, HGNN_EINVAL, "hgnn_sddmm: F = H*D = %d is odd; pad the feature length to the next even number", F);
  HGNN_REQUIRE(ldu >= F && ldv >= F && ldu % 2 == 0 && ldv % 2 == 0, HGNN_EINVAL, "hgnn_sddmm: bad leading dimension");
  HGNN_REQUIRE(g->eid == nullptr, HGNN_EUNSUPPORTED, "hgnn_sddmm: an edge-id map is not supported here");
  if (g->nnz == 0) return HGNN_OK;
  HGNN_REQUIRE(U && Vt && out, HGNN_EINVAL, "hgnn_sddmm: U, Vt or out is NULL");
  const bool score = op == HGNN_SDDMM_GAT_SCORE;
  HGNN_REQUIRE(!score || (a_l && a_r), HGNN_EINVAL, "hgnn_sddmm: GAT_SCORE needs a_l and a_r");
  if (p)
    HGNN_REQUIRE(p->nrows == g->nrows && p->ncols == g->ncols && p->nnz == g->nnz, HGNN_EINVAL,
                 "hgnn_sddmm: the plan was built for another graph");
  const int* erow = g->row ? g->row : (p ? p->edge_row : nullptr);
  HGNN_REQUIRE(erow != nullptr, HGNN_EINVAL, "hgnn_sddmm: needs COO row ids (g->row) or a plan");
  hipStream_t s = static_cast<hipStream_t>(stream);
  SddmmArgs a{};
  a.col = g->col;
  a.erow = erow;
  a.U = reinterpret_cast<const half_t*>(U);
  a.Vt = reinterpret_cast<const half_t*>(Vt);
  a.a_l = reinterpret_cast<const half_t*>(a_l);
  a.a_r = reinterpret_cast<const half_t*>(a_r);
  a.out = reinterpret_cast<half_t*>(out);
  a.ldu = ldu;
  a.ldv = ldv;
  a.nnz = g->nnz;
  a.nrows = g->nrows;
  a.ncols = g->ncols;
  a.H = H;
  a.D = D;
  a.F = F;
  a.slope = neg_slope;
  const int LH = D / 8;
  const bool vec = D % 8 == 0 && (LH & (LH - 1)) == 0 && F <= 512 && ldu % 8 == 0 && ldv % 8 == 0 && aligned16(U) &&
                   aligned16(Vt) && (!score || (aligned16(a_l) && aligned16(a_r))) &&
                   size_t(kTile) * H * sizeof(hgnn_half) * kWavesPerBlock <= 65536;
  if (!vec) {
    dim3 grid(unsigned(ceil_div(g->nnz * H, kBlock)));
    if (score) sddmm_scalar_kernel<true><<<grid, kBlock, 0, s>>>(a);
    else sddmm_scalar_kernel<false><<<grid, kBlock, 0, s>>>(a);
    HGNN_LAUNCH_CHECK("sddmm_scalar_kernel");
    return HGNN_OK;
  }
  const int L = pow2_at_least(F / 8);
  if (score && p && H <= p->max_H) {
    // project every vertex once, then one add per (edge, head)
    const int G = kWave / L;
    a.el = p->vscratch;
    a.er = p->vscratch + size_t(g->nrows) * H;
    launch_proj(L, dim3(unsigned(ceil_div(g->nrows, int64_t(kWavesPerBlock) * G))), s, a.U, ldu, g->nrows, a.a_l, F, D,
                a.el, H);
    HGNN_LAUNCH_CHECK("vertex_proj_kernel");
    launch_proj(L, dim3(unsigned(ceil_div(g->ncols, int64_t(kWavesPerBlock) * G))), s, a.Vt, ldv, g->ncols, a.a_r, F, D,
                a.er, H);
    HGNN_LAUNCH_CHECK("vertex_proj_kernel");
    edge_score_kernel<<<dim3(unsigned(ceil_div(g->nnz * H, kBlock))), kBlock, 0, s>>>(a);
    HGNN_LAUNCH_CHECK("edge_score_kernel");
    return HGNN_OK;
  }
  const size_t lds = size_t(kTile) * H * sizeof(hgnn_half) * kWavesPerBlock;
  dim3 grid(unsigned(ceil_div(g->nnz, int64_t(kTile) * kWavesPerBlock)));
  if (score) launch_edge<true>(L, grid, lds, s, a);
  else launch_edge<false>(L, grid, lds, s, a);
  HGNN_LAUNCH_CHECK("sddmm_edge_kernel");
  return HGNN_OK;
}
