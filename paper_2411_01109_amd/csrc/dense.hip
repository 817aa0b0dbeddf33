// The dense side of a layer on the matrix cores: the projection h = X.W that feeds the sparse kernels
// (paper section 3.1.3, Eq. 2: the linear layer's output is the dense input of the SpMM; section 6: the
// input width is projected to the intermediate width by a GeMM; section 3.1.1: dense products are what
// matrix units are for, the sparse kernels are not), its two gradients, and the small dense pieces that tie
// the fused GAT backward to it.
//
// All three products are skinny (n rows in the millions, K and F in the tens to hundreds), so they are bound
// by streaming X / Y once through HBM, not by MFMA rate; the tiling below is chosen for full-width 16-byte
// loads and stores per lane, with the small operand (W) resident in LDS.
//
// MFMA shape used everywhere: v_mfma_f32_32x32x16_f16.  Operand A is 32 x 16: lane l holds row l % 32,
// columns 8*(l / 32) .. +7.  Operand B is 16 x 32: lane l holds column l % 32, rows 8*(l / 32) .. +7.
// The 32 x 32 result: lane l holds column l % 32; its element r (0..15) is row 8*(r / 4) + 4*(l / 32) + r % 4.
#include <algorithm>
#include <cstdio>

#include "common.h"

namespace hgnn {

typedef float float16_t __attribute__((ext_vector_type(16)));

constexpr int kRowsPerWave = 32;                           // rows of X one wave multiplies per step
constexpr int kRowsPerBlock = kRowsPerWave * kWavesPerBlock;
constexpr int kLinearLdsHalves = 28 * 1024;                // LDS budget of the weight tile, in halves (56 KB)

struct LinearArgs {
  int64_t n;
  int K, F;
  const half_t* X;
  int64_t ldx;
  const half_t* W;
  int64_t ldw;
  int trans;  // 0: W is [K][F]; 1: W is [F][K]
  half_t* Y;
  int64_t ldy;
  int KC;  // columns of X (rows of W) held in LDS at a time; a multiple of 16
};

__device__ __forceinline__ unsigned pack2(float a, float b) {
  const half2_t h = {half_t(a), half_t(b)};
  return __builtin_bit_cast(unsigned, h);
}

// Y[r, fc0 .. fc0 + 32*NT) for the 128 rows of a workgroup pass; fc0 = blockIdx.y * 32 * NT.  The weight tile
// sits in LDS transposed (Wt[f][k], pitch KC + 8 halves so that the 16-byte reads of 32 consecutive f are
// spread over the banks); it is loaded once per workgroup when K fits (KC >= K) and the workgroup then walks
// row blocks grid-stride, otherwise once per row block and chunk of K.  The product is formed transposed
// (features x rows), which leaves every lane with values of ONE row of Y: after one exchange between the two
// half-waves a lane stores two 16-byte pieces.
// the four 16-byte pieces of X that one lane feeds into four consecutive MFMA steps (64 columns from k0 on)
struct XGroup {
  half8_t b[4];
};

__device__ __forceinline__ XGroup load_xgroup(const half_t* xrow, bool row_ok, int k0, int kn, int hf) {
  XGroup g;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const half8_t zero = {0, 0, 0, 0, 0, 0, 0, 0};
    const int kk = k0 + 16 * u + 8 * hf;
    g.b[u] = (row_ok && kk < kn) ? *reinterpret_cast<const half8_t*>(xrow + kk) : zero;
  }
  return g;
}

template <int NT>
__global__ __launch_bounds__(kBlock, NT == 4 ? 3 : 4) void linear_kernel(LinearArgs a) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  half_t* Wt = reinterpret_cast<half_t*>(lds_raw);
  const int pitch = a.KC + 8;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int m = lane & 31, hf = lane >> 5;
  const int fc0 = blockIdx.y * 32 * NT;
  const int nchunks = (a.K + a.KC - 1) / a.KC;
  const int64_t nrb = (a.n + kRowsPerBlock - 1) / kRowsPerBlock;
  bool loaded = false;
  // The loads of X run one group (64 columns) ahead of the products, across chunk and row-block borders, so
  // that a wave always has memory requests in flight while it multiplies and stores.
  XGroup next{};
  if (int64_t(blockIdx.x) < nrb) {
    const int64_t row = int64_t(blockIdx.x) * kRowsPerBlock + wave * kRowsPerWave + m;
    next = load_xgroup(a.X + (row < a.n ? row : 0) * a.ldx, row < a.n, 0, min(a.KC, a.K), hf);
  }
  for (int64_t rb = blockIdx.x; rb < nrb; rb += gridDim.x) {
    const int64_t row = rb * kRowsPerBlock + wave * kRowsPerWave + m;
    const bool row_ok = row < a.n;
    const half_t* xrow = a.X + (row_ok ? row : 0) * a.ldx;
    float16_t acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
    for (int c = 0; c < nchunks; ++c) {
      const int kc = c * a.KC;
      const int kn = min(a.KC, a.K - kc);  // a multiple of 8
      if (!loaded || nchunks > 1) {
        if (loaded) __syncthreads();  // everyone is done with the previous tile
        const int total = 32 * NT * a.KC;
        if (a.trans) {
          for (int idx = threadIdx.x; idx < total; idx += kBlock) {
            const int fl = idx / a.KC, k = idx - fl * a.KC;
            const bool ok = k < kn && fc0 + fl < a.F;
            Wt[fl * pitch + k] = ok ? a.W[int64_t(fc0 + fl) * a.ldw + kc + k] : half_t(0);
          }
        } else {
          for (int idx = threadIdx.x; idx < total; idx += kBlock) {
            const int k = idx / (32 * NT), fl = idx - k * (32 * NT);
            const bool ok = k < kn && fc0 + fl < a.F;
            Wt[fl * pitch + k] = ok ? a.W[int64_t(kc + k) * a.ldw + fc0 + fl] : half_t(0);
          }
        }
        __syncthreads();
        loaded = true;
      }
      for (int k0 = 0; k0 < kn; k0 += 64) {
        const XGroup cur = next;
        // what comes after this group: more of this chunk, the next chunk of the row, or the next row block
        if (k0 + 64 < kn) {
          next = load_xgroup(xrow + kc, row_ok, k0 + 64, kn, hf);
        } else if (c + 1 < nchunks) {
          next = load_xgroup(xrow + kc + a.KC, row_ok, 0, min(a.KC, a.K - kc - a.KC), hf);
        } else if (rb + gridDim.x < nrb) {
          const int64_t nrow = row + int64_t(gridDim.x) * kRowsPerBlock;
          next = load_xgroup(a.X + (nrow < a.n ? nrow : 0) * a.ldx, nrow < a.n, 0, min(a.KC, a.K), hf);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          if (k0 + 16 * u < kn) {  // uniform; keeps the LDS reads inside the tile
#pragma unroll
            for (int t = 0; t < NT; ++t) {
              const half8_t w = *reinterpret_cast<const half8_t*>(Wt + (32 * t + m) * pitch + k0 + 16 * u + 8 * hf);
              acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(w, cur.b[u], acc[t], 0, 0, 0);
            }
          }
        }
      }
    }
    // acc[t][4q + i] = Y[row][fc0 + 32t + 8q + 4hf + i].  The lower half-wave keeps the groups q = 0, 1 and
    // gets the partner's halves of them, the upper one keeps q = 2, 3.
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const float16_t c = acc[t];
      const unsigned p0 = pack2(c[0], c[1]), p1 = pack2(c[2], c[3]), p2 = pack2(c[4], c[5]), p3 = pack2(c[6], c[7]);
      const unsigned p4 = pack2(c[8], c[9]), p5 = pack2(c[10], c[11]), p6 = pack2(c[12], c[13]), p7 = pack2(c[14], c[15]);
      const unsigned k0 = hf ? p4 : p0, k1 = hf ? p5 : p1, k2 = hf ? p6 : p2, k3 = hf ? p7 : p3;  // kept
      const unsigned g0 = unsigned(__shfl_xor(int(hf ? p0 : p4), 32)), g1 = unsigned(__shfl_xor(int(hf ? p1 : p5), 32));
      const unsigned g2 = unsigned(__shfl_xor(int(hf ? p2 : p6), 32)), g3 = unsigned(__shfl_xor(int(hf ? p3 : p7), 32));
      if (row_ok) {
        // lower half-wave: its own values are features 0..3 of a group, the partner's 4..7; upper: the other way
        const int4_t va = hf ? int4_t{int(g0), int(g1), int(k0), int(k1)} : int4_t{int(k0), int(k1), int(g0), int(g1)};
        const int4_t vb = hf ? int4_t{int(g2), int(g3), int(k2), int(k3)} : int4_t{int(k2), int(k3), int(g2), int(g3)};
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const int f = fc0 + 32 * t + 8 * (2 * hf + j);
          const int4_t v = j ? vb : va;
          half_t* dst = a.Y + row * a.ldy + f;
          if (f + 8 <= a.F) {
            *reinterpret_cast<int4_t*>(dst) = v;
          } else if (f < a.F) {
            const half8_t h = __builtin_bit_cast(half8_t, v);
#pragma unroll
            for (int i = 0; i < 8; ++i)
              if (i < a.F - f) dst[i] = h[i];
          }
        }
      }
    }
  }
}

// ---- weight gradient ---------------------------------------------------------------------------------
struct WgradArgs {
  int64_t n;
  int K, F;
  const half_t* X;
  int64_t ldx;
  const half_t* dY;
  int64_t ldy;
  float* part;  // [parts][K][F] fp32
  int parts;    // partial results = waves along blockIdx.x
};

constexpr int kWgradRows = 16;                 // rows of X and dY per MFMA step
constexpr int kWgradTile = 64;                 // a wave owns a 64 x 64 block of dW
constexpr int kWgradPitch = kWgradTile + 8;    // halves; 16-byte aligned rows, half-waves on different banks

// dW[kc0 .. kc0+64, fc0 .. fc0+64) = sum over rows of X[:, k] * dY[:, f].  Every wave walks groups of 16 rows
// grid-stride, keeps a 64 x 64 fp32 block in registers and leaves it as partial number p in the workspace
// (summed in a fixed order afterwards: no atomics, the same bits on every run).  The two operands are wanted
// column-wise (eight consecutive ROWS of one column per lane), so a wave loads its 16 x 64 tiles with 16-byte
// row reads, parks them in its private LDS region and picks the columns from there.
__global__ __launch_bounds__(kBlock) void wgrad_kernel(WgradArgs a) {
  __shared__ __align__(16) half_t lds[kWavesPerBlock][2][kWgradRows * kWgradPitch];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int m = lane & 31, hf = lane >> 5;
  const int kc0 = blockIdx.y * kWgradTile, fc0 = blockIdx.z * kWgradTile;
  half_t* xs = lds[wave][0];
  half_t* ys = lds[wave][1];
  const int p = blockIdx.x * kWavesPerBlock + wave;
  const int64_t ngroups = (a.n + kWgradRows - 1) / kWgradRows;
  float16_t acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  // lane -> (row of the group, 16-byte piece of the 64-column tile): 16 rows x 8 pieces = 128 pieces, 2 per lane
  const int pr = lane >> 3, pc = (lane & 7) * 8;
  for (int64_t g = p; g < ngroups; g += a.parts) {
    const int64_t r0 = g * kWgradRows;
    half8_t vx[2], vy[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int64_t row = r0 + pr + 8 * u;
      const half8_t zero = {0, 0, 0, 0, 0, 0, 0, 0};
      vx[u] = zero;
      vy[u] = zero;
      if (row < a.n) {
        // K and F are multiples of 8 here, so a piece is inside the matrix or outside it as a whole
        if (kc0 + pc < a.K) vx[u] = *reinterpret_cast<const half8_t*>(a.X + row * a.ldx + kc0 + pc);
        if (fc0 + pc < a.F) vy[u] = *reinterpret_cast<const half8_t*>(a.dY + row * a.ldy + fc0 + pc);
      }
    }
    wave_sync();  // the previous step's column reads are done
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      *reinterpret_cast<half8_t*>(xs + (pr + 8 * u) * kWgradPitch + pc) = vx[u];
      *reinterpret_cast<half8_t*>(ys + (pr + 8 * u) * kWgradPitch + pc) = vy[u];
    }
    wave_sync();
    half8_t xa[2], yb[2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        xa[t][j] = xs[(8 * hf + j) * kWgradPitch + 32 * t + m];
        yb[t][j] = ys[(8 * hf + j) * kWgradPitch + 32 * t + m];
      }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(xa[i], yb[j], acc[i][j], 0, 0, 0);
  }
  float* out = a.part + int64_t(p) * a.K * a.F;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int k = kc0 + 32 * i + 8 * (r / 4) + 4 * hf + (r % 4);
        const int f = fc0 + 32 * j + m;
        if (k < a.K && f < a.F) out[int64_t(k) * a.F + f] = acc[i][j][r];
      }
}

// out[q][e] = sum_{j < group} in[q*group + j][e] (j ascending, partials in_stride apart), e < elems; e = k*F + f lands at
// out + q*out_stride + k*out_ld + f.  Two rounds of this add the partial results in a fixed order.
__global__ __launch_bounds__(kBlock) void partial_sum_kernel(const float* __restrict__ in, int64_t in_stride, int nparts, int group,
                                                            int64_t elems, int F, float* __restrict__ out, int64_t out_stride,
                                                            int64_t out_ld) {
  const int64_t e = int64_t(blockIdx.x) * kBlock + threadIdx.x;
  const int q = blockIdx.y;
  if (e >= elems) return;
  const int j0 = q * group, j1 = min(nparts, j0 + group);
  float s = 0.f;
#pragma unroll 8
  for (int j = j0; j < j1; ++j) s += in[int64_t(j) * in_stride + e];
  const int64_t k = e / F, f = e - k * F;
  out[int64_t(q) * out_stride + k * out_ld + f] = s;
}

// ---- feature gradient of a GAT layer -------------------------------------------------------------------
struct FeatGradArgs {
  int64_t n;
  int H, D, F;
  const half_t* dV;
  int64_t lddv;
  const half_t* d_el;
  const half_t* d_er;
  const half_t* a_l;
  const half_t* a_r;
  const half_t* hfeat;
  int64_t ldh;
  half_t* dh;
  int64_t lddh;
  float* part;  // [gridDim.x][2][F]
};

// dh[i, f] = dV[i, f] + d_el[i, head f] * a_l[f] + d_er[i, head f] * a_r[f] (one fp16 rounding), and per
// workgroup the partial sums of da_l[f] = sum_i d_el[i, head f] * h[i, f] and da_r likewise.  LP lanes per row
// (a power of two >= F / 8), 8 features per lane; a thread keeps its feature group for all its rows, so the
// column sums stay in registers until the end, where the workgroup adds them in a fixed order through LDS.
template <int LP>
__global__ __launch_bounds__(kBlock) void gat_feature_grad_kernel(FeatGradArgs a) {
  constexpr int RPB = kBlock / LP;  // rows per workgroup pass
  __shared__ float red[2][kBlock][8];
  const int l = threadIdx.x % LP, rr = threadIdx.x / LP;
  const int f0 = 8 * l;
  const bool live = f0 < a.F;  // D % 8 == 0: a feature group lies in one head
  const int h = live ? f0 / a.D : 0;
  float al[8], ar[8], sl[8], sr[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    al[i] = live ? float(a.a_l[f0 + i]) : 0.f;
    ar[i] = live ? float(a.a_r[f0 + i]) : 0.f;
    sl[i] = 0.f;
    sr[i] = 0.f;
  }
  if (live) {
    for (int64_t row = int64_t(blockIdx.x) * RPB + rr; row < a.n; row += int64_t(gridDim.x) * RPB) {
      const half8_t v = *reinterpret_cast<const half8_t*>(a.dV + row * a.lddv + f0);
      const half8_t x = *reinterpret_cast<const half8_t*>(a.hfeat + row * a.ldh + f0);
      const float gl = float(a.d_el[row * a.H + h]), gr = float(a.d_er[row * a.H + h]);
      half8_t o;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        o[i] = half_t(float(v[i]) + gl * al[i] + gr * ar[i]);
        sl[i] += gl * float(x[i]);
        sr[i] += gr * float(x[i]);
      }
      *reinterpret_cast<half8_t*>(a.dh + row * a.lddh + f0) = o;
    }
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    red[0][threadIdx.x][i] = sl[i];
    red[1][threadIdx.x][i] = sr[i];
  }
  __syncthreads();
  // thread t < 2 * F sums one feature of one side over the RPB row slots, in slot order
  for (int t = threadIdx.x; t < 2 * a.F; t += kBlock) {
    const int side = t / a.F, f = t - side * a.F;
    float s = 0.f;
    for (int r = 0; r < RPB; ++r) s += red[side][r * LP + f / 8][f % 8];
    a.part[(int64_t(blockIdx.x) * 2 + side) * a.F + f] = s;
  }
}

static int linear_chunk(int K, int NT) {
  // largest multiple of 16 with 32*NT * (KC + 8) halves inside the LDS budget, at most K rounded up to 16
  int kc = kLinearLdsHalves / (32 * NT) - 8;
  kc = kc / 16 * 16;
  const int k16 = (K + 15) / 16 * 16;
  return kc < k16 ? kc : k16;
}

static int wgrad_parts(int K, int F) {
  // fewer partial results for larger weights: the workspace stays near 32 MB
  int64_t p = (int64_t(1) << 23) / (int64_t(K) * F);
  p = p < 64 ? 64 : (p > 1024 ? 1024 : p);
  int q = 64;
  while (q * 2 <= p) q *= 2;
  return q;
}

constexpr int kSumGroup = 32;
constexpr int kFeatGradBlocks = 1024;

}  // namespace hgnn

using namespace hgnn;

extern "C" {

hgnn_status hgnn_linear(int64_t n, int32_t K, int32_t F, const hgnn_half* X, int64_t ldx, const hgnn_half* W, int64_t ldw,
                        int32_t trans_w, hgnn_half* Y, int64_t ldy, void* stream) {
  clear_error();
  const char* who = "hgnn_linear";
  HGNN_REQUIRE(n >= 0 && K > 0 && F > 0, HGNN_EINVAL, "%s: n = %lld, K = %d, F = %d", who, static_cast<long long>(n), K, F);
  HGNN_REQUIRE(ldx >= K && ldy >= F && ldw >= (trans_w ? K : F), HGNN_EINVAL, "%s: leading dimension smaller than the row", who);
  HGNN_REQUIRE(K <= 65536 && F <= 65536, HGNN_EUNSUPPORTED, "%s: K = %d / F = %d above 65536", who, K, F);
  if (n == 0) return HGNN_OK;
  HGNN_REQUIRE(X && W && Y, HGNN_EINVAL, "%s: NULL argument", who);
  HGNN_REQUIRE(K % 8 == 0 && ldx % 8 == 0 && ldy % 8 == 0 && aligned16(X) && aligned16(Y), HGNN_EUNSUPPORTED,
               "%s: needs K %% 8 == 0, ldx %% 8 == 0, ldy %% 8 == 0 and 16-byte aligned X, Y (pad with zeros)", who);
  LinearArgs a{n, K, F, reinterpret_cast<const half_t*>(X), ldx, reinterpret_cast<const half_t*>(W), ldw, trans_w ? 1 : 0,
               reinterpret_cast<half_t*>(Y), ldy, 0};
  const int tiles = int(ceil_div(F, 32));
  const int NT = tiles >= 4 ? 4 : (tiles >= 2 ? 2 : 1);
  a.KC = linear_chunk(K, NT);
  const size_t lds = size_t(32 * NT) * size_t(a.KC + 8) * sizeof(half_t);
  const int64_t nrb = ceil_div(n, kRowsPerBlock);
  const int fy = int(ceil_div(tiles, NT));
  // when the whole weight fits in LDS a workgroup keeps it and takes several row blocks
  const int64_t want = a.KC >= K ? std::min<int64_t>(nrb, 2048) : nrb;
  HGNN_REQUIRE(want <= 0x7fffffff && fy <= 65535, HGNN_EUNSUPPORTED, "%s: grid too large", who);
  const dim3 grid{unsigned(want), unsigned(fy), 1u};
  hipStream_t s = static_cast<hipStream_t>(stream);
  switch (NT) {
    case 1: linear_kernel<1><<<grid, kBlock, lds, s>>>(a); break;
    case 2: linear_kernel<2><<<grid, kBlock, lds, s>>>(a); break;
    default: linear_kernel<4><<<grid, kBlock, lds, s>>>(a); break;
  }
  HGNN_LAUNCH_CHECK("linear_kernel");
  return HGNN_OK;
}

size_t hgnn_linear_wgrad_workspace(int32_t K, int32_t F) {
  if (K <= 0 || F <= 0) return 0;
  const int parts = wgrad_parts(K, F);
  return size_t(parts + parts / kSumGroup) * size_t(K) * size_t(F) * sizeof(float);
}

hgnn_status hgnn_linear_wgrad(int64_t n, int32_t K, int32_t F, const hgnn_half* X, int64_t ldx, const hgnn_half* dY,
                              int64_t ldy, float* dW, int64_t lddw, void* workspace, size_t workspace_bytes, void* stream) {
  clear_error();
  const char* who = "hgnn_linear_wgrad";
  HGNN_REQUIRE(n >= 0 && K > 0 && F > 0, HGNN_EINVAL, "%s: n = %lld, K = %d, F = %d", who, static_cast<long long>(n), K, F);
  HGNN_REQUIRE(ldx >= K && ldy >= F && lddw >= F, HGNN_EINVAL, "%s: leading dimension smaller than the row", who);
  HGNN_REQUIRE(K <= 4096 && F <= 4096, HGNN_EUNSUPPORTED, "%s: K = %d / F = %d above 4096", who, K, F);
  HGNN_REQUIRE(dW != nullptr, HGNN_EINVAL, "%s: dW is NULL", who);
  HGNN_REQUIRE(n == 0 || (X && dY), HGNN_EINVAL, "%s: NULL argument", who);
  HGNN_REQUIRE(workspace != nullptr && workspace_bytes >= hgnn_linear_wgrad_workspace(K, F), HGNN_EINVAL,
               "%s: workspace of %zu bytes, needs %zu (hgnn_linear_wgrad_workspace)", who, workspace_bytes,
               hgnn_linear_wgrad_workspace(K, F));
  HGNN_REQUIRE(K % 8 == 0 && F % 8 == 0 && ldx % 8 == 0 && ldy % 8 == 0 && aligned16(X) && aligned16(dY) &&
                   (reinterpret_cast<uintptr_t>(workspace) & 3u) == 0,
               HGNN_EUNSUPPORTED, "%s: needs K, F, ldx, ldy %% 8 == 0 and 16-byte aligned X, dY (pad with zeros)", who);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int parts = wgrad_parts(K, F);
  float* part = static_cast<float*>(workspace);
  float* part2 = part + size_t(parts) * size_t(K) * size_t(F);
  WgradArgs a{n, K, F, reinterpret_cast<const half_t*>(X), ldx, reinterpret_cast<const half_t*>(dY), ldy, part, parts};
  const dim3 grid{unsigned(parts / kWavesPerBlock), unsigned(ceil_div(K, kWgradTile)), unsigned(ceil_div(F, kWgradTile))};
  wgrad_kernel<<<grid, kBlock, 0, s>>>(a);
  HGNN_LAUNCH_CHECK("wgrad_kernel");
  const int64_t elems = int64_t(K) * F;
  const int mid = parts / kSumGroup;
  partial_sum_kernel<<<dim3(unsigned(ceil_div(elems, kBlock)), unsigned(mid)), kBlock, 0, s>>>(part, elems, parts, kSumGroup, elems,
                                                                                            F, part2, elems, F);
  HGNN_LAUNCH_CHECK("partial_sum_kernel");
  partial_sum_kernel<<<dim3(unsigned(ceil_div(elems, kBlock)), 1), kBlock, 0, s>>>(part2, elems, mid, mid, elems, F, dW, 0, lddw);
  HGNN_LAUNCH_CHECK("partial_sum_kernel");
  return HGNN_OK;
}

size_t hgnn_gat_feature_grad_workspace(int32_t H, int32_t D) {
  if (H <= 0 || D <= 0) return 0;
  return size_t(kFeatGradBlocks + kFeatGradBlocks / kSumGroup) * 2 * size_t(H) * size_t(D) * sizeof(float);
}

hgnn_status hgnn_gat_feature_grad(int64_t n, int32_t H, int32_t D, const hgnn_half* dV, int64_t lddv, const hgnn_half* d_el,
                                  const hgnn_half* d_er, const hgnn_half* a_l, const hgnn_half* a_r, const hgnn_half* hfeat,
                                  int64_t ldh, hgnn_half* dh, int64_t lddh, float* da_l, float* da_r, void* workspace,
                                  size_t workspace_bytes, void* stream) {
  clear_error();
  const char* who = "hgnn_gat_feature_grad";
  HGNN_REQUIRE(n >= 0 && H >= 1 && D >= 1 && int64_t(H) * D <= 512, HGNN_EINVAL, "%s: n = %lld, H = %d, D = %d out of range", who,
               static_cast<long long>(n), H, D);
  const int F = H * D;
  HGNN_REQUIRE(lddv >= F && ldh >= F && lddh >= F, HGNN_EINVAL, "%s: leading dimension smaller than F", who);
  HGNN_REQUIRE(da_l && da_r, HGNN_EINVAL, "%s: da_l or da_r is NULL", who);
  HGNN_REQUIRE(n == 0 || (dV && d_el && d_er && a_l && a_r && hfeat && dh), HGNN_EINVAL, "%s: NULL argument", who);
  HGNN_REQUIRE(workspace != nullptr && workspace_bytes >= hgnn_gat_feature_grad_workspace(H, D), HGNN_EINVAL,
               "%s: workspace of %zu bytes, needs %zu (hgnn_gat_feature_grad_workspace)", who, workspace_bytes,
               hgnn_gat_feature_grad_workspace(H, D));
  HGNN_REQUIRE(D % 8 == 0 && lddv % 8 == 0 && ldh % 8 == 0 && lddh % 8 == 0 && aligned16(dV) && aligned16(hfeat) && aligned16(dh) &&
                   (reinterpret_cast<uintptr_t>(workspace) & 3u) == 0,
               HGNN_EUNSUPPORTED, "%s: needs D %% 8 == 0, ld %% 8 == 0 and 16-byte aligned dV, hfeat, dh", who);
  hipStream_t s = static_cast<hipStream_t>(stream);
  float* part = static_cast<float*>(workspace);
  float* part2 = part + size_t(kFeatGradBlocks) * 2 * size_t(F);
  FeatGradArgs a{n, H, D, F, reinterpret_cast<const half_t*>(dV), lddv, reinterpret_cast<const half_t*>(d_el),
                 reinterpret_cast<const half_t*>(d_er), reinterpret_cast<const half_t*>(a_l), reinterpret_cast<const half_t*>(a_r),
                 reinterpret_cast<const half_t*>(hfeat), ldh, reinterpret_cast<half_t*>(dh), lddh, part};
  const int LP = pow2_at_least(F / 8);
  dim3 grid(kFeatGradBlocks);
  switch (LP) {
    case 1: gat_feature_grad_kernel<1><<<grid, kBlock, 0, s>>>(a); break;
    case 2: gat_feature_grad_kernel<2><<<grid, kBlock, 0, s>>>(a); break;
    case 4: gat_feature_grad_kernel<4><<<grid, kBlock, 0, s>>>(a); break;
    case 8: gat_feature_grad_kernel<8><<<grid, kBlock, 0, s>>>(a); break;
    case 16: gat_feature_grad_kernel<16><<<grid, kBlock, 0, s>>>(a); break;
    case 32: gat_feature_grad_kernel<32><<<grid, kBlock, 0, s>>>(a); break;
    default: gat_feature_grad_kernel<64><<<grid, kBlock, 0, s>>>(a); break;
  }
  HGNN_LAUNCH_CHECK("gat_feature_grad_kernel");
  // the partial of workgroup b is [2][F]: treat it as one row of 2F elements
  const int64_t elems = 2 * int64_t(F);
  const int mid = kFeatGradBlocks / kSumGroup;
  partial_sum_kernel<<<dim3(unsigned(ceil_div(elems, kBlock)), unsigned(mid)), kBlock, 0, s>>>(part, elems, kFeatGradBlocks,
                                                                                            kSumGroup, elems, int(elems), part2, elems,
                                                                                            elems);
  HGNN_LAUNCH_CHECK("partial_sum_kernel");
  // second round: the two sides go to two output arrays
  partial_sum_kernel<<<dim3(unsigned(ceil_div(F, kBlock)), 1), kBlock, 0, s>>>(part2, elems, mid, mid, F, F, da_l, 0, F);
  HGNN_LAUNCH_CHECK("partial_sum_kernel");
  partial_sum_kernel<<<dim3(unsigned(ceil_div(F, kBlock)), 1), kBlock, 0, s>>>(part2 + F, elems, mid, mid, F, F, da_r, 0, F);
  HGNN_LAUNCH_CHECK("partial_sum_kernel");
  return HGNN_OK;
}

}  // extern "C"
