// fp16 SDDMM for gfx950 (paper sections 2.1.2 and 5.1): per non-zero, a reduction along the
// feature dimension of the row vertex's and the column vertex's vectors.
//
// Edge-parallel over the plan's segments: a wave owns one segment of consecutive non-zeros and
// each group of L lanes takes a contiguous chunk of it, four non-zeros per step.  Every lane
// loads 16 bytes (8 halves) of the column vertex's row -- the wide per-lane load of section
// 5.1.3 -- while the row vertex's vector stays in registers for as long as the row does not
// change.  The four partial dot products of a step are reduced across the lanes of a head with a
// transposing butterfly (each exchange halves the number of live values), so a step costs 2+1
// exchanges instead of 4*log2(D/8).  Results are collected in LDS and written back coalesced.
#include "common.h"

namespace hgnn {

struct SddmmArgs {
  const int* rowptr;
  const int* col;
  const int* erow;  // COO row ids from the caller, or nullptr (then the row is searched in rowptr)
  const int* seg_lo;
  const int* seg_hi;
  const int* eid;  // result slot of every non-zero (column-blocked plans), or nullptr: slot = position
  const half_t* U;
  const half_t* Vt;
  const half_t* a_l;
  const half_t* a_r;
  half_t* out;
  const float* lse;  // [nrows][H] or nullptr; when set the edge score kernel writes exp(score - lse[row]) = alpha
  float* el;  // [nrows][H] fp32 scratch (factorised GAT score)
  float* er;  // [ncols][H]
  int64_t ldu, ldv, nnz, nseg;
  int nrows, ncols;
  int H, D, F, S;
  float slope;
  // all column blocks of a plan in one launch (workgroups numbered block after block): the table of the blocks'
  // arrays, or nullptr when the arrays above describe the one graph of the launch
  const hgnn_seg_block* blocks;
  int nblocks;
};

constexpr int kTile = 256;  // non-zeros per wave in the kernels that run without a plan

__device__ __forceinline__ float dot8(const half8_t& a, const half8_t& b) {
  float p = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) p = fmaf(float(a[i]), float(b[i]), p);
  return p;
}

struct SddmmLds {
  int per, spad, col_off, row_off, blk_off, out_off, total;
};
__host__ __device__ inline SddmmLds sddmm_lds_layout(int S, int H) {
  SddmmLds o;
  o.per = 4 * ((S + 255) / 256);
  o.spad = kWave * o.per;
  o.col_off = 0;
  o.row_off = o.spad * 4;
  o.blk_off = o.row_off + o.spad * 4;
  o.out_off = o.blk_off + ((o.spad + 15) & ~15);
  o.total = o.out_off + ((o.spad * H * 2 + 15) & ~15);
  return o;
}

// DOT over one plan segment per wave:  out[k,h] = <U[row k, h], Vt[col k, h]>
// MASK: one head whose length is not a multiple of 8 -- the group's lanes cover the padded row pitch and
// the elements past D are forced to zero on both operands (whatever the padding columns hold).
// VW = halves per lane and load: 8 (16 bytes), or 4 / 2 for the vector-width study of section 6.3.1 (a head
// then spans D/VW lanes and the reduction across lanes has more rounds).
template <int L, int VW, bool MASK>
__global__ __launch_bounds__(kBlock, 8) void sddmm_seg_kernel(SddmmArgs a) {
  constexpr int G = kWave / L;
  typedef _Float16 hv_t __attribute__((ext_vector_type(VW)));
  extern __shared__ __align__(16) unsigned char smem[];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int g = lane / L, l = lane % L;
  const int f0 = VW * l;
  const bool active = f0 < a.F;
  const int f0c = active ? f0 : 0;
  const int LH = MASK ? L : a.D / VW;  // lanes per head (power of two)
  const int head = f0c / a.D;
  const int nvalid = active ? a.F - f0 : 0;  // MASK: elements of this lane's vector that exist
  const bool writer = MASK || active;         // MASK: every lane of the group may end up holding a result
  auto load8 = [&](const half_t* p) -> hv_t {
    hv_t v = *reinterpret_cast<const hv_t*>(p);
    if (MASK && nvalid < VW) {
#pragma unroll
      for (int i = 0; i < VW; ++i)
        if (i >= nvalid) v[i] = half_t(0);
    }
    return v;
  };
  auto dot = [&](const hv_t& x, const hv_t& y) -> float {
    float p = 0.f;
#pragma unroll
    for (int i = 0; i < VW; ++i) p = fmaf(float(x[i]), float(y[i]), p);
    return p;
  };
  const int lh = l % LH;
  const int S = a.S;
  const SddmmLds lay = sddmm_lds_layout(S, a.H);
  unsigned char* base = smem + size_t(wave) * lay.total;
  int* s_col = reinterpret_cast<int*>(base + lay.col_off);
  int* s_row = reinterpret_cast<int*>(base + lay.row_off);
  int* s_blk = reinterpret_cast<int*>(base + lay.blk_off);
  half_t* s_out = reinterpret_cast<half_t*>(base + lay.out_off);

  const int wpb = int(blockDim.x) / kWave;
  int64_t wg = blockIdx.x;
  if (a.blocks) {  // find this workgroup's block and take over its arrays
    int b = 0;
    for (;;) {
      const int64_t c = (a.blocks[b].nseg + wpb - 1) / wpb;
      if (wg < c || b + 1 == a.nblocks) break;
      wg -= c;
      ++b;
    }
    const hgnn_seg_block& B = a.blocks[b];
    a.rowptr = B.rowptr;
    a.col = B.col;
    a.eid = B.eid;
    a.seg_lo = B.seg_lo;
    a.seg_hi = B.seg_hi;
    a.nseg = B.nseg;
    a.nnz = B.nnz;
  }
  const int64_t seg = wg * wpb + wave;
  const bool valid = seg < a.nseg;
  const int64_t e0 = seg * S;
  const int n = valid ? int(a.nnz - e0 < S ? a.nnz - e0 : S) : 0;
  const int row_lo = valid ? a.seg_lo[seg] : 0, row_hi = valid ? a.seg_hi[seg] : -1;
  seg_stage_cols(a.col, e0, lane, lay.spad, n, stream_nontemporal(a.nnz), [&](int i, int c) { s_col[i] = c; });
  seg_stage_rows(s_row, s_blk, lane, lay.per, n, row_lo, row_hi, a.rowptr, e0);

  const int C = 4 * ((S + 4 * G - 1) / (4 * G));
  const int c0 = g * C < n ? g * C : n;
  const int c1 = c0 + C < n ? c0 + C : n;
  int cur = -1;
  hv_t u = hv_t(0);
  if (c0 < c1) {
    cur = s_row[c0];
    u = load8(a.U + int64_t(cur) * a.ldu + f0c);
  }
  for (int i = c0; i < c1; i += 4) {
    const int4_t cols = *reinterpret_cast<const int4_t*>(s_col + i);
    const int blk = s_blk[i >> 2];
    hv_t v[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) v[q] = load8(a.Vt + int64_t(cols[q]) * a.ldv + f0c);
    float p[4];
    if (blk == cur) {
#pragma unroll
      for (int q = 0; q < 4; ++q) p[q] = dot(u, v[q]);
    } else {
      const int4_t rows = *reinterpret_cast<const int4_t*>(s_row + i);
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        p[q] = 0.f;
        if (i + q < c1) {
          if (rows[q] != cur) {
            cur = rows[q];
            u = load8(a.U + int64_t(cur) * a.ldu + f0c);
          }
          p[q] = dot(u, v[q]);
        }
      }
    }
    // transposing butterfly over the LH lanes of a head: 4 values -> 2 -> 1, then plain exchanges
    if (LH >= 2) {
      const bool b0 = lh & 1;
      const float r0 = __shfl_xor(b0 ? p[0] : p[2], 1);
      const float r1 = __shfl_xor(b0 ? p[1] : p[3], 1);
      p[0] = (b0 ? p[2] : p[0]) + r0;  // edges {0,1} on even lanes, {2,3} on odd lanes
      p[1] = (b0 ? p[3] : p[1]) + r1;
      if (LH >= 4) {
        const bool b1 = (lh >> 1) & 1;
        const float r = __shfl_xor(b1 ? p[0] : p[1], 2);
        p[0] = (b1 ? p[1] : p[0]) + r;  // edge 2*b0 + b1
        for (int off = 4; off < LH; off <<= 1) p[0] += __shfl_xor(p[0], off);
        const int e = i + 2 * int(b0) + int(b1);
        if (writer && lh < 4 && e < c1) s_out[e * a.H + head] = half_t(p[0]);
      } else {
        const int e = i + 2 * int(b0);
        if (active && e < c1) s_out[e * a.H + head] = half_t(p[0]);
        if (active && e + 1 < c1) s_out[(e + 1) * a.H + head] = half_t(p[1]);
      }
    } else if (active) {
#pragma unroll
      for (int q = 0; q < 4; ++q)
        if (i + q < c1) s_out[(i + q) * a.H + head] = half_t(p[q]);
    }
  }
  wave_sync();
  // coalesced write-back, 16 bytes per lane where the destination allows it
  const int tot = n * a.H;
  half_t* dst = a.out + e0 * a.H;
  if (a.eid) {  // a column block: the non-zeros of a row piece are consecutive in the result, pieces are not
    for (int j = lane; j < tot; j += kWave) {
      const int k = j / a.H;
      a.out[int64_t(a.eid[e0 + k]) * a.H + (j - k * a.H)] = s_out[j];
    }
  } else if ((reinterpret_cast<uintptr_t>(dst) & 15u) == 0) {
    const int nv = tot / 8;
    for (int j = lane; j < nv; j += kWave)
      reinterpret_cast<half8_t*>(dst)[j] = reinterpret_cast<const half8_t*>(s_out)[j];
    for (int j = nv * 8 + lane; j < tot; j += kWave) dst[j] = s_out[j];
  } else {
    for (int j = lane; j < tot; j += kWave) dst[j] = s_out[j];
  }
}

// Without a plan: tiles of kTile non-zeros, row ids from the caller's COO array.
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
        const int r = a.erow ? a.erow[k] : row_of_edge(a.rowptr, a.nrows, k);
        u[q] = *reinterpret_cast<const half8_t*>(a.U + int64_t(r) * a.ldu + f0);
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
  wave_sync();
  for (int j = lane; j < n * a.H; j += kWave) a.out[e0 * a.H + j] = s_out[j];
}

// Scalar path: one thread per (non-zero, head).
template <bool SCORE>
__global__ __launch_bounds__(kBlock) void sddmm_scalar_kernel(SddmmArgs a) {
  const int64_t idx = int64_t(blockIdx.x) * kBlock + threadIdx.x;
  if (idx >= a.nnz * a.H) return;
  const int64_t k = idx / a.H;
  const int h = int(idx % a.H);
  const int r = a.erow ? a.erow[k] : row_of_edge(a.rowptr, a.nrows, k);
  const half_t* u = a.U + int64_t(r) * a.ldu + h * a.D;
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

// step 2, one plan segment per wave: e[k,h] = LeakyReLU(el[row k, h] + er[col k, h]); row ids
// come from the offset array (staged in LDS), so the only per-edge stream read is the column id.
template <int HT>
__global__ __launch_bounds__(kBlock) void edge_score_seg_kernel(SddmmArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int S = a.S;
  const int per = seg_slots_per_lane(S), spad = kWave * per;
  int* s_row = reinterpret_cast<int*>(smem) + size_t(wave) * (spad + spad / 4);
  int* s_blk = s_row + spad;
  const int64_t seg = int64_t(blockIdx.x) * kWavesPerBlock + wave;
  const bool valid = seg < a.nseg;
  const int64_t e0 = seg * S;
  const int n = valid ? int(a.nnz - e0 < S ? a.nnz - e0 : S) : 0;
  seg_stage_rows<true>(s_row, s_blk, lane, per, n, valid ? a.seg_lo[seg] : 0, valid ? a.seg_hi[seg] : -1, a.rowptr, e0);
  if (HT == 0) {  // any head count: one output element per lane and step
    const int tot = n * a.H;
    for (int j = lane; j < tot; j += kWave) {
      const int k = j / a.H, h = j - k * a.H;
      float s = a.el[int64_t(s_row[k]) * a.H + h] + a.er[int64_t(a.col[e0 + k]) * a.H + h];
      s = s > 0.f ? s : a.slope * s;
      if (a.lse) s = __expf(s - a.lse[int64_t(s_row[k]) * a.H + h]);
      a.out[e0 * a.H + j] = half_t(s);
    }
    return;
  }
  // H in {1,2,4,8}: a lane produces 8 consecutive outputs (8/H non-zeros) and stores them as 16 bytes
  constexpr int H = HT > 0 ? HT : 1;
  constexpr int EPL = 8 / H;
  typedef float fv_t __attribute__((ext_vector_type(H)));
  half_t* dst = a.out + e0 * H;
  const bool vec_ok = (reinterpret_cast<uintptr_t>(dst) & 15u) == 0;
  for (int kb = lane * EPL; kb < n; kb += kWave * EPL) {
    half8_t o = half8_t(0);
    int rows[EPL], cols[EPL];
    if (EPL >= 4 && kb + EPL <= n && (reinterpret_cast<uintptr_t>(a.col + e0 + kb) & 15u) == 0) {  // 16-byte loads of ids
#pragma unroll
      for (int v = 0; v < EPL / 4; ++v) {
        const int4_t c4 = *reinterpret_cast<const int4_t*>(a.col + e0 + kb + 4 * v);
        const int4_t r4 = *reinterpret_cast<const int4_t*>(s_row + kb + 4 * v);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          cols[4 * v + q] = c4[q];
          rows[4 * v + q] = r4[q];
        }
      }
    } else {
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        const int k = kb + e < n ? kb + e : n - 1;
        cols[e] = a.col[e0 + k];
        rows[e] = s_row[k];
      }
    }
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      const fv_t vl = *reinterpret_cast<const fv_t*>(a.el + int64_t(rows[e]) * H);
      const fv_t vr = *reinterpret_cast<const fv_t*>(a.er + int64_t(cols[e]) * H);
#pragma unroll
      for (int h = 0; h < H; ++h) {
        float s = vl[h] + vr[h];
        s = s > 0.f ? s : a.slope * s;
        if (a.lse) s = __expf(s - a.lse[int64_t(rows[e]) * H + h]);
        o[e * H + h] = half_t(s);
      }
    }
    if (vec_ok && kb + EPL <= n) {
      *reinterpret_cast<half8_t*>(dst + kb * H) = o;
    } else {
#pragma unroll
      for (int q = 0; q < 8; ++q)
        if (kb * H + q < n * H) dst[kb * H + q] = o[q];
    }
  }
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

template <int VW>
static void launch_seg_vw(int L, bool mask, dim3 grid, int threads, size_t lds, hipStream_t s, const SddmmArgs& a) {
#define LAUNCH_SEG(LL)                                                                   \
  do {                                                                                  \
    if (mask && VW == 8) sddmm_seg_kernel<LL, 8, true><<<grid, threads, lds, s>>>(a);   \
    else sddmm_seg_kernel<LL, VW, false><<<grid, threads, lds, s>>>(a);                 \
  } while (0)
  switch (L) {
    case 1: LAUNCH_SEG(1); break;
    case 2: LAUNCH_SEG(2); break;
    case 4: LAUNCH_SEG(4); break;
    case 8: LAUNCH_SEG(8); break;
    case 16: LAUNCH_SEG(16); break;
    case 32: LAUNCH_SEG(32); break;
    default: LAUNCH_SEG(64); break;
  }
#undef LAUNCH_SEG
}

static void launch_seg(int L, int vw, bool mask, dim3 grid, int threads, size_t lds, hipStream_t s, const SddmmArgs& a) {
  if (vw == 8) launch_seg_vw<8>(L, mask, grid, threads, lds, s, a);
  else if (vw == 4) launch_seg_vw<4>(L, false, grid, threads, lds, s, a);
  else launch_seg_vw<2>(L, false, grid, threads, lds, s, a);
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

static hgnn_status launch_edge_score(const SddmmArgs& a, int64_t seg_blocks, hipStream_t s) {
  const int spad = kWave * 4 * ((a.S + 255) / 256);
  const size_t lds = size_t(spad + spad / 4) * sizeof(int) * kWavesPerBlock;
  const dim3 gs{unsigned(seg_blocks > 0 ? seg_blocks : 1), 1u, 1u};
  switch (a.H) {
    case 1: edge_score_seg_kernel<1><<<gs, kBlock, lds, s>>>(a); break;
    case 2: edge_score_seg_kernel<2><<<gs, kBlock, lds, s>>>(a); break;
    case 4: edge_score_seg_kernel<4><<<gs, kBlock, lds, s>>>(a); break;
    case 8: edge_score_seg_kernel<8><<<gs, kBlock, lds, s>>>(a); break;
    default: edge_score_seg_kernel<0><<<gs, kBlock, lds, s>>>(a); break;
  }
  HGNN_LAUNCH_CHECK("edge_score_seg_kernel");
  return HGNN_OK;
}

hgnn_status gat_project(const hgnn_plan* p, const hgnn_csr* g, int H, int D, const hgnn_half* U, int64_t ldu,
                        const hgnn_half* Vt, int64_t ldv, const hgnn_half* a_l, const hgnn_half* a_r, hipStream_t s,
                        const char* who) {
  const int F = H * D, LH = D / 8;
  // Vt == nullptr: only the row side is wanted
  HGNN_REQUIRE(D % 8 == 0 && (LH & (LH - 1)) == 0 && F <= 512 && ldu % 8 == 0 && ldv % 8 == 0 && aligned16(U) &&
                   aligned16(Vt) && aligned16(a_l) && aligned16(a_r),
               HGNN_EUNSUPPORTED,
               "%s: the per-vertex projection needs D = 8 * 2^k, H * D <= 512, ld %% 8 == 0 and 16-byte aligned U, Vt, a_l, a_r",
               who);
  HGNN_REQUIRE(H <= p->max_H, HGNN_EINVAL, "%s: H = %d exceeds the plan's max_H = %d", who, H, p->max_H);
  const int L = pow2_at_least(F / 8), G = kWave / L;
  float* el = p->vscratch;
  float* er = p->vscratch + size_t(g->nrows) * H;
  launch_proj(L, dim3(unsigned(ceil_div(g->nrows, int64_t(kWavesPerBlock) * G))), s, reinterpret_cast<const half_t*>(U), ldu,
              g->nrows, reinterpret_cast<const half_t*>(a_l), F, D, el, H);
  HGNN_LAUNCH_CHECK("vertex_proj_kernel");
  if (Vt) {
    launch_proj(L, dim3(unsigned(ceil_div(g->ncols, int64_t(kWavesPerBlock) * G))), s, reinterpret_cast<const half_t*>(Vt),
                ldv, g->ncols, reinterpret_cast<const half_t*>(a_r), F, D, er, H);
    HGNN_LAUNCH_CHECK("vertex_proj_kernel");
  }
  return HGNN_OK;
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
  hipStream_t s = static_cast<hipStream_t>(stream);
  SddmmArgs a{};
  a.rowptr = g->rowptr;
  a.col = g->col;
  a.erow = g->row;
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
  if (p) {
    a.seg_lo = p->seg_row_lo;
    a.seg_hi = p->seg_row_hi;
    a.nseg = p->nseg;
    a.S = p->S;
  }
  const int LH = D / 8;
  const bool wide = F <= 512 && ldu % 8 == 0 && ldv % 8 == 0 && aligned16(U) && aligned16(Vt);
  const bool vec = wide && D % 8 == 0 && (LH & (LH - 1)) == 0 && (!score || (aligned16(a_l) && aligned16(a_r)));
  // one head of any even length: 16-byte loads up to the padded pitch, the tail masked (DOT over a plan only)
  const bool masked = wide && !vec && !score && H == 1 && p != nullptr;
  const int L = (vec || masked) ? pow2_at_least((F + 7) / 8) : 0;
  const int64_t seg_blocks = p ? ceil_div(p->nseg, kWavesPerBlock) : 0;

  if (vec && score && p && H <= p->max_H) {
    // project every vertex once, then one add per (edge, head)
    hgnn_status st2 = gat_project(p, g, H, D, U, ldu, Vt, ldv, a_l, a_r, s, "hgnn_sddmm");
    if (st2 != HGNN_OK) return st2;
    a.el = p->vscratch;
    a.er = p->vscratch + size_t(g->nrows) * H;
    if (H == 1 && p->ns > 0) return slice_edge_score(p, g, a.el, a.er, nullptr, neg_slope, out, s);
    return launch_edge_score(a, seg_blocks, s);
  }
  if ((vec || masked) && !score && p) {
    // halves per lane: the plan's setting, when the shape allows a narrower load than 16 bytes
    int vw = p->vec_halves;
    int Ls = L;
    if (vw != 8) {
      const int lh = D / vw;
      HGNN_REQUIRE(vec && F <= kWave * vw && D % vw == 0 && (lh & (lh - 1)) == 0, HGNN_EUNSUPPORTED,
                   "hgnn_sddmm: %d halves per lane needs F <= %d and D / %d a power of two", vw, kWave * vw, vw);
      Ls = pow2_at_least(F / vw);
    }
    const size_t seg_per_wave = size_t(sddmm_lds_layout(a.S, H).total);
    const int wpb = waves_per_block_for_lds(seg_per_wave, true);
    const size_t lds = seg_per_wave * wpb;
    if (lds <= 65536 && p->nb > 1 && !p->block_eid) {  // (a plan built over an edge-id map maps its blocks to that map's slots)
      // column-blocked plan: block after block, so that the gathered slice of Vt stays cache resident; on the plan's
      // finer cut where it has one (no partial rows here, so narrower blocks cost nothing)
      if (p->fine) p = p->fine;
      // one launch over all blocks: workgroups numbered block after block and dispatched in that order
      SddmmArgs ab = a;
      ab.blocks = p->bdesc;
      ab.nblocks = p->nb;
      int64_t wgs = 0;
      for (const hgnn_plan* q : p->sub) wgs += ceil_div(q->nseg, wpb);
      if (wgs > 0) {
        launch_seg(Ls, vw, masked, dim3(unsigned(wgs)), wpb * kWave, lds, s, ab);
        HGNN_LAUNCH_CHECK("sddmm_seg_kernel");
      }
      return HGNN_OK;
    }
    if (lds <= 65536) {
      launch_seg(Ls, vw, masked, dim3(unsigned(ceil_div(p->nseg, wpb))), wpb * kWave, lds, s, a);
      HGNN_LAUNCH_CHECK("sddmm_seg_kernel");
      return HGNN_OK;
    }
  }
  const size_t lds_tile = size_t(kTile) * H * sizeof(hgnn_half) * kWavesPerBlock;
  if (vec && lds_tile <= 65536) {
    dim3 grid(unsigned(ceil_div(g->nnz, int64_t(kTile) * kWavesPerBlock)));
    if (score) launch_edge<true>(L, grid, lds_tile, s, a);
    else launch_edge<false>(L, grid, lds_tile, s, a);
    HGNN_LAUNCH_CHECK("sddmm_edge_kernel");
    return HGNN_OK;
  }
  dim3 grid(unsigned(ceil_div(g->nnz * H, kBlock)));
  if (score) sddmm_scalar_kernel<true><<<grid, kBlock, 0, s>>>(a);
  else sddmm_scalar_kernel<false><<<grid, kBlock, 0, s>>>(a);
  HGNN_LAUNCH_CHECK("sddmm_scalar_kernel");
  return HGNN_OK;
}

extern "C" hgnn_status hgnn_gat_alpha(const hgnn_csr* g, const hgnn_plan* p, int32_t H, int32_t D, const hgnn_half* U,
                                      int64_t ldu, const hgnn_half* Vt, int64_t ldv, const hgnn_half* a_l,
                                      const hgnn_half* a_r, float neg_slope, const float* lse, hgnn_half* alpha,
                                      void* stream) {
  clear_error();
  const char* who = "hgnn_gat_alpha";
  hgnn_status st = check_csr_args(g, who);
  if (st != HGNN_OK) return st;
  HGNN_REQUIRE(p != nullptr, HGNN_EINVAL, "%s: plan is NULL", who);
  HGNN_REQUIRE(p->nrows == g->nrows && p->ncols == g->ncols && p->nnz == g->nnz, HGNN_EINVAL,
               "%s: the plan was built for another graph", who);
  HGNN_REQUIRE(g->eid == nullptr, HGNN_EUNSUPPORTED, "%s: an edge-id map is not supported here", who);
  HGNN_REQUIRE(H >= 1 && D >= 1 && int64_t(H) * D <= 512, HGNN_EINVAL, "%s: H = %d, D = %d out of range", who, H, D);
  if (g->nnz == 0) return HGNN_OK;
  HGNN_REQUIRE(U && Vt && a_l && a_r && lse && alpha, HGNN_EINVAL, "%s: NULL argument", who);
  hipStream_t s = static_cast<hipStream_t>(stream);
  st = gat_project(p, g, H, D, U, ldu, Vt, ldv, a_l, a_r, s, who);
  if (st != HGNN_OK) return st;
  SddmmArgs a{};
  a.rowptr = g->rowptr;
  a.col = g->col;
  a.out = reinterpret_cast<half_t*>(alpha);
  a.nnz = g->nnz;
  a.nrows = g->nrows;
  a.ncols = g->ncols;
  a.H = H;
  a.D = D;
  a.F = H * D;
  a.slope = neg_slope;
  a.seg_lo = p->seg_row_lo;
  a.seg_hi = p->seg_row_hi;
  a.nseg = p->nseg;
  a.S = p->S;
  a.el = p->vscratch;
  a.er = p->vscratch + size_t(g->nrows) * H;
  a.lse = lse;
  if (H == 1 && p->ns > 0) return slice_edge_score(p, g, a.el, a.er, lse, neg_slope, alpha, s);
  return launch_edge_score(a, ceil_div(p->nseg, kWavesPerBlock), s);
}
