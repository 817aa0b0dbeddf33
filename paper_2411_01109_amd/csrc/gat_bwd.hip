// Backward of the single-pass GAT aggregation for gfx950, again without any per-edge tensor.
//
// With alpha rebuilt from per-vertex scalars, alpha_ij = exp(LeakyReLU(el_i + er_j) - lse_i), and
// t_i = sum_j alpha_ij * dalpha_ij = <dOut_i, out_i> known per vertex, every per-edge quantity of
// the backward pass (sections 2.1.2 and 3.1.2: SDDMM for dalpha, Eq. 1 differentiated, the
// alpha-weighted SpMM on the transpose) follows from one gathered feature row and a few scalars:
//   dalpha_ij = <dOut_i, h_j>,   ds_ij = alpha_ij * (dalpha_ij - t_i) * LeakyReLU'(el_i + er_j)
// Two passes over the graph, both on the segment design (no atomics, staged pieces, follow-up):
//   transposed pass (rows j, gathers dOut_i):  dV_j = sum_i alpha_ij * dOut_i,  d_er_j = sum_i ds_ij
//   forward pass    (rows i, gathers h_j):     d_el_i = sum_j ds_ij
// The destination vertex's scalars (el, lse, t) sit in one 16-byte entry per (vertex, head), so the
// transposed pass fetches them with a single gather from a table that stays in L2; the weight and
// the mask are formed once per edge and wave while the segment is staged.  Because the sum of ds over
// any piece of a row is linear in the gathered vectors, no dot product is formed per edge: the
// kernels accumulate the mask-weighted vector sum and one scalar, and take the dot product with the
// row-side vector once per piece.
#include "common.h"

namespace hgnn {

struct GatBwdArgs {
  const int* rowptr;
  const int* col;
  const half_t* X;     // gathered, column-side vectors [ncols of this graph][ldx]
  const half_t* R;     // row-side vectors [nrows of this graph][ldr]
  half_t* Y;           // VEC kernels: [nrows][ldy] = sum over the row of alpha * X[col]
  int64_t ldx, ldr, ldy, nnz;
  int nrows, F, H, D;
  float slope;
  const float4* vtab;  // [destination vertex][H]: (el, lse, t, unused)
  const float* er;     // [source vertex][H]
  int dst_is_col;      // 1: the destination vertex of a non-zero is its column (transposed pass), 0: its row
  half_t* dsum;        // [nrows][H] sum over the row of ds (fp16), or
  float* dsum_f32;     // column blocks: this block's partial sums in fp32
  int S;
  int64_t nseg;
  const int* seg_lo;
  const int* seg_hi;
  half_t* staging;     // [2*nseg][stage_ld]
  float* stage_ds;     // [2*nseg][H][2], first float = partial sum of ds
  int stage_ld;
  const int* split_row;
  const int* split_lo;
  const int* split_hi;
  int n_split;
  // all column blocks of a plan in one launch (workgroups numbered block after block): the table of the blocks'
  // arrays, or nullptr when the fields above describe the one graph of the launch.  Y and dsum_f32 then point at
  // block 0's partial results and advance by the strides per block.
  const hgnn_seg_block* blocks;
  int nblocks;
  int64_t y_stride, ds_stride;
};

// Finds the block of workgroup wg (cnt(B) workgroups per block), rewrites `a` to that block and returns the
// workgroup's number inside the block; wg_count receives the block's workgroup count.
template <class Count>
__device__ __forceinline__ int64_t gat_bwd_enter_block(GatBwdArgs& a, int64_t wg, int64_t& wg_count, Count cnt) {
  int b = 0;
  for (;;) {
    const int64_t c = cnt(a.blocks[b]);
    wg_count = c;
    if (wg < c || b + 1 == a.nblocks) break;
    wg -= c;
    ++b;
  }
  const hgnn_seg_block& B = a.blocks[b];
  a.rowptr = B.rowptr;
  a.col = B.col;
  a.nnz = B.nnz;
  a.seg_lo = B.seg_lo;
  a.seg_hi = B.seg_hi;
  a.nseg = B.nseg;
  a.staging = reinterpret_cast<half_t*>(B.staging);
  a.stage_ds = B.stage_mz;
  a.split_row = B.split_row;
  a.split_lo = B.split_lo;
  a.split_hi = B.split_hi;
  a.n_split = B.n_split;
  if (a.Y) a.Y += int64_t(b) * a.y_stride;
  a.dsum_f32 += int64_t(b) * a.ds_stride;
  return wg;
}

struct GatBwdLds {
  int per, spad, col_off, row_off, blk_off, a_off, t_off, vec_off, ds_off, flag_off, total;
};
// fly: no per (edge, head) tables; a copy of the raw column ids instead where s_col holds byte offsets (off32)
__host__ __device__ inline GatBwdLds gat_bwd_lds_layout(int S, int H, int L, bool vec, bool fly, bool off32) {
  GatBwdLds o;
  const int G = kWave / L;
  o.per = 4 * ((S + 255) / 256);
  o.spad = kWave * o.per;
  o.col_off = 0;
  o.row_off = o.col_off + o.spad * 4;
  o.blk_off = o.row_off + o.spad * 4;
  o.a_off = o.blk_off + ((o.spad + 15) & ~15);
  o.t_off = o.a_off + (fly ? (off32 ? o.spad * 4 : 0) : o.spad * H * 4);
  o.vec_off = o.t_off + (fly ? 0 : o.spad * H * 4);
  o.ds_off = o.vec_off + (vec ? G * 8 * L * 4 : 0);  // one parked piece per lane group: the one that entered its chunk
  o.flag_off = o.ds_off + G * L * 4;
  o.total = o.flag_off + ((3 * G * 4 + 15) & ~15);
  return o;
}

// one finished row: the vector (VEC) and the head's scalar
template <bool VEC>
__device__ __forceinline__ void bwd_row_store(const GatBwdArgs& a, int64_t row, int f0, int head, bool leader,
                                              const float (&acc)[8], float ds) {
  if (VEC) {
    half8_t h;
#pragma unroll
    for (int i = 0; i < 8; ++i) h[i] = half_t(acc[i]);
    *reinterpret_cast<half8_t*>(a.Y + row * a.ldy + f0) = h;
  }
  if (leader) {
    if (a.dsum_f32) a.dsum_f32[row * a.H + head] = ds;
    else a.dsum[row * a.H + head] = half_t(ds);
  }
}

template <bool VEC>
__device__ __forceinline__ void bwd_stage_store(const GatBwdArgs& a, int64_t slot, int f0, int head, bool leader,
                                                const float (&acc)[8], float ds) {
  if (VEC) {
    half8_t h;
#pragma unroll
    for (int i = 0; i < 8; ++i) h[i] = half_t(acc[i]);
    *reinterpret_cast<half8_t*>(a.staging + slot * a.stage_ld + f0) = h;
  }
  if (leader) a.stage_ds[(slot * a.H + head) * 2] = ds;
}

// VEC = true is the pass over the transposed graph (the destination vertex of a non-zero is its column).
// FLY = true: the weight of an edge is formed in the main loop from the destination's packed scalars and the
// source's er, one of them gathered per edge and the other fetched when the row changes; no per-edge tables in
// LDS, so more waves fit a compute unit (wins with several heads, where the tables are large, and with one head
// of up to 64 features, whose few lanes repeat little of the scalar work).  FLY = false: formed once per
// (edge, head) while the segment is staged.
template <int L, bool OFF32, bool VEC, bool FLY>
__global__ __launch_bounds__(kBlock, VEC ? 1 : 6) void gat_bwd_seg_kernel(GatBwdArgs a) {
  constexpr int G = kWave / L;
  constexpr int VECF = 8 * L;
  extern __shared__ __align__(16) unsigned char smem[];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int g = lane / L, l = lane % L;
  const int f0 = 8 * l;
  const bool active = f0 < a.F;
  const int f0c = active ? f0 : 0;
  const int head = f0c / a.D;
  const bool leader = active && (f0 % a.D) == 0;
  const int LH = a.D / 8;
  const int S = a.S;
  const GatBwdLds lay = gat_bwd_lds_layout(S, a.H, L, VEC, FLY, OFF32);
  unsigned char* base = smem + size_t(wave) * lay.total;
  int* s_col = reinterpret_cast<int*>(base + lay.col_off);
  int* s_row = reinterpret_cast<int*>(base + lay.row_off);
  int* s_blk = reinterpret_cast<int*>(base + lay.blk_off);
  float* s_a = reinterpret_cast<float*>(base + lay.a_off);    // [spad][H]: alpha, negated where the score is <= 0
  int* s_raw = OFF32 ? reinterpret_cast<int*>(base + lay.a_off) : s_col;  // FLY: [spad] column ids (s_a's place)
  float* s_t = reinterpret_cast<float*>(base + lay.t_off);    // [spad][H]: alpha * mask * t of the destination vertex
  // the piece that entered a group's chunk is parked here when its row ends; the piece that leaves the chunk stays
  // in the group's registers, from where the merge reads it (no LDS allocation: more waves per compute unit)
  float* m_vec = reinterpret_cast<float*>(base + lay.vec_off);  // [G][VECF] parked vectors (VEC)
  float* m_ds = reinterpret_cast<float*>(base + lay.ds_off);    // [G][L] parked ds sums, per lane
  int* m_flag = reinterpret_cast<int*>(base + lay.flag_off);
  int* m_hrow = m_flag + G;
  int* m_trow = m_hrow + G;

  const int wpb = int(blockDim.x) / kWave;  // 4 waves per workgroup, fewer when the heads' LDS tables are large
  int64_t wg = blockIdx.x, wg_count = gridDim.x;
  if (a.blocks)
    wg = gat_bwd_enter_block(a, wg, wg_count, [&](const hgnn_seg_block& B) {
      const int64_t c = (B.nseg + wpb - 1) / wpb;
      return c > 0 ? c : int64_t(1);
    });
  const int64_t wid = wg * wpb + wave;
  const int64_t seg = wid;
  const bool valid = seg < a.nseg;
  const int64_t e0 = seg * S;
  const int n = valid ? int(a.nnz - e0 < S ? a.nnz - e0 : S) : 0;
  const int per = lay.per, spad = lay.spad;
  int row_lo = 0, row_hi = -1;
  bool seg_left_open = false, seg_right_open = false;
  if (valid) {
    row_lo = a.seg_lo[seg];
    row_hi = a.seg_hi[seg];
    seg_left_open = int64_t(a.rowptr[row_lo]) < e0;
    seg_right_open = int64_t(a.rowptr[row_hi + 1]) > e0 + n;
  }

  // ---- phase 1: column ids, row ids, then per (edge, head) the attention weight with the LeakyReLU branch in
  // its sign, and u = alpha * mask * t of the destination vertex
  seg_stage_cols(a.col, e0, lane, spad, n, stream_nontemporal(a.nnz), [&](int i, int c) {
    if (FLY && OFF32) {
      s_raw[i] = c;
      s_col[i] = int(uint32_t(c) * uint32_t(a.ldx) * 2u);
    } else {
      s_col[i] = c;
    }
  });
  if (lane < G) m_flag[lane] = 0;
  seg_stage_rows(s_row, s_blk, lane, per, n, row_lo, row_hi, a.rowptr, e0);
  if (!FLY) {
    for (int i = lane; i < spad; i += kWave) {
      const bool in = i < n;
      const int c = s_col[i];
      const int r = in ? s_row[i] : 0;
      const int64_t dst = a.dst_is_col ? c : r, src = a.dst_is_col ? r : c;
      for (int h = 0; h < a.H; ++h) {
        float av = 0.f, uv = 0.f;
        if (in) {
          const float4 v = a.vtab[dst * a.H + h];
          const float sc = v.x + a.er[src * a.H + h];
          const float alpha = __expf((sc > 0.f ? sc : a.slope * sc) - v.y);
          av = sc > 0.f ? alpha : -alpha;
          uv = (sc > 0.f ? alpha : a.slope * alpha) * v.z;
        }
        s_a[i * a.H + h] = av;
        s_t[i * a.H + h] = uv;
      }
      if (OFF32) s_col[i] = int(uint32_t(c) * uint32_t(a.ldx) * 2u);
    }
  }
  wave_sync();

  // ---- phase 2.  The sum of ds over a piece of a row is linear in the gathered vectors:
  //   sum_k alpha_k m_k (<r, x_k> - t_k) = <r, sum_k alpha_k m_k x_k> - sum_k alpha_k m_k t_k
  // (r = the row-side vector, m = the LeakyReLU slope of the edge), so the inner loop only accumulates the
  // mask-weighted vector wacc beside acc and one scalar; the dot product with r and the exchange between
  // the lanes of a head happen once per piece, when it is flushed.
  const int C = 4 * ((S + 4 * G - 1) / (4 * G));
  const int c0 = g * C < n ? g * C : n;
  const int c1 = c0 + C < n ? c0 + C : n;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};   // sum alpha * x          (VEC)
  float wacc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};  // sum alpha * m * x
  float csum = 0.f;                                           // sum alpha * m * t
  int cur = -1;
  bool lo = false;
  float leave_ds = 0.f;     // ds sum of the piece that leaves this chunk (its vector stays in acc)
  half8_t ur = half8_t(0);  // this lane's slice of the current row's row-side vector
  float4 v_row = make_float4(0.f, 0.f, 0.f, 0.f);  // FLY, pass over the graph: the row's (el, lse, t)
  float er_row = 0.f;                              // FLY, transposed pass: the row's er
  auto load_row_vec = [&](int r) {
    ur = *reinterpret_cast<const half8_t*>(a.R + int64_t(r) * a.ldr + f0c);
    if (FLY) {
      if (VEC) er_row = a.er[int64_t(r) * a.H + head];
      else v_row = a.vtab[int64_t(r) * a.H + head];
    }
  };
  auto flush = [&](bool ro) {
    float d = 0.f;
    if (active) {
#pragma unroll
      for (int q = 0; q < 8; ++q) d = fmaf(wacc[q], float(ur[q]), d);
    }
    const float dsv = head_sum1(d, LH) - csum;
    if (!lo && !ro) {
      if (active) bwd_row_store<VEC>(a, cur, f0, head, leader, acc, dsv);
    } else if (lo) {
      if (VEC && active) {
        float* dst = m_vec + g * VECF + f0;
#pragma unroll
        for (int i = 0; i < 8; ++i) dst[i] = acc[i];
      }
      m_ds[g * L + l] = dsv;
      if (l == 0) {
        m_flag[g] |= ro ? 3 : 1;
        m_hrow[g] = cur;
      }
    } else {  // leaves into the next chunk (only the last flush of a chunk gets here)
      leave_ds = dsv;
      if (l == 0) {
        m_flag[g] |= 4;
        m_trow[g] = cur;
      }
    }
  };
  auto gather = [&](int c) -> half8_t {
    if (OFF32) {
      const uint32_t boff = uint32_t(c) + uint32_t(f0c) * 2u;
      return *reinterpret_cast<const half8_t*>(reinterpret_cast<const char*>(a.X) + boff);
    }
    return *reinterpret_cast<const half8_t*>(a.X + int64_t(c) * a.ldx + f0c);
  };
  // FLY: av = the destination's el, uv = the source's er, lse and t beside them; else the staged pair
  auto add_edge = [&](float av, float uv, float lse, float tt, const half8_t& x) {
    float alpha, am;
    if (FLY) {
      const float sc = av + uv;
      alpha = __expf((sc > 0.f ? sc : a.slope * sc) - lse);
      am = sc > 0.f ? alpha : a.slope * alpha;
      csum = fmaf(am, tt, csum);
    } else {
      alpha = fabsf(av);
      am = av > 0.f ? av : -a.slope * av;
      csum += uv;
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const float xf = float(x[q]);
      if (VEC) acc[q] = fmaf(alpha, xf, acc[q]);
      wacc[q] = fmaf(am, xf, wacc[q]);
    }
  };

  if (c0 < c1) {
    cur = s_row[c0];
    lo = c0 > 0 ? s_row[c0 - 1] == cur : seg_left_open;
    load_row_vec(cur);
  }
  for (int i = c0; i < c1; i += 4) {
    const int4_t cols = *reinterpret_cast<const int4_t*>(s_col + i);
    const int blk = s_blk[i >> 2];
    half8_t x[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) x[u] = gather(cols[u]);
    float av[4], uv[4], ls[4], tt[4];
    if (FLY) {
      const int4_t raw = OFF32 ? *reinterpret_cast<const int4_t*>(s_raw + i) : cols;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (VEC) {
          const float4 v = a.vtab[int64_t(raw[u]) * a.H + head];
          av[u] = v.x;
          ls[u] = v.y;
          tt[u] = v.z;
        } else {
          uv[u] = a.er[int64_t(raw[u]) * a.H + head];
        }
      }
    } else {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        av[u] = s_a[(i + u) * a.H + head];
        uv[u] = s_t[(i + u) * a.H + head];
        ls[u] = tt[u] = 0.f;
      }
    }
    // the row-side half of a FLY edge is read when the edge is added: the row may have changed by then
    auto add = [&](int u) {
      if (FLY && VEC) add_edge(av[u], er_row, ls[u], tt[u], x[u]);
      else if (FLY) add_edge(v_row.x, uv[u], v_row.y, v_row.z, x[u]);
      else add_edge(av[u], uv[u], 0.f, 0.f, x[u]);
    };
    if (blk == cur) {
#pragma unroll
      for (int u = 0; u < 4; ++u) add(u);
    } else {
      const int4_t rows = *reinterpret_cast<const int4_t*>(s_row + i);
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (i + u < c1) {
          if (rows[u] != cur) {
            flush(false);
#pragma unroll
            for (int q = 0; q < 8; ++q) {
              acc[q] = 0.f;
              wacc[q] = 0.f;
            }
            csum = 0.f;
            cur = rows[u];
            lo = false;
            load_row_vec(cur);
          }
          add(u);
        }
      }
    }
  }
  if (c0 < c1) flush(c1 < n ? s_row[c1] == cur : seg_right_open);
  wave_sync();

  // ---- merge: group 0 sews the pieces together in chunk order (all lanes take part in the cross-lane reads)
  if (valid) {
    float run[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    float rds = 0.f;
    bool open = false, from_before = false;
    int run_row = -1;
    const bool me = g == 0 && active;
    for (int gg = 0; gg < G; ++gg) {
      const int fl = m_flag[gg];  // the same value on every lane
      if (fl & 1) {
        if (g == 0) {
          if (VEC) {
            const float* src = m_vec + gg * VECF + f0c;
#pragma unroll
            for (int i = 0; i < 8; ++i) run[i] += src[i];
          }
          rds += m_ds[gg * L + l];
        }
        if (gg == 0) {
          from_before = true;
          open = true;
          run_row = m_hrow[0];
        }
        if (!(fl & 2)) {
          if (me) {
            if (from_before) bwd_stage_store<VEC>(a, 2 * seg, f0, head, leader, run, rds);
            else bwd_row_store<VEC>(a, run_row, f0, head, leader, run, rds);
          }
#pragma unroll
          for (int i = 0; i < 8; ++i) run[i] = 0.f;
          rds = 0.f;
          open = false;
          from_before = false;
        }
      }
      if (fl & 4) {  // the piece that left chunk gg: from the registers of group gg
        const int src = gg * L + l;
        if (VEC) {
#pragma unroll
          for (int i = 0; i < 8; ++i) run[i] = __shfl(acc[i], src);
        }
        rds = __shfl(leave_ds, src);
        run_row = m_trow[gg];
        open = true;
        from_before = false;
      }
    }
    if (open && me) bwd_stage_store<VEC>(a, 2 * seg + (from_before ? 0 : 1), f0, head, leader, run, rds);
  }

  // ---- this wave's share of the empty rows
  const int64_t nw = wg_count * wpb;
  const int rpw = int((a.nrows + nw - 1) / nw);
  const int64_t r0 = wid * rpw;
  const int64_t r1 = r0 + rpw < a.nrows ? r0 + rpw : a.nrows;
  if (active) {
    const float zero[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int64_t r = r0 + g; r < r1; r += G)
      if (a.rowptr[r] == a.rowptr[r + 1]) bwd_row_store<VEC>(a, r, f0, head, leader, zero, 0.f);
  }
}

// Follow-up kernel: sums the staged pieces of every row that crosses a segment border, in segment order.
template <int L, bool VEC>
__global__ __launch_bounds__(kBlock) void gat_bwd_finish_kernel(GatBwdArgs a) {
  constexpr int G = kWave / L;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int g = lane / L, l = lane % L;
  const int f0 = 8 * l;
  const bool active = f0 < a.F;
  const int f0c = active ? f0 : 0;
  const int head = f0c / a.D;
  const bool leader = active && (f0 % a.D) == 0;
  int64_t wg = blockIdx.x, wg_count = gridDim.x;
  if (a.blocks)
    wg = gat_bwd_enter_block(a, wg, wg_count, [&](const hgnn_seg_block& B) {
      return (int64_t(B.n_split) + kWavesPerBlock * G - 1) / (kWavesPerBlock * G);
    });
  const int64_t i0 = (wg * kWavesPerBlock + wave) * G;
  if (i0 >= a.n_split) return;
  const int64_t idx = i0 + g;
  int r = 0, sa = 0, sb = -1;
  if (idx < a.n_split) {
    r = a.split_row[idx];
    sa = a.split_lo[idx];
    sb = a.split_hi[idx];
  }
  auto take = [&](float (&acc)[8], float& ds, int64_t slot) {
    if (VEC) {
      const half8_t o = *reinterpret_cast<const half8_t*>(a.staging + slot * a.stage_ld + f0c);
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] += float(o[i]);
    }
    ds += a.stage_ds[(slot * a.H + head) * 2];
  };
  if (idx < a.n_split && sb - sa <= 8) {
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    float ds = 0.f;
    take(acc, ds, 2 * int64_t(sa) + 1);
    for (int64_t k = int64_t(sa) + 1; k <= sb; ++k) take(acc, ds, 2 * k);
    if (active) bwd_row_store<VEC>(a, r, f0, head, leader, acc, ds);
  }
  for (int j = 0; j < G; ++j) {
    const int rj = __shfl(r, j * L), sj = __shfl(sa, j * L), ej = __shfl(sb, j * L);
    if (ej - sj <= 8) continue;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    float ds = 0.f;
    if (g == 0) take(acc, ds, 2 * int64_t(sj) + 1);
    for (int64_t k = int64_t(sj) + 1 + g; k <= ej; k += G) take(acc, ds, 2 * k);
#pragma unroll
    for (int off = L; off < kWave; off <<= 1) {
      if (VEC) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] += __shfl_xor(acc[i], off);
      }
      ds += __shfl_xor(ds, off);
    }
    if (g == 0 && active) bwd_row_store<VEC>(a, rj, f0, head, leader, acc, ds);
  }
}

// Column-blocked plans: adds the nb partial rows (fp16 vectors, fp32 ds sums) of every row.
template <int L, bool VEC>
__global__ __launch_bounds__(kBlock) void gat_bwd_block_sum_kernel(GatBwdArgs a, const half_t* __restrict__ part,
                                                                   int part_ld, const float* __restrict__ part_ds,
                                                                   int64_t ds_stride, int nb) {
  constexpr int G = kWave / L;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int g = lane / L, l = lane % L;
  const int f0 = 8 * l;
  const int64_t r = (int64_t(blockIdx.x) * kWavesPerBlock + wave) * G + g;
  if (r >= a.nrows || f0 >= a.F) return;
  const int head = f0 / a.D;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  float ds = 0.f;
  for (int b = 0; b < nb; ++b) {
    if (VEC) {
      const half8_t o = *reinterpret_cast<const half8_t*>(part + (int64_t(b) * a.nrows + r) * part_ld + f0);
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] += float(o[i]);
    }
    ds += part_ds[b * ds_stride + r * a.H + head];
  }
  bwd_row_store<VEC>(a, r, f0, head, (f0 % a.D) == 0, acc, ds);
}

// vtab[i,h] = (el[i,h], lse[i,h], t[i,h] = <dOut[i,h], out[i,h]>, 0) for every destination vertex.  With the masked
// result and weight sum that the saving forward pass left (outm, csum), the gradient of the row-side score term is
// a per-vertex expression and is written here: d_el[i,h] = <dOut[i,h], outm[i,h]> - t[i,h] * csum[i,h].
template <int L>
__global__ __launch_bounds__(kBlock) void gat_vtab_kernel(const float* __restrict__ el, const float* __restrict__ lse,
                                                           const half_t* __restrict__ dOut, int64_t lddo,
                                                           const half_t* __restrict__ out, int64_t ldo, int nv, int F, int D,
                                                           int H, float4* __restrict__ vtab, const half_t* __restrict__ outm,
                                                           int64_t ldom, const float* __restrict__ csum,
                                                           half_t* __restrict__ d_el) {
  constexpr int G = kWave / L;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int g = lane / L, l = lane % L;
  const int f0 = 8 * l;
  const bool active = f0 < F;
  const int LH = D / 8;
  const int64_t v = (int64_t(blockIdx.x) * kWavesPerBlock + wave) * G + g;
  float p = 0.f, pm = 0.f;
  if (active && v < nv) {
    const half8_t x = *reinterpret_cast<const half8_t*>(dOut + v * lddo + f0);
    const half8_t y = *reinterpret_cast<const half8_t*>(out + v * ldo + f0);
#pragma unroll
    for (int i = 0; i < 8; ++i) p = fmaf(float(x[i]), float(y[i]), p);
    if (outm) {
      const half8_t ym = *reinterpret_cast<const half8_t*>(outm + v * ldom + f0);
#pragma unroll
      for (int i = 0; i < 8; ++i) pm = fmaf(float(x[i]), float(ym[i]), pm);
    }
  }
  for (int off = 1; off < LH; off <<= 1) {
    p += __shfl_xor(p, off);
    pm += __shfl_xor(pm, off);
  }
  if (active && v < nv && (l % LH) == 0) {
    const int64_t k = v * H + l / LH;
    vtab[k] = make_float4(el[k], lse[k], p, 0.f);
    if (outm) d_el[k] = half_t(pm - p * csum[k]);
  }
}

template <bool OFF32, bool VEC, bool FLY>
static void launch_bwd_seg(int L, dim3 grid, int threads, size_t lds, hipStream_t s, const GatBwdArgs& a) {
  switch (L) {
    case 1: gat_bwd_seg_kernel<1, OFF32, VEC, FLY><<<grid, threads, lds, s>>>(a); break;
    case 2: gat_bwd_seg_kernel<2, OFF32, VEC, FLY><<<grid, threads, lds, s>>>(a); break;
    case 4: gat_bwd_seg_kernel<4, OFF32, VEC, FLY><<<grid, threads, lds, s>>>(a); break;
    case 8: gat_bwd_seg_kernel<8, OFF32, VEC, FLY><<<grid, threads, lds, s>>>(a); break;
    case 16: gat_bwd_seg_kernel<16, OFF32, VEC, FLY><<<grid, threads, lds, s>>>(a); break;
    case 32: gat_bwd_seg_kernel<32, OFF32, VEC, FLY><<<grid, threads, lds, s>>>(a); break;
    default: gat_bwd_seg_kernel<64, OFF32, VEC, FLY><<<grid, threads, lds, s>>>(a); break;
  }
}

template <bool VEC>
static void launch_bwd_finish(int L, dim3 grid, hipStream_t s, const GatBwdArgs& a) {
  switch (L) {
    case 1: gat_bwd_finish_kernel<1, VEC><<<grid, kBlock, 0, s>>>(a); break;
    case 2: gat_bwd_finish_kernel<2, VEC><<<grid, kBlock, 0, s>>>(a); break;
    case 4: gat_bwd_finish_kernel<4, VEC><<<grid, kBlock, 0, s>>>(a); break;
    case 8: gat_bwd_finish_kernel<8, VEC><<<grid, kBlock, 0, s>>>(a); break;
    case 16: gat_bwd_finish_kernel<16, VEC><<<grid, kBlock, 0, s>>>(a); break;
    case 32: gat_bwd_finish_kernel<32, VEC><<<grid, kBlock, 0, s>>>(a); break;
    default: gat_bwd_finish_kernel<64, VEC><<<grid, kBlock, 0, s>>>(a); break;
  }
}

template <bool VEC>
static void launch_bwd_block_sum(int L, dim3 grid, hipStream_t s, const GatBwdArgs& a, const half_t* part, int part_ld,
                                 const float* part_ds, int64_t ds_stride, int nb) {
  switch (L) {
    case 1: gat_bwd_block_sum_kernel<1, VEC><<<grid, kBlock, 0, s>>>(a, part, part_ld, part_ds, ds_stride, nb); break;
    case 2: gat_bwd_block_sum_kernel<2, VEC><<<grid, kBlock, 0, s>>>(a, part, part_ld, part_ds, ds_stride, nb); break;
    case 4: gat_bwd_block_sum_kernel<4, VEC><<<grid, kBlock, 0, s>>>(a, part, part_ld, part_ds, ds_stride, nb); break;
    case 8: gat_bwd_block_sum_kernel<8, VEC><<<grid, kBlock, 0, s>>>(a, part, part_ld, part_ds, ds_stride, nb); break;
    case 16: gat_bwd_block_sum_kernel<16, VEC><<<grid, kBlock, 0, s>>>(a, part, part_ld, part_ds, ds_stride, nb); break;
    case 32: gat_bwd_block_sum_kernel<32, VEC><<<grid, kBlock, 0, s>>>(a, part, part_ld, part_ds, ds_stride, nb); break;
    default: gat_bwd_block_sum_kernel<64, VEC><<<grid, kBlock, 0, s>>>(a, part, part_ld, part_ds, ds_stride, nb); break;
  }
}

struct VtabSaved {
  const half_t* outm;
  int64_t ldom;
  const float* csum;
  half_t* d_el;
};

static void launch_vtab(int L, dim3 grid, hipStream_t s, const float* el, const float* lse, const half_t* dOut, int64_t lddo,
                        const half_t* out, int64_t ldo, int nv, int F, int D, int H, float4* vtab, const VtabSaved& q) {
#define HGNN_VTAB(LL) \
  gat_vtab_kernel<LL><<<grid, kBlock, 0, s>>>(el, lse, dOut, lddo, out, ldo, nv, F, D, H, vtab, q.outm, q.ldom, q.csum, q.d_el)
  switch (L) {
    case 1: HGNN_VTAB(1); break;
    case 2: HGNN_VTAB(2); break;
    case 4: HGNN_VTAB(4); break;
    case 8: HGNN_VTAB(8); break;
    case 16: HGNN_VTAB(16); break;
    case 32: HGNN_VTAB(32); break;
    default: HGNN_VTAB(64); break;
  }
#undef HGNN_VTAB
}

// one pass (segment kernel + follow-up) over the graph in `a` with the segment arrays of plan q
template <bool VEC>
static hgnn_status run_bwd_segments(const hgnn_plan* q, GatBwdArgs a, int ncols, hipStream_t s) {
  a.seg_lo = q->seg_row_lo;
  a.seg_hi = q->seg_row_hi;
  a.S = q->S;
  a.nseg = q->nseg;
  a.staging = reinterpret_cast<half_t*>(q->staging);
  a.stage_ds = q->stage_mz;
  a.stage_ld = q->max_F;
  a.split_row = q->split_row;
  a.split_lo = q->split_seg_lo;
  a.split_hi = q->split_seg_hi;
  a.n_split = q->n_split;
  const int L = pow2_at_least(a.F / 8);
  const bool off32 = uint64_t(ncols) * uint64_t(a.ldx) * 2u < (uint64_t(1) << 32);
  // weights formed in the main loop: measured 0.26 -> 0.17 ms for the transposed pass with 4 heads of 16 (12 -> 20
  // waves per compute unit); with one head 3-15 % faster up to 64 features, 1-3 % slower from 128 on (every lane of
  // the head repeats the scalar work)
  const bool fly = a.H >= 2 || a.D <= 64;
  const size_t per_wave = size_t(gat_bwd_lds_layout(a.S, a.H, L, VEC, fly, off32).total);
  const int wpb = waves_per_block_for_lds(per_wave, true);
  const size_t lds = per_wave * wpb;
  HGNN_REQUIRE(lds <= 65536, HGNN_EUNSUPPORTED,
               "hgnn_gat_backward_fused: seg_edges = %d with H = %d needs %zu bytes of LDS per wavefront (limit 65536)", a.S,
               a.H, lds);
  const int64_t nblk = ceil_div(q->nseg, wpb);
  dim3 grid(unsigned(nblk > 0 ? nblk : 1));
  if (fly) {
    if (off32) launch_bwd_seg<true, VEC, true>(L, grid, wpb * kWave, lds, s, a);
    else launch_bwd_seg<false, VEC, true>(L, grid, wpb * kWave, lds, s, a);
  } else {
    if (off32) launch_bwd_seg<true, VEC, false>(L, grid, wpb * kWave, lds, s, a);
    else launch_bwd_seg<false, VEC, false>(L, grid, wpb * kWave, lds, s, a);
  }
  HGNN_LAUNCH_CHECK("gat_bwd_seg_kernel");
  if (a.n_split > 0) {
    launch_bwd_finish<VEC>(L, dim3(unsigned(ceil_div(a.n_split, int64_t(kWavesPerBlock) * (kWave / L)))), s, a);
    HGNN_LAUNCH_CHECK("gat_bwd_finish_kernel");
  }
  return HGNN_OK;
}

// a pass over graph gg with plan q (column-blocked or not)
template <bool VEC>
static hgnn_status run_bwd_pass(const hgnn_plan* q, const hgnn_csr* gg, GatBwdArgs a, hipStream_t s) {
  if (q->nb <= 1) return run_bwd_segments<VEC>(q, a, gg->ncols, s);
  const size_t V = size_t(q->nrows);
  const int64_t ds_stride = int64_t(V) * q->max_H * 2;
  const int L = pow2_at_least(a.F / 8);
  {
    // all blocks in one launch of each kernel: workgroups numbered block after block and dispatched in that order
    GatBwdArgs ab = a;
    ab.Y = reinterpret_cast<half_t*>(q->bstage);
    ab.ldy = q->max_F;
    ab.dsum = nullptr;
    ab.dsum_f32 = q->bsum;
    ab.blocks = q->bdesc;
    ab.nblocks = q->nb;
    ab.y_stride = int64_t(V) * q->max_F;
    ab.ds_stride = ds_stride;
    ab.S = q->S;
    ab.stage_ld = q->max_F;
    const bool off32 = uint64_t(gg->ncols) * uint64_t(ab.ldx) * 2u < (uint64_t(1) << 32);
    const bool fly = ab.H >= 2 || ab.D <= 64;  // as in run_bwd_segments
    const size_t per_wave = size_t(gat_bwd_lds_layout(ab.S, ab.H, L, VEC, fly, off32).total);
    const int wpb = waves_per_block_for_lds(per_wave, true);
    const size_t lds = per_wave * wpb;
    HGNN_REQUIRE(lds <= 65536, HGNN_EUNSUPPORTED,
                 "hgnn_gat_backward_fused: seg_edges = %d with H = %d needs %zu bytes of LDS per wavefront (limit 65536)", ab.S,
                 ab.H, lds);
    int64_t wgs = 0, wgs2 = 0;
    for (const hgnn_plan* sub : q->sub) {
      const int64_t c = ceil_div(sub->nseg, wpb);
      wgs += c > 0 ? c : 1;
      wgs2 += ceil_div(sub->n_split, int64_t(kWavesPerBlock) * (kWave / L));
    }
    const dim3 grid{unsigned(wgs)};
    if (fly) {
      if (off32) launch_bwd_seg<true, VEC, true>(L, grid, wpb * kWave, lds, s, ab);
      else launch_bwd_seg<false, VEC, true>(L, grid, wpb * kWave, lds, s, ab);
    } else {
      if (off32) launch_bwd_seg<true, VEC, false>(L, grid, wpb * kWave, lds, s, ab);
      else launch_bwd_seg<false, VEC, false>(L, grid, wpb * kWave, lds, s, ab);
    }
    HGNN_LAUNCH_CHECK("gat_bwd_seg_kernel");
    if (wgs2 > 0) {
      launch_bwd_finish<VEC>(L, dim3(unsigned(wgs2)), s, ab);
      HGNN_LAUNCH_CHECK("gat_bwd_finish_kernel");
    }
  }
  launch_bwd_block_sum<VEC>(L, dim3(unsigned(ceil_div(gg->nrows, int64_t(kWavesPerBlock) * (kWave / L)))), s, a,
                            reinterpret_cast<const half_t*>(q->bstage), q->max_F, q->bsum, ds_stride, q->nb);
  HGNN_LAUNCH_CHECK("gat_bwd_block_sum_kernel");
  return HGNN_OK;
}

}  // namespace hgnn

using namespace hgnn;

// out_masked / csum: what hgnn_gat_forward_fused_save left (then d_el is a per-vertex expression and the pass over g
// is not needed), or nullptr
static hgnn_status gat_backward_impl(const char* who, const hgnn_csr* g, const hgnn_plan* p, const hgnn_csr* gt,
                                     const hgnn_plan* pt, int32_t H, int32_t D, const hgnn_half* U, int64_t ldu,
                                     const hgnn_half* Vt, int64_t ldv, const hgnn_half* a_l, const hgnn_half* a_r,
                                     float neg_slope, const hgnn_half* out, int64_t ldo, const float* lse,
                                     const hgnn_half* out_masked, int64_t ldom, const float* csum, const hgnn_half* dOut,
                                     int64_t lddo, hgnn_half* dV, int64_t lddv, hgnn_half* d_el, hgnn_half* d_er,
                                     void* stream) {
  clear_error();
  hgnn_status st = check_csr_args(g, who);
  if (st != HGNN_OK) return st;
  st = check_csr_args(gt, who);
  if (st != HGNN_OK) return st;
  HGNN_REQUIRE(p != nullptr && pt != nullptr, HGNN_EINVAL, "%s: plan is NULL", who);
  HGNN_REQUIRE(p->nrows == g->nrows && p->ncols == g->ncols && p->nnz == g->nnz, HGNN_EINVAL,
               "%s: plan p was built for another graph than g", who);
  HGNN_REQUIRE(pt->nrows == gt->nrows && pt->ncols == gt->ncols && pt->nnz == gt->nnz, HGNN_EINVAL,
               "%s: plan pt was built for another graph than gt", who);
  HGNN_REQUIRE(gt->nrows == g->ncols && gt->ncols == g->nrows && gt->nnz == g->nnz, HGNN_EINVAL,
               "%s: gt is not the transpose of g", who);
  HGNN_REQUIRE(g->eid == nullptr, HGNN_EUNSUPPORTED, "%s: g must not carry an edge-id map", who);
  HGNN_REQUIRE(H >= 1 && D >= 1 && int64_t(H) * D <= 512, HGNN_EINVAL, "%s: H = %d, D = %d out of range", who, H, D);
  const int F = H * D;
  HGNN_REQUIRE(H <= p->max_H && F <= p->max_F && H <= pt->max_H && F <= pt->max_F, HGNN_EINVAL,
               "%s: H = %d / F = %d exceed a plan's max_H / max_F", who, H, F);
  HGNN_REQUIRE(ldu >= F && ldv >= F && ldo >= F && lddo >= F && lddv >= F, HGNN_EINVAL,
               "%s: leading dimension smaller than F", who);
  if (g->nrows == 0 && g->ncols == 0) return HGNN_OK;
  HGNN_REQUIRE(U && Vt && a_l && a_r && out && lse && dOut && dV && d_el && d_er, HGNN_EINVAL, "%s: NULL argument", who);
  HGNN_REQUIRE(ldo % 8 == 0 && lddo % 8 == 0 && lddv % 8 == 0 && aligned16(out) && aligned16(dOut) && aligned16(dV),
               HGNN_EUNSUPPORTED, "%s: needs ld %% 8 == 0 and 16-byte aligned out, dOut, dV", who);
  const bool saved = out_masked != nullptr;
  HGNN_REQUIRE(!saved || (csum != nullptr && ldom >= F), HGNN_EINVAL, "%s: out_masked needs csum and ldom >= F", who);
  HGNN_REQUIRE(!saved || (ldom % 8 == 0 && aligned16(out_masked)), HGNN_EUNSUPPORTED,
               "%s: needs ldom %% 8 == 0 and a 16-byte aligned out_masked", who);
  hipStream_t s = static_cast<hipStream_t>(stream);
  // per-vertex scalars in plan p's scratch: el, er, then (el, lse, t) packed per destination vertex
  st = gat_project(p, g, H, D, U, ldu, Vt, ldv, a_l, a_r, s, who);
  if (st != HGNN_OK) return st;
  const int L = pow2_at_least(F / 8), G = kWave / L;
  const float* el = p->vscratch;
  const float* er = p->vscratch + size_t(g->nrows) * H;
  float4* vtab = reinterpret_cast<float4*>(p->vtab);
  if (g->nrows > 0) {
    launch_vtab(L, dim3(unsigned(ceil_div(g->nrows, int64_t(kWavesPerBlock) * G))), s, el, lse,
                reinterpret_cast<const half_t*>(dOut), lddo, reinterpret_cast<const half_t*>(out), ldo, g->nrows, F, D, H,
                vtab, VtabSaved{reinterpret_cast<const half_t*>(out_masked), ldom, csum, reinterpret_cast<half_t*>(d_el)});
    HGNN_LAUNCH_CHECK("gat_vtab_kernel");
  }
  GatBwdArgs a{};
  a.F = F;
  a.H = H;
  a.D = D;
  a.slope = neg_slope;
  a.vtab = vtab;
  a.er = er;
  // transposed pass: rows j (sources), gathers dOut_i; dV_j and d_er_j
  if (gt->nrows > 0) {
    GatBwdArgs t = a;
    t.rowptr = gt->rowptr;
    t.col = gt->col;
    t.nnz = gt->nnz;
    t.nrows = gt->nrows;
    t.X = reinterpret_cast<const half_t*>(dOut);
    t.ldx = lddo;
    t.R = reinterpret_cast<const half_t*>(Vt);
    t.ldr = ldv;
    t.Y = reinterpret_cast<half_t*>(dV);
    t.ldy = lddv;
    t.dsum = reinterpret_cast<half_t*>(d_er);
    t.dst_is_col = 1;
    st = run_bwd_pass<true>(pt, gt, t, s);
    if (st != HGNN_OK) return st;
  }
  // forward pass: rows i (destinations), gathers h_j; d_el_i only (already written above from the saved tensors)
  if (g->nrows > 0 && !saved) {
    GatBwdArgs f = a;
    f.rowptr = g->rowptr;
    f.col = g->col;
    f.nnz = g->nnz;
    f.nrows = g->nrows;
    f.X = reinterpret_cast<const half_t*>(Vt);
    f.ldx = ldv;
    f.R = reinterpret_cast<const half_t*>(dOut);
    f.ldr = lddo;
    f.dsum = reinterpret_cast<half_t*>(d_el);
    f.dst_is_col = 0;
    st = run_bwd_pass<false>(p, g, f, s);
    if (st != HGNN_OK) return st;
  }
  return HGNN_OK;
}

extern "C" hgnn_status hgnn_gat_backward_fused(const hgnn_csr* g, const hgnn_plan* p, const hgnn_csr* gt,
                                               const hgnn_plan* pt, int32_t H, int32_t D, const hgnn_half* U, int64_t ldu,
                                               const hgnn_half* Vt, int64_t ldv, const hgnn_half* a_l, const hgnn_half* a_r,
                                               float neg_slope, const hgnn_half* out, int64_t ldo, const float* lse,
                                               const hgnn_half* dOut, int64_t lddo, hgnn_half* dV, int64_t lddv,
                                               hgnn_half* d_el, hgnn_half* d_er, void* stream) {
  return gat_backward_impl("hgnn_gat_backward_fused", g, p, gt, pt, H, D, U, ldu, Vt, ldv, a_l, a_r, neg_slope, out, ldo, lse,
                           nullptr, 0, nullptr, dOut, lddo, dV, lddv, d_el, d_er, stream);
}

extern "C" hgnn_status hgnn_gat_backward_fused_saved(const hgnn_csr* g, const hgnn_plan* p, const hgnn_csr* gt,
                                                     const hgnn_plan* pt, int32_t H, int32_t D, const hgnn_half* U,
                                                     int64_t ldu, const hgnn_half* Vt, int64_t ldv, const hgnn_half* a_l,
                                                     const hgnn_half* a_r, float neg_slope, const hgnn_half* out, int64_t ldo,
                                                     const float* lse, const hgnn_half* out_masked, int64_t ldom,
                                                     const float* csum, const hgnn_half* dOut, int64_t lddo, hgnn_half* dV,
                                                     int64_t lddv, hgnn_half* d_el, hgnn_half* d_er, void* stream) {
  const char* who = "hgnn_gat_backward_fused_saved";
  if (out_masked == nullptr || csum == nullptr) {
    clear_error();
    return fail(HGNN_EINVAL, "%s: out_masked and csum are required", who);
  }
  return gat_backward_impl(who, g, p, gt, pt, H, D, U, ldu, Vt, ldv, a_l, a_r, neg_slope, out, ldo, lse, out_masked, ldom, csum,
                           dOut, lddo, dV, lddv, d_el, d_er, stream);
}
