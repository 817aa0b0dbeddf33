// Single-pass GAT aggregation for gfx950: score, edge softmax and weighted sum of the neighbours'
// features in one read of the graph, with no per-edge tensor written (the paper, sections 3.1.2 and
// 5.2, keeps them as three kernels with an |E| x H score tensor and an |E| x H alpha tensor between
// them; this fuses them on top of the same discretized, atomic-free segment design).
//
//   s_k = el[i,h] + er[col k,h],  e_k = LeakyReLU(s_k),  alpha_k = softmax over row i (Eq. 1),
//   out[i, h*D+d] = sum_k alpha_k * X[col k, h*D+d],    lse[i,h] = log sum_k exp(e_k)
//
// el[i,h] = a_l.U[i,h] is a per-vertex projection (fp32, formed once per vertex); er[j,h] = a_r.X[j,h] is formed
// per edge from the gathered row X[j] itself.
// A partial result over any subset of a row's edges is kept as a triple (m, z, acc): m = largest
// score met, z = sum exp(e - m), acc = sum exp(e - m) * x.  Two triples of the same row merge by
// rescaling both to the larger m (the online form of Eq. 1's shift by the row maximum), so the
// segment kernel can cut rows anywhere: lane groups carry a running triple along their chunk,
// pieces that touch a chunk border meet in LDS, pieces that cross a segment border are staged as
// (m, z) in fp32 plus the normalised vector acc/z in fp16 -- a convex combination of feature rows,
// hence never larger than the features themselves (the discretized-scaling idea of section 5.2.2
// applied to the softmax weights) -- and a follow-up kernel merges them.  No atomics, one writer per
// output row, fixed merge order.
//
// SAVE kernels also keep, per row and head, what the backward pass needs to form the gradient of the row-side
// score term without another pass over the edges: with mu_k = 1 where s_k > 0 and the LeakyReLU slope elsewhere,
//   out_masked[i, h*D+d] = sum_k alpha_k * mu_k * X[col k, h*D+d],   csum[i,h] = sum_k alpha_k * mu_k
// (then sum_k ds_k = <dOut_i, out_masked_i> - <dOut_i, out_i> * csum_i).  They ride on the same gathered rows:
// a second accumulator and a second sum in every triple, rescaled with the first.
#include "common.h"

namespace hgnn {

struct GatArgs {
  const int* rowptr;
  const int* col;
  const half_t* X;  // column-side features [ncols][ldx]
  half_t* Y;        // [nrows][ldy]: the result, or (part_mz set) this block's normalised partial rows
  int64_t ldx, ldy, nnz;
  int nrows, F, H, D;
  float slope;
  const float* el;  // [nrows][H]
  const half_t* a_r;  // [H*D]
  float* lse;       // [nrows][H] or nullptr
  float* part_mz;   // column blocks: [nrows][H][2] (m, z) of this block's partial rows; else nullptr
  half_t* Ym;       // SAVE: [nrows][ldym] masked result (or this block's normalised partial rows)
  int64_t ldym;
  float* csum;      // SAVE: [nrows][H] masked weight sum (or, with part_mz, this block's share, relative to its z)
  half_t* staging_m;  // SAVE: [2*nseg][stage_ld] masked counterpart of staging
  float* stage_c;     // SAVE: [2*nseg][H] masked weight sum of a staged piece, relative to its z
  int S;
  int64_t nseg;
  const int* seg_lo;
  const int* seg_hi;
  half_t* staging;  // [2*nseg][stage_ld] normalised vectors of the pieces that cross a segment border
  float* stage_mz;  // [2*nseg][H][2]
  int stage_ld;
  const int* split_row;
  const int* split_lo;
  const int* split_hi;
  int n_split;
  // all column blocks of a plan in one launch (workgroups numbered block after block): the table of the blocks'
  // arrays, or nullptr when the fields above describe the one graph of the launch.  Y, part_mz, Ym and csum then
  // point at block 0's partial results and advance by the strides per block.
  const hgnn_seg_block* blocks;
  int nblocks, max_F, max_H;
  int64_t y_stride, mz_stride, c_stride;
};

// Finds the block of workgroup wg (cnt(B) workgroups per block), rewrites `a` to that block and returns the
// workgroup's number inside the block; wg_count receives the block's workgroup count.
template <class Count>
__device__ __forceinline__ int64_t gat_enter_block(GatArgs& a, int64_t wg, int64_t& wg_count, Count cnt) {
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
  a.stage_mz = B.stage_mz;
  a.staging_m = a.staging + size_t(2) * size_t(B.nseg) * size_t(a.max_F);
  a.stage_c = B.stage_mz + size_t(4) * size_t(B.nseg) * size_t(a.max_H);
  a.split_row = B.split_row;
  a.split_lo = B.split_lo;
  a.split_hi = B.split_hi;
  a.n_split = B.n_split;
  a.Y += int64_t(b) * a.y_stride;
  a.part_mz += int64_t(b) * a.mz_stride;
  if (a.Ym) {
    a.Ym += int64_t(b) * a.y_stride;
    a.csum += int64_t(b) * a.c_stride;
  }
  return wg;
}

// A partial result of one row and head over some of its edges, as held by one lane (8 features):
// m = largest score met, z = sum exp(e - m), acc = sum exp(e - m) * x; SAVE adds zm = sum exp(e - m) * mu and
// accm = sum exp(e - m) * mu * x.
template <bool SAVE>
struct Soft {
  float m = -INFINITY, z = 0.f, zm = 0.f;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  float accm[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  __device__ __forceinline__ void clear() {
    m = -INFINITY;
    z = 0.f;
    zm = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      acc[i] = 0.f;
      accm[i] = 0.f;
    }
  }
  __device__ __forceinline__ void scale(float f) {
    z *= f;
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] *= f;
    if (SAVE) {
      zm *= f;
#pragma unroll
      for (int i = 0; i < 8; ++i) accm[i] *= f;
    }
  }
  // one more edge with weight p = exp(e - m) (relative to the current m) and features x
  __device__ __forceinline__ void add(float p, float e, float slope, const half8_t& x) {
    z += p;
#pragma unroll
    for (int q = 0; q < 8; ++q) acc[q] = fmaf(p, float(x[q]), acc[q]);
    if (SAVE) {
      const float pm = e > 0.f ? p : p * slope;
      zm += pm;
#pragma unroll
      for (int q = 0; q < 8; ++q) accm[q] = fmaf(pm, float(x[q]), accm[q]);
    }
  }
};

// a <- a merged with b (both rescaled to the larger maximum)
template <bool SAVE>
__device__ __forceinline__ void soft_merge(Soft<SAVE>& a, const Soft<SAVE>& b) {
  const float M = fmaxf(a.m, b.m);
  if (M == -INFINITY) return;  // both empty
  const float fa = __expf(a.m - M), fb = __expf(b.m - M);  // exp(-inf) = 0 drops an empty side
  a.z = a.z * fa + b.z * fb;
#pragma unroll
  for (int i = 0; i < 8; ++i) a.acc[i] = a.acc[i] * fa + b.acc[i] * fb;
  if (SAVE) {
    a.zm = a.zm * fa + b.zm * fb;
#pragma unroll
    for (int i = 0; i < 8; ++i) a.accm[i] = a.accm[i] * fa + b.accm[i] * fb;
  }
  a.m = M;
}

// merge a staged piece: (mp, zp), its normalised vector o = acc/z and, SAVE, cp = zm/z and om = accm/z
template <bool SAVE>
__device__ __forceinline__ void soft_merge_normalised(Soft<SAVE>& a, float mp, float zp, float cp, const half8_t& o,
                                                      const half8_t& om) {
  const float M = fmaxf(a.m, mp);
  if (M == -INFINITY) return;
  const float fa = __expf(a.m - M), fb = __expf(mp - M) * zp;
  a.z = a.z * fa + fb;
#pragma unroll
  for (int i = 0; i < 8; ++i) a.acc[i] = a.acc[i] * fa + fb * float(o[i]);
  if (SAVE) {
    a.zm = a.zm * fa + fb * cp;
#pragma unroll
    for (int i = 0; i < 8; ++i) a.accm[i] = a.accm[i] * fa + fb * float(om[i]);
  }
  a.m = M;
}

__device__ __forceinline__ void store_vec8(half_t* p, int f0, const float (&v)[8], float s) {
  half8_t h;
#pragma unroll
  for (int i = 0; i < 8; ++i) h[i] = half_t(v[i] * s);
  *reinterpret_cast<half8_t*>(p + f0) = h;
}

// a finished row (or, with part_mz, a finished partial row of a column block)
template <bool SAVE>
__device__ __forceinline__ void row_store(const GatArgs& a, int64_t row, int f0, int head, bool leader, const Soft<SAVE>& t) {
  const float inv = t.z > 0.f ? 1.f / t.z : 0.f;
  store_vec8(a.Y + row * a.ldy, f0, t.acc, inv);
  if (SAVE) store_vec8(a.Ym + row * a.ldym, f0, t.accm, inv);
  if (!leader) return;
  if (SAVE) a.csum[row * a.H + head] = t.zm * inv;
  if (a.part_mz) {
    a.part_mz[(row * a.H + head) * 2] = t.m;
    a.part_mz[(row * a.H + head) * 2 + 1] = t.z;
  } else if (a.lse) {
    a.lse[row * a.H + head] = t.z > 0.f ? t.m + __logf(t.z) : 0.f;
  }
}

template <bool SAVE>
__device__ __forceinline__ void stage_store(const GatArgs& a, int64_t slot, int f0, int head, bool leader, const Soft<SAVE>& t) {
  const float inv = t.z > 0.f ? 1.f / t.z : 0.f;
  store_vec8(a.staging + slot * a.stage_ld, f0, t.acc, inv);
  if (SAVE) store_vec8(a.staging_m + slot * a.stage_ld, f0, t.accm, inv);
  if (leader) {
    a.stage_mz[(slot * a.H + head) * 2] = t.m;
    a.stage_mz[(slot * a.H + head) * 2 + 1] = t.z;
    if (SAVE) a.stage_c[slot * a.H + head] = t.zm * inv;
  }
}

struct GatLds {
  int per, spad, col_off, row_off, blk_off, vec_off, mz_off, flag_off, total;
};
__host__ __device__ inline GatLds gat_lds_layout(int S, int L, bool save) {
  GatLds o;
  const int G = kWave / L;
  const int nv = save ? 2 : 1, ns = save ? 3 : 2;  // vectors and scalars of a parked piece
  o.per = 4 * ((S + 255) / 256);
  o.spad = kWave * o.per;
  o.col_off = 0;
  o.row_off = o.col_off + o.spad * 4;
  o.blk_off = o.row_off + o.spad * 4;
  o.vec_off = o.blk_off + ((o.spad + 15) & ~15);
  o.mz_off = o.vec_off + G * nv * 8 * L * 4;  // one parked piece per lane group: the one that entered its chunk
  o.flag_off = o.mz_off + G * L * ns * 4;
  o.total = o.flag_off + ((3 * G * 4 + 15) & ~15);
  return o;
}

// The score of an edge is formed in the main loop, with no per-edge table and no per-edge scalar fetched: the
// column-side term a_r.X[col] from the gathered row itself (four two-way dot products per lane and an exchange
// among the lanes of a head), the row-side term el[row] from a register that is refilled when the row changes.
// Staging finished scores per (edge, head) in LDS instead (one 4-byte gather of er[col] per edge and head) was
// slower for every head width from 8 to 512: the table costs waves per compute unit, the gather a cache request.
template <int L, bool OFF32, bool SAVE>
__global__ __launch_bounds__(kBlock) void gat_seg_kernel(GatArgs a) {
  constexpr int G = kWave / L;
  constexpr int VEC = 8 * L;
  constexpr int NV = SAVE ? 2 : 1, NS = SAVE ? 3 : 2;
  extern __shared__ __align__(16) unsigned char smem[];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int g = lane / L, l = lane % L;
  const int f0 = 8 * l;
  const bool active = f0 < a.F;
  const int f0c = active ? f0 : 0;
  const int head = f0c / a.D;
  const bool leader = active && (f0 % a.D) == 0;  // the lane that writes its head's scalars
  const int S = a.S;
  const GatLds lay = gat_lds_layout(S, L, SAVE);
  unsigned char* base = smem + size_t(wave) * lay.total;
  int* s_col = reinterpret_cast<int*>(base + lay.col_off);
  int* s_row = reinterpret_cast<int*>(base + lay.row_off);
  int* s_blk = reinterpret_cast<int*>(base + lay.blk_off);
  // The piece that entered a group's chunk is parked in LDS when its row ends; the piece that leaves the chunk stays
  // in the group's registers and the merge reads it from there (cross-lane reads take no LDS allocation, and the
  // kernel's speed follows the number of waves that fit a compute unit).
  float* m_vec = reinterpret_cast<float*>(base + lay.vec_off);  // [G][NV][VEC]: the entering piece of group g
  float* m_mz = reinterpret_cast<float*>(base + lay.mz_off);    // [G][L][NS]: its (m, z[, zm]), per lane
  int* m_flag = reinterpret_cast<int*>(base + lay.flag_off);    // bit0 entering, bit1 runs through, bit2 leaving
  int* m_hrow = m_flag + G;
  int* m_trow = m_hrow + G;

  const int wpb = int(blockDim.x) / kWave;  // waves per workgroup (4, 2 or 1, chosen on the host for LDS packing)
  int64_t wg = blockIdx.x, wg_count = gridDim.x;
  if (a.blocks)
    wg = gat_enter_block(a, wg, wg_count, [&](const hgnn_seg_block& B) {
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
  if (valid) {
    row_lo = a.seg_lo[seg];
    row_hi = a.seg_hi[seg];
  }

  // ---- phase 1: column ids (as byte offsets of the neighbour's row where they fit 32 bits) and row ids
  seg_stage_cols(a.col, e0, lane, spad, n, stream_nontemporal(a.nnz),
                 [&](int i, int c) { s_col[i] = OFF32 ? int(uint32_t(c) * uint32_t(a.ldx) * 2u) : c; });
  if (lane < G) m_flag[lane] = 0;
  bool seg_open[2];
  seg_stage_rows(s_row, s_blk, lane, per, n, row_lo, row_hi, a.rowptr, e0, seg_open);
  const bool seg_left_open = seg_open[0], seg_right_open = seg_open[1];
  wave_sync();

  // ---- phase 2: running (m, z, acc) over this group's chunk
  const int C = 4 * ((S + 4 * G - 1) / (4 * G));
  const int c0 = g * C < n ? g * C : n;
  const int c1 = c0 + C < n ? c0 + C : n;
  Soft<SAVE> t;
  int cur = -1;
  bool lo = false;  // current piece began before this chunk

  auto park = [&](int slot, const Soft<SAVE>& v) {
    if (active) {
      float* dst = m_vec + slot * NV * VEC + f0;
#pragma unroll
      for (int i = 0; i < 8; ++i) dst[i] = v.acc[i];
      if (SAVE) {
#pragma unroll
        for (int i = 0; i < 8; ++i) dst[VEC + i] = v.accm[i];
      }
    }
    m_mz[(slot * L + l) * NS] = v.m;
    m_mz[(slot * L + l) * NS + 1] = v.z;
    if (SAVE) m_mz[(slot * L + l) * NS + 2] = v.zm;
  };
  auto unpark = [&](int slot) -> Soft<SAVE> {
    Soft<SAVE> v;
    const float* src = m_vec + slot * NV * VEC + f0c;
#pragma unroll
    for (int i = 0; i < 8; ++i) v.acc[i] = src[i];
    if (SAVE) {
#pragma unroll
      for (int i = 0; i < 8; ++i) v.accm[i] = src[VEC + i];
    }
    v.m = m_mz[(slot * L + l) * NS];
    v.z = m_mz[(slot * L + l) * NS + 1];
    if (SAVE) v.zm = m_mz[(slot * L + l) * NS + 2];
    return v;
  };
  auto flush = [&](bool ro) {
    if (!lo && !ro) {
      if (active) row_store<SAVE>(a, cur, f0, head, leader, t);
    } else if (lo) {
      park(g, t);
      if (l == 0) {
        m_flag[g] |= ro ? 3 : 1;
        m_hrow[g] = cur;
      }
    } else if (l == 0) {  // leaves into the next chunk (only the last flush of a chunk gets here): stays in t
      m_flag[g] |= 4;
      m_trow[g] = cur;
    }
  };
  auto gather = [&](int c) -> half8_t {
    if (OFF32) {
      const uint32_t boff = uint32_t(c) + uint32_t(f0c) * 2u;
      return *reinterpret_cast<const half8_t*>(reinterpret_cast<const char*>(a.X) + boff);
    }
    return *reinterpret_cast<const half8_t*>(a.X + int64_t(c) * a.ldx + f0c);
  };

  float el_cur = 0.f;  // the row-side score term of the current row, fetched when the row changes
  if (c0 < c1) {
    cur = s_row[c0];
    lo = c0 > 0 ? s_row[c0 - 1] == cur : seg_left_open;
    el_cur = a.el[int64_t(cur) * a.H + head];
  }
  const int LH = a.D / 8;  // lanes per head (power of two)
  typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
  half2_t ar2[4];
  {
    const half8_t t = *reinterpret_cast<const half8_t*>(a.a_r + f0c);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      ar2[q][0] = active ? t[2 * q] : half_t(0);
      ar2[q][1] = active ? t[2 * q + 1] : half_t(0);
    }
  }
  // the lanes of a group share their chunk, so the exchanges between the lanes of a head always meet
  for (int i = c0; i < c1; i += 4) {
    const int4_t cols = *reinterpret_cast<const int4_t*>(s_col + i);
    const int blk = s_blk[i >> 2];
    half8_t x[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) x[u] = gather(cols[u]);
    float sc[4];  // column-side term a_r.x from the row just gathered, summed over the lanes of the head
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      float d = 0.f;
#pragma unroll
      for (int q = 0; q < 4; ++q) {  // two fp16 products per instruction, fp32 sum
        half2_t xv;
        xv[0] = x[u][2 * q];
        xv[1] = x[u][2 * q + 1];
        d = __builtin_amdgcn_fdot2(ar2[q], xv, d, false);
      }
      sc[u] = d;
    }
    head_sum4(sc, LH);
    if (blk == cur) {  // four more edges of the current row: one rescale, four terms
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const float v = sc[u] + el_cur;
        sc[u] = v > 0.f ? v : a.slope * v;
      }
      const float mn = fmaxf(fmaxf(t.m, fmaxf(sc[0], sc[1])), fmaxf(sc[2], sc[3]));
      t.scale(__expf(t.m - mn));
#pragma unroll
      for (int u = 0; u < 4; ++u) t.add(__expf(sc[u] - mn), sc[u], a.slope, x[u]);
      t.m = mn;
    } else {
      const int4_t rows = *reinterpret_cast<const int4_t*>(s_row + i);
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (i + u < c1) {
          if (rows[u] != cur) {
            flush(false);
            t.clear();
            cur = rows[u];
            lo = false;
            el_cur = a.el[int64_t(cur) * a.H + head];
          }
          const float v = sc[u] + el_cur;
          const float e = v > 0.f ? v : a.slope * v;
          const float mn = fmaxf(t.m, e);
          t.scale(__expf(t.m - mn));
          t.add(__expf(e - mn), e, a.slope, x[u]);
          t.m = mn;
        }
      }
    }
  }
  if (c0 < c1) flush(c1 < n ? s_row[c1] == cur : seg_right_open);
  wave_sync();

  // ---- merge: group 0 sews the parked pieces together in chunk order
  if (valid) {  // all lanes take part in the cross-lane reads; only group 0 keeps and stores the result
    Soft<SAVE> run;
    bool open = false, from_before = false;
    int run_row = -1;
    const bool me = g == 0 && active;
    for (int gg = 0; gg < G; ++gg) {
      const int fl = m_flag[gg];  // the same value on every lane
      if (fl & 1) {
        if (g == 0) soft_merge<SAVE>(run, unpark(gg));
        if (gg == 0) {
          from_before = true;
          open = true;
          run_row = m_hrow[0];
        }
        if (!(fl & 2)) {  // the row ends inside chunk gg
          if (me) {
            if (from_before) stage_store<SAVE>(a, 2 * seg, f0, head, leader, run);
            else row_store<SAVE>(a, run_row, f0, head, leader, run);
          }
          run.clear();
          open = false;
          from_before = false;
        }
      }
      if (fl & 4) {  // the piece that left chunk gg: from the registers of group gg
        const int src = gg * L + l;
        run.m = __shfl(t.m, src);
        run.z = __shfl(t.z, src);
#pragma unroll
        for (int i = 0; i < 8; ++i) run.acc[i] = __shfl(t.acc[i], src);
        if (SAVE) {
          run.zm = __shfl(t.zm, src);
#pragma unroll
          for (int i = 0; i < 8; ++i) run.accm[i] = __shfl(t.accm[i], src);
        }
        run_row = m_trow[gg];
        open = true;
        from_before = false;
      }
    }
    if (open && me)  // leaves into the next segment; a piece that also entered uses slot 2*seg
      stage_store<SAVE>(a, 2 * seg + (from_before ? 0 : 1), f0, head, leader, run);
  }

  // ---- this wave's share of the empty rows
  const int64_t nw = wg_count * wpb;
  const int rpw = int((a.nrows + nw - 1) / nw);
  const int64_t r0 = wid * rpw;
  const int64_t r1 = r0 + rpw < a.nrows ? r0 + rpw : a.nrows;
  if (active) {
    const Soft<SAVE> none;
    for (int64_t r = r0 + g; r < r1; r += G)
      if (a.rowptr[r] == a.rowptr[r + 1]) row_store<SAVE>(a, r, f0, head, leader, none);
  }
}

// Follow-up kernel: merges the staged pieces of every row that crosses a segment border (the tail
// piece of its first segment, then the head pieces of the following ones) and stores the row.
// A wave owns G split rows; rows of up to kShortPieces pieces are merged by their own lane group,
// hubs by the whole wave with a final merge across the groups.
constexpr int kShortPieces = 8;

template <int L, bool SAVE>
__global__ __launch_bounds__(kBlock) void gat_finish_kernel(GatArgs a) {
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
    wg = gat_enter_block(a, wg, wg_count, [&](const hgnn_seg_block& B) {
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
  auto take = [&](Soft<SAVE>& t, int64_t slot) {
    const half8_t o = *reinterpret_cast<const half8_t*>(a.staging + slot * a.stage_ld + f0c);
    half8_t om = o;
    float cp = 0.f;
    if (SAVE) {
      om = *reinterpret_cast<const half8_t*>(a.staging_m + slot * a.stage_ld + f0c);
      cp = a.stage_c[slot * a.H + head];
    }
    soft_merge_normalised<SAVE>(t, a.stage_mz[(slot * a.H + head) * 2], a.stage_mz[(slot * a.H + head) * 2 + 1], cp, o, om);
  };
  if (idx < a.n_split && sb - sa <= kShortPieces) {
    Soft<SAVE> t;
    take(t, 2 * int64_t(sa) + 1);
    for (int64_t k = int64_t(sa) + 1; k <= sb; ++k) take(t, 2 * k);
    if (active) row_store<SAVE>(a, r, f0, head, leader, t);
  }
  for (int j = 0; j < G; ++j) {
    const int rj = __shfl(r, j * L), sj = __shfl(sa, j * L), ej = __shfl(sb, j * L);
    if (ej - sj <= kShortPieces) continue;
    Soft<SAVE> t;
    if (g == 0) take(t, 2 * int64_t(sj) + 1);
    for (int64_t k = int64_t(sj) + 1 + g; k <= ej; k += G) take(t, 2 * k);
#pragma unroll
    for (int off = L; off < kWave; off <<= 1) {
      Soft<SAVE> o;
      o.m = __shfl_xor(t.m, off);
      o.z = __shfl_xor(t.z, off);
#pragma unroll
      for (int i = 0; i < 8; ++i) o.acc[i] = __shfl_xor(t.acc[i], off);
      if (SAVE) {
        o.zm = __shfl_xor(t.zm, off);
#pragma unroll
        for (int i = 0; i < 8; ++i) o.accm[i] = __shfl_xor(t.accm[i], off);
      }
      soft_merge<SAVE>(t, o);
    }
    if (g == 0 && active) row_store<SAVE>(a, rj, f0, head, leader, t);
  }
}

// Column-blocked plans: merges the nb partial rows (normalised fp16 vectors + (m, z[, zm/z])) of every row.
struct GatBlockParts {
  const half_t* vec;    // [nb][nrows][ld]
  const half_t* vec_m;  // SAVE: the masked counterpart
  int ld;
  const float* mz;      // [nb] x mz_stride: [nrows][H][2]
  int64_t mz_stride;
  const float* c;       // SAVE: [nb] x c_stride: [nrows][H]
  int64_t c_stride;
  int nb;
};

template <int L, bool SAVE>
__global__ __launch_bounds__(kBlock) void gat_block_merge_kernel(GatArgs a, GatBlockParts q) {
  constexpr int G = kWave / L;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int g = lane / L, l = lane % L;
  const int f0 = 8 * l;
  const int64_t r = (int64_t(blockIdx.x) * kWavesPerBlock + wave) * G + g;
  if (r >= a.nrows || f0 >= a.F) return;
  const int head = f0 / a.D;
  Soft<SAVE> t;
  for (int b = 0; b < q.nb; ++b) {
    const int64_t pr = int64_t(b) * a.nrows + r;
    const half8_t o = *reinterpret_cast<const half8_t*>(q.vec + pr * q.ld + f0);
    half8_t om = o;
    float cp = 0.f;
    if (SAVE) {
      om = *reinterpret_cast<const half8_t*>(q.vec_m + pr * q.ld + f0);
      cp = q.c[b * q.c_stride + r * a.H + head];
    }
    const float* mz = q.mz + b * q.mz_stride + (r * a.H + head) * 2;
    soft_merge_normalised<SAVE>(t, mz[0], mz[1], cp, o, om);
  }
  row_store<SAVE>(a, r, f0, head, (f0 % a.D) == 0, t);
}

template <int L, bool OFF32>
static void launch_gat_seg_l(bool save, dim3 grid, int threads, size_t lds, hipStream_t s, const GatArgs& a) {
  if (save) gat_seg_kernel<L, OFF32, true><<<grid, threads, lds, s>>>(a);
  else gat_seg_kernel<L, OFF32, false><<<grid, threads, lds, s>>>(a);
}

template <bool OFF32>
static void launch_gat_seg(int L, bool save, dim3 grid, int threads, size_t lds, hipStream_t s, const GatArgs& a) {
  switch (L) {
    case 1: launch_gat_seg_l<1, OFF32>(save, grid, threads, lds, s, a); break;
    case 2: launch_gat_seg_l<2, OFF32>(save, grid, threads, lds, s, a); break;
    case 4: launch_gat_seg_l<4, OFF32>(save, grid, threads, lds, s, a); break;
    case 8: launch_gat_seg_l<8, OFF32>(save, grid, threads, lds, s, a); break;
    case 16: launch_gat_seg_l<16, OFF32>(save, grid, threads, lds, s, a); break;
    case 32: launch_gat_seg_l<32, OFF32>(save, grid, threads, lds, s, a); break;
    default: launch_gat_seg_l<64, OFF32>(save, grid, threads, lds, s, a); break;
  }
}

template <int L>
static void launch_gat_finish_l(bool save, dim3 grid, hipStream_t s, const GatArgs& a) {
  if (save) gat_finish_kernel<L, true><<<grid, kBlock, 0, s>>>(a);
  else gat_finish_kernel<L, false><<<grid, kBlock, 0, s>>>(a);
}

static void launch_gat_finish(int L, bool save, dim3 grid, hipStream_t s, const GatArgs& a) {
  switch (L) {
    case 1: launch_gat_finish_l<1>(save, grid, s, a); break;
    case 2: launch_gat_finish_l<2>(save, grid, s, a); break;
    case 4: launch_gat_finish_l<4>(save, grid, s, a); break;
    case 8: launch_gat_finish_l<8>(save, grid, s, a); break;
    case 16: launch_gat_finish_l<16>(save, grid, s, a); break;
    case 32: launch_gat_finish_l<32>(save, grid, s, a); break;
    default: launch_gat_finish_l<64>(save, grid, s, a); break;
  }
}

template <int L>
static void launch_gat_block_merge_l(bool save, dim3 grid, hipStream_t s, const GatArgs& a, const GatBlockParts& q) {
  if (save) gat_block_merge_kernel<L, true><<<grid, kBlock, 0, s>>>(a, q);
  else gat_block_merge_kernel<L, false><<<grid, kBlock, 0, s>>>(a, q);
}

static void launch_gat_block_merge(int L, bool save, dim3 grid, hipStream_t s, const GatArgs& a, const GatBlockParts& q) {
  switch (L) {
    case 1: launch_gat_block_merge_l<1>(save, grid, s, a, q); break;
    case 2: launch_gat_block_merge_l<2>(save, grid, s, a, q); break;
    case 4: launch_gat_block_merge_l<4>(save, grid, s, a, q); break;
    case 8: launch_gat_block_merge_l<8>(save, grid, s, a, q); break;
    case 16: launch_gat_block_merge_l<16>(save, grid, s, a, q); break;
    case 32: launch_gat_block_merge_l<32>(save, grid, s, a, q); break;
    default: launch_gat_block_merge_l<64>(save, grid, s, a, q); break;
  }
}

// segment pass + follow-up pass for the graph in `a` with the segment arrays of plan q
static hgnn_status run_gat_segments(const hgnn_plan* q, GatArgs a, int ncols, hipStream_t s) {
  a.seg_lo = q->seg_row_lo;
  a.seg_hi = q->seg_row_hi;
  a.S = q->S;
  a.nseg = q->nseg;
  a.staging = reinterpret_cast<half_t*>(q->staging);
  a.stage_mz = q->stage_mz;
  a.stage_ld = q->max_F;
  const bool save = a.Ym != nullptr;
  // the plan holds a second set of staging vectors and a third scalar per staged piece behind the first
  a.staging_m = a.staging + size_t(2) * size_t(q->nseg) * size_t(q->max_F);
  a.stage_c = q->stage_mz + size_t(4) * size_t(q->nseg) * size_t(q->max_H);
  a.split_row = q->split_row;
  a.split_lo = q->split_seg_lo;
  a.split_hi = q->split_seg_hi;
  a.n_split = q->n_split;
  const int L = pow2_at_least(a.F / 8);
  const size_t per_wave = size_t(gat_lds_layout(a.S, L, save).total);
  const int wpb = waves_per_block_for_lds(per_wave, true);
  const size_t lds = per_wave * wpb;
  HGNN_REQUIRE(lds <= 65536, HGNN_EUNSUPPORTED,
               "hgnn_gat_forward_fused: seg_edges = %d with H = %d needs %zu bytes of LDS per workgroup (limit 65536)", a.S,
               a.H, lds);
  const int64_t nblk = ceil_div(q->nseg, wpb);
  dim3 grid(unsigned(nblk > 0 ? nblk : 1));
  const int threads = wpb * kWave;
  const bool off32 = uint64_t(ncols) * uint64_t(a.ldx) * 2u < (uint64_t(1) << 32);
  if (off32) launch_gat_seg<true>(L, save, grid, threads, lds, s, a);
  else launch_gat_seg<false>(L, save, grid, threads, lds, s, a);
  HGNN_LAUNCH_CHECK("gat_seg_kernel");
  if (a.n_split > 0) {
    launch_gat_finish(L, save, dim3(unsigned(ceil_div(a.n_split, int64_t(kWavesPerBlock) * (kWave / L)))), s, a);
    HGNN_LAUNCH_CHECK("gat_finish_kernel");
  }
  return HGNN_OK;
}

}  // namespace hgnn

using namespace hgnn;

// out_masked / csum: nullptr, or the tensors a later backward call wants (see the SAVE kernels)
static hgnn_status gat_forward_impl(const char* who, const hgnn_csr* g, const hgnn_plan* p, int32_t H, int32_t D,
                                    const hgnn_half* U, int64_t ldu, const hgnn_half* Vt, int64_t ldv, const hgnn_half* a_l,
                                    const hgnn_half* a_r, float neg_slope, hgnn_half* out, int64_t ldo, float* lse,
                                    hgnn_half* out_masked, int64_t ldom, float* csum, void* stream) {
  clear_error();
  hgnn_status st = check_csr_args(g, who);
  if (st != HGNN_OK) return st;
  HGNN_REQUIRE(p != nullptr, HGNN_EINVAL, "%s: plan is NULL", who);
  HGNN_REQUIRE(p->nrows == g->nrows && p->ncols == g->ncols && p->nnz == g->nnz, HGNN_EINVAL,
               "%s: the plan was built for another graph", who);
  HGNN_REQUIRE(g->eid == nullptr, HGNN_EUNSUPPORTED, "%s: an edge-id map is not supported here", who);
  HGNN_REQUIRE(H >= 1 && D >= 1 && int64_t(H) * D <= 512, HGNN_EINVAL, "%s: H = %d, D = %d out of range", who, H, D);
  const int F = H * D;
  HGNN_REQUIRE(H <= p->max_H && F <= p->max_F, HGNN_EINVAL, "%s: H = %d / F = %d exceed the plan's max_H = %d / max_F = %d",
               who, H, F, p->max_H, p->max_F);
  HGNN_REQUIRE(ldo >= F && ldv >= F && ldu >= F, HGNN_EINVAL, "%s: leading dimension smaller than F", who);
  HGNN_REQUIRE((out_masked == nullptr) == (csum == nullptr), HGNN_EINVAL, "%s: out_masked and csum go together", who);
  HGNN_REQUIRE(out_masked == nullptr || (ldom >= F && neg_slope >= 0.f), HGNN_EINVAL,
               "%s: out_masked needs ldom >= F and a slope >= 0", who);
  HGNN_REQUIRE(g->nrows == 0 || out != nullptr, HGNN_EINVAL, "%s: out is NULL", who);
  if (g->nrows == 0) return HGNN_OK;
  HGNN_REQUIRE(U && Vt && a_l && a_r, HGNN_EINVAL, "%s: U, Vt, a_l or a_r is NULL", who);
  HGNN_REQUIRE(D % 8 == 0 && ldv % 8 == 0 && ldo % 8 == 0 && aligned16(Vt) && aligned16(out), HGNN_EUNSUPPORTED,
               "%s: needs D %% 8 == 0, ld %% 8 == 0 and 16-byte aligned Vt, out", who);
  HGNN_REQUIRE(out_masked == nullptr || (ldom % 8 == 0 && aligned16(out_masked)), HGNN_EUNSUPPORTED,
               "%s: needs ldom %% 8 == 0 and a 16-byte aligned out_masked", who);
  hipStream_t s = static_cast<hipStream_t>(stream);
  // per-vertex projection into the plan's fp32 scratch: el[i,h] = a_l[h].U[i,h]; the column-side term is formed in
  // the kernel from the gathered row
  st = gat_project(p, g, H, D, U, ldu, nullptr, ldv, a_l, a_r, s, who);
  if (st != HGNN_OK) return st;
  GatArgs a{};
  a.rowptr = g->rowptr;
  a.col = g->col;
  a.X = reinterpret_cast<const half_t*>(Vt);
  a.Y = reinterpret_cast<half_t*>(out);
  a.ldx = ldv;
  a.ldy = ldo;
  a.nnz = g->nnz;
  a.nrows = g->nrows;
  a.F = F;
  a.H = H;
  a.D = D;
  a.slope = neg_slope;
  a.el = p->vscratch;
  a.a_r = reinterpret_cast<const half_t*>(a_r);
  a.lse = lse;
  a.Ym = reinterpret_cast<half_t*>(out_masked);
  a.ldym = ldom;
  a.csum = csum;
  const bool save = out_masked != nullptr;
  if (p->nb <= 1) return run_gat_segments(p, a, g->ncols, s);
  // column-blocked plan: every block leaves normalised partial rows and their (m, z[, zm/z]) per row; one pass merges them
  const size_t V = size_t(p->nrows);
  const size_t flat = size_t(p->nb) * V;
  half_t* bstage = reinterpret_cast<half_t*>(p->bstage);
  half_t* bstage_m = bstage + flat * size_t(p->max_F);    // the plan holds a second set of partial rows behind the first
  float* bsum_c = p->bsum + 2 * flat * size_t(p->max_H);  // and a third scalar per partial row
  const int L = pow2_at_least(F / 8);
  {
    // all blocks in one launch of each kernel: workgroups numbered block after block and dispatched in that order
    GatArgs ab = a;
    ab.Y = bstage;
    ab.ldy = p->max_F;
    ab.lse = nullptr;
    ab.part_mz = p->bsum;
    ab.Ym = save ? bstage_m : nullptr;
    ab.ldym = p->max_F;
    ab.csum = save ? bsum_c : nullptr;
    ab.blocks = p->bdesc;
    ab.nblocks = p->nb;
    ab.max_F = p->max_F;
    ab.max_H = p->max_H;
    ab.y_stride = int64_t(V) * p->max_F;
    ab.mz_stride = int64_t(V) * p->max_H * 2;
    ab.c_stride = int64_t(V) * p->max_H;
    ab.S = p->S;
    ab.stage_ld = p->max_F;
    const size_t per_wave = size_t(gat_lds_layout(ab.S, L, save).total);
    const int wpb = waves_per_block_for_lds(per_wave, true);
    const size_t lds = per_wave * wpb;
    HGNN_REQUIRE(lds <= 65536, HGNN_EUNSUPPORTED,
                 "%s: seg_edges = %d with H = %d needs %zu bytes of LDS per workgroup (limit 65536)", who, ab.S, ab.H, lds);
    int64_t wgs = 0, wgs2 = 0;
    for (const hgnn_plan* q : p->sub) {
      const int64_t c = ceil_div(q->nseg, wpb);
      wgs += c > 0 ? c : 1;
      wgs2 += ceil_div(q->n_split, int64_t(kWavesPerBlock) * (kWave / L));
    }
    const bool off32 = uint64_t(g->ncols) * uint64_t(ab.ldx) * 2u < (uint64_t(1) << 32);
    if (off32) launch_gat_seg<true>(L, save, dim3(unsigned(wgs)), wpb * kWave, lds, s, ab);
    else launch_gat_seg<false>(L, save, dim3(unsigned(wgs)), wpb * kWave, lds, s, ab);
    HGNN_LAUNCH_CHECK("gat_seg_kernel");
    if (wgs2 > 0) {
      launch_gat_finish(L, save, dim3(unsigned(wgs2)), s, ab);
      HGNN_LAUNCH_CHECK("gat_finish_kernel");
    }
  }
  const GatBlockParts parts{bstage, bstage_m, p->max_F, p->bsum, int64_t(V) * p->max_H * 2, bsum_c, int64_t(V) * p->max_H, p->nb};
  launch_gat_block_merge(L, save, dim3(unsigned(ceil_div(g->nrows, int64_t(kWavesPerBlock) * (kWave / L)))), s, a, parts);
  HGNN_LAUNCH_CHECK("gat_block_merge_kernel");
  return HGNN_OK;
}

extern "C" {

hgnn_status hgnn_gat_forward_fused(const hgnn_csr* g, const hgnn_plan* p, int32_t H, int32_t D, const hgnn_half* U,
                                   int64_t ldu, const hgnn_half* Vt, int64_t ldv, const hgnn_half* a_l,
                                   const hgnn_half* a_r, float neg_slope, hgnn_half* out, int64_t ldo, float* lse,
                                   void* stream) {
  return gat_forward_impl("hgnn_gat_forward_fused", g, p, H, D, U, ldu, Vt, ldv, a_l, a_r, neg_slope, out, ldo, lse, nullptr, 0,
                          nullptr, stream);
}

hgnn_status hgnn_gat_forward_fused_save(const hgnn_csr* g, const hgnn_plan* p, int32_t H, int32_t D, const hgnn_half* U,
                                        int64_t ldu, const hgnn_half* Vt, int64_t ldv, const hgnn_half* a_l,
                                        const hgnn_half* a_r, float neg_slope, hgnn_half* out, int64_t ldo, float* lse,
                                        hgnn_half* out_masked, int64_t ldom, float* csum, void* stream) {
  const char* who = "hgnn_gat_forward_fused_save";
  if (out_masked == nullptr || csum == nullptr || lse == nullptr) {
    clear_error();
    return fail(HGNN_EINVAL, "%s: lse, out_masked and csum are required", who);
  }
  return gat_forward_impl(who, g, p, H, D, U, ldu, Vt, ldv, a_l, a_r, neg_slope, out, ldo, lse, out_masked, ldom, csum, stream);
}

}  // extern "C"
