// Edge softmax (paper Eq. 1), its backward, and row sums of edge tensors, for gfx950.
//
// The scores of one row (neighbourhood) are the contiguous slice e[rowptr[i]*H, rowptr[i+1]*H),
// element j of the whole tensor belonging to head j % H.  A "team" of lanes owns a row: a
// sub-wave group of LR lanes (LR chosen from the mean row length, so short rows do not idle a
// whole wave) or a whole wave; rows longer than the plan's threshold are cut into chunks, a
// workgroup each, whose partial results a second launch combines.
// Every lane moves 16 bytes (8 halves) per access: the slice is walked in 8-element vectors
// aligned to the tensor's base, the ragged first and last vector are masked, and because H
// divides 8 the head of each of a lane's 8 elements is fixed.  A row that fits the lanes'
// registers is read once.  exp, sums and the division stay in fp32; the exponent is <= 0, so
// the numerator is in (0,1] (section 3.1.2) and alpha is rounded once.
#include "common.h"

namespace hgnn {

constexpr int kKeepVec = 2;     // 8-element vectors per lane held in registers
constexpr int kTeamThreads = 64;  // workgroup size of the team kernel: its waves never meet, so one wave each

struct EdgeRowArgs {
  const int* rowptr;
  const int* big_row;
  const int* row_list;  // when set, the team kernel takes its rows from this list of n_list rows
  int n_list;
  const int* eid;
  const half_t* x0;  // forward: e.          backward: alpha.   rowsum: t
  const half_t* x1;  //                      backward: dalpha
  const half_t* x2;  //                      backward: e (LeakyReLU mask) or nullptr
  half_t* out;       // forward: alpha.      backward: de.      rowsum: [nrows][H]
  float* out_f32;    // rowsum only: when set, the sums are written here in fp32 instead of out
  int64_t total;     // nnz * H
  int nrows, H;
  int skip_above;    // rows longer than this are left to a later tier (0 = none)
  int skip_below;    // rows of at most this many non-zeros were done by an earlier tier (-1 = none)
  float slope;
};

// ---- teams -----------------------------------------------------------------------------------------
// One step of an all-reduce (sum or maximum) among aligned groups of lanes: with the partner inside a row of 16
// lanes the exchange is a DPP operand of the VALU instruction (lane ^ 1, lane ^ 2, then mirrors inside 8 and 16
// lanes, which pair a lane with one from the other half, whose partial result is the same on all its lanes);
// across rows it goes through ds_bpermute.
template <int OFF, bool IS_MAX>
__device__ __forceinline__ float team_step(float v) {
  float o;
  if (OFF == 1) o = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xf, 0xf, false));
  else if (OFF == 2) o = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xf, 0xf, false));
  else if (OFF == 4) o = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xf, 0xf, false));
  else if (OFF == 8) o = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xf, 0xf, false));
  else o = __shfl_xor(v, OFF);
  return IS_MAX ? fmaxf(v, o) : v + o;
}

template <int N, int H, bool IS_MAX>  // all-reduce over aligned groups of N lanes (N a power of two up to 64)
__device__ __forceinline__ void team_reduce(float (&v)[H]) {
#pragma unroll
  for (int h = 0; h < H; ++h) {
    if (N > 1) v[h] = team_step<1, IS_MAX>(v[h]);
    if (N > 2) v[h] = team_step<2, IS_MAX>(v[h]);
    if (N > 4) v[h] = team_step<4, IS_MAX>(v[h]);
    if (N > 8) v[h] = team_step<8, IS_MAX>(v[h]);
    if (N > 16) v[h] = team_step<16, IS_MAX>(v[h]);
    if (N > 32) v[h] = team_step<32, IS_MAX>(v[h]);
  }
}

template <int LR>
struct SubWaveTeam {  // LR consecutive lanes of a wave
  static constexpr int size = LR;
  int rank;
  __device__ SubWaveTeam() : rank((threadIdx.x & (kWave - 1)) % LR) {}
  template <int H, bool IS_MAX>
  __device__ __forceinline__ void reduce(float (&v)[H]) const {
    team_reduce<LR, H, IS_MAX>(v);
  }
};

// 8 elements starting at the 8-aligned index b; a vector that would cross the end of the tensor is read by element
__device__ __forceinline__ half8_t load_vec(const half_t* p, int64_t b, int64_t total) {
  if (b + 8 <= total) return *reinterpret_cast<const half8_t*>(p + b);
  half8_t v = half8_t(0);
#pragma unroll
  for (int q = 0; q < 8; ++q)
    if (b + q < total) v[q] = p[b + q];
  return v;
}
// load_vec with the elements outside [j0, j1) replaced by `fill` (the neutral value of what the caller does with
// them), so that the passes over the vector need no bounds checks of their own: two 32-bit compares and a select
// per element, once, instead of two 64-bit compares per element and pass
__device__ __forceinline__ half8_t load_vec_in(const half_t* p, int64_t b, int64_t total, int64_t j0, int64_t j1, half_t fill) {
  half8_t v = load_vec(p, b, total);
  const int lo = j0 > b ? int(j0 - b) : 0;          // first valid element
  const int hi = j1 - b < 8 ? int(j1 - b) : 8;      // one past the last valid element
#pragma unroll
  for (int q = 0; q < 8; ++q)
    if (q < lo || q >= hi) v[q] = fill;
  return v;
}
__device__ __forceinline__ void store_vec(half_t* p, int64_t b, const half8_t& v, int64_t j0, int64_t j1) {
  if (b >= j0 && b + 8 <= j1) {
    *reinterpret_cast<half8_t*>(p + b) = v;
  } else {
#pragma unroll
    for (int q = 0; q < 8; ++q)
      if (b + q >= j0 && b + q < j1) p[b + q] = v[q];
  }
}

// ---- forward: one row by one team ----------------------------------------------------------------------
template <int H, class Team>
__device__ __forceinline__ void softmax_fwd_row(const EdgeRowArgs& a, const Team& team, int64_t j0, int64_t j1) {
  const int64_t a0 = j0 & ~int64_t(7);
  const int64_t nvec = (j1 - a0 + 7) >> 3;
  half8_t keep[kKeepVec];
  float m[H];
#pragma unroll
  for (int h = 0; h < H; ++h) m[h] = -INFINITY;
  // elements of a vector that lie outside the row are read as -inf: they lose every maximum and add exp(-inf) = 0
  const half_t ninf = half_t(-INFINITY);
  auto visit_max = [&](const half8_t& v) {
#pragma unroll
    for (int q = 0; q < 8; ++q) m[q % H] = fmaxf(m[q % H], float(v[q]));
  };
#pragma unroll
  for (int i = 0; i < kKeepVec; ++i) {
    const int64_t t = team.rank + int64_t(Team::size) * i;
    keep[i] = half8_t(ninf);
    if (t < nvec) {
      keep[i] = load_vec_in(a.x0, a0 + 8 * t, a.total, j0, j1, ninf);
      visit_max(keep[i]);
    }
  }
  for (int64_t t = team.rank + int64_t(Team::size) * kKeepVec; t < nvec; t += Team::size)
    visit_max(load_vec_in(a.x0, a0 + 8 * t, a.total, j0, j1, ninf));
  team.template reduce<H, true>(m);
  float z[H];
#pragma unroll
  for (int h = 0; h < H; ++h) z[h] = 0.f;
  auto visit_sum = [&](const half8_t& v) {
#pragma unroll
    for (int q = 0; q < 8; ++q) z[q % H] += __expf(float(v[q]) - m[q % H]);
  };
  float ex[kKeepVec][8];  // the exponentials of the vectors held in registers, formed once
#pragma unroll
  for (int i = 0; i < kKeepVec; ++i) {
    const int64_t t = team.rank + int64_t(Team::size) * i;
#pragma unroll
    for (int q = 0; q < 8; ++q) ex[i][q] = 0.f;
    if (t < nvec) {
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        ex[i][q] = __expf(float(keep[i][q]) - m[q % H]);
        z[q % H] += ex[i][q];
      }
    }
  }
  for (int64_t t = team.rank + int64_t(Team::size) * kKeepVec; t < nvec; t += Team::size)
    visit_sum(load_vec_in(a.x0, a0 + 8 * t, a.total, j0, j1, ninf));
  team.template reduce<H, false>(z);
  float inv[H];
#pragma unroll
  for (int h = 0; h < H; ++h) inv[h] = 1.f / z[h];
  auto emit = [&](const half8_t& v, int64_t b) {
    half8_t o;
#pragma unroll
    for (int q = 0; q < 8; ++q) o[q] = half_t(__expf(float(v[q]) - m[q % H]) * inv[q % H]);
    store_vec(a.out, b, o, j0, j1);
  };
#pragma unroll
  for (int i = 0; i < kKeepVec; ++i) {
    const int64_t t = team.rank + int64_t(Team::size) * i;
    if (t < nvec) {
      half8_t o;
#pragma unroll
      for (int q = 0; q < 8; ++q) o[q] = half_t(ex[i][q] * inv[q % H]);
      store_vec(a.out, a0 + 8 * t, o, j0, j1);
    }
  }
  for (int64_t t = team.rank + int64_t(Team::size) * kKeepVec; t < nvec; t += Team::size)
    emit(load_vec(a.x0, a0 + 8 * t, a.total), a0 + 8 * t);
}

// ---- backward: t = sum alpha*dalpha (per head); de = alpha*(dalpha - t) [* LeakyReLU'(e)] --------------
template <int H, class Team>
__device__ __forceinline__ void softmax_bwd_row(const EdgeRowArgs& a, const Team& team, int64_t j0, int64_t j1) {
  const int64_t a0 = j0 & ~int64_t(7);
  const int64_t nvec = (j1 - a0 + 7) >> 3;
  half8_t ka[kKeepVec], kd[kKeepVec];
  float t[H];
#pragma unroll
  for (int h = 0; h < H; ++h) t[h] = 0.f;
  // elements outside the row are read as zero on both sides, so their products vanish (a neighbouring row's
  // infinity times zero would not)
  auto visit = [&](const half8_t& va, const half8_t& vd) {
#pragma unroll
    for (int q = 0; q < 8; ++q) t[q % H] = fmaf(float(va[q]), float(vd[q]), t[q % H]);
  };
#pragma unroll
  for (int i = 0; i < kKeepVec; ++i) {
    const int64_t v = team.rank + int64_t(Team::size) * i;
    ka[i] = half8_t(0);
    kd[i] = half8_t(0);
    if (v < nvec) {
      ka[i] = load_vec_in(a.x0, a0 + 8 * v, a.total, j0, j1, half_t(0));
      kd[i] = load_vec_in(a.x1, a0 + 8 * v, a.total, j0, j1, half_t(0));
      visit(ka[i], kd[i]);
    }
  }
  for (int64_t v = team.rank + int64_t(Team::size) * kKeepVec; v < nvec; v += Team::size)
    visit(load_vec_in(a.x0, a0 + 8 * v, a.total, j0, j1, half_t(0)), load_vec_in(a.x1, a0 + 8 * v, a.total, j0, j1, half_t(0)));
  team.template reduce<H, false>(t);
  auto emit = [&](const half8_t& va, const half8_t& vd, int64_t b) {
    half8_t o;
    half8_t ve = half8_t(1);
    if (a.x2) ve = load_vec(a.x2, b, a.total);
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      float d = float(va[q]) * (float(vd[q]) - t[q % H]);
      if (!(float(ve[q]) > 0.f)) d *= a.slope;
      o[q] = half_t(d);
    }
    store_vec(a.out, b, o, j0, j1);
  };
#pragma unroll
  for (int i = 0; i < kKeepVec; ++i) {
    const int64_t v = team.rank + int64_t(Team::size) * i;
    if (v < nvec) emit(ka[i], kd[i], a0 + 8 * v);
  }
  for (int64_t v = team.rank + int64_t(Team::size) * kKeepVec; v < nvec; v += Team::size)
    emit(load_vec(a.x0, a0 + 8 * v, a.total), load_vec(a.x1, a0 + 8 * v, a.total), a0 + 8 * v);
}

// ---- row sums: out[row,h] = sum over the row of t[slot(k), h] -------------------------------------------
template <int H, class Team>
__device__ __forceinline__ void rowsum_row(const EdgeRowArgs& a, const Team& team, int row, int beg, int end) {
  float s[H];
#pragma unroll
  for (int h = 0; h < H; ++h) s[h] = 0.f;
  if (a.eid) {  // transposed view: one lane per non-zero, its H values are contiguous at slot eid[k]
    typedef _Float16 hv_t __attribute__((ext_vector_type(H)));
    for (int k = beg + team.rank; k < end; k += Team::size) {
      const int64_t slot = a.eid[k];
      if (H == 1) {
        s[0] += float(a.x0[slot]);
      } else {
        const hv_t v = *reinterpret_cast<const hv_t*>(a.x0 + slot * H);
#pragma unroll
        for (int h = 0; h < H; ++h) s[h] += float(v[h]);
      }
    }
  } else {
    const int64_t j0 = int64_t(beg) * H, j1 = int64_t(end) * H;
    const int64_t a0 = j0 & ~int64_t(7);
    const int64_t nvec = (j1 - a0 + 7) >> 3;
    for (int64_t t = team.rank; t < nvec; t += Team::size) {
      const int64_t b = a0 + 8 * t;
      const half8_t v = load_vec(a.x0, b, a.total);
#pragma unroll
      for (int q = 0; q < 8; ++q)
        if (b + q >= j0 && b + q < j1) s[q % H] += float(v[q]);
    }
  }
  team.template reduce<H, false>(s);
  if (team.rank == 0) {
#pragma unroll
    for (int h = 0; h < H; ++h) {
      if (a.out_f32) a.out_f32[int64_t(row) * H + h] = s[h];
      else a.out[int64_t(row) * H + h] = half_t(s[h]);
    }
  }
}

enum { kFwd = 0, kBwd = 1, kSum = 2 };

template <int OP, int LR, int H>
__global__ __launch_bounds__(kBlock) void edge_row_team_kernel(EdgeRowArgs a) {
  constexpr int GR = kWave / LR;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  int64_t row = (int64_t(blockIdx.x) * (int(blockDim.x) / kWave) + wave) * GR + lane / LR;
  if (a.row_list) {
    if (row >= a.n_list) return;
    row = a.row_list[row];
  }
  if (row >= a.nrows) return;
  const int beg = a.rowptr[row], end = a.rowptr[row + 1];
  if ((a.skip_above > 0 && end - beg > a.skip_above) || end - beg <= a.skip_below) return;
  const SubWaveTeam<LR> team;
  if (OP == kSum) {
    rowsum_row<H>(a, team, int(row), beg, end);
  } else if (end > beg) {
    if (OP == kFwd) softmax_fwd_row<H>(a, team, int64_t(beg) * H, int64_t(end) * H);
    else softmax_bwd_row<H>(a, team, int64_t(beg) * H, int64_t(end) * H);
  }
}

// ---- long rows in chunks ------------------------------------------------------------------------------
// A row above the plan's long-row threshold is cut into chunks of kHubEdges non-zeros (the plan lists them): a
// workgroup of kHubThreads per chunk leaves the chunk's partial result per head -- (max, sum of exp) for the
// softmax, sum of alpha * dalpha for its backward, the sum for the row sums -- and a second launch combines the
// partials of a row (a few dozen at most) and writes the chunk's outputs, or the row's sum.  The latency of a long
// row is then that of one chunk, and a graph's longest rows keep many compute units busy instead of one each.
constexpr int kHubThreads = 256;

struct HubChunks {
  const int* row;    // [n] row of the chunk
  const int* first;  // [n] slot of the first chunk of that row
  const int* count;  // [n] chunks of that row
  float* part;       // [n][H][2]
};

template <int H, bool IS_MAX>
__device__ __forceinline__ void hub_block_reduce(float (&v)[H], float* sm) {  // sm: [kHubThreads / kWave][8]
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  team_reduce<kWave, H, IS_MAX>(v);
  __syncthreads();  // protects sm against the previous use
  if (lane == 0)
#pragma unroll
    for (int h = 0; h < H; ++h) sm[wave * 8 + h] = v[h];
  __syncthreads();
#pragma unroll
  for (int h = 0; h < H; ++h) {
    float r = sm[h];
    for (int w = 1; w < kHubThreads / kWave; ++w) r = IS_MAX ? fmaxf(r, sm[w * 8 + h]) : r + sm[w * 8 + h];
    v[h] = r;
  }
}

// the chunk's non-zeros [beg, end) of its row
__device__ __forceinline__ void hub_chunk_range(const EdgeRowArgs& a, const HubChunks& c, int slot, int& beg, int& end) {
  const int row = c.row[slot];
  beg = a.rowptr[row] + (slot - c.first[slot]) * kHubEdges;
  const int row_end = a.rowptr[row + 1];
  end = beg + kHubEdges < row_end ? beg + kHubEdges : row_end;
}

template <int OP, int H>
__global__ __launch_bounds__(kHubThreads) void edge_hub_partial_kernel(EdgeRowArgs a, HubChunks c) {
  __shared__ float sm[(kHubThreads / kWave) * 8];
  const int slot = blockIdx.x;
  int beg, end;
  hub_chunk_range(a, c, slot, beg, end);
  const int64_t j0 = int64_t(beg) * H, j1 = int64_t(end) * H;
  const int64_t a0 = j0 & ~int64_t(7);
  const int64_t nvec = (j1 - a0 + 7) >> 3;
  float r0[H], r1[H];
#pragma unroll
  for (int h = 0; h < H; ++h) {
    r0[h] = OP == kFwd ? -INFINITY : 0.f;
    r1[h] = 0.f;
  }
  if (OP == kSum && a.eid) {
    typedef _Float16 hv_t __attribute__((ext_vector_type(H)));
    for (int k = beg + int(threadIdx.x); k < end; k += kHubThreads) {
      const int64_t s = a.eid[k];
      if (H == 1) {
        r0[0] += float(a.x0[s]);
      } else {
        const hv_t v = *reinterpret_cast<const hv_t*>(a.x0 + s * H);
#pragma unroll
        for (int h = 0; h < H; ++h) r0[h] += float(v[h]);
      }
    }
  } else {
    for (int64_t t = threadIdx.x; t < nvec; t += kHubThreads) {
      const int64_t b = a0 + 8 * t;
      const half8_t v = load_vec(a.x0, b, a.total);
      half8_t d = half8_t(0);
      if (OP == kBwd) d = load_vec(a.x1, b, a.total);
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        if (b + q < j0 || b + q >= j1) continue;
        if (OP == kFwd) r0[q % H] = fmaxf(r0[q % H], float(v[q]));
        else if (OP == kBwd) r0[q % H] = fmaf(float(v[q]), float(d[q]), r0[q % H]);
        else r0[q % H] += float(v[q]);
      }
    }
  }
  hub_block_reduce<H, OP == kFwd>(r0, sm);
  if (OP == kFwd) {  // second walk (cache resident): the sum of exp relative to the chunk's maximum
    for (int64_t t = threadIdx.x; t < nvec; t += kHubThreads) {
      const int64_t b = a0 + 8 * t;
      const half8_t v = load_vec(a.x0, b, a.total);
#pragma unroll
      for (int q = 0; q < 8; ++q)
        if (b + q >= j0 && b + q < j1) r1[q % H] += __expf(float(v[q]) - r0[q % H]);
    }
    hub_block_reduce<H, false>(r1, sm);
  }
  if (threadIdx.x < H) {
    float v0 = 0.f, v1 = 0.f;
#pragma unroll
    for (int h = 0; h < H; ++h)
      if (int(threadIdx.x) == h) {
        v0 = r0[h];
        v1 = r1[h];
      }
    c.part[(int64_t(slot) * H + threadIdx.x) * 2] = v0;
    c.part[(int64_t(slot) * H + threadIdx.x) * 2 + 1] = v1;
  }
}

// softmax forward / backward: the row's partials combined, then this chunk's outputs
template <int OP, int H>
__global__ __launch_bounds__(kHubThreads) void edge_hub_emit_kernel(EdgeRowArgs a, HubChunks c) {
  const int slot = blockIdx.x;
  int beg, end;
  hub_chunk_range(a, c, slot, beg, end);
  const int first = c.first[slot], cnt = c.count[slot];
  float M[H], S[H];  // forward: row maximum and 1 / sum of exp; backward: S = sum of alpha * dalpha
#pragma unroll
  for (int h = 0; h < H; ++h) {
    M[h] = -INFINITY;
    S[h] = 0.f;
  }
  if (OP == kFwd) {
    for (int i = 0; i < cnt; ++i)
#pragma unroll
      for (int h = 0; h < H; ++h) M[h] = fmaxf(M[h], c.part[(int64_t(first + i) * H + h) * 2]);
  }
  for (int i = 0; i < cnt; ++i)
#pragma unroll
    for (int h = 0; h < H; ++h) {
      const float p0 = c.part[(int64_t(first + i) * H + h) * 2], p1 = c.part[(int64_t(first + i) * H + h) * 2 + 1];
      S[h] += OP == kFwd ? p1 * __expf(p0 - M[h]) : p0;
    }
  if (OP == kFwd) {
#pragma unroll
    for (int h = 0; h < H; ++h) S[h] = 1.f / S[h];
  }
  const int64_t j0 = int64_t(beg) * H, j1 = int64_t(end) * H;
  const int64_t a0 = j0 & ~int64_t(7);
  const int64_t nvec = (j1 - a0 + 7) >> 3;
  for (int64_t t = threadIdx.x; t < nvec; t += kHubThreads) {
    const int64_t b = a0 + 8 * t;
    const half8_t v = load_vec(a.x0, b, a.total);
    half8_t o;
    if (OP == kFwd) {
#pragma unroll
      for (int q = 0; q < 8; ++q) o[q] = half_t(__expf(float(v[q]) - M[q % H]) * S[q % H]);
    } else {
      const half8_t d = load_vec(a.x1, b, a.total);
      half8_t e = half8_t(1);
      if (a.x2) e = load_vec(a.x2, b, a.total);
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        float g = float(v[q]) * (float(d[q]) - S[q % H]);
        if (!(float(e[q]) > 0.f)) g *= a.slope;
        o[q] = half_t(g);
      }
    }
    store_vec(a.out, b, o, j0, j1);
  }
}

// row sums of the long rows: one thread per (row, head) adds the row's partial sums in chunk order
__global__ __launch_bounds__(kBlock) void edge_hub_rowsum_kernel(EdgeRowArgs a, HubChunks c, const int* __restrict__ big_first,
                                                                 int n_big) {
  const int i = blockIdx.x * kBlock + threadIdx.x;
  if (i >= n_big * a.H) return;
  const int r = i / a.H, h = i - r * a.H;
  const int first = big_first[r], cnt = c.count[first];
  float s = 0.f;
  for (int k = 0; k < cnt; ++k) s += c.part[(int64_t(first + k) * a.H + h) * 2];
  const int64_t o = int64_t(a.big_row[r]) * a.H + h;
  if (a.out_f32) a.out_f32[o] = s;
  else a.out[o] = half_t(s);
}

// Scalar path for head counts that do not divide 8: one thread per (row, head).
template <int OP>
__global__ __launch_bounds__(kBlock) void edge_row_scalar_kernel(EdgeRowArgs a) {
  const int64_t idx = int64_t(blockIdx.x) * kBlock + threadIdx.x;
  if (idx >= int64_t(a.nrows) * a.H) return;
  const int row = int(idx / a.H), h = int(idx % a.H);
  const int beg = a.rowptr[row], end = a.rowptr[row + 1];
  if (OP == kSum) {
    float s = 0.f;
    for (int k = beg; k < end; ++k) s += float(a.x0[(a.eid ? int64_t(a.eid[k]) : int64_t(k)) * a.H + h]);
    if (a.out_f32) a.out_f32[idx] = s;
    else a.out[idx] = half_t(s);
    return;
  }
  if (beg == end) return;
  if (OP == kFwd) {
    float m = -INFINITY, z = 0.f;
    for (int k = beg; k < end; ++k) m = fmaxf(m, float(a.x0[int64_t(k) * a.H + h]));
    for (int k = beg; k < end; ++k) z += __expf(float(a.x0[int64_t(k) * a.H + h]) - m);
    const float inv = 1.f / z;
    for (int k = beg; k < end; ++k)
      a.out[int64_t(k) * a.H + h] = half_t(__expf(float(a.x0[int64_t(k) * a.H + h]) - m) * inv);
  } else {
    float t = 0.f;
    for (int k = beg; k < end; ++k) t = fmaf(float(a.x0[int64_t(k) * a.H + h]), float(a.x1[int64_t(k) * a.H + h]), t);
    for (int k = beg; k < end; ++k) {
      const int64_t i = int64_t(k) * a.H + h;
      float d = float(a.x0[i]) * (float(a.x1[i]) - t);
      if (a.x2 && !(float(a.x2[i]) > 0.f)) d *= a.slope;
      a.out[i] = half_t(d);
    }
  }
}

template <int OP, int H>
static void launch_team_h(int LR, dim3 grid, hipStream_t s, const EdgeRowArgs& a) {
  switch (LR) {
    case 4: edge_row_team_kernel<OP, 4, H><<<grid, kTeamThreads, 0, s>>>(a); break;
    case 8: edge_row_team_kernel<OP, 8, H><<<grid, kTeamThreads, 0, s>>>(a); break;
    case 16: edge_row_team_kernel<OP, 16, H><<<grid, kTeamThreads, 0, s>>>(a); break;
    case 32: edge_row_team_kernel<OP, 32, H><<<grid, kTeamThreads, 0, s>>>(a); break;
    default: edge_row_team_kernel<OP, 64, H><<<grid, kTeamThreads, 0, s>>>(a); break;
  }
}

// Launches the team kernel (and the chunked kernels when a plan lists long rows) for H in {1,2,4,8}.
template <int OP>
static hgnn_status launch_edge_rows(const hgnn_csr* g, const hgnn_plan* p, EdgeRowArgs a, hipStream_t s) {
  const int H = a.H;
  // the chunked long-row kernels keep partial results in the plan, sized for its max_H heads: with more heads than
  // that the call runs as it does without a plan (a wave for every row above the sub-wave tier)
  if (p && H > p->max_H) p = nullptr;
  if (!(H == 1 || H == 2 || H == 4 || H == 8) || !aligned16(a.x0) || !aligned16(a.out) ||
      (a.x1 && !aligned16(a.x1)) || (a.x2 && !aligned16(a.x2))) {
    edge_row_scalar_kernel<OP><<<dim3(unsigned(ceil_div(int64_t(g->nrows) * H, kBlock))), kBlock, 0, s>>>(a);
    HGNN_LAUNCH_CHECK("edge_row_scalar_kernel");
    return HGNN_OK;
  }
  // lanes per row: about one 8-element vector per lane for the mean row (rowsum over an edge-id map
  // walks one non-zero per lane instead)
  // (with a plan that lists the longer rows for the tiers below: the mean over the rows it does not list, which on
  // a power-law graph is far below the mean over all rows)
  double mean_len = double(g->nnz) / double(g->nrows > 0 ? g->nrows : 1);
  if (p && p->n_mid + p->n_big > 0 && int64_t(p->n_mid) + p->n_big < g->nrows / 2)  // the listed rows are the exception
    mean_len = double(g->nnz - p->listed_nnz) / double(g->nrows - p->n_mid - p->n_big);
  const double per_row = mean_len * ((OP == kSum && a.eid) ? 1.0 : H / 8.0);
  int LR = 4;
  while (LR < kWave && LR < per_row) LR <<= 1;
  const int big = (p && p->n_big > 0) ? p->big_deg : 0;
  a.big_row = p ? p->big_row : nullptr;
  // tier 1: sub-wave teams take the rows they can hold in registers; tier 2: a whole wave per row
  // for the rows between that and the plan's long-row threshold; tier 3: the long rows in chunks.
  int t1 = (OP == kSum && a.eid) ? LR * 4 : LR * 8 * kKeepVec / H;
  // a plan lists the rows between its mid and long thresholds: the wave-per-row tier then walks that list
  // instead of starting a wave for every row of the graph only to find most of them done
  const bool mid_list = p && LR < kWave && (big == 0 || big > p->mid_deg);
  if (mid_list && t1 < p->mid_deg) t1 = p->mid_deg;  // the sub-wave tier takes what the list leaves out
  for (int tier = 0; tier < 2; ++tier) {
    const int lr = tier == 0 ? LR : kWave;
    if (tier == 1 && (LR == kWave || (big > 0 && t1 >= big))) break;
    a.skip_below = tier == 0 ? -1 : t1;
    a.skip_above = (tier == 0 && LR < kWave) ? (big > 0 && big < t1 ? big : t1) : big;
    int64_t nrows_tier = g->nrows;
    a.row_list = nullptr;
    a.n_list = 0;
    if (tier == 1 && mid_list) {
      if (p->n_mid == 0) break;
      a.row_list = p->mid_row;
      a.n_list = p->n_mid;
      nrows_tier = p->n_mid;
    }
    dim3 grid(unsigned(ceil_div(nrows_tier, int64_t(kTeamThreads / kWave) * (kWave / lr))));
    switch (H) {
      case 1: launch_team_h<OP, 1>(lr, grid, s, a); break;
      case 2: launch_team_h<OP, 2>(lr, grid, s, a); break;
      case 4: launch_team_h<OP, 4>(lr, grid, s, a); break;
      default: launch_team_h<OP, 8>(lr, grid, s, a); break;
    }
    HGNN_LAUNCH_CHECK("edge_row_team_kernel");
  }
  if (big > 0) {
    const HubChunks c{p->hub_chunk_row, p->hub_chunk_first, p->hub_chunk_count, p->hub_part};
    dim3 gc(unsigned(p->n_hub_chunks));
    switch (H) {
      case 1: edge_hub_partial_kernel<OP, 1><<<gc, kHubThreads, 0, s>>>(a, c); break;
      case 2: edge_hub_partial_kernel<OP, 2><<<gc, kHubThreads, 0, s>>>(a, c); break;
      case 4: edge_hub_partial_kernel<OP, 4><<<gc, kHubThreads, 0, s>>>(a, c); break;
      default: edge_hub_partial_kernel<OP, 8><<<gc, kHubThreads, 0, s>>>(a, c); break;
    }
    HGNN_LAUNCH_CHECK("edge_hub_partial_kernel");
    if (OP == kSum) {
      edge_hub_rowsum_kernel<<<dim3(unsigned(ceil_div(int64_t(p->n_big) * H, kBlock))), kBlock, 0, s>>>(a, c, p->big_first,
                                                                                                       p->n_big);
      HGNN_LAUNCH_CHECK("edge_hub_rowsum_kernel");
    } else {
      switch (H) {
        case 1: edge_hub_emit_kernel<OP, 1><<<gc, kHubThreads, 0, s>>>(a, c); break;
        case 2: edge_hub_emit_kernel<OP, 2><<<gc, kHubThreads, 0, s>>>(a, c); break;
        case 4: edge_hub_emit_kernel<OP, 4><<<gc, kHubThreads, 0, s>>>(a, c); break;
        default: edge_hub_emit_kernel<OP, 8><<<gc, kHubThreads, 0, s>>>(a, c); break;
      }
      HGNN_LAUNCH_CHECK("edge_hub_emit_kernel");
    }
  }
  return HGNN_OK;
}

// column-blocked row sums: out[i] = sum over the blocks of their fp32 partial sums
__global__ __launch_bounds__(kBlock) void rowsum_block_sum_kernel(const float* __restrict__ part, int nb, int64_t n,
                                                                   half_t* __restrict__ out) {
  const int64_t i = int64_t(blockIdx.x) * kBlock + threadIdx.x;
  if (i >= n) return;
  float s = 0.f;
  for (int b = 0; b < nb; ++b) s += part[int64_t(b) * n + i];
  out[i] = half_t(s);
}

static hgnn_status edge_rows_common(const char* who, const hgnn_csr* g, const hgnn_plan* p, int H, bool allow_eid) {
  hgnn_status st = check_csr_args(g, who);
  if (st != HGNN_OK) return st;
  HGNN_REQUIRE(H >= 1, HGNN_EINVAL, "%s: H = %d must be positive", who, H);
  HGNN_REQUIRE(allow_eid || g->eid == nullptr, HGNN_EUNSUPPORTED, "%s: an edge-id map is not supported here", who);
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
  hgnn_status st = edge_rows_common("hgnn_edge_softmax", g, p, H, false);
  if (st != HGNN_OK) return st;
  if (g->nnz == 0 || g->nrows == 0) return HGNN_OK;
  HGNN_REQUIRE(e && alpha, HGNN_EINVAL, "hgnn_edge_softmax: e or alpha is NULL");
  EdgeRowArgs a{};
  a.rowptr = g->rowptr;
  a.x0 = reinterpret_cast<const half_t*>(e);
  a.out = reinterpret_cast<half_t*>(alpha);
  a.total = g->nnz * H;
  a.nrows = g->nrows;
  a.H = H;
  return launch_edge_rows<kFwd>(g, p, a, static_cast<hipStream_t>(stream));
}

hgnn_status hgnn_edge_softmax_bwd(const hgnn_csr* g, const hgnn_plan* p, int32_t H, const hgnn_half* alpha,
                                  const hgnn_half* dalpha, const hgnn_half* e, float neg_slope, hgnn_half* de,
                                  void* stream) {
  clear_error();
  hgnn_status st = edge_rows_common("hgnn_edge_softmax_bwd", g, p, H, false);
  if (st != HGNN_OK) return st;
  if (g->nnz == 0 || g->nrows == 0) return HGNN_OK;
  HGNN_REQUIRE(alpha && dalpha && de, HGNN_EINVAL, "hgnn_edge_softmax_bwd: alpha, dalpha or de is NULL");
  EdgeRowArgs a{};
  a.rowptr = g->rowptr;
  a.x0 = reinterpret_cast<const half_t*>(alpha);
  a.x1 = reinterpret_cast<const half_t*>(dalpha);
  a.x2 = reinterpret_cast<const half_t*>(e);
  a.out = reinterpret_cast<half_t*>(de);
  a.total = g->nnz * H;
  a.nrows = g->nrows;
  a.H = H;
  a.slope = neg_slope;
  return launch_edge_rows<kBwd>(g, p, a, static_cast<hipStream_t>(stream));
}

hgnn_status hgnn_edge_rowsum(const hgnn_csr* g, const hgnn_plan* p, int32_t H, const hgnn_half* t, hgnn_half* out,
                             void* stream) {
  clear_error();
  hgnn_status st = edge_rows_common("hgnn_edge_rowsum", g, p, H, true);
  if (st != HGNN_OK) return st;
  if (g->nrows == 0) return HGNN_OK;
  HGNN_REQUIRE(out != nullptr && (g->nnz == 0 || t != nullptr), HGNN_EINVAL, "hgnn_edge_rowsum: t or out is NULL");
  EdgeRowArgs a{};
  a.rowptr = g->rowptr;
  a.eid = g->eid;
  a.x0 = reinterpret_cast<const half_t*>(t);
  a.out = reinterpret_cast<half_t*>(out);
  a.total = g->nnz * H;
  a.nrows = g->nrows;
  a.H = H;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (!(p && p->nb > 1 && g->eid && p->block_eid && H <= p->max_H && g->nnz > 0)) return launch_edge_rows<kSum>(g, p, a, s);
  // column-blocked plan of a graph with an edge-id map (the transposed view): the slots a block reads
  // lie in one contiguous part of the edge tensor, so block after block the random reads stay cache
  // resident; fp32 partial sums per block, then one pass adds them
  const int64_t nout = int64_t(g->nrows) * H;
  for (int b = 0; b < p->nb; ++b) {
    hgnn_csr view{g->nrows, g->ncols, p->boff[size_t(b) + 1] - p->boff[size_t(b)],
                  p->brp + size_t(b) * (size_t(g->nrows) + 1), p->bcol + p->boff[size_t(b)], nullptr,
                  p->beid + p->boff[size_t(b)]};
    EdgeRowArgs ab = a;
    ab.rowptr = view.rowptr;
    ab.eid = view.eid;
    ab.out_f32 = p->bsum + size_t(b) * size_t(nout);
    st = launch_edge_rows<kSum>(&view, nullptr, ab, s);
    if (st != HGNN_OK) return st;
  }
  rowsum_block_sum_kernel<<<dim3(unsigned(ceil_div(nout, kBlock))), kBlock, 0, s>>>(p->bsum, p->nb, nout, a.out);
  HGNN_LAUNCH_CHECK("rowsum_block_sum_kernel");
  return HGNN_OK;
}

}  // extern "C"
