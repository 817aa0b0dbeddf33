// fp16 CSR SpMM for gfx950 (wave64): the vertex-parallel kernel behind hgnn_spmm and the
// edge-parallel discretized-reduction kernels behind hgnn_spmm_discretized
// (paper sections 2.1.2, 4.1, 5.2).
//
// Lane mapping (the wave64 form of the paper's sub-warps, section 4.1): a feature row of F
// halves is covered by L = pow2 >= F/8 lanes that load 16 bytes (8 halves) each, so a wave
// holds G = 64/L such groups and touches G different neighbour rows per load instruction.
// Products are formed and accumulated in fp32 (v_fma_mix), fp16 only when a value is stored.
#include "common.h"

#include <algorithm>
#include <climits>

namespace hgnn {

struct SpmmArgs {
  const int* rowptr;
  const int* deg_rowptr;  // offset array that defines deg(i) for MEAN (the whole graph's, also when a column block runs)
  const int* col;
  const int* eid;
  const int* delta;  // column blocks of a graph without edge-id map: slot of non-zero k of row r = k + delta[r]
  const half_t* w;  // [nnz][H] or nullptr
  const half_t* X;
  half_t* Y;
  const float* row_scale;
  int64_t ldx, ldy;
  int64_t nnz;
  int nrows;
  int F, H, D;
  int reduce;
  float one;  // 1.0f
  int rows_per_wave;  // spmm_row_kernel: rows a wave owns, 1 or 64/L
  int long_row;       // plan-free kernels: rows longer than this go to the chunked hub kernels
  // fused scaling and epilogue (discretized kernels): Y = self_coef*self + sum of partials, every partial
  // = agg_coef * s_i * sum_batch w * col_scale[j] * x_j
  const float* col_scale;  // [ncols] or nullptr
  const half_t* self;      // [nrows][ld_self] or nullptr
  int64_t ld_self;
  float self_coef, agg_coef;
  // discretized kernels
  int S;
  int64_t nseg;
  const int* seg_lo;  // row of the first / last edge of every segment
  const int* seg_hi;
  half_t* staging;  // [2*nseg][stage_ld]
  int stage_ld;
  const int* split_row;
  const int* split_lo;
  const int* split_hi;
  int n_split;
  int atomic_y;  // 1: conflicting pieces are added to Y with packed fp16 atomics instead of being staged (comparison variant)
  // all column blocks of a plan in one launch: workgroups are numbered block after block (they are dispatched in that
  // order, so the compute units still gather from one slice of X at a time, without a drain between the blocks)
  const hgnn_seg_block* blocks;  // nullptr: the arrays above describe the one graph of the launch
  int nblocks;
  int use_eid;             // the call's graph has an edge-id map: slots through the blocks' copy of it, else through delta
  int64_t block_y_stride;  // halves between the blocks' partial outputs
};

// Finds the block of workgroup `wg` when blocks are walked in one launch (per block cnt(b) workgroups, at least one
// so that an empty block still zero-fills its partial output), rewrites `a` to that block's arrays and returns the
// workgroup's number inside the block; wg_count receives the block's workgroup count.
template <class Count>
__device__ __forceinline__ int64_t enter_block(SpmmArgs& a, int64_t wg, int64_t& wg_count, Count cnt) {
  int b = 0;
  int64_t first = 0;
  for (;;) {
    const int64_t c = cnt(a.blocks[b]);
    if (wg < first + c || b + 1 == a.nblocks) {
      wg_count = c;
      break;
    }
    first += c;
    ++b;
  }
  const hgnn_seg_block& B = a.blocks[b];
  a.rowptr = B.rowptr;
  a.col = B.col;
  a.eid = a.use_eid ? B.eid : nullptr;
  a.delta = a.use_eid ? nullptr : B.delta;
  a.seg_lo = B.seg_lo;
  a.seg_hi = B.seg_hi;
  a.staging = reinterpret_cast<half_t*>(B.staging);
  a.split_row = B.split_row;
  a.split_lo = B.split_lo;
  a.split_hi = B.split_hi;
  a.nnz = B.nnz;
  a.nseg = B.nseg;
  a.n_split = B.n_split;
  a.Y += int64_t(b) * a.block_y_stride;
  return wg - first;
}

__device__ __forceinline__ float scale_of(const SpmmArgs& a, int r) {
  float s = 1.f;
  if (a.reduce == HGNN_MEAN) {
    int d = a.deg_rowptr[r + 1] - a.deg_rowptr[r];
    s = 1.f / float(d > 1 ? d : 1);
  }
  if (a.row_scale) s *= a.row_scale[r];
  return s * a.agg_coef;
}

__device__ __forceinline__ void store8(half_t* p, const float (&v)[8], float s) {
  half8_t h;
#pragma unroll
  for (int i = 0; i < 8; ++i) h[i] = half_t(v[i] * s);
  *reinterpret_cast<half8_t*>(p) = h;
}

// Y[row, f0..f0+7] = self_coef * self[row] + s * v  (the self term only when the call carries one)
__device__ __forceinline__ void store_row(const SpmmArgs& a, int64_t row, int f0, const float (&v)[8], float s) {
  half8_t h;
  if (a.self) {
    const half8_t sv = *reinterpret_cast<const half8_t*>(a.self + row * a.ld_self + f0);
#pragma unroll
    for (int i = 0; i < 8; ++i) h[i] = half_t(fmaf(a.self_coef, float(sv[i]), v[i] * s));
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) h[i] = half_t(v[i] * s);
  }
  half_t* y = a.Y + row * a.ldy + f0;
  if (f0 + 8 <= a.F) {
    __builtin_nontemporal_store(h, reinterpret_cast<half8_t*>(y));
  } else {  // F is not a multiple of 8: the last lane of a row owns fewer than 8 features
#pragma unroll
    for (int i = 0; i < 8; ++i)
      if (f0 + i < a.F) y[i] = h[i];
  }
}

__device__ __forceinline__ void fma8(float (&acc)[8], float w, const half8_t& x) {
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = fmaf(w, float(x[i]), acc[i]);
}

// p[0..7] += v with four packed fp16 atomic adds (the conflict-write scheme the paper removes, section 5.2.3)
__device__ __forceinline__ void atomic_add8(half_t* p, const float (&v)[8], int nvalid) {
  typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    if (2 * q >= nvalid) break;  // F is even, so a pair is valid as a whole
    half2_t h;
    h[0] = half_t(v[2 * q]);
    h[1] = half_t(v[2 * q + 1]);
    (void)__builtin_amdgcn_flat_atomic_fadd_v2f16(reinterpret_cast<half2_t*>(p) + q, h);
  }
}

// ---------------------------------------------------------------------------------------------------
// Vertex-parallel SpMM (no plan).  A wave owns G = 64/L consecutive rows.  Rows of at most kShortRow
// non-zeros are reduced by one lane group each, all G of them at once and with no exchange between
// lanes; every longer row is reduced by the whole wave, the groups striding over its non-zeros
// and their fp32 partial vectors added across groups with lane shuffles.  Rows longer than
// the hub threshold (SpmmArgs::long_row) are hubs: they are left to the chunked kernels further down.
// ---------------------------------------------------------------------------------------------------
constexpr int kShortRow = 32;
constexpr int kLongRowMin = 256, kLongRowMax = 1024;  // the hub threshold is 8 * mean row length within these, see hgnn_spmm

// acc += sum over the non-zeros k = first, first + STRIDE, ... < end of w_k * X[col_k, f0..f0+7],
// U of them in flight at a time; the column ids of the next U are fetched while the rows of
// the current U are on their way, so one trip through the loop costs one memory latency, not two
template <int STRIDE, bool HAS_W, int U>
__device__ __forceinline__ void edges_accumulate(const SpmmArgs& a, int first, int end, int f0c, int head,
                                                 float (&acc)[8]) {
  int c[U];
#pragma unroll
  for (int u = 0; u < U; ++u) c[u] = first + u * STRIDE < end ? a.col[first + u * STRIDE] : 0;
  for (int k = first; k < end; k += STRIDE * U) {
    half8_t x[U];
    float wv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int kk = k + u * STRIDE;
      x[u] = half8_t(0);
      wv[u] = 0.f;
      if (kk < end) {
        x[u] = *reinterpret_cast<const half8_t*>(a.X + int64_t(c[u]) * a.ldx + f0c);
        if (HAS_W) {
          const int64_t slot = a.eid ? a.eid[kk] : kk;
          wv[u] = float(a.w[slot * a.H + head]);
        } else {
          wv[u] = a.one;
        }
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int kn = k + (U + u) * STRIDE;
      c[u] = kn < end ? a.col[kn] : 0;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) fma8(acc, wv[u], x[u]);
  }
}

// every lane ends up with the sum of its feature slice over the wave's G groups
template <int L>
__device__ __forceinline__ void groups_reduce(float (&acc)[8]) {
#pragma unroll
  for (int off = L; off < kWave; off <<= 1) {
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] += __shfl_xor(acc[i], off);
  }
}

// the rows of workgroup `wg` (of blockDim.x / 64 waves)
template <int L, bool HAS_W>
__device__ __forceinline__ void spmm_row_body(const SpmmArgs& a, int64_t wg) {
  constexpr int G = kWave / L;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int g = lane / L, l = lane % L;
  const int rw = a.rows_per_wave;  // 1 or G
  const int64_t r0 = (wg * (int(blockDim.x) / kWave) + wave) * rw;
  if (r0 >= a.nrows) return;
  const int f0 = 8 * l;
  const bool active = f0 < a.F;
  const int f0c = active ? f0 : 0;
  const int head = f0c / a.D;
  // the group's own row
  const int64_t rg = r0 + g;
  const bool has_row = g < rw && rg < a.nrows;
  int beg_g = 0, end_g = 0;
  if (has_row) {
    beg_g = a.rowptr[rg];
    end_g = a.rowptr[rg + 1];
  }
  if (has_row && end_g - beg_g <= kShortRow) {
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    edges_accumulate<1, HAS_W, 4>(a, beg_g, end_g, f0c, head, acc);
    if (active) store_row(a, rg, f0, acc, scale_of(a, int(rg)));
  }
  // the wave's mid-length rows, one after the other
  for (int j = 0; j < rw; ++j) {
    const int beg = __shfl(beg_g, j * L), end = __shfl(end_g, j * L);
    if (end - beg <= kShortRow || end - beg > a.long_row) continue;  // done above / a hub
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    edges_accumulate<G, HAS_W, 4>(a, beg + g, end, f0c, head, acc);
    groups_reduce<L>(acc);
    if (g == 0 && active) store_row(a, r0 + j, f0, acc, scale_of(a, int(r0 + j)));
  }
}

template <int L, bool HAS_W>
__global__ __launch_bounds__(kBlock) void spmm_row_kernel(SpmmArgs a) {
  spmm_row_body<L, HAS_W>(a, blockIdx.x);
}

// Hubs.  A row longer than the hub threshold is cut into chunks of kHubChunk non-zeros, one wave per chunk,
// so that a hub of 10^5 edges keeps dozens of compute units busy instead of one.  Three
// launches: hub_scan_kernel lists the hubs and hands every one a run of consecutive chunk slots
// (the slot numbers depend on the order in which the atomic counter is reached, the values
// computed do not); spmm_hub_kernel reduces one chunk per wave into an fp32 partial row in
// scratch memory; spmm_hub_sum_kernel adds a hub's partial rows in chunk order and stores the row.
// No atomics touch feature data and the summation order is fixed.
constexpr int kHubChunk = 512;
constexpr int kHubGrid = 131072;  // single-wave workgroups walking the chunk list with a grid stride (with 16384 of them the
                                  // plain SpMM of a 62 M-edge power-law graph took 5 % longer; an idle launch costs 25 us)

struct HubLists {
  int* count;      // [0] chunks handed out, [1] hubs listed
  int* chunk_row;  // [max_chunks] the hub a chunk slot belongs to
  int* chunk_no;   // [max_chunks] its number within the hub
  int* hub_row;    // [max_hubs]
  int* hub_base;   // [max_hubs] first chunk slot of the hub
  float* part;     // [max_chunks][F rounded up to a multiple of 8]
  int max_chunks, max_hubs;
};

__global__ __launch_bounds__(kBlock) void hub_zero_kernel(HubLists h) {
  if (threadIdx.x < 2) h.count[threadIdx.x] = 0;
}

constexpr int kScanRows = 16;  // rows per thread in hub_scan_kernel

// A workgroup looks at kBlock * kScanRows rows, adds up what its hubs need in LDS and reserves it with one
// pair of atomic adds (thousands of single adds on one address would take longer than the SpMM of a small graph).
__global__ __launch_bounds__(kBlock) void hub_scan_kernel(SpmmArgs a, HubLists h) {
  __shared__ int s_chunks[kBlock], s_hubs[kBlock];
  __shared__ int s_base[2];
  const int64_t r0 = int64_t(blockIdx.x) * (kBlock * kScanRows);
  int my_chunks = 0, my_hubs = 0;
  for (int u = 0; u < kScanRows; ++u) {
    const int64_t r = r0 + u * kBlock + threadIdx.x;
    if (r >= a.nrows) break;
    const int deg = a.rowptr[r + 1] - a.rowptr[r];
    if (deg > a.long_row) {
      my_chunks += (deg + kHubChunk - 1) / kHubChunk;
      ++my_hubs;
    }
  }
  s_chunks[threadIdx.x] = my_chunks;
  s_hubs[threadIdx.x] = my_hubs;
  __syncthreads();
  // inclusive scan over the workgroup (Hillis-Steele; kBlock is small)
  for (int off = 1; off < kBlock; off <<= 1) {
    const int c = int(threadIdx.x) >= off ? s_chunks[threadIdx.x - off] : 0;
    const int n = int(threadIdx.x) >= off ? s_hubs[threadIdx.x - off] : 0;
    __syncthreads();
    s_chunks[threadIdx.x] += c;
    s_hubs[threadIdx.x] += n;
    __syncthreads();
  }
  if (threadIdx.x == kBlock - 1) {
    s_base[0] = s_chunks[kBlock - 1] > 0 ? atomicAdd(&h.count[0], s_chunks[kBlock - 1]) : 0;
    s_base[1] = s_hubs[kBlock - 1] > 0 ? atomicAdd(&h.count[1], s_hubs[kBlock - 1]) : 0;
  }
  __syncthreads();
  if (my_hubs == 0) return;
  int base = s_base[0] + s_chunks[threadIdx.x] - my_chunks;
  int i = s_base[1] + s_hubs[threadIdx.x] - my_hubs;
  for (int u = 0; u < kScanRows; ++u) {
    const int64_t r = r0 + u * kBlock + threadIdx.x;
    if (r >= a.nrows) break;
    const int deg = a.rowptr[r + 1] - a.rowptr[r];
    if (deg <= a.long_row) continue;
    const int nch = (deg + kHubChunk - 1) / kHubChunk;
    if (base + nch <= h.max_chunks && i < h.max_hubs) {  // always true for a valid rowptr
      h.hub_row[i] = int(r);
      h.hub_base[i] = base;
      for (int c = 0; c < nch; ++c) {
        h.chunk_row[base + c] = int(r);
        h.chunk_no[base + c] = c;
      }
    }
    base += nch;
    ++i;
  }
}

// one wave per chunk, single-wave workgroups walking the chunk list with a grid stride
// the chunks first, first + stride, ... of the list, one wave
template <int L, bool HAS_W>
__device__ __forceinline__ void spmm_hub_body(const SpmmArgs& a, const HubLists& h, int64_t first, int64_t stride) {
  constexpr int G = kWave / L;
  const int nchunks = h.count[0] < h.max_chunks ? h.count[0] : h.max_chunks;
  const int lane = threadIdx.x;
  const int g = lane / L, l = lane % L;
  const int f0 = 8 * l;
  const bool active = f0 < a.F;
  const int f0c = active ? f0 : 0;
  const int pitch = (a.F + 7) & ~7;
  for (int64_t c = first; c < nchunks; c += stride) {
    const int row = h.chunk_row[c];
    const int row_end = a.rowptr[row + 1];
    const int b = a.rowptr[row] + h.chunk_no[c] * kHubChunk;
    const int e = b + kHubChunk < row_end ? b + kHubChunk : row_end;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    edges_accumulate<G, HAS_W, 4>(a, b + g, e, f0c, f0c / a.D, acc);
    groups_reduce<L>(acc);
    if (g == 0 && active) {
      float* out = h.part + c * pitch + f0;
#pragma unroll
      for (int i = 0; i < 8; ++i) out[i] = acc[i];
    }
  }
}

template <int L, bool HAS_W>
__global__ __launch_bounds__(kWave) void spmm_hub_kernel(SpmmArgs a, HubLists h) {
  spmm_hub_body<L, HAS_W>(a, h, blockIdx.x, gridDim.x);
}

// Rows and hub chunks in one launch of single-wave workgroups: the row workgroups first, then hub_wgs workgroups that
// walk the chunk list.  Neither kind of work depends on the other (the lists are there when the launch begins), so
// the chunks start while the last rows are still being reduced instead of waiting for the row kernel to drain:
// 1 % on a 62 M-edge power-law graph, 9-14 % on graphs of 2-5 M edges.  The order matters on the large graph:
// chunks first, or chunk walkers spread among the row workgroups, were 8 % slower than rows first.
template <int L, bool HAS_W>
__global__ __launch_bounds__(kWave) void spmm_row_hub_kernel(SpmmArgs a, HubLists h, int hub_wgs) {
  const int64_t bid = blockIdx.x;
  const int64_t row_wgs = int64_t(gridDim.x) - hub_wgs;
  if (bid < row_wgs) spmm_row_body<L, HAS_W>(a, bid);
  else spmm_hub_body<L, HAS_W>(a, h, bid - row_wgs, hub_wgs);
}

// one wave per hub; its groups stride over the hub's partial rows
template <int L>
__global__ __launch_bounds__(kBlock) void spmm_hub_sum_kernel(SpmmArgs a, HubLists h) {
  constexpr int G = kWave / L;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int g = lane / L, l = lane % L;
  const int nhubs = h.count[1] < h.max_hubs ? h.count[1] : h.max_hubs;
  const int i = int(blockIdx.x) * kWavesPerBlock + wave;
  if (i >= nhubs) return;
  const int f0 = 8 * l;
  const bool active = f0 < a.F;
  const int f0c = active ? f0 : 0;
  const int row = h.hub_row[i];
  const int nch = (a.rowptr[row + 1] - a.rowptr[row] + kHubChunk - 1) / kHubChunk;
  const int pitch = (a.F + 7) & ~7;
  const float* part = h.part + int64_t(h.hub_base[i]) * pitch + f0c;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int c = g; c < nch; c += G) {
    const float4 lo = *reinterpret_cast<const float4*>(part + int64_t(c) * pitch);
    const float4 hi = *reinterpret_cast<const float4*>(part + int64_t(c) * pitch + 4);
    acc[0] += lo.x, acc[1] += lo.y, acc[2] += lo.z, acc[3] += lo.w;
    acc[4] += hi.x, acc[5] += hi.y, acc[6] += hi.z, acc[7] += hi.w;
  }
  groups_reduce<L>(acc);
  if (g == 0 && active) store_row(a, row, f0, acc, scale_of(a, row));
}

// ---------------------------------------------------------------------------------------------------
// Column passes of the plan-free SpMM.  Where the feature table misses the L2s but rows are long (hundreds of
// non-zeros), waves that each sweep their own row from its first column to its last are spread all over the table at
// any moment and share little in the L2s.  The passes align them: the columns are cut into npass equal ranges and
// the launch walks pass after pass (workgroups are numbered pass-major and dispatched in that order), a wave reducing
// the piece of its row that falls into the pass's range -- contiguous, because columns ascend inside a row -- into an
// fp32 partial row in the caller's workspace; one more kernel adds a row's npass partials in pass order, scales and
// rounds once.  Same arithmetic as one sweep (fp32 sums, one rounding), fixed summation order, no atomics.
// ---------------------------------------------------------------------------------------------------
constexpr int kPassLongRow = 16384;  // rows beyond this still go to the hub kernels

// First position p of [lo, hi) with col[p] >= key (hi if there is none), found by all 64 lanes of a wave together; every
// lane passes the same arguments and receives the same answer: 64 evenly spaced samples narrow the range 64-fold per
// step.  Reads stay inside [lo, hi) whatever the entries hold (an unsorted row gives a wrong cut, never a position
// outside the row).
__device__ __forceinline__ int wave_lower_bound(const int* __restrict__ col, int lo, int hi, int64_t key, int lane) {
  while (hi - lo > kWave) {
    const int n = hi - lo;
    const int v = col[lo + int((int64_t(lane) * n) >> 6)];
    const int cnt = __popcll(__ballot(int64_t(v) < key));
    if (cnt == 0) return lo;
    const int nlo = lo + int((int64_t(cnt - 1) * n) >> 6) + 1;
    const int nhi = cnt == kWave ? hi : lo + int((int64_t(cnt) * n) >> 6);
    lo = nlo;
    hi = nhi;
  }
  const int v = lo + lane < hi ? col[lo + lane] : INT_MAX;
  return lo + __popcll(__ballot(int64_t(v) < key));
}

constexpr int kMaxPasses = 16;

// cuts[r*(npass+1) + b] = first CSR position of row r whose column is >= b*width (b = npass: end of the row).
// One wave per row.  Every border is first looked for in a window of 64 entries around the place that an even spread
// of the columns over the row would give it; the windows of all borders are loaded together, so a row whose borders
// lie inside them costs one memory latency after its offsets.  A border outside its window is searched in the part
// of the row that the window rules in.
__global__ __launch_bounds__(kBlock) void row_cuts_kernel(const int* __restrict__ rowptr, const int* __restrict__ col,
                                                           int nrows, int ncols, int npass, int width, int long_row,
                                                           int* __restrict__ cuts) {
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int64_t r = int64_t(blockIdx.x) * kWavesPerBlock + wave;
  if (r >= nrows) return;
  const int beg = rowptr[r], end = rowptr[r + 1];
  const int n = end - beg;
  int* out = cuts + r * (npass + 1);
  if (n == 0 || n > long_row) {  // nothing to cut / a hub: its passes are empty
    if (lane <= npass) out[lane] = lane == npass && n <= long_row ? end : beg;
    return;
  }
  int wlo[kMaxPasses], v[kMaxPasses];
#pragma unroll
  for (int b = 1; b < kMaxPasses; ++b) {
    wlo[b] = beg;
    v[b] = INT_MAX;
    if (b < npass) {
      int w = beg + int(int64_t(n) * b * width / ncols) - kWave / 2;
      if (w > end - kWave) w = end - kWave;
      if (w < beg) w = beg;
      wlo[b] = w;
      if (w + lane < end) v[b] = col[w + lane];
    }
  }
  int cut = lane == 0 ? beg : end;
#pragma unroll
  for (int b = 1; b < kMaxPasses; ++b) {
    if (b < npass) {
      const int64_t key = int64_t(b) * width;
      const int whi = wlo[b] + kWave < end ? wlo[b] + kWave : end;
      const int cnt = __popcll(__ballot(int64_t(v[b]) < key));
      int c;
      if (cnt > 0 && cnt < whi - wlo[b]) c = wlo[b] + cnt;                          // inside the window
      else if (cnt == 0) c = wlo[b] == beg ? beg : wave_lower_bound(col, beg, wlo[b], key, lane);  // before it
      else c = whi == end ? end : wave_lower_bound(col, whi, end, key, lane);       // after it
      if (lane == b) cut = c;
    }
  }
  if (lane <= npass) out[lane] = cut;
}

// one single-wave workgroup per (pass, row), pass-major
template <int L, bool HAS_W>
__global__ __launch_bounds__(kWave) void spmm_row_pass_kernel(SpmmArgs a, const int* __restrict__ cuts,
                                                              float* __restrict__ part, int npass) {
  constexpr int G = kWave / L;
  const int lane = threadIdx.x;
  const int g = lane / L, l = lane % L;
  const int b = int(blockIdx.x / unsigned(a.nrows));
  const int64_t r = blockIdx.x % unsigned(a.nrows);
  const int f0 = 8 * l;
  const bool active = f0 < a.F;
  const int f0c = active ? f0 : 0;
  const int beg = cuts[r * (npass + 1) + b], end = cuts[r * (npass + 1) + b + 1];
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  edges_accumulate<G, HAS_W, 4>(a, beg + g, end, f0c, f0c / a.D, acc);
  groups_reduce<L>(acc);
  if (g == 0 && active) {
    const int pitch = (a.F + 7) & ~7;
    float* out = part + (int64_t(b) * a.nrows + r) * pitch + f0;
    *reinterpret_cast<float4*>(out) = make_float4(acc[0], acc[1], acc[2], acc[3]);
    *reinterpret_cast<float4*>(out + 4) = make_float4(acc[4], acc[5], acc[6], acc[7]);
  }
}

// a lane group per row: adds the row's partials in pass order and stores the row (hubs are left to spmm_hub_sum_kernel)
template <int L>
__global__ __launch_bounds__(kBlock) void spmm_pass_sum_kernel(SpmmArgs a, const float* __restrict__ part, int npass) {
  constexpr int G = kWave / L;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int g = lane / L, l = lane % L;
  const int64_t r = (int64_t(blockIdx.x) * kWavesPerBlock + wave) * G + g;
  const int f0 = 8 * l;
  if (r >= a.nrows || f0 >= a.F) return;
  if (a.rowptr[r + 1] - a.rowptr[r] > a.long_row) return;
  const int pitch = (a.F + 7) & ~7;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int b = 0; b < npass; ++b) {
    const float* p = part + (int64_t(b) * a.nrows + r) * pitch + f0;
    const float4 lo = *reinterpret_cast<const float4*>(p);
    const float4 hi = *reinterpret_cast<const float4*>(p + 4);
    acc[0] += lo.x, acc[1] += lo.y, acc[2] += lo.z, acc[3] += lo.w;
    acc[4] += hi.x, acc[5] += hi.y, acc[6] += hi.z, acc[7] += hi.w;
  }
  store_row(a, r, f0, acc, scale_of(a, int(r)));
}

// Scalar path for shapes the 16-byte path cannot take: one thread per (row, feature).
__global__ __launch_bounds__(kBlock) void spmm_scalar_kernel(SpmmArgs a) {
  const int64_t idx = int64_t(blockIdx.x) * kBlock + threadIdx.x;
  if (idx >= int64_t(a.nrows) * a.F) return;
  const int row = int(idx / a.F), f = int(idx % a.F);
  const int head = f / a.D;
  float acc = 0.f;
  for (int k = a.rowptr[row]; k < a.rowptr[row + 1]; ++k) {
    float wv = 1.f;
    if (a.w) {
      const int64_t slot = a.eid ? a.eid[k] : k;
      wv = float(a.w[slot * a.H + head]);
    }
    acc = fmaf(wv, float(a.X[int64_t(a.col[k]) * a.ldx + f]), acc);
  }
  a.Y[int64_t(row) * a.ldy + f] = half_t(acc * scale_of(a, row));
}

// ---------------------------------------------------------------------------------------------------
// Discretized-reduction SpMM, pass 1 (section 5.2): one wave per segment of S edges.
//  phase 1  the wave loads the segment's column ids and edge values once, coalesced, into LDS
//           (the two-phase load of section 4.1; LDS reads broadcast to a group) and derives the
//           row id of every edge from the offset array: the rows seg_row_lo..seg_row_hi mark
//           their first edge in LDS and a wave-wide running maximum spreads the ids.  No per-edge
//           row array is read from memory.
//  phase 2  group g walks its contiguous chunk of the segment, four edges per step, with a
//           running reduction; a row piece that starts and ends inside the chunk is scaled and
//           stored straight to Y;
//  merge    pieces that touch a chunk border are parked in LDS (fp32, scaled) and group 0 sews
//           them together in order: rows that lie inside the segment are stored to Y, the piece
//           entering from the previous segment and the piece leaving into the next go to the
//           staging buffer as fp16 (each covers at most S edges, so it cannot overflow where
//           S * max|w x| fits fp16).  No atomics; every Y row has exactly one writer.
// The wave also zero-fills its share of the empty rows.
// ---------------------------------------------------------------------------------------------------
__host__ __device__ inline int align16i(int v) { return (v + 15) & ~15; }

struct SegLds {
  int per;   // LDS entries per lane (multiple of 4); the padded segment holds 64*per edges
  int spad;
  int col_off, row_off, blk_off, w_off, vec_off, flag_off, total;
};
// wm: 0 = no per-edge factor, 1 = fp16 edge values, 2 = fp32 factor (edge value times column scale)
__host__ __device__ inline SegLds seg_lds_layout(int S, int H, int wm, int L) {
  SegLds o;
  const int G = kWave / L;
  o.per = 4 * ((S + 255) / 256);  // = seg_slots_per_lane(S)
  o.spad = kWave * o.per;
  o.col_off = 0;
  o.row_off = o.col_off + o.spad * 4;
  o.blk_off = o.row_off + o.spad * 4;
  o.w_off = o.blk_off + align16i(o.spad);  // one int per 4 edges
  o.vec_off = o.w_off + (wm == 0 ? 0 : align16i(o.spad * H * (wm == 2 ? 4 : 2)));
  o.flag_off = o.vec_off + G * 8 * L * 4;  // one parked vector per lane group (the piece that entered its chunk)
  o.total = o.flag_off + align16i(3 * G * 4);
  return o;
}

// Edge values of four staged edges (i0 + q * kWave, q = 0..3) into the LDS table: fp16 as they are (WM == 1) or
// as fp32 factors times the column scale cs (WM == 2; no values: the scale alone).  HV = 1, 2, 4, 8: the H values of
// an edge are read as one vector (H == HV, base aligned to it); HV = 0: any head count, one value at a time.
// All four edges' loads of a level are issued before the first LDS store.
template <int WM, int HV>
__device__ __forceinline__ void seg_stage_values(const SpmmArgs& a, int i0, int n, const int64_t (&slot)[4],
                                                 const float (&cs)[4], half_t* s_w, float* s_wf) {
  const bool have = WM == 1 || a.w != nullptr;
  if (HV == 0) {
    for (int h = 0; h < a.H; ++h) {
      half_t wv[4];
#pragma unroll
      for (int q = 0; q < 4; ++q)
        wv[q] = (i0 + q * kWave < n && have) ? a.w[slot[q] * a.H + h] : half_t(WM == 1 ? 0 : 1);
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int i = i0 + q * kWave;
        if (WM == 1) s_w[i * a.H + h] = wv[q];
        else s_wf[i * a.H + h] = float(wv[q]) * cs[q];
      }
    }
    return;
  }
  constexpr int N = HV > 0 ? HV : 1;
  typedef _Float16 hv_t __attribute__((ext_vector_type(N)));
  hv_t wv[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    wv[q] = hv_t(half_t(WM == 1 ? 0 : 1));
    if (i0 + q * kWave < n && have) wv[q] = *reinterpret_cast<const hv_t*>(a.w + slot[q] * N);
  }
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int i = i0 + q * kWave;
    if (WM == 1) {
      *reinterpret_cast<hv_t*>(s_w + i * N) = wv[q];
    } else {
#pragma unroll
      for (int h = 0; h < N; ++h) s_wf[i * N + h] = float(wv[q][h]) * cs[q];
    }
  }
}

template <int WM>
__device__ __forceinline__ void seg_stage_values_any(const SpmmArgs& a, int i0, int n, const int64_t (&slot)[4],
                                                     const float (&cs)[4], half_t* s_w, float* s_wf) {
  const uintptr_t wa = reinterpret_cast<uintptr_t>(a.w);
  if (a.H == 1) seg_stage_values<WM, 1>(a, i0, n, slot, cs, s_w, s_wf);
  else if (a.H == 4 && (wa & 7u) == 0) seg_stage_values<WM, 4>(a, i0, n, slot, cs, s_w, s_wf);
  else if (a.H == 2 && (wa & 3u) == 0) seg_stage_values<WM, 2>(a, i0, n, slot, cs, s_w, s_wf);
  else if (a.H == 8 && (wa & 15u) == 0) seg_stage_values<WM, 8>(a, i0, n, slot, cs, s_w, s_wf);
  else seg_stage_values<WM, 0>(a, i0, n, slot, cs, s_w, s_wf);
}

// MAPPED = false: the call has no edge-id map (only instantiated for WM == 1, where the code of the map costs the
// registers of a seventh wave per SIMD)
template <int L, int WM, bool OFF32, bool MAPPED = true>
__global__ __launch_bounds__(kBlock, WM == 0 ? 8 : ((WM == 1 && !MAPPED) ? 7 : 1)) void spmm_seg_kernel(SpmmArgs a) {
  constexpr int G = kWave / L;
  constexpr int VEC = 8 * L;  // floats per parked vector
  extern __shared__ __align__(16) unsigned char smem[];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int g = lane / L, l = lane % L;
  const int f0 = 8 * l;
  const bool active = f0 < a.F;
  const int f0c = active ? f0 : 0;  // idle lanes of a group load a valid address and drop the result
  const int head = f0c / a.D;
  const int S = a.S;
  const SegLds lay = seg_lds_layout(S, a.H, WM, L);
  unsigned char* base = smem + size_t(wave) * lay.total;
  int* s_col = reinterpret_cast<int*>(base + lay.col_off);
  int* s_row = reinterpret_cast<int*>(base + lay.row_off);  // row id of every edge of the segment
  int* s_blk = reinterpret_cast<int*>(base + lay.blk_off);  // per 4 edges: their common row id, or -1
  half_t* s_w = reinterpret_cast<half_t*>(base + lay.w_off);   // WM == 1
  float* s_wf = reinterpret_cast<float*>(base + lay.w_off);    // WM == 2
  // A group's piece that entered its chunk from the previous one is parked in LDS when its row ends; the piece that
  // leaves into the next chunk simply stays in the group's registers and is fetched from there by the merge
  // (cross-lane reads need no LDS allocation).  Every KB of LDS less per wave is more waves per compute unit, and
  // this latency-bound gather speeds up almost in proportion.
  float* m_vec = reinterpret_cast<float*>(base + lay.vec_off);  // [G][VEC]: the entering piece of group g
  int* m_flag = reinterpret_cast<int*>(base + lay.flag_off);    // bit0 entering, bit1 runs through, bit2 leaving
  int* m_hrow = m_flag + G;
  int* m_trow = m_hrow + G;

  const int wpb = int(blockDim.x) / kWave;  // waves per workgroup (4, 2 or 1, chosen on the host for LDS packing)
  int64_t wg = blockIdx.x, wg_count = gridDim.x;
  if (a.blocks)
    wg = enter_block(a, wg, wg_count, [&](const hgnn_seg_block& B) {
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

  // ---- phase 1: coalesced stage of column ids and edge values, then the row id of every edge.  spad is a
  // multiple of 4 * kWave; a lane keeps its four loads of a round in flight together (column ids, then the
  // edge-id map, then the values behind it), so a round costs one memory latency per level, not four.
  const bool nt = stream_nontemporal(a.nnz);
  for (int i0 = lane; i0 < spad; i0 += 4 * kWave) {
    int c[4];
    int64_t slot[4] = {0, 0, 0, 0};
    if (nt) stream_load4<true>(a.col + e0, i0, n, c);
    else stream_load4<false>(a.col + e0, i0, n, c);
    if (WM != 0 && !a.delta) {
      if (MAPPED && a.eid) {
        int e[4];
        if (nt) stream_load4<true>(a.eid + e0, i0, n, e);
        else stream_load4<false>(a.eid + e0, i0, n, e);
#pragma unroll
        for (int q = 0; q < 4; ++q) slot[q] = e[q];
      } else {
#pragma unroll
        for (int q = 0; q < 4; ++q) slot[q] = i0 + q * kWave < n ? e0 + i0 + q * kWave : 0;
      }
    }
#pragma unroll
    for (int q = 0; q < 4; ++q)  // OFF32: byte offset of the neighbour's row
      s_col[i0 + q * kWave] = OFF32 ? int(uint32_t(c[q]) * uint32_t(a.ldx) * 2u) : c[q];
    if (WM != 0 && !a.delta) {
      float cs[4] = {1.f, 1.f, 1.f, 1.f};
      if (WM == 2) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const bool in = i0 + q * kWave < n;
          cs[q] = (in && a.col_scale) ? a.col_scale[c[q]] : (in ? 1.f : 0.f);
        }
      }
      seg_stage_values_any<WM>(a, i0, n, slot, cs, s_w, s_wf);
    }
  }
  if (lane < G) m_flag[lane] = 0;
  seg_stage_rows(s_row, s_blk, lane, per, n, row_lo, row_hi, a.rowptr, e0);
  if (WM != 0 && a.delta) {
    // a row piece of a column block is a run of consecutive slots: slot = position + delta[row], so the
    // edge values are read coalesced without an edge-id array (the row ids are known only now)
    for (int i0 = lane; i0 < spad; i0 += 4 * kWave) {  // four in flight per level, as above
      int64_t slot[4];
      float cs[4] = {1.f, 1.f, 1.f, 1.f};
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int i = i0 + q * kWave;
        slot[q] = i < n ? e0 + i + a.delta[s_row[i]] : 0;
      }
      if (WM == 2) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int i = i0 + q * kWave;
          cs[q] = i < n ? (a.col_scale ? a.col_scale[a.col[e0 + i]] : 1.f) : 0.f;
        }
      }
      seg_stage_values_any<WM>(a, i0, n, slot, cs, s_w, s_wf);
    }
    wave_sync();
  }

  // ---- phase 2: running reduction over this group's chunk
  const int C = 4 * ((S + 4 * G - 1) / (4 * G));  // edges per group, a multiple of 4
  const int c0 = g * C < n ? g * C : n;
  const int c1 = c0 + C < n ? c0 + C : n;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  int cur = -1;
  bool lo = false;  // current piece began before this chunk

  // the scale of the current row (1/degree, row factor) is requested when the row begins, so that its latency has
  // passed by the time the row ends; fetched at the flush it would stall the lane group once per row
  float sc = 0.f;
  auto flush = [&](bool ro) {
    if (!lo && !ro) {
      if (active) store_row(a, cur, f0, acc, sc);
    } else if (lo) {
      if (active) {
        float* dst = m_vec + g * VEC + f0;
#pragma unroll
        for (int i = 0; i < 8; ++i) dst[i] = acc[i] * sc;
      }
      if (l == 0) {
        m_flag[g] |= ro ? 3 : 1;
        m_hrow[g] = cur;
      }
    } else {  // leaves into the next chunk (only the last flush of a chunk gets here): stays in acc, scaled
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] *= sc;
      if (l == 0) {
        m_flag[g] |= 4;
        m_trow[g] = cur;
      }
    }
  };
  auto gather = [&](int c) -> half8_t {
    if (OFF32) {  // byte offset in 32 bits: scalar base address + per-lane offset
      const uint32_t boff = uint32_t(c) + uint32_t(f0c) * 2u;
      return *reinterpret_cast<const half8_t*>(reinterpret_cast<const char*>(a.X) + boff);
    }
    return *reinterpret_cast<const half8_t*>(a.X + int64_t(c) * a.ldx + f0c);
  };

  if (c0 < c1) {
    cur = s_row[c0];
    lo = c0 > 0 ? s_row[c0 - 1] == cur : seg_left_open;
    sc = scale_of(a, cur);
  }
  for (int i = c0; i < c1; i += 4) {
    const int4_t cols = *reinterpret_cast<const int4_t*>(s_col + i);
    const int blk = s_blk[i >> 2];
    half8_t x[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) x[u] = gather(cols[u]);
    float wv[4] = {a.one, a.one, a.one, a.one};  // 1.0 the compiler cannot fold: keeps convert+add in one v_fma_mix
    if (WM == 1) {
      if (a.H == 1) {
        const half4_t w4 = *reinterpret_cast<const half4_t*>(s_w + i);
#pragma unroll
        for (int u = 0; u < 4; ++u) wv[u] = float(w4[u]);
      } else {
#pragma unroll
        for (int u = 0; u < 4; ++u) wv[u] = float(s_w[(i + u) * a.H + head]);
      }
    } else if (WM == 2) {
      if (a.H == 1) {
        const float4 w4 = *reinterpret_cast<const float4*>(s_wf + i);
        wv[0] = w4.x;
        wv[1] = w4.y;
        wv[2] = w4.z;
        wv[3] = w4.w;
      } else {
#pragma unroll
        for (int u = 0; u < 4; ++u) wv[u] = s_wf[(i + u) * a.H + head];
      }
    }
    if (blk == cur) {  // the four edges continue the current row: no bookkeeping at all
#pragma unroll
      for (int u = 0; u < 4; ++u) fma8(acc, wv[u], x[u]);
    } else {
      const int4_t rows = *reinterpret_cast<const int4_t*>(s_row + i);
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (i + u < c1) {
          if (rows[u] != cur) {
            flush(false);
#pragma unroll
            for (int q = 0; q < 8; ++q) acc[q] = 0.f;
            cur = rows[u];
            lo = false;
            sc = scale_of(a, cur);
          }
          fma8(acc, wv[u], x[u]);
        }
      }
    }
  }
  if (c0 < c1) flush(c1 < n ? s_row[c1] == cur : seg_right_open);
  wave_sync();

  // ---- merge: group 0 sews the pieces together in chunk order (all lanes take part in the cross-lane reads)
  if (valid) {
    float run[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    bool open = false, from_before = false;
    int run_row = -1;
    const bool me = g == 0 && active;
    for (int gg = 0; gg < G; ++gg) {
      const int fl = m_flag[gg];  // the same value on every lane
      if (fl & 1) {
        if (me) {
          const float* src = m_vec + gg * VEC + f0;
#pragma unroll
          for (int i = 0; i < 8; ++i) run[i] += src[i];
        }
        if (gg == 0) {
          from_before = true;
          open = true;
          run_row = m_hrow[0];
        }
        if (!(fl & 2)) {  // the row ends inside chunk gg
          if (me) {
            if (!from_before) store_row(a, run_row, f0, run, 1.f);
            else if (a.atomic_y) atomic_add8(a.Y + int64_t(run_row) * a.ldy + f0, run, a.F - f0);
            else store8(a.staging + (2 * seg) * a.stage_ld + f0, run, 1.f);
          }
#pragma unroll
          for (int i = 0; i < 8; ++i) run[i] = 0.f;
          open = false;
          from_before = false;
        }
      }
      if (fl & 4) {  // the piece that left chunk gg: from the registers of group gg
#pragma unroll
        for (int i = 0; i < 8; ++i) run[i] = __shfl(acc[i], gg * L + l);
        run_row = m_trow[gg];
        open = true;
        from_before = false;
      }
    }
    if (open && me) {  // leaves into the next segment; a piece that also entered is a "middle" and uses slot 2*seg
      if (a.atomic_y) atomic_add8(a.Y + int64_t(run_row) * a.ldy + f0, run, a.F - f0);
      else store8(a.staging + (2 * seg + (from_before ? 0 : 1)) * a.stage_ld + f0, run, 1.f);
    }
  }

  // ---- zero-fill this wave's share of the empty rows
  const int64_t nw = wg_count * wpb;
  const int rpw = int((a.nrows + nw - 1) / nw);
  const int64_t r0 = wid * rpw;
  const int64_t r1 = r0 + rpw < a.nrows ? r0 + rpw : a.nrows;
  if (active) {
    const float zero[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int64_t r = r0 + g; r < r1; r += G)
      if (a.rowptr[r] == a.rowptr[r + 1]) store_row(a, r, f0, zero, 0.f);
  }
}

// Pass 2, the follow-up kernel (section 5.2.3): adds the staged fp16 partials of every split row
// (fp32, fixed order) and stores the row once.  A wave owns G split rows: a row of at most
// kFinishShort pieces is summed by its own lane group, a hub that spans more segments by the
// whole wave, the groups striding over its pieces.
constexpr int kFinishShort = 8;

// acc += staging rows MUL*k for k = first, first + STRIDE, ... <= last
template <int STRIDE, int MUL = 2>
__device__ __forceinline__ void pieces_accumulate(const SpmmArgs& a, int64_t first, int64_t last, int f0,
                                                  float (&acc)[8]) {
  constexpr int U = 4;
  for (int64_t k = first; k <= last; k += STRIDE * U) {
    half8_t t[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t kk = k + u * STRIDE;
      t[u] = half8_t(0);
      if (kk <= last) t[u] = *reinterpret_cast<const half8_t*>(a.staging + (MUL * kk) * a.stage_ld + f0);
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] += float(t[u][i]);
  }
}

template <int L>
__global__ __launch_bounds__(kBlock) void spmm_finish_kernel(SpmmArgs a) {
  constexpr int G = kWave / L;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int g = lane / L, l = lane % L;
  const int f0 = 8 * l;
  const bool active = f0 < a.F;
  const int f0c = active ? f0 : 0;
  int64_t wg = blockIdx.x, wg_count = gridDim.x;
  if (a.blocks)
    wg = enter_block(a, wg, wg_count,
                     [&](const hgnn_seg_block& B) { return (int64_t(B.n_split) + kWavesPerBlock * G - 1) / (kWavesPerBlock * G); });
  const int64_t i0 = (wg * kWavesPerBlock + wave) * G;
  if (i0 >= a.n_split) return;
  const int64_t idx = i0 + g;
  int r = 0, sa = 0, sb = -1;
  if (idx < a.n_split) {
    r = a.split_row[idx];
    sa = a.split_lo[idx];
    sb = a.split_hi[idx];
  }
  // the tail piece of segment sa, then the head pieces of segments sa+1 .. sb
  if (idx < a.n_split && sb - sa <= kFinishShort) {
    float acc[8];
    const half8_t t = *reinterpret_cast<const half8_t*>(a.staging + (2 * int64_t(sa) + 1) * a.stage_ld + f0c);
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = float(t[i]);
    pieces_accumulate<1>(a, int64_t(sa) + 1, sb, f0c, acc);
    if (active) store_row(a, r, f0, acc, 1.f);
  }
  for (int j = 0; j < G; ++j) {
    const int rj = __shfl(r, j * L), sj = __shfl(sa, j * L), ej = __shfl(sb, j * L);
    if (ej - sj <= kFinishShort) continue;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (g == 0) {
      const half8_t t = *reinterpret_cast<const half8_t*>(a.staging + (2 * int64_t(sj) + 1) * a.stage_ld + f0c);
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] = float(t[i]);
    }
    pieces_accumulate<G>(a, int64_t(sj) + 1 + g, ej, f0c, acc);
    groups_reduce<L>(acc);
    if (g == 0 && active) store_row(a, rj, f0, acc, 1.f);
  }
}

// ---------------------------------------------------------------------------------------------------
// Vertex-parallel variant of the discretized SpMM (section 5.4): a wave reduces one neighbour group,
// at most ng non-zeros of a single row, so there is no row change inside a wave and no merge; what
// is left of the conflict is between the waves that share a long row.  A row with one group is
// stored directly; the groups of a longer row store their scaled fp16 partials in staging slots of
// their own and spmm_vgroup_finish_kernel adds them.  Edge values of a group start at an arbitrary
// position of the edge tensor: with one value per edge they are fetched as aligned pairs, starting
// one position early when the group starts at an odd position, and the pair is taken apart while it
// is copied to LDS.
// ---------------------------------------------------------------------------------------------------
struct VGroupArgs {
  const int* grp_row;
  const int* goff;
  const int* moff;
  int64_t n_groups;
  int ng;
  int pair_loads;  // edge values: one per edge, no edge-id map, 4-byte aligned base
  int acc16;       // products and sums of a lane's chunk in packed fp16 (the paper's arithmetic, section 4.2)
};

__host__ __device__ inline int vgroup_lds_bytes(int ng, int H, bool has_w) {
  const int spad = kWave * 4 * ((ng + 255) / 256);
  return spad * 4 + (has_w ? align16i(spad * H * 2) : 0);
}

// VW = halves per lane and load: 8 (16 bytes), 4 or 2 -- the narrower forms exist for the vector-width
// study (section 6.3.1 carried over to SpMM); a row of F halves then takes L = pow2 >= F/VW lanes.
template <int L, int VW, bool HAS_W, bool OFF32>
__global__ __launch_bounds__(kBlock) void spmm_vgroup_kernel(SpmmArgs a, VGroupArgs v) {
  constexpr int G = kWave / L;
  typedef _Float16 hv_t __attribute__((ext_vector_type(VW)));
  extern __shared__ __align__(16) unsigned char smem[];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int g = lane / L, l = lane % L;
  const int f0 = VW * l;
  const bool active = f0 < a.F;
  const int f0c = active ? f0 : 0;
  const int head = f0c / a.D;
  const int spad = kWave * 4 * ((v.ng + 255) / 256);
  unsigned char* base = smem + size_t(wave) * vgroup_lds_bytes(v.ng, a.H, HAS_W);
  int* s_col = reinterpret_cast<int*>(base);
  half_t* s_w = reinterpret_cast<half_t*>(base + spad * 4);

  const int64_t j = int64_t(blockIdx.x) * (int(blockDim.x) / kWave) + wave;
  const bool valid = j < v.n_groups;
  int row = 0, idx = 0, cnt = 1, k0 = 0, n = 0;
  if (valid) {
    row = v.grp_row[j];
    idx = int(j - v.goff[row]);
    cnt = v.goff[row + 1] - v.goff[row];
    k0 = a.rowptr[row] + idx * v.ng;
    const int left = a.rowptr[row + 1] - k0;
    n = left < v.ng ? left : v.ng;
  }

  // ---- phase 1: coalesced stage of column ids (as byte offsets) and edge values
  const bool pairs = HAS_W && v.pair_loads;
  for (int i = lane; i < spad; i += kWave) {
    const bool in = i < n;
    const int c = in ? a.col[k0 + i] : 0;
    s_col[i] = OFF32 ? int(uint32_t(c) * uint32_t(a.ldx) * 2u) : c;
    if (HAS_W) {
      if (!pairs) {
        const int64_t slot = in ? (a.eid ? int64_t(a.eid[k0 + i]) : int64_t(k0 + i)) : 0;
        for (int h = 0; h < a.H; ++h) s_w[i * a.H + h] = in ? a.w[slot * a.H + h] : half_t(0);
      } else if (!in) {
        s_w[i] = half_t(0);
      }
    }
  }
  if (pairs) {
    typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
    const int odd = k0 & 1;
    const int64_t b = int64_t(k0) - odd;  // even position at or just before the group's first value
    for (int i = lane; 2 * i < n + odd; i += kWave) {
      half2_t pr;
      if (b + 2 * i + 1 < a.nnz) {
        pr = *reinterpret_cast<const half2_t*>(a.w + b + 2 * i);
      } else {
        pr[0] = a.w[b + 2 * i];
        pr[1] = half_t(0);
      }
      const int i0 = 2 * i - odd;
      if (i0 >= 0 && i0 < n) s_w[i0] = pr[0];
      if (i0 + 1 < n) s_w[i0 + 1] = pr[1];
    }
  }
  wave_sync();

  // ---- phase 2: the groups of lanes take consecutive chunks of the neighbour group
  const int C = 4 * ((v.ng + 4 * G - 1) / (4 * G));
  const int c0 = g * C < n ? g * C : n;
  const int c1 = c0 + C < n ? c0 + C : n;
  float acc[VW];
#pragma unroll
  for (int q = 0; q < VW; ++q) acc[q] = 0.f;
  half2_t acc2[VW / 2 > 0 ? VW / 2 : 1];
#pragma unroll
  for (int q = 0; q < VW / 2; ++q) acc2[q] = half2_t{half_t(0), half_t(0)};
  auto gather = [&](int c) -> hv_t {
    if (OFF32) {
      const uint32_t boff = uint32_t(c) + uint32_t(f0c) * 2u;
      return *reinterpret_cast<const hv_t*>(reinterpret_cast<const char*>(a.X) + boff);
    }
    return *reinterpret_cast<const hv_t*>(a.X + int64_t(c) * a.ldx + f0c);
  };
  for (int i = c0; i < c1; i += 4) {
    const int4_t cols = *reinterpret_cast<const int4_t*>(s_col + i);
    hv_t x[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) x[u] = gather(cols[u]);  // padding holds offset 0, a valid row
    float wv[4] = {a.one, a.one, a.one, a.one};
    if (HAS_W) {
      if (a.H == 1) {
        const half4_t w4 = *reinterpret_cast<const half4_t*>(s_w + i);
#pragma unroll
        for (int u = 0; u < 4; ++u) wv[u] = float(w4[u]);
      } else {
#pragma unroll
        for (int u = 0; u < 4; ++u) wv[u] = float(s_w[(i + u) * a.H + head]);
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (i + 4 <= c1 || i + u < c1) {
        if (VW == 8 && v.acc16) {
          // section 4.2: the edge value mirrored into both halves of a pair multiplies two features per
          // instruction (v_pk_fma_f16); the sum of this lane's chunk stays in fp16
          const half2_t w2 = {half_t(wv[u]), half_t(wv[u])};
#pragma unroll
          for (int q = 0; q < VW / 2; ++q) {
            const half2_t x2 = {x[u][2 * q], x[u][2 * q + 1]};
            acc2[q] = x2 * w2 + acc2[q];
          }
        } else {
#pragma unroll
          for (int q = 0; q < VW; ++q) acc[q] = fmaf(wv[u], float(x[u][q]), acc[q]);
        }
      }
    }
  }
  if (VW == 8 && v.acc16) {
#pragma unroll
    for (int q = 0; q < VW / 2; ++q) {
      acc[2 * q] = float(acc2[q][0]);
      acc[2 * q + 1] = float(acc2[q][1]);
    }
  }
#pragma unroll
  for (int off = L; off < kWave; off <<= 1) {
#pragma unroll
    for (int q = 0; q < VW; ++q) acc[q] += __shfl_xor(acc[q], off);
  }
  if (valid && g == 0 && active) {
    const float sc = scale_of(a, row);
    hv_t h;
#pragma unroll
    for (int q = 0; q < VW; ++q) h[q] = half_t(acc[q] * sc);
    half_t* dst = cnt == 1 ? a.Y + int64_t(row) * a.ldy + f0 : a.staging + (int64_t(v.moff[row]) + idx) * a.stage_ld + f0;
    if (cnt != 1 || f0 + VW <= a.F) {  // staging rows are padded to a multiple of 8
      *reinterpret_cast<hv_t*>(dst) = h;
    } else {
#pragma unroll
      for (int q = 0; q < VW; ++q)
        if (f0 + q < a.F) dst[q] = h[q];
    }
  }
}

// Follow-up kernel of the vertex-parallel variant; it also writes the empty rows.  A wave looks at G
// rows: rows with up to kFinishShort groups are summed by their own lane group, longer ones by the wave.
template <int L>
__global__ __launch_bounds__(kBlock) void spmm_vgroup_finish_kernel(SpmmArgs a, VGroupArgs v) {
  constexpr int G = kWave / L;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int g = lane / L, l = lane % L;
  const int f0 = 8 * l;
  const bool active = f0 < a.F;
  const int f0c = active ? f0 : 0;
  const int64_t r0 = (int64_t(blockIdx.x) * kWavesPerBlock + wave) * G;
  if (r0 >= a.nrows) return;
  const int64_t r = r0 + g;
  int cnt = 1, first = 0;  // cnt = 1: nothing to do
  if (r < a.nrows) {
    cnt = v.goff[r + 1] - v.goff[r];
    first = v.moff[r];
  }
  if (cnt == 0 && active) {
    const float zero[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    store_row(a, r, f0, zero, 0.f);
  }
  if (cnt > 1 && cnt <= kFinishShort) {
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    pieces_accumulate<1, 1>(a, first, int64_t(first) + cnt - 1, f0c, acc);
    if (active) store_row(a, r, f0, acc, 1.f);
  }
  for (int j = 0; j < G; ++j) {
    const int cj = __shfl(cnt, j * L), fj = __shfl(first, j * L);
    if (cj <= kFinishShort) continue;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    pieces_accumulate<G, 1>(a, int64_t(fj) + g, int64_t(fj) + cj - 1, f0c, acc);
    groups_reduce<L>(acc);
    if (g == 0 && active) store_row(a, r0 + j, f0, acc, 1.f);
  }
}

// zero the rows whose pieces the atomic comparison variant adds into Y
template <int L>
__global__ __launch_bounds__(kBlock) void zero_split_rows_kernel(SpmmArgs a) {
  constexpr int G = kWave / L;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int g = lane / L, l = lane % L;
  const int64_t idx = (int64_t(blockIdx.x) * kWavesPerBlock + wave) * G + g;
  if (idx >= a.n_split || 8 * l >= a.F) return;
  const float zero[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  SpmmArgs b = a;
  b.self = nullptr;
  store_row(b, a.split_row[idx], 8 * l, zero, 0.f);
}

// ---------------------------------------------------------------------------------------------------
hgnn_status check_spmm_args(const char* who, const hgnn_csr* g, const hgnn_half* w, int H, const hgnn_half* X,
                                   int64_t ldx, hgnn_half* Y, int64_t ldy, int F, hgnn_reduce op) {
  hgnn_status st = check_csr_args(g, who);
  if (st != HGNN_OK) return st;
  HGNN_REQUIRE(F > 0, HGNN_EINVAL, "%s: F = %d must be positive", who, F);
  HGNN_REQUIRE(F % 2 == 0, HGNN_EINVAL, "%s: F = %d is odd; pad the feature length to the next even number", who, F);
  HGNN_REQUIRE(H >= 1 && F % H == 0, HGNN_EINVAL, "%s: H = %d does not divide F = %d", who, H, F);
  HGNN_REQUIRE(ldx >= F && ldy >= F, HGNN_EINVAL, "%s: leading dimension smaller than F", who);
  HGNN_REQUIRE(ldx % 2 == 0 && ldy % 2 == 0, HGNN_EINVAL, "%s: odd leading dimension", who);
  HGNN_REQUIRE(op == HGNN_SUM || op == HGNN_MEAN, HGNN_EINVAL, "%s: unknown reduce op %d", who, int(op));
  HGNN_REQUIRE(g->nrows == 0 || Y != nullptr, HGNN_EINVAL, "%s: Y is NULL", who);
  HGNN_REQUIRE(g->nnz == 0 || X != nullptr, HGNN_EINVAL, "%s: X is NULL", who);
  (void)w;
  return HGNN_OK;
}

static bool vector_path_ok(const hgnn_half* w, int H, const hgnn_half* X, int64_t ldx, const hgnn_half* Y, int64_t ldy,
                           int F) {
  // F itself need not be a multiple of 8: rows are read in 16-byte pieces up to the padded pitch and the
  // last piece is stored by element
  if (F > 512 || ldx % 8 != 0 || ldy % 8 != 0) return false;
  if (!aligned16(X) || !aligned16(Y)) return false;
  if (w && H > 1 && (F / H) % 8 != 0) return false;
  return true;
}

static SpmmArgs make_args(const hgnn_csr* g, const hgnn_half* w, int H, const hgnn_half* X, int64_t ldx, hgnn_half* Y,
                          int64_t ldy, int F, hgnn_reduce op, const float* row_scale) {
  SpmmArgs a{};
  a.rowptr = g->rowptr;
  a.deg_rowptr = g->rowptr;
  a.col = g->col;
  a.eid = g->eid;
  a.w = reinterpret_cast<const half_t*>(w);
  a.X = reinterpret_cast<const half_t*>(X);
  a.Y = reinterpret_cast<half_t*>(Y);
  a.row_scale = row_scale;
  a.ldx = ldx;
  a.ldy = ldy;
  a.nnz = g->nnz;
  a.nrows = g->nrows;
  a.F = F;
  a.H = w ? H : 1;  // without edge values the head structure is irrelevant
  a.D = F / a.H;
  a.reduce = int(op);
  a.one = 1.0f;
  a.agg_coef = 1.0f;
  a.self_coef = 0.0f;
  return a;
}

template <int L, bool HAS_W>
static void launch_row_set(dim3 grid, hipStream_t s, const SpmmArgs& a, const HubLists* h) {
  if (!h) {
    spmm_row_kernel<L, HAS_W><<<grid, kWave, 0, s>>>(a);  // its waves never meet: single-wave workgroups
    return;
  }
  const int64_t hub_wgs = h->max_chunks < kHubGrid ? h->max_chunks : kHubGrid;
  const int64_t row_wgs = grid.x;
  if (row_wgs + hub_wgs >= (int64_t(1) << 31)) {
    spmm_row_kernel<L, HAS_W><<<grid, kWave, 0, s>>>(a);
    spmm_hub_kernel<L, HAS_W><<<dim3(unsigned(hub_wgs)), kWave, 0, s>>>(a, *h);
  } else {
    spmm_row_hub_kernel<L, HAS_W><<<dim3(unsigned(row_wgs + hub_wgs)), kWave, 0, s>>>(a, *h, int(hub_wgs));
  }
  spmm_hub_sum_kernel<L><<<dim3(unsigned(ceil_div(h->max_hubs, kWavesPerBlock))), kBlock, 0, s>>>(a, *h);
}

template <int L, bool HAS_W>
static void launch_pass_set(hipStream_t s, const SpmmArgs& a, const HubLists* h, const int* cuts, float* part, int npass) {
  constexpr int G = kWave / L;
  spmm_row_pass_kernel<L, HAS_W><<<dim3(unsigned(int64_t(npass) * a.nrows)), kWave, 0, s>>>(a, cuts, part, npass);
  spmm_pass_sum_kernel<L><<<dim3(unsigned(ceil_div(a.nrows, int64_t(kWavesPerBlock) * G))), kBlock, 0, s>>>(a, part, npass);
  if (h) {
    // only rows beyond kPassLongRow are left to the chunks here: a small grid walks the list
    constexpr int kGrid = 8192;
    spmm_hub_kernel<L, HAS_W><<<dim3(unsigned(h->max_chunks < kGrid ? h->max_chunks : kGrid)), kWave, 0, s>>>(a, *h);
    const int64_t max_hubs = std::min<int64_t>(h->max_hubs, a.nnz / kPassLongRow + 1);
    spmm_hub_sum_kernel<L><<<dim3(unsigned(ceil_div(max_hubs, kWavesPerBlock))), kBlock, 0, s>>>(a, *h);
  }
}

template <bool HAS_W>
static void launch_pass(int L, hipStream_t s, const SpmmArgs& a, const HubLists* h, const int* cuts, float* part, int npass) {
  switch (L) {
    case 1: launch_pass_set<1, HAS_W>(s, a, h, cuts, part, npass); break;
    case 2: launch_pass_set<2, HAS_W>(s, a, h, cuts, part, npass); break;
    case 4: launch_pass_set<4, HAS_W>(s, a, h, cuts, part, npass); break;
    case 8: launch_pass_set<8, HAS_W>(s, a, h, cuts, part, npass); break;
    case 16: launch_pass_set<16, HAS_W>(s, a, h, cuts, part, npass); break;
    case 32: launch_pass_set<32, HAS_W>(s, a, h, cuts, part, npass); break;
    default: launch_pass_set<64, HAS_W>(s, a, h, cuts, part, npass); break;
  }
}

template <bool HAS_W>
static void launch_row(int L, dim3 grid, hipStream_t s, const SpmmArgs& a, const HubLists* h) {
  switch (L) {
    case 1: launch_row_set<1, HAS_W>(grid, s, a, h); break;
    case 2: launch_row_set<2, HAS_W>(grid, s, a, h); break;
    case 4: launch_row_set<4, HAS_W>(grid, s, a, h); break;
    case 8: launch_row_set<8, HAS_W>(grid, s, a, h); break;
    case 16: launch_row_set<16, HAS_W>(grid, s, a, h); break;
    case 32: launch_row_set<32, HAS_W>(grid, s, a, h); break;
    default: launch_row_set<64, HAS_W>(grid, s, a, h); break;
  }
}

// Scratch of the hub kernels: chunk and hub lists and one fp32 partial row per chunk, in one block of device memory
// that the caller hands over (hgnn_spmm) or that sits in the library's static device array (hgnn_spmm_static).
// The sizes are worst-case bounds taken from the graph's sizes alone, so that they are known without a look at the
// graph: the sum over the hubs of ceil(deg / chunk) is at most nnz / chunk + the number of hubs, and there are
// fewer than nnz / long_row hubs.
static int hub_threshold(int64_t nrows, int64_t nnz) {
  // hubs: rows longer than 8 times the mean, but never a threshold below 256 or above 1024 non-zeros (on sparse
  // power-law graphs 256 balanced better than 1024: 17 % on an R-MAT of mean degree 16, 1-3 % at mean degree
  // 21-26; with rows of 500 on average 1024 was 2 % better than 4000)
  const int64_t mean = nrows > 0 ? nnz / nrows : 0;
  return int(std::min<int64_t>(std::max<int64_t>(kLongRowMin, 8 * mean), kLongRowMax));
}

struct HubLayout {
  int64_t o_count, o_crow, o_cno, o_hrow, o_hbase, o_part, bytes;
  int64_t max_chunks, max_hubs;
};

static HubLayout hub_layout(int64_t nnz, int long_row, int F) {
  HubLayout o{};
  if (nnz <= long_row) return o;  // no row can be a hub: bytes = 0
  o.max_hubs = nnz / long_row + 1;
  o.max_chunks = nnz / kHubChunk + o.max_hubs + 1;
  auto up = [](int64_t b) { return (b + 255) / 256 * 256; };
  o.o_count = 0;
  o.o_crow = o.o_count + 256;
  o.o_cno = o.o_crow + up(o.max_chunks * 4);
  o.o_hrow = o.o_cno + up(o.max_chunks * 4);
  o.o_hbase = o.o_hrow + up(o.max_hubs * 4);
  o.o_part = o.o_hbase + up(o.max_hubs * 4);
  o.bytes = o.o_part + up(o.max_chunks * int64_t((F + 7) & ~7) * 4);
  return o;
}

// Column passes are taken under the rule that makes a plan cut its graph into column blocks: the table (ncols rows of
// F halves) is beyond three L2s, fits three quarters of the cache behind them, and rows average 128 non-zeros or more;
// about two L2 sizes of feature rows per pass.  1 = one sweep.
static int row_passes(int64_t nrows, int64_t ncols, int64_t nnz, int F) {
  if (nrows <= 0 || nnz / nrows < 128) return 1;
  int64_t l2 = 0, llc = 0;
  device_cache_bytes(&l2, &llc);
  const double table = double(ncols) * F * 2.0;
  if (!(table > 3.0 * double(l2) && table < 0.75 * double(llc))) return 1;
  if (int64_t(16) * nrows >= (int64_t(1) << 31)) return 1;  // one workgroup per (pass, row)
  int np = int(table / (2.0 * double(l2)) + 0.5);
  return np < 2 ? 2 : (np > kMaxPasses ? kMaxPasses : np);
}

struct PassLayout {
  int64_t o_cuts, o_part, bytes;  // offsets from the end of the hub scratch
};

static PassLayout pass_layout(int64_t nrows, int npass, int F) {
  PassLayout o{};
  auto up = [](int64_t b) { return (b + 255) / 256 * 256; };
  o.o_cuts = 0;
  o.o_part = up(nrows * (npass + 1) * 4);
  o.bytes = o.o_part + up(int64_t(npass) * nrows * ((F + 7) & ~7) * 4);
  return o;
}

static HubLists hub_lists_at(void* base, const HubLayout& o) {
  HubLists h{};
  char* p = static_cast<char*>(base);
  h.count = reinterpret_cast<int*>(p + o.o_count);
  h.chunk_row = reinterpret_cast<int*>(p + o.o_crow);
  h.chunk_no = reinterpret_cast<int*>(p + o.o_cno);
  h.hub_row = reinterpret_cast<int*>(p + o.o_hrow);
  h.hub_base = reinterpret_cast<int*>(p + o.o_hbase);
  h.part = reinterpret_cast<float*>(p + o.o_part);
  h.max_chunks = int(o.max_chunks);
  h.max_hubs = int(o.max_hubs);
  return h;
}

template <int WM, bool OFF32>
static void launch_seg(int L, dim3 grid, int threads, size_t lds, hipStream_t s, const SpmmArgs& a) {
  if (WM == 1 && !a.eid && !(a.blocks && a.use_eid)) {  // edge values at the graph's own positions
    switch (L) {
      case 1: spmm_seg_kernel<1, WM, OFF32, WM != 1><<<grid, threads, lds, s>>>(a); break;
      case 2: spmm_seg_kernel<2, WM, OFF32, WM != 1><<<grid, threads, lds, s>>>(a); break;
      case 4: spmm_seg_kernel<4, WM, OFF32, WM != 1><<<grid, threads, lds, s>>>(a); break;
      case 8: spmm_seg_kernel<8, WM, OFF32, WM != 1><<<grid, threads, lds, s>>>(a); break;
      case 16: spmm_seg_kernel<16, WM, OFF32, WM != 1><<<grid, threads, lds, s>>>(a); break;
      case 32: spmm_seg_kernel<32, WM, OFF32, WM != 1><<<grid, threads, lds, s>>>(a); break;
      default: spmm_seg_kernel<64, WM, OFF32, WM != 1><<<grid, threads, lds, s>>>(a); break;
    }
    return;
  }
  switch (L) {
    case 1: spmm_seg_kernel<1, WM, OFF32><<<grid, threads, lds, s>>>(a); break;
    case 2: spmm_seg_kernel<2, WM, OFF32><<<grid, threads, lds, s>>>(a); break;
    case 4: spmm_seg_kernel<4, WM, OFF32><<<grid, threads, lds, s>>>(a); break;
    case 8: spmm_seg_kernel<8, WM, OFF32><<<grid, threads, lds, s>>>(a); break;
    case 16: spmm_seg_kernel<16, WM, OFF32><<<grid, threads, lds, s>>>(a); break;
    case 32: spmm_seg_kernel<32, WM, OFF32><<<grid, threads, lds, s>>>(a); break;
    default: spmm_seg_kernel<64, WM, OFF32><<<grid, threads, lds, s>>>(a); break;
  }
}

static void launch_finish(int L, dim3 grid, hipStream_t s, const SpmmArgs& a) {
  switch (L) {
    case 1: spmm_finish_kernel<1><<<grid, kBlock, 0, s>>>(a); break;
    case 2: spmm_finish_kernel<2><<<grid, kBlock, 0, s>>>(a); break;
    case 4: spmm_finish_kernel<4><<<grid, kBlock, 0, s>>>(a); break;
    case 8: spmm_finish_kernel<8><<<grid, kBlock, 0, s>>>(a); break;
    case 16: spmm_finish_kernel<16><<<grid, kBlock, 0, s>>>(a); break;
    case 32: spmm_finish_kernel<32><<<grid, kBlock, 0, s>>>(a); break;
    default: spmm_finish_kernel<64><<<grid, kBlock, 0, s>>>(a); break;
  }
}

static void launch_zero_split(int L, dim3 grid, hipStream_t s, const SpmmArgs& a) {
  switch (L) {
    case 1: zero_split_rows_kernel<1><<<grid, kBlock, 0, s>>>(a); break;
    case 2: zero_split_rows_kernel<2><<<grid, kBlock, 0, s>>>(a); break;
    case 4: zero_split_rows_kernel<4><<<grid, kBlock, 0, s>>>(a); break;
    case 8: zero_split_rows_kernel<8><<<grid, kBlock, 0, s>>>(a); break;
    case 16: zero_split_rows_kernel<16><<<grid, kBlock, 0, s>>>(a); break;
    case 32: zero_split_rows_kernel<32><<<grid, kBlock, 0, s>>>(a); break;
    default: zero_split_rows_kernel<64><<<grid, kBlock, 0, s>>>(a); break;
  }
}

template <int L, int VW>
static void launch_vgroup_main(bool has_w, bool off32, dim3 grid, int threads, size_t lds, hipStream_t s, const SpmmArgs& a,
                               const VGroupArgs& v) {
  if (has_w) {
    if (off32) spmm_vgroup_kernel<L, VW, true, true><<<grid, threads, lds, s>>>(a, v);
    else if (VW == 8) spmm_vgroup_kernel<L, 8, true, false><<<grid, threads, lds, s>>>(a, v);
  } else {
    if (off32) spmm_vgroup_kernel<L, VW, false, true><<<grid, threads, lds, s>>>(a, v);
    else if (VW == 8) spmm_vgroup_kernel<L, 8, false, false><<<grid, threads, lds, s>>>(a, v);
  }
}

template <int VW>
static void launch_vgroup_vw(int L, bool has_w, bool off32, dim3 grid, int threads, size_t lds, hipStream_t s, const SpmmArgs& a,
                             const VGroupArgs& v) {
  switch (L) {
    case 1: launch_vgroup_main<1, VW>(has_w, off32, grid, threads, lds, s, a, v); break;
    case 2: launch_vgroup_main<2, VW>(has_w, off32, grid, threads, lds, s, a, v); break;
    case 4: launch_vgroup_main<4, VW>(has_w, off32, grid, threads, lds, s, a, v); break;
    case 8: launch_vgroup_main<8, VW>(has_w, off32, grid, threads, lds, s, a, v); break;
    case 16: launch_vgroup_main<16, VW>(has_w, off32, grid, threads, lds, s, a, v); break;
    case 32: launch_vgroup_main<32, VW>(has_w, off32, grid, threads, lds, s, a, v); break;
    default: launch_vgroup_main<64, VW>(has_w, off32, grid, threads, lds, s, a, v); break;
  }
}

static void launch_vgroup_finish(int L, dim3 grid, hipStream_t s, const SpmmArgs& a, const VGroupArgs& v) {
  switch (L) {
    case 1: spmm_vgroup_finish_kernel<1><<<grid, kBlock, 0, s>>>(a, v); break;
    case 2: spmm_vgroup_finish_kernel<2><<<grid, kBlock, 0, s>>>(a, v); break;
    case 4: spmm_vgroup_finish_kernel<4><<<grid, kBlock, 0, s>>>(a, v); break;
    case 8: spmm_vgroup_finish_kernel<8><<<grid, kBlock, 0, s>>>(a, v); break;
    case 16: spmm_vgroup_finish_kernel<16><<<grid, kBlock, 0, s>>>(a, v); break;
    case 32: spmm_vgroup_finish_kernel<32><<<grid, kBlock, 0, s>>>(a, v); break;
    default: spmm_vgroup_finish_kernel<64><<<grid, kBlock, 0, s>>>(a, v); break;
  }
}

// The vertex-parallel variant for the graph in `a` with the neighbour groups of plan p.
static hgnn_status run_vgroups(const hgnn_plan* p, SpmmArgs a, int ncols, bool acc16, hipStream_t s) {
  VGroupArgs v{};
  v.acc16 = acc16 ? 1 : 0;
  v.grp_row = p->grp_row;
  v.goff = p->goff;
  v.moff = p->moff;
  v.n_groups = p->n_groups;
  v.ng = p->ng;
  v.pair_loads = (a.w && a.H == 1 && !a.eid && (reinterpret_cast<uintptr_t>(a.w) & 3u) == 0) ? 1 : 0;
  a.staging = reinterpret_cast<half_t*>(p->gstage);
  a.stage_ld = p->max_F;
  // halves per lane: 8 unless the plan's setting asks for a narrower load and the shape allows it
  int vw = acc16 ? 8 : p->vec_halves;
  const bool off32 = uint64_t(ncols) * uint64_t(a.ldx) * 2u < (uint64_t(1) << 32);
  if (vw != 8) {
    HGNN_REQUIRE(off32 && a.F <= kWave * vw && a.D % vw == 0, HGNN_EUNSUPPORTED,
                 "hgnn_spmm_discretized_variant: %d halves per lane needs F <= %d, D %% %d == 0 and a feature table below 4 GiB",
                 vw, kWave * vw, vw);
  }
  const int L = pow2_at_least((a.F + vw - 1) / vw);   // lanes per row in the main kernel
  const int L8 = pow2_at_least((a.F + 7) / 8);        // the follow-up kernel always moves 16 bytes per lane
  const size_t vg_per_wave = size_t(vgroup_lds_bytes(v.ng, a.H, a.w != nullptr));
  const int wpb = waves_per_block_for_lds(vg_per_wave, a.w != nullptr);
  const size_t lds = vg_per_wave * wpb;
  HGNN_REQUIRE(lds <= 65536, HGNN_EUNSUPPORTED,
               "hgnn_spmm_discretized_variant: group_edges = %d with H = %d needs %zu bytes of LDS per workgroup (limit 65536)",
               v.ng, a.H, lds);
  dim3 grid(unsigned(ceil_div(v.n_groups > 0 ? v.n_groups : 1, wpb)));
  dim3 grid2(unsigned(ceil_div(a.nrows, int64_t(kWavesPerBlock) * (kWave / L8))));
  const bool has_w = a.w != nullptr;
  if (v.n_groups > 0) {
    if (vw == 8) launch_vgroup_vw<8>(L, has_w, off32, grid, wpb * kWave, lds, s, a, v);
    else if (vw == 4) launch_vgroup_vw<4>(L, has_w, off32, grid, wpb * kWave, lds, s, a, v);
    else launch_vgroup_vw<2>(L, has_w, off32, grid, wpb * kWave, lds, s, a, v);
  }
  launch_vgroup_finish(L8, grid2, s, a, v);
  HGNN_LAUNCH_CHECK("spmm_vgroup_kernel / spmm_vgroup_finish_kernel");
  return HGNN_OK;
}

// Pass 1 and pass 2 of the discretized SpMM for the graph in `a` with the segment arrays of plan q.
static hgnn_status run_segments(const hgnn_plan* q, SpmmArgs a, int ncols, hipStream_t s) {
  const int wm = a.col_scale ? 2 : (a.w ? 1 : 0);
  a.seg_lo = q->seg_row_lo;
  a.seg_hi = q->seg_row_hi;
  a.S = q->S;
  a.nseg = q->nseg;
  a.staging = reinterpret_cast<half_t*>(q->staging);
  a.stage_ld = q->max_F;
  a.split_row = q->split_row;
  a.split_lo = q->split_seg_lo;
  a.split_hi = q->split_seg_hi;
  a.n_split = q->n_split;
  const int L = pow2_at_least((a.F + 7) / 8);
  const SegLds lay = seg_lds_layout(a.S, a.H, wm, L);
  const int wpb = waves_per_block_for_lds(size_t(lay.total), wm != 0);
  const int threads = wpb * kWave;
  const size_t lds = size_t(lay.total) * wpb;
  HGNN_REQUIRE(lds <= 65536, HGNN_EUNSUPPORTED,
               "hgnn_spmm_discretized: seg_edges = %d with H = %d needs %zu bytes of LDS per workgroup (limit 65536)", a.S,
               a.H, lds);
  const int64_t nblk = ceil_div(q->nseg, wpb);
  dim3 grid(unsigned(nblk > 0 ? nblk : 1));
  // feature table below 2^32 bytes: 32-bit byte offsets from a scalar base address
  const bool off32 = uint64_t(ncols) * uint64_t(a.ldx) * 2u < (uint64_t(1) << 32);
  if (a.atomic_y && a.n_split > 0) {
    launch_zero_split(L, dim3(unsigned(ceil_div(a.n_split, int64_t(kWavesPerBlock) * (kWave / L)))), s, a);
    HGNN_LAUNCH_CHECK("zero_split_rows_kernel");
  }
  if (wm == 2) {
    if (off32) launch_seg<2, true>(L, grid, threads, lds, s, a);
    else launch_seg<2, false>(L, grid, threads, lds, s, a);
  } else if (wm == 1) {
    if (off32) launch_seg<1, true>(L, grid, threads, lds, s, a);
    else launch_seg<1, false>(L, grid, threads, lds, s, a);
  } else {
    if (off32) launch_seg<0, true>(L, grid, threads, lds, s, a);
    else launch_seg<0, false>(L, grid, threads, lds, s, a);
  }
  HGNN_LAUNCH_CHECK("spmm_seg_kernel");
  if (a.n_split > 0 && !a.atomic_y) {
    const int G = kWave / L;
    dim3 grid2(unsigned(ceil_div(a.n_split, int64_t(kWavesPerBlock) * G)));
    launch_finish(L, grid2, s, a);
    HGNN_LAUNCH_CHECK("spmm_finish_kernel");
  }
  return HGNN_OK;
}

// Pass 1 and pass 2 over all column blocks of plan p, one launch each: a.Y / a.ldy / a.block_y_stride describe the
// blocks' partial outputs.
static hgnn_status run_segments_blocked(const hgnn_plan* p, SpmmArgs a, int ncols, hipStream_t s) {
  const int wm = a.col_scale ? 2 : (a.w ? 1 : 0);
  a.blocks = p->bdesc;
  a.nblocks = p->nb;
  a.S = p->S;
  a.stage_ld = p->max_F;
  const int L = pow2_at_least((a.F + 7) / 8);
  const int G = kWave / L;
  const SegLds lay = seg_lds_layout(a.S, a.H, wm, L);
  const int wpb = waves_per_block_for_lds(size_t(lay.total), wm != 0);
  const size_t lds = size_t(lay.total) * wpb;
  HGNN_REQUIRE(lds <= 65536, HGNN_EUNSUPPORTED,
               "hgnn_spmm_discretized: seg_edges = %d with H = %d needs %zu bytes of LDS per workgroup (limit 65536)", a.S,
               a.H, lds);
  int64_t wgs = 0, wgs2 = 0;
  for (const hgnn_plan* q : p->sub) {
    const int64_t c = ceil_div(q->nseg, wpb);
    wgs += c > 0 ? c : 1;
    wgs2 += ceil_div(q->n_split, int64_t(kWavesPerBlock) * G);
  }
  const bool off32 = uint64_t(ncols) * uint64_t(a.ldx) * 2u < (uint64_t(1) << 32);
  dim3 grid{unsigned(wgs)};
  const int threads = wpb * kWave;
  if (wm == 2) {
    if (off32) launch_seg<2, true>(L, grid, threads, lds, s, a);
    else launch_seg<2, false>(L, grid, threads, lds, s, a);
  } else if (wm == 1) {
    if (off32) launch_seg<1, true>(L, grid, threads, lds, s, a);
    else launch_seg<1, false>(L, grid, threads, lds, s, a);
  } else {
    if (off32) launch_seg<0, true>(L, grid, threads, lds, s, a);
    else launch_seg<0, false>(L, grid, threads, lds, s, a);
  }
  HGNN_LAUNCH_CHECK("spmm_seg_kernel");
  if (wgs2 > 0) {
    launch_finish(L, dim3(unsigned(wgs2)), s, a);
    HGNN_LAUNCH_CHECK("spmm_finish_kernel");
  }
  return HGNN_OK;
}

// Column-blocked plans: Y[r] = sum over the blocks of their (already scaled, fp16) partial rows; fp32 sum in
// block order, one store per row.
template <int L>
__global__ __launch_bounds__(kBlock) void spmm_block_sum_kernel(SpmmArgs a, const half_t* __restrict__ part, int nb,
                                                                 int part_ld) {
  constexpr int G = kWave / L;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int g = lane / L, l = lane % L;
  const int f0 = 8 * l;
  const int64_t r = (int64_t(blockIdx.x) * kWavesPerBlock + wave) * G + g;
  if (r >= a.nrows || f0 >= a.F) return;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int b = 0; b < nb; ++b) {
    const half8_t t = *reinterpret_cast<const half8_t*>(part + (int64_t(b) * a.nrows + r) * part_ld + f0);
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] += float(t[i]);
  }
  store_row(a, r, f0, acc, 1.f);
}

static void launch_block_sum(int L, dim3 grid, hipStream_t s, const SpmmArgs& a, const half_t* part, int nb, int part_ld) {
  switch (L) {
    case 1: spmm_block_sum_kernel<1><<<grid, kBlock, 0, s>>>(a, part, nb, part_ld); break;
    case 2: spmm_block_sum_kernel<2><<<grid, kBlock, 0, s>>>(a, part, nb, part_ld); break;
    case 4: spmm_block_sum_kernel<4><<<grid, kBlock, 0, s>>>(a, part, nb, part_ld); break;
    case 8: spmm_block_sum_kernel<8><<<grid, kBlock, 0, s>>>(a, part, nb, part_ld); break;
    case 16: spmm_block_sum_kernel<16><<<grid, kBlock, 0, s>>>(a, part, nb, part_ld); break;
    case 32: spmm_block_sum_kernel<32><<<grid, kBlock, 0, s>>>(a, part, nb, part_ld); break;
    default: spmm_block_sum_kernel<64><<<grid, kBlock, 0, s>>>(a, part, nb, part_ld); break;
  }
}

// The plan-free SpMM with its hub scratch at `scratch` (scratch_bytes of device memory, may be null: then no row is
// treated as a hub and a long row is reduced by one wave).
hgnn_status spmm_rows(const char* who, const hgnn_csr* g, const hgnn_half* edge_val, int32_t H, const hgnn_half* X,
                             int64_t ldx, hgnn_half* Y, int64_t ldy, int32_t F, hgnn_reduce op, const float* row_scale,
                             void* scratch, size_t scratch_bytes, hipStream_t s) {
  SpmmArgs a = make_args(g, edge_val, H, X, ldx, Y, ldy, F, op, row_scale);
  if (!vector_path_ok(edge_val, H, X, ldx, Y, ldy, F)) {
    dim3 grid(unsigned(ceil_div(int64_t(g->nrows) * F, kBlock)));
    spmm_scalar_kernel<<<grid, kBlock, 0, s>>>(a);
    HGNN_LAUNCH_CHECK("spmm_scalar_kernel");
    return HGNN_OK;
  }
  const int L = pow2_at_least((F + 7) / 8);
  // sparse rows: a wave takes one row per lane group; dense rows: one row per wave, for balance
  a.rows_per_wave = g->nnz / g->nrows >= 64 ? 1 : kWave / L;
  dim3 grid(unsigned(ceil_div(g->nrows, a.rows_per_wave)));
  a.long_row = hub_threshold(g->nrows, g->nnz);
  const HubLayout lay = hub_layout(g->nnz, a.long_row, F);
  HubLists h{};
  const bool hubs = lay.bytes > 0 && scratch != nullptr;
  const int npass = scratch ? row_passes(g->nrows, g->ncols, g->nnz, F) : 1;
  const PassLayout pl = pass_layout(g->nrows, npass, F);
  if (npass > 1 && scratch_bytes >= size_t(lay.bytes + pl.bytes)) {
    HGNN_REQUIRE((reinterpret_cast<uintptr_t>(scratch) & 15u) == 0, HGNN_EINVAL, "%s: the workspace must be 16-byte aligned", who);
    a.long_row = kPassLongRow > a.long_row ? kPassLongRow : a.long_row;
    if (hubs) {
      h = hub_lists_at(scratch, lay);
      hub_zero_kernel<<<1, kBlock, 0, s>>>(h);
      hub_scan_kernel<<<dim3(unsigned(ceil_div(g->nrows, kBlock * kScanRows))), kBlock, 0, s>>>(a, h);
    } else {
      a.long_row = INT_MAX;
    }
    char* base = static_cast<char*>(scratch) + lay.bytes;
    int* cuts = reinterpret_cast<int*>(base + pl.o_cuts);
    float* part = reinterpret_cast<float*>(base + pl.o_part);
    const int width = int(ceil_div(g->ncols, npass));
    row_cuts_kernel<<<dim3(unsigned(ceil_div(g->nrows, kWavesPerBlock))), kBlock, 0, s>>>(g->rowptr, g->col, g->nrows, g->ncols,
                                                                                        npass, width, a.long_row, cuts);
    if (edge_val) launch_pass<true>(L, s, a, hubs ? &h : nullptr, cuts, part, npass);
    else launch_pass<false>(L, s, a, hubs ? &h : nullptr, cuts, part, npass);
    HGNN_LAUNCH_CHECK("spmm_row_pass_kernel");
    return HGNN_OK;
  }
  if (hubs) {
    HGNN_REQUIRE(scratch_bytes >= size_t(lay.bytes), HGNN_EINVAL, "%s: the workspace holds %zu bytes, this graph needs %lld", who,
                 scratch_bytes, (long long)lay.bytes);
    HGNN_REQUIRE((reinterpret_cast<uintptr_t>(scratch) & 15u) == 0, HGNN_EINVAL, "%s: the workspace must be 16-byte aligned", who);
    h = hub_lists_at(scratch, lay);
    hub_zero_kernel<<<1, kBlock, 0, s>>>(h);
    hub_scan_kernel<<<dim3(unsigned(ceil_div(g->nrows, kBlock * kScanRows))), kBlock, 0, s>>>(a, h);
  } else {
    a.long_row = INT_MAX;  // no scratch: every row above the short-row limit is reduced by one wave
  }
  if (edge_val) launch_row<true>(L, grid, s, a, hubs ? &h : nullptr);
  else launch_row<false>(L, grid, s, a, hubs ? &h : nullptr);
  HGNN_LAUNCH_CHECK("spmm_row_kernel");
  return HGNN_OK;
}

size_t spmm_hub_scratch_bytes(int32_t nrows, int64_t nnz, int32_t F) {
  if (nrows <= 0 || nnz <= 0 || F <= 0) return 0;
  return size_t(hub_layout(nnz, hub_threshold(nrows, nnz), F).bytes);
}

}  // namespace hgnn

using namespace hgnn;

extern "C" {

size_t hgnn_spmm_workspace(int32_t nrows, int32_t ncols, int64_t nnz, int32_t F) {
  if (nrows <= 0 || nnz <= 0 || F <= 0) return 0;
  size_t need = spmm_hub_scratch_bytes(nrows, nnz, F);
  const int npass = ncols > 0 ? row_passes(nrows, ncols, nnz, F) : 1;
  if (npass > 1) need += size_t(pass_layout(nrows, npass, F).bytes);
  return need;
}

hgnn_status hgnn_spmm(const hgnn_csr* g, const hgnn_half* edge_val, int32_t H, const hgnn_half* X, int64_t ldx,
                      hgnn_half* Y, int64_t ldy, int32_t F, hgnn_reduce op, const float* row_scale, void* workspace,
                      size_t workspace_bytes, void* stream) {
  clear_error();
  hgnn_status st = check_spmm_args("hgnn_spmm", g, edge_val, H, X, ldx, Y, ldy, F, op);
  if (st != HGNN_OK) return st;
  if (g->nrows == 0) return HGNN_OK;
  return spmm_rows("hgnn_spmm", g, edge_val, H, X, ldx, Y, ldy, F, op, row_scale, workspace, workspace_bytes,
                   static_cast<hipStream_t>(stream));
}

hgnn_status hgnn_spmm_discretized_fused(const hgnn_plan* p, const hgnn_csr* g, const hgnn_half* edge_val, int32_t H,
                                        const hgnn_half* X, int64_t ldx, hgnn_half* Y, int64_t ldy, int32_t F,
                                        hgnn_reduce op, const float* row_scale, const hgnn_spmm_fusion* fz,
                                        void* stream) {
  clear_error();
  const char* who = "hgnn_spmm_discretized";
  hgnn_status st = check_spmm_args(who, g, edge_val, H, X, ldx, Y, ldy, F, op);
  if (st != HGNN_OK) return st;
  HGNN_REQUIRE(p != nullptr, HGNN_EINVAL, "%s: plan is NULL", who);
  HGNN_REQUIRE(p->nrows == g->nrows && p->ncols == g->ncols && p->nnz == g->nnz, HGNN_EINVAL,
               "%s: the plan was built for another graph", who);
  HGNN_REQUIRE(F <= p->max_F, HGNN_EINVAL, "%s: F = %d exceeds the plan's max_F = %d", who, F, p->max_F);
  HGNN_REQUIRE(vector_path_ok(edge_val, H, X, ldx, Y, ldy, F), HGNN_EUNSUPPORTED,
               "%s: needs F <= 512, ld %% 8 == 0, 16-byte aligned X, Y, and D %% 8 == 0 when edge values have several heads", who);
  if (fz && fz->self)
    HGNN_REQUIRE(fz->ld_self >= F && fz->ld_self % 8 == 0 && aligned16(fz->self), HGNN_EINVAL,
                 "%s: self features need ld_self >= F, ld_self %% 8 == 0 and a 16-byte aligned base", who);
  const bool prescale = fz && fz->col_scale && fz->scaled_x;
  if (prescale)
    HGNN_REQUIRE(fz->ld_scaled >= F && fz->ld_scaled % 8 == 0 && aligned16(fz->scaled_x), HGNN_EINVAL,
                 "%s: the scaled_x workspace needs ld_scaled >= F, ld_scaled %% 8 == 0 and a 16-byte aligned base", who);
  if (g->nrows == 0) return HGNN_OK;
  hipStream_t s = static_cast<hipStream_t>(stream);
  SpmmArgs a = make_args(g, edge_val, H, X, ldx, Y, ldy, F, op, row_scale);
  if (prescale) {
    // the column scale goes onto the table once; the kernels then run without a per-edge factor
    st = hgnn_scale_rows(g->ncols, F, X, ldx, fz->col_scale, fz->scaled_x, fz->ld_scaled, stream);
    if (st != HGNN_OK) return st;
    a.X = reinterpret_cast<const half_t*>(fz->scaled_x);
    a.ldx = fz->ld_scaled;
  }
  if (fz) {
    a.col_scale = prescale ? nullptr : fz->col_scale;
    a.self = reinterpret_cast<const half_t*>(fz->self);
    a.ld_self = fz->ld_self;
    a.self_coef = fz->self_coef;
    a.agg_coef = fz->agg_coef;
    if (a.col_scale && !edge_val) {  // the per-edge factor is the column scale alone; heads are irrelevant
      a.H = 1;
      a.D = F;
    }
  }
  // blocks that the automatic rule chose (for max_F) are used when the table of this call is beyond an L2 too
  const bool use_blocks = p->nb > 1 && (!p->auto_blocks || double(g->ncols) * double(a.ldx) * 2.0 > 3.0 * double(p->l2_bytes));
  if (!use_blocks) return run_segments(p, a, g->ncols, s);
  HGNN_REQUIRE(!(edge_val && g->eid && !p->block_eid), HGNN_EINVAL,
               "%s: the column-blocked plan was built from a graph without an edge-id map; build the plan from the graph "
               "that carries the map", who);
  // column-blocked plan: one discretized SpMM per block into that block's partial output, blocks one
  // after the other so that all compute units gather from the same slice of X, then one pass adds
  // the partials of every row (and the self term, once).  Scales are applied per partial (section 5.2.2).
  // edge values behind an edge-id map: the plan's finer blocks, where it has them
  if (edge_val && g->eid && p->fine) p = p->fine;
  {
    // all blocks in one launch of each kernel (workgroups numbered block after block), into the blocks' partial outputs.
    // Slots in the edge tensors: a graph without an edge-id map reads at its own CSR positions (block position + the
    // row's offset, a coalesced read); a graph with one reads through the blocked copy of the map
    SpmmArgs ab = a;
    ab.use_eid = g->eid ? 1 : 0;
    ab.Y = reinterpret_cast<half_t*>(p->bstage);
    ab.ldy = p->max_F;
    ab.block_y_stride = int64_t(p->nrows) * p->max_F;
    ab.self = nullptr;
    st = run_segments_blocked(p, ab, g->ncols, s);
    if (st != HGNN_OK) return st;
  }
  const int L = pow2_at_least((F + 7) / 8);
  const int G = kWave / L;
  launch_block_sum(L, dim3(unsigned(ceil_div(g->nrows, int64_t(kWavesPerBlock) * G))), s, a,
                   reinterpret_cast<const half_t*>(p->bstage), p->nb, p->max_F);
  HGNN_LAUNCH_CHECK("spmm_block_sum_kernel");
  return HGNN_OK;
}

hgnn_status hgnn_spmm_discretized(const hgnn_plan* p, const hgnn_csr* g, const hgnn_half* edge_val, int32_t H,
                                  const hgnn_half* X, int64_t ldx, hgnn_half* Y, int64_t ldy, int32_t F,
                                  hgnn_reduce op, const float* row_scale, void* stream) {
  return hgnn_spmm_discretized_fused(p, g, edge_val, H, X, ldx, Y, ldy, F, op, row_scale, nullptr, stream);
}

hgnn_status hgnn_spmm_discretized_variant(const hgnn_plan* p, const hgnn_csr* g, const hgnn_half* edge_val, int32_t H,
                                          const hgnn_half* X, int64_t ldx, hgnn_half* Y, int64_t ldy, int32_t F,
                                          hgnn_reduce op, const float* row_scale, hgnn_spmm_variant variant,
                                          void* stream) {
  if (variant == HGNN_EDGE_SEGMENTS)
    return hgnn_spmm_discretized_fused(p, g, edge_val, H, X, ldx, Y, ldy, F, op, row_scale, nullptr, stream);
  clear_error();
  const char* who = "hgnn_spmm_discretized_variant";
  HGNN_REQUIRE(variant == HGNN_EDGE_SEGMENTS_ATOMIC || variant == HGNN_VERTEX_GROUPS || variant == HGNN_VERTEX_GROUPS_HALF2,
               HGNN_EINVAL, "%s: unknown variant %d", who, int(variant));
  hgnn_status st = check_spmm_args(who, g, edge_val, H, X, ldx, Y, ldy, F, op);
  if (st != HGNN_OK) return st;
  HGNN_REQUIRE(p != nullptr, HGNN_EINVAL, "%s: plan is NULL", who);
  HGNN_REQUIRE(p->nrows == g->nrows && p->ncols == g->ncols && p->nnz == g->nnz, HGNN_EINVAL,
               "%s: the plan was built for another graph", who);
  HGNN_REQUIRE(F <= p->max_F, HGNN_EINVAL, "%s: F = %d exceeds the plan's max_F = %d", who, F, p->max_F);
  HGNN_REQUIRE(vector_path_ok(edge_val, H, X, ldx, Y, ldy, F), HGNN_EUNSUPPORTED,
               "%s: needs F <= 512, ld %% 8 == 0, 16-byte aligned X, Y, and D %% 8 == 0 when edge values have several heads", who);
  HGNN_REQUIRE(variant == HGNN_EDGE_SEGMENTS_ATOMIC || p->ng > 0, HGNN_EINVAL,
               "%s: the plan holds no neighbour groups (hgnn_plan_add_groups)", who);
  if (g->nrows == 0) return HGNN_OK;
  hipStream_t s = static_cast<hipStream_t>(stream);
  SpmmArgs a = make_args(g, edge_val, H, X, ldx, Y, ldy, F, op, row_scale);
  if (variant != HGNN_EDGE_SEGMENTS_ATOMIC) return run_vgroups(p, a, g->ncols, variant == HGNN_VERTEX_GROUPS_HALF2, s);
  a.atomic_y = 1;  // always on the whole graph: column blocks are not used by the comparison variants
  return run_segments(p, a, g->ncols, s);
}

}  // extern "C"
