// Internal definitions shared by the translation units of libhgnn.so (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "hgnn.h"

namespace hgnn {

constexpr int kWave = 64;          // CDNA wavefront
constexpr int kWavesPerBlock = 4;  // 256-thread workgroups: one wave per SIMD of a CU
constexpr int kBlock = kWave * kWavesPerBlock;

typedef _Float16 half_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));  // 16 bytes: one global_load_dwordx4 per lane

// ---- status plumbing -------------------------------------------------------------------------
hgnn_status fail(hgnn_status s, const char* fmt, ...);  // records the thread-local message, returns s
void clear_error();

#define HGNN_REQUIRE(cond, status, ...)                  \
  do {                                                   \
    if (!(cond)) return ::hgnn::fail(status, __VA_ARGS__); \
  } while (0)

#define HGNN_HIP(call)                                                                              \
  do {                                                                                              \
    hipError_t err__ = (call);                                                                      \
    if (err__ != hipSuccess)                                                                        \
      return ::hgnn::fail(err__ == hipErrorOutOfMemory ? HGNN_ENOMEM : HGNN_EHIP, "%s: %s", #call, \
                          hipGetErrorString(err__));                                                \
  } while (0)

#define HGNN_LAUNCH_CHECK(name)                                                     \
  do {                                                                              \
    hipError_t err__ = hipGetLastError();                                           \
    if (err__ != hipSuccess)                                                        \
      return ::hgnn::fail(HGNN_EHIP, "launch of %s: %s", name, hipGetErrorString(err__)); \
  } while (0)

// Waves per workgroup for a kernel whose waves work independently on private LDS regions of per_wave bytes
// (no workgroup barrier anywhere, so the choice is free).  Measured on MI355X: kernels that stage per-edge
// values or scores before their main loop (a dependent chain of global loads whose length varies from wave to
// wave) run 5-15 % faster as single-wave workgroups -- a workgroup's LDS and wave slots are only released
// when its last wave ends, and small allocations pack the 160 KB of LDS better -- while the plain
// unweighted segment kernel runs 4 % faster in workgroups of four (fewer dispatches, waves of consecutive
// segments start together).  independent_waves selects the former; either way the workgroup must fit 64 KB.
inline int waves_per_block_for_lds(size_t per_wave, bool independent_waves) {
  int w = independent_waves ? 1 : 4;
  while (w > 1 && per_wave * size_t(w) > 65536) w >>= 1;
  return w;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// smallest power of two >= v (v >= 1)
inline int pow2_at_least(int v) {
  int p = 1;
  while (p < v) p <<= 1;
  return p;
}

hgnn_status check_csr_args(const hgnn_csr* g, const char* who);

// row that holds CSR position k: the last r with rowptr[r] <= k (an upper bound minus one, so
// empty rows are skipped)
__host__ __device__ inline int row_of_edge(const int* rowptr, int nrows, int64_t k) {
  int lo = 0, hi = nrows + 1;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (int64_t(rowptr[mid]) <= k) lo = mid + 1;
    else hi = mid;
  }
  return lo - 1;
}

// Orders the LDS accesses of one wave: what its lanes wrote before is visible to all its lanes after.
// The kernels that stage a segment give every wave a private LDS region, so nothing wider than the
// wave has to meet; a workgroup barrier there would only put the four waves in lock step and stall
// three of them whenever one waits for memory.
__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// v += the value of the lane that the data-parallel-primitive control CTRL pairs this lane with (one VALU
// instruction, no trip through the LDS crossbar).  Controls used: quad_perm [1,0,3,2] = 0xB1 and [2,3,0,1] =
// 0x4E (lane ^ 1, lane ^ 2), row_half_mirror = 0x141 (lane i <-> 7 - i of each 8), row_mirror = 0x140
// (i <-> 15 - i of each 16).
template <int CTRL>
__device__ __forceinline__ float dpp_add(float v) {
  const int t = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false);
  return v + __int_as_float(t);
}

// All-reduce (sum) over the LH consecutive, LH-aligned lanes of a head; LH is a power of two.  After the
// quads are summed, a mirror inside 8 (16) lanes pairs every lane with one of the other quad (half), whose
// partial sum is the same on all its lanes; beyond a row of 16 lanes the exchange goes through ds_bpermute.
__device__ __forceinline__ float head_sum1(float v, int LH) {
  if (LH >= 2) v = dpp_add<0xB1>(v);
  if (LH >= 4) v = dpp_add<0x4E>(v);
  if (LH >= 8) v = dpp_add<0x141>(v);
  if (LH >= 16) v = dpp_add<0x140>(v);
  for (int off = 16; off < LH; off <<= 1) v += __shfl_xor(v, off);
  return v;
}

// the same for four independent values at once (four chains in flight)
__device__ __forceinline__ void head_sum4(float (&v)[4], int LH) {
  if (LH >= 2) {
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = dpp_add<0xB1>(v[u]);
  }
  if (LH >= 4) {
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = dpp_add<0x4E>(v[u]);
  }
  if (LH >= 8) {
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = dpp_add<0x141>(v[u]);
  }
  if (LH >= 16) {
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = dpp_add<0x140>(v[u]);
  }
  for (int off = 16; off < LH; off <<= 1) {
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] += __shfl_xor(v[u], off);
  }
}

typedef int int4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));

// ---- per-edge row ids of one plan segment, staged in LDS by one wave ---------------------------------
// A segment of n <= S consecutive edges starting at e0 touches the rows row_lo..row_hi (plan arrays).
// Every non-empty row after row_lo marks the slot of its first edge, then a wave-wide running
// maximum spreads the ids: s_row[i] = row of edge e0+i for i < n, -2 for the padding up to
// 64*per slots; s_blk[i/4] = common row id of the aligned group of four edges, or -1 when they
// differ or touch the padding.  Lane t owns the slots [t*per, (t+1)*per); per is a multiple of 4.
// s_row / s_blk are private to the calling wave, so wave-level ordering is enough; BLOCK_SYNC = true uses
// workgroup barriers instead (every wave of the workgroup must then call it, n = 0 without a segment),
// which keeps the four waves of a streaming kernel in step on consecutive segments.
__device__ __forceinline__ int seg_slots_per_lane(int S) { return 4 * ((S + 255) / 256); }

// The index arrays (column ids, edge ids) are read once per pass.  On graphs whose arrays are far larger than the
// caches a non-temporal load keeps them from displacing the feature rows that the gathers reuse (config 5: 1-2 %
// on every segment kernel, config 4 up to 3 %); on graphs that fit the Infinity Cache it would push the arrays out
// between kernels (config 3: the next kernel's reads of the column ids 15 % slower), hence the size rule.
__host__ __device__ inline bool stream_nontemporal(int64_t nnz) { return nnz * 4 > (int64_t(64) << 20); }

// four consecutive rounds of a lane's reads from an index array, in flight together: v[q] = p[i0 + q * kWave], or 0
// from position n on.  NT is a template parameter because a run-time choice between two loads of one address is
// folded into a single ordinary load by the compiler.
template <bool NT>
__device__ __forceinline__ void stream_load4(const int* __restrict__ p, int i0, int n, int (&v)[4]) {
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int i = i0 + q * kWave;
    v[q] = 0;
    if (i < n) v[q] = NT ? __builtin_nontemporal_load(p + i) : p[i];
  }
}

// Reads the n column ids of a segment (0 beyond n) and hands them to put(i, c) for i in [0, spad); spad is a
// multiple of 4 * kWave (see seg_slots_per_lane).  A lane has its four loads of a round in flight together: a loop
// of one load and one LDS store per turn waits for every load in turn, four memory latencies per 256 edges.
template <class Put>
__device__ __forceinline__ void seg_stage_cols(const int* __restrict__ col, int64_t e0, int lane, int spad, int n, bool nt,
                                               Put&& put) {
  for (int i0 = lane; i0 < spad; i0 += 4 * kWave) {
    int c[4];
    if (nt) stream_load4<true>(col + e0, i0, n, c);
    else stream_load4<false>(col + e0, i0, n, c);
#pragma unroll
    for (int q = 0; q < 4; ++q) put(i0 + q * kWave, c[q]);
  }
}

template <bool BLOCK_SYNC = false>
__device__ __forceinline__ void seg_stage_rows(int* s_row, int* s_blk, int lane, int per, int n, int row_lo, int row_hi,
                                               const int* __restrict__ rowptr, int64_t e0, bool* open = nullptr) {
  const int r0 = row_lo + 1 + lane;
  int p0 = 0, q0 = 0, b_lo = 0, b_hi = 0;
  if (open && n > 0) {  // a segment of the plan: row_lo <= row_hi are rows of the graph
    const int rc = r0 <= row_hi ? r0 : row_lo;
    p0 = rowptr[rc];
    q0 = rowptr[rc + 1];
    b_lo = rowptr[row_lo];
    b_hi = rowptr[row_hi + 1];
  }
  for (int i = lane; i < kWave * per; i += kWave) s_row[i] = i == 0 ? row_lo : -1;
  if (BLOCK_SYNC) __syncthreads();
  else wave_sync();
  if (open) {
    if (r0 <= row_hi && q0 > p0) s_row[p0 - int(e0)] = r0;
    open[0] = n > 0 && int64_t(b_lo) < e0;
    open[1] = n > 0 && int64_t(b_hi) > e0 + n;
  }
  for (int r = open ? r0 + kWave : r0; r <= row_hi; r += kWave) {
    const int p = rowptr[r], q = rowptr[r + 1];
    if (q > p) s_row[p - int(e0)] = r;
  }
  if (BLOCK_SYNC) __syncthreads();
  else wave_sync();
  const int b0 = lane * per;
  int run = -1;
  for (int j = 0; j < per; ++j) {
    run = max(run, s_row[b0 + j]);
    s_row[b0 + j] = run;
  }
  int inc = run;
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    const int t = __shfl_up(inc, d);
    if (lane >= d) inc = max(inc, t);
  }
  int excl = __shfl_up(inc, 1);
  if (lane == 0) excl = -1;
  for (int j = 0; j < per; j += 4) {
    int v[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      v[q] = max(s_row[b0 + j + q], excl);
      if (b0 + j + q >= n) v[q] = -2;
      s_row[b0 + j + q] = v[q];
    }
    s_blk[(b0 + j) >> 2] = (v[0] == v[1] && v[1] == v[2] && v[2] == v[3]) ? v[0] : -1;
  }
  if (BLOCK_SYNC) __syncthreads();
  else wave_sync();
}

}  // namespace hgnn

// One column block of a blocked plan as the kernels see it when all blocks run in one launch (device array in the plan).
struct hgnn_seg_block {
  const int32_t* rowptr;   // the block's own offset array [nrows+1]
  const int32_t* col;
  const int32_t* eid;      // slots of the creating graph's edge-id map (or CSR positions), block order
  const int32_t* delta;    // [nrows] CSR position in the whole graph = block position + delta[row]
  const int32_t* seg_lo;
  const int32_t* seg_hi;
  hgnn_half* staging;
  const int32_t* split_row;
  const int32_t* split_lo;
  const int32_t* split_hi;
  int64_t nnz, nseg;
  int32_t n_split, pad;
  float* stage_mz;         // scalars of the staged pieces of the fused GAT passes
};

// The plan object behind the opaque handle of the C ABI.
constexpr int kHubEdges = 2048;  // non-zeros per chunk of a long row in the edge-row kernels

struct hgnn_plan {
  int32_t nrows = 0, ncols = 0;
  int64_t nnz = 0;
  int32_t S = 0;        // edges per segment
  int64_t nseg = 0;     // ceil(nnz / S)
  int32_t n_split = 0;  // rows whose edges span more than one segment
  int32_t n_big = 0;    // rows longer than big_deg (edge softmax hands them to a whole workgroup)
  int32_t n_mid = 0;    // rows longer than mid_deg and at most big_deg (edge softmax: one wave each)
  int32_t mid_deg = 0;
  int32_t big_deg = 0;
  int64_t listed_nnz = 0;  // non-zeros of the rows in mid_row and big_row (the rest belong to rows of at most mid_deg)
  int32_t max_F = 0, max_H = 0;
  int64_t l2_bytes = 0, llc_bytes = 0;  // cache sizes of the device the plan was built on (an XCD's L2, the cache behind the L2s)
  int32_t vec_halves = 8;  // halves a lane moves per feature load in the kernels that exist in several widths (8, 4 or 2)
  bool auto_blocks = false;  // the blocks were chosen by the automatic rule (col_blocks = 0): a call whose own table is small runs unblocked
  bool block_eid = false;  // column blocks: built from a graph that carried an edge-id map (beid holds that map's slots)
  int32_t* seg_row_lo = nullptr;    // [nseg]
  int32_t* seg_row_hi = nullptr;    // [nseg]
  int32_t* split_row = nullptr;     // [n_split]
  int32_t* split_seg_lo = nullptr;  // [n_split]
  int32_t* split_seg_hi = nullptr;  // [n_split]
  int32_t* big_row = nullptr;       // [n_big]
  int32_t* mid_row = nullptr;       // [n_mid]
  // the rows of big_row cut into chunks of kHubEdges non-zeros for the edge-row kernels (softmax, its backward, row
  // sums): a workgroup per chunk leaves partial results, a second pass combines those of a row
  int32_t n_hub_chunks = 0;
  int32_t* hub_chunk_row = nullptr;    // [n_hub_chunks] the row a chunk belongs to
  int32_t* hub_chunk_first = nullptr;  // [n_hub_chunks] slot of the first chunk of that row (slot - first = chunk number)
  int32_t* hub_chunk_count = nullptr;  // [n_hub_chunks] chunks of that row
  int32_t* big_first = nullptr;        // [n_big] slot of the first chunk of big_row[i]
  float* hub_part = nullptr;           // [n_hub_chunks][max_H][2] partial results
  hgnn_half* staging = nullptr;     // [2][2*nseg][max_F] (second set: masked vectors of the saving GAT pass)
  float* stage_mz = nullptr;        // [2*nseg][max_H][2] softmax (max, sum) of the staged pieces of the fused GAT pass, then [2*nseg][max_H] masked sums
  float* vscratch = nullptr;        // [(nrows + ncols) * max_H] fp32
  float* vtab = nullptr;            // [nrows][max_H][4] fp32 per-vertex (el, lse, t, -) of the fused GAT backward
  // column blocking of the SpMM (nb > 1): block b holds the non-zeros whose column lies in
  // [b*block_width, (b+1)*block_width), stored block after block as a CSR of their own
  int32_t nb = 1;
  int32_t block_width = 0;
  int32_t* brp = nullptr;           // [nb][nrows+1] offset arrays of the blocks
  int32_t* bcol = nullptr;          // [nnz] column ids, block-major
  int32_t* beid = nullptr;          // [nnz] slot in the edge tensors of every blocked non-zero: the creating graph's eid, else its CSR position
  int32_t* bdelta = nullptr;        // [nb][nrows] CSR position in the whole graph of a blocked non-zero = its block position + bdelta[b][row]
  std::vector<int64_t> boff;        // [nb+1] first non-zero of every block in bcol / beid
  std::vector<hgnn_plan*> sub;      // [nb] segment plans of the blocks
  hgnn_seg_block* bdesc = nullptr;  // [nb] the blocks' arrays, for kernels that walk all blocks in one launch
  hgnn_plan* fine = nullptr;        // the same graph in twice the blocks (blocked arrays only), for the SpMM that gathers edge
                                    // values through the edge-id map and for the SDDMM; only where the automatic rule
                                    // chose the blocks
  hgnn_half* bstage = nullptr;      // [2][nb][nrows][max_F] per-block partial outputs (second set: masked GAT partials)
  float* bsum = nullptr;            // [nb][nrows][max_H][2] per-block partial row sums of edge tensors / GAT (max, sum), then [nb][nrows][max_H] masked sums
  // neighbour groups of the vertex-parallel variant (hgnn_plan_add_groups): row r owns the groups
  // goff[r] .. goff[r+1]-1, group j of the row covers the non-zeros rowptr[r] + j*ng ...
  int32_t ng = 0;                   // neighbours per group; 0 = not built
  int64_t n_groups = 0;
  int64_t n_gslots = 0;             // groups that belong to rows with more than one group
  int32_t* goff = nullptr;          // [nrows+1]
  int32_t* moff = nullptr;          // [nrows+1] first staging slot of a row with more than one group
  int32_t* grp_row = nullptr;       // [n_groups]
  hgnn_half* gstage = nullptr;      // [n_gslots][max_F]
  // column slices (hgnn_plan_add_slices): slice s holds the columns [s*slice_w, (s+1)*slice_w); the edge-score and
  // column-sum kernels keep one slice's per-column scalars in LDS
  int32_t ns = 0;                   // slices; 0 = not built
  int32_t slice_w = 0;
  int32_t nch = 0;                  // row chunks of about nnz / nch non-zeros each (a multiple of 8)
  int32_t* scut = nullptr;          // [ns+1][nrows] first CSR position of row r whose column is >= s*slice_w
  int32_t* chunk_row = nullptr;     // [nch+1]
  unsigned long long* col_part = nullptr;  // [nch][ncols] fixed-point partial column sums of the row chunks
  float* col_poison = nullptr;      // [ncols] sums of non-finite inputs; zero between calls
};

namespace hgnn {
// el[i,h] = a_l[h].U[i,h] and er[j,h] = a_r[h].Vt[j,h] into the plan's fp32 scratch (el first, then er;
// Vt == nullptr skips er)
hgnn_status gat_project(const hgnn_plan* p, const hgnn_csr* g, int H, int D, const hgnn_half* U, int64_t ldu,
                        const hgnn_half* Vt, int64_t ldv, const hgnn_half* a_l, const hgnn_half* a_r, hipStream_t s,
                        const char* who);
// argument checks shared by the SpMM entry points, and the plan-free SpMM with the scratch of its hub kernels at
// `scratch` (scratch_bytes of device memory; null: no row is treated as a hub)
hgnn_status check_spmm_args(const char* who, const hgnn_csr* g, const hgnn_half* w, int H, const hgnn_half* X, int64_t ldx,
                            hgnn_half* Y, int64_t ldy, int F, hgnn_reduce op);
hgnn_status spmm_rows(const char* who, const hgnn_csr* g, const hgnn_half* edge_val, int32_t H, const hgnn_half* X,
                      int64_t ldx, hgnn_half* Y, int64_t ldy, int32_t F, hgnn_reduce op, const float* row_scale,
                      void* scratch, size_t scratch_bytes, hipStream_t s);
void device_cache_bytes(int64_t* l2, int64_t* llc);  // of the current device
size_t spmm_hub_scratch_bytes(int32_t nrows, int64_t nnz, int32_t F);  // scratch of the plan-free SpMM's hub kernels alone
hgnn_status plan_build_arrays(hgnn_plan* p, const hgnn_csr* g, hipStream_t s, bool sub);
hgnn_status build_col_blocks(hgnn_plan* p, const hgnn_csr* g, int nb, hipStream_t s);
constexpr int kSliceMaxCols = 16384;  // columns per slice: 8 bytes each fill 128 KB of the 160 KB of LDS a workgroup may hold
hgnn_status build_col_slices(hgnn_plan* p, const hgnn_csr* g, int W, hipStream_t s);
hgnn_status slice_edge_score(const hgnn_plan* p, const hgnn_csr* g, const float* el, const float* er, const float* lse,
                             float slope, hgnn_half* out, hipStream_t s);
}  // namespace hgnn
