// Internal definitions shared by the translation units of libhgnn.so (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

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

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// smallest power of two >= v (v >= 1)
inline int pow2_at_least(int v) {
  int p = 1;
  while (p < v) p <<= 1;
  return p;
}

hgnn_status check_csr_args(const hgnn_csr* g, const char* who);

}  // namespace hgnn

// The plan object behind the opaque handle of the C ABI.
struct hgnn_plan {
  int32_t nrows = 0, ncols = 0;
  int64_t nnz = 0;
  int32_t S = 0;        // edges per segment
  int64_t nseg = 0;     // ceil(nnz / S)
  int32_t n_split = 0;  // rows whose edges span more than one segment
  int32_t n_big = 0;    // rows longer than big_deg (edge softmax hands them to a whole workgroup)
  int32_t big_deg = 0;
  int32_t max_F = 0, max_H = 0;
  int32_t* seg_row_lo = nullptr;    // [nseg]
  int32_t* seg_row_hi = nullptr;    // [nseg]
  int32_t* split_row = nullptr;     // [n_split]
  int32_t* split_seg_lo = nullptr;  // [n_split]
  int32_t* split_seg_hi = nullptr;  // [n_split]
  int32_t* big_row = nullptr;       // [n_big]
  int32_t* edge_row = nullptr;      // [nnz] COO row ids (owned copy, built from rowptr)
  hgnn_half* staging = nullptr;     // [2*nseg][max_F]
  float* vscratch = nullptr;        // [(nrows + ncols) * max_H] fp32
};
