// hgnn_spmm_static: the plan-free SpMM for callers that cannot allocate and have no workspace to hand over (code under
// HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  Same kernels as hgnn_spmm; the scratch of
// the hub kernels (chunk and hub lists, one fp32 partial row per 512-edge chunk of a long row) is a static device array
// of kStaticScratchBytes instead of a caller's workspace.  Every device the library runs on holds its own copy of
// the array until the process ends.  All calls on one device share it: it keeps the previous call's contents (the
// kernels reset the two counters they start from and overwrite what they read), and calls that overlap in time on one
// device race.
#include "common.h"

#include <mutex>

namespace hgnn {

// In host code the array's name is only a handle for hipGetSymbolAddress; the address that kernels use is looked up
// once per device (with that device current) and kept.
constexpr size_t kStaticScratchBytes = size_t(32) << 20;
static __device__ __align__(256) unsigned char g_spmm_scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices] = {};
static std::mutex g_scratch_mutex;

static hgnn_status static_scratch(void** out) {
  int dev = 0;
  HGNN_HIP(hipGetDevice(&dev));
  HGNN_REQUIRE(dev >= 0 && dev < kMaxDevices, HGNN_EUNSUPPORTED, "hgnn_spmm_static: device ordinal %d not supported", dev);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    HGNN_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_spmm_scratch)));
    HGNN_REQUIRE(ptr != nullptr, HGNN_EHIP, "hgnn_spmm_static: the scratch array has no device address");
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return HGNN_OK;
}

}  // namespace hgnn

using namespace hgnn;

extern "C" {

size_t hgnn_spmm_static_limit(void) { return kStaticScratchBytes; }

hgnn_status hgnn_spmm_static(const hgnn_csr* g, const hgnn_half* edge_val, int32_t H, const hgnn_half* X, int64_t ldx,
                             hgnn_half* Y, int64_t ldy, int32_t F, hgnn_reduce op, const float* row_scale, void* stream) {
  clear_error();
  const char* who = "hgnn_spmm_static";
  hgnn_status st = check_spmm_args(who, g, edge_val, H, X, ldx, Y, ldy, F, op);
  if (st != HGNN_OK) return st;
  if (g->nrows == 0) return HGNN_OK;
  const size_t need = spmm_hub_scratch_bytes(g->nrows, g->nnz, F);
  HGNN_REQUIRE(need <= kStaticScratchBytes, HGNN_EUNSUPPORTED,
               "%s: a graph of %lld non-zeros with F = %d needs %zu bytes of scratch, the static array holds %zu; use hgnn_spmm "
               "with a workspace", who, (long long)g->nnz, F, need, kStaticScratchBytes);
  void* scratch = nullptr;
  st = static_scratch(&scratch);
  if (st != HGNN_OK) return st;
  // the array is offered as the scratch of the long rows and nothing more: one sweep per row, never column passes
  return spmm_rows(who, g, edge_val, H, X, ldx, Y, ldy, F, op, row_scale, scratch, need, static_cast<hipStream_t>(stream));
}

}  // extern "C"
