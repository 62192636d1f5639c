// Selected-row attention for callers that cannot allocate device memory (code under HIP graph
// capture, tight serving loops, harnesses that forbid hipMalloc): the scratch that
// ct_selected_attention takes from the caller's workspace lives in a device array of this
// library instead.
//
// Every GPU the library runs on holds its own copy of the array, at its own address, until the
// process ends.  The array's name is a host-side stand-in in host code, not a device address: the
// address is looked up once per device with hipGetSymbolAddress and that pointer is what the
// kernels get.  All calls on one GPU share the array: calls that overlap in time on one GPU race.
#include <mutex>

#include "ct_internal.h"

namespace ct {

namespace {

constexpr size_t kStaticScratchBytes = (size_t)64 << 20;   // 64 MiB per GPU
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {nullptr};

// Device address of `scratch` on the current device (looked up on the first call on that device).
ct_status static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) return fail(CT_ERR_UNSUPPORTED, "device ordinal %d is beyond %d", dev, kMaxDevices - 1);
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress (static scratch)");
    if (p == nullptr || ((uintptr_t)p & 255) != 0) return fail(CT_ERR_HIP, "static scratch has no usable device address");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return CT_OK;
}

}  // namespace

}  // namespace ct

using namespace ct;

extern "C" {

size_t ct_static_scratch_bytes(void) { return kStaticScratchBytes; }

ct_status ct_selected_attention_static(const ct_layer_cfg* cfg, const void* q_sel, const void* k_buf, const void* v_buf,
                                       int32_t n_ctx, const int32_t* sel_idx, int32_t n_sel, void* out, float* lse,
                                       void* stream) {
  ct_status st = check_cfg(cfg);
  if (st != CT_OK) return st;
  if (n_ctx <= 0 || n_sel < 0) return fail(CT_ERR_SHAPE, "bad size (n_ctx %d, n_sel %d)", n_ctx, n_sel);
  if (n_sel > n_ctx) return fail(CT_ERR_SHAPE, "n_sel %d exceeds n_ctx %d", n_sel, n_ctx);
  if (n_sel == 0) return CT_OK;
  if (!q_sel || !k_buf || !v_buf || !sel_idx || !out)
    return fail(CT_ERR_NULL, "q_sel, k_buf, v_buf, sel_idx and out must be non-NULL");
  if ((st = check_kv_extent(cfg, n_ctx)) != CT_OK) return st;
  const size_t need = attention_scratch_bytes(cfg, n_ctx, n_sel);
  if (need > kStaticScratchBytes)
    return fail(CT_ERR_WORKSPACE,
                "this problem (n_ctx %d, n_sel %d) needs %zu bytes of scratch, the static array holds %zu: "
                "use ct_selected_attention with a workspace of the caller's",
                n_ctx, n_sel, need, kStaticScratchBytes);
  void* ptr = nullptr;
  if ((st = static_scratch(&ptr)) != CT_OK) return st;
  return launch_attention(cfg, q_sel, k_buf, v_buf, n_ctx, sel_idx, n_sel, out, lse, ptr, static_cast<hipStream_t>(stream));
}

}  // extern "C"
