// Host side of libcachetune: argument validation (before any HIP call), error reporting,
// opt-in event profiling and the stream/event orchestration of one partial-prefill layer
// (Sec. 4.2: Transfer stream + Recompute stream coordinated by events; cost model Eq. 9).
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>
#include <vector>

#include "ct_internal.h"

namespace ct {

// ------------------------------------------------------------------------------ errors
static thread_local char g_err[512] = "";

ct_status fail(ct_status code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

ct_status hip_fail(hipError_t e, const char* what) {
  return fail(CT_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

static bool is_pow2(int x) { return x > 0 && (x & (x - 1)) == 0; }

ct_status check_cfg(const ct_layer_cfg* cfg) {
  if (cfg == nullptr) return fail(CT_ERR_NULL, "cfg is NULL");
  if (cfg->hidden <= 0 || cfg->n_q_heads <= 0 || cfg->n_kv_heads <= 0 || cfg->head_dim <= 0)
    return fail(CT_ERR_SHAPE, "cfg sizes must be positive (hidden %d, heads %d/%d, head_dim %d)", cfg->hidden,
                cfg->n_q_heads, cfg->n_kv_heads, cfg->head_dim);
  if (cfg->n_q_heads % cfg->n_kv_heads != 0)
    return fail(CT_ERR_SHAPE, "n_q_heads %d is not a multiple of n_kv_heads %d", cfg->n_q_heads, cfg->n_kv_heads);
  if (cfg->head_dim != 64 && cfg->head_dim != 128)
    return fail(CT_ERR_UNSUPPORTED, "head_dim %d: only 64 and 128 are supported", cfg->head_dim);
  const int g = cfg->n_q_heads / cfg->n_kv_heads;
  if (!is_pow2(g) || g > 16) return fail(CT_ERR_UNSUPPORTED, "group size %d: supported are 1, 2, 4, 8, 16", g);
  if (cfg->hidden % 64 != 0) return fail(CT_ERR_UNSUPPORTED, "hidden %d is not a multiple of 64", cfg->hidden);
  if (cfg->rope_style != 0 && cfg->rope_style != 1)
    return fail(CT_ERR_UNSUPPORTED, "rope_style %d: 0 (half-split) or 1 (interleaved)", cfg->rope_style);
  if (!(cfg->rope_theta > 0.0) || !isfinite(cfg->rope_theta))
    return fail(CT_ERR_SHAPE, "rope_theta must be positive and finite");
  if (!(cfg->softmax_scale >= 0.0f) || !isfinite(cfg->softmax_scale))
    return fail(CT_ERR_SHAPE, "softmax_scale must be >= 0 (0 selects 1/sqrt(head_dim))");
  return CT_OK;
}

void fill_rope_table(const ct_layer_cfg* cfg, RopeTable* t) {
  const int half = cfg->head_dim / 2;
  const double two_pi = 6.283185307179586476925286766559;
  for (int j = 0; j < 64; ++j) {
    t->turns[j] = j < half ? pow(cfg->rope_theta, -2.0 * (double)j / (double)cfg->head_dim) / two_pi : 0.0;
  }
}

// ------------------------------------------------------------------------------ profiling
struct ProfClass {
  std::vector<hipEvent_t> start, stop;
  size_t used = 0;
};
static std::mutex g_prof_mu;
static bool g_prof_on = false;
static ProfClass g_prof[KC_COUNT];

void prof_events(KernelClass kc, hipEvent_t* start, hipEvent_t* stop) {
  *start = nullptr;
  *stop = nullptr;
  if (!g_prof_on) return;
  std::lock_guard<std::mutex> lk(g_prof_mu);
  ProfClass& p = g_prof[kc];
  if (p.used == p.start.size()) {
    hipEvent_t a, b;
    if (hipEventCreate(&a) != hipSuccess) return;
    if (hipEventCreate(&b) != hipSuccess) {
      (void)hipEventDestroy(a);
      return;
    }
    p.start.push_back(a);
    p.stop.push_back(b);
  }
  const size_t slot = p.used++;
  *start = p.start[slot];
  *stop = p.stop[slot];
}

// ------------------------------------------------------------------------------ stream-ordering events
ct_status pooled_events(size_t n, hipEvent_t** out) {
  static thread_local std::vector<hipEvent_t> pool;
  while (pool.size() < n) {
    hipEvent_t e;
    hipError_t err = hipEventCreateWithFlags(&e, hipEventDisableTiming);
    if (err != hipSuccess) return hip_fail(err, "hipEventCreate");
    pool.push_back(e);
  }
  *out = pool.data();
  return CT_OK;
}

// ------------------------------------------------------------------------------ planning
AttnPlan plan_attention(const ct_layer_cfg* cfg, int n_ctx, int n_sel) {
  AttnPlan p;
  const int g = cfg->n_q_heads / cfg->n_kv_heads;
  p.tile_tokens = 256 / g;
  p.n_tiles = (n_sel + p.tile_tokens - 1) / p.tile_tokens;
  p.n_splits = 1;
  p.split_keys = n_ctx;
  p.ws_bytes = 0;
  // Split the key range only when the (tile, kv head) pairs alone leave compute units idle:
  // measured on MI355X, an unsplit launch wins as soon as there are about 1.5 pairs per
  // compute unit (each split costs an fp32 partial (O, m, l) round trip and a merge kernel).
  const long pairs = (long)p.n_tiles * cfg->n_kv_heads;
  static const long target = []() {                     // tuning knob: split below this many (tile, head) pairs
    const char* v = getenv("CT_ATTN_SPLIT_TARGET");
    return v != nullptr && atol(v) > 0 ? atol(v) : 384L;  // 1.5 x 256 compute units
  }();
  if (pairs > 0 && pairs < target && n_ctx > 2048) {
    int want = (int)((target + pairs - 1) / pairs);
    int keys = (n_ctx + want - 1) / want;
    keys = ((keys + 1023) / 1024) * 1024;               // whole K tiles, not too small
    if (keys < 2048) keys = 2048;
    static const int forced = []() {                    // tuning knob: keys per split
      const char* v = getenv("CT_ATTN_SPLIT_KEYS");
      return v != nullptr ? atoi(v) : 0;
    }();
    if (forced >= 64) keys = (forced + 63) / 64 * 64;
    int ns = (n_ctx + keys - 1) / keys;
    if (ns > 1) {
      p.n_splits = ns;
      p.split_keys = keys;
      const size_t cols = 256;
      const size_t per_item = cols * (size_t)(cfg->head_dim + 2) * sizeof(float);
      p.ws_bytes = (size_t)p.n_tiles * cfg->n_kv_heads * ns * per_item;
    }
  }
  return p;
}

size_t attention_scratch_bytes(const ct_layer_cfg* cfg, int n_ctx, int n_sel) {
  return plan_attention(cfg, n_ctx, n_sel).ws_bytes;
}

size_t attention_state_bytes(const ct_layer_cfg* cfg, int n_ctx, int n_sel) {
  const AttnPlan p = plan_attention(cfg, n_ctx, n_sel);
  return (size_t)p.n_tiles * cfg->n_kv_heads * 256 * (size_t)(cfg->head_dim + 2) * sizeof(float);
}

// The attention kernel forms key-row byte offsets in 32 bits from a 24-bit row number.
ct_status check_kv_extent(const ct_layer_cfg* cfg, int64_t n_ctx) {
  if ((uint64_t)n_ctx * cfg->n_kv_heads * cfg->head_dim * 2 > 0xffffffffull)
    return fail(CT_ERR_UNSUPPORTED, "K/V buffers beyond 4 GiB each (n_ctx %lld) are not supported", (long long)n_ctx);
  if (n_ctx >= (1 << 24)) return fail(CT_ERR_UNSUPPORTED, "n_ctx %lld: at most 2^24 - 1 rows are supported", (long long)n_ctx);
  return CT_OK;
}

// The projection kernel forms byte offsets into `hidden` and `wqkv` in 32 bits.
static ct_status check_qkv_extent(const ct_layer_cfg* cfg, int64_t hidden_rows_spanned) {
  const uint64_t o = (uint64_t)(cfg->n_q_heads + 2 * cfg->n_kv_heads) * cfg->head_dim;
  if (o * cfg->hidden * 2 > 0xffffffffull) return fail(CT_ERR_UNSUPPORTED, "wqkv beyond 4 GiB is not supported");
  if ((uint64_t)hidden_rows_spanned * cfg->hidden * 2 > 0xffffffffull)
    return fail(CT_ERR_UNSUPPORTED, "hidden rows beyond 4 GiB from the base (%lld rows of %d) are not supported",
                (long long)hidden_rows_spanned, cfg->hidden);
  return CT_OK;
}

static ct_status check_indices_host(const int32_t* idx, int32_t n_sel, int32_t n_ctx) {
  for (int32_t i = 0; i < n_sel; ++i) {
    if (idx[i] < 0 || idx[i] >= n_ctx)
      return fail(CT_ERR_INDEX, "index %d at ordinal %d is outside [0, %d)", idx[i], i, n_ctx);
    if (i > 0 && idx[i] <= idx[i - 1])
      return fail(CT_ERR_INDEX, "indices not strictly ascending at ordinal %d (%d after %d)", i, idx[i], idx[i - 1]);
  }
  return CT_OK;
}

// Nothing but MFMAs on four independent accumulators per wave: the rate the matrix cores
// sustain on this device (power-limited well below the published peak).
__global__ __launch_bounds__(512) void mfma_rate_kernel(float* out, int iters) {
  bf16x8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    // operands that look like data (uniform in [-2, 2)): the rate is power-limited and depends on
    // how many bits toggle - small integers run at nearly the published peak, such data does not
    uint32_t h = (threadIdx.x * 8u + i + blockIdx.x * 4099u) * 2654435761u;
    h ^= h >> 15;
    a[i] = (__bf16)(((int)(h & 0xffff) - 32768) * (1.0f / 16384.0f));
    b[i] = (__bf16)(((int)(h >> 16) - 32768) * (1.0f / 16384.0f));
  }
  f32x16 c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
      c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
      c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
      c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
    }
  }
  out[blockIdx.x * 512 + threadIdx.x] = c0[0] + c1[1] + c2[2] + c3[3];
}

// Device-visible address of pinned host memory, or nullptr when `p` is not mapped for the device
// (pageable memory, or anything the runtime does not know).
static const void* device_view_of_host(const void* p) {
  hipPointerAttribute_t attr;
  memset(&attr, 0, sizeof(attr));
  if (hipPointerGetAttributes(&attr, p) != hipSuccess) {
    (void)hipGetLastError();   // unknown pointer: not an error of ours
    return nullptr;
  }
  if (attr.type != hipMemoryTypeHost || attr.devicePointer == nullptr) return nullptr;
  return attr.devicePointer;
}

// Workgroups (of 1024 threads) of the stream-in kernel.  Eight keep the host link at about 55 GB/s
// on MI355X (four: 45 GB/s); every further one takes a compute unit away from the kernels of the recompute
// stream and slows them more than the faster transfer gains.
int stream_in_blocks() {
  static const int v = []() {
    const char* e = getenv("CT_STREAM_IN_BLOCKS");
    const int n = e != nullptr ? atoi(e) : 0;
    return n > 0 ? n : 8;
  }();
  return v;
}

bool stream_in_skips_selected() {
  static const bool v = []() {
    const char* e = getenv("CT_STREAM_IN_SKIP_SELECTED");
    return e == nullptr || atoi(e) != 0;
  }();
  return v;
}

ct_status stream_in_host_chunks(const ct_layer_cfg* cfg, const ct_chunk* chunks, int n_chunks, const ChunkTable& tab,
                                void* k_buf, void* v_buf, const int32_t* sel_idx, int32_t n_sel, hipStream_t xs,
                                bool* done, const int* group_sizes, int n_groups, stream_in_group_fn after_group,
                                void* ctx) {
  *done = false;
  static const bool enabled = []() {
    const char* e = getenv("CT_STREAM_IN");
    return e == nullptr || atoi(e) != 0;
  }();
  if (!enabled) return CT_OK;
  const void* kview[64];
  const void* vview[64];
  for (int c = 0; c < n_chunks; ++c) {
    if (chunks[c].location == 0) continue;
    kview[c] = device_view_of_host(chunks[c].k);
    vview[c] = device_view_of_host(chunks[c].v);
    if (kview[c] == nullptr || vview[c] == nullptr) {
      if (chunks[c].location == 2)
        return fail(CT_ERR_UNSUPPORTED, "chunk %d: a compact pool must be in pinned host memory the device can address", c);
      return CT_OK;   // caller falls back to copies
    }
  }
  ReropeChunks rc;
  memset(&rc, 0, sizeof(rc));
  const bool skip_selected = stream_in_skips_selected();
  int last_chunk = -1, group = 0;
  auto flush = [&]() -> ct_status {
    if (rc.n == 0) return CT_OK;
    ++group;
    rc.tok_start[rc.n] = rc.total_tokens;
    rc.skip_rows = (skip_selected || rc.compact_mask != 0) && n_sel > 0 ? sel_idx : nullptr;
    rc.n_skip = n_sel;
    ct_status r = launch_rerope_chunks(cfg, k_buf, v_buf, &rc, stream_in_blocks(), xs);
    rc.n = 0;
    rc.total_tokens = 0;
    rc.compact_mask = 0;
    if (r == CT_OK && after_group != nullptr) r = after_group(ctx, last_chunk);
    return r;
  };
  auto per_launch = [&]() {   // chunks the launch being filled may hold
    const int want = group_sizes != nullptr && group < n_groups - 1 ? group_sizes[group] : 32;
    return want > 0 && want < 32 ? want : 32;
  };
  for (int c = 0; c < n_chunks; ++c) {
    const ct_chunk& ch = chunks[c];
    if (ch.location == 0) continue;
    const int i = rc.n++;
    if (ch.location == 2) rc.compact_mask |= 1u << i;
    rc.tok_start[i] = rc.total_tokens;
    rc.total_tokens += ch.n_tokens;
    rc.k_src[i] = kview[c];
    rc.v_src[i] = vview[c];
    rc.row_start[i] = tab.row_start[c];
    rc.delta0[i] = ch.raw_keys ? ch.new_pos_start : ch.new_pos_start - ch.old_pos_start;
    rc.delta_step[i] = ch.raw_keys ? 1 : 0;
    last_chunk = c;
    if (rc.n == per_launch()) {
      ct_status st = flush();
      if (st != CT_OK) return st;
    }
  }
  ct_status st = flush();
  if (st != CT_OK) return st;
  *done = true;
  return CT_OK;
}

}  // namespace ct

using namespace ct;

// ================================================================================ C ABI
extern "C" {

const char* ct_last_error(void) { return g_err; }
const char* ct_version(void) { return "cachetune-gfx950 0.1"; }

void ct_set_profiling(int32_t on) {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  g_prof_on = on != 0;
}



ct_status ct_measure_mfma_rate(void* scratch, int32_t iters, void* stream, double* tflops) {
  if (scratch == nullptr || tflops == nullptr) return fail(CT_ERR_NULL, "scratch and tflops must be non-NULL");
  if (iters <= 0 || iters > (1 << 20)) return fail(CT_ERR_SHAPE, "iters %d out of range", iters);
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipEvent_t e0, e1;
  hipError_t e;
  if ((e = hipEventCreate(&e0)) != hipSuccess) return hip_fail(e, "hipEventCreate");
  if ((e = hipEventCreate(&e1)) != hipSuccess) {
    (void)hipEventDestroy(e0);
    return hip_fail(e, "hipEventCreate");
  }
  const int blocks = 256;
  hipLaunchKernelGGL(mfma_rate_kernel, dim3(blocks), dim3(512), 0, s, static_cast<float*>(scratch), 8);   // warm-up
  e = hipEventRecord(e0, s);
  hipLaunchKernelGGL(mfma_rate_kernel, dim3(blocks), dim3(512), 0, s, static_cast<float*>(scratch), iters);
  if (e == hipSuccess) e = hipEventRecord(e1, s);
  if (e == hipSuccess) e = hipEventSynchronize(e1);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (e != hipSuccess) return hip_fail(e, "mfma rate measurement");
  const double flops = (double)blocks * 8 * (double)iters * 64 * 2.0 * 32 * 32 * 16;
  *tflops = flops / ((double)ms * 1e-3) / 1e12;
  return CT_OK;
}

void ct_profile_reset(void) {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  for (int i = 0; i < KC_COUNT; ++i) g_prof[i].used = 0;
}

ct_status ct_profile_read(int32_t kernel_class, int64_t* launches, double* total_ms) {
  if (launches == nullptr || total_ms == nullptr) return fail(CT_ERR_NULL, "launches / total_ms is NULL");
  if (kernel_class < 0 || kernel_class >= KC_COUNT) return fail(CT_ERR_SHAPE, "kernel class %d unknown", kernel_class);
  std::lock_guard<std::mutex> lk(g_prof_mu);
  ProfClass& p = g_prof[kernel_class];
  double sum = 0.0;
  for (size_t i = 0; i < p.used; ++i) {
    hipError_t e = hipEventSynchronize(p.stop[i]);
    if (e != hipSuccess) return hip_fail(e, "hipEventSynchronize (profile)");
    float ms = 0.f;
    e = hipEventElapsedTime(&ms, p.start[i], p.stop[i]);
    if (e != hipSuccess) return hip_fail(e, "hipEventElapsedTime (profile)");
    sum += ms;
  }
  *launches = (int64_t)p.used;
  *total_ms = sum;
  return CT_OK;
}

ct_status ct_validate_indices(const int32_t* host_idx, int32_t n_sel, int32_t n_ctx) {
  if (n_sel < 0 || n_ctx < 0) return fail(CT_ERR_SHAPE, "negative size (n_sel %d, n_ctx %d)", n_sel, n_ctx);
  if (n_sel > n_ctx) return fail(CT_ERR_SHAPE, "n_sel %d exceeds n_ctx %d", n_sel, n_ctx);
  if (n_sel > 0 && host_idx == nullptr) return fail(CT_ERR_NULL, "host_idx is NULL");
  return check_indices_host(host_idx, n_sel, n_ctx);
}

size_t ct_workspace_bytes(const ct_layer_cfg* cfg, int32_t n_ctx, int32_t n_sel) {
  if (check_cfg(cfg) != CT_OK || n_ctx <= 0 || n_sel < 0 || n_sel > n_ctx) return 0;
  // selected-row attention partials (if the key range is split) + the layer call's staging of
  // recomputed q, k, v rows, each region 256-byte aligned
  AttnPlan p = plan_attention(cfg, n_ctx, n_sel);
  auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
  const size_t q = up((size_t)n_sel * cfg->n_q_heads * cfg->head_dim * 2);
  const size_t kv = up((size_t)n_sel * cfg->n_kv_heads * cfg->head_dim * 2);
  return up(p.ws_bytes) + q + 2 * kv + 256;
}

size_t ct_attention_state_bytes(const ct_layer_cfg* cfg, int32_t n_ctx, int32_t n_sel) {
  if (check_cfg(cfg) != CT_OK || n_ctx <= 0 || n_sel <= 0 || n_sel > n_ctx) return 0;
  return (attention_state_bytes(cfg, n_ctx, n_sel) + 255) & ~(size_t)255;
}

ct_status ct_attention_rows_read(const ct_layer_cfg* cfg, const int32_t* sel_idx_host, int32_t n_sel, int32_t n_ctx,
                                 int32_t key_after, int32_t key_upto, int32_t with_state, int32_t* first_row,
                                 int32_t* last_row) {
  ct_status st = check_cfg(cfg);
  if (st != CT_OK) return st;
  if (!sel_idx_host || !first_row || !last_row) return fail(CT_ERR_NULL, "sel_idx_host, first_row and last_row must be non-NULL");
  if (n_ctx <= 0 || n_sel <= 0 || n_sel > n_ctx) return fail(CT_ERR_SHAPE, "bad size (n_ctx %d, n_sel %d)", n_ctx, n_sel);
  if (key_after < 0 || key_upto <= key_after)
    return fail(CT_ERR_SHAPE, "key range [%d, %d) is empty or negative", key_after, key_upto);
  if ((st = check_indices_host(sel_idx_host, n_sel, n_ctx)) != CT_OK) return st;
  return attention_rows_read(cfg, sel_idx_host, n_sel, n_ctx, key_after, key_upto, with_state != 0, first_row, last_row);
}

ct_status ct_qkv_selected(const ct_layer_cfg* cfg, const void* hidden, const int32_t* hidden_rows,
                          const int32_t* sel_pos, int32_t n_sel, const void* wqkv, const void* bias, void* q_out,
                          void* k_out, void* v_out, void* stream) {
  ct_status st = check_cfg(cfg);
  if (st != CT_OK) return st;
  if (n_sel < 0) return fail(CT_ERR_SHAPE, "n_sel %d is negative", n_sel);
  if (n_sel == 0) return CT_OK;
  if (!hidden || !sel_pos || !wqkv || !q_out || !k_out || !v_out)
    return fail(CT_ERR_NULL, "hidden, sel_pos, wqkv, q_out, k_out and v_out must be non-NULL");
  if ((((uintptr_t)hidden | (uintptr_t)wqkv | (uintptr_t)q_out | (uintptr_t)k_out | (uintptr_t)v_out) & 15) != 0)
    return fail(CT_ERR_UNSUPPORTED, "hidden, wqkv, q_out, k_out and v_out must be 16-byte aligned");
  // with a row gather the rows read are the caller's to keep within 4 GiB of the base (device data)
  if ((st = check_qkv_extent(cfg, hidden_rows != nullptr ? 0 : n_sel)) != CT_OK) return st;
  return launch_qkv(cfg, hidden, hidden_rows, sel_pos, nullptr, nullptr, n_sel, wqkv, bias, q_out, k_out, v_out,
                    static_cast<hipStream_t>(stream));
}

ct_status ct_rerope_keys(const ct_layer_cfg* cfg, const void* k_src, void* k_dst, const int32_t* old_pos,
                         const int32_t* new_pos, int32_t n_tokens, void* stream) {
  ct_status st = check_cfg(cfg);
  if (st != CT_OK) return st;
  if (n_tokens < 0) return fail(CT_ERR_SHAPE, "n_tokens %d is negative", n_tokens);
  if (n_tokens == 0) return CT_OK;
  if (!k_src || !k_dst || !new_pos) return fail(CT_ERR_NULL, "k_src, k_dst and new_pos must be non-NULL");
  return launch_rerope(cfg, k_src, k_dst, nullptr, nullptr, old_pos, new_pos, 0, 0, n_tokens,
                       static_cast<hipStream_t>(stream));
}

ct_status ct_rerope_keys_skip(const ct_layer_cfg* cfg, const void* k_src, void* k_dst, const int32_t* old_pos,
                              const int32_t* new_pos, int32_t n_tokens, const int32_t* skip_rows, int32_t n_skip,
                              void* stream) {
  ct_status st = check_cfg(cfg);
  if (st != CT_OK) return st;
  if (n_tokens < 0 || n_skip < 0) return fail(CT_ERR_SHAPE, "negative size (n_tokens %d, n_skip %d)", n_tokens, n_skip);
  if (n_skip > n_tokens) return fail(CT_ERR_SHAPE, "n_skip %d exceeds n_tokens %d", n_skip, n_tokens);
  if (n_tokens == 0) return CT_OK;
  if (!k_src || !k_dst || !new_pos) return fail(CT_ERR_NULL, "k_src, k_dst and new_pos must be non-NULL");
  if (n_skip > 0 && !skip_rows) return fail(CT_ERR_NULL, "skip_rows is NULL but n_skip is %d", n_skip);
  return launch_rerope(cfg, k_src, k_dst, nullptr, nullptr, old_pos, new_pos, 0, 0, n_tokens,
                       static_cast<hipStream_t>(stream), skip_rows, n_skip);
}

ct_status ct_rerope_chunk(const ct_layer_cfg* cfg, const void* k_src, void* k_dst, const void* v_src, void* v_dst,
                          int32_t n_tokens, int32_t old_pos_start, int32_t new_pos_start, int32_t raw_keys,
                          void* stream) {
  ct_status st = check_cfg(cfg);
  if (st != CT_OK) return st;
  if (n_tokens < 0) return fail(CT_ERR_SHAPE, "n_tokens %d is negative", n_tokens);
  if (n_tokens == 0) return CT_OK;
  if (!k_src || !k_dst) return fail(CT_ERR_NULL, "k_src and k_dst must be non-NULL");
  if ((v_src == nullptr) != (v_dst == nullptr)) return fail(CT_ERR_NULL, "v_src and v_dst must be given together");
  const bool copy_v = v_src != nullptr && v_src != v_dst;
  const int32_t d0 = raw_keys ? new_pos_start : new_pos_start - old_pos_start;
  return launch_rerope(cfg, k_src, k_dst, copy_v ? v_src : nullptr, copy_v ? v_dst : nullptr, nullptr, nullptr, d0,
                       raw_keys ? 1 : 0, n_tokens, static_cast<hipStream_t>(stream));
}

ct_status ct_scatter_kv(const ct_layer_cfg* cfg, void* k_buf, void* v_buf, int32_t n_ctx, const void* k_sel,
                        const void* v_sel, const int32_t* sel_idx, int32_t n_sel, void* stream) {
  ct_status st = check_cfg(cfg);
  if (st != CT_OK) return st;
  if (n_ctx < 0 || n_sel < 0) return fail(CT_ERR_SHAPE, "negative size (n_ctx %d, n_sel %d)", n_ctx, n_sel);
  if (n_sel > n_ctx) return fail(CT_ERR_SHAPE, "n_sel %d exceeds n_ctx %d", n_sel, n_ctx);
  if (n_sel == 0) return CT_OK;
  if (!k_buf || !v_buf || !k_sel || !v_sel || !sel_idx)
    return fail(CT_ERR_NULL, "k_buf, v_buf, k_sel, v_sel and sel_idx must be non-NULL");
  return launch_scatter(cfg, k_buf, v_buf, k_sel, v_sel, sel_idx, n_sel, static_cast<hipStream_t>(stream));
}

ct_status ct_selected_attention(const ct_layer_cfg* cfg, const void* q_sel, const void* k_buf, const void* v_buf,
                                int32_t n_ctx, const int32_t* sel_idx, int32_t n_sel, void* out, float* lse,
                                void* workspace, size_t workspace_bytes, void* stream) {
  ct_status st = check_cfg(cfg);
  if (st != CT_OK) return st;
  if (n_ctx <= 0 || n_sel < 0) return fail(CT_ERR_SHAPE, "bad size (n_ctx %d, n_sel %d)", n_ctx, n_sel);
  if (n_sel > n_ctx) return fail(CT_ERR_SHAPE, "n_sel %d exceeds n_ctx %d", n_sel, n_ctx);
  if (n_sel == 0) return CT_OK;
  if (!q_sel || !k_buf || !v_buf || !sel_idx || !out)
    return fail(CT_ERR_NULL, "q_sel, k_buf, v_buf, sel_idx and out must be non-NULL");
  if ((st = check_kv_extent(cfg, n_ctx)) != CT_OK) return st;
  AttnPlan p = plan_attention(cfg, n_ctx, n_sel);
  if (p.ws_bytes > 0) {
    if (workspace == nullptr) return fail(CT_ERR_WORKSPACE, "workspace is NULL but %zu bytes are needed", p.ws_bytes);
    if (workspace_bytes < p.ws_bytes)
      return fail(CT_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, p.ws_bytes);
    if (((uintptr_t)workspace & 255) != 0) return fail(CT_ERR_WORKSPACE, "workspace is not 256-byte aligned");
  }
  return launch_attention(cfg, q_sel, k_buf, v_buf, n_ctx, sel_idx, n_sel, out, lse, workspace,
                          static_cast<hipStream_t>(stream));
}

ct_status ct_partial_prefill_layer(const ct_layer_cfg* cfg, const ct_chunk* chunks, int32_t n_chunks,
                                   const void* hidden, const int32_t* hidden_rows, const int32_t* sel_idx,
                                   int32_t n_sel, double recompute_ratio, const void* wqkv, const void* bias,
                                   void* k_buf, void* v_buf, void* attn_out, void* workspace,
                                   size_t workspace_bytes, void* compute_stream, void* copy_stream) {
  ct_status st = check_cfg(cfg);
  if (st != CT_OK) return st;
  if (chunks == nullptr) return fail(CT_ERR_NULL, "chunks is NULL");
  if (n_chunks <= 0) return fail(CT_ERR_SHAPE, "n_chunks %d must be positive", n_chunks);
  if (n_chunks > 64) return fail(CT_ERR_UNSUPPORTED, "n_chunks %d: at most 64 chunks per call", n_chunks);
  if (n_sel < 0) return fail(CT_ERR_SHAPE, "n_sel %d is negative", n_sel);

  ChunkTable tab;
  memset(&tab, 0, sizeof(tab));
  tab.n = n_chunks;
  int64_t n_ctx64 = 0;
  bool any_host = false, any_compact = false;
  for (int c = 0; c < n_chunks; ++c) {
    const ct_chunk& ch = chunks[c];
    if (ch.n_tokens <= 0) return fail(CT_ERR_SHAPE, "chunk %d has n_tokens %d", c, ch.n_tokens);
    if (ch.k == nullptr || ch.v == nullptr) return fail(CT_ERR_NULL, "chunk %d has a NULL k or v", c);
    if (ch.location < 0 || ch.location > 2) return fail(CT_ERR_SHAPE, "chunk %d has location %d", c, ch.location);
    if (ch.new_pos_start < 0) return fail(CT_ERR_SHAPE, "chunk %d has negative new_pos_start", c);
    if (c > 0) {
      const ct_chunk& pr = chunks[c - 1];
      if ((int64_t)ch.new_pos_start < (int64_t)pr.new_pos_start + pr.n_tokens)
        return fail(CT_ERR_SHAPE, "chunk %d starts at position %d, before chunk %d ends (%lld)", c, ch.new_pos_start,
                    c - 1, (long long)pr.new_pos_start + pr.n_tokens);
    }
    any_host |= ch.location != 0;
    any_compact |= ch.location == 2;
    tab.row_start[c] = (int32_t)n_ctx64;
    tab.new_start[c] = ch.new_pos_start;
    n_ctx64 += ch.n_tokens;
    if (n_ctx64 > 0x7fffffff / 2) return fail(CT_ERR_SHAPE, "context too long");
  }
  const int32_t n_ctx = (int32_t)n_ctx64;
  tab.row_start[n_chunks] = n_ctx;
  if (n_sel > n_ctx) return fail(CT_ERR_SHAPE, "n_sel %d exceeds n_ctx %d", n_sel, n_ctx);
  if ((st = check_kv_extent(cfg, n_ctx)) != CT_OK) return st;
  // hidden_rows, when given, index the context's rows of `hidden`
  if (n_sel > 0 && (st = check_qkv_extent(cfg, hidden_rows != nullptr ? n_ctx : n_sel)) != CT_OK) return st;
  if (recompute_ratio >= 0.0) {
    if (!(recompute_ratio <= 1.0)) return fail(CT_ERR_RATIO, "recompute_ratio %g is above 1", recompute_ratio);
    int64_t want = (int64_t)floor(recompute_ratio * (double)n_ctx + 1e-9);
    if (recompute_ratio > 0.0 && want < 1) want = 1;
    if (want != n_sel)
      return fail(CT_ERR_RATIO, "n_sel %d but floor(%g * %d) = %lld", n_sel, recompute_ratio, n_ctx, (long long)want);
  }
  if (!k_buf || !v_buf) return fail(CT_ERR_NULL, "k_buf and v_buf must be non-NULL");
  if (n_sel > 0) {
    if (!hidden || !sel_idx || !wqkv || !attn_out)
      return fail(CT_ERR_NULL, "hidden, sel_idx, wqkv and attn_out must be non-NULL when n_sel > 0");
    const size_t need = ct_workspace_bytes(cfg, n_ctx, n_sel);
    if (workspace == nullptr) return fail(CT_ERR_WORKSPACE, "workspace is NULL but %zu bytes are needed", need);
    if (workspace_bytes < need) return fail(CT_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, need);
    if (((uintptr_t)workspace & 255) != 0) return fail(CT_ERR_WORKSPACE, "workspace is not 256-byte aligned");
  }
  if (any_host && compute_stream == copy_stream)
    return fail(CT_ERR_SHAPE, "pinned-host chunks need a copy_stream different from compute_stream");

  hipStream_t cs = static_cast<hipStream_t>(compute_stream);
  hipStream_t xs = static_cast<hipStream_t>(copy_stream);
  const size_t row_bytes = (size_t)cfg->n_kv_heads * cfg->head_dim * 2;
  auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };

  // workspace layout: [attention partials][q rows][k rows][v rows]
  char* ws = static_cast<char*>(workspace);
  void *q_rows = nullptr, *k_rows = nullptr, *v_rows = nullptr;
  float* attn_state = nullptr;
  if (n_sel > 0) {
    AttnPlan p = plan_attention(cfg, n_ctx, n_sel);
    size_t off = up(p.ws_bytes);
    q_rows = ws + off;
    off += up((size_t)n_sel * cfg->n_q_heads * cfg->head_dim * 2);
    k_rows = ws + off;
    off += up((size_t)n_sel * row_bytes);
    v_rows = ws + off;
    off += up((size_t)n_sel * row_bytes);
    // room behind the staging rows for the attention state: the attention of host-pool layers can
    // then follow the chunk groups key range by key range
    const size_t state_bytes = attention_state_bytes(cfg, n_ctx, n_sel);
    if (p.n_splits == 1 && workspace_bytes >= off + state_bytes) attn_state = reinterpret_cast<float*>(ws + off);
  }

  // Transfer stream: enqueue every pinned-host chunk's transfer first so the link starts at once.
  // Events (from the per-thread pool): one fence, one per launch of the stream-in kernel (at most
  // 8 groups), or - when the chunks have to be copied - one per chunk.
  hipEvent_t* ev_pool = nullptr;
  if (any_host && (st = pooled_events((size_t)1 + 8 + n_chunks, &ev_pool)) != CT_OK) return st;
  hipEvent_t* landed = ev_pool != nullptr ? ev_pool + 9 : nullptr;   // landed[c]: chunk c has been copied
  // one event per launch of the stream-in kernel, and the last chunk that launch brought in
  struct GroupEvents {
    hipStream_t xs;
    hipEvent_t* ev;
    int n = 0;
    int last_chunk[8];
    static ct_status record(void* self, int last) {
      GroupEvents* g = static_cast<GroupEvents*>(self);
      if (g->n >= 8) return fail(CT_ERR_HIP, "more than 8 stream-in launches in one layer");
      hipError_t err = hipEventRecord(g->ev[g->n], g->xs);
      if (err != hipSuccess) return hip_fail(err, "event after a stream-in launch");
      g->last_chunk[g->n++] = last;
      return CT_OK;
    }
  } groups;
  bool streamed = false, pipelined = false;
  hipError_t e;
  if (any_host) {
    // the copies write k_buf / v_buf: they must not overtake earlier work of the compute
    // stream that still reads the buffers (the previous layer's attention)
    hipEvent_t fence = ev_pool[0];
    e = hipEventRecord(fence, cs);
    if (e == hipSuccess) e = hipStreamWaitEvent(xs, fence, 0);
    if (e != hipSuccess) return hip_fail(e, "fence compute->copy stream");
    // Preferred: a kernel on the transfer stream reads the pinned chunks over the host link,
    // rotates the keys on the way and writes keys and values to their buffer rows (Eq. 8 overlapped
    // with the transfer); one event says that all of them are in place.
    // The chunks go in groups, one launch and one event each, so that the attention of the
    // selected rows that see only the first groups can start while the later ones are still on
    // the link (the chunk-wise overlap of transfer and recomputation of Sec. 4.2).
    int host_chunks = 0;
    for (int c = 0; c < n_chunks; ++c) host_chunks += chunks[c].location != 0;
    pipelined = n_sel > 0 && host_chunks >= 2 && stream_in_skips_selected() &&
                plan_attention(cfg, n_ctx, n_sel).n_splits == 1;
    groups.xs = xs;
    groups.ev = ev_pool + 1;
    // Equal groups of chunks.  Without room for the attention state: as many as leave every
    // attention launch some 200 workgroups (a
    // launch computes the tiles of selected rows between two group ends, for every KV head; with
    // fewer the chip is underfilled and the launches together take longer than the overlap
    // gains: at config 4, 824 tile-head pairs, 4 groups give 13.2 ms, 8 groups 14.9, 2 groups
    // 15.2, one launch after the last chunk 16.9; groups that end at equal attention work
    // instead of equal rows are worse, 13.9 ms at best).
    int sizes[8];
    int n_groups = 0;
    if (pipelined) {
      const AttnPlan plan = plan_attention(cfg, n_ctx, n_sel);
      int G = (int)((int64_t)plan.n_tiles * cfg->n_kv_heads / 200);
      // With room for the attention state a launch takes all unfinished tiles through the keys of
      // one group, so the launches are full whatever the number of groups, and what is left when
      // the transfer ends is the last group's keys: 1 / G^2 of the attention work.  Every further
      // stream-in launch costs the link about 0.1 ms (measured at config 4: 9.34 ms in 2 launches,
      // 9.98 in 8), so G = cbrt(2 x attention time / 0.1 ms) with the attention time estimated at
      // 1.1 PFLOP/s: 5 groups at config 4 (equal groups: 10.3 ms; 4 groups 10.4, 8 groups 10.5, 2
      // groups 12.0).
      if (attn_state != nullptr) {
        static const int forced = []() {                  // tuning knob: number of chunk groups
          const char* v = getenv("CT_ATTN_GROUPS");
          return v != nullptr ? atoi(v) : 0;
        }();
        const double attn_ms = 4.0 * cfg->head_dim * cfg->n_q_heads * (0.5 * (double)n_sel * n_ctx) / 1.1e12;
        G = forced >= 2 ? forced : (int)lround(cbrt(2.0 * attn_ms / 0.1));
        if (G < 2) G = 2;
      }
      if (G > 8) G = 8;
      if (G > host_chunks) G = host_chunks;
      if (G < 2) {
        pipelined = false;
      } else {
        // With the attention state the last group is `last_share` of the others: what is left
        // after the transfer is that group's keys alone, and the work in them goes with the
        // square of the group's size (config 4: 10.0 ms against 10.3 with equal groups; tuning
        // knob CT_ATTN_LAST_GROUP, in per cent).
        static const int last_pct = []() {
          const char* v = getenv("CT_ATTN_LAST_GROUP");
          const int x = v != nullptr ? atoi(v) : 50;
          return x >= 10 && x <= 100 ? x : 50;
        }();
        const double last_share = attn_state != nullptr ? last_pct / 100.0 : 1.0;
        const double unit = host_chunks / (G - 1 + last_share);
        int done_chunks = 0;
        for (int g = 0; g < G; ++g) {
          int upto = g + 1 == G ? host_chunks : (int)lround(unit * (g + 1));
          if (upto <= done_chunks) upto = done_chunks + 1;
          if (upto > host_chunks - (G - 1 - g)) upto = host_chunks - (G - 1 - g);   // every group holds a chunk
          if (upto - done_chunks > 32) upto = done_chunks + 32;   // one launch holds 32 chunks at most
          sizes[n_groups++] = upto - done_chunks;
          done_chunks = upto;
        }
      }
    }
    st = stream_in_host_chunks(cfg, chunks, n_chunks, tab, k_buf, v_buf, sel_idx, n_sel, xs, &streamed,
                               pipelined ? sizes : nullptr, n_groups, &GroupEvents::record, &groups);
    if (st != CT_OK) return st;
    if (!streamed && any_compact) return fail(CT_ERR_UNSUPPORTED, "compact pools are read by the stream-in kernel only");
    // Otherwise (host memory the device cannot address): plain copies, one event per chunk.
    for (int c = 0; c < n_chunks && !streamed; ++c) {
      const ct_chunk& ch = chunks[c];
      if (ch.location != 1) continue;
      char* kd = static_cast<char*>(k_buf) + (size_t)tab.row_start[c] * row_bytes;
      char* vd = static_cast<char*>(v_buf) + (size_t)tab.row_start[c] * row_bytes;
      const size_t bytes = (size_t)ch.n_tokens * row_bytes;
      e = hipMemcpyAsync(kd, ch.k, bytes, hipMemcpyHostToDevice, xs);
      if (e == hipSuccess) e = hipMemcpyAsync(vd, ch.v, bytes, hipMemcpyHostToDevice, xs);
      if (e == hipSuccess) e = hipEventRecord(landed[c], xs);
      if (e != hipSuccess) return hip_fail(e, "host->device chunk copy");
    }
  }

  // The recomputed keys and values go straight from the projection's epilogue to their rows of
  // the layer buffers (the scatter of Sec. 4.2 fused into the GEMM) when nothing else writes those
  // rows afterwards: the launch that rotates device chunks writes every row of its chunks and is
  // issued first; the stream-in kernel leaves the selected rows alone; plain host copies (memory
  // the device cannot address) overwrite them at a time of their own, so then the rows wait in
  // the workspace and a scatter launch follows the copies.
  const bool direct = n_sel > 0 && (!any_host || (streamed && stream_in_skips_selected()));
  // Device-resident chunks: rotated (and their values copied) into place in as few launches
  // as the table size allows; they do not wait for any copy.  Rows of the recompute set are left
  // out: the projection's epilogue (or the scatter) writes them next.
  {
    ReropeChunks rc;
    auto flush = [&]() -> ct_status {
      if (rc.n == 0) return CT_OK;
      rc.tok_start[rc.n] = rc.total_tokens;
      rc.skip_rows = n_sel > 0 ? sel_idx : nullptr;
      rc.n_skip = n_sel;
      ct_status r = launch_rerope_chunks(cfg, k_buf, v_buf, &rc, 0, cs);
      rc.n = 0;
      rc.total_tokens = 0;
      return r;
    };
    memset(&rc, 0, sizeof(rc));
    for (int c = 0; c < n_chunks; ++c) {
      const ct_chunk& ch = chunks[c];
      if (ch.location != 0) continue;
      const char* vd = static_cast<const char*>(v_buf) + (size_t)tab.row_start[c] * row_bytes;
      const int i = rc.n++;
      rc.tok_start[i] = rc.total_tokens;
      rc.total_tokens += ch.n_tokens;
      rc.k_src[i] = ch.k;
      rc.v_src[i] = (ch.v == (const void*)vd) ? nullptr : ch.v;   // already in place: leave the values
      rc.row_start[i] = tab.row_start[c];
      rc.delta0[i] = ch.raw_keys ? ch.new_pos_start : ch.new_pos_start - ch.old_pos_start;
      rc.delta_step[i] = ch.raw_keys ? 1 : 0;
      if (rc.n == 32 && (st = flush()) != CT_OK) return st;
    }
    if ((st = flush()) != CT_OK) return st;
  }
  // Recompute stream: projection of the selected rows runs while the copies are in flight.
  if (n_sel > 0) {
    st = direct ? launch_qkv(cfg, hidden, hidden_rows, nullptr, sel_idx, &tab, n_sel, wqkv, bias, q_rows, k_buf, v_buf, cs,
                             sel_idx)
                : launch_qkv(cfg, hidden, hidden_rows, nullptr, sel_idx, &tab, n_sel, wqkv, bias, q_rows, k_rows, v_rows, cs);
    if (st != CT_OK) return st;
  }
  // Pinned-host chunks: already rotated by the stream-in kernel, or rotated in place chunk by
  // chunk as soon as each copy has landed.
  if (streamed && pipelined) {
    // The recomputed rows are not among those the stream-in kernel writes, so they are in their
    // slots already; one attention launch per group of chunks, each for the selected rows whose
    // last visible key that group completes.
    int32_t seen = 0;
    for (int j = 0; j < groups.n; ++j) {
      if ((e = hipStreamWaitEvent(cs, groups.ev[j], 0)) != hipSuccess)
        return hip_fail(e, "hipStreamWaitEvent (chunk group streamed in)");
      const int32_t upto = j + 1 == groups.n ? 0x7fffffff : tab.row_start[groups.last_chunk[j] + 1];
      st = launch_attention(cfg, q_rows, k_buf, v_buf, n_ctx, sel_idx, n_sel, attn_out, nullptr, workspace, cs, seen, upto,
                            attn_state);
      if (st != CT_OK) return st;
      seen = upto;
    }
    return CT_OK;
  }
  if (streamed && groups.n > 0 && (e = hipStreamWaitEvent(cs, groups.ev[groups.n - 1], 0)) != hipSuccess)
    return hip_fail(e, "hipStreamWaitEvent (chunks streamed in)");
  for (int c = 0; c < n_chunks && any_host && !streamed; ++c) {
    const ct_chunk& ch = chunks[c];
    if (ch.location != 1) continue;
    char* kd = static_cast<char*>(k_buf) + (size_t)tab.row_start[c] * row_bytes;
    if ((e = hipStreamWaitEvent(cs, landed[c], 0)) != hipSuccess) return hip_fail(e, "hipStreamWaitEvent (chunk landed)");
    const int32_t d0 = ch.raw_keys ? ch.new_pos_start : ch.new_pos_start - ch.old_pos_start;
    // (rotates the chunk's stale selected rows too; the scatter below overwrites them)
    if ((st = launch_rerope(cfg, kd, kd, nullptr, nullptr, nullptr, nullptr, d0, ch.raw_keys ? 1 : 0, ch.n_tokens, cs)) != CT_OK)
      return st;
  }
  if (n_sel == 0) return CT_OK;
  if (!direct && (st = launch_scatter(cfg, k_buf, v_buf, k_rows, v_rows, sel_idx, n_sel, cs)) != CT_OK) return st;
  return launch_attention(cfg, q_rows, k_buf, v_buf, n_ctx, sel_idx, n_sel, attn_out, nullptr, workspace, cs);
}

}  // extern "C"
