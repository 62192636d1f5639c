// The rest of a transformer layer on the selected rows, and the multi-layer partial prefill.
//
// After the check layer every layer works on the selected tokens only (Sec. 4.2: fusion
// layers): RMSNorm -> selective QKV recompute, KV fusion, selected-row attention -> output
// projection + residual -> RMSNorm -> SwiGLU FFN + residual.  The stack entry point chains
// the layers and streams each layer's reused KV from pinned host memory one layer ahead on
// the transfer stream into one of two layer buffers (Sec. 4.2 "Hiding external-cache transfer
// overhead"; steady-state cost model Eq. 10).
#include <string.h>

#include "ct_internal.h"

namespace ct {

namespace {

// One wave per row: sum of squares in fp32, wave reduction, second pass scales and rounds.
// The launch asks for kKeepOutLdsBytes of dynamic LDS that the kernel does not use: that keeps the
// workgroups off the compute units on which the stream-in kernel of the transfer stream sits (which
// claims the other half), where every memory access would wait behind that kernel's loads from host
// memory.
constexpr int kNormRows = 16;
__global__ __launch_bounds__(64 * kNormRows) void rmsnorm_kernel(const uint16_t* __restrict__ x,
                                                                const uint16_t* __restrict__ w,
                                                                uint16_t* __restrict__ out, int32_t n_tok, int32_t width,
                                                                float eps) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * kNormRows + (threadIdx.x >> 6);
  if (row >= n_tok) return;
  const u32x4* xr = reinterpret_cast<const u32x4*>(x + row * width);
  const u32x4* wr = reinterpret_cast<const u32x4*>(w);
  u32x4* orow = reinterpret_cast<u32x4*>(out + row * width);
  const int pieces = width / 8;
  float ss = 0.f;
  for (int p = lane; p < pieces; p += 64) {
    const u32x4 v = xr[p];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float a = bf16_lo(v[i]), b = bf16_hi(v[i]);
      ss += a * a + b * b;
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) ss += __shfl_xor(ss, off);
  const float scale = 1.0f / sqrtf(ss / (float)width + eps);
  for (int p = lane; p < pieces; p += 64) {
    const u32x4 v = xr[p];
    const u32x4 g = wr[p];
    u32x4 r;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      r[i] = pack_bf16(bf16_lo(v[i]) * scale * bf16_lo(g[i]), bf16_hi(v[i]) * scale * bf16_hi(g[i]));
    orow[p] = r;
  }
}

size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }

struct StackLayout {
  size_t attn_ws, x_norm, q, k, v, attn_out, act, gemm_ws, gemm_ws_bytes, total;
};

StackLayout stack_layout(const ct_layer_cfg* cfg, int32_t ffn_dim, int32_t n_ctx, int32_t n_sel) {
  StackLayout L;
  const AttnPlan p = plan_attention(cfg, n_ctx, n_sel);
  size_t off = 0;
  L.attn_ws = off;  off += up256(p.ws_bytes);
  L.x_norm = off;   off += up256((size_t)n_sel * cfg->hidden * 2);
  L.q = off;        off += up256((size_t)n_sel * cfg->n_q_heads * cfg->head_dim * 2);
  L.k = off;        off += up256((size_t)n_sel * cfg->n_kv_heads * cfg->head_dim * 2);
  L.v = off;        off += up256((size_t)n_sel * cfg->n_kv_heads * cfg->head_dim * 2);
  L.attn_out = off; off += up256((size_t)n_sel * cfg->n_q_heads * cfg->head_dim * 2);
  L.act = off;      off += up256((size_t)n_sel * ffn_dim * 2);
  // scratch of the two linear launches (output projection, FFN down projection)
  const size_t g1 = linear_workspace_bytes(n_sel, cfg->n_q_heads * cfg->head_dim, cfg->hidden);
  const size_t g2 = linear_workspace_bytes(n_sel, ffn_dim, cfg->hidden);
  L.gemm_ws_bytes = g1 > g2 ? g1 : g2;
  L.gemm_ws = off;  off += up256(L.gemm_ws_bytes);
  L.total = off + 256;
  return L;
}

}  // namespace

ct_status launch_rmsnorm(const void* x, const void* w, float eps, int32_t n_tok, int32_t width, void* out, hipStream_t s) {
  if (n_tok == 0) return CT_OK;
  static const hipError_t allowed = hipFuncSetAttribute(reinterpret_cast<const void*>(rmsnorm_kernel),
                                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)kKeepOutLdsBytes);
  if (allowed != hipSuccess) return hip_fail(allowed, "hipFuncSetAttribute (rmsnorm kernel LDS)");
  launch_kernel(KC_NORM, rmsnorm_kernel, dim3((n_tok + kNormRows - 1) / kNormRows), dim3(64 * kNormRows), kKeepOutLdsBytes, s,
                static_cast<const uint16_t*>(x), static_cast<const uint16_t*>(w), static_cast<uint16_t*>(out), n_tok, width,
                eps);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(e, "rmsnorm kernel launch");
  return CT_OK;
}

}  // namespace ct

using namespace ct;

extern "C" {

ct_status ct_rmsnorm(const void* x, const void* weight, float eps, int32_t n_tokens, int32_t width, void* out, void* stream) {
  if (n_tokens < 0 || width <= 0) return fail(CT_ERR_SHAPE, "bad size (n_tokens %d, width %d)", n_tokens, width);
  if (width % 8 != 0) return fail(CT_ERR_UNSUPPORTED, "width %d is not a multiple of 8", width);
  if (!(eps >= 0.f)) return fail(CT_ERR_SHAPE, "eps must be >= 0");
  if (n_tokens == 0) return CT_OK;
  if (!x || !weight || !out) return fail(CT_ERR_NULL, "x, weight and out must be non-NULL");
  return launch_rmsnorm(x, weight, eps, n_tokens, width, out, static_cast<hipStream_t>(stream));
}

static ct_status check_gemm_shape(int32_t n_tokens, int32_t k_len, int32_t n_out) {
  if (n_tokens < 0 || k_len <= 0 || n_out <= 0)
    return fail(CT_ERR_SHAPE, "bad size (n_tokens %d, k_len %d, n_out %d)", n_tokens, k_len, n_out);
  if (k_len % 64 != 0) return fail(CT_ERR_UNSUPPORTED, "k_len %d is not a multiple of 64", k_len);
  if (n_out % 64 != 0) return fail(CT_ERR_UNSUPPORTED, "n_out %d is not a multiple of 64", n_out);
  if ((uint64_t)n_out * k_len * 2 > 0xffffffffull || (uint64_t)n_tokens * k_len * 2 > 0xffffffffull)
    return fail(CT_ERR_UNSUPPORTED, "operands beyond 4 GiB are not supported");
  return CT_OK;
}

ct_status ct_linear(const void* x, int32_t n_tokens, int32_t k_len, const void* w, int32_t n_out, const void* residual,
                    void* out, void* stream) {
  ct_status st = check_gemm_shape(n_tokens, k_len, n_out);
  if (st != CT_OK) return st;
  if (n_tokens == 0) return CT_OK;
  if (!x || !w || !out) return fail(CT_ERR_NULL, "x, w and out must be non-NULL");
  if ((((uintptr_t)x | (uintptr_t)w | (uintptr_t)out | (uintptr_t)residual) & 15) != 0)
    return fail(CT_ERR_UNSUPPORTED, "x, w, residual and out must be 16-byte aligned");
  return launch_linear(x, n_tokens, k_len, w, n_out, residual, out, nullptr, 0, kNumCUs, static_cast<hipStream_t>(stream));
}

size_t ct_linear_workspace_bytes(int32_t n_tokens, int32_t k_len, int32_t n_out) {
  if (n_tokens <= 0 || k_len <= 0 || n_out <= 0) return 0;
  return linear_workspace_bytes(n_tokens, k_len, n_out);
}

ct_status ct_linear_ws(const void* x, int32_t n_tokens, int32_t k_len, const void* w, int32_t n_out, const void* residual,
                       void* out, void* workspace, size_t workspace_bytes, void* stream) {
  return ct_linear_ws_cus(x, n_tokens, k_len, w, n_out, residual, out, workspace, workspace_bytes, kNumCUs, stream);
}

ct_status ct_linear_ws_cus(const void* x, int32_t n_tokens, int32_t k_len, const void* w, int32_t n_out, const void* residual,
                           void* out, void* workspace, size_t workspace_bytes, int32_t n_compute_units, void* stream) {
  ct_status st = check_gemm_shape(n_tokens, k_len, n_out);
  if (st != CT_OK) return st;
  if (n_compute_units < 1 || n_compute_units > kNumCUs)
    return fail(CT_ERR_SHAPE, "n_compute_units %d is outside [1, %d]", n_compute_units, kNumCUs);
  if (n_tokens == 0) return CT_OK;
  if (!x || !w || !out) return fail(CT_ERR_NULL, "x, w and out must be non-NULL");
  if ((((uintptr_t)x | (uintptr_t)w | (uintptr_t)out | (uintptr_t)residual) & 15) != 0)
    return fail(CT_ERR_UNSUPPORTED, "x, w, residual and out must be 16-byte aligned");
  if (workspace != nullptr && ((uintptr_t)workspace & 15) != 0)
    return fail(CT_ERR_WORKSPACE, "workspace is not 16-byte aligned");
  return launch_linear(x, n_tokens, k_len, w, n_out, residual, out, workspace, workspace_bytes, n_compute_units,
                       static_cast<hipStream_t>(stream));
}

ct_status ct_swiglu(const void* x, int32_t n_tokens, int32_t k_len, const void* w_gate, const void* w_up, int32_t n_out,
                    void* out, void* stream) {
  ct_status st = check_gemm_shape(n_tokens, k_len, n_out);
  if (st != CT_OK) return st;
  if (n_tokens == 0) return CT_OK;
  if (!x || !w_gate || !w_up || !out) return fail(CT_ERR_NULL, "x, w_gate, w_up and out must be non-NULL");
  if ((((uintptr_t)x | (uintptr_t)w_gate | (uintptr_t)w_up | (uintptr_t)out) & 15) != 0)
    return fail(CT_ERR_UNSUPPORTED, "x, w_gate, w_up and out must be 16-byte aligned");
  return launch_swiglu(x, n_tokens, k_len, w_gate, w_up, n_out, out, static_cast<hipStream_t>(stream));
}

size_t ct_stack_workspace_bytes(const ct_layer_cfg* cfg, int32_t ffn_dim, int32_t n_ctx, int32_t n_sel) {
  if (check_cfg(cfg) != CT_OK || ffn_dim <= 0 || n_ctx <= 0 || n_sel < 0 || n_sel > n_ctx) return 0;
  return stack_layout(cfg, ffn_dim, n_ctx, n_sel).total;
}

ct_status ct_partial_prefill_stack(const ct_layer_cfg* cfg, int32_t ffn_dim, float rms_eps, const ct_layer_weights* layers,
                                   int32_t n_layers, int32_t n_chunks, void* hidden_sel, const int32_t* sel_idx,
                                   int32_t n_sel, double recompute_ratio, void* k_bufs, void* v_bufs, void* workspace,
                                   size_t workspace_bytes, void* compute_stream, void* copy_stream) {
  return ct_partial_prefill_stack_tap(cfg, ffn_dim, rms_eps, layers, n_layers, n_chunks, hidden_sel, sel_idx, n_sel,
                                      recompute_ratio, k_bufs, v_bufs, workspace, workspace_bytes, compute_stream,
                                      copy_stream, nullptr);
}

ct_status ct_partial_prefill_stack_tap(const ct_layer_cfg* cfg, int32_t ffn_dim, float rms_eps,
                                       const ct_layer_weights* layers, int32_t n_layers, int32_t n_chunks,
                                       void* hidden_sel, const int32_t* sel_idx, int32_t n_sel, double recompute_ratio,
                                       void* k_bufs, void* v_bufs, void* workspace, size_t workspace_bytes,
                                       void* compute_stream, void* copy_stream, void* layer_inputs) {
  ct_status st = check_cfg(cfg);
  if (st != CT_OK) return st;
  if (layers == nullptr) return fail(CT_ERR_NULL, "layers is NULL");
  if (n_layers <= 0) return fail(CT_ERR_SHAPE, "n_layers %d must be positive", n_layers);
  if (n_chunks <= 0) return fail(CT_ERR_SHAPE, "n_chunks %d must be positive", n_chunks);
  if (n_chunks > 64) return fail(CT_ERR_UNSUPPORTED, "n_chunks %d: at most 64 chunks per layer", n_chunks);
  if (ffn_dim <= 0 || ffn_dim % 64 != 0) return fail(CT_ERR_UNSUPPORTED, "ffn_dim %d must be a positive multiple of 64", ffn_dim);
  if (!(rms_eps >= 0.f)) return fail(CT_ERR_SHAPE, "rms_eps must be >= 0");
  if (n_sel <= 0) return fail(CT_ERR_SHAPE, "n_sel %d: the stack needs at least one selected row", n_sel);
  if (cfg->n_q_heads * cfg->head_dim % 64 != 0) return fail(CT_ERR_UNSUPPORTED, "n_q_heads * head_dim must be a multiple of 64");

  // chunk geometry must be the same in every layer (same prompt): take it from layer 0, check the rest
  ChunkTable tab;
  memset(&tab, 0, sizeof(tab));
  tab.n = n_chunks;
  int64_t n_ctx64 = 0;
  bool any_host = false, any_compact = false;
  for (int l = 0; l < n_layers; ++l) {
    const ct_layer_weights& lw = layers[l];
    if (!lw.attn_norm || !lw.wqkv || !lw.wo || !lw.ffn_norm || !lw.w_gate || !lw.w_up || !lw.w_down)
      return fail(CT_ERR_NULL, "layer %d has a NULL weight", l);
    if (lw.chunks == nullptr) return fail(CT_ERR_NULL, "layer %d has no chunk table", l);
    int64_t rows = 0;
    for (int c = 0; c < n_chunks; ++c) {
      const ct_chunk& ch = lw.chunks[c];
      if (ch.n_tokens <= 0) return fail(CT_ERR_SHAPE, "layer %d chunk %d has n_tokens %d", l, c, ch.n_tokens);
      if (ch.location < 0 || ch.location > 2) return fail(CT_ERR_SHAPE, "layer %d chunk %d has location %d", l, c, ch.location);
      if (ch.new_pos_start < 0) return fail(CT_ERR_SHAPE, "layer %d chunk %d has negative new_pos_start", l, c);
      if (l == 0) {
        if (c > 0 && (int64_t)ch.new_pos_start < (int64_t)lw.chunks[c - 1].new_pos_start + lw.chunks[c - 1].n_tokens)
          return fail(CT_ERR_SHAPE, "chunk %d starts before chunk %d ends", c, c - 1);
        tab.row_start[c] = (int32_t)rows;
        tab.new_start[c] = ch.new_pos_start;
      } else if (ch.n_tokens != layers[0].chunks[c].n_tokens || ch.new_pos_start != layers[0].chunks[c].new_pos_start) {
        return fail(CT_ERR_SHAPE, "layer %d chunk %d differs in geometry from layer 0", l, c);
      }
      any_host |= ch.location != 0;
      any_compact |= ch.location == 2;
      rows += ch.n_tokens;
      if (rows > 0x7fffffff / 2) return fail(CT_ERR_SHAPE, "context too long");
    }
    if (l == 0) n_ctx64 = rows;
  }
  const int32_t n_ctx = (int32_t)n_ctx64;
  tab.row_start[n_chunks] = n_ctx;
  if (n_sel > n_ctx) return fail(CT_ERR_SHAPE, "n_sel %d exceeds n_ctx %d", n_sel, n_ctx);
  const bool full = n_sel == n_ctx;   // full recompute: every buffer row is overwritten, no cached KV is needed
  if (!full) {
    for (int l = 0; l < n_layers; ++l)
      for (int c = 0; c < n_chunks; ++c)
        if (!layers[l].chunks[c].k || !layers[l].chunks[c].v) return fail(CT_ERR_NULL, "layer %d chunk %d has a NULL k or v", l, c);
  }
  if ((st = check_kv_extent(cfg, n_ctx)) != CT_OK) return st;
  if (recompute_ratio >= 0.0) {
    if (!(recompute_ratio <= 1.0)) return fail(CT_ERR_RATIO, "recompute_ratio %g is above 1", recompute_ratio);
    int64_t want = (int64_t)floor(recompute_ratio * (double)n_ctx + 1e-9);
    if (recompute_ratio > 0.0 && want < 1) want = 1;
    if (want != n_sel) return fail(CT_ERR_RATIO, "n_sel %d but floor(%g * %d) = %lld", n_sel, recompute_ratio, n_ctx, (long long)want);
  }
  if (!hidden_sel || !sel_idx || !k_bufs || !v_bufs) return fail(CT_ERR_NULL, "hidden_sel, sel_idx, k_bufs and v_bufs must be non-NULL");
  st = check_gemm_shape(n_sel, cfg->hidden, ffn_dim);
  if (st != CT_OK) return st;
  st = check_gemm_shape(n_sel, ffn_dim, cfg->hidden);
  if (st != CT_OK) return st;
  const StackLayout L = stack_layout(cfg, ffn_dim, n_ctx, n_sel);
  if (workspace == nullptr) return fail(CT_ERR_WORKSPACE, "workspace is NULL but %zu bytes are needed", L.total);
  if (workspace_bytes < L.total) return fail(CT_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, L.total);
  if (((uintptr_t)workspace & 255) != 0) return fail(CT_ERR_WORKSPACE, "workspace is not 256-byte aligned");
  if (any_host && !full && compute_stream == copy_stream)
    return fail(CT_ERR_SHAPE, "pinned-host chunks need a copy_stream different from compute_stream");

  hipStream_t cs = static_cast<hipStream_t>(compute_stream);
  hipStream_t xs = static_cast<hipStream_t>(copy_stream);
  char* ws = static_cast<char*>(workspace);
  const size_t row_bytes = (size_t)cfg->n_kv_heads * cfg->head_dim * 2;
  const size_t buf_bytes = (size_t)n_ctx * row_bytes;   // one layer buffer; k_bufs / v_bufs hold two
  const int32_t qd = cfg->n_q_heads * cfg->head_dim;

  // events: one "landed" per (layer parity, chunk), one "attention done" per layer parity, one fence
  hipEvent_t* ev = nullptr;
  st = pooled_events((size_t)2 * n_chunks + 3, &ev);
  if (st != CT_OK) return st;
  auto landed = [&](int l, int c) { return ev[(size_t)(l & 1) * n_chunks + c]; };
  auto attn_done = [&](int l) { return ev[(size_t)2 * n_chunks + (l & 1)]; };
  hipEvent_t fence = ev[(size_t)2 * n_chunks + 2];
  hipError_t e;

  // Transfer stream: layer l's pinned-host chunks go to buffer slot l & 1.  The copies may start as
  // soon as the attention of layer l - 2 (the previous user of that slot) is done.
  bool streamed[2] = {false, false};
  auto enqueue_copies = [&](int l) -> ct_status {
    if (full || !any_host) return CT_OK;
    if (l >= 2) {
      if ((e = hipStreamWaitEvent(xs, attn_done(l), 0)) != hipSuccess) return hip_fail(e, "hipStreamWaitEvent (slot free)");
    } else if (l == 0) {
      // the first copies must not overtake earlier work of the compute stream that still uses the buffers
      if ((e = hipEventRecord(fence, cs)) != hipSuccess) return hip_fail(e, "hipEventRecord (fence)");
      if ((e = hipStreamWaitEvent(xs, fence, 0)) != hipSuccess) return hip_fail(e, "hipStreamWaitEvent (fence)");
    }
    char* kb = static_cast<char*>(k_bufs) + (size_t)(l & 1) * buf_bytes;
    char* vb = static_cast<char*>(v_bufs) + (size_t)(l & 1) * buf_bytes;
    // preferred: one kernel streams the chunks in and rotates the keys on the way
    bool done = false;
    ct_status sst = stream_in_host_chunks(cfg, layers[l].chunks, n_chunks, tab, kb, vb, sel_idx, n_sel, xs, &done);
    if (sst != CT_OK) return sst;
    streamed[l & 1] = done;
    if (!done && any_compact) return fail(CT_ERR_UNSUPPORTED, "compact pools are read by the stream-in kernel only");
    if (done) {
      if ((e = hipEventRecord(landed(l, 0), xs)) != hipSuccess) return hip_fail(e, "hipEventRecord (chunks streamed in)");
      return CT_OK;
    }
    for (int c = 0; c < n_chunks; ++c) {
      const ct_chunk& ch = layers[l].chunks[c];
      if (ch.location != 1) continue;
      const size_t bytes = (size_t)ch.n_tokens * row_bytes;
      const size_t off = (size_t)tab.row_start[c] * row_bytes;
      e = hipMemcpyAsync(kb + off, ch.k, bytes, hipMemcpyHostToDevice, xs);
      if (e == hipSuccess) e = hipMemcpyAsync(vb + off, ch.v, bytes, hipMemcpyHostToDevice, xs);
      if (e == hipSuccess) e = hipEventRecord(landed(l, c), xs);
      if (e != hipSuccess) return hip_fail(e, "host->device chunk copy");
    }
    return CT_OK;
  };

  if ((st = enqueue_copies(0)) != CT_OK) return st;
  for (int l = 0; l < n_layers; ++l) {
    const ct_layer_weights& lw = layers[l];
    if (l + 1 < n_layers && (st = enqueue_copies(l + 1)) != CT_OK) return st;
    char* kb = static_cast<char*>(k_bufs) + (size_t)(l & 1) * buf_bytes;
    char* vb = static_cast<char*>(v_bufs) + (size_t)(l & 1) * buf_bytes;
    if (layer_inputs != nullptr) {   // hand out the rows as they enter this layer
      const size_t bytes = (size_t)n_sel * cfg->hidden * 2;
      e = hipMemcpyAsync(static_cast<char*>(layer_inputs) + (size_t)l * bytes, hidden_sel, bytes, hipMemcpyDeviceToDevice, cs);
      if (e != hipSuccess) return hip_fail(e, "copy of a layer's input rows");
    }

    // attention block on the selected rows
    if ((st = launch_rmsnorm(hidden_sel, lw.attn_norm, rms_eps, n_sel, cfg->hidden, ws + L.x_norm, cs)) != CT_OK) return st;
    // The projection's epilogue writes the recomputed keys and values straight to their rows of
    // the layer buffers unless plain host copies, which overwrite those rows at a time of their
    // own, bring this layer's chunks in; device chunks are rotated into place first.
    bool host_here = false;
    for (int c = 0; c < n_chunks && !full; ++c) host_here |= lw.chunks[c].location != 0;
    const bool direct = full || !host_here || (streamed[l & 1] && stream_in_skips_selected());
    if (!full) {
      ReropeChunks rc;
      memset(&rc, 0, sizeof(rc));
      auto flush = [&]() -> ct_status {
        if (rc.n == 0) return CT_OK;
        rc.tok_start[rc.n] = rc.total_tokens;
        rc.skip_rows = sel_idx;   // the projection's epilogue (or the scatter) overwrites these rows next
        rc.n_skip = n_sel;
        ct_status r = launch_rerope_chunks(cfg, kb, vb, &rc, 0, cs);
        rc.n = 0;
        rc.total_tokens = 0;
        return r;
      };
      for (int c = 0; c < n_chunks; ++c) {
        const ct_chunk& ch = lw.chunks[c];
        if (ch.location != 0) continue;
        const int i = rc.n++;
        rc.tok_start[i] = rc.total_tokens;
        rc.total_tokens += ch.n_tokens;
        rc.k_src[i] = ch.k;
        rc.v_src[i] = (ch.v == (const void*)(vb + (size_t)tab.row_start[c] * row_bytes)) ? nullptr : ch.v;
        rc.row_start[i] = tab.row_start[c];
        rc.delta0[i] = ch.raw_keys ? ch.new_pos_start : ch.new_pos_start - ch.old_pos_start;
        rc.delta_step[i] = ch.raw_keys ? 1 : 0;
        if (rc.n == 32 && (st = flush()) != CT_OK) return st;
      }
      if ((st = flush()) != CT_OK) return st;
    }
    if ((st = direct ? launch_qkv(cfg, ws + L.x_norm, nullptr, nullptr, sel_idx, &tab, n_sel, lw.wqkv, nullptr, ws + L.q, kb, vb,
                                  cs, sel_idx)
                     : launch_qkv(cfg, ws + L.x_norm, nullptr, nullptr, sel_idx, &tab, n_sel, lw.wqkv, nullptr, ws + L.q,
                                  ws + L.k, ws + L.v, cs)) != CT_OK)
      return st;
    if (!full) {
      if (streamed[l & 1] && (e = hipStreamWaitEvent(cs, landed(l, 0), 0)) != hipSuccess)
        return hip_fail(e, "hipStreamWaitEvent (chunks streamed in)");
      for (int c = 0; c < n_chunks && !streamed[l & 1]; ++c) {
        const ct_chunk& ch = lw.chunks[c];
        if (ch.location != 1) continue;
        if ((e = hipStreamWaitEvent(cs, landed(l, c), 0)) != hipSuccess) return hip_fail(e, "hipStreamWaitEvent (chunk landed)");
        char* kd = kb + (size_t)tab.row_start[c] * row_bytes;
        const int32_t d0 = ch.raw_keys ? ch.new_pos_start : ch.new_pos_start - ch.old_pos_start;
        if ((st = launch_rerope(cfg, kd, kd, nullptr, nullptr, nullptr, nullptr, d0, ch.raw_keys ? 1 : 0, ch.n_tokens, cs)) != CT_OK)
          return st;   // (rotates the chunk's stale selected rows too; the scatter below overwrites them)
      }
    }
    if (!direct && (st = launch_scatter(cfg, kb, vb, ws + L.k, ws + L.v, sel_idx, n_sel, cs)) != CT_OK) return st;
    if ((st = launch_attention(cfg, ws + L.q, kb, vb, n_ctx, sel_idx, n_sel, ws + L.attn_out, nullptr, ws + L.attn_ws, cs)) != CT_OK)
      return st;
    if ((e = hipEventRecord(attn_done(l), cs)) != hipSuccess) return hip_fail(e, "hipEventRecord (attention done)");
    // output projection + residual, FFN + residual (the residual stream is updated in place).
    // The chunks of layer l + 2 start streaming in when this layer's attention is done, so that
    // kernel runs beside these GEMMs and its workgroups hold compute units of their own: the GEMM
    // rounds are planned for what is left.  A launch's workgroups go to the eight XCDs in turn, so
    // what counts is the XCD with the fewest free units, and the stream-in workgroups do not
    // spread one per XCD: with 8 of them, launches planned for 216-224 units (28 per XCD) finish
    // in one round, launches planned for 232 or more do not (measured on the 32-layer stack).
    const int gemm_cus = (l + 2 < n_layers && (streamed[0] || streamed[1]))
                             ? kNumCUs - kCUsHeldPerStreamInBlock * stream_in_blocks() : kNumCUs;
    if ((st = launch_linear(ws + L.attn_out, n_sel, qd, lw.wo, cfg->hidden, hidden_sel, hidden_sel, ws + L.gemm_ws,
                            L.gemm_ws_bytes, gemm_cus, cs)) != CT_OK) return st;
    if ((st = launch_rmsnorm(hidden_sel, lw.ffn_norm, rms_eps, n_sel, cfg->hidden, ws + L.x_norm, cs)) != CT_OK) return st;
    if ((st = launch_swiglu(ws + L.x_norm, n_sel, cfg->hidden, lw.w_gate, lw.w_up, ffn_dim, ws + L.act, cs)) != CT_OK) return st;
    if ((st = launch_linear(ws + L.act, n_sel, ffn_dim, lw.w_down, cfg->hidden, hidden_sel, hidden_sel, ws + L.gemm_ws,
                            L.gemm_ws_bytes, gemm_cus, cs)) != CT_OK) return st;
  }
  return CT_OK;
}

}  // extern "C"
