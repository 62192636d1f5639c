// Internal declarations shared by the translation units of libcachetune (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "cachetune.h"

namespace ct {

// ---- the one chip this library is written for (MI355X, gfx950) --------------------------------
constexpr int kNumCUs = 256;    // compute units
constexpr int kNumXCDs = 8;     // accelerator dies; consecutive workgroup ids of a launch go to them in turn
// Compute units a linear launch of the recompute stream should leave out of its plan for every
// workgroup of the stream-in kernel that runs beside it (measured on the 32-layer stack: the
// stream-in workgroups do not spread one per XCD, and the XCD with the fewest free units sets
// the round).
constexpr int kCUsHeldPerStreamInBlock = 4;

// ---- kernel classes for the opt-in event profiling ------------------------------------
enum KernelClass { KC_QKV = 0, KC_REROPE = 1, KC_SCATTER = 2, KC_ATTN = 3, KC_MERGE = 4, KC_LINEAR = 5, KC_NORM = 6, KC_FREQ = 7, KC_TOPK = 8, KC_COUNT = 9 };

ct_status fail(ct_status code, const char* fmt, ...);
ct_status hip_fail(hipError_t e, const char* what);
ct_status check_cfg(const ct_layer_cfg* cfg);
// K/V buffers of n_ctx rows must stay below 2^24 rows and 4 GiB (32-bit byte offsets in the attention kernel).
ct_status check_kv_extent(const ct_layer_cfg* cfg, int64_t n_ctx);

// A pair of events for one launch of class `kc` when profiling is on (both NULL when it is off).
void prof_events(KernelClass kc, hipEvent_t* start, hipEvent_t* stop);

// `n` timing-disabled events for stream ordering, reused from call to call (created on first use,
// kept until the process ends, one set per calling thread).  Re-recording an event does not
// disturb waits that were enqueued on its earlier record.
ct_status pooled_events(size_t n, hipEvent_t** out);

#if defined(__HIPCC__)
// Every kernel of the library is launched through this.  With profiling on, the two events ride on
// the kernel's own dispatch (hipExtLaunchKernelGGL) and take its begin and end timestamps, the
// same interval a kernel trace reports.  (Events recorded before and after a launch also span the
// gaps around it: 12.2 us instead of 9.6 us for the scatter of the 32K workload.)
template <typename Kernel, typename... Args>
inline void launch_kernel(KernelClass kc, Kernel kernel, dim3 grid, dim3 block, unsigned lds_bytes, hipStream_t s,
                          Args... args) {
  hipEvent_t e0 = nullptr, e1 = nullptr;
  prof_events(kc, &e0, &e1);
  if (e0 != nullptr)
    hipExtLaunchKernelGGL(kernel, grid, block, lds_bytes, s, e0, e1, 0, args...);
  else
    hipLaunchKernelGGL(kernel, grid, block, lds_bytes, s, args...);
}
#endif

// RoPE frequencies in turns: omega_j / (2 pi), j < head_dim / 2 <= 64, computed on the
// host in double precision and handed to kernels by value.
struct RopeTable {
  double turns[64];
};
void fill_rope_table(const ct_layer_cfg* cfg, RopeTable* t);

// Attention launch geometry chosen on the host from the problem size.
struct AttnPlan {
  int tile_tokens;   // selected tokens per workgroup tile (256 / group size)
  int n_tiles;       // ceil(n_sel / tile_tokens)
  int n_splits;      // key-range splits per tile (1 = no workspace traffic)
  int split_keys;    // keys per split (multiple of the K tile), meaningful when n_splits > 1
  size_t ws_bytes;   // workspace bytes needed
};
AttnPlan plan_attention(const ct_layer_cfg* cfg, int n_ctx, int n_sel);
// Lowest and highest key row the attention launch over keys [key_after, key_upto) reads (host replay).
ct_status attention_rows_read(const ct_layer_cfg* cfg, const int32_t* sel_idx_host, int32_t n_sel, int32_t n_ctx,
                              int32_t key_after, int32_t key_upto, bool resumable, int32_t* first_row,
                              int32_t* last_row);
// Scratch bytes launch_attention needs behind its `workspace` pointer for this problem size.
size_t attention_scratch_bytes(const ct_layer_cfg* cfg, int n_ctx, int n_sel);

// ---- launchers implemented next to their kernels ---------------------------------------
// skip_rows (optional, device memory, sorted ascending, n_skip entries): token rows that are neither
// read nor written (the recompute set, whose keys the scatter overwrites).
ct_status launch_rerope(const ct_layer_cfg* cfg, const void* k_src, void* k_dst, const void* v_src, void* v_dst,
                        const int32_t* old_pos, const int32_t* new_pos, int32_t delta0, int32_t delta_step,
                        int32_t n_tokens, hipStream_t s, const int32_t* skip_rows = nullptr, int32_t n_skip = 0);
// Several device-resident chunks rotated (and their values copied) into the layer buffers
// in one launch.  v_src[c] == NULL leaves the values of chunk c alone.
struct ReropeChunks {
  int32_t n;
  int32_t pad;
  int64_t total_tokens;
  int64_t tok_start[33];   // ordinal of the first token of chunk c among the listed chunks
  const void* k_src[32];
  const void* v_src[32];
  int32_t row_start[32];   // buffer row the chunk's first token goes to
  int32_t delta0[32];
  int32_t delta_step[32];
  const int32_t* skip_rows;   // optional: sorted buffer rows that are not to be brought in (device memory)
  int32_t n_skip;
  uint32_t compact_mask;      // bit c: the source of chunk c holds only its rows that are not in skip_rows
};
// LDS that the small kernels of the recompute stream claim without using it (the large ones need
// at least as much anyway): together with the 80 KiB the stream-in kernel claims, it keeps the two
// streams' workgroups on different compute units.  It is asked for as dynamic LDS at the launch.
constexpr unsigned kKeepOutLdsBytes = 96 * 1024;
constexpr unsigned kStreamInLdsBytes = 80 * 1024;
// max_blocks > 0 caps the grid (threads then stride over the tokens).
ct_status launch_rerope_chunks(const ct_layer_cfg* cfg, void* k_buf, void* v_buf, const ReropeChunks* chunks,
                               int max_blocks, hipStream_t s);
// Pinned-host chunks (location 1) read by a kernel on stream `xs` straight from host memory:
// keys rotated on the way, values copied, both written to their rows of the layer buffers.
// *done is false, and nothing was enqueued, when some chunk's memory is not addressable by the
// device; the caller then copies.
struct ChunkTable;
// Rows listed in sel_idx (the recompute set: their K/V are overwritten by the scatter) are not
// transferred - the index-aware transfer of Sec. 4.2.
// group_sizes != NULL: launch g covers the next group_sizes[g] host chunks (the last group takes
// what is left), and after each launch `after_group(ctx, c)` is called with the index of the
// last chunk it covers (to record an event, say).
typedef ct_status (*stream_in_group_fn)(void* ctx, int last_chunk);
ct_status stream_in_host_chunks(const ct_layer_cfg* cfg, const ct_chunk* chunks, int n_chunks, const ChunkTable& tab,
                                void* k_buf, void* v_buf, const int32_t* sel_idx, int32_t n_sel, hipStream_t xs,
                                bool* done, const int* group_sizes = nullptr, int n_groups = 0,
                                stream_in_group_fn after_group = nullptr, void* ctx = nullptr);
// Whether the stream-in kernel leaves the rows of the recompute set alone (it does unless switched off).
bool stream_in_skips_selected();
ct_status launch_scatter(const ct_layer_cfg* cfg, void* k_buf, void* v_buf, const void* k_sel, const void* v_sel,
                         const int32_t* sel_idx, int32_t n_sel, hipStream_t s);
// pos_of_row != NULL: position of selected token s is pos_of_row[s]; otherwise it is looked up
// through the chunk table (positions of buffer rows) with sel_idx.
struct ChunkTable {
  int32_t n;
  int32_t row_start[65];   // buffer row where chunk c starts; row_start[n] = n_ctx
  int32_t new_start[64];
};
ct_status launch_qkv(const ct_layer_cfg* cfg, const void* hidden, const int32_t* hidden_rows, const int32_t* sel_pos,
                     const int32_t* sel_idx, const ChunkTable* chunks, int32_t n_sel, const void* wqkv,
                     const void* bias, void* q_out, void* k_out, void* v_out, hipStream_t s,
                     const int32_t* kv_rows = nullptr);   // kv_rows != NULL: keys and values of selected row t go
                                                          // to row kv_rows[t] of k_out / v_out (the layer buffers)
// out[t, :] = x[t, :] * w^T (+ residual[t, :]);  x [n_tok, k_len], w [n_out, k_len], bf16
// ws (optional, linear_workspace_bytes() bytes): scratch that lets a launch whose last round of
// workgroups would leave most compute units idle split the reduction of those tiles.  n_cu: the
// compute units the launch can count on (256, less what a concurrent stream-in kernel holds).
ct_status launch_linear(const void* x, int32_t n_tok, int32_t k_len, const void* w, int32_t n_out, const void* residual,
                        void* out, void* ws, size_t ws_bytes, int n_cu, hipStream_t s);
// Workgroups of the kernel that streams host chunks in (each keeps a compute unit to itself).
int stream_in_blocks();
size_t linear_workspace_bytes(int32_t n_tok, int32_t k_len, int32_t n_out);
// out[t, :] = silu(x[t, :] * w_gate^T) * (x[t, :] * w_up^T);  both weights [n_out, k_len]
ct_status launch_swiglu(const void* x, int32_t n_tok, int32_t k_len, const void* w_gate, const void* w_up, int32_t n_out,
                        void* out, hipStream_t s);
// out[t, :] = x[t, :] / sqrt(mean(x[t, :]^2) + eps) * w;  x, out [n_tok, width] bf16, w [width] bf16
ct_status launch_rmsnorm(const void* x, const void* w, float eps, int32_t n_tok, int32_t width, void* out, hipStream_t s);
// key_after / key_upto, the unsplit plan only.  state == NULL: the launch computes only the tiles
// of selected rows whose last row r has key_after < r + 1 <= key_upto (all tiles by default).
// state != NULL (attention_state_bytes() bytes): the launch takes every tile that sees keys past
// key_after through the keys [key_after, key_upto) alone; tiles that need later keys leave their
// fp32 (O, m, l) in `state`, where the launch for the next key range picks them up.
ct_status launch_attention(const ct_layer_cfg* cfg, const void* q_sel, const void* k_buf, const void* v_buf,
                           int32_t n_ctx, const int32_t* sel_idx, int32_t n_sel, void* out, float* lse,
                           void* workspace, hipStream_t s, int32_t key_after = 0, int32_t key_upto = 0x7fffffff,
                           float* state = nullptr);
size_t attention_state_bytes(const ct_layer_cfg* cfg, int n_ctx, int n_sel);

}  // namespace ct

// ---- device helpers ----------------------------------------------------------------------
#if defined(__HIPCC__)
namespace ct {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// two fp32 -> packed bf16 pair, round to nearest even (v_cvt_pk_bf16_f32 on gfx950)
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  f32x2 v = {lo, hi};
  bf16x2 p = __builtin_convertvector(v, bf16x2);
  return *reinterpret_cast<uint32_t*>(&p);
}

// cos and sin of the angle steps * omega, with omega given in turns (omega / 2pi).
// The product and its reduction to [-1/2, 1/2] turns are done in fp64, so the angle is good
// to ~1e-11 rad at any position; the hardware sin/cos take their argument in turns.
__device__ __forceinline__ void sincos_turns(int32_t steps, double omega_turns, float& c, float& s) {
  double t = (double)steps * omega_turns;
  t -= rint(t);
  float f = (float)t;
  s = __builtin_amdgcn_sinf(f);
  c = __builtin_amdgcn_cosf(f);
}

}  // namespace ct
#endif
