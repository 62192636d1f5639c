// Bandwidth-bound steps of the partial-prefill layer: deferred RoPE recovery of reused keys
// (Eq. 8, delta form) and scatter fusion of recomputed K/V rows (Sec. 4.2).
//
// Both kernels move every byte exactly once with 128-bit accesses.  Key rows are
// [n_kv_heads, head_dim] bf16; a thread owns 8 rotation pairs of one token and walks over
// all KV heads, so the 8 sin/cos values (angle reduced in fp64) are computed once per
// token and pair and reused for every head.
#include "ct_internal.h"

namespace ct {

namespace {

constexpr int kReropeThreads = 256;

// Streaming accesses.  Cached keys and values are read once: their loads do not allocate in the
// caches (measured cold: +3 % out of place).  A rotation in place also writes lines nobody reads
// soon, so its stores bypass the caches as well (+17 % at 64 MiB, 5.3 -> 6.0 TB/s at 256 MiB);
// rows written into a layer buffer are read by the attention kernel next and are stored normally.
template <bool NT>
__device__ __forceinline__ u32x4 ld16(const uint16_t* p) {
  if (NT) return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  return *reinterpret_cast<const u32x4*>(p);
}
template <bool NT>
__device__ __forceinline__ void st16(uint16_t* p, u32x4 v) {
  if (NT) __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(p));
  else *reinterpret_cast<u32x4*>(p) = v;
}

// Rotate (and optionally copy V for) one token's share owned by this thread.
// STYLE 0: pairs (j, j + D/2); STYLE 1: pairs (2j, 2j + 1).  HEADS > 0 fixes the head count
// at compile time (full unroll, all loads in flight before the first use).
// k_src/k_dst (and v_src/v_dst) may be the same row: a thread reads all it owns before it
// writes, and no two threads own the same bytes.
template <int D, int STYLE, int HEADS, bool NT_STORE = false>
__device__ __forceinline__ void rerope_token(const uint16_t* k_src, uint16_t* k_dst, const uint16_t* v_src,
                                             uint16_t* v_dst, int32_t delta, int jg, int n_heads_rt,
                                             const RopeTable& table) {
  const int n_heads = HEADS > 0 ? HEADS : n_heads_rt;
  float cs[8], sn[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) sincos_turns(delta, table.turns[jg * 8 + i], cs[i], sn[i]);

  // element offsets (in bf16) of the two 16-byte pieces this thread owns inside a head row
  const int off_a = STYLE == 0 ? jg * 8 : jg * 16;
  const int off_b = STYLE == 0 ? jg * 8 + D / 2 : jg * 16 + 8;

  auto rotate_head = [&](u32x4 a, u32x4 b, u32x4& ra, u32x4& rb) {
    if (STYLE == 0) {
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        float a0 = bf16_lo(a[w]), a1 = bf16_hi(a[w]);
        float b0 = bf16_lo(b[w]), b1 = bf16_hi(b[w]);
        float c0 = cs[2 * w], s0 = sn[2 * w], c1 = cs[2 * w + 1], s1 = sn[2 * w + 1];
        ra[w] = pack_bf16(a0 * c0 - b0 * s0, a1 * c1 - b1 * s1);
        rb[w] = pack_bf16(a0 * s0 + b0 * c0, a1 * s1 + b1 * c1);
      }
    } else {
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        float x = bf16_lo(a[w]), y = bf16_hi(a[w]);
        ra[w] = pack_bf16(x * cs[w] - y * sn[w], x * sn[w] + y * cs[w]);
        float x2 = bf16_lo(b[w]), y2 = bf16_hi(b[w]);
        rb[w] = pack_bf16(x2 * cs[4 + w] - y2 * sn[4 + w], x2 * sn[4 + w] + y2 * cs[4 + w]);
      }
    }
  };

  if (HEADS > 0) {
    u32x4 a[HEADS > 0 ? HEADS : 1], b[HEADS > 0 ? HEADS : 1];
#pragma unroll
    for (int h = 0; h < HEADS; ++h) {
      a[h] = ld16<true>(k_src + h * D + off_a);
      b[h] = ld16<true>(k_src + h * D + off_b);
    }
#pragma unroll
    for (int h = 0; h < HEADS; ++h) {
      u32x4 ra, rb;
      rotate_head(a[h], b[h], ra, rb);
      st16<NT_STORE>(k_dst + h * D + off_a, ra);
      st16<NT_STORE>(k_dst + h * D + off_b, rb);
    }
    if (v_src != nullptr) {
#pragma unroll
      for (int h = 0; h < HEADS; ++h) {
        a[h] = ld16<true>(v_src + h * D + off_a);
        b[h] = ld16<true>(v_src + h * D + off_b);
      }
#pragma unroll
      for (int h = 0; h < HEADS; ++h) {
        st16<NT_STORE>(v_dst + h * D + off_a, a[h]);
        st16<NT_STORE>(v_dst + h * D + off_b, b[h]);
      }
    }
  } else {
    for (int h = 0; h < n_heads; ++h) {
      u32x4 a = ld16<true>(k_src + h * D + off_a);
      u32x4 b = ld16<true>(k_src + h * D + off_b);
      u32x4 ra, rb;
      rotate_head(a, b, ra, rb);
      st16<NT_STORE>(k_dst + h * D + off_a, ra);
      st16<NT_STORE>(k_dst + h * D + off_b, rb);
      if (v_src != nullptr) {
        u32x4 va = ld16<true>(v_src + h * D + off_a);
        u32x4 vb = ld16<true>(v_src + h * D + off_b);
        st16<NT_STORE>(v_dst + h * D + off_a, va);
        st16<NT_STORE>(v_dst + h * D + off_b, vb);
      }
    }
  }
}

// Sorted skip lists (the recompute set: rows that are overwritten by the scatter and need not be
// moved).  count_below: number of listed rows < row, by binary search.
__device__ __forceinline__ int count_below(const int32_t* __restrict__ list, int n, int32_t row) {
  int lo = 0, hi = n;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (list[mid] < row) lo = mid + 1; else hi = mid;
  }
  return lo;
}
// The rows of one workgroup lie next to each other: one search for the workgroup's first row
// (the same for every thread, so its loads are scalar), then a walk over the few entries up to
// this thread's row.  Rows far from the first one (a gap between chunks) search on their own.
__device__ __forceinline__ int count_below_near(const int32_t* __restrict__ list, int n, int32_t first_row,
                                                int first_below, int32_t row) {
  if (row < first_row || row - first_row > 512) return count_below(list, n, row);
  int i = first_below;
  while (i < n && list[i] < row) ++i;
  return i;
}

// Per-token positions, or one arithmetic progression of deltas (delta0 + delta_step * t).
template <int D, int STYLE, int HEADS, bool NT_STORE>
__global__ __launch_bounds__(kReropeThreads) void rerope_kernel(
    const uint16_t* k_src, uint16_t* k_dst, const uint16_t* v_src, uint16_t* v_dst,
    const int32_t* __restrict__ old_pos, const int32_t* __restrict__ new_pos, int32_t delta0, int32_t delta_step,
    int32_t n_tokens, int32_t n_heads_rt, RopeTable table, const int32_t* __restrict__ skip_rows, int32_t n_skip) {
  constexpr int GROUPS = D / 16;  // threads per token: each owns 8 pairs = 16 elements per head
  const int64_t gid = (int64_t)blockIdx.x * kReropeThreads + threadIdx.x;
  const int64_t token = gid / GROUPS;
  const int jg = (int)(gid % GROUPS);
  if (token >= n_tokens) return;
  if (skip_rows != nullptr) {
    const int32_t first = (int32_t)((int64_t)blockIdx.x * (kReropeThreads / GROUPS));
    const int at = count_below_near(skip_rows, n_skip, first, count_below(skip_rows, n_skip, first), (int32_t)token);
    if (at < n_skip && skip_rows[at] == (int32_t)token) return;
  }
  int32_t delta;
  if (new_pos != nullptr) {
    delta = new_pos[token] - (old_pos != nullptr ? old_pos[token] : 0);
  } else {
    delta = delta0 + delta_step * (int32_t)token;
  }
  const int64_t row = token * (int64_t)(HEADS > 0 ? HEADS : n_heads_rt) * D;
  rerope_token<D, STYLE, HEADS, NT_STORE>(k_src + row, k_dst + row, v_src ? v_src + row : nullptr,
                                v_dst ? v_dst + row : nullptr, delta, jg, n_heads_rt, table);
}

// Several chunks in one launch: buffer row -> chunk by search in the (small) table.
// NEAR: the grid covers every token once, so a workgroup's rows are neighbours and share one search
// of the skip list; otherwise (few workgroups striding over the tokens) every token searches.
template <int D, int STYLE, int HEADS, bool NEAR>
__device__ __forceinline__ void rerope_chunk_tokens(uint16_t* k_buf, uint16_t* v_buf, int32_t n_heads_rt,
                                                    const RopeTable& table, const ReropeChunks& chunks, int threads) {
  constexpr int GROUPS = D / 16;
  const int64_t gid = (int64_t)blockIdx.x * threads + threadIdx.x;
  const int jg = (int)(gid % GROUPS);
  const int64_t t_step = (int64_t)gridDim.x * (threads / GROUPS);
  int32_t first_row = 0;
  int first_below = 0;
  if (NEAR && chunks.skip_rows != nullptr) {
    const int64_t t0 = (int64_t)blockIdx.x * (threads / GROUPS);   // the workgroup's first token
    int c0 = 0;
    while (c0 + 1 < chunks.n && t0 >= chunks.tok_start[c0 + 1]) ++c0;
    first_row = chunks.row_start[c0] + (int32_t)(t0 - chunks.tok_start[c0]);
    first_below = count_below(chunks.skip_rows, chunks.n_skip, first_row);
  }
  for (int64_t t_all = gid / GROUPS; t_all < chunks.total_tokens; t_all += t_step) {   // ordinal among the listed tokens
    int c = 0;
    while (c + 1 < chunks.n && t_all >= chunks.tok_start[c + 1]) ++c;
    const int32_t t = (int32_t)(t_all - chunks.tok_start[c]);
    int32_t t_src = t;   // row inside the chunk's source
    if (chunks.skip_rows != nullptr) {   // is this buffer row in the sorted skip list?
      const int32_t row = chunks.row_start[c] + t;
      const int lo = NEAR ? count_below_near(chunks.skip_rows, chunks.n_skip, first_row, first_below, row)
                          : count_below(chunks.skip_rows, chunks.n_skip, row);
      if (lo < chunks.n_skip && chunks.skip_rows[lo] == row) continue;
      // a compact source holds only the rows that are kept: step over the skipped ones before this row
      if ((chunks.compact_mask >> c) & 1u) t_src = t - (lo - count_below(chunks.skip_rows, chunks.n_skip, chunks.row_start[c]));
    }
    const int64_t heads = HEADS > 0 ? HEADS : n_heads_rt;
    const int64_t src_row = (int64_t)t_src * heads * D;
    const int64_t dst_row = ((int64_t)chunks.row_start[c] + t) * heads * D;
    const uint16_t* ks = static_cast<const uint16_t*>(chunks.k_src[c]) + src_row;
    const uint16_t* vs = chunks.v_src[c] ? static_cast<const uint16_t*>(chunks.v_src[c]) + src_row : nullptr;
    const int32_t delta = chunks.delta0[c] + chunks.delta_step[c] * t;
    rerope_token<D, STYLE, HEADS>(ks, k_buf + dst_row, vs, v_buf + dst_row, delta, jg, n_heads_rt, table);
  }
}

template <int D, int STYLE, int HEADS>
__global__ __launch_bounds__(kReropeThreads) void rerope_chunks_kernel(uint16_t* k_buf, uint16_t* v_buf,
                                                                      int32_t n_heads_rt, RopeTable table,
                                                                      ReropeChunks chunks) {
  rerope_chunk_tokens<D, STYLE, HEADS, true>(k_buf, v_buf, n_heads_rt, table, chunks, kReropeThreads);
}

// The same work for chunks in pinned host memory, read over the host link by a few resident
// workgroups that stride over the tokens (Sec. 4.2: RoPE recovery overlapped with the transfer).
// What it is shaped by, measured on MI355X:
//  - a load from host memory takes microseconds, and while it is pending it holds a slot in the
//    memory pipeline of its compute unit and in the L2 channel's queue to the fabric; waves of
//    other kernels on the same compute unit, and L2 misses of any kernel in the same XCD, wait
//    behind it.  So a thread keeps only one head's two 16-byte loads in flight (about 128 KiB
//    over the whole grid already keeps the link at 45-50 GB/s; more only lengthens the queues);
//  - the launch asks for 80 KiB of (dynamic) LDS that the kernel does not use: they keep the
//    workgroups of the GEMM and attention kernels, which need 96-160 KiB, off the few compute units
//    this kernel sits on, where they would run at the speed of the host link.
constexpr int kStreamInThreads = 1024;
template <int D, int STYLE>
__global__ __launch_bounds__(kStreamInThreads) void stream_in_kernel(uint16_t* k_buf, uint16_t* v_buf, int32_t n_heads_rt,
                                                                    RopeTable table, ReropeChunks chunks) {
  rerope_chunk_tokens<D, STYLE, 0, false>(k_buf, v_buf, n_heads_rt, table, chunks, kStreamInThreads);
}

// One 16-byte piece per thread and loop step; a selected row's K and V are `row_vec`
// pieces each.  Pieces of consecutive threads are consecutive in memory.
// The launch asks for kKeepOutLdsBytes of dynamic LDS that the kernel does not use (see there).
__global__ __launch_bounds__(1024) void scatter_kernel(u32x4* __restrict__ k_buf, u32x4* __restrict__ v_buf,
                                                      const u32x4* __restrict__ k_sel,
                                                      const u32x4* __restrict__ v_sel,
                                                      const int32_t* __restrict__ sel_idx, int32_t n_sel,
                                                      int32_t row_vec) {
  const int64_t total = (int64_t)n_sel * row_vec;
  for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < total; p += (int64_t)gridDim.x * blockDim.x) {
    const int64_t s = p / row_vec;
    const int c = (int)(p - s * row_vec);
    const int64_t dst = (int64_t)sel_idx[s] * row_vec + c;
    u32x4 kv = k_sel[p];
    u32x4 vv = v_sel[p];
    k_buf[dst] = kv;
    v_buf[dst] = vv;
  }
}

// Arguments of the per-token form, bundled for the dispatch over (head_dim, style, head count).
struct ReropeLaunch {
  const uint16_t* ks; uint16_t* kd; const uint16_t* vs; uint16_t* vd;
  const int32_t* old_pos; const int32_t* new_pos; int32_t delta0, delta_step, n_tokens;
  const int32_t* skip_rows; int32_t n_skip;
};

template <int D, int STYLE, int HEADS>
void launch_rerope_one(dim3 grid, hipStream_t s, const ReropeLaunch& r, int H, const RopeTable& t,
                       const ReropeChunks* chunks, bool big_blocks) {
  if (chunks != nullptr) {
    if (big_blocks)
      launch_kernel(KC_REROPE, stream_in_kernel<D, STYLE>, grid, dim3(kStreamInThreads), kStreamInLdsBytes, s, r.kd, r.vd,
                    H, t, *chunks);
    else
      launch_kernel(KC_REROPE, rerope_chunks_kernel<D, STYLE, HEADS>, grid, dim3(kReropeThreads), 0, s, r.kd, r.vd, H, t,
                    *chunks);
  } else {
    if (r.ks == r.kd)   // in place
      launch_kernel(KC_REROPE, rerope_kernel<D, STYLE, HEADS, true>, grid, dim3(kReropeThreads), 0, s, r.ks, r.kd, r.vs,
                    r.vd, r.old_pos, r.new_pos, r.delta0, r.delta_step, r.n_tokens, H, t, r.skip_rows, r.n_skip);
    else
      launch_kernel(KC_REROPE, rerope_kernel<D, STYLE, HEADS, false>, grid, dim3(kReropeThreads), 0, s, r.ks, r.kd, r.vs,
                    r.vd, r.old_pos, r.new_pos, r.delta0, r.delta_step, r.n_tokens, H, t, r.skip_rows, r.n_skip);
  }
}

template <int D, int STYLE>
void launch_rerope_heads(int H, dim3 grid, hipStream_t s, const ReropeLaunch& r, const RopeTable& t,
                         const ReropeChunks* chunks, bool big_blocks) {
  if (H == 8)
    launch_rerope_one<D, STYLE, 8>(grid, s, r, H, t, chunks, big_blocks);
  else if (H == 2)
    launch_rerope_one<D, STYLE, 2>(grid, s, r, H, t, chunks, big_blocks);
  else
    launch_rerope_one<D, STYLE, 0>(grid, s, r, H, t, chunks, big_blocks);
}

// The stream-in and scatter kernels are launched with more dynamic LDS than the default limit
// of a kernel: raise the limit once per kernel.
template <typename Kernel>
hipError_t allow_dynamic_lds(Kernel kernel, unsigned bytes) {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

ct_status launch_rerope_any(const ct_layer_cfg* cfg, const ReropeLaunch& r, int64_t n_tokens, const ReropeChunks* chunks,
                            int max_blocks, hipStream_t s) {
  if (n_tokens == 0) return CT_OK;
  RopeTable table;
  fill_rope_table(cfg, &table);
  const int D = cfg->head_dim, H = cfg->n_kv_heads;
  const int64_t threads = n_tokens * (D / 16);
  const bool big_blocks = chunks != nullptr && max_blocks > 0;   // sources in pinned host memory
  const int per_block = big_blocks ? kStreamInThreads : kReropeThreads;
  int64_t blocks = (threads + per_block - 1) / per_block;
  if (big_blocks && blocks > max_blocks) blocks = max_blocks;
  dim3 grid((unsigned)blocks);
  if (big_blocks) {
    static const hipError_t allowed = []() {
      hipError_t e = allow_dynamic_lds(stream_in_kernel<128, 0>, kStreamInLdsBytes);
      if (e == hipSuccess) e = allow_dynamic_lds(stream_in_kernel<128, 1>, kStreamInLdsBytes);
      if (e == hipSuccess) e = allow_dynamic_lds(stream_in_kernel<64, 0>, kStreamInLdsBytes);
      if (e == hipSuccess) e = allow_dynamic_lds(stream_in_kernel<64, 1>, kStreamInLdsBytes);
      return e;
    }();
    if (allowed != hipSuccess) return hip_fail(allowed, "hipFuncSetAttribute (stream-in kernel LDS)");
  }
  if (D == 128) {
    if (cfg->rope_style == 0)
      launch_rerope_heads<128, 0>(H, grid, s, r, table, chunks, big_blocks);
    else
      launch_rerope_heads<128, 1>(H, grid, s, r, table, chunks, big_blocks);
  } else {
    if (cfg->rope_style == 0)
      launch_rerope_heads<64, 0>(H, grid, s, r, table, chunks, big_blocks);
    else
      launch_rerope_heads<64, 1>(H, grid, s, r, table, chunks, big_blocks);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(e, "re-RoPE kernel launch");
  return CT_OK;
}

}  // namespace

ct_status launch_rerope(const ct_layer_cfg* cfg, const void* k_src, void* k_dst, const void* v_src, void* v_dst,
                        const int32_t* old_pos, const int32_t* new_pos, int32_t delta0, int32_t delta_step,
                        int32_t n_tokens, hipStream_t s, const int32_t* skip_rows, int32_t n_skip) {
  ReropeLaunch r = {static_cast<const uint16_t*>(k_src), static_cast<uint16_t*>(k_dst), static_cast<const uint16_t*>(v_src),
                    static_cast<uint16_t*>(v_dst), old_pos, new_pos, delta0, delta_step, n_tokens,
                    n_skip > 0 ? skip_rows : nullptr, n_skip};
  return launch_rerope_any(cfg, r, n_tokens, nullptr, 0, s);
}

ct_status launch_rerope_chunks(const ct_layer_cfg* cfg, void* k_buf, void* v_buf, const ReropeChunks* chunks,
                               int max_blocks, hipStream_t s) {
  ReropeLaunch r = {nullptr, static_cast<uint16_t*>(k_buf), nullptr, static_cast<uint16_t*>(v_buf), nullptr, nullptr, 0, 0, 0,
                    nullptr, 0};
  return launch_rerope_any(cfg, r, chunks->total_tokens, chunks, max_blocks, s);
}

ct_status launch_scatter(const ct_layer_cfg* cfg, void* k_buf, void* v_buf, const void* k_sel, const void* v_sel,
                         const int32_t* sel_idx, int32_t n_sel, hipStream_t s) {
  if (n_sel == 0) return CT_OK;
  static const hipError_t allowed = allow_dynamic_lds(scatter_kernel, kKeepOutLdsBytes);
  if (allowed != hipSuccess) return hip_fail(allowed, "hipFuncSetAttribute (scatter kernel LDS)");
  const int row_vec = cfg->n_kv_heads * cfg->head_dim / 8;  // 16-byte pieces per row
  const int64_t total = (int64_t)n_sel * row_vec;
  int64_t blocks = (total + 1023) / 1024;
  if (blocks > 2048) blocks = 2048;
  launch_kernel(KC_SCATTER, scatter_kernel, dim3((unsigned)blocks), dim3(1024), kKeepOutLdsBytes, s,
                static_cast<u32x4*>(k_buf), static_cast<u32x4*>(v_buf), static_cast<const u32x4*>(k_sel),
                static_cast<const u32x4*>(v_sel), sel_idx, n_sel, row_vec);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(e, "scatter kernel launch");
  return CT_OK;
}

}  // namespace ct
