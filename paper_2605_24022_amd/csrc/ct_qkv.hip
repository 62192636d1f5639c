// Selective recompute of Q, K, V for the selected tokens (Eq. 1) with RoPE at their true
// positions (Sec. 4.2, last paragraph), as one bf16 MFMA GEMM with a fused epilogue.
//
// The kernel computes the transposed product  C^T[f, t] = sum_e W[f, e] * X[row(t), e]
// (features in the MFMA M dimension, tokens in N) so that, in the 32x32 accumulator layout,
// a lane holds one token (column) and groups of four consecutive features (rows):
//   - both elements of every RoPE pair of a token sit in the same lane (no cross-lane
//     traffic in the epilogue), and the token's position is a per-lane scalar;
//   - results leave as 8-byte stores of four consecutive bf16 features.
// Both operands are K-contiguous in memory (W is out-features major, X is token major).
// Tiles go from global memory straight into LDS (global_load_lds_dwordx4, no register
// staging): a wave-wide load fills 8 rows of 128 bytes, the 16-byte pieces of a row are
// XOR-swizzled so that the 128-bit fragment reads of 16 consecutive rows hit distinct banks.
//
// Workgroup: 512 threads = 8 waves (2 feature halves x 4 token quarters), tile 256 features x
// 256 tokens x 64 (K step), wave tile 128 x 64 = 4 x 2 MFMA tiles of
// v_mfma_f32_32x32x16_bf16, two LDS stages of 64 KiB, one barrier per K step.  Two waves
// share a SIMD, so one wave's fragment reads and waits hide behind the other's MFMAs.
// Workgroups are numbered so that the ones resident on one XCD (ids congruent mod 8) cover a
// patch of neighbouring tiles and share their W and X tiles in that XCD's L2.
#include "ct_internal.h"

namespace ct {

namespace {

constexpr int BF = 256;           // features per workgroup
constexpr int BT = 256;           // tokens per workgroup
constexpr int BK = 64;            // reduction elements per stage
constexpr int ROWB = BK * 2;      // LDS row in bytes (unpadded, swizzled)
constexpr int A_BYTES = BF * ROWB;
constexpr int B_BYTES = BT * ROWB;
constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
constexpr int NWAVES = 8;
constexpr int A_LOADS = BF / 8 / NWAVES;   // wave-wide loads (8 rows each) per wave and stage
constexpr int B_LOADS = BT / 8 / NWAVES;

struct QkvArgs {
  const uint16_t* hidden;
  const int32_t* hidden_rows;
  const int32_t* sel_pos;
  const int32_t* sel_idx;
  const uint16_t* wqkv;
  const uint16_t* bias;
  uint16_t* q_out;
  uint16_t* k_out;
  uint16_t* v_out;
  int32_t n_sel, E, O, Hq, Hkv;
  int32_t nF, nT;
};

__device__ __forceinline__ int32_t position_of_row(const ChunkTable& tab, int32_t r) {
  int c = 0;
  while (c + 1 < tab.n && r >= tab.row_start[c + 1]) ++c;
  return tab.new_start[c] + (r - tab.row_start[c]);
}

// swizzle of the 16-byte pieces of LDS row r (rows are 128 bytes: two rows per 256-byte bank span)
__device__ __forceinline__ int swz(int r) { return (r >> 1) & 7; }

template <int D, int STYLE>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) void qkv_kernel(QkvArgs a, RopeTable rope,
                                                                                            ChunkTable chunks) {
  __shared__ __align__(1024) unsigned char lds[2 * STAGE_BYTES];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hi = lane >> 5;

  // ---- workgroup -> tile, XCD aware (consecutive ids go to different XCDs) ----------------
  const int total = a.nF * a.nT;
  const int per_xcd = (total + 7) / 8;
  const int v = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (v >= total) return;
  constexpr int PF = 4, PT = 8;
  const int tp = v / (PT * a.nF);
  const int rem = v - tp * PT * a.nF;
  const int th = min(PT, a.nT - tp * PT);
  const int fp = rem / (PF * th);
  const int r2 = rem - fp * PF * th;
  const int fw = min(PF, a.nF - fp * PF);
  const int f_blk = (fp * PF + r2 % fw) * BF;
  const int t_blk = (tp * PT + r2 / fw) * BT;

  // ---- global -> LDS loads -------------------------------------------------------------------
  // load j of this wave fills LDS rows (NWAVES * j + wave) * 8 .. + 7 of the A (or B) tile; this
  // lane supplies physical piece lane % 8 of row lane / 8, i.e. logical piece (that ^ swizzle).
  // Byte offsets from the tensor bases fit 32 bits (checked on the host); the K step advances
  // the scalar base, so the per-lane offsets are loop invariant.
  uint32_t a_off[A_LOADS], b_off[B_LOADS];
#pragma unroll
  for (int j = 0; j < A_LOADS; ++j) {
    const int row = (NWAVES * j + wave) * 8 + (lane >> 3);
    const int f = min(f_blk + row, a.O - 1);
    a_off[j] = ((uint32_t)f * a.E + (((lane & 7) ^ swz(row)) * 8)) * 2;
  }
#pragma unroll
  for (int j = 0; j < B_LOADS; ++j) {
    const int row = (NWAVES * j + wave) * 8 + (lane >> 3);
    const int t = min(t_blk + row, a.n_sel - 1);
    const uint32_t xr = a.hidden_rows ? (uint32_t)a.hidden_rows[t] : (uint32_t)t;
    b_off[j] = (xr * a.E + (((lane & 7) ^ swz(row)) * 8)) * 2;
  }
  typedef __attribute__((address_space(3))) void* lds_ptr_t;
  const uint32_t lds_addr0 = (uint32_t)(uintptr_t)(lds_ptr_t)lds;
  auto dma16 = [&](const uint16_t* base, uint32_t byte_off, uint32_t lds_addr) __attribute__((always_inline)) {
    const uint32_t m0 = __builtin_amdgcn_readfirstlane(lds_addr);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(m0), "v"(byte_off), "s"(base) : "memory");
  };
  auto issue_stage = [&](int k0, int stage) __attribute__((always_inline)) {
    const uint16_t* wk = a.wqkv + k0;      // scalar bases advanced to the K step
    const uint16_t* xk = a.hidden + k0;
    const uint32_t st = lds_addr0 + stage * STAGE_BYTES;
#pragma unroll
    for (int j = 0; j < A_LOADS; ++j) dma16(wk, a_off[j], st + (NWAVES * j + wave) * 1024);
#pragma unroll
    for (int j = 0; j < B_LOADS; ++j) dma16(xk, b_off[j], st + A_BYTES + (NWAVES * j + wave) * 1024);
  };

  const int wf = wave & 1, wt = wave >> 1;
  // fragment read offsets inside a stage (bytes): row base + swizzled piece, per k-step
  int a_frag[BK / 16], b_frag[BK / 16];
#pragma unroll
  for (int ks = 0; ks < BK / 16; ++ks) {
    a_frag[ks] = (wf * 128 + l32) * ROWB + (((2 * ks + hi) ^ swz(l32)) * 16);
    b_frag[ks] = A_BYTES + (wt * 64 + l32) * ROWB + (((2 * ks + hi) ^ swz(l32)) * 16);
  }

  f32x16 acc[4][2];
#pragma unroll
  for (int m = 0; m < 4; ++m)
#pragma unroll
    for (int n = 0; n < 2; ++n)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[m][n][i] = 0.f;

  const int nk = a.E / BK;
  __builtin_amdgcn_s_waitcnt(0x0f70);   // ordinary loads so far (row indices) are complete
  issue_stage(0, 0);
  for (int kt = 0; kt < nk; ++kt) {
    const int buf = kt & 1;
    __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0): this wave's part of stage kt has landed
    __syncthreads();                      // everybody's has; everybody is done reading the other stage
    if (kt + 1 < nk) issue_stage((kt + 1) * BK, buf ^ 1);
    const unsigned char* base = lds + buf * STAGE_BYTES;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 fa[4], fb[2];
#pragma unroll
      for (int m = 0; m < 4; ++m) fa[m] = *reinterpret_cast<const bf16x8*>(base + a_frag[ks] + m * 32 * ROWB);
#pragma unroll
      for (int n = 0; n < 2; ++n) fb[n] = *reinterpret_cast<const bf16x8*>(base + b_frag[ks] + n * 32 * ROWB);
#pragma unroll
      for (int m = 0; m < 4; ++m)
#pragma unroll
        for (int n = 0; n < 2; ++n)
          acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[m], fb[n], acc[m][n], 0, 0, 0);
    }
  }

  // ---- epilogue: bias, RoPE, round, store ---------------------------------------------------
  // accumulator element i of tile (m, n): feature f0 + m*32 + 8*(i/4) + 4*hi + i%4, token = column l32
  const int f0 = f_blk + wf * 128;
  const int rope_end = (a.Hq + a.Hkv) * D;   // features below this are q or k heads
  const int q_end = a.Hq * D;
#pragma unroll
  for (int n = 0; n < 2; ++n) {
    const int t = t_blk + wt * 64 + n * 32 + l32;
    const bool t_ok = t < a.n_sel;
    const int tc = t_ok ? t : a.n_sel - 1;
    const int32_t pos = a.sel_pos ? a.sel_pos[tc] : position_of_row(chunks, a.sel_idx[tc]);

    if (a.bias != nullptr) {
#pragma unroll
      for (int m = 0; m < 4; ++m)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int f = min(f0 + m * 32 + 8 * (i >> 2) + 4 * hi + (i & 3), a.O - 1);
          acc[m][n][i] += bf16_lo((uint32_t)a.bias[f]);
        }
    }

    if (STYLE == 0) {
      // pairs (j, j + D/2): D = 128 couples tiles (m, m+2); D = 64 couples (m, m+1) for m even
      constexpr int STEP = D / 64;          // tile distance between the two halves of a pair
#pragma unroll
      for (int m = 0; m < 4; ++m) {
        if ((D == 128 && m >= 2) || (D == 64 && (m & 1))) continue;
        const int fa0 = f0 + m * 32;        // first feature of the "a" half tile
        if (fa0 >= rope_end) continue;      // v heads are not rotated
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int j = (fa0 % D) + 8 * (i >> 2) + 4 * hi + (i & 3);
          float c, s;
          sincos_turns(pos, rope.turns[j], c, s);
          const float x = acc[m][n][i], y = acc[m + STEP][n][i];
          acc[m][n][i] = x * c - y * s;
          acc[m + STEP][n][i] = x * s + y * c;
        }
      }
    } else {
#pragma unroll
      for (int m = 0; m < 4; ++m) {
        const int fa0 = f0 + m * 32;
        if (fa0 >= rope_end) continue;
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
          const int j = ((fa0 % D) + 8 * (i >> 2) + 4 * hi + (i & 3)) >> 1;
          float c, s;
          sincos_turns(pos, rope.turns[j], c, s);
          const float x = acc[m][n][i], y = acc[m][n][i + 1];
          acc[m][n][i] = x * c - y * s;
          acc[m][n][i + 1] = x * s + y * c;
        }
      }
    }

    if (!t_ok) continue;
#pragma unroll
    for (int m = 0; m < 4; ++m) {
      const int fm = f0 + m * 32;
      if (fm >= a.O) continue;
      uint16_t* dst;
      if (fm < q_end)
        dst = a.q_out + (size_t)t * q_end + fm;
      else if (fm < rope_end)
        dst = a.k_out + (size_t)t * (a.Hkv * D) + (fm - q_end);
      else
        dst = a.v_out + (size_t)t * (a.Hkv * D) + (fm - rope_end);
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        u32x2 w;
        w[0] = pack_bf16(acc[m][n][4 * g + 0], acc[m][n][4 * g + 1]);
        w[1] = pack_bf16(acc[m][n][4 * g + 2], acc[m][n][4 * g + 3]);
        *reinterpret_cast<u32x2*>(dst + 8 * g + 4 * hi) = w;
      }
    }
  }
}

}  // namespace

ct_status launch_qkv(const ct_layer_cfg* cfg, const void* hidden, const int32_t* hidden_rows, const int32_t* sel_pos,
                     const int32_t* sel_idx, const ChunkTable* chunks, int32_t n_sel, const void* wqkv,
                     const void* bias, void* q_out, void* k_out, void* v_out, hipStream_t s) {
  if (n_sel == 0) return CT_OK;
  QkvArgs a;
  a.hidden = static_cast<const uint16_t*>(hidden);
  a.hidden_rows = hidden_rows;
  a.sel_pos = sel_pos;
  a.sel_idx = sel_idx;
  a.wqkv = static_cast<const uint16_t*>(wqkv);
  a.bias = static_cast<const uint16_t*>(bias);
  a.q_out = static_cast<uint16_t*>(q_out);
  a.k_out = static_cast<uint16_t*>(k_out);
  a.v_out = static_cast<uint16_t*>(v_out);
  a.n_sel = n_sel;
  a.E = cfg->hidden;
  a.Hq = cfg->n_q_heads;
  a.Hkv = cfg->n_kv_heads;
  a.O = (cfg->n_q_heads + 2 * cfg->n_kv_heads) * cfg->head_dim;
  a.nF = (a.O + BF - 1) / BF;
  a.nT = (n_sel + BT - 1) / BT;
  RopeTable rope;
  fill_rope_table(cfg, &rope);
  ChunkTable tab;
  if (chunks != nullptr) {
    tab = *chunks;
  } else {
    tab.n = 1;
    tab.row_start[0] = 0;
    tab.row_start[1] = 0x7fffffff;
    tab.new_start[0] = 0;
  }
  const int total = a.nF * a.nT;
  const int per_xcd = (total + 7) / 8;
  dim3 grid(per_xcd * 8), block(512);
  auto launch = [&](auto kernel) -> hipError_t {
    int slot = prof_begin(KC_QKV, s);
    hipLaunchKernelGGL(kernel, grid, block, 0, s, a, rope, tab);
    prof_end(KC_QKV, slot, s);
    return hipGetLastError();
  };
  hipError_t e;
  if (cfg->head_dim == 128)
    e = cfg->rope_style == 0 ? launch(qkv_kernel<128, 0>) : launch(qkv_kernel<128, 1>);
  else
    e = cfg->rope_style == 0 ? launch(qkv_kernel<64, 0>) : launch(qkv_kernel<64, 1>);
  if (e != hipSuccess) return hip_fail(e, "qkv kernel launch");
  return CT_OK;
}

}  // namespace ct
