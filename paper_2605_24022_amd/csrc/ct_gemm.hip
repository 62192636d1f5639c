// The bf16 MFMA GEMM of the selected rows with fused epilogues:
//   - selective recompute of Q, K, V (Eq. 1) with RoPE at the rows' true positions
//     (Sec. 4.2, last paragraph);
//   - the other linear maps a transformer layer applies to the selected rows only
//     (Sec. 4.2: every layer after the check layer works on the selected tokens): output
//     projection and FFN down projection with the residual added, and the SwiGLU gate/up pair.
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
// v_mfma_f32_32x32x16_bf16, three weight-tile and two token-tile LDS slots of 32 KiB (loads run
// two and one K steps ahead), one barrier per K step, placed before the step's last MFMA group so
// that it passes while the matrix core is busy.  Two waves share a SIMD, so one wave's other
// waits hide behind the other's MFMAs.
// Workgroups are numbered so that the ones resident on one XCD (ids congruent mod 8) cover a
// patch of neighbouring tiles and share their W and X tiles in that XCD's L2.
#include <string.h>

#include "ct_internal.h"

namespace ct {

namespace {

constexpr int BF = 256;           // features per workgroup
// tokens per workgroup: 128 * NB, NB = MFMA column tiles per wave (template parameter; 2 unless the
// grid would otherwise end in a mostly empty last round of workgroups)
constexpr int BK = 64;            // reduction elements per stage
constexpr int ROWB = BK * 2;      // LDS row in bytes (unpadded, swizzled)
constexpr int A_BYTES = BF * ROWB;
constexpr int A_SLOTS = 3, B_SLOTS = 2;   // LDS slots per operand tile

enum Epilogue { EPI_QKV_ROPE = 0, EPI_LINEAR = 1, EPI_SWIGLU = 2, EPI_PARTIAL = 3 };

struct GemmArgs {
  const uint16_t* hidden;        // B operand X [*, E], token major
  const int32_t* hidden_rows;    // optional row gather
  const uint16_t* wqkv;          // A operand W [O, E], feature major (SwiGLU: the gate matrix)
  const uint16_t* w_up;          // SwiGLU only: the up matrix [O, E]
  int32_t n_sel, E, O;           // tokens, reduction length, features (rows of W)
  int32_t nF, nT;                // tiles
  // this launch covers tiles v_begin .. v_begin + v_count - 1 (in the patch order below), each by
  // k_parts workgroups that take consecutive parts of the reduction (k_parts > 1: EPI_PARTIAL)
  int32_t v_begin, v_count, k_parts;
  float* partial;                // EPI_PARTIAL: fp32 [v_count * k_parts][256 tokens][256 features]
  // EPI_QKV_ROPE
  const int32_t* sel_pos;
  const int32_t* sel_idx;
  const uint16_t* bias;
  uint16_t* q_out;
  uint16_t* k_out;
  uint16_t* v_out;
  // optional: row of k_out / v_out that takes the keys and values of selected row t (the layer
  // buffers with kv_rows = sel_idx: the scatter of the recomputed rows done by the epilogue)
  const int32_t* kv_rows;
  int32_t Hq, Hkv;
  // EPI_LINEAR / EPI_SWIGLU: out[t, f] (+ residual[t, f]), row length O
  const uint16_t* residual;
  uint16_t* out;
};
typedef GemmArgs QkvArgs;

__device__ __forceinline__ int32_t position_of_row(const ChunkTable& tab, int32_t r) {
  int c = 0;
  while (c + 1 < tab.n && r >= tab.row_start[c + 1]) ++c;
  return tab.new_start[c] + (r - tab.row_start[c]);
}

// swizzle of the 16-byte pieces of LDS row r (rows are 128 bytes: two rows per 256-byte bank span)
__device__ __forceinline__ int swz(int r) { return (r >> 1) & 7; }

// Tile number -> (feature tile, token tile): tiles are numbered patch by patch (4 feature tiles x
// 8 token tiles), so that the workgroups resident on one XCD cover neighbouring tiles.
__device__ __forceinline__ void tile_of(int v, int nF, int nT, int* f_tile, int* t_tile) {
  constexpr int PF = 4, PT = 8;
  const int tp = v / (PT * nF);
  const int rem = v - tp * PT * nF;
  const int th = min(PT, nT - tp * PT);
  const int fp = rem / (PF * th);
  const int r2 = rem - fp * PF * th;
  const int fw = min(PF, nF - fp * PF);
  *f_tile = fp * PF + r2 % fw;
  *t_tile = tp * PT + r2 / fw;
}

// EPI_SWIGLU: the 128 A rows of a wave are 64 gate rows followed by the 64 up rows of the same
// output features, so gate and up of one (feature, token) land in the same lane and register
// index of accumulator tiles (m, m + 2) - the same pairing the half-split RoPE uses.
template <int EPI, int D, int STYLE, int NB, int NW>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(NW / 4, NW / 4))) void gemm_kernel(
    GemmArgs a, RopeTable rope, ChunkTable chunks) {
  constexpr int NWAVES = NW;                 // 8: two waves per SIMD, wave tile 128 x 32 NB; 4: one, 128 x 64 NB
  constexpr int A_LOADS = BF / 8 / NWAVES;   // wave-wide loads (8 rows each) per wave and stage
  constexpr int TW = 8 * NB / NW;            // 32-token MFMA tiles per wave
  constexpr int BT = 128 * NB;
  constexpr int B_BYTES = BT * ROWB;
  constexpr int B_LOADS = BT / 8 / NWAVES;
  __shared__ __align__(1024) unsigned char lds[A_SLOTS * A_BYTES + B_SLOTS * B_BYTES];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hi = lane >> 5;

  // ---- workgroup -> tile, XCD aware (consecutive ids go to different XCDs) ----------------
  const int items = a.v_count * a.k_parts;
  const int per_xcd = (items + kNumXCDs - 1) / kNumXCDs;
  const int item = (blockIdx.x % kNumXCDs) * per_xcd + blockIdx.x / kNumXCDs;
  if (item >= items) return;
  const int kp = item % a.k_parts;
  int f_tile, t_tile;
  tile_of(a.v_begin + item / a.k_parts, a.nF, a.nT, &f_tile, &t_tile);
  const int f_blk = f_tile * (EPI == EPI_SWIGLU ? BF / 2 : BF);   // first output feature
  const int t_blk = t_tile * BT;

  // ---- global -> LDS loads -------------------------------------------------------------------
  // load j of this wave fills LDS rows (NWAVES * j + wave) * 8 .. + 7 of the A (or B) tile; this
  // lane supplies physical piece lane % 8 of row lane / 8, i.e. logical piece (that ^ swizzle).
  // Byte offsets from the tensor bases fit 32 bits (the entry points check the extents of the
  // weights and of compact token matrices; gathered rows are the caller's contract); the K step advances
  // the scalar base, so the per-lane offsets are loop invariant.
  uint32_t a_off[A_LOADS], b_off[B_LOADS];
#pragma unroll
  for (int j = 0; j < A_LOADS; ++j) {
    const int row = (NWAVES * j + wave) * 8 + (lane >> 3);
    // SwiGLU: tile row -> (wave half, gate | up, feature within the wave's 64)
    const int frow = EPI == EPI_SWIGLU ? f_blk + (row >> 7) * 64 + (row & 63) : f_blk + row;
    const int f = min(frow, a.O - 1);
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
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(m0), "v"(byte_off), "s"(base) : "memory", "m0");
  };
  // A (weight) tiles cycle through three LDS slots, B (token) tiles through two.  `half` selects
  // the first or second half of a tile's loads.
  auto issue_a = [&](int k0, int slot, int half) __attribute__((always_inline)) {
    const uint16_t* wk = a.wqkv + k0;      // scalar bases advanced to the K step
    const uint16_t* uk = EPI == EPI_SWIGLU ? a.w_up + k0 : wk;
    const uint32_t st = lds_addr0 + slot * A_BYTES;
#pragma unroll
    for (int j = half * (A_LOADS / 2); j < (half + 1) * (A_LOADS / 2); ++j) {
      // a wave-wide load covers 8 consecutive tile rows: all gate or all up
      const bool up = EPI == EPI_SWIGLU && ((((NWAVES * j + wave) * 8) >> 6) & 1);
      dma16(up ? uk : wk, a_off[j], st + (NWAVES * j + wave) * 1024);
    }
  };
  auto issue_b = [&](int k0, int slot, int half) __attribute__((always_inline)) {
    const uint16_t* xk = a.hidden + k0;
    const uint32_t st = lds_addr0 + A_SLOTS * A_BYTES + slot * B_BYTES;
#pragma unroll
    for (int j = half * (B_LOADS / 2); j < (half + 1) * (B_LOADS / 2); ++j)
      dma16(xk, b_off[j], st + (NWAVES * j + wave) * 1024);
  };

  const int wf = wave & 1, wt = wave >> 1;
  // fragment read offsets inside a stage (bytes): row base + swizzled piece, per k-step
  int a_frag[BK / 16], b_frag[BK / 16];
#pragma unroll
  for (int ks = 0; ks < BK / 16; ++ks) {
    a_frag[ks] = (wf * 128 + l32) * ROWB + (((2 * ks + hi) ^ swz(l32)) * 16);
    b_frag[ks] = (wt * 32 * TW + l32) * ROWB + (((2 * ks + hi) ^ swz(l32)) * 16);
  }

  f32x16 acc[4][TW];
#pragma unroll
  for (int m = 0; m < 4; ++m)
#pragma unroll
    for (int n = 0; n < TW; ++n)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[m][n][i] = 0.f;

  // Pipeline.  The weight tile of K step kt + 2 and the token tile of step kt + 1 are in flight
  // while step kt is multiplied (all 160 KiB of LDS: 3 + 2 slots of 32 KiB); with one step in
  // flight the load path alone (issue, L2 latency, barrier) takes as long as the MFMAs of a step.
  // Loads are issued in the order B(kt + 1), A(kt + 2), so when step kt + 1 is about to start
  // everything but the newest A_LOADS loads - A(kt + 2) - is waited for.  Past the end the last
  // step is loaded again into the free slots, which keeps the number of loads in flight, and the
  // wait, uniform.
  // The workgroup barrier of a step sits before its last MFMA group, not after it: a wave waits
  // for its loads of the next step, meets the others, issues the first fragment reads of the
  // next step and only then issues the last 4 x TW MFMAs of this step, so the barrier and the
  // LDS latency that follows it pass while the matrix core still has work queued.  (All waves of
  // a workgroup stand at the barrier together, so the other wave of the SIMD cannot cover it.)
  // this workgroup's part of the reduction: K steps kbeg .. kbeg + nk - 1
  const int nk_all = a.E / BK;
  const int kbeg = (int)((long)kp * nk_all / a.k_parts);
  const int nk = (int)((long)(kp + 1) * nk_all / a.k_parts) - kbeg;
  const int kbase = kbeg * BK;
  constexpr int WAIT_STEP = (A_LOADS & 15) | 0x0f70;   // s_waitcnt vmcnt(A_LOADS)
  __builtin_amdgcn_s_waitcnt(0x0f70);   // ordinary loads so far (row indices) are complete
  issue_a(kbase, 0, 0); issue_a(kbase, 0, 1);
  issue_b(kbase, 0, 0); issue_b(kbase, 0, 1);
  issue_a(kbase + min(1, nk - 1) * BK, 1, 0); issue_a(kbase + min(1, nk - 1) * BK, 1, 1);
  int sa = 0, sb = 0;
  // The fragment reads of MFMA group ks + 1 are issued before the MFMAs of group ks (two register
  // sets), so a wave waits for LDS once per K step instead of once per group.
  bf16x8 fa[2][4], fb[2][TW];
  auto read_frags = [&](const unsigned char* a_base, const unsigned char* b_base, int ks, int set) __attribute__((always_inline)) {
#pragma unroll
    for (int n = 0; n < TW; ++n) fb[set][n] = *reinterpret_cast<const bf16x8*>(b_base + b_frag[ks] + n * 32 * ROWB);
#pragma unroll
    for (int m = 0; m < 4; ++m) fa[set][m] = *reinterpret_cast<const bf16x8*>(a_base + a_frag[ks] + m * 32 * ROWB);
  };
  auto mfma_group = [&](int set) __attribute__((always_inline)) {
#pragma unroll
    for (int m = 0; m < 4; ++m)
#pragma unroll
      for (int n = 0; n < TW; ++n)
        acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[set][m], fb[set][n], acc[m][n], 0, 0, 0);
  };
  __builtin_amdgcn_s_waitcnt(WAIT_STEP);   // this wave's loads of step 0 have landed
  __syncthreads();                         // everybody's have
  read_frags(lds, lds + A_SLOTS * A_BYTES, 0, 0);
  for (int kt = 0; kt < nk; ++kt) {
    const unsigned char* a_base = lds + sa * A_BYTES;
    const unsigned char* b_base = lds + A_SLOTS * A_BYTES + sb * B_BYTES;
    const int sa_free = sa == 0 ? A_SLOTS - 1 : sa - 1;   // slot of step kt - 1
    const int sb_free = sb ^ 1;
    const int sa_next = sa == A_SLOTS - 1 ? 0 : sa + 1;
    const int kb1 = kbase + min(kt + 1, nk - 1) * BK, ka2 = kbase + min(kt + 2, nk - 1) * BK;
#pragma unroll
    for (int ks = 0; ks < BK / 16 - 1; ++ks) {
      // the loads go out a part at a time, one part per MFMA group: a burst of all of them from
      // all waves would queue at the texture addresser.  B first: it is needed a step earlier.
      if (ks == 0) { issue_b(kb1, sb_free, 0); issue_b(kb1, sb_free, 1); }
      else issue_a(ka2, sa_free, ks - 1);
      read_frags(a_base, b_base, ks + 1, (ks + 1) & 1);
      __builtin_amdgcn_sched_barrier(0);
      mfma_group(ks & 1);
      __builtin_amdgcn_sched_barrier(0);
    }
    __builtin_amdgcn_s_waitcnt(WAIT_STEP & ~0x0f00);   // vmcnt(A_LOADS): this wave's loads of step kt + 1 have
                                                        // landed; lgkmcnt(0): its fragment reads of step kt are done
    __syncthreads();                         // everybody's have; everybody is done reading step kt
    read_frags(lds + sa_next * A_BYTES, lds + A_SLOTS * A_BYTES + sb_free * B_BYTES, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    mfma_group((BK / 16 - 1) & 1);
    __builtin_amdgcn_sched_barrier(0);
    sa = sa_next;
    sb = sb_free;
  }
  __builtin_amdgcn_s_waitcnt(0x0f70);   // the repeated loads of the last steps have landed before the LDS is released

  // ---- epilogues ---------------------------------------------------------------------------------
  // accumulator element i of tile (m, n): row f0 + m*32 + 8*(i/4) + 4*hi + i%4, token = column l32
  // In an accumulator tile the lanes l and l + 32 hold features 8g + 0..3 and 8g + 4..7 of one
  // token (g = 0..3).  v_permlane32_swap between the packed results of groups 2q and 2q + 1 gives
  // lane l all eight features of group 2q and lane l + 32 those of group 2q + 1, so a tile leaves as
  // two 16-byte stores per lane instead of four 8-byte ones.  `p` points at the token's row at the
  // tile's first feature.  Every lane of the wave must come here (the swap crosses the two halves
  // of the wave); `ok` gates the store alone.
  auto store_tile = [&](uint16_t* p, const f32x16& c, bool ok) __attribute__((always_inline)) {
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const int g0 = 8 * q, g1 = 8 * q + 4;
      const auto x0 = __builtin_amdgcn_permlane32_swap(pack_bf16(c[g0], c[g0 + 1]), pack_bf16(c[g1], c[g1 + 1]), false, false);
      const auto x1 = __builtin_amdgcn_permlane32_swap(pack_bf16(c[g0 + 2], c[g0 + 3]), pack_bf16(c[g1 + 2], c[g1 + 3]), false, false);
      const u32x4 out16 = {x0[0], x1[0], x0[1], x1[1]};
      if (ok) *reinterpret_cast<u32x4*>(p + 16 * q + 8 * hi) = out16;
    }
  };
  if constexpr (EPI == EPI_PARTIAL) {
    // fp32 partial sums of this part of the reduction, token major inside the tile, 16-byte stores
    float* dst = a.partial + (size_t)item * (BT * BF);
#pragma unroll
    for (int n = 0; n < TW; ++n) {
      const int tl = wt * 32 * TW + n * 32 + l32;
#pragma unroll
      for (int m = 0; m < 4; ++m)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const f32x4 w = {acc[m][n][4 * g + 0], acc[m][n][4 * g + 1], acc[m][n][4 * g + 2], acc[m][n][4 * g + 3]};
          *reinterpret_cast<f32x4*>(dst + (size_t)tl * BF + wf * 128 + m * 32 + 8 * g + 4 * hi) = w;
        }
    }
    return;
  } else if constexpr (EPI == EPI_LINEAR) {
    const int f0 = f_blk + wf * 128;
    // Residuals arrive the same way, as 16-byte loads of the lane's eight features, and are swapped
    // back into the accumulator layout.  All residual values of the wave's tile are fetched before
    // the first result is stored: `out` may be the residual buffer itself, so the compiler cannot
    // move these loads above stores on its own, and with few loads in flight per lane the epilogue
    // is bound by memory latency.
    u32x4 res[TW][4][2];
    if (a.residual != nullptr) {
#pragma unroll
      for (int n = 0; n < TW; ++n) {
        const int t = min(t_blk + wt * 32 * TW + n * 32 + l32, a.n_sel - 1);
#pragma unroll
        for (int m = 0; m < 4; ++m) {
          const int fm = min(f0 + m * 32, a.O - 32);
          const size_t row = (size_t)t * a.O + fm + 8 * hi;
#pragma unroll
          for (int q = 0; q < 2; ++q) res[n][m][q] = *reinterpret_cast<const u32x4*>(a.residual + row + 16 * q);
        }
      }
    }
#pragma unroll
    for (int n = 0; n < TW; ++n) {
      const int t = t_blk + wt * 32 * TW + n * 32 + l32;
      const bool t_ok = t < a.n_sel;
#pragma unroll
      for (int m = 0; m < 4; ++m) {
        const int fm = f0 + m * 32;
        if (fm >= a.O) continue;            // uniform for the wave
        if (a.residual != nullptr) {
#pragma unroll
          for (int q = 0; q < 2; ++q) {
            // r[0], r[1]: features +0..3 of the lane's eight, r[2], r[3]: +4..7
            const u32x4 r = res[n][m][q];
            const auto d0 = __builtin_amdgcn_permlane32_swap(r[0], r[2], false, false);   // dword 0 of groups 2q, 2q + 1
            const auto d1 = __builtin_amdgcn_permlane32_swap(r[1], r[3], false, false);   // dword 1
#pragma unroll
            for (int e = 0; e < 2; ++e) {
              const int i0 = 4 * (2 * q + e);
              acc[m][n][i0 + 0] += bf16_lo(d0[e]);
              acc[m][n][i0 + 1] += bf16_hi(d0[e]);
              acc[m][n][i0 + 2] += bf16_lo(d1[e]);
              acc[m][n][i0 + 3] += bf16_hi(d1[e]);
            }
          }
        }
        store_tile(a.out + (size_t)(t_ok ? t : 0) * a.O + fm, acc[m][n], t_ok);
      }
    }
    return;
  } else if constexpr (EPI == EPI_SWIGLU) {
    const int f0 = f_blk + wf * 64;          // output features of this wave: f0 .. f0 + 63
#pragma unroll
    for (int n = 0; n < TW; ++n) {
      const int t = t_blk + wt * 32 * TW + n * 32 + l32;
      const bool t_ok = t < a.n_sel;
#pragma unroll
      for (int m = 0; m < 2; ++m) {          // gate tile m, up tile m + 2
        const int fm = f0 + m * 32;
        if (fm >= a.O) continue;             // uniform for the wave
        f32x16 y;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float gate = acc[m][n][i], up = acc[m + 2][n][i];
          y[i] = gate / (1.0f + __builtin_amdgcn_exp2f(-gate * 1.4426950408889634f)) * up;   // silu(gate) * up
        }
        store_tile(a.out + (size_t)(t_ok ? t : 0) * a.O + fm, y, t_ok);
      }
    }
    return;
  } else {
    // accumulator element i of tile (m, n): feature f0 + m*32 + 8*(i/4) + 4*hi + i%4, token = column l32
    const int f0 = f_blk + wf * 128;
    const int rope_end = (a.Hq + a.Hkv) * D;   // features below this are q or k heads
    const int q_end = a.Hq * D;
  #pragma unroll
    for (int n = 0; n < TW; ++n) {
      const int t = t_blk + wt * 32 * TW + n * 32 + l32;
      const bool t_ok = t < a.n_sel;
      const int tc = t_ok ? t : a.n_sel - 1;
      const int32_t pos = a.sel_pos ? a.sel_pos[tc] : position_of_row(chunks, a.sel_idx[tc]);
      const int32_t kv_row = a.kv_rows ? a.kv_rows[tc] : tc;

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

  #pragma unroll
      for (int m = 0; m < 4; ++m) {
        const int fm = f0 + m * 32;
        if (fm >= a.O) continue;             // uniform for the wave
        uint16_t* dst;
        if (fm < q_end)
          dst = a.q_out + (size_t)tc * q_end + fm;
        else if (fm < rope_end)
          dst = a.k_out + (size_t)kv_row * (a.Hkv * D) + (fm - q_end);
        else
          dst = a.v_out + (size_t)kv_row * (a.Hkv * D) + (fm - rope_end);
        store_tile(dst, acc[m][n], t_ok);
      }
    }
  }
}

// Sum of the k_parts partial tiles of EPI_PARTIAL (+ residual), rounded to bf16 and written to
// out[t, f].  One thread per token and four consecutive features; a workgroup covers 4 tokens.
__global__ __launch_bounds__(256) void gemm_reduce_kernel(GemmArgs a) {
  const int tile_local = blockIdx.x >> 6;                 // 64 workgroups per 256 x 256 tile
  const int tl = ((blockIdx.x & 63) << 2) + (threadIdx.x >> 6);
  const int fl = (threadIdx.x & 63) << 2;
  int f_tile, t_tile;
  tile_of(a.v_begin + tile_local, a.nF, a.nT, &f_tile, &t_tile);
  const int t = t_tile * 256 + tl, f = f_tile * BF + fl;
  if (t >= a.n_sel || f >= a.O) return;
  const float* src = a.partial + ((size_t)tile_local * a.k_parts * 256 + tl) * BF + fl;
  f32x4 sum = *reinterpret_cast<const f32x4*>(src);
  for (int kp = 1; kp < a.k_parts; ++kp) {
    const f32x4 p = *reinterpret_cast<const f32x4*>(src + (size_t)kp * (256 * BF));
    sum += p;
  }
  const size_t o = (size_t)t * a.O + f;
  if (a.residual != nullptr) {
    const u32x2 r = *reinterpret_cast<const u32x2*>(a.residual + o);
    sum[0] += bf16_lo(r[0]); sum[1] += bf16_hi(r[0]); sum[2] += bf16_lo(r[1]); sum[3] += bf16_hi(r[1]);
  }
  u32x2 w;
  w[0] = pack_bf16(sum[0], sum[1]);
  w[1] = pack_bf16(sum[2], sum[3]);
  *reinterpret_cast<u32x2*>(a.out + o) = w;
}

}  // namespace

static void fill_tiles(GemmArgs* a, bool swiglu, int nb) {
  a->nF = (a->O + (swiglu ? BF / 2 : BF) - 1) / (swiglu ? BF / 2 : BF);
  a->nT = (a->n_sel + 128 * nb - 1) / (128 * nb);
  a->v_begin = 0;
  a->v_count = a->nF * a->nT;
  a->k_parts = 1;
}

// Token tile width for a launch: 256 tokens per workgroup unless the workgroups then fill the last
// round over the 256 compute units so badly that 128-token tiles (about 0.56 of the time of a
// 256-token tile each) finish earlier.
static int pick_nb(const GemmArgs& a, bool swiglu) {
  GemmArgs t = a;
  double cost[3] = {0, 0, 0};
  for (int nb = 1; nb <= 2; ++nb) {
    fill_tiles(&t, swiglu, nb);
    const long wgs = (long)t.nF * t.nT;
    cost[nb] = (double)((wgs + kNumCUs - 1) / kNumCUs) * (nb == 2 ? 1.0 : 0.56);
  }
  return cost[1] < cost[2] ? 1 : 2;
}

template <typename Kernel>
static ct_status launch_gemm(Kernel kernel, int threads, const GemmArgs& a, const RopeTable& rope, const ChunkTable& tab,
                             KernelClass kc, hipStream_t s) {
  const int items = a.v_count * a.k_parts;
  const int per_xcd = (items + kNumXCDs - 1) / kNumXCDs;
  dim3 grid(per_xcd * kNumXCDs), block(threads);
  launch_kernel(kc, kernel, grid, block, 0, s, a, rope, tab);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(e, "gemm kernel launch");
  return CT_OK;
}

template <int EPI, int D, int STYLE, int NB>
static ct_status launch_variant(const GemmArgs& a, const RopeTable& rope, const ChunkTable& tab, KernelClass kc,
                                hipStream_t s) {
  // Eight waves.  Four (one per SIMD, 128 x 128 wave tiles, half the LDS reads per MFMA) compile
  // from the same source and were measured: no faster on any layer shape.
  return launch_gemm(gemm_kernel<EPI, D, STYLE, NB, 8>, 512, a, rope, tab, kc, s);
}

ct_status launch_qkv(const ct_layer_cfg* cfg, const void* hidden, const int32_t* hidden_rows, const int32_t* sel_pos,
                     const int32_t* sel_idx, const ChunkTable* chunks, int32_t n_sel, const void* wqkv,
                     const void* bias, void* q_out, void* k_out, void* v_out, hipStream_t s,
                     const int32_t* kv_rows) {
  if (n_sel == 0) return CT_OK;
  GemmArgs a;
  memset(&a, 0, sizeof(a));
  a.hidden = static_cast<const uint16_t*>(hidden);
  a.hidden_rows = hidden_rows;
  a.kv_rows = kv_rows;
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
  const int nb = pick_nb(a, false);
  fill_tiles(&a, false, nb);
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
  if (nb == 2) {
    if (cfg->head_dim == 128)
      return cfg->rope_style == 0 ? launch_variant<EPI_QKV_ROPE, 128, 0, 2>(a, rope, tab, KC_QKV, s)
                                  : launch_variant<EPI_QKV_ROPE, 128, 1, 2>(a, rope, tab, KC_QKV, s);
    return cfg->rope_style == 0 ? launch_variant<EPI_QKV_ROPE, 64, 0, 2>(a, rope, tab, KC_QKV, s)
                                : launch_variant<EPI_QKV_ROPE, 64, 1, 2>(a, rope, tab, KC_QKV, s);
  }
  if (cfg->head_dim == 128)
    return cfg->rope_style == 0 ? launch_variant<EPI_QKV_ROPE, 128, 0, 1>(a, rope, tab, KC_QKV, s)
                                : launch_variant<EPI_QKV_ROPE, 128, 1, 1>(a, rope, tab, KC_QKV, s);
  return cfg->rope_style == 0 ? launch_variant<EPI_QKV_ROPE, 64, 0, 1>(a, rope, tab, KC_QKV, s)
                              : launch_variant<EPI_QKV_ROPE, 64, 1, 1>(a, rope, tab, KC_QKV, s);
}

// The last round of 256-token tiles of a linear launch, when it would leave most compute units
// idle, is run with the reduction of each tile split over several workgroups (fp32 partial tiles
// in `ws`, then a small kernel that adds them, and the residual, and rounds).  Returns the number
// of parts, or 1 when splitting is not worth it or `ws` is too small.
static int split_plan(const GemmArgs& a256, size_t ws_bytes, double cost_unsplit, int n_cu, int* full_tiles) {
  const int tiles = a256.nF * a256.nT;
  const int rem = tiles % n_cu;
  const int nk = a256.E / BK;
  *full_tiles = tiles - rem;
  if (rem == 0 || rem > n_cu / 2) return 1;
  int parts = n_cu / rem;
  if (parts > 8) parts = 8;
  if (parts > nk / 8) parts = nk / 8;
  if (parts < 2) return 1;
  if (ws_bytes < (size_t)rem * parts * 256 * BF * sizeof(float)) return 1;
  // in units of one round of 256-token tiles: the split round, plus the partial tiles' trip
  // through memory and the two extra launches (measured: 0.45 of a round for 256 partial tiles at
  // K = 4096, where a round takes 100 us; in proportion less for longer reductions)
  const double cost = (double)(*full_tiles / n_cu) + 1.05 / parts + 0.45 * (64.0 / nk) * (rem * parts / 256.0);
  return cost < cost_unsplit ? parts : 1;
}

size_t linear_workspace_bytes(int32_t n_tok, int32_t k_len, int32_t n_out) {
  GemmArgs a;
  memset(&a, 0, sizeof(a));
  a.n_sel = n_tok;
  a.E = k_len;
  a.O = n_out;
  fill_tiles(&a, false, 2);
  // at most one partial tile per compute unit, whatever share of the chip the launch is planned for
  const int tiles = a.nF * a.nT;
  return (size_t)(tiles < kNumCUs ? tiles * 8 < kNumCUs ? tiles * 8 : kNumCUs : kNumCUs) * 256 * BF * sizeof(float);
}

ct_status launch_linear(const void* x, int32_t n_tok, int32_t k_len, const void* w, int32_t n_out, const void* residual,
                        void* out, void* ws, size_t ws_bytes, int n_cu, hipStream_t s) {
  if (n_tok == 0) return CT_OK;
  GemmArgs a;
  memset(&a, 0, sizeof(a));
  a.hidden = static_cast<const uint16_t*>(x);
  a.wqkv = static_cast<const uint16_t*>(w);
  a.residual = static_cast<const uint16_t*>(residual);
  a.out = static_cast<uint16_t*>(out);
  a.n_sel = n_tok;
  a.E = k_len;
  a.O = n_out;
  RopeTable rope;
  memset(&rope, 0, sizeof(rope));
  ChunkTable tab;
  memset(&tab, 0, sizeof(tab));
  const int nb = pick_nb(a, false);
  if (ws != nullptr) {
    GemmArgs t2 = a, t1 = a;
    fill_tiles(&t2, false, 2);
    fill_tiles(&t1, false, 1);
    if (n_cu <= 0 || n_cu > kNumCUs) n_cu = kNumCUs;
    const double c2 = (double)((t2.nF * t2.nT + n_cu - 1) / n_cu), c1 = 0.56 * (double)((t1.nF * t1.nT + n_cu - 1) / n_cu);
    int full = 0;
    const int parts = split_plan(t2, ws_bytes, c1 < c2 ? c1 : c2, n_cu, &full);
    if (parts > 1) {
      ct_status st = CT_OK;
      a = t2;
      if (full > 0) {
        a.v_count = full;
        if ((st = launch_variant<EPI_LINEAR, 128, 0, 2>(a, rope, tab, KC_LINEAR, s)) != CT_OK) return st;
      }
      a.v_begin = full;
      a.v_count = t2.nF * t2.nT - full;
      a.k_parts = parts;
      a.partial = static_cast<float*>(ws);
      if ((st = launch_variant<EPI_PARTIAL, 128, 0, 2>(a, rope, tab, KC_LINEAR, s)) != CT_OK) return st;
      launch_kernel(KC_LINEAR, gemm_reduce_kernel, dim3(a.v_count * 64), dim3(256), 0, s, a);
      hipError_t e = hipGetLastError();
      if (e != hipSuccess) return hip_fail(e, "gemm reduce launch");
      return CT_OK;
    }
  }
  fill_tiles(&a, false, nb);
  return nb == 2 ? launch_variant<EPI_LINEAR, 128, 0, 2>(a, rope, tab, KC_LINEAR, s)
                 : launch_variant<EPI_LINEAR, 128, 0, 1>(a, rope, tab, KC_LINEAR, s);
}

ct_status launch_swiglu(const void* x, int32_t n_tok, int32_t k_len, const void* w_gate, const void* w_up, int32_t n_out,
                        void* out, hipStream_t s) {
  if (n_tok == 0) return CT_OK;
  GemmArgs a;
  memset(&a, 0, sizeof(a));
  a.hidden = static_cast<const uint16_t*>(x);
  a.wqkv = static_cast<const uint16_t*>(w_gate);
  a.w_up = static_cast<const uint16_t*>(w_up);
  a.out = static_cast<uint16_t*>(out);
  a.n_sel = n_tok;
  a.E = k_len;
  a.O = n_out;
  const int nb = pick_nb(a, true);
  fill_tiles(&a, true, nb);
  RopeTable rope;
  memset(&rope, 0, sizeof(rope));
  ChunkTable tab;
  memset(&tab, 0, sizeof(tab));
  return nb == 2 ? launch_variant<EPI_SWIGLU, 128, 0, 2>(a, rope, tab, KC_LINEAR, s)
                 : launch_variant<EPI_SWIGLU, 128, 0, 1>(a, rope, tab, KC_LINEAR, s);
}

}  // namespace ct
