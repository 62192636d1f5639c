// Causal attention for the selected query rows over the fused layer KV (Sec. 4.2: the
// check / fusion layers compute attention for the selected tokens alone), GQA aware.
//
// Formulation.  Everything is computed transposed so that a lane owns a query column:
//   S^T = K Q^T            A = K tile rows (keys) from LDS,       B = Q^T kept in registers
//   O^T += V^T P^T         A = V^T (head_dim x keys) from LDS,    B = P^T taken straight from
//                                                                     the S^T accumulators
// In the 32x32 MFMA accumulator layout lane l holds column l%32 (one query) and 16 rows
// (keys), so the row maximum and row sum of the softmax are in-lane reductions plus one
// exchange with lane l^32, the rescale factor of the online softmax is a per-lane scalar,
// and the probabilities need no trip through LDS: accumulator registers 8t..8t+7 of an
// S^T tile are exactly the B operand of PV step t once V^T is stored in LDS with the same
// key order (keys of a 32-key sub-tile are laid out as 16-byte units (t, lane-half) holding
// keys 16t + 8a + 4*half + b, a in {0,1}, b in 0..3).
//
// Work decomposition.  A workgroup (8 waves, two per SIMD) owns one KV head and a tile of 256
// query columns = (256 / G) selected tokens x the G query heads of that KV head; every wave
// owns 32 columns and all keys.  K and V tiles of 64 keys are staged once per workgroup in LDS
// by direct global->LDS loads (three stages each); V^T fragments come out of LDS with
// transposing reads.  The selected rows are sorted, so a tile needs keys [0, last position of
// the tile]; only key tiles that straddle a query position of the wave evaluate the causal mask.
// When (tile, head) pairs are too few to fill the chip, the key range is split and fp32
// partial (O, m, l) are merged by a second kernel; tiles whose keys fit one split write their
// result directly.
// Workgroup ids map KV head = id mod n_kv_heads, so with 8 KV heads every XCD streams the
// keys of one head through its own L2; tiles are issued heaviest first.
#include <math.h>
#include <stdlib.h>

#include "ct_internal.h"

namespace ct {

namespace {

constexpr int BN = 64;                 // keys per LDS tile

struct AttnArgs {
  const uint16_t* q;
  const uint16_t* k;
  const uint16_t* v;
  const int32_t* sel_idx;
  uint16_t* out;
  float* lse;
  float* partial;     // workspace when n_splits > 1
  int32_t n_sel, n_ctx, Hq, Hkv, G, TM, tm_shift, cols;
  int32_t n_tiles, n_splits, split_keys;
  // state == NULL: only tiles whose visible key count lies in (key_after, key_upto] are computed by
  // this launch (the rest by other launches, each started when the rows it needs are in place).
  // state != NULL: this launch takes every tile that sees keys past key_after through the keys
  // [key_after, key_upto) and no further; a tile that needs later keys leaves its fp32
  // (O, m, l) in `state` ([tile][kv head][256 columns][D], then m[256], l[256]) and the launch
  // for the next key range resumes from there.
  int32_t key_after, key_upto;
  float* state;
  float scale_log2;   // softmax scale * log2(e)
};

// The keys one workgroup (tile, key-range split) of a launch works through: [k_lo, k_hi), or nothing.
// Shared by the kernel and by the host-side check of the rows a launch reads.
struct ItemRange {
  int k_lo, k_hi;
  bool active;
};
__host__ __device__ inline ItemRange item_range(int kmax, int split, int split_keys, bool resumable, int key_after,
                                                int key_upto) {
  ItemRange r = {0, 0, false};
  if (kmax <= key_after || (!resumable && kmax > key_upto)) return r;   // another launch's tile
  r.k_lo = resumable ? key_after : split * split_keys;
  if (r.k_lo >= kmax) return r;                                          // empty split
  r.k_hi = resumable ? (key_upto < kmax ? key_upto : kmax)
                     : (r.k_lo + split_keys < kmax ? r.k_lo + split_keys : kmax);
  r.active = true;
  return r;
}
// Row of the K (or V) buffer behind row `row_in_tile` of the LDS tile that starts at key k0: rows from
// k_hi on (the end of the item's key range) are replaced by row k_hi - 1.
__host__ __device__ inline int tile_load_row(int k0, int row_in_tile, int k_hi) {
  const int key = k0 + row_in_tile;
  return key < k_hi - 1 ? key : k_hi - 1;
}

// v_permlane32_swap exchanges the upper half of the first operand with the lower half of
// the second: with both operands x, result[0] is (x | partner) and result[1] is
// (partner | x) over (lanes 0-31 | lanes 32-63), so any commutative combination of the two
// results combines every lane with lane ^ 32.
__device__ __forceinline__ float max_with_lane_xor32(float x) {
  const uint32_t u = __float_as_uint(x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_with_lane_xor32(float x) {
  const uint32_t u = __float_as_uint(x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((address_space(3))) void* lds_ptr_t;

// Swizzles of the 16-byte pieces inside a key row of the LDS tiles (rows are unpadded:
// direct global->LDS loads write 64 lanes x 16 bytes contiguously).  K rows are read one
// row per lane (ds_read_b128), V rows four rows per 16-lane block (ds_read_b64_tr_b16).
template <int D>
__device__ __forceinline__ int swz_k(int r) { return D == 128 ? (r & 15) : ((r >> 1) & 7); }
template <int D>
__device__ __forceinline__ int swz_v(int r) {
  return D == 128 ? (((r & 3) << 2) | ((r >> 2) & 3)) : (((r & 1) << 2) | ((r >> 1) & 3));
}

// A workgroup has 8 waves, two per SIMD; every wave owns 32 query columns (one MFMA column
// tile) and all keys, so the workgroup owns 256 query columns.
//
// Ping-pong schedule.  The work of a wave on key tile i splits into a matrix-core part
//   M(i): O^T += V^T(i-1) P^T(i-1), then S^T(i) = K(i) Q^T            (32 MFMAs)
// and a vector-ALU part
//   V(i): causal mask, online softmax of S^T(i) into P^T(i), rescale of O^T.
// The loop runs in periods separated by one workgroup barrier.  Waves 0-3 (one per SIMD) run
// M(i) and then V(i) in period i; waves 4-7 run V(i-1) and then M(i).  The two parts take about
// the same time, so each SIMD has one wave feeding the matrix cores and one wave doing softmax
// arithmetic for most of the period without a barrier between the halves (a second barrier
// there makes every wave wait for the slowest of eight twice per period: measured 2 % slower).
// K(i) and V(i-1) are the tiles in use during period i; K(i+2) and V(i+1) are fetched during
// it with direct global->LDS loads into three K and three V stages.
template <int D>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_kernel(AttnArgs a) {
  constexpr int NWAVES = 8;
  constexpr int COLS = 32 * NWAVES;            // query columns per workgroup
  constexpr int NST = 3;                       // LDS stages per tensor
  constexpr int ROWB = D * 2;                  // bytes per key row in LDS (no padding)
  constexpr int TILE_BYTES = BN * ROWB;        // one K (or V) tile
  constexpr int KS = D / 16;                   // MFMA k-steps over head_dim
  constexpr int MT = D / 32;                   // O^T row tiles
  constexpr int PCS = D / 8;                   // 16-byte pieces per key row
  constexpr int RPI = 64 / PCS;                // key rows covered by one wave-wide 16-byte load
  constexpr int INSTS = BN / RPI / NWAVES;     // such loads per wave, tile and tensor
  static_assert(INSTS >= 1 && (NWAVES * RPI) % 16 == 0, "tile / wave count mismatch");

  __shared__ __align__(1024) unsigned char k_lds[NST * TILE_BYTES];
  __shared__ __align__(1024) unsigned char v_lds[NST * TILE_BYTES];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hi = lane >> 5;
  const bool group_b = wave >= NWAVES / 2;

  // ---- work item ---------------------------------------------------------------------------
  const int g = blockIdx.x % a.Hkv;
  const int rest = blockIdx.x / a.Hkv;
  // split-major order: the workgroups resident on an XCD at one time work on neighbouring
  // tiles of the same key range and share its K/V lines in that XCD's L2
  const int split = rest / a.n_tiles;
  const int tile = a.n_tiles - 1 - rest % a.n_tiles;    // heaviest (latest) tiles first
  const int tok0 = tile * a.TM;
  const int last_tok = min(tok0 + a.TM, a.n_sel) - 1;
  const int kmax = a.sel_idx[last_tok] + 1;              // keys this tile can see
  const bool resumable = a.state != nullptr;
  const ItemRange item = item_range(kmax, split, a.split_keys, resumable, a.key_after, a.key_upto);
  if (!item.active) return;                              // uniform for the workgroup
  const int k_lo = item.k_lo, k_hi = item.k_hi;
  const int n_kt = (k_hi - k_lo + BN - 1) / BN;

  // ---- this lane's query column ------------------------------------------------------------------
  const int col = wave * 32 + l32;
  const int tok_raw = tok0 + (col & (a.TM - 1));
  const bool valid = tok_raw < a.n_sel;
  const int tokv = valid ? tok_raw : a.n_sel - 1;
  const int hq = g * a.G + (col >> a.tm_shift);
  // keys from k_hi on belong to a later launch (or to nobody): the causal mask is taken against
  // min(position, k_hi - 1), which cuts the last key tile of the range where the range ends
  const int pos = min(a.sel_idx[tokv], k_hi - 1);
  int wmin = pos;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) wmin = min(wmin, __shfl_xor(wmin, off));
  wmin = __builtin_amdgcn_readfirstlane(wmin);

  // Q^T fragments: B operand, lane = column, 8 consecutive head_dim elements per k-step
  bf16x8 qf[KS];
  {
    const uint16_t* qp = a.q + ((size_t)tokv * a.Hq + hq) * D + hi * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16);
  }

  // ---- global -> LDS staging (direct loads, no registers) ----------------------------------
  // load i of this wave fills LDS rows (NWAVES * i + wave) * RPI .. + RPI - 1 of a tile; this
  // lane supplies physical piece lane % PCS of row lane / PCS, i.e. logical piece
  // (that ^ swizzle); NWAVES * RPI is a multiple of 16 rows, so the swizzle is the same for all i
  const int ld_row = wave * RPI + lane / PCS;
  const int ld_pk = (lane % PCS) ^ swz_k<D>(ld_row);
  const int ld_pv = (lane % PCS) ^ swz_v<D>(ld_row);
  // byte offsets from the tensor bases fit 32 bits and row numbers 24 (checked on the host)
  const uint32_t kv_row_bytes = (uint32_t)a.Hkv * D * 2;
  const uint32_t k_lane_off = ((uint32_t)g * D + ld_pk * 8) * 2;
  const uint32_t v_lane_off = ((uint32_t)g * D + ld_pv * 8) * 2;
  // The loads are inline assembly (M0 = LDS base of the wave's 1 KiB slot, each lane lands at
  // +16 * lane): the compiler neither reorders them nor adds waits of its own; the pipeline
  // below orders them against the fragment reads with explicit vmcnt waits and barriers.
  auto dma16 = [&](const uint16_t* base, uint32_t byte_off, uint32_t lds_addr) __attribute__((always_inline)) {
    const uint32_t m0 = __builtin_amdgcn_readfirstlane(lds_addr);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(m0), "v"(byte_off), "s"(base) : "memory", "m0");
  };
  const uint32_t k_lds_addr = (uint32_t)(uintptr_t)(lds_ptr_t)k_lds;
  const uint32_t v_lds_addr = (uint32_t)(uintptr_t)(lds_ptr_t)v_lds;
  // One wave-wide load: rows (NWAVES * idx + wave) * RPI .. of the tile that starts at key k0.
  // Rows from k_hi on (the end of this item's key range) are replaced by row k_hi - 1: they are
  // masked (their probabilities are zero), or belong to look-ahead tiles that are never consumed,
  // but what stands in those rows may not have been written yet - a later group of chunks still on
  // the host link - and a non-finite bit pattern there would turn 0 * v into NaN in the PV product.
  auto issue_one = [&](const uint16_t* base, uint32_t lane_off, int k0, uint32_t stage_addr, int idx) __attribute__((always_inline)) {
    const int key = tile_load_row(k0, ld_row + NWAVES * RPI * idx, k_hi);
    dma16(base, __umul24(key, kv_row_bytes) + lane_off, stage_addr + (NWAVES * idx + wave) * 1024);
  };
  auto issue_rows = [&](const uint16_t* base, uint32_t lane_off, int k0, uint32_t stage_addr) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < INSTS; ++i) issue_one(base, lane_off, k0, stage_addr, i);
  };

  // ---- per-lane LDS read offsets ----------------------------------------------------------------
  // K fragment (sub-tile u, k-step ks): row 32u + l32, logical piece 2ks + hi, i.e. byte offset
  //   l32 * ROWB + ((2ks + hi) ^ swizzle) * 16 + u * 32 * ROWB  =  (k_a ^ (ks << 5)) + u * 32 * ROWB,
  // because the swizzle is an exclusive-or on bits the row term leaves clear: one register holds
  // k_a and every fragment address is that register exclusive-or a constant.
  const int k_a = l32 * ROWB + ((hi ^ swz_k<D>(l32)) * 16);
  // V^T fragment (row tile m, sub-tile u, step t, half a2): 16-lane block b reads 4 key rows x
  // 16 head_dim columns; lane j of the block addresses row j / 4, 8-byte chunk j % 4:
  //   r = 8 a2 + 4 hi + j / 4 (+ 32u + 16t, which leave the swizzle unchanged), piece pc = 4m + 2 (lane / 16 % 2) + j % 4 / 2,
  //   offset r * ROWB + (pc ^ swizzle(r)) * 16 + 8 (j % 2)  =  (v_a ^ (m << 6) ^ (a2 << 5, D = 128 only)) + a2 * 8 * ROWB
  // for the same reason (checked for every lane, m and a2 on the host when this was written).
  const int vj = lane & 15, vdh = (lane >> 4) & 1;
  const int v_a = (4 * hi + (vj >> 2)) * ROWB + (((2 * vdh + ((vj & 3) >> 1)) ^ swz_v<D>(4 * hi + (vj >> 2))) * 16) + 8 * (vj & 1);
  constexpr int V_A2_XOR = D == 128 ? 32 : 0;

  // ---- state ---------------------------------------------------------------------------------------
  f32x16 o[MT];
#pragma unroll
  for (int m = 0; m < MT; ++m)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[m][i] = 0.f;
  float m_run = -INFINITY;
  float l_run = 0.f;   // per-lane partial row sum; lanes l and l^32 are added at the end
  if (resumable && k_lo > 0) {   // what the launch for the previous key range left
    const float* base = a.state + ((size_t)tile * a.Hkv + g) * (size_t)(COLS * (D + 2));
    const float* op = base + (size_t)col * D + 4 * hi;
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const f32x4 w = *reinterpret_cast<const f32x4*>(op + m * 32 + 8 * q4);
#pragma unroll
        for (int e = 0; e < 4; ++e) o[m][4 * q4 + e] = w[e];
      }
    m_run = base[COLS * D + col];
    l_run = hi == 0 ? base[COLS * D + COLS + col] : 0.f;
  }
  f32x16 s[2];         // S^T of the tile whose scores were computed last (two 32-key sub-tiles)
  bf16x8 pf[2][2];     // P^T fragments (sub-tile u, 16-key step t) of the tile whose softmax was done last
#pragma unroll
  for (int u = 0; u < 2; ++u)
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int e = 0; e < 8; ++e) pf[u][t][e] = (__bf16)0.0f;

  typedef __attribute__((ext_vector_type(8))) short s16x8;
  auto load_vfrag = [&](const unsigned char* vrow, int m) __attribute__((always_inline)) -> bf16x8 {
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(vrow + (v_a ^ (m << 6))));
    const s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) s16x4*)(vrow + ((v_a ^ (m << 6) ^ V_A2_XOR) + 8 * ROWB)));
    const s16x8 both = __builtin_shufflevector(lo, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
    return *reinterpret_cast<const bf16x8*>(&both);
  };

  // ---- M part: O^T += V^T P^T (previous tile), S^T = K Q^T (this tile) ----------------------------
  // One stream of NPV + NQK (fragment read, MFMA) steps.  A step needs one A fragment from LDS;
  // with one wave per SIMD in this part nothing else hides the LDS latency, so the reads run PD
  // fragments (PD * 32 MFMA cycles) ahead of their MFMAs through a ring of PD + 1 fragment
  // registers, across the PV -> QK boundary as well.  The first PD fragments are read before the
  // first MFMA can issue (a wave issues in order, one LDS instruction per ~15 cycles), so the
  // distance is no longer than the LDS latency asks for: 3 or 4 (7 costs 1.5 %, 2 costs 1 %).
  // The wave runs it at raised priority: its instruction stream is sparse and must not queue
  // behind the dense softmax stream of the other wave on the SIMD.
  // The first period has no previous tile and the last one no next tile; both still run the
  // whole stream (P^T = 0 in the first, S^T unused in the last, the stages hold loaded data).
  constexpr int NPV = 4 * MT, NQK = 2 * KS;
#ifndef CT_ATTN_PD
#define CT_ATTN_PD 4
#endif
  constexpr int PD = CT_ATTN_PD;
  auto load_frag = [&](int j, const unsigned char* vb, const unsigned char* kb) __attribute__((always_inline)) -> bf16x8 {
    if (j < NPV) return load_vfrag(vb + 16 * (j / MT) * ROWB, j % MT);
    const int ks = (j - NPV) >> 1, u = (j - NPV) & 1;
    return *reinterpret_cast<const bf16x8*>(kb + (k_a ^ (ks << 5)) + u * 32 * ROWB);
  };
  auto part_m = [&](const unsigned char* vb, const unsigned char* kb, auto&& dma) __attribute__((always_inline)) {
    __builtin_amdgcn_s_setprio(3);
    bf16x8 fr[PD + 1];
#pragma unroll
    for (int j = 0; j < PD; ++j) fr[j] = load_frag(j, vb, kb);
    dma();   // behind the first fragment reads: issued while the wave would wait for them anyway
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int i = 0; i < 16; ++i) s[u][i] = 0.f;
#pragma unroll
    for (int j = 0; j < NPV + NQK; ++j) {
      if (j + PD < NPV + NQK) fr[(j + PD) % (PD + 1)] = load_frag(j + PD, vb, kb);
      if (j < NPV) {
        const int gi = j / MT, m = j % MT;
        o[m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[j % (PD + 1)], pf[gi >> 1][gi & 1], o[m], 0, 0, 0);
      } else {
        const int ks = (j - NPV) >> 1, u = (j - NPV) & 1;
        s[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[j % (PD + 1)], qf[ks], s[u], 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);   // keep the read-ahead distance as written
    }
    __builtin_amdgcn_s_setprio(0);
  };

  // ---- V part: causal mask, online softmax, P^T fragments, rescale of O^T -------------------------
  auto part_v = [&](int k0) __attribute__((always_inline)) {
    if (k0 + BN - 1 > wmin) {   // only tiles that reach past the earliest query of this wave
      const int rel = pos - k0 - 4 * hi;   // key offsets (32u + 8(i/4) + i%4) <= rel are visible
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int i = 0; i < 16; ++i)
          if (32 * u + 8 * (i >> 2) + (i & 3) > rel) s[u][i] = -INFINITY;
    }
    float mx = s[0][0];
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s[u][i]);
    mx = max_with_lane_xor32(mx);
    // The reference of the exponents follows the running maximum lazily: it moves only when the
    // tile's maximum exceeds it by more than 2^8, so probabilities stay below 256 (bf16 keeps
    // their relative precision, the sums are fp32) and the rescale of O^T becomes rare.  A
    // rescale in one wave holds up the whole workgroup at the next barrier, and with the exact
    // maximum some wave of the eight has one in most periods.
    const float m_tile = mx * a.scale_log2;
    const bool changed = m_tile > m_run + 8.0f;
    const float m_new = changed ? m_tile : m_run;
    const float m_use = m_new == -INFINITY ? 0.f : m_new;
    const float alpha = changed ? __builtin_amdgcn_exp2f(m_run - m_use) : 1.0f;
    m_run = m_new;
    float rs0 = 0.f, rs1 = 0.f;
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int i = 0; i < 16; i += 2) {
        const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[u][i], a.scale_log2, -m_use));
        const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[u][i + 1], a.scale_log2, -m_use));
        s[u][i] = p0;
        s[u][i + 1] = p1;
        rs0 += p0;
        rs1 += p1;
      }
    l_run = l_run * alpha + (rs0 + rs1);
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        u32x4 w;
#pragma unroll
        for (int e = 0; e < 4; ++e) w[e] = pack_bf16(s[u][8 * t + 2 * e], s[u][8 * t + 2 * e + 1]);
        pf[u][t] = *reinterpret_cast<bf16x8*>(&w);
      }
    if (__any(changed)) {
#pragma unroll
      for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[m][i] *= alpha;
    }
  };

  // ---- the period loop -----------------------------------------------------------------------------
  // Loads past the last tile are still issued (row index clamped) so that the number of loads
  // outstanding at the wait, and with it the wait itself, is the same in every period.
  constexpr int LPP = 2 * INSTS;                                              // loads per wave and period
  constexpr int WAIT_OLDER = (LPP & 15) | ((LPP >> 4) << 14) | 0x0f70;        // s_waitcnt vmcnt(LPP)
  // Every ordinary global load so far (indices, Q fragments) is waited for here, once: the
  // compiler would otherwise guard their first use inside the loop with vmcnt waits that also
  // wait for the look-ahead tile loads.
  __builtin_amdgcn_s_waitcnt(0x0f70);
  issue_rows(a.k, k_lane_off, k_lo, k_lds_addr);                           // K(0)
  issue_rows(a.v, v_lane_off, k_lo, v_lds_addr + 2 * TILE_BYTES);          // stands in for V(-1): keeps the load count uniform
  issue_rows(a.k, k_lane_off, k_lo + BN, k_lds_addr + TILE_BYTES);         // K(1)
  issue_rows(a.v, v_lane_off, k_lo, v_lds_addr);                           // V(0)
  __builtin_amdgcn_s_waitcnt(WAIT_OLDER);                                  // K(0) has landed (and the stand-in)
  __syncthreads();
  auto end_of_period = [&]() __attribute__((always_inline)) {
    __builtin_amdgcn_s_waitcnt(WAIT_OLDER);     // this wave's loads of the previous period have landed
    __syncthreads();                            // everybody's have; everybody is done with K(i), V(i-1)
  };
  // Period i uses K(i) and V(i-1); its M parts fetch K(i+2) and V(i+1) into the stages of
  // K(i-1) and V(i-2), which nobody reads any more.  The two groups run separate loops with
  // the same number of barriers; nothing but the order of the two parts differs, and no barrier
  // is needed between them: both groups read the same tiles for the whole period.
  // The look-ahead loads of period i (K(i+2), V(i+1)) are issued by each wave at the start of its
  // M part, right behind the first fragment reads: the wave has to wait for those anyway, so the
  // queueing of the four waves' loads at the texture addresser costs it nothing there (measured:
  // anywhere later in the MFMA stream it costs 4.5 %, before the softmax part 1.5 %).
  auto refill = [&](int i, int st_im1, int st_ip1) __attribute__((always_inline)) {
    issue_rows(a.k, k_lane_off, k_lo + (i + 2) * BN, k_lds_addr + st_im1 * TILE_BYTES);
    issue_rows(a.v, v_lane_off, k_lo + (i + 1) * BN, v_lds_addr + st_ip1 * TILE_BYTES);
  };
  int st_i = 0, st_im1 = 2;                     // stage indices of tiles i and i - 1 (i mod 3)
  if (!group_b) {
    for (int i = 0; i <= n_kt; ++i) {
      const int st_ip1 = st_i == 2 ? 0 : st_i + 1;
      part_m(v_lds + st_im1 * TILE_BYTES, k_lds + st_i * TILE_BYTES, [&]() __attribute__((always_inline)) { refill(i, st_im1, st_ip1); });
      if (i < n_kt) part_v(k_lo + i * BN);
      end_of_period();
      st_im1 = st_i;
      st_i = st_ip1;
    }
  } else {
    for (int i = 0; i <= n_kt; ++i) {
      const int st_ip1 = st_i == 2 ? 0 : st_i + 1;
      if (i >= 1) part_v(k_lo + (i - 1) * BN);
      part_m(v_lds + st_im1 * TILE_BYTES, k_lds + st_i * TILE_BYTES, [&]() __attribute__((always_inline)) { refill(i, st_im1, st_ip1); });
      end_of_period();
      st_im1 = st_i;
      st_i = st_ip1;
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0f70);           // drain the look-ahead loads before the LDS is released

  // ---- epilogue -------------------------------------------------------------------------------
  const float l_tot = sum_with_lane_xor32(l_run);
  if (resumable ? k_hi == kmax : kmax <= a.split_keys) {   // the tile's key range ends here: final result
    if (valid) {
      const float inv = 1.0f / l_tot;
      uint16_t* op = a.out + ((size_t)tokv * a.Hq + hq) * D + 4 * hi;
#pragma unroll
      for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          u32x2 w;
          w[0] = pack_bf16(o[m][4 * q4 + 0] * inv, o[m][4 * q4 + 1] * inv);
          w[1] = pack_bf16(o[m][4 * q4 + 2] * inv, o[m][4 * q4 + 3] * inv);
          *reinterpret_cast<u32x2*>(op + m * 32 + 8 * q4) = w;
        }
      if (a.lse != nullptr && hi == 0)
        a.lse[(size_t)tokv * a.Hq + hq] = (m_run + __builtin_log2f(l_tot)) * 0.69314718055994531f;
    }
  } else {
    // partial results: [item][COLS columns][D] fp32, then m[COLS], l[COLS]
    const size_t item = ((size_t)tile * a.Hkv + g) * a.n_splits + split;
    float* base = (resumable ? a.state : a.partial) + item * (size_t)(COLS * (D + 2));
    float* op = base + (size_t)col * D + 4 * hi;
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        f32x4 w = {o[m][4 * q4 + 0], o[m][4 * q4 + 1], o[m][4 * q4 + 2], o[m][4 * q4 + 3]};
        *reinterpret_cast<f32x4*>(op + m * 32 + 8 * q4) = w;
      }
    if (hi == 0) {
      base[COLS * D + col] = m_run;
      base[COLS * D + COLS + col] = l_tot;
    }
  }
}

// Merge of the key-range splits: out = sum_i w_i O_i / sum_i w_i l_i, w_i = 2^(m_i - max m).
// One thread owns 4 head_dim elements of one (token, query head).
template <int D>
__global__ __launch_bounds__(256) void attn_merge_kernel(AttnArgs a) {
  constexpr int TPR = D / 4;                       // threads per (token, head) row
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t rowid = gid / TPR;
  const int d4 = (int)(gid % TPR) * 4;
  if (rowid >= (int64_t)a.n_sel * a.Hq) return;
  const int tok = (int)(rowid / a.Hq), h = (int)(rowid % a.Hq);
  const int g = h / a.G, hg = h % a.G;
  const int tile = tok / a.TM;
  const int col = hg * a.TM + (tok - tile * a.TM);
  const int last_tok = min(tile * a.TM + a.TM, a.n_sel) - 1;
  const int kmax = a.sel_idx[last_tok] + 1;
  const int ns = min(a.n_splits, (kmax + a.split_keys - 1) / a.split_keys);
  if (ns == 1) return;                             // written by the attention kernel itself
  const size_t item0 = ((size_t)tile * a.Hkv + g) * a.n_splits;
  const int C = a.cols;
  const size_t istride = (size_t)C * (D + 2);
  float mx = -INFINITY;
  for (int i = 0; i < ns; ++i) mx = fmaxf(mx, a.partial[(item0 + i) * istride + (size_t)C * D + col]);
  float L = 0.f;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int i = 0; i < ns; ++i) {
    const float* base = a.partial + (item0 + i) * istride;
    const float mi = base[(size_t)C * D + col];
    const float w = __builtin_amdgcn_exp2f(mi - mx);     // 0 for a split with nothing visible (m = -inf)
    L += w * base[(size_t)C * D + C + col];
    const f32x4 oi = *reinterpret_cast<const f32x4*>(base + (size_t)col * D + d4);
    if (w > 0.f) acc += w * oi;
  }
  const float inv = 1.0f / L;
  u32x2 w2;
  w2[0] = pack_bf16(acc[0] * inv, acc[1] * inv);
  w2[1] = pack_bf16(acc[2] * inv, acc[3] * inv);
  *reinterpret_cast<u32x2*>(a.out + ((size_t)tok * a.Hq + h) * D + d4) = w2;
  if (a.lse != nullptr && d4 == 0)
    a.lse[(size_t)tok * a.Hq + h] = (mx + __builtin_log2f(L)) * 0.69314718055994531f;
}

}  // namespace

ct_status launch_attention(const ct_layer_cfg* cfg, const void* q_sel, const void* k_buf, const void* v_buf,
                           int32_t n_ctx, const int32_t* sel_idx, int32_t n_sel, void* out, float* lse,
                           void* workspace, hipStream_t s, int32_t key_after, int32_t key_upto, float* state) {
  if (n_sel == 0) return CT_OK;
  const AttnPlan p = plan_attention(cfg, n_ctx, n_sel);
  AttnArgs a;
  a.q = static_cast<const uint16_t*>(q_sel);
  a.k = static_cast<const uint16_t*>(k_buf);
  a.v = static_cast<const uint16_t*>(v_buf);
  a.sel_idx = sel_idx;
  a.out = static_cast<uint16_t*>(out);
  a.lse = lse;
  a.partial = static_cast<float*>(workspace);
  a.n_sel = n_sel;
  a.n_ctx = n_ctx;
  a.Hq = cfg->n_q_heads;
  a.Hkv = cfg->n_kv_heads;
  a.G = cfg->n_q_heads / cfg->n_kv_heads;
  a.TM = p.tile_tokens;
  a.cols = 256;
  a.tm_shift = 0;
  while ((1 << a.tm_shift) < a.TM) ++a.tm_shift;
  a.n_tiles = p.n_tiles;
  a.n_splits = p.n_splits;
  a.split_keys = p.split_keys;
  a.key_after = key_after;
  a.key_upto = key_upto;
  a.state = state;
  const float scale = cfg->softmax_scale > 0.f ? cfg->softmax_scale : 1.0f / sqrtf((float)cfg->head_dim);
  a.scale_log2 = scale * 1.4426950408889634f;

  const int D = cfg->head_dim;
  dim3 grid((unsigned)((size_t)p.n_tiles * cfg->n_kv_heads * p.n_splits));
  hipError_t e;
  if (D == 128)
    launch_kernel(KC_ATTN, attn_kernel<128>, grid, dim3(512), 0, s, a);
  else
    launch_kernel(KC_ATTN, attn_kernel<64>, grid, dim3(512), 0, s, a);
  e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(e, "attention kernel launch");
  if (p.n_splits > 1) {
    const int64_t threads = (int64_t)n_sel * cfg->n_q_heads * (D / 4);
    dim3 mgrid((unsigned)((threads + 255) / 256)), block(256);
    if (D == 128)
      launch_kernel(KC_MERGE, attn_merge_kernel<128>, mgrid, block, 0, s, a);
    else
      launch_kernel(KC_MERGE, attn_merge_kernel<64>, mgrid, block, 0, s, a);
    e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "attention merge kernel launch");
  }
  return CT_OK;
}

// Host-side replay of the key rows one launch reads (same item and row functions as the kernel, same
// tile loads: the prologue's K(0), K(1), V(0) and stand-in, then K(i + 2) and V(i + 1) in period i).
ct_status attention_rows_read(const ct_layer_cfg* cfg, const int32_t* sel_idx_host, int32_t n_sel, int32_t n_ctx,
                              int32_t key_after, int32_t key_upto, bool resumable, int32_t* first_row,
                              int32_t* last_row) {
  const AttnPlan p = plan_attention(cfg, n_ctx, n_sel);
  int lo = 0x7fffffff, hi = -1;
  for (int tile = 0; tile < p.n_tiles; ++tile) {
    const int last_tok = (tile * p.tile_tokens + p.tile_tokens < n_sel ? tile * p.tile_tokens + p.tile_tokens : n_sel) - 1;
    const int kmax = sel_idx_host[last_tok] + 1;
    for (int split = 0; split < p.n_splits; ++split) {
      const ItemRange it = item_range(kmax, split, p.split_keys, resumable, key_after, key_upto);
      if (!it.active) continue;
      const int n_kt = (it.k_hi - it.k_lo + BN - 1) / BN;
      for (int t = 0; t <= n_kt + 2; ++t)          // tiles 0 .. n_kt + 2 of the item are loaded
        for (int r = 0; r < BN; r += BN - 1) {     // first and last row of a tile bound the others
          const int row = tile_load_row(it.k_lo + t * BN, r, it.k_hi);
          lo = row < lo ? row : lo;
          hi = row > hi ? row : hi;
        }
    }
  }
  *first_row = hi < 0 ? -1 : lo;
  *last_row = hi;
  return CT_OK;
}

}  // namespace ct
