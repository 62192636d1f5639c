// Causal attention for the selected query rows over the fused layer KV (Sec. 4.2: the
// check / fusion layers compute attention "only for the corresponding tokens"), GQA aware.
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
// Work decomposition.  A workgroup (4 waves) owns one KV head and a tile of 256 query
// columns = (256 / G) selected tokens x the G query heads of that KV head; every wave owns
// 64 columns and all keys.  K and V tiles of 64 keys are staged once per workgroup in LDS
// (double buffered); V is transposed on the way in with byte permutes.  The selected rows
// are sorted, so a tile needs keys [0, last position of the tile]; tiles past a wave's last
// query are skipped and only tiles that straddle a query position evaluate the causal mask.
// When (tile, head) pairs are too few to fill the chip, the key range is split and fp32
// partial (O, m, l) are merged by a second kernel.
// Workgroup ids map KV head = id mod n_kv_heads, so with 8 KV heads every XCD streams the
// keys of one head through its own L2; tiles are issued heaviest first.
#include <math.h>

#include "ct_internal.h"

namespace ct {

namespace {

constexpr int BN = 64;                 // keys per LDS tile
constexpr int VT_ROWB = BN * 2 + 16;   // bytes per head_dim row of V^T in LDS

struct AttnArgs {
  const uint16_t* q;
  const uint16_t* k;
  const uint16_t* v;
  const int32_t* sel_idx;
  uint16_t* out;
  float* lse;
  float* partial;     // workspace when n_splits > 1
  int32_t n_sel, n_ctx, Hq, Hkv, G, TM, tm_shift;
  int32_t n_tiles, n_splits, split_keys;
  float scale_log2;   // softmax scale * log2(e)
};

// value held by lane ^ 32
__device__ __forceinline__ float lane_xor32(float x) { return __shfl_xor(x, 32); }

template <int D>
__global__ __launch_bounds__(256) void attn_kernel(AttnArgs a) {
  constexpr int K_ROWB = D * 2 + 16;
  constexpr int K_BYTES = BN * K_ROWB;
  constexpr int VT_BYTES = D * VT_ROWB;
  constexpr int STAGE = K_BYTES + VT_BYTES;
  constexpr int KS = D / 16;        // MFMA k-steps over head_dim
  constexpr int MT = D / 32;        // O^T row tiles
  constexpr int PCS = D / 8;        // 16-byte pieces per key row
  constexpr int KEYS_PER_PASS = 256 / PCS;       // keys covered by one piece per thread
  constexpr int K_PIECES = BN / KEYS_PER_PASS;   // pieces per thread for the K tile
  // V: a thread owns a block of 4 consecutive keys x 8 head_dim elements; the tile has
  // (BN / 4) * PCS such blocks: 256 for D = 128, 128 for D = 64 (then half the threads idle here)
  constexpr int V_UNITS = 1;
  static_assert((BN / 4) * PCS <= 256, "V tile has more 4x8 blocks than threads");

  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, hi = lane >> 5;

  // ---- work item ---------------------------------------------------------------------------
  const int g = blockIdx.x % a.Hkv;
  const int rest = blockIdx.x / a.Hkv;
  const int split = rest % a.n_splits;
  const int tile = a.n_tiles - 1 - rest / a.n_splits;   // heaviest (latest) tiles first
  const int tok0 = tile * a.TM;
  const int last_tok = min(tok0 + a.TM, a.n_sel) - 1;
  const int kmax = a.sel_idx[last_tok] + 1;              // keys this tile can see
  const int k_lo = split * a.split_keys;
  if (k_lo >= kmax) return;                              // empty split (uniform for the workgroup)
  const int k_hi = min(k_lo + a.split_keys, kmax);
  const int n_kt = (k_hi - k_lo + BN - 1) / BN;

  // ---- this lane's two query columns ---------------------------------------------------------
  int pos[2], tokv[2], hq[2];
  bool valid[2];
#pragma unroll
  for (int n = 0; n < 2; ++n) {
    const int col = wave * 64 + n * 32 + l32;
    const int tl = col & (a.TM - 1);
    const int t = tok0 + tl;
    valid[n] = t < a.n_sel;
    tokv[n] = valid[n] ? t : a.n_sel - 1;
    hq[n] = g * a.G + (col >> a.tm_shift);
    pos[n] = a.sel_idx[tokv[n]];
  }
  int wmax = max(pos[0], pos[1]), wmin = min(pos[0], pos[1]);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    wmax = max(wmax, __shfl_xor(wmax, off));
    wmin = min(wmin, __shfl_xor(wmin, off));
  }

  // Q^T fragments: B operand, lane = column, 8 consecutive head_dim elements per k-step
  bf16x8 qf[2][KS];
#pragma unroll
  for (int n = 0; n < 2; ++n) {
    const uint16_t* qp = a.q + ((size_t)tokv[n] * a.Hq + hq[n]) * D + hi * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[n][ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16);
  }

  // ---- staging maps --------------------------------------------------------------------------
  const int pc_col = tid % PCS;          // 16-byte piece inside a key row
  const int pc_key = tid / PCS;          // key inside a pass
  const size_t kv_row = (size_t)a.Hkv * D;
  const uint16_t* kbase = a.k + (size_t)g * D + pc_col * 8;
  const uint16_t* vbase = a.v + (size_t)g * D + pc_col * 8;
  const bool v_active = pc_key < BN / 4;   // pc_key doubles as the 4-key group of the V block
  u32x4 kr[K_PIECES];
  u32x4 vr[V_UNITS][4];

  auto load_tile = [&](int k0) {
#pragma unroll
    for (int i = 0; i < K_PIECES; ++i) {
      const int key = min(k0 + i * KEYS_PER_PASS + pc_key, a.n_ctx - 1);
      kr[i] = *reinterpret_cast<const u32x4*>(kbase + key * kv_row);
    }
    if (v_active) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int key = min(k0 + pc_key * 4 + i, a.n_ctx - 1);
        vr[0][i] = *reinterpret_cast<const u32x4*>(vbase + key * kv_row);
      }
    }
  };
  auto store_tile = [&](int buf) {
    unsigned char* kb = smem + buf * STAGE;
    unsigned char* vb = kb + K_BYTES;
#pragma unroll
    for (int i = 0; i < K_PIECES; ++i)
      *reinterpret_cast<u32x4*>(kb + (i * KEYS_PER_PASS + pc_key) * K_ROWB + pc_col * 16) = kr[i];
    if (v_active) {
      constexpr int u = 0;
      const int kg = pc_key;                              // group of 4 keys inside the tile, 0..15
      const int sub = kg >> 3, kgl = kg & 7;
      const int unit = sub * 4 + (kgl >> 2) * 2 + (kgl & 1);   // 16-byte unit (sub-tile, t, half)
      const int inner = ((kgl >> 1) & 1) * 8;             // a = 0 / 1 inside the unit
      const int sw = pc_col & 7;                          // (d >> 3) & 7 for all 8 rows of this thread
      unsigned char* dst = vb + (pc_col * 8) * VT_ROWB + ((unit ^ sw) * 16) + inner;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        u32x2 lo, hi2;
        lo[0] = __builtin_amdgcn_perm(vr[u][1][w], vr[u][0][w], 0x05040100u);
        lo[1] = __builtin_amdgcn_perm(vr[u][3][w], vr[u][2][w], 0x05040100u);
        hi2[0] = __builtin_amdgcn_perm(vr[u][1][w], vr[u][0][w], 0x07060302u);
        hi2[1] = __builtin_amdgcn_perm(vr[u][3][w], vr[u][2][w], 0x07060302u);
        *reinterpret_cast<u32x2*>(dst + (2 * w) * VT_ROWB) = lo;
        *reinterpret_cast<u32x2*>(dst + (2 * w + 1) * VT_ROWB) = hi2;
      }
    }
  };

  // ---- accumulators ---------------------------------------------------------------------------
  f32x16 o[MT][2];
#pragma unroll
  for (int m = 0; m < MT; ++m)
#pragma unroll
    for (int n = 0; n < 2; ++n)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[m][n][i] = 0.f;
  float m_run[2] = {-INFINITY, -INFINITY};
  float l_run[2] = {0.f, 0.f};   // per-lane partial row sums; lanes l and l^32 are added at the end

  const int k_frag = l32 * K_ROWB + hi * 16;
  const int v_sw = l32 >> 3;            // (d >> 3) & 3 of this lane's row inside a 32-row tile

  load_tile(k_lo);
  store_tile(0);
  __syncthreads();

  for (int it = 0; it < n_kt; ++it) {
    const int k0 = k_lo + it * BN;
    const int buf = it & 1;
    const bool more = it + 1 < n_kt;
    if (more) load_tile(k0 + BN);

    if (k0 <= wmax) {
      const unsigned char* kb = smem + buf * STAGE;
      const unsigned char* vb = kb + K_BYTES;

      // ---- S^T = K Q^T for two 32-key sub-tiles x two 32-column tiles ------------------------
      f32x16 s[2][2];
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int n = 0; n < 2; ++n)
#pragma unroll
          for (int i = 0; i < 16; ++i) s[u][n][i] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        bf16x8 kf[2];
#pragma unroll
        for (int u = 0; u < 2; ++u)
          kf[u] = *reinterpret_cast<const bf16x8*>(kb + k_frag + u * 32 * K_ROWB + ks * 32);
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
          for (int n = 0; n < 2; ++n)
            s[u][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[u], qf[n][ks], s[u][n], 0, 0, 0);
      }

      // ---- causal mask (only tiles that reach past the earliest query of this wave) --------
      if (k0 + BN - 1 > wmin) {
#pragma unroll
        for (int n = 0; n < 2; ++n) {
          const int rel = pos[n] - k0 - 4 * hi;   // key offsets (32u + 8(i/4) + i%4) <= rel are visible
#pragma unroll
          for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int i = 0; i < 16; ++i)
              if (32 * u + 8 * (i >> 2) + (i & 3) > rel) s[u][n][i] = -INFINITY;
        }
      }

      // ---- online softmax ----------------------------------------------------------------------
      float alpha[2];
      bool changed = false;
#pragma unroll
      for (int n = 0; n < 2; ++n) {
        float mx = s[0][n][0];
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
          for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s[u][n][i]);
        mx = fmaxf(mx, lane_xor32(mx));
        const float m_new = fmaxf(m_run[n], mx * a.scale_log2);
        const float m_use = m_new == -INFINITY ? 0.f : m_new;
        alpha[n] = __builtin_amdgcn_exp2f(m_run[n] - m_use);
        changed |= m_new > m_run[n];
        m_run[n] = m_new;
        float rs = 0.f;
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[u][n][i], a.scale_log2, -m_use));
            s[u][n][i] = p;
            rs += p;
          }
        l_run[n] = l_run[n] * alpha[n] + rs;
      }
      if (__any(changed)) {
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
          for (int n = 0; n < 2; ++n)
#pragma unroll
            for (int i = 0; i < 16; ++i) o[m][n][i] *= alpha[n];
      }

      // ---- O^T += V^T P^T ------------------------------------------------------------------------
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          bf16x8 pf[2];
#pragma unroll
          for (int n = 0; n < 2; ++n) {
            u32x4 w;
#pragma unroll
            for (int e = 0; e < 4; ++e) w[e] = pack_bf16(s[u][n][8 * t + 2 * e], s[u][n][8 * t + 2 * e + 1]);
            pf[n] = *reinterpret_cast<bf16x8*>(&w);
          }
          const int unit = u * 4 + t * 2 + hi;
#pragma unroll
          for (int m = 0; m < MT; ++m) {
            const int sw = v_sw + 4 * (m & 1);
            const bf16x8 vf =
                *reinterpret_cast<const bf16x8*>(vb + (m * 32 + l32) * VT_ROWB + ((unit ^ sw) * 16));
#pragma unroll
            for (int n = 0; n < 2; ++n)
              o[m][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[n], o[m][n], 0, 0, 0);
          }
        }
    }

    if (more) store_tile(buf ^ 1);
    __syncthreads();
  }

  // ---- epilogue -------------------------------------------------------------------------------
  float l_tot[2];
#pragma unroll
  for (int n = 0; n < 2; ++n) l_tot[n] = l_run[n] + lane_xor32(l_run[n]);

  if (a.n_splits == 1) {
#pragma unroll
    for (int n = 0; n < 2; ++n) {
      if (!valid[n]) continue;
      const float inv = 1.0f / l_tot[n];
      uint16_t* op = a.out + ((size_t)tokv[n] * a.Hq + hq[n]) * D + 4 * hi;
#pragma unroll
      for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          u32x2 w;
          w[0] = pack_bf16(o[m][n][4 * q4 + 0] * inv, o[m][n][4 * q4 + 1] * inv);
          w[1] = pack_bf16(o[m][n][4 * q4 + 2] * inv, o[m][n][4 * q4 + 3] * inv);
          *reinterpret_cast<u32x2*>(op + m * 32 + 8 * q4) = w;
        }
      if (a.lse != nullptr && hi == 0)
        a.lse[(size_t)tokv[n] * a.Hq + hq[n]] = (m_run[n] + __builtin_log2f(l_tot[n])) * 0.69314718055994531f;
    }
  } else {
    // partial results: [item][256 columns][D] fp32, then m[256], l[256]
    const size_t item = ((size_t)tile * a.Hkv + g) * a.n_splits + split;
    float* base = a.partial + item * (size_t)(256 * (D + 2));
#pragma unroll
    for (int n = 0; n < 2; ++n) {
      const int col = wave * 64 + n * 32 + l32;
      float* op = base + (size_t)col * D + 4 * hi;
#pragma unroll
      for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          f32x4 w = {o[m][n][4 * q4 + 0], o[m][n][4 * q4 + 1], o[m][n][4 * q4 + 2], o[m][n][4 * q4 + 3]};
          *reinterpret_cast<f32x4*>(op + m * 32 + 8 * q4) = w;
        }
      if (hi == 0) {
        base[256 * D + col] = m_run[n];
        base[256 * D + 256 + col] = l_tot[n];
      }
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
  const size_t item0 = ((size_t)tile * a.Hkv + g) * a.n_splits;
  const size_t istride = (size_t)(256 * (D + 2));
  float mx = -INFINITY;
  for (int i = 0; i < ns; ++i) mx = fmaxf(mx, a.partial[(item0 + i) * istride + 256 * D + col]);
  float L = 0.f;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int i = 0; i < ns; ++i) {
    const float* base = a.partial + (item0 + i) * istride;
    const float mi = base[256 * D + col];
    const float w = __builtin_amdgcn_exp2f(mi - mx);     // 0 for a split with nothing visible (m = -inf)
    L += w * base[256 * D + 256 + col];
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
                           void* workspace, hipStream_t s) {
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
  a.tm_shift = 0;
  while ((1 << a.tm_shift) < a.TM) ++a.tm_shift;
  a.n_tiles = p.n_tiles;
  a.n_splits = p.n_splits;
  a.split_keys = p.split_keys;
  const float scale = cfg->softmax_scale > 0.f ? cfg->softmax_scale : 1.0f / sqrtf((float)cfg->head_dim);
  a.scale_log2 = scale * 1.4426950408889634f;

  const int D = cfg->head_dim;
  const size_t shmem = 2 * (size_t)(BN * (D * 2 + 16) + D * VT_ROWB);
  dim3 grid((unsigned)((size_t)p.n_tiles * cfg->n_kv_heads * p.n_splits)), block(256);
  hipError_t e;
  const void* fn = D == 128 ? reinterpret_cast<const void*>(attn_kernel<128>) : reinterpret_cast<const void*>(attn_kernel<64>);
  e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
  if (e != hipSuccess) return hip_fail(e, "hipFuncSetAttribute (attention)");
  int slot = prof_begin(KC_ATTN, s);
  if (D == 128)
    hipLaunchKernelGGL(attn_kernel<128>, grid, block, shmem, s, a);
  else
    hipLaunchKernelGGL(attn_kernel<64>, grid, block, shmem, s, a);
  prof_end(KC_ATTN, slot, s);
  e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(e, "attention kernel launch");
  if (p.n_splits > 1) {
    const int64_t threads = (int64_t)n_sel * cfg->n_q_heads * (D / 4);
    dim3 mgrid((unsigned)((threads + 255) / 256));
    slot = prof_begin(KC_MERGE, s);
    if (D == 128)
      hipLaunchKernelGGL(attn_merge_kernel<128>, mgrid, block, 0, s, a);
    else
      hipLaunchKernelGGL(attn_merge_kernel<64>, mgrid, block, 0, s, a);
    prof_end(KC_MERGE, slot, s);
    e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "attention merge kernel launch");
  }
  return CT_OK;
}

}  // namespace ct
