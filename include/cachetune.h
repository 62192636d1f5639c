/*
 * cachetune.h - C ABI of the MI355X (gfx950) selective-recompute partial-prefill library.
 *
 * The library implements one layer of CacheTune's online sparse-reuse pipeline (paper
 * Sec. 4.2, "KV Cache Offloading and Sparse Reuse"): cached KV chunks are reused at new
 * positions, only the tokens of a recompute index set are projected again, the two parts
 * are fused in one layer buffer and the selected tokens' queries attend causally over it.
 *
 * Conventions shared by every entry point
 *   - All tensors are dense, row-major bfloat16 unless stated otherwise; index and position
 *     vectors are int32.  "device" pointers are HIP device memory of the current device,
 *     "host" pointers are ordinary process memory, "pinned host" is hipHostMalloc memory.
 *   - KV layout is token-major [tokens, n_kv_heads, head_dim] (the paper's N x H x D).
 *   - The caller owns every buffer and both streams.  The library allocates no device or host
 *     buffers and keeps no state besides a thread-local error string, the opt-in profiling events
 *     and a small per-thread pool of HIP events (created on first use, reused by every later call
 *     of that thread) that order the two streams in the layer and stack calls.  `stream`
 *     arguments are hipStream_t values passed as void* (NULL = the default stream).
 *   - Calls only enqueue work: no entry point synchronises the device or the host with it.
 *     Results are valid once the stream has passed the call's last kernel.
 *   - Every host-checkable condition (NULL pointers, shapes, chunk tiling, workspace size,
 *     the ratio) is checked before the first HIP call and reported as a negative status;
 *     nothing is thrown and nothing aborts.  ct_last_error() describes the last failure of
 *     the calling thread.
 *   - Supported shapes: head_dim in {64, 128}; n_q_heads a multiple of n_kv_heads with
 *     group size n_q_heads / n_kv_heads in {1, 2, 4, 8, 16}; hidden a multiple of 64; K/V
 *     buffers of fewer than 2^24 rows and at most 4 GiB each; weight matrices and the rows read
 *     of activation matrices within 4 GiB of their base (CT_ERR_UNSUPPORTED otherwise).
 */
#ifndef CACHETUNE_H
#define CACHETUNE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  CT_OK = 0,
  CT_ERR_NULL = -1,        /* a required pointer is NULL */
  CT_ERR_SHAPE = -2,       /* a size is negative, zero where it may not be, or inconsistent */
  CT_ERR_INDEX = -3,       /* host index set not strictly ascending / out of range */
  CT_ERR_RATIO = -4,       /* n_sel does not equal floor(recompute_ratio * n_ctx) */
  CT_ERR_WORKSPACE = -5,   /* workspace missing or smaller than ct_workspace_bytes() */
  CT_ERR_HIP = -6,         /* a HIP runtime call failed; see ct_last_error() */
  CT_ERR_UNSUPPORTED = -7  /* a shape outside the supported set listed above */
} ct_status;

/* One attention layer's shape.  RoPE: omega_j = rope_theta^(-2j/head_dim); rope_style 0
 * couples elements (j, j + head_dim/2), rope_style 1 couples (2j, 2j + 1).
 * softmax_scale 0 means 1/sqrt(head_dim). */
typedef struct {
  int32_t hidden;
  int32_t n_q_heads;
  int32_t n_kv_heads;
  int32_t head_dim;
  double rope_theta;
  int32_t rope_style;
  float softmax_scale;
} ct_layer_cfg;

/* One reusable KV chunk (the paper's unit of storage and transfer, Sec. 3 and 4.2).
 * k, v: bf16 [n_tokens, n_kv_heads, head_dim], device memory (location 0) or pinned host
 * memory (location 1).  Location 2 is a pool that dropped the recompute set when the chunk was
 * offloaded (Sec. 4.2, index-aware offloading): pinned host memory holding, in order, only the
 * chunk's rows that are NOT in sel_idx - n_tokens minus the number of selected rows of the
 * chunk; n_tokens still counts all tokens of the chunk (k and v must be non-NULL even when no row
 * of the chunk is kept: nothing is read then).  In the new context token t of the chunk sits at position
 * new_pos_start + t.  raw_keys = 0: the keys were cached after RoPE at positions
 * old_pos_start + t and are rotated by new_pos_start - old_pos_start.  raw_keys = 1: the
 * keys were cached before RoPE (the paper's own scheme, Eq. 8) and token t is rotated by
 * new_pos_start + t; old_pos_start is ignored. */
typedef struct {
  const void* k;
  const void* v;
  int32_t n_tokens;
  int32_t old_pos_start;
  int32_t new_pos_start;
  int32_t location;
  int32_t raw_keys;
  int32_t reserved;
} ct_chunk;

/* Step "selective recompute" (Eq. 1 and Sec. 4.2 last paragraph: standard RoPE at the true
 * positions).  For s in [0, n_sel): x = hidden[hidden_rows ? hidden_rows[s] : s, :],
 * [q|k|v] = x * wqkv^T (+ bias), RoPE on every q and k head at position sel_pos[s],
 * results rounded to bf16 (nearest even) from fp32 accumulators.
 *   hidden      device bf16 [*, hidden]; rows read must lie within 4 GiB of the base
 *   hidden_rows device int32 [n_sel] or NULL (hidden is already compact)
 *   sel_pos     device int32 [n_sel]
 *   wqkv        device bf16 [(n_q_heads + 2 n_kv_heads) * head_dim, hidden]: one row per
 *               output feature (q heads, then k heads, then v heads)
 *   bias        device bf16 [(n_q_heads + 2 n_kv_heads) * head_dim] or NULL
 *   q_out       device bf16 [n_sel, n_q_heads, head_dim]
 *   k_out,v_out device bf16 [n_sel, n_kv_heads, head_dim]
 * hidden, wqkv and the three outputs must be 16-byte aligned.  n_sel = 0 is legal and does nothing. */
ct_status ct_qkv_selected(const ct_layer_cfg* cfg, const void* hidden, const int32_t* hidden_rows,
                          const int32_t* sel_pos, int32_t n_sel, const void* wqkv, const void* bias,
                          void* q_out, void* k_out, void* v_out, void* stream);

/* Step "deferred RoPE recovery" (Eq. 8) in delta form: key row t is rotated by the angle
 * (new_pos[t] - old_pos[t]) * omega_j in fp32 (angle reduced in fp64) and rounded to bf16.
 *   k_src, k_dst device bf16 [n_tokens, n_kv_heads, head_dim]; k_dst may equal k_src
 *                (in place) but may not otherwise overlap it
 *   old_pos      device int32 [n_tokens] or NULL (= all zero: a raw pre-RoPE cache)
 *   new_pos      device int32 [n_tokens] */
ct_status ct_rerope_keys(const ct_layer_cfg* cfg, const void* k_src, void* k_dst, const int32_t* old_pos,
                         const int32_t* new_pos, int32_t n_tokens, void* stream);

/* ct_rerope_keys for the reused rows alone (Eq. 8 applies to reused keys; Sec. 4.2, index-aware
 * I/O: rows of the recompute set are not moved): rows listed in skip_rows are neither read nor
 * written - the scatter overwrites them.
 *   skip_rows    device int32 [n_skip], strictly ascending, in [0, n_tokens); may be NULL when
 *                n_skip = 0 (the call is then ct_rerope_keys) */
ct_status ct_rerope_keys_skip(const ct_layer_cfg* cfg, const void* k_src, void* k_dst, const int32_t* old_pos,
                              const int32_t* new_pos, int32_t n_tokens, const int32_t* skip_rows, int32_t n_skip,
                              void* stream);

/* Same rotation for one chunk whose positions are contiguous (Eq. 8): token t moves from
 * old_pos_start + t to new_pos_start + t, so every token shares one delta; with
 * raw_keys != 0 token t is rotated by new_pos_start + t instead.  If v_src and v_dst are
 * both non-NULL and differ, the chunk's values are copied alongside (values carry no
 * position: Sec. 4.2 corrects Keys only). */
ct_status ct_rerope_chunk(const ct_layer_cfg* cfg, const void* k_src, void* k_dst, const void* v_src,
                          void* v_dst, int32_t n_tokens, int32_t old_pos_start, int32_t new_pos_start,
                          int32_t raw_keys, void* stream);

/* Step "scatter fusion" (Sec. 4.2): k_buf[sel_idx[s]] = k_sel[s], v_buf[sel_idx[s]] = v_sel[s],
 * bit for bit; no other row is touched.
 *   k_buf, v_buf device bf16 [n_ctx, n_kv_heads, head_dim] (in/out)
 *   k_sel, v_sel device bf16 [n_sel, n_kv_heads, head_dim]
 *   sel_idx      device int32 [n_sel], strictly ascending, in [0, n_ctx) (not checked on
 *                the device; use ct_validate_indices on a host copy) */
ct_status ct_scatter_kv(const ct_layer_cfg* cfg, void* k_buf, void* v_buf, int32_t n_ctx, const void* k_sel,
                        const void* v_sel, const int32_t* sel_idx, int32_t n_sel, void* stream);

/* Step "attention only for the selected tokens" (Sec. 4.2, check/fusion layers): for every
 * selected token s and query head h,
 *   out[s,h,:] = sum_{j <= sel_idx[s]} softmax_j(q[s,h,:] . k_buf[j,g,:] * scale) v_buf[j,g,:],
 * g = h / (n_q_heads / n_kv_heads).  bf16 operands, fp32 scores / softmax / accumulation.
 *   q_sel  device bf16 [n_sel, n_q_heads, head_dim]
 *   out    device bf16 [n_sel, n_q_heads, head_dim]
 *   lse    device fp32 [n_sel, n_q_heads] natural-log sum-exp of the scaled scores, or NULL
 *   workspace device scratch of at least ct_workspace_bytes(cfg, n_ctx, n_sel) bytes,
 *          256-byte aligned; contents are undefined afterwards. */
ct_status ct_selected_attention(const ct_layer_cfg* cfg, const void* q_sel, const void* k_buf, const void* v_buf,
                                int32_t n_ctx, const int32_t* sel_idx, int32_t n_sel, void* out, float* lse,
                                void* workspace, size_t workspace_bytes, void* stream);

/* ct_selected_attention for callers that cannot allocate device memory or bring a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * results and kernels; the scratch lives in a device array inside the library (one copy per GPU,
 * ct_static_scratch_bytes() = 64 MiB, held until the process ends) instead of a workspace.  The
 * call allocates nothing.  A problem whose scratch exceeds the array is rejected with
 * CT_ERR_WORKSPACE before anything is launched.  Every call on a GPU uses that GPU's one array:
 * calls that overlap in time on the same GPU (two streams, two threads) race; calls ordered on
 * one stream do not.  The array keeps the last call's contents; the call clears what it needs
 * cleared itself. */
ct_status ct_selected_attention_static(const ct_layer_cfg* cfg, const void* q_sel, const void* k_buf,
                                       const void* v_buf, int32_t n_ctx, const int32_t* sel_idx, int32_t n_sel,
                                       void* out, float* lse, void* stream);
size_t ct_static_scratch_bytes(void);

/* One fusion-layer step of the online pipeline (Sec. 4.2; its cost model is Eq. 9):
 *   compute stream: device chunks are read from chunk.k / chunk.v, rotated and written to
 *                   the buffers (all but the rows listed in sel_idx, which are recomputed); a
 *                   device chunk whose k already points at its rows of k_buf is rotated in
 *                   place and its v is left alone
 *   compute stream: selective recompute of q/k/v for the selected rows; the projection writes
 *                   the new keys and values straight to rows sel_idx[s] of k_buf / v_buf (the
 *                   scatter fusion of Sec. 4.2 done by the GEMM's epilogue), except when host
 *                   chunks arrive by plain copies (below): then they wait in the workspace and
 *                   are scattered once the copies have landed
 *   copy stream   : chunks in pinned host memory (the "Transfer stream"): a kernel reads
 *                   them over the host link, rotates the keys on the way (Eq. 8 overlapped with
 *                   the transfer) and writes K and V to their rows of k_buf / v_buf; rows
 *                   listed in sel_idx are not transferred.  The chunks go in equal groups
 *                   (one launch and one event each; two to eight groups, as many as leave
 *                   every attention launch about 200 workgroups, or - with the attention
 *                   state - as balance the work left after the last group against the cost
 *                   of a further launch).  Host memory the device cannot
 *                   address is copied instead (one event per chunk) and rotated in place on
 *                   the compute stream
 *   compute stream: per group of host chunks, wait for the group and compute
 *                   the attention of the selected rows whose visible keys it completes - or,
 *                   with the extra workspace of ct_attention_state_bytes(), of all unfinished
 *                   rows over that group's keys (the
 *                   chunk-wise overlap of transfer and recomputation of Sec. 4.2); with no
 *                   host chunks, or a context so short that the key range is split over
 *                   workgroups, one wait and one attention launch.
 * Chunks must tile buffer rows [0, n_ctx) in order (n_ctx = sum of n_tokens) with ascending
 * new positions, so that "key position <= query position" is "key row <= query row".
 *   hidden / hidden_rows / wqkv / bias as in ct_qkv_selected (hidden_rows, when given, are rows
 *   of a [n_ctx, hidden] matrix); the RoPE position of selected token s is the new position of
 *   buffer row sel_idx[s].
 *   sel_idx      device int32 [n_sel] strictly ascending
 *   recompute_ratio  r in [0,1]: n_sel must equal floor(r * n_ctx) (1 at least when r > 0);
 *                a negative value disables the check
 *   attn_out     device bf16 [n_sel, n_q_heads, head_dim]
 *   workspace    at least ct_workspace_bytes(cfg, n_ctx, n_sel) bytes
 *   copy_stream  used only when a chunk has location 1 or 2; must differ from compute_stream
 *                for the copy to overlap.
 * On return (stream ordered) k_buf / v_buf hold the fused layer KV.  n_sel = 0 is the Full
 * KV Reuse case: the buffers are assembled and no attention output is produced. */
ct_status ct_partial_prefill_layer(const ct_layer_cfg* cfg, const ct_chunk* chunks, int32_t n_chunks,
                                   const void* hidden, const int32_t* hidden_rows, const int32_t* sel_idx,
                                   int32_t n_sel, double recompute_ratio, const void* wqkv, const void* bias,
                                   void* k_buf, void* v_buf, void* attn_out, void* workspace,
                                   size_t workspace_bytes, void* compute_stream, void* copy_stream);

/* Scratch bytes ct_selected_attention / ct_partial_prefill_layer need for this problem
 * size (0 on invalid arguments). */
size_t ct_workspace_bytes(const ct_layer_cfg* cfg, int32_t n_ctx, int32_t n_sel);

/* Optional extra workspace of ct_partial_prefill_layer for layers whose chunks come from host
 * memory (Sec. 4.2, overlap of transfer and recomputation): with a workspace of at least
 * ct_workspace_bytes() + ct_attention_state_bytes() bytes the attention launch that follows a
 * group of chunks takes every unfinished tile of selected rows through that group's keys and
 * keeps the fp32 running (O, max, sum) of the tiles that still wait for later keys there, so
 * only the last group's keys are left when the transfer ends.  With less the launches go tile
 * by tile: a tile is computed once all its keys have arrived.  Host function, no GPU call;
 * 0 for an invalid configuration or n_sel = 0. */
size_t ct_attention_state_bytes(const ct_layer_cfg* cfg, int32_t n_ctx, int32_t n_sel);

/* Which rows of k_buf / v_buf one attention launch of a host-pool layer reads (Sec. 4.2: the
 * attention follows the chunk groups while later groups are still on the host link, so a launch over
 * the keys [key_after, key_upto) must not touch a row from key_upto on).  Replays, on the host, the
 * tile loads of the launch that ct_partial_prefill_layer issues for that key range - with_state != 0:
 * the launch with the attention state, every unfinished tile through the range; 0: the tile-by-tile
 * launch, tiles whose last visible key lies in the range - with the index arithmetic the kernel uses.
 * sel_idx_host: host memory, n_sel strictly ascending rows.  first_row / last_row receive the lowest
 * and highest row read (-1 and -1 when the launch has no work).  Host function, no GPU call.
 * Errors: CT_ERR_NULL, CT_ERR_SHAPE (sizes, key range), CT_ERR_INDEX (indices). */
ct_status ct_attention_rows_read(const ct_layer_cfg* cfg, const int32_t* sel_idx_host, int32_t n_sel, int32_t n_ctx,
                                 int32_t key_after, int32_t key_upto, int32_t with_state, int32_t* first_row,
                                 int32_t* last_row);

/* ---- The rest of a transformer layer on the selected rows, and the multi-layer partial prefill.
 * After the check layer every layer of the model runs on the selected tokens only (Sec. 4.2,
 * fusion layers); the non-selected tokens contribute their cached K/V and nothing else. ---- */

/* out[t,:] = x[t,:] / sqrt(mean(x[t,:]^2) + eps) * weight, fp32 arithmetic, bf16 in and out.
 *   x, out device bf16 [n_tokens, width] (out may equal x); weight device bf16 [width];
 *   width a multiple of 8. */
ct_status ct_rmsnorm(const void* x, const void* weight, float eps, int32_t n_tokens, int32_t width, void* out,
                     void* stream);

/* out[t,:] = x[t,:] * w^T (+ residual[t,:]), bf16 MFMA, fp32 accumulation, bf16 result.
 *   x device bf16 [n_tokens, k_len]; w device bf16 [n_out, k_len] (one row per output feature);
 *   residual device bf16 [n_tokens, n_out] or NULL; out device bf16 [n_tokens, n_out], may equal
 *   residual (each element is read before it is written), may not overlap x.
 *   k_len and n_out multiples of 64; all four pointers 16-byte aligned. */
ct_status ct_linear(const void* x, int32_t n_tokens, int32_t k_len, const void* w, int32_t n_out, const void* residual,
                    void* out, void* stream);

/* ct_linear with scratch memory.  When the 256 x 256 output tiles do not fill the last round over
 * the compute units (say 320 tiles on 256 units), the tiles of that round are each computed by
 * several workgroups that split the reduction, as fp32 partial tiles in `workspace`, and a second
 * kernel adds the parts and the residual before the one rounding to bf16.  Same result layout
 * and rounding as ct_linear; sums are formed in a different order.
 *   workspace  device memory, 16-byte aligned, ct_linear_workspace_bytes() bytes (less, or NULL,
 *              is legal: the call then behaves like ct_linear). */
ct_status ct_linear_ws(const void* x, int32_t n_tokens, int32_t k_len, const void* w, int32_t n_out,
                       const void* residual, void* out, void* workspace, size_t workspace_bytes, void* stream);
size_t ct_linear_workspace_bytes(int32_t n_tokens, int32_t k_len, int32_t n_out);

/* ct_linear_ws planned for n_compute_units of the chip's 256 compute units instead of all of
 * them, for a launch that runs beside kernels which keep compute units to themselves (the stack
 * call plans the GEMMs that run beside the transfer of a later layer's chunks this way: Sec. 4.2,
 * transfer overlapped with recomputation).  Same result as ct_linear_ws up to the order of the
 * fp32 sums.  n_compute_units in [1, 256], CT_ERR_SHAPE otherwise. */
ct_status ct_linear_ws_cus(const void* x, int32_t n_tokens, int32_t k_len, const void* w, int32_t n_out,
                           const void* residual, void* out, void* workspace, size_t workspace_bytes,
                           int32_t n_compute_units, void* stream);

/* out[t,:] = silu(x[t,:] * w_gate^T) * (x[t,:] * w_up^T) (SwiGLU), one kernel, bf16 result.
 *   w_gate, w_up device bf16 [n_out, k_len]; out device bf16 [n_tokens, n_out]; pointers
 *   16-byte aligned. */
ct_status ct_swiglu(const void* x, int32_t n_tokens, int32_t k_len, const void* w_gate, const void* w_up, int32_t n_out,
                    void* out, void* stream);

/* Weights and cached KV of one layer.  All weights device bf16, one row per output feature:
 * attn_norm, ffn_norm [hidden]; wqkv [(n_q_heads + 2 n_kv_heads) head_dim, hidden];
 * wo [hidden, n_q_heads head_dim]; w_gate, w_up [ffn_dim, hidden]; w_down [hidden, ffn_dim].
 * chunks: this layer's n_chunks cached KV chunks (same token counts and positions in every
 * layer; k / v may be NULL when every row is recomputed). */
typedef struct {
  const void* attn_norm;
  const void* wqkv;
  const void* wo;
  const void* ffn_norm;
  const void* w_gate;
  const void* w_up;
  const void* w_down;
  const ct_chunk* chunks;
} ct_layer_weights;

/* Partial prefill of n_layers layers on the selected rows (pre-norm blocks: RMSNorm, selected
 * attention over the fused KV, output projection + residual, RMSNorm, SwiGLU FFN + residual).
 *   hidden_sel device bf16 [n_sel, hidden]: in, the layer-0 input rows of the selected tokens
 *              (compact, in sel_idx order); out, the last layer's output rows.
 *   k_bufs, v_bufs device bf16 [2, n_ctx, n_kv_heads, head_dim]: two layer buffers used in
 *              turn, so that layer l+1's pinned-host chunks are copied on copy_stream while
 *              layer l computes.  On return slot (n_layers-1) % 2 holds the last layer's fused KV.
 *   n_sel == n_ctx is ordinary full prefill: no cached KV is read or copied.
 *   workspace  at least ct_stack_workspace_bytes() bytes, 256-byte aligned.
 * Events are taken from the calling thread's pool. */
ct_status ct_partial_prefill_stack(const ct_layer_cfg* cfg, int32_t ffn_dim, float rms_eps, const ct_layer_weights* layers,
                                   int32_t n_layers, int32_t n_chunks, void* hidden_sel, const int32_t* sel_idx,
                                   int32_t n_sel, double recompute_ratio, void* k_bufs, void* v_bufs, void* workspace,
                                   size_t workspace_bytes, void* compute_stream, void* copy_stream);
size_t ct_stack_workspace_bytes(const ct_layer_cfg* cfg, int32_t ffn_dim, int32_t n_ctx, int32_t n_sel);

/* ct_partial_prefill_stack that also hands out what enters every layer (Sec. 4.2: the fusion
 * layers' inputs are the selected tokens' hidden states): layer_inputs, device bf16
 * [n_layers, n_sel, hidden], receives the rows of hidden_sel as layer l reads them (a device copy
 * on compute_stream per layer); layer l's output is layer l + 1's input, the last layer's is
 * hidden_sel.  For inspecting or checking single layers of a run; NULL makes the call
 * ct_partial_prefill_stack. */
ct_status ct_partial_prefill_stack_tap(const ct_layer_cfg* cfg, int32_t ffn_dim, float rms_eps,
                                       const ct_layer_weights* layers, int32_t n_layers, int32_t n_chunks,
                                       void* hidden_sel, const int32_t* sel_idx, int32_t n_sel, double recompute_ratio,
                                       void* k_bufs, void* v_bufs, void* workspace, size_t workspace_bytes,
                                       void* compute_stream, void* copy_stream, void* layer_inputs);

/* ---- Choice of the recomputation ratio for a given GPU and cache pool (Sec. 4.3).  Host code. ---- */

/* Per-layer latency model, Eq. 9: max(r N t_c, (1 - r) N t_i) + t_o.  t_c: recomputation cost
 * per token and layer, t_i: transfer cost per token and layer, t_o: fixed cost per layer (all
 * in the same unit of time; the result is in that unit).  Multiply by the number of layers for
 * the steady-state TTFT of Eq. 10. */
double ct_layer_latency_model(double r, double n_tokens, double t_c, double t_i, double t_o);

/* Crossover of the two branches of Eq. 9 (Eq. 11): t_i / (t_c + t_i), clipped to
 * [r_min, r_max] (r_min is the quality floor of Sec. 4.3, 0.15 in the paper). */
double ct_ratio_prior(double t_c, double t_i, double r_min, double r_max);

/* Golden-section search for the ratio with the least measured latency (Alg. 1), warm-started at
 * the prior r0: `eval(r, user)` returns the mean TTFT of the calibration set at ratio r and is
 * called once per iteration after the first two probes.  Stops when the bracket is narrower than
 * eps or after max_evals evaluations; *r_star is the midpoint of the final bracket, *n_evals
 * (may be NULL) the number of evaluations made.  Two departures from the listing, both needed
 * because r0 is not at a golden point of [r_min, r_max]: each new probe is the golden-section
 * point of the larger part that the surviving probe leaves of the bracket (the listing's
 * expression whenever the survivor is at a golden point; off it the listing's point can meet or
 * pass the survivor and the minimum is lost), and a prior that sits on a bound is moved inside
 * by a hundredth of the interval.  Errors: CT_ERR_NULL (eval, r_star), CT_ERR_RATIO (bounds not
 * 0 <= r_min <= r_max <= 1), CT_ERR_SHAPE (eps <= 0, max_evals < 2). */
typedef double (*ct_ttft_fn)(double r, void* user);
ct_status ct_ratio_search(ct_ttft_fn eval, void* user, double r0, double r_min, double r_max, double eps,
                          int32_t max_evals, double* r_star, int32_t* n_evals);

/* ---- Offline choice of the tokens to recompute (Sec. 4.1): done once per chunk and layer when
 * the chunk's cache is generated; its result is the index set the calls above consume. ---- */

/* Low-frequency energy scores, Eq. 2-6.  For each of n_batch sequences (say, the layers of one
 * chunk): real FFT of every (head, dim) column of K and of V along the tokens, bins
 * k >= c = floor(alpha * (floor(N/2) + 1)) zeroed, inverse real FFT back to N samples, then
 * scores[b, i] = (||K~_i||_2 + ||V~_i||_2) / 2 with the norms over the row_elems = H * D values
 * of token i.  fp32 arithmetic on bf16 inputs; the result does not depend on launch order.
 *   k, v        device bf16 [n_batch][n_tokens, row_elems], sequence b at element offset
 *               b * batch_stride (batch_stride >= n_tokens * row_elems)
 *   scores      device fp32 [n_batch, n_tokens]
 *   workspace   at least ct_frequency_workspace_bytes() bytes of device memory
 * n_tokens must be of the form 2^a 3^b 5^c; row_elems even.  Up to 4096 tokens the transform of a
 * strip of columns is done inside one compute unit's LDS; longer sequences (below 2^24 tokens, with
 * a divisor pair N1 N2 = n_tokens, both at most 4096) are transformed in two factors through one
 * complex fp32 copy of a tensor in the workspace (n_tokens * row_elems * 4 bytes; the workspace
 * must then be 256-byte aligned).  CT_ERR_UNSUPPORTED otherwise. */
ct_status ct_frequency_scores(const void* k, const void* v, int32_t n_batch, int64_t batch_stride, int32_t n_tokens,
                              int32_t row_elems, double alpha, float* scores, void* workspace, size_t workspace_bytes,
                              void* stream);
size_t ct_frequency_workspace_bytes(int32_t n_batch, int32_t n_tokens, int32_t row_elems);

/* TopK, Eq. 7: for each of n_batch score rows the k positions with the largest scores, written
 * in ascending position order (int32 [n_batch, k]).  Equal scores: the lower position wins, so
 * the set is unique.  Scores must not be NaN.  k = 0 writes nothing. */
ct_status ct_topk_indices(const float* scores, int32_t n_batch, int32_t n_tokens, int32_t k, int32_t* idx_out,
                          void* stream);

/* floor(ratio * n_tokens), at least 1 when ratio > 0: the size of the recomputation set. */
int32_t ct_frequency_n_selected(int32_t n_tokens, double ratio);

/* Eq. 2-7 in one call: scores (also returned, [n_batch, n_tokens]) and the recomputation sets
 * idx_out [n_batch, ct_frequency_n_selected(n_tokens, ratio)], each ascending. */
ct_status ct_select_frequency(const void* k, const void* v, int32_t n_batch, int64_t batch_stride, int32_t n_tokens,
                              int32_t row_elems, double alpha, double ratio, int32_t* idx_out, float* scores,
                              void* workspace, size_t workspace_bytes, void* stream);

/* Host-side check of an index set: strictly ascending and inside [0, n_ctx). */
ct_status ct_validate_indices(const int32_t* host_idx, int32_t n_sel, int32_t n_ctx);

/* Per-kernel timing for measurement runs.  With profiling on, every kernel launch the
 * library makes carries a pair of HIP events on its own dispatch (begin and end of that kernel
 * on the launch stream); nothing is put into the stream between kernels.
 * ct_profile_read waits for the recorded events of one kernel class, adds their elapsed
 * times and returns the number of launches and the summed milliseconds; ct_profile_reset
 * forgets what was recorded.  Classes: 0 qkv projection, 1 re-RoPE, 2 scatter,
 * 3 selected attention (main kernel), 4 attention split merge, 5 linear / SwiGLU GEMMs,
 * 6 RMSNorm, 7 frequency scores, 8 TopK.  Profiling is process wide,
 * off by default, creates events on first use and is not meant for concurrent callers. */
void ct_set_profiling(int32_t on);
void ct_profile_reset(void);
/* Measurement aid: the matrix-core rate this device sustains.  Runs a kernel that does nothing
 * but dependent-free v_mfma_f32_32x32x16_bf16 (one workgroup of eight waves per compute unit,
 * `iters` x 64 MFMAs per wave) on `stream`, waits for it, and stores the achieved TFLOP/s in
 * *tflops (host pointer).  `scratch` is device memory of at least 256 * 512 * 4 bytes that the
 * kernel writes its (meaningless) results to.  This is the ceiling the MFMA-bound kernels are
 * measured against besides the published peak; it is not part of the partial-prefill path. */
ct_status ct_measure_mfma_rate(void* scratch, int32_t iters, void* stream, double* tflops);
ct_status ct_profile_read(int32_t kernel_class, int64_t* launches, double* total_ms);

/* Message for the last non-OK status returned on this thread ("" if none). */
const char* ct_last_error(void);

/* Library version string. */
const char* ct_version(void);

#ifdef __cplusplus
}
#endif
#endif /* CACHETUNE_H */
