"""CPU oracle for the selective-recompute partial prefill (TEST INFRASTRUCTURE ONLY).

A plain, slow, float64 NumPy statement of what one layer of CacheTune's online sparse-reuse
pipeline computes (paper Sec. 4.2, "KV Cache Offloading and Sparse Reuse"), used by the
tests, the smoke check and the bench's CPU-baseline leg to judge the HIP kernels.  It is
not part of the product path, shares no code with it and must never be called from it.

The online path is exact given its inputs (the approximation of the method lies in *which*
tokens are recomputed and in reusing stale KV, both of which are inputs here), so every
function below is the definition written out, in float64, on bf16-valued inputs, with no
intermediate rounding:

  qkv_selected        Eq. 1 (k = h W_K, v = h W_V, and likewise q) for the selected tokens,
                      then standard RoPE at their true positions (Sec. 4.2, "Preserving
                      positional consistency", last paragraph).
  rerope_keys         Eq. 8 (deferred RoPE recovery) in its delta form: a key cached after
                      rotation at `old_pos` is rotated by (new_pos - old_pos).  The paper's
                      raw pre-RoPE cache is the special case old_pos = 0.
  scatter_kv          scatter fusion (Sec. 4.2, "Reducing online recomputation and fusion
                      overhead"): recomputed rows overwrite their slots of the layer buffer.
  selected_attention  the check/fusion-layer attention, computed for the selected tokens alone:
                      causal softmax attention of the selected queries over the fused KV.
  partial_prefill_layer  the composition of the four.
  rmsnorm, swiglu_ffn, layer_tail, partial_prefill_stack
                      the rest of a pre-norm transformer layer applied to the selected rows
                      only (Sec. 4.2: every layer after the check layer is a fusion layer that
                      works on the selected tokens) and the chain of layers.  The paper names
                      the models (Sec. 5) but not these formulas; they are the standard RMSNorm
                      and SwiGLU definitions of those models.

  layer_latency_model, ratio_prior, ratio_search
                      the hardware-aware choice of the recomputation ratio (Sec. 4.3): the
                      latency model of Eq. 9, its crossover (Eq. 11) and the warm-started
                      golden-section search of Alg. 1.  The search is an iteration, so it is
                      written step by step in the algorithm's notation.

  frequency_scores, topk_indices, select_frequency
                      the offline frequency-domain choice of the tokens to recompute (Sec. 4.1):
                      rFFT along the sequence (Eq. 2), low-pass (Eq. 3), inverse rFFT (Eq. 4),
                      per-token norms (Eq. 5), joint score (Eq. 6), TopK (Eq. 7).  NumPy's FFT
                      is the library step; everything else is the equations as written.

Readings where the paper is silent (RoPE pair convention and frequencies, softmax scale,
GQA head mapping, floor for r*N, V being position independent) are stated at the function
that uses them.  All pins live in tests/test_oracle_pins.py.
"""
from __future__ import annotations

import numpy as np

HALF_SPLIT = 0   # pair j couples elements (j, j + D/2)
INTERLEAVED = 1  # pair j couples elements (2j, 2j + 1)


# ----------------------------------------------------------------------------- RoPE
def rope_frequencies(head_dim: int, theta: float) -> np.ndarray:
    """omega_j = theta^(-2j/D), j = 0..D/2-1 (the paper only says "RoPE"; this is the
    standard definition with no long-context scaling)."""
    j = np.arange(head_dim // 2, dtype=np.float64)
    return np.float64(theta) ** (-2.0 * j / np.float64(head_dim))


def rotate(x: np.ndarray, steps: np.ndarray, theta: float, style: int = HALF_SPLIT) -> np.ndarray:
    """Rotate every pair of x[t, h, :] by the angle steps[t] * omega_j.

    x: [T, H, D] float64; steps: [T] integers (a position, or a position difference).
    (x_a, x_b) -> (x_a cos - x_b sin, x_a sin + x_b cos).
    """
    x = np.asarray(x, dtype=np.float64)
    T, H, D = x.shape
    half = D // 2
    ang = np.asarray(steps, dtype=np.float64)[:, None] * rope_frequencies(D, theta)[None, :]  # [T, D/2]
    c = np.cos(ang)[:, None, :]
    s = np.sin(ang)[:, None, :]
    out = np.empty_like(x)
    if style == HALF_SPLIT:
        a, b = x[..., :half], x[..., half:]
        out[..., :half] = a * c - b * s
        out[..., half:] = a * s + b * c
    elif style == INTERLEAVED:
        a, b = x[..., 0::2], x[..., 1::2]
        out[..., 0::2] = a * c - b * s
        out[..., 1::2] = a * s + b * c
    else:
        raise ValueError("rope style")
    return out


# ----------------------------------------------------------------------------- step a1
def qkv_selected(hidden_sel, wqkv, bias, sel_pos, n_q_heads, n_kv_heads, head_dim, theta,
                 style: int = HALF_SPLIT):
    """Fresh Q, K, V for the selected tokens (Eq. 1) with RoPE on Q and K at `sel_pos`.

    hidden_sel: [n, E]; wqkv: [O, E] with O = (Hq + 2 Hkv) D, rows ordered Q heads, K heads,
    V heads (out-features major, so y = x W^T); bias: [O] or None; sel_pos: [n].
    Returns q [n, Hq, D], k [n, Hkv, D], v [n, Hkv, D].
    """
    x = np.asarray(hidden_sel, dtype=np.float64)
    w = np.asarray(wqkv, dtype=np.float64)
    y = x @ w.T
    if bias is not None:
        y = y + np.asarray(bias, dtype=np.float64)[None, :]
    n = x.shape[0]
    nq = n_q_heads * head_dim
    nk = n_kv_heads * head_dim
    q = y[:, :nq].reshape(n, n_q_heads, head_dim)
    k = y[:, nq:nq + nk].reshape(n, n_kv_heads, head_dim)
    v = y[:, nq + nk:nq + 2 * nk].reshape(n, n_kv_heads, head_dim).copy()
    q = rotate(q, sel_pos, theta, style)
    k = rotate(k, sel_pos, theta, style)
    return q, k, v


# ----------------------------------------------------------------------------- step a3
def rerope_keys(k_cached, old_pos, new_pos, theta, style: int = HALF_SPLIT):
    """Deferred RoPE recovery (Eq. 8), delta form: rotate row i by new_pos[i] - old_pos[i]."""
    delta = np.asarray(new_pos, dtype=np.int64) - np.asarray(old_pos, dtype=np.int64)
    return rotate(k_cached, delta, theta, style)


# ----------------------------------------------------------------------------- step a4
def scatter_kv(k_buf, v_buf, k_sel, v_sel, sel_idx):
    """Scatter fusion: rows sel_idx of the buffers take the recomputed rows; returns copies."""
    k_out = np.array(k_buf, copy=True)
    v_out = np.array(v_buf, copy=True)
    idx = np.asarray(sel_idx, dtype=np.int64)
    k_out[idx] = k_sel
    v_out[idx] = v_sel
    return k_out, v_out


# ----------------------------------------------------------------------------- step a5
def selected_attention(q_sel, k_buf, v_buf, sel_idx, rows=None, scale=None):
    """Causal attention of the selected queries over the fused layer KV.

    q_sel: [n, Hq, D]; k_buf, v_buf: [N, Hkv, D]; sel_idx: [n] buffer rows of the queries.
    Query s sees keys at buffer rows 0..sel_idx[s] inclusive (its own fresh K/V included).
    Query head h reads KV head h // (Hq/Hkv).  scale defaults to 1/sqrt(D).
    `rows`: optional ordinals into the selected set; only those outputs are evaluated
    (each output row depends on no other query, so a subset is exact).
    Returns out [len(rows), Hq, D] and lse [len(rows), Hq] (natural-log sum of exp of the
    scaled scores).
    """
    q = np.asarray(q_sel, dtype=np.float64)
    k = np.asarray(k_buf, dtype=np.float64)
    v = np.asarray(v_buf, dtype=np.float64)
    idx = np.asarray(sel_idx, dtype=np.int64)
    if rows is not None:
        rows = np.asarray(rows, dtype=np.int64)
        q = q[rows]
        idx = idx[rows]
    n, Hq, D = q.shape
    N, Hkv, _ = k.shape
    G = Hq // Hkv
    if scale is None:
        scale = 1.0 / np.sqrt(np.float64(D))
    out = np.zeros((n, Hq, D), dtype=np.float64)
    lse = np.zeros((n, Hq), dtype=np.float64)
    if n == 0:
        return out, lse
    visible = np.arange(N, dtype=np.int64)[None, :] <= idx[:, None]   # [n, N]
    for h in range(Hq):
        g = h // G
        s = (q[:, h, :] @ k[:, g, :].T) * scale                        # [n, N]
        s = np.where(visible, s, -np.inf)
        m = s.max(axis=1, keepdims=True)
        p = np.exp(s - m)
        l = p.sum(axis=1, keepdims=True)
        # masked columns carry weight exp(-inf) = 0; zero the operand too so that a
        # non-finite value parked in an invisible row cannot leak through 0 * inf
        vh = v[:, g, :]
        out[:, h, :] = _masked_matmul(p, vh, visible) / l
        lse[:, h] = (m + np.log(l))[:, 0]
    return out, lse


def _masked_matmul(p, vh, visible):
    """sum_j p[i, j] * vh[j, :] over the visible j only."""
    if np.isfinite(vh).all():
        return p @ vh
    out = np.empty((p.shape[0], vh.shape[1]), dtype=np.float64)
    for i in range(p.shape[0]):
        cols = np.flatnonzero(visible[i])
        out[i] = p[i, cols] @ vh[cols]
    return out


# ----------------------------------------------------------------------------- step a6
def partial_prefill_layer(hidden_sel, wqkv, bias, k_cache, v_cache, old_pos, new_pos, sel_idx,
                          n_q_heads, n_kv_heads, head_dim, theta, style: int = HALF_SPLIT,
                          rows=None):
    """One fusion-layer step: recompute the selected tokens, re-rotate the reused keys,
    scatter, attend.  Returns (attention output for the selected rows, fused K, fused V)."""
    sel_idx = np.asarray(sel_idx, dtype=np.int64)
    sel_pos = np.asarray(new_pos, dtype=np.int64)[sel_idx]
    q, k_new, v_new = qkv_selected(hidden_sel, wqkv, bias, sel_pos, n_q_heads, n_kv_heads,
                                   head_dim, theta, style)
    k_rot = rerope_keys(k_cache, old_pos, new_pos, theta, style)
    k_fused, v_fused = scatter_kv(k_rot, np.asarray(v_cache, dtype=np.float64), k_new, v_new, sel_idx)
    out, lse = selected_attention(q, k_fused, v_fused, sel_idx, rows=rows)
    return out, lse, k_fused, v_fused


# ----------------------------------------------------------------------------- step a7
def rmsnorm(x, weight, eps):
    """y = x / sqrt(mean(x^2) + eps) * weight over the last axis."""
    x = np.asarray(x, dtype=np.float64)
    ms = (x * x).mean(axis=-1, keepdims=True)
    return x / np.sqrt(ms + np.float64(eps)) * np.asarray(weight, dtype=np.float64)


def silu(x):
    return x / (1.0 + np.exp(-x))


def swiglu_ffn(x, w_gate, w_up, w_down):
    """(silu(x Wg^T) * (x Wu^T)) Wd^T with weights stored one row per output feature."""
    x = np.asarray(x, dtype=np.float64)
    g = x @ np.asarray(w_gate, dtype=np.float64).T
    u = x @ np.asarray(w_up, dtype=np.float64).T
    return (silu(g) * u) @ np.asarray(w_down, dtype=np.float64).T


def layer_tail(h, attn_out, wo, ffn_norm, w_gate, w_up, w_down, eps):
    """Output projection + residual, then RMSNorm -> SwiGLU FFN + residual.
    h: [n, E] layer input rows; attn_out: [n, Hq, D]."""
    h = np.asarray(h, dtype=np.float64)
    a = np.asarray(attn_out, dtype=np.float64).reshape(h.shape[0], -1)
    h1 = h + a @ np.asarray(wo, dtype=np.float64).T
    return h1 + swiglu_ffn(rmsnorm(h1, ffn_norm, eps), w_gate, w_up, w_down)


def transformer_layer(h_sel, lw, old_pos, new_pos, sel_idx, n_q_heads, n_kv_heads, head_dim, theta, eps,
                      style: int = HALF_SPLIT):
    """One layer on the selected rows.  lw: dict with attn_norm, wqkv, wo, ffn_norm, w_gate, w_up,
    w_down, k_cache, v_cache.  Returns (output rows, fused K, fused V)."""
    x = rmsnorm(h_sel, lw["attn_norm"], eps)
    attn, _, kf, vf = partial_prefill_layer(x, lw["wqkv"], None, lw["k_cache"], lw["v_cache"], old_pos, new_pos,
                                            sel_idx, n_q_heads, n_kv_heads, head_dim, theta, style)
    return layer_tail(h_sel, attn, lw["wo"], lw["ffn_norm"], lw["w_gate"], lw["w_up"], lw["w_down"], eps), kf, vf


def partial_prefill_stack(h_sel, layers, old_pos, new_pos, sel_idx, n_q_heads, n_kv_heads, head_dim, theta, eps,
                          style: int = HALF_SPLIT, keep_inputs: bool = False):
    """Chain of layers on the selected rows; the same index set in every layer.
    Returns the last layer's output rows (and, with keep_inputs, the list of per-layer inputs)."""
    h = np.asarray(h_sel, dtype=np.float64)
    inputs = []
    for lw in layers:
        if keep_inputs:
            inputs.append(h)
        h, _, _ = transformer_layer(h, lw, old_pos, new_pos, sel_idx, n_q_heads, n_kv_heads, head_dim, theta, eps, style)
    return (h, inputs) if keep_inputs else h


# ----------------------------------------------------------------------------- ratio scheduling (Sec. 4.3)
def layer_latency_model(r, n_tokens, t_c, t_i, t_o):
    """Eq. 9: recomputation of r N tokens overlaps the transfer of the other (1 - r) N; the
    slower of the two plus the fixed per-layer cost is the layer's latency."""
    return max(r * n_tokens * t_c, (1.0 - r) * n_tokens * t_i) + t_o


def ratio_prior(t_c, t_i, r_min, r_max):
    """Eq. 11, clipped to the semantic bounds as Alg. 1 requires of its input."""
    r0 = t_i / (t_c + t_i) if (t_c + t_i) > 0.0 else r_min
    return min(max(r0, r_min), r_max)


def ratio_search(f, r0, r_min, r_max, eps, max_evals=64):
    """Alg. 1: golden-section search on [r_min, r_max] with the prior r0 as one of the first two
    probes.  Returns (r_star, probes), probes being the ratios f was evaluated at, in order.

    Readings.  (1) The listing places each new probe at b - phi (b - a) or a + phi (b - a) and
    makes the surviving probe the other one.  That is right when the survivor sits at a golden
    point of the shrunken bracket, which textbook starting probes guarantee and r0 does not: with
    an off-golden survivor the new probe can coincide with it or land on its wrong side, and the
    next comparison then discards the part of the bracket that holds the minimum.  Here the new
    probe is the golden-section point of the larger of the two parts into which the survivor
    splits the bracket (the usual golden step of bracketing minimisers); it equals the listing's
    expression whenever the survivor is at a golden point, and keeps a < x1 < x2 < b always.
    (2) An r0 that was clipped onto a bound is moved inside by 1 % of the bracket: a probe at the
    bound cannot tell the search which side the minimum is on.  (3) max_evals bounds the loop,
    since f is a noisy measurement in practice."""
    a, b = float(r_min), float(r_max)
    r0 = min(max(float(r0), a), b)
    phi = (np.sqrt(5.0) - 1.0) / 2.0
    probes = []

    def evaluate(x):
        probes.append(x)
        return f(x)

    if b - a < eps:
        return (a + b) / 2.0, probes
    inset = 0.01 * (b - a)
    if r0 <= (a + b) / 2.0:
        x1, x2 = max(r0, a + inset), a + phi * (b - a)
    else:
        x1, x2 = b - phi * (b - a), min(r0, b - inset)
    f1 = evaluate(x1)
    f2 = evaluate(x2)
    while abs(b - a) >= eps and len(probes) < max_evals:
        if f1 < f2:          # the minimum lies in [a, x2]; x1 survives
            b, s, fs = x2, x1, f1
        else:                # the minimum lies in [x1, b]; x2 survives
            a, s, fs = x1, x2, f2
        if s - a > b - s:    # new probe left of the survivor
            x1, x2, f2 = s - (1.0 - phi) * (s - a), s, fs
            f1 = evaluate(x1)
        else:                # new probe right of the survivor
            x1, x2, f1 = s, s + (1.0 - phi) * (b - s), fs
            f2 = evaluate(x2)
    return (a + b) / 2.0, probes


# ----------------------------------------------------------------------------- frequency-guided selection (Sec. 4.1)
def lowpass_cutoff(n_tokens: int, alpha: float) -> int:
    """Eq. 3: c = floor(alpha * (floor(N/2) + 1)); bins k >= c are zeroed.  (A 1e-9 guard keeps a
    product that is an integer in exact arithmetic from falling below it in floating point.)"""
    return int(np.floor(alpha * (n_tokens // 2 + 1) + 1e-9))


def lowpass_reconstruction(x, alpha: float):
    """Eq. 2-4 for one tensor x [N, ...]: transform along axis 0, zero the bins from the cutoff
    on, transform back to N samples."""
    x = np.asarray(x, dtype=np.float64)
    n = x.shape[0]
    spec = np.fft.rfft(x, axis=0)
    spec[lowpass_cutoff(n, alpha):] = 0.0
    return np.fft.irfft(spec, n=n, axis=0)


def frequency_scores(k, v, alpha: float):
    """Eq. 5-6: s_i = (||K~_i||_2 + ||V~_i||_2) / 2, the norms taken over all heads and
    dimensions of token i.  k, v: [N, H, D] (or [N, H*D]).  Returns float64 [N]."""
    kt = lowpass_reconstruction(k, alpha)
    vt = lowpass_reconstruction(v, alpha)
    n = kt.shape[0]
    s_k = np.sqrt((kt.reshape(n, -1) ** 2).sum(axis=1))
    s_v = np.sqrt((vt.reshape(n, -1) ** 2).sum(axis=1))
    return 0.5 * (s_k + s_v)


def topk_indices(scores, k: int):
    """Eq. 7: the k tokens with the largest scores, returned in ascending index order (the form
    the online path takes its index set in).  Reading: among equal scores the lower index wins,
    which makes the set unique."""
    scores = np.asarray(scores)
    n = scores.shape[0]
    order = sorted(range(n), key=lambda i: (-float(scores[i]), i))
    return np.array(sorted(order[:k]), dtype=np.int32)


def select_frequency(k, v, alpha: float, ratio: float):
    """The recomputation set of one chunk and layer: TopK of the scores with floor(r N) entries
    (at least one when r > 0).  Returns (indices, scores)."""
    s = frequency_scores(k, v, alpha)
    n = s.shape[0]
    n_sel = n if ratio >= 1.0 else int(np.floor(ratio * n + 1e-9))
    if ratio > 0.0 and n_sel < 1:
        n_sel = 1
    return topk_indices(s, n_sel), s
