"""Seeded synthetic inputs for the partial-prefill hot path.

This module only *makes data*: bf16 bit patterns, position vectors, index sets and chunk
tables.  It contains none of the method's arithmetic (no projection, no rotation, no
softmax) so that the CPU oracle and the HIP path can both be fed from it while sharing
no computation.

The inputs stand in for the paper's workloads (multi-chunk RAG / QA prompts, Sec. 5):
several independently cached fixed-length chunks are concatenated into one context, the
keys of every chunk were cached at chunk-local positions 0..L-1, and a fraction r of the
tokens (default 15 %, the paper's quality floor, Sec. 4.3) is selected for recomputation.

Recipe (all draws from numpy's PCG64 ``default_rng([seed, stream_id])``):
  stream 0 hidden states  ~ N(0,1)                     [rows, E]
  stream 1 Wqkv           ~ N(0,1)/sqrt(E)             [O, E]   (out-features major)
  stream 2 cached K       ~ N(0,1)                     [N, Hkv, D]
  stream 3 cached V       ~ N(0,1)                     [N, Hkv, D]
  stream 4 index set      (see ``_select_*``)
every float is rounded to bf16 (round-to-nearest-even) and handed out as uint16 bits.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np


# --------------------------------------------------------------------------- bf16 format
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 values to bfloat16 (nearest, ties to even); returns uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + (np.uint32(0x7FFF) + lsb)
    out = (r >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        out = np.where(nan, np.uint16(0x7FC0), out)
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f32(b).astype(np.float64)


def _normal_bf16(seed: int, stream: int, shape, scale: float = 1.0, slab: int = 1 << 24) -> np.ndarray:
    """N(0,1)*scale as bf16 bits, generated in slabs so peak memory stays small."""
    rng = np.random.default_rng([seed, stream])
    total = int(np.prod(shape))
    out = np.empty(total, dtype=np.uint16)
    for lo in range(0, total, slab):
        hi = min(total, lo + slab)
        v = rng.standard_normal(hi - lo, dtype=np.float32)
        if scale != 1.0:
            v *= np.float32(scale)
        out[lo:hi] = f32_to_bf16_bits(v)
    return out.reshape(shape)


# --------------------------------------------------------------------------- shapes
@dataclass(frozen=True)
class LayerShape:
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    rope_theta: float
    rope_style: int = 0  # 0 = half-split pairs (j, j+D/2); 1 = interleaved pairs (2j, 2j+1)

    @property
    def qkv_width(self) -> int:
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads


TINY = LayerShape(hidden=512, n_q_heads=8, n_kv_heads=2, head_dim=64, rope_theta=1.0e4)
LLAMA3_8B = LayerShape(hidden=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, rope_theta=5.0e5)


@dataclass(frozen=True)
class WorkloadSpec:
    name: str
    shape: LayerShape
    n_chunks: int
    chunk_len: int
    ratio_pct: int          # recompute ratio in percent
    selection: str          # "uniform" | "forced16" | "clustered" | "all"
    seed: int
    compact_hidden: bool = False   # True: hidden holds only the selected rows

    @property
    def n_ctx(self) -> int:
        return self.n_chunks * self.chunk_len

    @property
    def n_sel(self) -> int:
        return n_selected(self.n_ctx, self.ratio_pct)


def n_selected(n_ctx: int, ratio_pct: int) -> int:
    """floor(r*N), at least one row when r > 0, all rows when r = 100 %."""
    if ratio_pct <= 0:
        return 0
    if ratio_pct >= 100:
        return n_ctx
    return max(1, (ratio_pct * n_ctx) // 100)


def spec(config: int, ratio_pct: Optional[int] = None) -> WorkloadSpec:
    """The five synthetic configurations (1-based, as in the baseline description)."""
    if config == 1:
        return WorkloadSpec("cfg1-tiny-1k", TINY, 4, 256, ratio_pct or 15, "uniform", 1001)
    if config == 2:
        return WorkloadSpec("cfg2-llama8b-8k", LLAMA3_8B, 8, 1024, ratio_pct or 15, "forced16", 1002)
    if config == 3:
        r = ratio_pct or 15
        k = {5: 0, 10: 1, 15: 2, 30: 3, 100: 4}.get(r, 5)
        return WorkloadSpec(f"cfg3-llama8b-32k-r{r}", LLAMA3_8B, 16, 2048, r,
                            "all" if r >= 100 else "uniform", 1003 + 10 * k)
    if config == 4:
        return WorkloadSpec("cfg4-llama8b-128k", LLAMA3_8B, 32, 4096, ratio_pct or 5, "clustered", 1004,
                            compact_hidden=True)
    if config == 5:
        return WorkloadSpec("cfg5-llama8b-32k-stack", LLAMA3_8B, 16, 2048, ratio_pct or 15, "uniform", 1005)
    raise ValueError(f"unknown config {config}")


def custom_spec(name: str, shape: LayerShape, n_chunks: int, chunk_len: int, ratio_pct: int,
                selection: str = "uniform", seed: int = 7, compact_hidden: bool = False) -> WorkloadSpec:
    return WorkloadSpec(name, shape, n_chunks, chunk_len, ratio_pct, selection, seed, compact_hidden)


# --------------------------------------------------------------------------- index sets
def _select_uniform(rng, n_ctx, n_sel):
    return np.sort(rng.choice(n_ctx, size=n_sel, replace=False))


def _select_forced16(rng, n_chunks, chunk_len, n_sel):
    """First 16 tokens of every chunk are always selected and count toward the budget."""
    n_ctx = n_chunks * chunk_len
    forced = (np.arange(n_chunks)[:, None] * chunk_len + np.arange(min(16, chunk_len))[None, :]).ravel()
    forced = forced[:n_sel]
    mask = np.ones(n_ctx, dtype=bool)
    mask[forced] = False
    rest = np.flatnonzero(mask)
    extra = rng.choice(rest, size=n_sel - forced.size, replace=False)
    return np.sort(np.concatenate([forced, extra]))


def _select_clustered(rng, n_chunks, chunk_len, n_sel, edge=64, share=0.7):
    """`share` of the budget from tokens within `edge` of a chunk boundary, rest uniform.

    When the boundary pool is smaller than the requested share the pool is taken whole
    (dense runs at every chunk edge) and the remainder is drawn from the interior.
    """
    n_ctx = n_chunks * chunk_len
    off = np.arange(chunk_len)
    near = (off < edge) | (off >= chunk_len - edge)
    pool = (np.arange(n_chunks)[:, None] * chunk_len + off[None, :])[:, near].ravel()
    want = min(int(share * n_sel), pool.size, n_sel)
    clustered = pool if want == pool.size else rng.choice(pool, size=want, replace=False)
    mask = np.ones(n_ctx, dtype=bool)
    mask[clustered] = False
    rest = np.flatnonzero(mask)
    extra = rng.choice(rest, size=n_sel - clustered.size, replace=False)
    return np.sort(np.concatenate([clustered, extra]))


def select_indices(sp: WorkloadSpec, n_sel: Optional[int] = None) -> np.ndarray:
    """The selected token indices, ascending.  `n_sel` overrides the count that follows from the
    spec's percentage (for ratios that are not whole percents)."""
    rng = np.random.default_rng([sp.seed, 4])
    n_ctx = sp.n_ctx
    n_sel = sp.n_sel if n_sel is None else int(n_sel)
    if n_sel == 0:
        idx = np.empty(0, dtype=np.int64)
    elif sp.selection == "all" or n_sel == n_ctx:
        idx = np.arange(n_ctx)
    elif sp.selection == "uniform":
        idx = _select_uniform(rng, n_ctx, n_sel)
    elif sp.selection == "forced16":
        idx = _select_forced16(rng, sp.n_chunks, sp.chunk_len, n_sel)
    elif sp.selection == "clustered":
        idx = _select_clustered(rng, sp.n_chunks, sp.chunk_len, n_sel)
    else:
        raise ValueError(sp.selection)
    return idx.astype(np.int32)


# --------------------------------------------------------------------------- full workload
@dataclass
class Workload:
    spec: WorkloadSpec
    hidden: np.ndarray          # uint16 bf16 bits, [N, E] or [n_sel, E] when compact
    hidden_rows: Optional[np.ndarray]  # int32 [n_sel] rows of `hidden` holding the selected tokens, None = compact
    wqkv: np.ndarray            # uint16 [O, E]
    k_cache: np.ndarray         # uint16 [N, Hkv, D]  keys as cached (rotated at old_pos)
    v_cache: np.ndarray         # uint16 [N, Hkv, D]
    old_pos: np.ndarray         # int32 [N]
    new_pos: np.ndarray         # int32 [N]
    sel_idx: np.ndarray         # int32 [n_sel], ascending, unique
    chunk_rows: np.ndarray = field(default=None)   # int32 [C+1] buffer row where each chunk starts
    chunk_old_start: np.ndarray = field(default=None)  # int32 [C]
    chunk_new_start: np.ndarray = field(default=None)  # int32 [C]

    @property
    def sel_pos(self) -> np.ndarray:
        return self.new_pos[self.sel_idx]


def make_workload(sp: WorkloadSpec, with_hidden: bool = True) -> Workload:
    sh = sp.shape
    n_ctx = sp.n_ctx
    sel = select_indices(sp)
    if sp.compact_hidden:
        hidden = _normal_bf16(sp.seed, 0, (sel.size, sh.hidden)) if with_hidden else None
        rows = None
    else:
        hidden = _normal_bf16(sp.seed, 0, (n_ctx, sh.hidden)) if with_hidden else None
        rows = sel.copy()
    wqkv = _normal_bf16(sp.seed, 1, (sh.qkv_width, sh.hidden), scale=1.0 / np.sqrt(sh.hidden))
    k = _normal_bf16(sp.seed, 2, (n_ctx, sh.n_kv_heads, sh.head_dim))
    v = _normal_bf16(sp.seed, 3, (n_ctx, sh.n_kv_heads, sh.head_dim))
    i = np.arange(n_ctx, dtype=np.int32)
    old_pos = (i % sp.chunk_len).astype(np.int32)       # every chunk cached at positions 0..L-1
    new_pos = i.copy()                                  # concatenated context
    c = np.arange(sp.n_chunks, dtype=np.int32)
    return Workload(sp, hidden, rows, wqkv, k, v, old_pos, new_pos, sel,
                    chunk_rows=np.concatenate([c * sp.chunk_len, [n_ctx]]).astype(np.int32),
                    chunk_old_start=np.zeros(sp.n_chunks, dtype=np.int32),
                    chunk_new_start=(c * sp.chunk_len).astype(np.int32))


def sample_rows(n_sel: int, count: int, seed: int = 0) -> np.ndarray:
    """A bounded, seeded subset of selected-row ordinals: first, last and a uniform fill."""
    if n_sel <= count:
        return np.arange(n_sel, dtype=np.int64)
    rng = np.random.default_rng([seed, 99])
    pick = set([0, 1, n_sel // 2, n_sel - 2, n_sel - 1])
    pick.update(rng.choice(n_sel, size=count - len(pick), replace=False).tolist())
    return np.array(sorted(pick))[:count].astype(np.int64)


# --------------------------------------------------------------------------- multi-layer stack
@dataclass
class StackWorkload:
    spec: WorkloadSpec
    ffn_dim: int
    rms_eps: float
    hidden0: np.ndarray          # uint16 [n_sel, E]: layer-0 input rows of the selected tokens
    layers: list                 # per layer: dict of uint16 arrays (attn_norm, wqkv, wo, ffn_norm, w_gate, w_up, w_down, k_cache, v_cache)
    old_pos: np.ndarray
    new_pos: np.ndarray
    sel_idx: np.ndarray
    chunk_rows: np.ndarray
    chunk_new_start: np.ndarray


def make_stack_workload(sp: WorkloadSpec, n_layers: int, ffn_dim: int, rms_eps: float = 1e-5,
                        unit_norm_weights: bool = False) -> StackWorkload:
    """Per layer (streams 100*l + k of the spec's seed): 0 attn_norm, 1 wqkv ~ N(0,1)/sqrt(E),
    2 wo ~ N(0,1)/sqrt(Hq*D), 3 ffn_norm, 4 w_gate, 5 w_up ~ N(0,1)/sqrt(E), 6 w_down ~ N(0,1)/sqrt(F),
    7 K cache, 8 V cache ~ N(0,1); norm weights are 1 (or 1 + 0.1 N(0,1) to exercise the multiply).
    Stream 0 of the spec's seed gives the layer-0 input rows."""
    sh = sp.shape
    E, qd = sh.hidden, sh.n_q_heads * sh.head_dim
    n_ctx = sp.n_ctx
    sel = select_indices(sp)

    def norm_w(stream):
        if unit_norm_weights:
            return f32_to_bf16_bits(np.ones(E, dtype=np.float32))
        rng = np.random.default_rng([sp.seed, stream])
        return f32_to_bf16_bits((1.0 + 0.1 * rng.standard_normal(E)).astype(np.float32))

    layers = []
    for l in range(n_layers):
        b = 100 * (l + 1)
        layers.append(dict(
            attn_norm=norm_w(b + 0),
            wqkv=_normal_bf16(sp.seed, b + 1, (sh.qkv_width, E), 1.0 / np.sqrt(E)),
            wo=_normal_bf16(sp.seed, b + 2, (E, qd), 1.0 / np.sqrt(qd)),
            ffn_norm=norm_w(b + 3),
            w_gate=_normal_bf16(sp.seed, b + 4, (ffn_dim, E), 1.0 / np.sqrt(E)),
            w_up=_normal_bf16(sp.seed, b + 5, (ffn_dim, E), 1.0 / np.sqrt(E)),
            w_down=_normal_bf16(sp.seed, b + 6, (E, ffn_dim), 1.0 / np.sqrt(ffn_dim)),
            k_cache=_normal_bf16(sp.seed, b + 7, (n_ctx, sh.n_kv_heads, sh.head_dim)),
            v_cache=_normal_bf16(sp.seed, b + 8, (n_ctx, sh.n_kv_heads, sh.head_dim)),
        ))
    i = np.arange(n_ctx, dtype=np.int32)
    c = np.arange(sp.n_chunks, dtype=np.int32)
    return StackWorkload(sp, ffn_dim, rms_eps, _normal_bf16(sp.seed, 0, (sel.size, E)), layers,
                         (i % sp.chunk_len).astype(np.int32), i.copy(), sel,
                         np.concatenate([c * sp.chunk_len, [n_ctx]]).astype(np.int32),
                         (c * sp.chunk_len).astype(np.int32))


# --------------------------------------------------------------------------- chunk K/V for the offline scoring
def make_spectral_kv(seed: int, n_tokens: int, row_elems: int, n_batch: int = 1):
    """Synthetic per-chunk K and V with structure along the sequence, standing in for the cached
    K/V of real chunks: per column a few slow sinusoids (random frequency below N/16, amplitude,
    phase) and a slow drift, white noise of comparable size on top, a per-token gain that makes
    about 3 % of the tokens stand out by 2-4x (attention-sink-like rows), so that low-pass
    scores separate tokens.  Returns two uint16 (bf16 bits) arrays [n_batch, n_tokens, row_elems]."""
    out = []
    for t in range(2):
        rng = np.random.default_rng([seed, 70 + t])
        n = np.arange(n_tokens, dtype=np.float64)[None, :, None]
        x = rng.standard_normal((n_batch, n_tokens, row_elems))
        for _ in range(3):
            f = rng.uniform(0.0, max(1.0, n_tokens / 16.0), (n_batch, 1, row_elems))
            a = rng.uniform(0.2, 1.0, (n_batch, 1, row_elems))
            ph = rng.uniform(0.0, 2 * np.pi, (n_batch, 1, row_elems))
            x += a * np.cos(2 * np.pi * f * n / n_tokens + ph)
        x += rng.standard_normal((n_batch, 1, row_elems)) * (n / max(1, n_tokens) - 0.5)
        gain = np.ones((n_batch, n_tokens, 1))
        hot = rng.random((n_batch, n_tokens, 1)) < 0.03
        gain[hot] = rng.uniform(2.0, 4.0, int(hot.sum()))
        out.append(f32_to_bf16_bits((x * gain).astype(np.float32)))
    return out[0], out[1]
