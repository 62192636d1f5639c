"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle, element by
element on the same seeded inputs.  Acceptance: bit-exact for scatter placement and copies;
max-abs <= 2e-2 and per-row relative L2 <= 1e-2 for bf16-in / fp32-accumulate outputs."""
import math

import numpy as np
import pytest
import torch

from oracle import ct_oracle as O
from paper_2605_24022_amd import binding as B
from paper_2605_24022_amd import workloads as W
from tests.gpu_util import (assert_close, bits_of, dev_bf16, dev_i32, f64_of, pinned_bf16, say)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "GPU tests need a GPU (run with -m 'not gpu' elsewhere)"
    B.load()
    torch.cuda.set_device(0)


def _shape(E, Hq, Hkv, D, theta, style=0):
    return W.LayerShape(E, Hq, Hkv, D, theta, style)


# ------------------------------------------------------------------------------ re-RoPE
@pytest.mark.parametrize("Hkv,D,theta,style", [(2, 64, 1e4, 0), (8, 128, 5e5, 0), (8, 128, 5e5, 1), (3, 64, 1e4, 1),
                                                 (4, 128, 1e4, 0)])
def test_rerope_per_token_positions(Hkv, D, theta, style):
    n = 1000 + 37                                    # ragged: not a multiple of the block's tokens
    rng = np.random.default_rng([11, Hkv, D, style])
    k_bits = W.f32_to_bf16_bits(rng.standard_normal((n, Hkv, D), dtype=np.float32))
    old = rng.integers(0, 4096, n).astype(np.int32)
    new = rng.integers(0, 131072, n).astype(np.int32)   # deltas of either sign, up to 1.3e5
    new[:4] = old[:4]                                 # delta 0 must be the identity
    cfg = B.make_cfg(Hkv * D * 2, Hkv * 2, Hkv, D, theta, style)
    say(f"rerope per-token Hkv={Hkv} D={D} style={style} n={n}")
    k = dev_bf16(k_bits)
    out = torch.empty_like(k)
    B.ct_rerope_keys(cfg, k, out, dev_i32(old), dev_i32(new), n)
    torch.cuda.synchronize()
    want = O.rerope_keys(W.bf16_bits_to_f64(k_bits), old, new, theta, style)
    assert_close(f64_of(out), want, "rerope src->dst", rel_l2=2.5e-3)
    assert np.array_equal(bits_of(out)[:4], k_bits[:4])
    # in place, and old_pos = NULL means a raw (never rotated) cache
    B.ct_rerope_keys(cfg, k, k, None, dev_i32(new), n)
    torch.cuda.synchronize()
    want0 = O.rerope_keys(W.bf16_bits_to_f64(k_bits), np.zeros(n, dtype=np.int64), new, theta, style)
    assert_close(f64_of(k), want0, "rerope in place, raw cache", rel_l2=2.5e-3)


@pytest.mark.parametrize("raw", [0, 1])
def test_rerope_chunk_with_value_copy(raw):
    Hkv, D, theta, n = 8, 128, 5e5, 513
    rng = np.random.default_rng([12, raw])
    k_bits = W.f32_to_bf16_bits(rng.standard_normal((n, Hkv, D), dtype=np.float32))
    v_bits = W.f32_to_bf16_bits(rng.standard_normal((n, Hkv, D), dtype=np.float32))
    cfg = B.make_cfg(4096, 32, Hkv, D, theta)
    old0, new0 = 7, 100000
    say(f"rerope chunk raw={raw}")
    k, v = dev_bf16(k_bits), dev_bf16(v_bits)
    ko, vo = torch.zeros_like(k), torch.zeros_like(v)
    B.ct_rerope_chunk(cfg, k, ko, v, vo, n, old0, new0, raw)
    torch.cuda.synchronize()
    t = np.arange(n)
    old = np.zeros(n, dtype=np.int64) if raw else old0 + t
    want = O.rerope_keys(W.bf16_bits_to_f64(k_bits), old, new0 + t, theta)
    assert_close(f64_of(ko), want, "rerope chunk", rel_l2=2.5e-3)
    assert np.array_equal(bits_of(vo), v_bits)


@pytest.mark.parametrize("Hkv,D,style,in_place", [(8, 128, 0, True), (8, 128, 0, False), (2, 64, 1, True), (3, 64, 0, False)])
def test_rerope_keys_skip_leaves_the_recompute_set_alone(Hkv, D, style, in_place):
    """Rows of the skip list are neither read nor written; every other row is rotated as by
    ct_rerope_keys.  The list has dense runs, isolated rows, the first and the last row."""
    n = 5000 + 13
    rng = np.random.default_rng([18, Hkv, D, style])
    k_bits = W.f32_to_bf16_bits(rng.standard_normal((n, Hkv, D), dtype=np.float32))
    old = rng.integers(0, 4096, n).astype(np.int32)
    new = rng.integers(0, 131072, n).astype(np.int32)
    skip = np.unique(np.concatenate([[0, n - 1], np.arange(100, 420), np.arange(2047, 2050),
                                     rng.choice(n, 600, replace=False)])).astype(np.int32)
    k_bits[skip] = 0x7FC0                       # whatever stands in skipped rows must not matter ...
    cfg = B.make_cfg(Hkv * D * 2, Hkv * 2, Hkv, D, 5e5, style)
    say(f"rerope with skip list Hkv={Hkv} D={D} style={style} in_place={in_place} n={n} n_skip={skip.size}")
    k = dev_bf16(k_bits)
    out = k if in_place else torch.full_like(k, -7.0)
    B.ct_rerope_keys_skip(cfg, k, out, dev_i32(old), dev_i32(new), n, dev_i32(skip), skip.size)
    torch.cuda.synchronize()
    keep = np.setdiff1d(np.arange(n), skip)
    want = O.rerope_keys(W.bf16_bits_to_f64(k_bits[keep]), old[keep], new[keep], 5e5, style)
    # one rounding to bf16 per element: 2^-9 relative on average rows, up to 2^-8 for a row whose
    # elements all sit at the bottom of their binades; short rows (3 x 64) scatter more than long ones
    assert_close(f64_of(out)[keep], want, "rerope (kept rows)", rel_l2=3e-3)
    got_skip = bits_of(out)[skip]               # ... and those rows are not written
    assert np.array_equal(got_skip, k_bits[skip] if in_place else np.full_like(got_skip, 0xC0E0))
    # an empty list is ct_rerope_keys
    a, b = torch.empty_like(k), torch.empty_like(k)
    k2 = dev_bf16(W.f32_to_bf16_bits(rng.standard_normal((n, Hkv, D), dtype=np.float32)))
    B.ct_rerope_keys_skip(cfg, k2, a, dev_i32(old), dev_i32(new), n, None, 0)
    B.ct_rerope_keys(cfg, k2, b, dev_i32(old), dev_i32(new), n)
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))


# ------------------------------------------------------------------------------ scatter
@pytest.mark.parametrize("Hkv,D", [(2, 64), (8, 128)])
def test_scatter_bit_exact(Hkv, D):
    n_ctx, n_sel = 3001, 457
    rng = np.random.default_rng([13, Hkv])
    kb = rng.integers(0, 65536, (n_ctx, Hkv, D)).astype(np.uint16)     # any bit pattern, NaNs included
    vb = rng.integers(0, 65536, (n_ctx, Hkv, D)).astype(np.uint16)
    ks = rng.integers(0, 65536, (n_sel, Hkv, D)).astype(np.uint16)
    vs = rng.integers(0, 65536, (n_sel, Hkv, D)).astype(np.uint16)
    sel = np.sort(rng.choice(n_ctx, n_sel, replace=False)).astype(np.int32)
    sel[0], sel[-1] = 0, n_ctx - 1
    sel = np.unique(sel).astype(np.int32)
    n_sel = sel.size
    ks, vs = ks[:n_sel], vs[:n_sel]
    cfg = B.make_cfg(Hkv * D * 2, Hkv * 2, Hkv, D, 1e4)
    say(f"scatter Hkv={Hkv} D={D}")
    k, v = dev_bf16(kb), dev_bf16(vb)
    B.ct_scatter_kv(cfg, k, v, n_ctx, dev_bf16(ks), dev_bf16(vs), dev_i32(sel), n_sel)
    torch.cuda.synchronize()
    k_want, v_want = O.scatter_kv(kb, vb, ks, vs, sel)
    assert np.array_equal(bits_of(k), k_want)
    assert np.array_equal(bits_of(v), v_want)


# ------------------------------------------------------------------------------ QKV projection
@pytest.mark.parametrize("E,Hq,Hkv,D,theta,style,n_rows,n_sel,bias", [
    (512, 8, 2, 64, 1e4, 0, 1024, 153, False),       # config-1 shape
    (512, 8, 2, 64, 1e4, 1, 300, 300, True),         # interleaved pairs, bias, all rows
    (1024, 8, 2, 128, 5e5, 0, 700, 333, True),       # ragged tile tails
    (1024, 6, 3, 64, 1e4, 0, 400, 129, False),       # odd head counts: k/v boundary inside a 128-feature tile
    (4096, 32, 8, 128, 5e5, 0, 600, 257, False),     # Llama-3-8B layer shape
])
def test_qkv_selected(E, Hq, Hkv, D, theta, style, n_rows, n_sel, bias):
    sh = _shape(E, Hq, Hkv, D, theta, style)
    rng = np.random.default_rng([14, E, Hq, n_sel])
    hid = W.f32_to_bf16_bits(rng.standard_normal((n_rows, E), dtype=np.float32))
    wq = W.f32_to_bf16_bits(rng.standard_normal((sh.qkv_width, E), dtype=np.float32) / np.float32(math.sqrt(E)))
    bs = W.f32_to_bf16_bits(rng.standard_normal(sh.qkv_width, dtype=np.float32) * np.float32(0.5)) if bias else None
    rows = np.sort(rng.choice(n_rows, n_sel, replace=False)).astype(np.int32)
    pos = (rows.astype(np.int64) * 37 + 5).astype(np.int32)           # positions up to ~4e4
    pos[-1] = 131071
    cfg = B.cfg_from_shape(sh)
    say(f"qkv E={E} Hq={Hq} Hkv={Hkv} D={D} style={style} n_sel={n_sel} bias={bias}")
    q = torch.zeros((n_sel, Hq, D), dtype=torch.bfloat16, device="cuda")
    k = torch.zeros((n_sel, Hkv, D), dtype=torch.bfloat16, device="cuda")
    v = torch.zeros((n_sel, Hkv, D), dtype=torch.bfloat16, device="cuda")
    B.ct_qkv_selected(cfg, dev_bf16(hid), dev_i32(rows), dev_i32(pos), n_sel, dev_bf16(wq),
                      None if bs is None else dev_bf16(bs), q, k, v)
    torch.cuda.synchronize()
    qw, kw, vw = O.qkv_selected(W.bf16_bits_to_f64(hid[rows]), W.bf16_bits_to_f64(wq),
                                None if bs is None else W.bf16_bits_to_f64(bs), pos, Hq, Hkv, D, theta, style)
    assert_close(f64_of(q), qw, "q")
    assert_close(f64_of(k), kw, "k")
    assert_close(f64_of(v), vw, "v")
    # compact hidden (hidden_rows = NULL) gives the same bits
    q2, k2, v2 = torch.zeros_like(q), torch.zeros_like(k), torch.zeros_like(v)
    B.ct_qkv_selected(cfg, dev_bf16(hid[rows]), None, dev_i32(pos), n_sel, dev_bf16(wq),
                      None if bs is None else dev_bf16(bs), q2, k2, v2)
    torch.cuda.synchronize()
    assert torch.equal(q, q2) and torch.equal(k, k2) and torch.equal(v, v2)


# ------------------------------------------------------------------------------ selected attention
def _attention_case(Hq, Hkv, D, n_ctx, sel, seed, rows=None, want_split=None, trend=0.0):
    rng = np.random.default_rng([15, seed])
    n_sel = sel.size
    q = rng.standard_normal((n_sel, Hq, D), dtype=np.float32)
    k = rng.standard_normal((n_ctx, Hkv, D), dtype=np.float32)
    if trend != 0.0:
        # scores that drift along the keys: every query gets a component along one direction u
        # and key j the component trend * j / n_ctx along it
        u = rng.standard_normal(D).astype(np.float32)
        u /= np.linalg.norm(u)
        q += 4.0 * u
        k += (trend * np.arange(n_ctx, dtype=np.float32) / n_ctx)[:, None, None] * u
    qb = W.f32_to_bf16_bits(q)
    kb = W.f32_to_bf16_bits(k)
    vb = W.f32_to_bf16_bits(rng.standard_normal((n_ctx, Hkv, D), dtype=np.float32))
    cfg = B.make_cfg(Hq * D, Hq, Hkv, D, 1e4)
    ws_bytes = B.ct_workspace_bytes(cfg, n_ctx, n_sel)
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device="cuda")
    say(f"attention Hq={Hq} Hkv={Hkv} D={D} n_ctx={n_ctx} n_sel={n_sel} ws={ws_bytes}")
    out = torch.full((n_sel, Hq, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    lse = torch.full((n_sel, Hq), float("nan"), dtype=torch.float32, device="cuda")
    B.ct_selected_attention(cfg, dev_bf16(qb), dev_bf16(kb), dev_bf16(vb), n_ctx, dev_i32(sel), n_sel, out, lse,
                            ws, ws_bytes)
    torch.cuda.synchronize()
    want, want_lse = O.selected_attention(W.bf16_bits_to_f64(qb), W.bf16_bits_to_f64(kb), W.bf16_bits_to_f64(vb),
                                          sel, rows=rows)
    got = f64_of(out)
    got_lse = lse.cpu().numpy().astype(np.float64)
    if rows is not None:
        assert np.isfinite(got).all()
        got, got_lse = got[rows], got_lse[rows]
    assert_close(got, want, "attention out")
    assert np.max(np.abs(got_lse - want_lse)) <= 2e-2, np.max(np.abs(got_lse - want_lse))


@pytest.mark.parametrize("Hq,Hkv,D,n_ctx,n_sel,seed", [
    (8, 2, 64, 1024, 153, 1),        # config-1 shape
    (8, 2, 64, 1000, 1000, 2),       # r = 100 %, ragged key tail (not a multiple of 64)
    (32, 8, 128, 2048, 307, 3),      # Llama head layout
    (4, 4, 128, 700, 50, 4),         # G = 1: 256-token tiles
    (16, 2, 128, 900, 77, 5),        # G = 8: 32-token tiles
    (4, 2, 128, 1500, 300, 8),       # G = 2: 128-token tiles
    (16, 1, 64, 1100, 40, 9),        # G = 16: 16-token tiles, one KV head
    (32, 2, 128, 3000, 90, 10),      # G = 16, D = 128, several tiles
    (32, 8, 128, 777, 1, 6),         # a single selected row
    (32, 8, 128, 8192, 400, 7),      # few tiles, long context -> key-range splits + merge
])
def test_selected_attention(Hq, Hkv, D, n_ctx, n_sel, seed):
    rng = np.random.default_rng([16, seed])
    sel = np.arange(n_ctx, dtype=np.int32) if n_sel == n_ctx else \
        np.sort(rng.choice(n_ctx, n_sel, replace=False)).astype(np.int32)
    if n_sel > 2:
        sel[0] = 0                    # a query that sees exactly one key
        sel = np.unique(sel).astype(np.int32)
    _attention_case(Hq, Hkv, D, n_ctx, sel, seed)


def test_selected_attention_clustered_rows():
    """Dense runs of selected rows next to sparse ones (the long-context selection pattern)."""
    n_ctx = 4096
    sel = np.unique(np.concatenate([np.arange(0, 64), np.arange(1000, 1128), [2000, 3000, 4095]])).astype(np.int32)
    _attention_case(32, 8, 128, n_ctx, sel, 21)


@pytest.mark.parametrize("trend", [113.0, -113.0])
def test_selected_attention_drifting_maximum(trend):
    """Scores that rise (or fall) by about 40 over the context, a little per key tile: the running
    maximum moves in most tiles by much less than the step at which the kernel moves its exponent
    reference, so probabilities above one and a lagging reference are exercised, on rows with
    and without key-range splits."""
    rng = np.random.default_rng([17, int(abs(trend))])
    for n_ctx, n_sel in ((4096, 300), (8192, 200)):
        sel = np.sort(rng.choice(n_ctx, n_sel, replace=False)).astype(np.int32)
        sel[-1] = n_ctx - 1
        _attention_case(32, 8, 128, n_ctx, np.unique(sel).astype(np.int32), 31, trend=trend)


# ------------------------------------------------------------------------------ whole layer
def _run_layer(wl, pinned=False, poison=True, in_place=False, pageable=False, compact=False, mixed=False, state=False,
               raw=False):
    """raw: the pool holds keys cached before RoPE (the paper's own scheme, Eq. 8): chunks are
    passed with raw_keys = 1 and the oracle rotates from position 0."""
    sp, sh = wl.spec, wl.spec.shape
    n_chunks = len(wl.chunk_rows) - 1
    cfg = B.cfg_from_shape(sh)
    n_ctx, n_sel = sp.n_ctx, sp.n_sel
    hidden = dev_bf16(wl.hidden)
    rows = None if wl.hidden_rows is None else dev_i32(wl.hidden_rows)
    wqkv = dev_bf16(wl.wqkv)
    sel = dev_i32(wl.sel_idx)
    k_cache, v_cache = wl.k_cache.copy(), wl.v_cache.copy()
    if poison:                        # stale K/V at the selected slots must never be read
        k_cache[wl.sel_idx] = 0x7FC0
        v_cache[wl.sel_idx] = 0x7FC0
    fill = float("nan") if poison else 0.0
    k_buf = torch.full((n_ctx, sh.n_kv_heads, sh.head_dim), fill, dtype=torch.bfloat16, device="cuda")
    v_buf = torch.full((n_ctx, sh.n_kv_heads, sh.head_dim), fill, dtype=torch.bfloat16, device="cuda")
    if pageable:   # ordinary host memory the device cannot address: the library has to copy
        k_pool = torch.from_numpy(np.ascontiguousarray(k_cache).view(np.int16)).view(torch.bfloat16)
        v_pool = torch.from_numpy(np.ascontiguousarray(v_cache).view(np.int16)).view(torch.bfloat16)
        pinned = True
    elif pinned or mixed:
        k_pool, v_pool = pinned_bf16(k_cache), pinned_bf16(v_cache)
        if mixed:   # every third chunk stays on the device, the others come from pinned host memory
            k_dev, v_dev = dev_bf16(k_cache), dev_bf16(v_cache)
    elif in_place:
        k_buf.copy_(dev_bf16(k_cache)); v_buf.copy_(dev_bf16(v_cache))
        k_pool, v_pool = k_buf, v_buf
    else:
        k_pool, v_pool = dev_bf16(k_cache), dev_bf16(v_cache)
    entries, keep_alive = [], []
    for c in range(n_chunks):
        lo, hi = int(wl.chunk_rows[c]), int(wl.chunk_rows[c + 1])
        if compact:   # the pool dropped the recompute set: only the other rows of the chunk, in order
            kept = np.setdiff1d(np.arange(lo, hi), wl.sel_idx)
            kc, vc = pinned_bf16(k_cache[kept]), pinned_bf16(v_cache[kept])
            keep_alive.append((kc, vc))
            entries.append(dict(k=kc, v=vc, n_tokens=hi - lo, old_pos_start=int(wl.chunk_old_start[c]),
                                new_pos_start=int(wl.chunk_new_start[c]), location=2, raw_keys=int(raw)))
            continue
        on_device = mixed and c % 3 == 1
        entries.append(dict(k=(k_dev if on_device else k_pool)[lo:hi], v=(v_dev if on_device else v_pool)[lo:hi],
                            n_tokens=hi - lo, old_pos_start=int(wl.chunk_old_start[c]),
                            new_pos_start=int(wl.chunk_new_start[c]),
                            location=0 if on_device else (1 if (pinned or mixed) else 0), raw_keys=int(raw)))
    chunks = B.make_chunks(entries)
    ws_bytes = B.ct_workspace_bytes(cfg, n_ctx, n_sel)
    if state:      # room for the running (O, max, sum): attention follows the chunk groups key range by key range
        ws_bytes += B.ct_attention_state_bytes(cfg, n_ctx, n_sel)
    ws = torch.full((max(ws_bytes, 256),), 0xff, dtype=torch.uint8, device="cuda")     # NaN patterns wherever read as fp32
    out = torch.full((n_sel, sh.n_q_heads, sh.head_dim), float("nan"), dtype=torch.bfloat16, device="cuda")
    compute, copy = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    say(f"layer {sp.name} n_ctx={n_ctx} n_sel={n_sel} chunks={n_chunks} pinned={pinned} pageable={pageable} "
        f"compact={compact} mixed={mixed} in_place={in_place} raw={raw} state={state} ws={ws_bytes}")
    B.ct_partial_prefill_layer(cfg, chunks, n_chunks, hidden, rows, sel, n_sel, sp.ratio_pct / 100.0, wqkv, None,
                               k_buf, v_buf, out, ws, ws_bytes, compute, copy)
    torch.cuda.synchronize()
    return out, k_buf, v_buf


def _oracle_layer(wl, rows=None, raw=False):
    sh = wl.spec.shape
    hid = W.bf16_bits_to_f64(wl.hidden if wl.hidden_rows is None else wl.hidden[wl.hidden_rows])
    old_pos = np.zeros_like(wl.old_pos) if raw else wl.old_pos     # a raw cache: keys never rotated
    return O.partial_prefill_layer(hid, W.bf16_bits_to_f64(wl.wqkv), None, W.bf16_bits_to_f64(wl.k_cache),
                                   W.bf16_bits_to_f64(wl.v_cache), old_pos, wl.new_pos, wl.sel_idx,
                                   sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.rope_theta, sh.rope_style, rows=rows)


def _check_layer(wl, out, k_buf, v_buf, rows=None, raw=False):
    want, _, k_want, v_want = _oracle_layer(wl, rows=rows, raw=raw)
    got = f64_of(out)
    assert np.isfinite(got).all(), "a stale or unwritten row leaked into the attention output"
    assert_close(got if rows is None else got[rows], want, f"{wl.spec.name} attention output")
    assert_close(f64_of(k_buf), k_want, f"{wl.spec.name} fused K")
    # reused values are copies, recomputed values are rounded fp32 results
    reused = np.setdiff1d(np.arange(wl.spec.n_ctx), wl.sel_idx)
    assert np.array_equal(bits_of(v_buf)[reused], wl.v_cache[reused]), "reused V rows must be bit-exact copies"
    assert_close(f64_of(v_buf)[wl.sel_idx], v_want[wl.sel_idx], f"{wl.spec.name} recomputed V")


@pytest.mark.parametrize("mode", ["pool", "in_place", "pinned", "pinned_state", "pageable", "compact", "compact_state"])
def test_layer_config1(mode):
    wl = W.make_workload(W.spec(1))
    state = mode.endswith("_state")      # workspace with room for the attention state
    mode = mode.replace("_state", "")
    out, kb, vb = _run_layer(wl, pinned=mode == "pinned", in_place=mode == "in_place", poison=mode != "in_place",
                             pageable=mode == "pageable", compact=mode == "compact", state=state)
    _check_layer(wl, out, kb, vb)


@pytest.mark.parametrize("mode", ["pool", "in_place", "pinned", "pinned_state", "pageable", "compact", "mixed"])
def test_layer_config1_raw_key_cache(mode):
    """The paper's own cache scheme (Eq. 8): the pool holds keys as they were before RoPE, and
    token t of a chunk is rotated by its global position new_pos_start + t - for a compact pool
    by the position of the row it stands for, not by its place in the pool."""
    wl = W.make_workload(W.spec(1))
    state = mode.endswith("_state")
    mode = mode.replace("_state", "")
    out, kb, vb = _run_layer(wl, pinned=mode == "pinned", in_place=mode == "in_place", poison=mode != "in_place",
                             pageable=mode == "pageable", compact=mode == "compact", mixed=mode == "mixed", state=state,
                             raw=True)
    _check_layer(wl, out, kb, vb, raw=True)


def _ragged_workload(shape, lengths, ratio_pct, seed):
    """A context of chunks of unequal lengths, none a multiple of the attention kernel's 64-key tile."""
    n_ctx = int(sum(lengths))
    wl = W.make_workload(W.custom_spec(f"ragged-{n_ctx}", shape, 1, n_ctx, ratio_pct, seed=seed))
    starts = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
    wl.chunk_rows = starts
    wl.chunk_new_start = starts[:-1].copy()
    wl.chunk_old_start = np.zeros(len(lengths), dtype=np.int32)
    wl.old_pos = np.concatenate([np.arange(n, dtype=np.int32) for n in lengths])   # every chunk cached at 0..len-1
    return wl


@pytest.mark.parametrize("mode", ["pool", "pinned", "pinned_state", "compact_state", "pageable"])
def test_layer_ragged_chunks_tiny(mode):
    """Chunks of 200 / 333 / 491 / ... tokens: with room for the attention state the launches end at
    chunk-group boundaries inside a 64-key tile, while the rows behind the boundary are still NaN."""
    wl = _ragged_workload(W.TINY, [200, 333, 491, 157, 400, 419], 15, seed=41)
    state = mode.endswith("_state")
    mode = mode.replace("_state", "")
    out, kb, vb = _run_layer(wl, pinned=mode == "pinned", pageable=mode == "pageable", compact=mode == "compact", state=state)
    _check_layer(wl, out, kb, vb)


@pytest.mark.parametrize("state", [False, True])
def test_layer_ragged_chunks_attention_follows_the_groups(state):
    """Llama head layout, 13 chunks of odd lengths in pinned host memory, r = 50 %: enough (tile,
    head) pairs (400) for one attention launch per group of chunks, tile by tile or - with the state -
    key range by key range; group ends fall inside 64-key tiles, and the buffers start as NaN."""
    lengths = [491, 333, 777, 200, 613, 509, 387, 451, 702, 299, 555, 641, 442]
    assert sum(lengths) == 6400
    wl = _ragged_workload(W.LLAMA3_8B, lengths, 50, seed=42)
    out, kb, vb = _run_layer(wl, pinned=True, state=state)
    ends = np.cumsum(lengths)
    near = np.flatnonzero(np.min(np.abs(wl.sel_idx[:, None] - ends[None, :]), axis=1) < 40)   # rows at the chunk boundaries
    rows = np.unique(np.concatenate([W.sample_rows(wl.spec.n_sel, 96, seed=42), near[::3][:64]]))
    _check_layer(wl, out, kb, vb, rows=rows)
    assert torch.isfinite(out.float()).all()


@pytest.mark.parametrize("ratio", [100, 0])
def test_layer_config1_ratio_edges(ratio):
    """r = 100 % is ordinary full causal prefill; r = 0 is full KV reuse (buffers only)."""
    sp = W.spec(1, ratio) if ratio else W.custom_spec("cfg1-r0", W.TINY, 4, 256, 0)
    wl = W.make_workload(sp)
    out, kb, vb = _run_layer(wl, poison=ratio != 0)
    if ratio:
        _check_layer(wl, out, kb, vb)
    else:
        k_want = O.rerope_keys(W.bf16_bits_to_f64(wl.k_cache), wl.old_pos, wl.new_pos, sp.shape.rope_theta)
        assert_close(f64_of(kb), k_want, "full reuse fused K", rel_l2=2.5e-3)
        assert np.array_equal(bits_of(vb), wl.v_cache)


def test_layer_config2():
    wl = W.make_workload(W.spec(2))
    out, kb, vb = _run_layer(wl)
    _check_layer(wl, out, kb, vb)


def test_layer_call_can_be_captured_in_a_hip_graph():
    """The layer call with a device-resident pool only enqueues kernels on the caller's stream (no
    allocation, no synchronisation, no memset), so a caller may capture it.  The graph is replayed
    three times with eager work and synchronisation between the replays and with the outputs wiped
    before each; every replay must give the bits of the eager call, which the oracle bounds."""
    wl = W.make_workload(W.spec(2))
    sp, sh = wl.spec, wl.spec.shape
    cfg = B.cfg_from_shape(sh)
    n_ctx, n_sel, n_chunks = sp.n_ctx, sp.n_sel, len(wl.chunk_rows) - 1
    hidden, wqkv, sel = dev_bf16(wl.hidden), dev_bf16(wl.wqkv), dev_i32(wl.sel_idx)
    rows = None if wl.hidden_rows is None else dev_i32(wl.hidden_rows)
    k_pool, v_pool = dev_bf16(wl.k_cache), dev_bf16(wl.v_cache)
    k_buf = torch.zeros((n_ctx, sh.n_kv_heads, sh.head_dim), dtype=torch.bfloat16, device="cuda")
    v_buf = torch.zeros_like(k_buf)
    chunks = B.make_chunks([dict(k=k_pool[int(wl.chunk_rows[c]):int(wl.chunk_rows[c + 1])],
                                 v=v_pool[int(wl.chunk_rows[c]):int(wl.chunk_rows[c + 1])],
                                 n_tokens=int(wl.chunk_rows[c + 1] - wl.chunk_rows[c]), old_pos_start=int(wl.chunk_old_start[c]),
                                 new_pos_start=int(wl.chunk_new_start[c]), location=0) for c in range(n_chunks)])
    ws_bytes = B.ct_workspace_bytes(cfg, n_ctx, n_sel)
    ws = torch.zeros(max(ws_bytes, 256), dtype=torch.uint8, device="cuda")
    out = torch.zeros((n_sel, sh.n_q_heads, sh.head_dim), dtype=torch.bfloat16, device="cuda")
    side = torch.cuda.Stream()

    def step(stream):
        B.ct_partial_prefill_layer(cfg, chunks, n_chunks, hidden, rows, sel, n_sel, sp.ratio_pct / 100.0, wqkv, None,
                                   k_buf, v_buf, out, ws, ws_bytes, stream, stream)

    say("layer cfg2, eager call on a side stream")
    step(side)
    torch.cuda.synchronize()
    want_out, want_k, want_v = out.clone(), k_buf.clone(), v_buf.clone()
    _check_layer(wl, want_out, want_k, want_v)
    say("layer cfg2, capture")
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step(torch.cuda.current_stream())
    for replay in range(3):
        out.fill_(float("nan")); k_buf.fill_(float("nan")); v_buf.fill_(float("nan")); ws.fill_(0xff)
        torch.cuda.synchronize()
        say(f"layer cfg2, graph replay {replay}")
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), want_out.view(torch.int16)), f"replay {replay}: attention output differs"
        assert torch.equal(k_buf.view(torch.int16), want_k.view(torch.int16)), f"replay {replay}: fused K differs"
        assert torch.equal(v_buf.view(torch.int16), want_v.view(torch.int16)), f"replay {replay}: fused V differs"
        step(side)                                     # eager work of the same kind between the replays
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), want_out.view(torch.int16))
