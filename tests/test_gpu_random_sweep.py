"""Seeded random sweeps over shapes and launch geometries that the hand-picked parity cases do not
name: attention (head dims, group sizes, context lengths around the 64-key tile, selection
patterns), the layer call (ragged chunk lengths, every pool mode, raw and rotated key caches) and
the offline scores (lengths of the form 2^a 3^b 5^c on both sides of the in-LDS limit).  Every case
is a valid input and is compared with the oracle at the bounds of the parity tests; buffers hold
NaN wherever nothing may be read."""
import numpy as np
import pytest
import torch

from oracle import ct_oracle as O
from paper_2605_24022_amd import binding as B
from paper_2605_24022_amd import workloads as W
from tests import test_gpu_frequency as TF
from tests import test_gpu_parity as TP
from tests.gpu_util import assert_close, dev_bf16, dev_i32, f64_of, say

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available()
    B.load()
    torch.cuda.set_device(0)


def _selection(rng, n_ctx):
    pattern = str(rng.choice(["uniform", "all", "first", "last", "clustered", "single"]))
    if pattern == "all":
        sel = np.arange(min(n_ctx, 4100))
    elif pattern == "single":
        sel = np.array([int(rng.integers(0, n_ctx))])
    else:
        n_sel = int(max(1, min(n_ctx, rng.integers(1, max(2, min(n_ctx, 3000))))))
        if pattern == "uniform":
            sel = np.sort(rng.choice(n_ctx, n_sel, replace=False))
        elif pattern == "first":
            sel = np.arange(n_sel)
        elif pattern == "last":
            sel = np.arange(n_ctx - n_sel, n_ctx)
        else:
            lo = max(0, int(rng.integers(0, n_ctx)) - n_sel // 2)
            sel = np.arange(lo, min(n_ctx, lo + n_sel))
    return pattern, sel.astype(np.int32)


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_attention_random_shapes(seed):
    rng = np.random.default_rng([7001, seed])
    for case in range(16):
        D = int(rng.choice([64, 128]))
        Hkv = int(rng.choice([1, 2, 4, 8]))
        G = int(rng.choice([1, 2, 4, 8, 16]))
        if Hkv * G > 64:
            G = 64 // Hkv
        Hq = Hkv * G
        n_ctx = int(rng.choice([1, 63, 64, 65, 200, 777, 2048, 2049, 4100, 9000, 20000]))
        pattern, sel = _selection(rng, n_ctx)
        n_sel = sel.size
        cfg = B.make_cfg(hidden=Hq * D, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, rope_theta=1e4)
        q = W.f32_to_bf16_bits(rng.standard_normal((n_sel, Hq, D), dtype=np.float32))
        k = W.f32_to_bf16_bits(rng.standard_normal((n_ctx, Hkv, D), dtype=np.float32))
        v = W.f32_to_bf16_bits(rng.standard_normal((n_ctx, Hkv, D), dtype=np.float32))
        kmax = int(sel[-1]) + 1
        k[kmax:] = 0x7FC0                     # nobody may read beyond the last visible key
        v[kmax:] = 0x7FC0
        out = torch.full((n_sel, Hq, D), float("nan"), dtype=torch.bfloat16, device="cuda")
        lse = torch.full((n_sel, Hq), float("nan"), dtype=torch.float32, device="cuda")
        ws_bytes = max(B.ct_workspace_bytes(cfg, n_ctx, n_sel), 256)
        ws = torch.full((ws_bytes,), 0xff, dtype=torch.uint8, device="cuda")
        say(f"random attention seed={seed} case={case}: D={D} Hq={Hq} Hkv={Hkv} n_ctx={n_ctx} n_sel={n_sel} {pattern}")
        B.ct_selected_attention(cfg, dev_bf16(q), dev_bf16(k), dev_bf16(v), n_ctx, dev_i32(sel), n_sel, out, lse, ws, ws_bytes)
        torch.cuda.synchronize()
        rows = np.arange(n_sel) if n_sel * kmax <= 3_000_000 else \
            np.unique(np.concatenate([[0, n_sel - 1], rng.choice(n_sel, 48)]))
        kz, vz = W.bf16_bits_to_f64(k), W.bf16_bits_to_f64(v)
        kz[kmax:] = 0.0
        vz[kmax:] = 0.0
        want, want_lse = O.selected_attention(W.bf16_bits_to_f64(q), kz, vz, sel, rows=rows)
        assert_close(f64_of(out)[rows], want, f"attention output (seed {seed}, case {case})")
        got_lse = lse.cpu().numpy().astype(np.float64)[rows]
        assert np.isfinite(got_lse).all() and np.abs(got_lse - want_lse).max() <= 2e-2


@pytest.mark.parametrize("seed", [1, 2])
def test_layer_random_chunk_geometry(seed):
    rng = np.random.default_rng([7002, seed])
    for case in range(12):
        shape = W.TINY if rng.random() < 0.6 else W.LLAMA3_8B
        n_chunks = int(rng.integers(1, 14))
        lengths = [int(rng.integers(1, 900)) for _ in range(n_chunks)]
        if shape is W.LLAMA3_8B and sum(lengths) > 5000:
            lengths = [max(1, n // 2) for n in lengths]
        n_ctx = sum(lengths)
        ratio = int(rng.choice([1, 5, 15, 30, 50, 80, 100]))
        if n_ctx * ratio // 100 < 1:
            ratio = 100
        mode = str(rng.choice(["pool", "pinned", "pinned_state", "compact", "compact_state", "pageable", "mixed", "mixed_state"]))
        raw = bool(rng.random() < 0.3)
        wl = TP._ragged_workload(shape, lengths, ratio, seed=1000 * seed + case)
        state = mode.endswith("_state")
        mode = mode.replace("_state", "")
        starts = np.concatenate([[0], np.cumsum(lengths)])
        if mode == "compact" and any(np.isin(np.arange(starts[c], starts[c + 1]), wl.sel_idx).all() for c in range(n_chunks)):
            mode = "pinned"       # a compact chunk that keeps no row has no memory to point at
        say(f"random layer seed={seed} case={case}: lengths={lengths} ratio={ratio} mode={mode} state={state} raw={raw}")
        out, kb, vb = TP._run_layer(wl, pinned=mode == "pinned", pageable=mode == "pageable", compact=mode == "compact",
                                    mixed=mode == "mixed", state=state, raw=raw)
        rows = None if wl.spec.n_sel * n_ctx < 4_000_000 else W.sample_rows(wl.spec.n_sel, 64, seed=case)
        TP._check_layer(wl, out, kb, vb, rows=rows, raw=raw)


def test_frequency_scores_random_lengths():
    rng = np.random.default_rng(7003)
    smooth = sorted({2 ** a * 3 ** b * 5 ** c for a in range(18) for b in range(8) for c in range(6)
                     if 2 ** a * 3 ** b * 5 ** c <= 300000})
    long_ones = [n for n in smooth if n > 4096]
    for case in range(14):
        n = int(rng.choice(smooth if case % 2 == 0 else long_ones))
        row = int(rng.choice([2, 6, 8, 16, 30, 64, 128, 250, 256, 1024]))
        if n * row > 20_000_000:
            row = max(2, (20_000_000 // n) // 2 * 2)
        n_batch = int(rng.integers(1, 4)) if n * row < 4_000_000 else 1
        alpha = float(rng.choice([0.0, 0.01, 0.1, 0.3, 0.5, 0.9, 1.0]))
        assert B.ct_frequency_workspace_bytes(n_batch, n, row) > 0
        say(f"random frequency case={case}: n={n} row={row} batch={n_batch} alpha={alpha}")
        kb, vb = W.make_spectral_kv(5000 + case, n, row, n_batch)
        got = TF._gpu_scores(kb, vb, alpha).cpu().numpy().astype(np.float64)
        want = TF._oracle_scores(kb, vb, alpha)
        assert np.isfinite(got).all()
        bound = TF.SCORE_REL * max(want.max(), 1e-30) if want.max() > 0 else 0.0
        assert np.abs(got - want).max() <= bound, (n, row, alpha)
