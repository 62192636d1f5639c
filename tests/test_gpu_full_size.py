"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.
The oracle evaluates a seeded sample of the selected rows (every output row depends on no
other query, so sampled rows are checked exactly) plus the whole fused K/V cache."""
import numpy as np
import pytest
import torch

from paper_2605_24022_amd import workloads as W
from tests.gpu_util import say
from tests.test_gpu_parity import _check_layer, _run_layer

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available()
    torch.cuda.set_device(0)


@pytest.mark.parametrize("ratio", [15, 5])
def test_layer_config3_sampled_rows(ratio):
    """32768-token context; r = 15 % is the headline point, r = 5 % exercises key-range splits."""
    wl = W.make_workload(W.spec(3, ratio))
    out, kb, vb = _run_layer(wl)
    rows = W.sample_rows(wl.spec.n_sel, 192, seed=ratio)
    say(f"oracle on {len(rows)} sampled rows of {wl.spec.n_sel}")
    _check_layer(wl, out, kb, vb, rows=rows)


def test_layer_config3_full_recompute_equals_full_prefill():
    """r = 100 %: every row is recomputed; the cache pool is poisoned and must not matter."""
    wl = W.make_workload(W.spec(3, 100))
    out, kb, vb = _run_layer(wl)
    rows = W.sample_rows(wl.spec.n_sel, 96, seed=100)
    _check_layer(wl, out, kb, vb, rows=rows)


@pytest.mark.parametrize("state", [False, True])
def test_layer_config4_pinned_host_chunks_clustered_rows(state):
    """131072-token context streamed from pinned host memory on a second stream, clustered rows;
    attention tile by tile as the chunk groups land, or (with room for its state) key range by key
    range."""
    wl = W.make_workload(W.spec(4))
    out, kb, vb = _run_layer(wl, pinned=True, state=state)
    rows = W.sample_rows(wl.spec.n_sel, 64, seed=4)
    _check_layer(wl, out, kb, vb, rows=rows)


@pytest.mark.parametrize("state", [False, True])
@pytest.mark.parametrize("pool", ["pinned", "mixed", "compact"])
def test_layer_config3_host_pools_attention_follows_the_chunk_groups(pool, state):
    """Config 3 at r = 15 % with the cached K/V outside the device: 16 chunks stream in in
    groups and one attention launch per group computes the rows that group completes (or, with
    room for the attention state, takes every unfinished row through that group's keys).  Pinned
    pool, a pool with every third chunk on the device, and a compact pool (reused rows only)."""
    wl = W.make_workload(W.spec(3, 15))
    out, kb, vb = _run_layer(wl, pinned=pool == "pinned", mixed=pool == "mixed", compact=pool == "compact", state=state)
    rows = W.sample_rows(wl.spec.n_sel, 192, seed=33)
    _check_layer(wl, out, kb, vb, rows=rows)
    assert torch.isfinite(out.float()).all()        # every tile was computed by exactly one of the launches


def test_layer_config2_compact_host_pool():
    """8192-token context, forced + uniform rows; the host pool holds only the rows that are reused."""
    wl = W.make_workload(W.spec(2))
    out, kb, vb = _run_layer(wl, compact=True)
    _check_layer(wl, out, kb, vb)


def test_stack_config5_one_layer_sampled_rows():
    """One layer of the config-5 stack at its full shape (hidden 4096, FFN 14336, 32768-token
    context, r = 15 %, cached K/V in pinned host memory) through ct_partial_prefill_stack.  The
    oracle computes Q, K, V of all selected rows and the whole fused cache, then attention, output
    projection and FFN for a sample of rows (the rest of the layer is row-wise)."""
    from oracle import ct_oracle as O
    from tests.gpu_util import assert_close, f64_of
    from tests.test_gpu_stack import _run_stack

    sp = W.spec(5)
    sh = sp.shape
    sw = W.make_stack_workload(sp, n_layers=1, ffn_dim=14336)
    h = _run_stack(sw, sw.hidden0, pinned=True)
    lw = {k: W.bf16_bits_to_f64(v) for k, v in sw.layers[0].items()}
    rows = W.sample_rows(sp.n_sel, 64, seed=5)
    say(f"oracle: projections of {sp.n_sel} rows, attention and FFN of {len(rows)} sampled rows")
    h0 = W.bf16_bits_to_f64(sw.hidden0)
    x = O.rmsnorm(h0, lw["attn_norm"], sw.rms_eps)
    attn, _, _, _ = O.partial_prefill_layer(x, lw["wqkv"], None, lw["k_cache"], lw["v_cache"], sw.old_pos, sw.new_pos,
                                            sw.sel_idx, sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.rope_theta,
                                            sh.rope_style, rows=rows)
    want = O.layer_tail(h0[rows], attn, lw["wo"], lw["ffn_norm"], lw["w_gate"], lw["w_up"], lw["w_down"], sw.rms_eps)
    assert_close(f64_of(h)[rows], want, "config-5 layer output (sampled rows)", ulp_slack=2.0 ** -8)
