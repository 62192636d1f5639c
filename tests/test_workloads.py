"""Host-side checks of the seeded input generators (no method arithmetic involved)."""
import numpy as np
import torch

from paper_2605_24022_amd import workloads as W


def test_bf16_rounding_matches_library_conversion():
    x = np.random.default_rng(3).standard_normal(200000, dtype=np.float32) * 7
    x[:5] = [0.0, -0.0, 1.00390625, 1.01171875, 3.4e38]
    ours = W.f32_to_bf16_bits(x)
    lib = torch.tensor(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, lib)
    assert np.array_equal(W.bf16_bits_to_f32(ours), torch.tensor(x).to(torch.bfloat16).float().numpy())


def test_selected_counts_follow_floor_rule():
    assert W.spec(1).n_sel == 153
    assert W.spec(2).n_sel == 1228
    assert [W.spec(3, r).n_sel for r in (5, 10, 15, 30, 100)] == [1638, 3276, 4915, 9830, 32768]
    assert W.spec(4).n_sel == 6553


def test_index_sets_are_sorted_unique_in_range_and_reproducible():
    for c in (1, 2, 3, 4):
        sp = W.spec(c)
        s = W.select_indices(sp)
        assert s.dtype == np.int32 and s.size == sp.n_sel
        assert (np.diff(s) > 0).all() and s[0] >= 0 and s[-1] < sp.n_ctx
        assert np.array_equal(s, W.select_indices(sp))


def test_forced_and_clustered_structure():
    sp = W.spec(2)
    s = set(W.select_indices(sp).tolist())
    for c in range(sp.n_chunks):
        assert all(c * sp.chunk_len + t in s for t in range(16))
    sp = W.spec(4)
    s = W.select_indices(sp)
    off = s % sp.chunk_len
    near = (off < 64) | (off >= sp.chunk_len - 64)
    assert near.sum() == 32 * 128          # the whole boundary pool (62.5 % of the budget)


def test_tiny_workload_shapes():
    w = W.make_workload(W.spec(1))
    assert w.hidden.shape == (1024, 512) and w.wqkv.shape == (768, 512)
    assert w.k_cache.shape == (1024, 2, 64) and w.k_cache.dtype == np.uint16
    assert np.array_equal(w.old_pos[:300], np.arange(300) % 256)
    assert np.array_equal(w.sel_pos, w.sel_idx)
