"""The C-ABI library loads without a GPU, exports every symbol the header declares and
rejects bad arguments before it touches HIP."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2605_24022_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000  # a non-NULL address that is never dereferenced by validation


@pytest.fixture(scope="module")
def lib():
    return B.load()


def _cfg(**kw):
    base = dict(hidden=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, rope_theta=5e5)
    base.update(kw)
    return B.make_cfg(**base)


def test_every_declared_symbol_is_exported(lib):
    text = open(os.path.join(ROOT, "include", "cachetune.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(ct_[a-z_]+)\s*\(", text))
    assert declared, "no declarations found"
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None
    assert B.ct_version().startswith("cachetune-gfx950")


def test_struct_layout_matches_header():
    assert ctypes.sizeof(B.LayerCfg) == 32
    assert ctypes.sizeof(B.Chunk) == 40


def _status(fn, *args, **kw):
    with pytest.raises(B.CacheTuneError) as ei:
        fn(*args, **kw)
    assert ei.value.message
    return ei.value.status


def test_cfg_validation():
    for bad, want in [(dict(head_dim=96), B.CT_ERR_UNSUPPORTED), (dict(n_q_heads=30), B.CT_ERR_SHAPE),
                      (dict(n_q_heads=24, n_kv_heads=8), B.CT_ERR_UNSUPPORTED), (dict(hidden=100), B.CT_ERR_UNSUPPORTED),
                      (dict(rope_style=2), B.CT_ERR_UNSUPPORTED), (dict(rope_theta=0.0), B.CT_ERR_SHAPE),
                      (dict(hidden=0), B.CT_ERR_SHAPE)]:
        st = _status(B.ct_rerope_keys, _cfg(**bad), FAKE, FAKE, None, FAKE, 16)
        assert st == want, (bad, st)
    assert B.ct_workspace_bytes(_cfg(head_dim=96), 1024, 10) == 0


def test_null_and_shape_errors():
    c = _cfg()
    assert _status(B.ct_rerope_keys, c, None, FAKE, None, FAKE, 16) == B.CT_ERR_NULL
    assert _status(B.ct_rerope_keys, c, FAKE, FAKE, None, None, 16) == B.CT_ERR_NULL
    assert _status(B.ct_rerope_keys, c, FAKE, FAKE, None, FAKE, -1) == B.CT_ERR_SHAPE
    assert _status(B.ct_rerope_chunk, c, FAKE, FAKE, FAKE, None, 16, 0, 0) == B.CT_ERR_NULL
    assert _status(B.ct_scatter_kv, c, FAKE, None, 64, FAKE, FAKE, FAKE, 4) == B.CT_ERR_NULL
    assert _status(B.ct_scatter_kv, c, FAKE, FAKE, 4, FAKE, FAKE, FAKE, 8) == B.CT_ERR_SHAPE
    assert _status(B.ct_qkv_selected, c, FAKE, None, None, 4, FAKE, None, FAKE, FAKE, FAKE) == B.CT_ERR_NULL
    assert _status(B.ct_qkv_selected, c, FAKE, None, FAKE, -4, FAKE, None, FAKE, FAKE, FAKE) == B.CT_ERR_SHAPE
    assert _status(B.ct_selected_attention, c, FAKE, FAKE, FAKE, 0, FAKE, 4, FAKE, None, None, 0) == B.CT_ERR_SHAPE
    assert _status(B.ct_selected_attention, c, None, FAKE, FAKE, 64, FAKE, 4, FAKE, None, None, 0) == B.CT_ERR_NULL
    # empty work is legal and needs no GPU
    B.ct_rerope_keys(c, None, None, None, None, 0)
    B.ct_scatter_kv(c, None, None, 64, None, None, None, 0)
    B.ct_qkv_selected(c, None, None, None, 0, None, None, None, None, None)
    B.ct_selected_attention(c, None, None, None, 64, None, 0, None, None, None, 0)


def test_extent_limits_are_rejected_on_the_host():
    """32-bit byte offsets and 24-bit row numbers inside the kernels: sizes beyond them are errors."""
    small = B.make_cfg(64, 1, 1, 64, 1e4)                    # 128-byte K/V rows: 2^24 rows stay below 4 GiB
    assert _status(B.ct_selected_attention, small, FAKE, FAKE, FAKE, 1 << 24, FAKE, 4, FAKE, None, FAKE, 1 << 30) \
        == B.CT_ERR_UNSUPPORTED
    c = _cfg()
    assert _status(B.ct_selected_attention, c, FAKE, FAKE, FAKE, 1 << 21, FAKE, 4, FAKE, None, FAKE, 1 << 30) \
        == B.CT_ERR_UNSUPPORTED                                 # 2^21 rows x 2 KiB = 4 GiB
    # compact hidden of n_sel rows x 4096 x 2 bytes beyond 4 GiB
    assert _status(B.ct_qkv_selected, c, FAKE, None, FAKE, 1 << 19, FAKE, None, FAKE, FAKE, FAKE) == B.CT_ERR_UNSUPPORTED
    wide = B.make_cfg(1 << 17, 128, 128, 128, 1e4)            # wqkv of 49152 x 131072 x 2 bytes
    assert _status(B.ct_qkv_selected, wide, FAKE, FAKE, FAKE, 4, FAKE, None, FAKE, FAKE, FAKE) == B.CT_ERR_UNSUPPORTED


def test_rerope_skip_and_planned_linear_validation():
    c = _cfg()
    assert _status(B.ct_rerope_keys_skip, c, FAKE, FAKE, None, FAKE, 16, None, 4) == B.CT_ERR_NULL
    assert _status(B.ct_rerope_keys_skip, c, FAKE, FAKE, None, FAKE, 16, FAKE, 17) == B.CT_ERR_SHAPE
    assert _status(B.ct_rerope_keys_skip, c, FAKE, FAKE, None, FAKE, 16, FAKE, -1) == B.CT_ERR_SHAPE
    assert _status(B.ct_rerope_keys_skip, c, None, FAKE, None, FAKE, 16, FAKE, 4) == B.CT_ERR_NULL
    B.ct_rerope_keys_skip(c, None, None, None, None, 0, None, 0)
    assert _status(B.ct_linear_ws_cus, FAKE, 4, 512, FAKE, 512, None, FAKE, FAKE, 1 << 20, 0) == B.CT_ERR_SHAPE
    assert _status(B.ct_linear_ws_cus, FAKE, 4, 512, FAKE, 512, None, FAKE, FAKE, 1 << 20, 257) == B.CT_ERR_SHAPE
    assert _status(B.ct_linear_ws_cus, FAKE, 4, 512, None, 512, None, FAKE, FAKE, 1 << 20, 224) == B.CT_ERR_NULL
    B.ct_linear_ws_cus(None, 0, 512, None, 512, None, None, None, 0, 224)


def test_static_scratch_entry_point_rejects_on_the_host():
    """ct_selected_attention_static: the same argument checks as ct_selected_attention, and a clear
    error - before any HIP call - for a problem whose scratch does not fit the library's array."""
    c = _cfg()
    assert B.ct_static_scratch_bytes() == 64 << 20
    assert _status(B.ct_selected_attention_static, c, None, FAKE, FAKE, 64, FAKE, 4, FAKE, None) == B.CT_ERR_NULL
    assert _status(B.ct_selected_attention_static, c, FAKE, FAKE, FAKE, 0, FAKE, 4, FAKE, None) == B.CT_ERR_SHAPE
    assert _status(B.ct_selected_attention_static, c, FAKE, FAKE, FAKE, 64, FAKE, 65, FAKE, None) == B.CT_ERR_SHAPE
    with pytest.raises(B.CacheTuneError) as e:      # 376 (tile, head) pairs split in two: 100 MB of partials
        B.ct_selected_attention_static(c, FAKE, FAKE, FAKE, 65536, FAKE, 3000, FAKE, None)
    assert e.value.status == B.CT_ERR_WORKSPACE and "static" in e.value.message
    B.ct_selected_attention_static(c, None, None, None, 64, None, 0, None, None)     # empty work is legal


def test_attention_launches_over_ragged_chunk_groups_stay_inside_their_key_range():
    """Sec. 4.2, chunk-wise overlap: the attention launch that follows a group of host chunks may read
    no key row of a later group (it may still be on the host link).  The host replay of the kernel's
    tile loads says which rows a launch reads; group ends that are no multiple of the 64-key tile are
    the case that matters.  Also: every row a launch needs is read, and argument errors are reported."""
    c = _cfg()
    rng = np.random.default_rng(7)
    n_ctx = 200 + 333 + 491 + 1000
    ends = [200, 533, 1024, n_ctx]                      # ragged group ends
    for n_sel in (1, 37, 300, n_ctx):
        sel = np.sort(rng.choice(n_ctx, n_sel, replace=False)).astype(np.int32)
        for with_state in (False, True):
            seen = 0
            for upto in ends:
                lo, hi = B.ct_attention_rows_read(c, sel, n_sel, n_ctx, seen, upto, with_state)
                # tiles of 256 / G = 64 selected rows; the last row of a tile decides what the tile sees
                lasts = np.array([sel[min(t + 64, n_sel) - 1] for t in range(0, n_sel, 64)])
                if with_state:
                    active = lasts >= seen                  # every tile that sees keys past `seen`
                    want_hi = min(upto, lasts[active].max() + 1) - 1 if active.any() else -1
                    want_lo = seen if active.any() else -1
                else:
                    active = (lasts >= seen) & (lasts < upto)
                    want_hi = lasts[active].max() if active.any() else -1
                    want_lo = 0 if active.any() else -1
                assert (lo, hi) == (want_lo, want_hi), (n_sel, with_state, seen, upto)
                assert hi < upto
                seen = upto
    sel = np.arange(8, dtype=np.int32)
    assert _status(B.ct_attention_rows_read, c, None, 8, 64, 0, 64, False) == B.CT_ERR_NULL
    assert _status(B.ct_attention_rows_read, c, sel, 8, 64, 10, 10, False) == B.CT_ERR_SHAPE
    assert _status(B.ct_attention_rows_read, c, sel[::-1].copy(), 8, 64, 0, 64, False) == B.CT_ERR_INDEX


def test_attention_workspace_checks():
    c = _cfg()
    need = B.ct_workspace_bytes(c, 32768, 1638)   # few tiles -> split keys -> partials in the workspace
    assert need > 0
    assert _status(B.ct_selected_attention, c, FAKE, FAKE, FAKE, 32768, FAKE, 1638, FAKE, None, None, 0) \
        == B.CT_ERR_WORKSPACE
    assert _status(B.ct_selected_attention, c, FAKE, FAKE, FAKE, 32768, FAKE, 1638, FAKE, None, FAKE, 1024) \
        == B.CT_ERR_WORKSPACE
    assert _status(B.ct_selected_attention, c, FAKE, FAKE, FAKE, 32768, FAKE, 1638, FAKE, None, FAKE + 8, need) \
        == B.CT_ERR_WORKSPACE


def _chunks(n=4, length=256, **kw):
    return B.make_chunks([dict(k=FAKE, v=FAKE, n_tokens=length, old_pos_start=0, new_pos_start=i * length, **kw)
                          for i in range(n)])


def test_layer_validation():
    c = B.make_cfg(512, 8, 2, 64, 1e4)
    ch = _chunks()
    args = dict(hidden=FAKE, hidden_rows=None, sel_idx=FAKE, n_sel=153, recompute_ratio=0.15, wqkv=FAKE, bias=None,
                k_buf=FAKE, v_buf=FAKE, attn_out=FAKE, workspace=None, workspace_bytes=0)

    def call(chunks=ch, n_chunks=4, **over):
        a = dict(args); a.update(over)
        return _status(B.ct_partial_prefill_layer, c, chunks, n_chunks, a["hidden"], a["hidden_rows"], a["sel_idx"],
                       a["n_sel"], a["recompute_ratio"], a["wqkv"], a["bias"], a["k_buf"], a["v_buf"],
                       a["attn_out"], a["workspace"], a["workspace_bytes"])

    assert call(n_sel=150) == B.CT_ERR_RATIO                 # floor(0.15 * 1024) = 153
    assert call(recompute_ratio=1.5) == B.CT_ERR_RATIO
    assert call() == B.CT_ERR_WORKSPACE                      # ratio fine, workspace missing
    assert call(recompute_ratio=-1.0, n_sel=150) == B.CT_ERR_WORKSPACE   # negative ratio disables the check
    assert call(n_chunks=0) == B.CT_ERR_SHAPE
    assert call(n_chunks=65) == B.CT_ERR_UNSUPPORTED
    assert call(n_sel=2000, recompute_ratio=-1.0) == B.CT_ERR_SHAPE
    assert call(k_buf=None) == B.CT_ERR_NULL
    assert call(hidden=None, workspace=FAKE, workspace_bytes=1 << 30) == B.CT_ERR_NULL
    bad = _chunks(); bad[2].new_pos_start = 100              # overlaps chunk 1 in position
    assert call(chunks=bad) == B.CT_ERR_SHAPE
    bad = _chunks(); bad[1].n_tokens = 0
    assert call(chunks=bad) == B.CT_ERR_SHAPE
    bad = _chunks(); bad[3].k = None
    assert call(chunks=bad) == B.CT_ERR_NULL
    bad = _chunks(); bad[0].location = 3
    assert call(chunks=bad) == B.CT_ERR_SHAPE
    host = _chunks(location=1)                               # pinned-host chunks need a second stream
    need = B.ct_workspace_bytes(c, 1024, 153)
    assert call(chunks=host, workspace=FAKE, workspace_bytes=need) == B.CT_ERR_SHAPE


def test_validate_indices():
    good = np.array([0, 3, 4, 9], dtype=np.int32)
    B.ct_validate_indices(good, 4, 10)
    B.ct_validate_indices(None, 0, 10)
    for bad in ([0, 3, 3, 9], [0, 5, 4, 9], [-1, 3, 4, 9], [0, 3, 4, 10]):
        assert _status(B.ct_validate_indices, np.array(bad, dtype=np.int32), 4, 10) == B.CT_ERR_INDEX
    assert _status(B.ct_validate_indices, good, 4, 3) == B.CT_ERR_SHAPE
    assert _status(B.ct_validate_indices, None, 4, 10) == B.CT_ERR_NULL


def test_workspace_size_covers_staging_and_partials():
    c = _cfg()
    for n_ctx, n_sel in [(8192, 1228), (32768, 4915), (32768, 1638), (131072, 6553)]:
        need = B.ct_workspace_bytes(c, n_ctx, n_sel)
        # q, k, v staging of the layer call must fit
        assert need >= n_sel * (32 + 16) * 128 * 2
        assert need % 256 == 0
    # few (tile, head) pairs -> the key range is split and fp32 partials need room as well
    staging = 1638 * (32 + 16) * 128 * 2
    assert B.ct_workspace_bytes(c, 32768, 1638) > staging + 26 * 8 * 2 * 256 * 128 * 4 - 1
    assert B.ct_workspace_bytes(c, 0, 0) == 0 and B.ct_workspace_bytes(c, 100, 200) == 0
    # the optional attention state: fp32 (O, m, l) of every 256-column tile and KV head
    assert B.ct_attention_state_bytes(c, 32768, 4915) == 77 * 8 * 256 * 130 * 4
    assert B.ct_attention_state_bytes(c, 32768, 0) == 0 and B.ct_attention_state_bytes(c, 100, 200) == 0


def test_norm_and_gemm_validation():
    assert _status(B.ct_rmsnorm, None, FAKE, 1e-5, 4, 512, FAKE) == B.CT_ERR_NULL
    assert _status(B.ct_rmsnorm, FAKE, FAKE, 1e-5, 4, 100, FAKE) == B.CT_ERR_UNSUPPORTED
    assert _status(B.ct_rmsnorm, FAKE, FAKE, -1.0, 4, 512, FAKE) == B.CT_ERR_SHAPE
    assert _status(B.ct_rmsnorm, FAKE, FAKE, 1e-5, -4, 512, FAKE) == B.CT_ERR_SHAPE
    assert _status(B.ct_linear, FAKE, 4, 512, None, 512, None, FAKE) == B.CT_ERR_NULL
    assert _status(B.ct_linear, FAKE, 4, 500, FAKE, 512, None, FAKE) == B.CT_ERR_UNSUPPORTED
    assert _status(B.ct_linear, FAKE, 4, 512, FAKE, 100, None, FAKE) == B.CT_ERR_UNSUPPORTED
    assert _status(B.ct_linear, FAKE, 4, 0, FAKE, 512, None, FAKE) == B.CT_ERR_SHAPE
    assert _status(B.ct_linear, FAKE, 1 << 20, 4096, FAKE, 4096, None, FAKE) == B.CT_ERR_UNSUPPORTED   # > 4 GiB
    assert _status(B.ct_linear_ws, FAKE, 4, 512, None, 512, None, FAKE, FAKE, 1 << 20) == B.CT_ERR_NULL
    assert _status(B.ct_linear_ws, FAKE, 4, 500, FAKE, 512, None, FAKE, FAKE, 1 << 20) == B.CT_ERR_UNSUPPORTED
    assert _status(B.ct_linear_ws, FAKE, 4, 512, FAKE, 512, None, FAKE, FAKE + 4, 1 << 20) == B.CT_ERR_WORKSPACE
    B.ct_linear_ws(None, 0, 512, None, 512, None, None, None, 0)
    # scratch: one fp32 tile per compute unit when the tiles leave a partial round, none for bad sizes
    assert B.ct_linear_workspace_bytes(4915, 14336, 4096) == 256 * 256 * 256 * 4
    assert B.ct_linear_workspace_bytes(100, 4096, 512) == 2 * 8 * 256 * 256 * 4
    assert B.ct_linear_workspace_bytes(0, 4096, 512) == 0 and B.ct_linear_workspace_bytes(16, -1, 512) == 0
    assert _status(B.ct_linear, FAKE + 8, 4, 512, FAKE, 512, None, FAKE) == B.CT_ERR_UNSUPPORTED       # alignment
    assert _status(B.ct_swiglu, FAKE, 4, 512, FAKE, FAKE + 2, 512, FAKE) == B.CT_ERR_UNSUPPORTED
    assert _status(B.ct_swiglu, FAKE, 4, 512, FAKE, None, 512, FAKE) == B.CT_ERR_NULL
    assert _status(B.ct_swiglu, FAKE, 4, 512, FAKE, FAKE, 96, FAKE) == B.CT_ERR_UNSUPPORTED
    # empty work is legal and needs no GPU
    B.ct_rmsnorm(None, None, 1e-5, 0, 512, None)
    B.ct_linear(None, 0, 512, None, 512, None, None)
    B.ct_swiglu(None, 0, 512, None, None, 512, None)


def test_mfma_rate_validation():
    assert _status(B.ct_measure_mfma_rate, None, 100) == B.CT_ERR_NULL
    assert _status(B.ct_measure_mfma_rate, FAKE, 0) == B.CT_ERR_SHAPE


def _layers(n_layers=2, n_chunks=4, length=256, **kw):
    entries = []
    for _ in range(n_layers):
        entries.append(dict(attn_norm=FAKE, wqkv=FAKE, wo=FAKE, ffn_norm=FAKE, w_gate=FAKE, w_up=FAKE, w_down=FAKE,
                            chunks=_chunks(n_chunks, length, **kw)))
    return entries


def test_stack_validation():
    assert ctypes.sizeof(B.LayerWeights) == 64
    c = B.make_cfg(512, 8, 2, 64, 1e4)
    need = B.ct_stack_workspace_bytes(c, 1536, 1024, 153)
    assert need > B.ct_workspace_bytes(c, 1024, 153) and need % 256 == 0
    assert B.ct_stack_workspace_bytes(c, 0, 1024, 153) == 0
    assert B.ct_stack_workspace_bytes(c, 1536, 100, 200) == 0

    def call(entries=None, n_layers=2, n_chunks=4, ffn=1536, eps=1e-5, hidden=FAKE, sel=FAKE, n_sel=153, ratio=0.15,
             kb=FAKE, vb=FAKE, ws=FAKE + 0xF0, ws_bytes=need, s1=None, s2=None):
        layers = B.make_layers(entries if entries is not None else _layers())
        return _status(B.ct_partial_prefill_stack, c, ffn, eps, layers, n_layers, n_chunks, hidden, sel, n_sel, ratio,
                       kb, vb, ws, ws_bytes, s1, s2)

    assert FAKE + 0xF0 & 255 != 0
    assert call() == B.CT_ERR_WORKSPACE                       # everything fine up to the misaligned workspace
    assert call(ws=None) == B.CT_ERR_WORKSPACE
    assert call(ws=FAKE, ws_bytes=need - 1) == B.CT_ERR_WORKSPACE
    assert call(n_layers=0) == B.CT_ERR_SHAPE
    assert call(n_chunks=0) == B.CT_ERR_SHAPE
    assert call(n_chunks=65) == B.CT_ERR_UNSUPPORTED
    assert call(ffn=1000) == B.CT_ERR_UNSUPPORTED
    assert call(eps=-1.0) == B.CT_ERR_SHAPE
    assert call(n_sel=0, ratio=-1.0) == B.CT_ERR_SHAPE
    assert call(n_sel=2000, ratio=-1.0) == B.CT_ERR_SHAPE
    assert call(n_sel=150) == B.CT_ERR_RATIO
    assert call(hidden=None) == B.CT_ERR_NULL
    assert call(kb=None) == B.CT_ERR_NULL
    bad = _layers(); bad[1]["wo"] = None
    assert call(entries=bad) == B.CT_ERR_NULL
    bad = _layers(); bad[1]["chunks"][2].n_tokens = 128      # geometry differs between layers
    assert call(entries=bad) == B.CT_ERR_SHAPE
    bad = _layers(); bad[0]["chunks"][2].new_pos_start = 100
    assert call(entries=bad) == B.CT_ERR_SHAPE
    bad = _layers(); bad[1]["chunks"][3].v = None
    assert call(entries=bad) == B.CT_ERR_NULL
    # pinned-host chunks need a second stream (both default here)
    assert call(entries=_layers(location=1), ws=FAKE) == B.CT_ERR_SHAPE


def test_frequency_selection_argument_checks():
    """Everything the host can reject is rejected before any HIP call."""
    lib = B.load()
    one = ctypes.c_void_p(256)     # never dereferenced: the checks fail first
    def scores(n_batch=1, stride=2048 * 1024, n=2048, row=1024, alpha=0.5, k=one, v=one, out=one, ws=one, ws_bytes=1 << 30):
        return lib.ct_frequency_scores(k, v, n_batch, stride, n, row, alpha, out, ws, ws_bytes, None)
    assert scores(n=7 * 128) == B.CT_ERR_UNSUPPORTED          # prime factor 7
    # beyond 4096 tokens the transform is split in two factors of at most 4096 each
    assert scores(n=2 * 4099, stride=2 * 4099 * 1024) == B.CT_ERR_UNSUPPORTED       # 4099 is prime
    assert scores(n=1 << 24, stride=(1 << 24) * 1024) == B.CT_ERR_UNSUPPORTED
    assert scores(n=8192, stride=8192 * 1024, ws_bytes=1 << 20) == B.CT_ERR_WORKSPACE
    assert scores(n=8192, stride=8192 * 1024, ws=ctypes.c_void_p(264)) == B.CT_ERR_WORKSPACE   # alignment
    assert scores(row=1023) == B.CT_ERR_SHAPE
    assert scores(alpha=1.5) == B.CT_ERR_RATIO and scores(alpha=-0.1) == B.CT_ERR_RATIO
    assert scores(k=None) == B.CT_ERR_NULL and scores(out=None) == B.CT_ERR_NULL
    assert scores(n_batch=2, stride=100) == B.CT_ERR_SHAPE
    assert scores(ws_bytes=16) == B.CT_ERR_WORKSPACE and scores(ws=None) == B.CT_ERR_WORKSPACE
    assert scores(n_batch=0) == B.CT_OK and scores(n=0) == B.CT_OK
    assert B.ct_frequency_workspace_bytes(1, 2048, 1024) == 2 * 64 * 2048 * 4
    # 8192 = 64 x 128: four strips of 128 complex columns per tensor, and one complex fp32 copy of a tensor
    assert B.ct_frequency_workspace_bytes(1, 8192, 1024) == 2 * 4 * 8192 * 4 + 8192 * 512 * 8
    assert B.ct_frequency_workspace_bytes(1, 2 * 4099, 1024) == 0 and B.ct_frequency_workspace_bytes(1, 7, 8) == 0
    assert lib.ct_topk_indices(one, 1, 10, 11, one, None) == B.CT_ERR_SHAPE
    assert lib.ct_topk_indices(None, 1, 10, 3, one, None) == B.CT_ERR_NULL
    assert lib.ct_topk_indices(one, 1, 10, 0, one, None) == B.CT_OK
    assert [B.ct_frequency_n_selected(32768, r) for r in (0.0, 0.15, 1e-9, 1.0)] == [0, 4915, 1, 32768]
    assert lib.ct_select_frequency(one, one, 1, 0, 2048, 1024, 0.5, 1.2, one, one, one, 1 << 30, None) == B.CT_ERR_RATIO
