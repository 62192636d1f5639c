"""The entry point that allocates nothing (ct_selected_attention_static) against the entry point it
is a variant of (ct_selected_attention with a caller's workspace): same kernels, so the same bits,
and against the oracle; two calls in a row on the library's one scratch array, the second with a
smaller input, which must not see anything the first one left there."""
import numpy as np
import pytest
import torch

from oracle import ct_oracle as O
from paper_2605_24022_amd import binding as B
from paper_2605_24022_amd import workloads as W
from tests.gpu_util import assert_close, dev_bf16, dev_i32, f64_of, say

pytestmark = pytest.mark.gpu


def _case(Hq, Hkv, D, n_ctx, n_sel, seed):
    rng = np.random.default_rng([61, seed])
    sel = np.sort(rng.choice(n_ctx, n_sel, replace=False)).astype(np.int32)
    sel[-1] = n_ctx - 1
    sel = np.unique(sel).astype(np.int32)
    q = W.f32_to_bf16_bits(rng.standard_normal((sel.size, Hq, D), dtype=np.float32))
    k = W.f32_to_bf16_bits(rng.standard_normal((n_ctx, Hkv, D), dtype=np.float32))
    v = W.f32_to_bf16_bits(rng.standard_normal((n_ctx, Hkv, D), dtype=np.float32))
    return sel, q, k, v


def test_static_scratch_attention_matches_the_workspace_entry_point():
    assert torch.cuda.is_available()
    torch.cuda.set_device(0)
    B.load()
    limit = B.ct_static_scratch_bytes()
    assert limit == 64 << 20
    # first a problem whose key range is split (fp32 partials go through the scratch), then a smaller
    # one with other head counts, then one that needs no scratch at all
    for Hq, Hkv, D, n_ctx, n_sel, seed in ((32, 8, 128, 8192, 400, 1), (8, 2, 64, 4096, 90, 2), (32, 8, 128, 2048, 307, 3)):
        sel, q, k, v = _case(Hq, Hkv, D, n_ctx, n_sel, seed)
        cfg = B.make_cfg(Hq * D, Hq, Hkv, D, 1e4)
        need = B.ct_workspace_bytes(cfg, n_ctx, sel.size)
        say(f"static-scratch attention Hq={Hq} Hkv={Hkv} D={D} n_ctx={n_ctx} n_sel={sel.size} (workspace entry point needs {need})")
        qd, kd, vd, sd = dev_bf16(q), dev_bf16(k), dev_bf16(v), dev_i32(sel)
        out_a = torch.full((sel.size, Hq, D), float("nan"), dtype=torch.bfloat16, device="cuda")
        lse_a = torch.full((sel.size, Hq), float("nan"), dtype=torch.float32, device="cuda")
        out_b, lse_b = out_a.clone(), lse_a.clone()
        B.ct_selected_attention_static(cfg, qd, kd, vd, n_ctx, sd, sel.size, out_a, lse_a)
        torch.cuda.synchronize()
        ws = torch.full((max(need, 256),), 0xff, dtype=torch.uint8, device="cuda")
        B.ct_selected_attention(cfg, qd, kd, vd, n_ctx, sd, sel.size, out_b, lse_b, ws, need)
        torch.cuda.synchronize()
        assert torch.equal(out_a.view(torch.int16), out_b.view(torch.int16)), "outputs differ from the workspace entry point's"
        assert torch.equal(lse_a.view(torch.int32), lse_b.view(torch.int32)), "LSE differs from the workspace entry point's"
        want, want_lse = O.selected_attention(W.bf16_bits_to_f64(q), W.bf16_bits_to_f64(k), W.bf16_bits_to_f64(v), sel)
        assert_close(f64_of(out_a), want, "static-scratch attention out")
        assert np.max(np.abs(lse_a.cpu().numpy().astype(np.float64) - want_lse)) <= 2e-2


def test_static_scratch_attention_rejects_what_does_not_fit():
    B.load()
    cfg = B.make_cfg(4096, 32, 8, 128, 5e5)
    # 47 tiles x 8 heads = 376 pairs, split in two: 752 partial tiles of 133 120 bytes > 64 MiB
    with pytest.raises(B.CacheTuneError) as e:
        B.ct_selected_attention_static(cfg, 0x10000, 0x10000, 0x10000, 65536, 0x10000, 3000, 0x10000, None)
    assert e.value.status == B.CT_ERR_WORKSPACE and "static" in e.value.message
