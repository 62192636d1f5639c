"""Helpers shared by the GPU parity tests: bf16 bit patterns <-> device tensors, and the
acceptance rule for bf16-in / fp32-accumulate outputs."""
import sys

import numpy as np
import torch

from paper_2605_24022_amd import workloads as W

MAX_ABS = 2e-2      # acceptance bounds for bf16-in / fp32-accumulate outputs
ROW_REL_L2 = 1e-2


def say(msg):
    """Name the case before the GPU step so that a fault leaves a trace."""
    print(f"[gpu-case] {msg}", flush=True)
    sys.stdout.flush()


def dev_bf16(bits: np.ndarray) -> torch.Tensor:
    """uint16 bf16 bit patterns -> bfloat16 tensor on cuda:0 (bit exact)."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def pinned_bf16(bits: np.ndarray) -> torch.Tensor:
    t = torch.empty(bits.shape, dtype=torch.int16, pin_memory=True)
    t.copy_(torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)))
    return t.view(torch.bfloat16)


def dev_i32(a) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def bits_of(t: torch.Tensor) -> np.ndarray:
    return t.detach().view(torch.int16).cpu().numpy().view(np.uint16)


def f64_of(t: torch.Tensor) -> np.ndarray:
    return W.bf16_bits_to_f64(bits_of(t))


def errors(got: np.ndarray, want: np.ndarray):
    """max-abs error and worst per-row (last axis) relative L2 error."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    diff = got - want
    max_abs = float(np.max(np.abs(diff))) if diff.size else 0.0
    num = np.sqrt((diff ** 2).sum(axis=-1))
    den = np.sqrt((want ** 2).sum(axis=-1))
    rel = float(np.max(num / np.maximum(den, 1e-30))) if diff.size else 0.0
    return max_abs, rel


def bf16_half_ulp(x: np.ndarray) -> np.ndarray:
    """Largest error that rounding a value of magnitude |x| to bfloat16 can add: half the spacing
    2^(floor(log2 |x|) - 7) of bf16 numbers at that magnitude (0 for x = 0)."""
    ax = np.abs(np.asarray(x, dtype=np.float64))
    e = np.floor(np.log2(np.where(ax > 0, ax, 1.0)))
    return np.where(ax > 0, 2.0 ** (e - 8.0), 0.0)


def assert_close(got, want, what, max_abs=MAX_ABS, rel_l2=ROW_REL_L2, ulp_slack=0.0, slack_above=0.0,
                 rounding_slack_from=None, unit_scale_rows=False):
    """max-abs and per-row relative L2 bounds.
    unit_scale_rows: the absolute bound is meant for data of unit scale; a row whose expected
    values have a root mean square above 1 (the residual stream deep in a stack) is held to
    max_abs times that root mean square.  The relative L2 bound is never scaled.
    rounding_slack_from = m: for elements with |want| >= m the absolute bound grows by the half
    spacing of bf16 at |want| (the error the final rounding of the stored result alone can add: from
    magnitude 4 on that is 0.0156 or more of the 0.02 allowed, from 8 on more than all of it).
    ulp_slack > 0: the bound grows by ulp_slack * |want| for elements with |want| > slack_above (a
    looser, relative form for results whose inputs already carry rounding from earlier layers)."""
    assert np.isfinite(np.asarray(got)).all(), f"{what}: non-finite values in the GPU result"
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    excess = np.abs(got - want) - ulp_slack * np.where(np.abs(want) > slack_above, np.abs(want), 0.0)
    if rounding_slack_from is not None:
        excess = excess - np.where(np.abs(want) >= rounding_slack_from, bf16_half_ulp(want), 0.0)
    if unit_scale_rows and excess.size:
        rms = np.sqrt((want ** 2).mean(axis=-1, keepdims=True))
        excess = excess / np.maximum(rms, 1.0)
        what = f"{what} [row rms up to {float(rms.max()):.2f}]"
    ma = float(excess.max()) if excess.size else 0.0
    _, rl = errors(got, want)
    slack_txt = " beyond the bf16 rounding slack" if (ulp_slack or rounding_slack_from is not None) else ""
    print(f"[parity] {what}: max-abs {ma:.3e} (<= {max_abs:g}{slack_txt}), "
          f"worst row rel-L2 {rl:.3e} (<= {rel_l2:g})", flush=True)
    assert ma <= max_abs, f"{what}: max-abs {ma} > {max_abs}"
    assert rl <= rel_l2, f"{what}: row relative L2 {rl} > {rel_l2}"
