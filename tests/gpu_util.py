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


def assert_close(got, want, what, max_abs=MAX_ABS, rel_l2=ROW_REL_L2, ulp_slack=0.0):
    """max-abs and per-row relative L2 bounds.  `ulp_slack` > 0 lets the absolute bound grow with
    the magnitude of the expected value (|err| <= max_abs + ulp_slack * |want|): a bf16 result
    above 8 in magnitude is rounded with a spacing of 2^-5 or more, which alone exceeds 2e-2."""
    assert np.isfinite(np.asarray(got)).all(), f"{what}: non-finite values in the GPU result"
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    excess = np.abs(got - want) - ulp_slack * np.abs(want)
    ma = float(excess.max()) if excess.size else 0.0
    _, rl = errors(got, want)
    print(f"[parity] {what}: max-abs {ma:.3e} (<= {max_abs:g}{' beyond the bf16 spacing slack' if ulp_slack else ''}), "
          f"worst row rel-L2 {rl:.3e} (<= {rel_l2:g})", flush=True)
    assert ma <= max_abs, f"{what}: max-abs {ma} > {max_abs}"
    assert rl <= rel_l2, f"{what}: row relative L2 {rl} > {rel_l2}"
