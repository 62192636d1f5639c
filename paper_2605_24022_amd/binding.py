"""ctypes binding over libcachetune.so: argument marshalling only.

Every function mirrors one C entry point of ``include/cachetune.h`` under the same name
and takes torch tensors (device or pinned host), Python ints and a stream handle.  No step
of the method is computed here; a missing library is an error, never a fallback.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, byref, c_char_p, c_double, c_float, c_int32, c_int64, c_size_t, c_void_p
from typing import Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libcachetune.so")

CT_OK = 0
CT_ERR_NULL, CT_ERR_SHAPE, CT_ERR_INDEX, CT_ERR_RATIO = -1, -2, -3, -4
CT_ERR_WORKSPACE, CT_ERR_HIP, CT_ERR_UNSUPPORTED = -5, -6, -7

KERNEL_CLASSES = {"qkv": 0, "rerope": 1, "scatter": 2, "attention": 3, "merge": 4, "linear": 5, "norm": 6, "frequency": 7, "topk": 8}

EXPORTS = [
    "ct_qkv_selected", "ct_rerope_keys", "ct_rerope_keys_skip", "ct_rerope_chunk", "ct_scatter_kv", "ct_selected_attention",
    "ct_selected_attention_static", "ct_static_scratch_bytes",
    "ct_partial_prefill_layer", "ct_workspace_bytes", "ct_attention_state_bytes", "ct_attention_rows_read", "ct_validate_indices", "ct_set_profiling",
    "ct_profile_reset", "ct_profile_read", "ct_last_error", "ct_version",
    "ct_rmsnorm", "ct_linear", "ct_linear_ws", "ct_linear_ws_cus", "ct_linear_workspace_bytes", "ct_swiglu", "ct_partial_prefill_stack", "ct_partial_prefill_stack_tap", "ct_stack_workspace_bytes",
    "ct_measure_mfma_rate", "ct_layer_latency_model", "ct_ratio_prior", "ct_ratio_search",
    "ct_frequency_scores", "ct_frequency_workspace_bytes", "ct_topk_indices", "ct_frequency_n_selected",
    "ct_select_frequency",
]


TTFT_FN = ctypes.CFUNCTYPE(c_double, c_double, c_void_p)


class LayerCfg(ctypes.Structure):
    _fields_ = [("hidden", c_int32), ("n_q_heads", c_int32), ("n_kv_heads", c_int32), ("head_dim", c_int32),
                ("rope_theta", c_double), ("rope_style", c_int32), ("softmax_scale", c_float)]


class Chunk(ctypes.Structure):
    _fields_ = [("k", c_void_p), ("v", c_void_p), ("n_tokens", c_int32), ("old_pos_start", c_int32),
                ("new_pos_start", c_int32), ("location", c_int32), ("raw_keys", c_int32), ("reserved", c_int32)]


class LayerWeights(ctypes.Structure):
    _fields_ = [("attn_norm", c_void_p), ("wqkv", c_void_p), ("wo", c_void_p), ("ffn_norm", c_void_p),
                ("w_gate", c_void_p), ("w_up", c_void_p), ("w_down", c_void_p), ("chunks", POINTER(Chunk))]


class CacheTuneError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"ct_status {status}: {message}")
        self.status = status
        self.message = message


_lib = None


def load() -> ctypes.CDLL:
    """Load the shared library (built by ``python -m paper_2605_24022_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2605_24022_amd.build` "
            "(there is no CPU fallback for the HIP path)")
    lib = ctypes.CDLL(LIB_PATH)
    P = c_void_p
    cfgp = POINTER(LayerCfg)
    lib.ct_qkv_selected.argtypes = [cfgp, P, P, P, c_int32, P, P, P, P, P, P]
    lib.ct_rerope_keys.argtypes = [cfgp, P, P, P, P, c_int32, P]
    lib.ct_rerope_keys_skip.argtypes = [cfgp, P, P, P, P, c_int32, P, c_int32, P]
    lib.ct_rerope_chunk.argtypes = [cfgp, P, P, P, P, c_int32, c_int32, c_int32, c_int32, P]
    lib.ct_scatter_kv.argtypes = [cfgp, P, P, c_int32, P, P, P, c_int32, P]
    lib.ct_selected_attention.argtypes = [cfgp, P, P, P, c_int32, P, c_int32, P, P, P, c_size_t, P]
    lib.ct_selected_attention_static.argtypes = [cfgp, P, P, P, c_int32, P, c_int32, P, P, P]
    lib.ct_selected_attention_static.restype = c_int32
    lib.ct_static_scratch_bytes.argtypes = []
    lib.ct_static_scratch_bytes.restype = c_size_t
    lib.ct_partial_prefill_layer.argtypes = [cfgp, POINTER(Chunk), c_int32, P, P, P, c_int32, c_double, P, P,
                                             P, P, P, P, c_size_t, P, P]
    lib.ct_rmsnorm.argtypes = [P, P, c_float, c_int32, c_int32, P, P]
    lib.ct_linear.argtypes = [P, c_int32, c_int32, P, c_int32, P, P, P]
    lib.ct_linear_ws.argtypes = [P, c_int32, c_int32, P, c_int32, P, P, P, c_size_t, P]
    lib.ct_linear_ws_cus.argtypes = [P, c_int32, c_int32, P, c_int32, P, P, P, c_size_t, c_int32, P]
    lib.ct_linear_workspace_bytes.argtypes = [c_int32, c_int32, c_int32]
    lib.ct_linear_workspace_bytes.restype = c_size_t
    lib.ct_swiglu.argtypes = [P, c_int32, c_int32, P, P, c_int32, P, P]
    lib.ct_partial_prefill_stack.argtypes = [cfgp, c_int32, c_float, POINTER(LayerWeights), c_int32, c_int32, P, P,
                                             c_int32, c_double, P, P, P, c_size_t, P, P]
    lib.ct_partial_prefill_stack_tap.argtypes = [cfgp, c_int32, c_float, POINTER(LayerWeights), c_int32, c_int32, P, P,
                                                 c_int32, c_double, P, P, P, c_size_t, P, P, P]
    lib.ct_partial_prefill_stack_tap.restype = c_int32
    lib.ct_stack_workspace_bytes.argtypes = [cfgp, c_int32, c_int32, c_int32]
    lib.ct_stack_workspace_bytes.restype = c_size_t
    lib.ct_workspace_bytes.argtypes = [cfgp, c_int32, c_int32]
    lib.ct_workspace_bytes.restype = c_size_t
    lib.ct_attention_state_bytes.argtypes = [cfgp, c_int32, c_int32]
    lib.ct_attention_state_bytes.restype = c_size_t
    lib.ct_attention_rows_read.argtypes = [cfgp, P, c_int32, c_int32, c_int32, c_int32, c_int32, POINTER(c_int32),
                                           POINTER(c_int32)]
    lib.ct_validate_indices.argtypes = [P, c_int32, c_int32]
    lib.ct_set_profiling.argtypes = [c_int32]
    lib.ct_set_profiling.restype = None
    lib.ct_profile_reset.argtypes = []
    lib.ct_profile_reset.restype = None
    lib.ct_profile_read.argtypes = [c_int32, POINTER(c_int64), POINTER(c_double)]
    lib.ct_frequency_scores.argtypes = [c_void_p, c_void_p, c_int32, c_int64, c_int32, c_int32, c_double, c_void_p,
                                        c_void_p, c_size_t, c_void_p]
    lib.ct_frequency_workspace_bytes.argtypes = [c_int32, c_int32, c_int32]
    lib.ct_frequency_workspace_bytes.restype = c_size_t
    lib.ct_topk_indices.argtypes = [c_void_p, c_int32, c_int32, c_int32, c_void_p, c_void_p]
    lib.ct_frequency_n_selected.argtypes = [c_int32, c_double]
    lib.ct_frequency_n_selected.restype = c_int32
    lib.ct_select_frequency.argtypes = [c_void_p, c_void_p, c_int32, c_int64, c_int32, c_int32, c_double, c_double,
                                        c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
    lib.ct_layer_latency_model.argtypes = [c_double] * 5
    lib.ct_layer_latency_model.restype = c_double
    lib.ct_ratio_prior.argtypes = [c_double] * 4
    lib.ct_ratio_prior.restype = c_double
    lib.ct_ratio_search.argtypes = [TTFT_FN, c_void_p, c_double, c_double, c_double, c_double, c_int32,
                                    POINTER(c_double), POINTER(c_int32)]
    lib.ct_ratio_search.restype = c_int32
    lib.ct_measure_mfma_rate.argtypes = [c_void_p, c_int32, c_void_p, POINTER(c_double)]
    lib.ct_measure_mfma_rate.restype = c_int32
    lib.ct_last_error.restype = c_char_p
    lib.ct_version.restype = c_char_p
    for name in ("ct_qkv_selected", "ct_rerope_keys", "ct_rerope_keys_skip", "ct_linear_ws_cus", "ct_rerope_chunk", "ct_scatter_kv", "ct_selected_attention",
                 "ct_partial_prefill_layer", "ct_validate_indices", "ct_profile_read", "ct_rmsnorm", "ct_linear",
                 "ct_linear_ws", "ct_swiglu", "ct_partial_prefill_stack"):
        getattr(lib, name).restype = c_int32
    _lib = lib
    return lib


def make_cfg(hidden: int, n_q_heads: int, n_kv_heads: int, head_dim: int, rope_theta: float,
             rope_style: int = 0, softmax_scale: float = 0.0) -> LayerCfg:
    return LayerCfg(hidden, n_q_heads, n_kv_heads, head_dim, float(rope_theta), rope_style, softmax_scale)


def cfg_from_shape(shape) -> LayerCfg:
    """From a workloads.LayerShape."""
    return make_cfg(shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.rope_theta,
                    shape.rope_style)


def _ptr(x) -> Optional[int]:
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()          # torch tensor (device or pinned host)


def _stream(s) -> Optional[int]:
    if s is None:
        return None
    if isinstance(s, int):
        return s or None
    return s.cuda_stream or None  # torch.cuda.Stream


def _check(status: int) -> None:
    if status != CT_OK:
        raise CacheTuneError(status, load().ct_last_error().decode())


def ct_version() -> str:
    return load().ct_version().decode()


def ct_last_error() -> str:
    return load().ct_last_error().decode()


def ct_workspace_bytes(cfg: LayerCfg, n_ctx: int, n_sel: int) -> int:
    return int(load().ct_workspace_bytes(byref(cfg), n_ctx, n_sel))


def ct_attention_state_bytes(cfg: LayerCfg, n_ctx: int, n_sel: int) -> int:
    return int(load().ct_attention_state_bytes(byref(cfg), n_ctx, n_sel))


def ct_attention_rows_read(cfg: LayerCfg, host_idx, n_sel: int, n_ctx: int, key_after: int, key_upto: int,
                           with_state: bool):
    """host_idx: numpy int32 array.  Returns (first_row, last_row) of the key rows that launch reads."""
    lo, hi = c_int32(0), c_int32(0)
    p = None if host_idx is None else host_idx.ctypes.data
    _check(load().ct_attention_rows_read(byref(cfg), p, n_sel, n_ctx, key_after, key_upto, int(bool(with_state)),
                                         byref(lo), byref(hi)))
    return lo.value, hi.value


def ct_validate_indices(host_idx, n_sel: int, n_ctx: int) -> None:
    """host_idx: numpy int32 array (or None)."""
    p = None if host_idx is None else host_idx.ctypes.data
    _check(load().ct_validate_indices(p, n_sel, n_ctx))


def ct_qkv_selected(cfg, hidden, hidden_rows, sel_pos, n_sel, wqkv, bias, q_out, k_out, v_out, stream=None) -> None:
    _check(load().ct_qkv_selected(byref(cfg), _ptr(hidden), _ptr(hidden_rows), _ptr(sel_pos), n_sel, _ptr(wqkv),
                                  _ptr(bias), _ptr(q_out), _ptr(k_out), _ptr(v_out), _stream(stream)))


def ct_rerope_keys(cfg, k_src, k_dst, old_pos, new_pos, n_tokens, stream=None) -> None:
    _check(load().ct_rerope_keys(byref(cfg), _ptr(k_src), _ptr(k_dst), _ptr(old_pos), _ptr(new_pos), n_tokens,
                                 _stream(stream)))


def ct_rerope_keys_skip(cfg, k_src, k_dst, old_pos, new_pos, n_tokens, skip_rows, n_skip, stream=None) -> None:
    _check(load().ct_rerope_keys_skip(byref(cfg), _ptr(k_src), _ptr(k_dst), _ptr(old_pos), _ptr(new_pos), n_tokens,
                                      _ptr(skip_rows), n_skip, _stream(stream)))


def ct_rerope_chunk(cfg, k_src, k_dst, v_src, v_dst, n_tokens, old_pos_start, new_pos_start, raw_keys=0,
                    stream=None) -> None:
    _check(load().ct_rerope_chunk(byref(cfg), _ptr(k_src), _ptr(k_dst), _ptr(v_src), _ptr(v_dst), n_tokens,
                                  old_pos_start, new_pos_start, raw_keys, _stream(stream)))


def ct_scatter_kv(cfg, k_buf, v_buf, n_ctx, k_sel, v_sel, sel_idx, n_sel, stream=None) -> None:
    _check(load().ct_scatter_kv(byref(cfg), _ptr(k_buf), _ptr(v_buf), n_ctx, _ptr(k_sel), _ptr(v_sel),
                                _ptr(sel_idx), n_sel, _stream(stream)))


def ct_selected_attention(cfg, q_sel, k_buf, v_buf, n_ctx, sel_idx, n_sel, out, lse, workspace, workspace_bytes,
                          stream=None) -> None:
    _check(load().ct_selected_attention(byref(cfg), _ptr(q_sel), _ptr(k_buf), _ptr(v_buf), n_ctx, _ptr(sel_idx),
                                        n_sel, _ptr(out), _ptr(lse), _ptr(workspace), workspace_bytes,
                                        _stream(stream)))


def ct_selected_attention_static(cfg, q_sel, k_buf, v_buf, n_ctx, sel_idx, n_sel, out, lse, stream=None) -> None:
    _check(load().ct_selected_attention_static(byref(cfg), _ptr(q_sel), _ptr(k_buf), _ptr(v_buf), n_ctx, _ptr(sel_idx),
                                               n_sel, _ptr(out), _ptr(lse), _stream(stream)))


def ct_static_scratch_bytes() -> int:
    return int(load().ct_static_scratch_bytes())


def make_chunks(entries: Sequence[dict]):
    """entries: dicts with k, v (tensors or addresses), n_tokens, old_pos_start, new_pos_start,
    location (0 device / 1 pinned host) and optional raw_keys."""
    arr = (Chunk * len(entries))()
    for i, e in enumerate(entries):
        arr[i] = Chunk(_ptr(e["k"]), _ptr(e["v"]), e["n_tokens"], e.get("old_pos_start", 0), e["new_pos_start"],
                       e.get("location", 0), e.get("raw_keys", 0), 0)
    return arr


def ct_partial_prefill_layer(cfg, chunks, n_chunks, hidden, hidden_rows, sel_idx, n_sel, recompute_ratio, wqkv,
                             bias, k_buf, v_buf, attn_out, workspace, workspace_bytes, compute_stream=None,
                             copy_stream=None) -> None:
    _check(load().ct_partial_prefill_layer(byref(cfg), chunks, n_chunks, _ptr(hidden), _ptr(hidden_rows),
                                           _ptr(sel_idx), n_sel, float(recompute_ratio), _ptr(wqkv), _ptr(bias),
                                           _ptr(k_buf), _ptr(v_buf), _ptr(attn_out), _ptr(workspace),
                                           workspace_bytes, _stream(compute_stream), _stream(copy_stream)))


def ct_rmsnorm(x, weight, eps, n_tokens, width, out, stream=None) -> None:
    _check(load().ct_rmsnorm(_ptr(x), _ptr(weight), float(eps), n_tokens, width, _ptr(out), _stream(stream)))


def ct_linear(x, n_tokens, k_len, w, n_out, residual, out, stream=None) -> None:
    _check(load().ct_linear(_ptr(x), n_tokens, k_len, _ptr(w), n_out, _ptr(residual), _ptr(out), _stream(stream)))


def ct_linear_workspace_bytes(n_tokens, k_len, n_out) -> int:
    return int(load().ct_linear_workspace_bytes(n_tokens, k_len, n_out))


def ct_linear_ws(x, n_tokens, k_len, w, n_out, residual, out, workspace, workspace_bytes, stream=None) -> None:
    _check(load().ct_linear_ws(_ptr(x), n_tokens, k_len, _ptr(w), n_out, _ptr(residual), _ptr(out), _ptr(workspace),
                               workspace_bytes, _stream(stream)))


def ct_linear_ws_cus(x, n_tokens, k_len, w, n_out, residual, out, workspace, workspace_bytes, n_compute_units,
                     stream=None) -> None:
    _check(load().ct_linear_ws_cus(_ptr(x), n_tokens, k_len, _ptr(w), n_out, _ptr(residual), _ptr(out), _ptr(workspace),
                                   workspace_bytes, n_compute_units, _stream(stream)))


def ct_swiglu(x, n_tokens, k_len, w_gate, w_up, n_out, out, stream=None) -> None:
    _check(load().ct_swiglu(_ptr(x), n_tokens, k_len, _ptr(w_gate), _ptr(w_up), n_out, _ptr(out), _stream(stream)))


def make_layers(entries: Sequence[dict]):
    """entries: dicts with attn_norm, wqkv, wo, ffn_norm, w_gate, w_up, w_down (tensors) and
    chunks (a Chunk array from make_chunks).  The returned array keeps the chunk arrays alive."""
    arr = (LayerWeights * len(entries))()
    keep = []
    for i, e in enumerate(entries):
        keep.append(e["chunks"])
        arr[i] = LayerWeights(_ptr(e["attn_norm"]), _ptr(e["wqkv"]), _ptr(e["wo"]), _ptr(e["ffn_norm"]),
                              _ptr(e["w_gate"]), _ptr(e["w_up"]), _ptr(e["w_down"]),
                              ctypes.cast(e["chunks"], POINTER(Chunk)))
    arr._keep = keep
    return arr


def ct_stack_workspace_bytes(cfg: LayerCfg, ffn_dim: int, n_ctx: int, n_sel: int) -> int:
    return int(load().ct_stack_workspace_bytes(byref(cfg), ffn_dim, n_ctx, n_sel))


def ct_partial_prefill_stack(cfg, ffn_dim, rms_eps, layers, n_layers, n_chunks, hidden_sel, sel_idx, n_sel,
                             recompute_ratio, k_bufs, v_bufs, workspace, workspace_bytes, compute_stream=None,
                             copy_stream=None) -> None:
    _check(load().ct_partial_prefill_stack(byref(cfg), ffn_dim, float(rms_eps), layers, n_layers, n_chunks,
                                           _ptr(hidden_sel), _ptr(sel_idx), n_sel, float(recompute_ratio),
                                           _ptr(k_bufs), _ptr(v_bufs), _ptr(workspace), workspace_bytes,
                                           _stream(compute_stream), _stream(copy_stream)))


def ct_partial_prefill_stack_tap(cfg, ffn_dim, rms_eps, layers, n_layers, n_chunks, hidden_sel, sel_idx, n_sel,
                                 recompute_ratio, k_bufs, v_bufs, workspace, workspace_bytes, compute_stream=None,
                                 copy_stream=None, layer_inputs=None) -> None:
    _check(load().ct_partial_prefill_stack_tap(byref(cfg), ffn_dim, float(rms_eps), layers, n_layers, n_chunks,
                                               _ptr(hidden_sel), _ptr(sel_idx), n_sel, float(recompute_ratio),
                                               _ptr(k_bufs), _ptr(v_bufs), _ptr(workspace), workspace_bytes,
                                               _stream(compute_stream), _stream(copy_stream), _ptr(layer_inputs)))


def ct_set_profiling(on: bool) -> None:
    load().ct_set_profiling(1 if on else 0)


def ct_profile_reset() -> None:
    load().ct_profile_reset()


def ct_frequency_workspace_bytes(n_batch, n_tokens, row_elems) -> int:
    return int(load().ct_frequency_workspace_bytes(n_batch, n_tokens, row_elems))


def ct_frequency_scores(k, v, n_batch, batch_stride, n_tokens, row_elems, alpha, scores, workspace, workspace_bytes,
                        stream=None):
    _check(load().ct_frequency_scores(_ptr(k), _ptr(v), n_batch, batch_stride, n_tokens, row_elems, alpha, _ptr(scores),
                                      _ptr(workspace), workspace_bytes, _stream(stream)))


def ct_topk_indices(scores, n_batch, n_tokens, k, idx_out, stream=None):
    _check(load().ct_topk_indices(_ptr(scores), n_batch, n_tokens, k, _ptr(idx_out), _stream(stream)))


def ct_frequency_n_selected(n_tokens, ratio) -> int:
    return int(load().ct_frequency_n_selected(n_tokens, ratio))


def ct_select_frequency(k, v, n_batch, batch_stride, n_tokens, row_elems, alpha, ratio, idx_out, scores, workspace,
                        workspace_bytes, stream=None):
    _check(load().ct_select_frequency(_ptr(k), _ptr(v), n_batch, batch_stride, n_tokens, row_elems, alpha, ratio,
                                      _ptr(idx_out), _ptr(scores), _ptr(workspace), workspace_bytes, _stream(stream)))


def ct_layer_latency_model(r, n_tokens, t_c, t_i, t_o) -> float:
    return float(load().ct_layer_latency_model(r, n_tokens, t_c, t_i, t_o))


def ct_ratio_prior(t_c, t_i, r_min, r_max) -> float:
    return float(load().ct_ratio_prior(t_c, t_i, r_min, r_max))


def ct_ratio_search(eval_fn, r0, r_min, r_max, eps, max_evals=64):
    """eval_fn(r) -> latency.  Returns (r_star, number of evaluations)."""
    cb = TTFT_FN(lambda r, _user: float(eval_fn(r)))
    out, n = c_double(0.0), c_int32(0)
    _check(load().ct_ratio_search(cb, None, r0, r_min, r_max, eps, max_evals, byref(out), byref(n)))
    return out.value, n.value


def ct_measure_mfma_rate(scratch, iters: int = 2000, stream=None) -> float:
    """TFLOP/s of a kernel that only issues bf16 MFMAs; `scratch`: device tensor of >= 512 KiB."""
    out = c_double(0.0)
    _check(load().ct_measure_mfma_rate(_ptr(scratch), iters, _stream(stream), byref(out)))
    return out.value


def ct_profile_read(kernel_class) -> tuple:
    """Returns (launches, total_ms) for a kernel class name or number."""
    kc = KERNEL_CLASSES[kernel_class] if isinstance(kernel_class, str) else int(kernel_class)
    n, ms = c_int64(0), c_double(0.0)
    _check(load().ct_profile_read(kc, byref(n), byref(ms)))
    return n.value, ms.value
