#!/usr/bin/env python3
"""Benchmark of the partial-prefill hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3] [--ratio 15]

A step is one call of ct_partial_prefill_layer (selective QKV recompute, re-RoPE of the
reused keys + value copy from the device-resident cache pool into the layer buffers,
scatter fusion, selected-row causal attention) over one batch of seeded synthetic input
that is already resident in HBM.  The default workload is the headline one: Llama-3-8B
layer shape, 32768-token context from 16 x 2048-token chunks, recompute ratio 15 %.

One JSON line is printed on stdout; progress goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E
# HBM bytes per attention launch from rocprofv3 FETCH_SIZE / WRITE_SIZE runs of this command (scaled
# by a plain-copy calibration).  Counters cannot be read live, so a figure is attached to the
# workload it was measured on AND to the attention kernel source it was measured with: it is
# reported only while the SHA-256 of csrc/ct_attention.hip still starts with the recorded prefix
# (a changed kernel makes it null until the counter runs are repeated and recorded here with the
# summary under profiles/).
MEASURED_ATTENTION_TRAFFIC = {
    # workload: (fetch MiB scaled, write MiB, sha256 prefix of ct_attention.hip, summary file)
    "cfg3-llama8b-32k-r15": (576.1, 40.8, "68d23583b46a9d35", "profiles/partial_prefill_layer_cfg3_r15.md"),
}


def attention_traffic(workload: str):
    """(bytes per launch, provenance) for this workload and the attention source as it stands, or (None, reason)."""
    import hashlib
    rec = MEASURED_ATTENTION_TRAFFIC.get(workload)
    if rec is None:
        return None, "no counter run recorded for this workload"
    fetch_mib, write_mib, sha, summary = rec
    src = os.path.join(ROOT, "paper_2605_24022_amd", "csrc", "ct_attention.hip")
    have = hashlib.sha256(open(src, "rb").read()).hexdigest()
    if not have.startswith(sha):
        return None, f"recorded with another version of the attention kernel ({sha}); see {summary}"
    return (fetch_mib + write_mib) * 1024 * 1024, f"{summary} (attention source {sha})"


def log(msg: str) -> None:
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def cpu_baseline(wl, sample_rows: int, O, W, np):
    """Time the fp64 oracle (as it stands) on the same layer: the projection, re-RoPE and scatter
    in full; attention in full as well (sample_rows = 0: nothing extrapolated), or on
    `sample_rows` selected rows with its time scaled by visible-key counts to the full row set."""
    from threadpoolctl import threadpool_info
    sh = wl.spec.shape
    t0 = time.perf_counter()
    hid = W.bf16_bits_to_f64(wl.hidden if wl.hidden_rows is None else wl.hidden[wl.hidden_rows])
    wq = W.bf16_bits_to_f64(wl.wqkv)
    kc, vc = W.bf16_bits_to_f64(wl.k_cache), W.bf16_bits_to_f64(wl.v_cache)
    t_conv = time.perf_counter() - t0
    t0 = time.perf_counter()
    q, k_new, v_new = O.qkv_selected(hid, wq, None, wl.sel_pos, sh.n_q_heads, sh.n_kv_heads, sh.head_dim,
                                     sh.rope_theta, sh.rope_style)
    t_qkv = time.perf_counter() - t0
    t0 = time.perf_counter()
    k_rot = O.rerope_keys(kc, wl.old_pos, wl.new_pos, sh.rope_theta, sh.rope_style)
    t_rope = time.perf_counter() - t0
    t0 = time.perf_counter()
    kf, vf = O.scatter_kv(k_rot, vc, k_new, v_new, wl.sel_idx)
    t_scat = time.perf_counter() - t0
    full = sample_rows <= 0 or sample_rows >= wl.spec.n_sel
    rows = None if full else W.sample_rows(wl.spec.n_sel, sample_rows, seed=wl.spec.seed)
    t0 = time.perf_counter()
    if full:   # a few hundred rows at a time: one call would hold [n_sel, n_ctx] score matrices of gigabytes
        for lo in range(0, wl.spec.n_sel, 512):
            O.selected_attention(q, kf, vf, wl.sel_idx, rows=np.arange(lo, min(lo + 512, wl.spec.n_sel)))
    else:
        O.selected_attention(q, kf, vf, wl.sel_idx, rows=rows)
    t_attn = time.perf_counter() - t0
    vis_all = float((wl.sel_idx.astype(np.int64) + 1).sum())
    vis_smp = vis_all if full else float((wl.sel_idx[rows].astype(np.int64) + 1).sum())
    t_attn_full = t_attn * vis_all / vis_smp
    total = t_qkv + t_rope + t_scat + t_attn_full
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    nproc = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    what = (f"attention for all {wl.spec.n_sel} selected rows ({t_attn:.2f}s, nothing extrapolated)" if full else
            f"attention on {len(rows)} of {wl.spec.n_sel} selected rows ({t_attn:.2f}s) scaled by visible keys "
            f"x{vis_all / vis_smp:.1f} (extrapolated)")
    return {
        "value": total * 1e3, "unit": "ms/layer", "cores": threads, "nproc": nproc, "kind": "oracle",
        "sample": (f"fp64 NumPy oracle, same workload: QKV projection, re-RoPE and scatter in full "
                   f"({t_qkv:.2f}s + {t_rope:.2f}s + {t_scat:.2f}s), {what}; "
                   f"bf16->f64 input conversion {t_conv:.2f}s not counted; {threads} BLAS threads on {nproc} host cores"),
        "extrapolated": not full,
        "measured_s": {"qkv": t_qkv, "rerope": t_rope, "scatter": t_scat,
                       "attention" if full else "attention_sample": t_attn},
    }


def cold_cache_bandwidth(B, cfg, wl, sp, torch, np, reps: int = 3):
    """Stand-alone bandwidth kernels under a cold-cache protocol: every launch works on a
    different buffer out of a ring of >= 1 GiB, so nothing it reads is left in the last-level
    cache by the launch before.  In-place re-RoPE of all N key rows (credited with the N - n rows
    that have to be rotated), scatter of the n recomputed rows, and a plain device copy of the
    same size as the re-RoPE traffic for the ceiling.  Durations come from the library's HIP
    events on the launch stream."""
    sh = sp.shape
    N, n = sp.n_ctx, sp.n_sel
    row = sh.n_kv_heads * sh.head_dim
    ring = max(2, (1 << 30) // (N * row * 2))
    kb = [torch.randn((N, sh.n_kv_heads, sh.head_dim), device="cuda", dtype=torch.float32).to(torch.bfloat16)
          for _ in range(ring)]
    vb = [torch.zeros_like(kb[0]) for _ in range(ring)]
    old = torch.from_numpy(wl.old_pos).cuda()
    new = torch.from_numpy(wl.new_pos).cuda()
    sel = torch.from_numpy(wl.sel_idx).cuda()
    ks = torch.randn((n, sh.n_kv_heads, sh.head_dim), device="cuda", dtype=torch.float32).to(torch.bfloat16)
    vs = torch.randn_like(ks)
    st = torch.cuda.current_stream()
    res = {"ring_buffers": ring, "ring_bytes": ring * N * row * 2 * 2}

    def timed_on(bufs, name, fn):
        fn(0)
        torch.cuda.synchronize()
        B.ct_profile_reset()
        B.ct_set_profiling(True)
        for r in range(reps):
            for i in range(len(bufs)):
                fn(i)
        torch.cuda.synchronize()
        B.ct_set_profiling(False)
        cnt, ms = B.ct_profile_read(name)
        B.ct_profile_reset()
        return ms / cnt * 1e-3

    def timed(name, fn):
        return timed_on(kb, name, fn)

    t = timed("rerope", lambda i: B.ct_rerope_keys(cfg, kb[i], kb[i], old, new, N, st))
    credited = 2.0 * (N - n) * row * 2 + 8.0 * (N - n)
    moved = 2.0 * N * row * 2 + 8.0 * N
    res["rerope_in_place"] = {"avg_us": t * 1e6, "gbs_credited": credited / t / 1e9, "gbs_moved": moved / t / 1e9,
                              "frac_of_hbm_peak_credited": credited / t / 1e9 / PEAK_HBM_GBS,
                              "frac_of_hbm_peak_moved": moved / t / 1e9 / PEAK_HBM_GBS}
    # the same rotation with the recompute set left out (rows that are overwritten by the scatter are
    # neither read nor written): what it moves is what it is credited with
    t = timed("rerope", lambda i: B.ct_rerope_keys_skip(cfg, kb[i], kb[i], old, new, N, sel, n, st))
    res["rerope_in_place_reused_rows_only"] = {"avg_us": t * 1e6, "gbs": credited / t / 1e9,
                                               "frac_of_hbm_peak": credited / t / 1e9 / PEAK_HBM_GBS}
    t = timed("scatter", lambda i: B.ct_scatter_kv(cfg, kb[i], vb[i], N, ks, vs, sel, n, st))
    sb = 2.0 * 2.0 * n * row * 2 + 4.0 * n
    res["scatter"] = {"avg_us": t * 1e6, "gbs": sb / t / 1e9, "frac_of_hbm_peak": sb / t / 1e9 / PEAK_HBM_GBS}
    if n < N:
        # the r = 100 % point of the same context (every row scattered: 268 MB), where the launch ramp
        # weighs less than at 40 MB; sources rotate through the K ring as well
        all_rows = torch.arange(N, device="cuda", dtype=torch.int32)
        t = timed("scatter", lambda i: B.ct_scatter_kv(cfg, kb[i], vb[i], N, kb[(i + ring // 2) % ring],
                                                       kb[(i + ring // 2 + 1) % ring], all_rows, N, st))
        sb_all = 2.0 * 2.0 * N * row * 2 + 4.0 * N
        res["scatter_all_rows"] = {"n_rows": N, "bytes": sb_all, "avg_us": t * 1e6, "gbs": sb_all / t / 1e9,
                                   "frac_of_hbm_peak": sb_all / t / 1e9 / PEAK_HBM_GBS}
    # ceiling: plain device copy K ring -> V ring, same bytes as the in-place rotation moves
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    vb[0].copy_(kb[0])
    torch.cuda.synchronize()
    e0.record()
    for r in range(reps):
        for i in range(ring):
            vb[i].copy_(kb[(i + ring // 2) % ring])
    e1.record()
    torch.cuda.synchronize()
    t = e0.elapsed_time(e1) * 1e-3 / (reps * ring)
    res["plain_copy"] = {"avg_us": t * 1e6, "gbs": 2.0 * N * row * 2 / t / 1e9}
    # the same in-place rotation on a 4x longer context (256 MiB of keys per launch), where the launch
    # ramp weighs less
    del vb
    n4 = 4 * N
    ring4 = max(2, ring // 4)
    k4 = [torch.cat(kb[4 * i:4 * i + 4]) for i in range(ring4)] if ring >= 8 else None
    if k4 is not None:
        old4 = torch.arange(n4, device="cuda", dtype=torch.int32) % sp.chunk_len
        new4 = torch.arange(n4, device="cuda", dtype=torch.int32)
        t = timed_on(k4, "rerope", lambda i: B.ct_rerope_keys(cfg, k4[i], k4[i], old4, new4, n4, st))
        m4 = 2.0 * n4 * row * 2 + 8.0 * n4
        res["rerope_in_place_4x_tokens"] = {"n_tokens": n4, "avg_us": t * 1e6, "gbs_moved": m4 / t / 1e9,
                                            "frac_of_hbm_peak_moved": m4 / t / 1e9 / PEAK_HBM_GBS}
        del k4
    return res


def bench_offline(args, B, W, np, torch) -> int:
    """Offline frequency-guided selection (Sec. 4.1) for one chunk of the config-3/5 shape, all
    layers in one call: K and V of `--layers` layers x 2048 tokens x 1024 values, alpha = 0.5,
    r = `--ratio` %.  A step is one ct_select_frequency call (scores + TopK); buffers rotate
    through a ring of more than 1 GiB so that no step finds its input in the last-level cache."""
    n, row, n_batch, alpha = 2048, 1024, args.layers, 0.5
    ratio = args.ratio / 100.0
    n_sel = B.ct_frequency_n_selected(n, ratio)
    log(f"generating spectral K/V for {n_batch} layers of a {n}-token chunk")
    kb, vb = W.make_spectral_kv(1006, n, row, min(n_batch, 4))
    reps = (n_batch + kb.shape[0] - 1) // kb.shape[0]

    def dev(bits):
        t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)
        return t.repeat(reps, 1, 1)[:n_batch].contiguous()
    bytes_per_step = n_batch * (2 * n * row * 2 + n * 4 + n_sel * 4)
    ring = max(2, -(-(1 << 30) // (n_batch * 2 * n * row * 2)) + 1)
    ks = [dev(kb) for _ in range(ring)]
    vs = [dev(vb) for _ in range(ring)]
    ws_bytes = B.ct_frequency_workspace_bytes(n_batch, n, row)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    scores = torch.empty((n_batch, n), dtype=torch.float32, device="cuda")
    idx = torch.empty((n_batch, n_sel), dtype=torch.int32, device="cuda")

    def step(i):
        B.ct_select_frequency(ks[i % ring], vs[i % ring], n_batch, n * row, n, row, alpha, ratio, idx, scores, ws, ws_bytes)
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    B.ct_profile_reset()
    B.ct_set_profiling(not args.no_profile_events)
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    B.ct_set_profiling(False)
    cnt_f, ms_f = B.ct_profile_read("frequency")
    cnt_t, ms_t = B.ct_profile_read("topk")
    B.ct_profile_reset()
    us_f = ms_f / args.steps * 1e3 if cnt_f else 0.0     # both score kernels of a step
    us_t = ms_t / args.steps * 1e3 if cnt_t else 0.0
    score_bytes = n_batch * (2 * n * row * 2 + n * 4)
    fft_flop = n_batch * 2 * (row // 2) * 2 * 5.0 * n * math.log2(n)
    cpu = None
    if not args.no_cpu_baseline:
        from threadpoolctl import threadpool_info
        from oracle import ct_oracle as O
        nb = min(4, n_batch)
        log(f"timing the CPU oracle on {nb} layers")
        kf, vf = W.bf16_bits_to_f64(kb[:nb]), W.bf16_bits_to_f64(vb[:nb])
        t0 = time.perf_counter()
        want = [O.select_frequency(kf[b], vf[b], alpha, ratio) for b in range(nb)]
        t_cpu = (time.perf_counter() - t0) / nb
        step(0)
        torch.cuda.synchronize()
        agree = [int(np.isin(want[b][0], idx[b].cpu().numpy()).sum()) for b in range(nb)]
        threads = max([d.get("num_threads", 1) for d in threadpool_info()] + [1])
        cpu = {"value": t_cpu * n_batch * 1e3, "unit": "ms", "cores": threads, "kind": "oracle",
               "sample": f"fp64 NumPy oracle (rfft, mask, irfft, norms, sort) on {nb} of {n_batch} layers, scaled; "
                         f"indices equal to the oracle's: {agree} of {n_sel} per layer"}
    line = {
        "metric": f"offline frequency-guided selection, {n_batch} layers of a {n}-token chunk, r={args.ratio}%",
        "value": ms, "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"offline-select-llama8b-chunk{n}-x{n_batch}", "n_tokens": n, "row_elems": row,
                   "alpha": alpha, "n_sel": n_sel},
        # bound by vector arithmetic: a forward and an inverse complex FFT of length N (5 N log2 N flop
        # each, the usual count) for each of the row_elems / 2 packed column pairs of K and of V
        "roofline": {"bound": "alu", "achieved": fft_flop / (us_f * 1e-6) / 1e12 if us_f else None, "peak": 157.3,
                     "unit": "TFLOP/s", "frac": fft_flop / (us_f * 1e-6) / 157.3e12 if us_f else None, "traffic": None,
                     "kernel": "freq_energy_kernel (+ freq_finish_kernel), cold cache"},
        "extra": {"scores_us": us_f, "topk_us": us_t, "algorithmic_bytes_per_step": bytes_per_step,
                  "algorithmic_flop_per_step": fft_flop,
                  "scores_hbm_GBps": score_bytes / (us_f * 1e-6) / 1e9 if us_f else None,
                  "scores_frac_of_hbm_peak": score_bytes / (us_f * 1e-6) / 8e12 if us_f else None,
                  "us_per_chunk_layer": ms * 1e3 / n_batch},
        "cpu_baseline": cpu,
    }
    print(json.dumps(line), flush=True)
    return 0


def bench_stack(args, B, W, np, torch) -> int:
    """Config 5: Llama-3-8B-shaped stack (hidden 4096, FFN 14336, 32/8 heads) over a 32768-token
    context; partial prefill at the given ratio with per-layer KV streamed from pinned host
    memory, against full prefill (r = 100 %, same kernels, nothing copied) on the same GPU.
    Weights and caches are random (torch generator, seed 1005) - created on the device because
    14 GB of weights would take minutes to draw on the host."""
    sp = W.spec(5, args.ratio)
    sh = sp.shape
    n_layers, ffn = args.layers, 14336
    cfg = B.cfg_from_shape(sh)
    g = torch.Generator(device="cuda").manual_seed(1005)
    E, qd, Hkv, D, N = sh.hidden, sh.n_q_heads * sh.head_dim, sh.n_kv_heads, sh.head_dim, sp.n_ctx

    def rnd(shape, scale):
        return (torch.randn(shape, generator=g, device="cuda", dtype=torch.float32) * scale).to(torch.bfloat16)

    log(f"creating {n_layers} layers of weights and {n_layers} x 128 MiB of pinned-host KV")
    ones = torch.ones(E, dtype=torch.bfloat16, device="cuda")
    weights, pools = [], []
    for _ in range(n_layers):
        weights.append(dict(attn_norm=ones, wqkv=rnd((sh.qkv_width, E), E ** -0.5), wo=rnd((E, qd), qd ** -0.5),
                            ffn_norm=ones, w_gate=rnd((ffn, E), E ** -0.5), w_up=rnd((ffn, E), E ** -0.5),
                            w_down=rnd((E, ffn), ffn ** -0.5)))
        if args.kv_pool in ("pinned", "compact"):
            kp = torch.empty((N, Hkv, D), dtype=torch.bfloat16, pin_memory=True)
            vp = torch.empty((N, Hkv, D), dtype=torch.bfloat16, pin_memory=True)
            kp.copy_(rnd((N, Hkv, D), 1.0))
            vp.copy_(rnd((N, Hkv, D), 1.0))
        else:
            kp, vp = rnd((N, Hkv, D), 1.0), rnd((N, Hkv, D), 1.0)
        pools.append((kp, vp))
    torch.cuda.synchronize()

    dev_pools = []

    def run(r, steps, warmup, kv_pool=args.kv_pool):
        """Mean latency of the stack at recompute ratio r (a fraction; floor(r N) rows)."""
        n_sel = N if r >= 1.0 else max(1, int(math.floor(r * N + 1e-9)))
        sel_np = W.select_indices(sp, n_sel)
        sel = torch.from_numpy(sel_np).cuda()
        entries, keep = [], []
        compact = kv_pool == "compact" and r < 1.0
        if kv_pool == "device" and args.kv_pool != "device" and not dev_pools:
            dev_pools.extend((kp.cuda(), vp.cuda()) for kp, vp in pools)
        use_pools = dev_pools if (kv_pool == "device" and args.kv_pool != "device") else pools
        if compact:   # per chunk: the rows that are not recomputed, gathered into a pool of their own
            kept = [torch.from_numpy(np.setdiff1d(np.arange(c * sp.chunk_len, (c + 1) * sp.chunk_len), sel_np))
                    for c in range(sp.n_chunks)]
        for lw, (kp, vp) in zip(weights, use_pools):
            if compact:
                parts = []
                for c in range(sp.n_chunks):
                    kc = torch.empty((len(kept[c]), Hkv, D), dtype=torch.bfloat16, pin_memory=True)
                    vc = torch.empty_like(kc).pin_memory()
                    kc.copy_(kp[kept[c]])
                    vc.copy_(vp[kept[c]])
                    parts.append((kc, vc))
                keep.append(parts)
                ch = B.make_chunks([dict(k=parts[c][0], v=parts[c][1], n_tokens=sp.chunk_len, old_pos_start=0,
                                         new_pos_start=c * sp.chunk_len, location=2) for c in range(sp.n_chunks)])
                keep.append(ch)
                d = dict(lw)
                d["chunks"] = ch
                entries.append(d)
                continue
            ch = B.make_chunks([dict(k=kp[c * sp.chunk_len:(c + 1) * sp.chunk_len], v=vp[c * sp.chunk_len:(c + 1) * sp.chunk_len],
                                     n_tokens=sp.chunk_len, old_pos_start=0, new_pos_start=c * sp.chunk_len,
                                     location=0 if kv_pool == "device" else 1)
                                for c in range(sp.n_chunks)])
            keep.append(ch)
            d = dict(lw)
            d["chunks"] = ch
            entries.append(d)
        layers = B.make_layers(entries)
        ws_bytes = B.ct_stack_workspace_bytes(cfg, ffn, N, n_sel)
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
        k_bufs = torch.zeros((2, N, Hkv, D), dtype=torch.bfloat16, device="cuda")
        v_bufs = torch.zeros_like(k_bufs)
        h0 = rnd((n_sel, E), 1.0)
        h = torch.empty_like(h0)
        s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()

        def step():
            h.copy_(h0)
            torch.cuda.current_stream().synchronize()
            B.ct_partial_prefill_stack(cfg, ffn, 1e-5, layers, n_layers, sp.n_chunks, h, sel, n_sel, min(r, 1.0),
                                       k_bufs, v_bufs, ws, ws_bytes, s1, s2)
        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        B.ct_profile_reset()
        B.ct_set_profiling(not args.no_profile_events)
        t0 = time.perf_counter()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        B.ct_set_profiling(False)
        kern = {}
        for name in B.KERNEL_CLASSES:
            cnt, kms = B.ct_profile_read(name)
            if cnt:
                kern[name] = {"launches_per_layer": cnt / steps / n_layers, "ms_per_layer": kms / steps / n_layers}
        B.ct_profile_reset()
        assert torch.isfinite(h.float()).all()
        return ms, n_sel, kern

    tuning = None
    ratio = sp.ratio_pct / 100.0
    if args.tune_ratio:
        # Sec. 4.3 on this machine.  Hardware profile: t_c and t_o from the compute-only stack
        # (device-resident pool) at two ratios, t_i from the transfer-dominated stack (this pool, 2 %);
        # then Alg. 1 over the measured latency of the stack, warm-started at the prior of Eq. 11.
        r_a, r_b, r_s = 0.15, 0.30, 0.02
        la = run(r_a, args.steps, 1, "device")[0] / n_layers
        lb = run(r_b, args.steps, 1, "device")[0] / n_layers
        t_c = (lb - la) / ((r_b - r_a) * N)
        t_o = la - r_a * N * t_c
        if args.kv_pool == "device":
            t_i = 0.0
        else:
            ls = run(r_s, args.steps, 1)[0] / n_layers
            t_i = max(0.0, (ls - t_o) / ((1.0 - r_s) * N))
        r0_raw = t_i / (t_c + t_i)
        r0 = B.ct_ratio_prior(t_c, t_i, args.r_min, args.r_max)
        log(f"profile: t_c {t_c * 1e6:.1f} ns/token/layer, t_i {t_i * 1e6:.1f} ns/token/layer, t_o {t_o * 1e3:.1f} us/layer; "
            f"crossover {r0_raw:.4f}, prior r0 {r0:.4f}")
        probes = []

        def ttft(r):
            ms = run(r, args.steps, 1)[0]
            probes.append({"r": r, "ms": ms, "model_ms": n_layers * B.ct_layer_latency_model(r, N, t_c, t_i, t_o)})
            log(f"  probe r={r:.4f}: {ms:.2f} ms (model {probes[-1]['model_ms']:.2f})")
            return ms
        r_star, n_evals = B.ct_ratio_search(ttft, r0, args.r_min, args.r_max, args.eps, 32)
        log(f"r* = {r_star:.4f} after {n_evals} evaluations")
        tuning = {"t_c_ns_per_token_layer": t_c * 1e6, "t_i_ns_per_token_layer": t_i * 1e6, "t_o_us_per_layer": t_o * 1e3,
                  "profile_points": {"device_pool_ms_per_layer": {str(r_a): la, str(r_b): lb},
                                     "this_pool_ms_per_layer": None if args.kv_pool == "device" else {str(r_s): ls}},
                  "crossover_unclipped": r0_raw, "r0": r0, "r_min": args.r_min, "r_max": args.r_max, "eps": args.eps,
                  "n_evals": n_evals, "r_star": r_star, "probes": probes,
                  "calibration_set": f"{args.steps} seeded synthetic steps per probe"}
        ratio = r_star
    rtxt = f"{ratio * 100:.1f}%" if args.tune_ratio else f"{sp.ratio_pct}%"
    log(f"partial prefill r={rtxt}")
    ms_part, n_sel, kern_part = run(ratio, args.steps, args.warmup)
    log("full prefill (r=100%)")
    ms_full, _, kern_full = run(1.0, max(1, args.steps // 4), 1)

    cpu = None
    if not args.no_cpu_baseline:
        # the oracle on layer 0 of the same stack: projections, re-RoPE and scatter in full, attention
        # and the row-wise rest of the layer on a sample of rows; scaled to all rows and all layers
        log("timing the CPU oracle on one layer (sampled rows)")
        from threadpoolctl import threadpool_info
        from oracle import ct_oracle as O

        def f64(t):
            return W.bf16_bits_to_f64(t.cpu().view(torch.int16).numpy().view(np.uint16))
        lw = {k: f64(v) for k, v in weights[0].items()}
        kc, vc = f64(pools[0][0]), f64(pools[0][1])
        sel_np = W.select_indices(sp, n_sel)
        h0 = np.random.default_rng(1005).standard_normal((n_sel, E))
        rows = W.sample_rows(n_sel, args.cpu_sample_rows if args.cpu_sample_rows > 0 else 96, seed=1005)
        old_pos = (np.arange(N) % sp.chunk_len).astype(np.int32)         # keys cached at chunk-local positions
        new_pos = np.arange(N, dtype=np.int32)
        t0 = time.perf_counter()
        x = O.rmsnorm(h0, lw["attn_norm"], 1e-5)
        q, k_new, v_new = O.qkv_selected(x, lw["wqkv"], None, new_pos[sel_np], sh.n_q_heads, sh.n_kv_heads, D,
                                         sh.rope_theta, sh.rope_style)
        k_rot = O.rerope_keys(kc, old_pos, new_pos, sh.rope_theta, sh.rope_style)
        kf, vf = O.scatter_kv(k_rot, vc, k_new, v_new, sel_np)
        t_full_parts = time.perf_counter() - t0
        t0 = time.perf_counter()
        attn, _ = O.selected_attention(q, kf, vf, sel_np, rows=rows)
        t_attn = time.perf_counter() - t0
        t0 = time.perf_counter()
        O.layer_tail(h0[rows], attn, lw["wo"], lw["ffn_norm"], lw["w_gate"], lw["w_up"], lw["w_down"], 1e-5)
        t_tail = time.perf_counter() - t0
        vis_all = int((sel_np.astype(np.int64) + 1).sum())
        vis_s = int((sel_np[rows].astype(np.int64) + 1).sum())
        per_layer = t_full_parts + t_attn * vis_all / vis_s + t_tail * n_sel / len(rows)
        threads = max([d.get("num_threads", 1) for d in threadpool_info()] + [1])
        cpu = {"value": per_layer * n_layers * 1e3, "unit": "ms", "cores": threads, "kind": "oracle",
               "sample": f"fp64 NumPy oracle on layer 0: RMSNorm, QKV projection, re-RoPE, scatter in full "
                         f"({t_full_parts:.2f}s); attention on {len(rows)} of {n_sel} rows ({t_attn:.2f}s, scaled by "
                         f"visible keys x{vis_all / vis_s:.1f}); output projection and FFN on the same rows "
                         f"({t_tail:.2f}s, scaled x{n_sel / len(rows):.1f}); times {n_layers} layers (extrapolated)"}
    line = {
        "metric": f"end-to-end partial prefill latency, {n_layers}-layer stack @{N // 1024}K ctx, r={rtxt}"
                  f"{' (tuned)' if args.tune_ratio else ''} (vs full prefill)",
        "value": ms_part, "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_part, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": sp.name, "layers": n_layers, "n_ctx": N, "n_sel": n_sel, "ffn_dim": ffn,
                   "kv_pool": {"pinned": "pinned host, streamed one layer ahead on a second stream",
                               "compact": "pinned host holding only the rows that are not recomputed, streamed one layer ahead",
                               "device": "device-resident"}[args.kv_pool]},
        "extra": {"full_prefill_ms": ms_full, "speedup_vs_full_prefill": ms_full / ms_part,
                  "ms_per_layer_partial": ms_part / n_layers, "ms_per_layer_full": ms_full / n_layers,
                  "host_to_device_bytes_per_layer": 0 if args.kv_pool == "device" else 2 * (N - n_sel) * Hkv * D * 2,
                  "kernels_partial": kern_part, "kernels_full": kern_full, "ratio_tuning": tuning},
        "cpu_baseline": cpu,
    }
    print(json.dumps(line), flush=True)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=3, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--layers", type=int, default=32, help="config 5 only: number of layers")
    ap.add_argument("--kv-pool", choices=["pinned", "compact", "device"], default="pinned",
                    help="config 5 only: where the per-layer cached K/V live (pinned host memory is the paper's CPU pool; "
                         "compact = pinned, holding only the rows that are not recomputed)")
    ap.add_argument("--ratio", type=int, default=None,
                    help="recompute ratio in percent (default: 15, and 5 for config 4, as the workloads are defined)")
    ap.add_argument("--offline-select", action="store_true",
                    help="time the offline frequency-guided selection (scores + TopK) instead of the online path")
    ap.add_argument("--tune-ratio", action="store_true",
                    help="config 5 only: profile t_c, t_i, t_o and search the ratio with the least measured latency")
    ap.add_argument("--r-min", type=float, default=0.15)
    ap.add_argument("--r-max", type=float, default=0.60)
    ap.add_argument("--eps", type=float, default=0.01)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-rows", type=int, default=-1,
                    help="selected rows the CPU oracle's attention is timed on (0 = all; default: all rows up to the "
                         "headline point's work, 96 rows beyond it)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="run one plain 512 MiB device copy before the timed region (reference for HBM byte counters)")
    ap.add_argument("--no-cold-cache", action="store_true",
                    help="skip the stand-alone re-RoPE / scatter bandwidth runs (outside the timed region)")
    ap.add_argument("--no-profile-events", action="store_true",
                    help="do not bracket kernels with HIP events inside the timed region")
    args = ap.parse_args()
    if args.ratio is None:
        args.ratio = 5 if args.config == 4 else 15
    if args.steps is None:
        args.steps = 4 if args.config == 5 else 50
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2605_24022_amd import binding as B
    from paper_2605_24022_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    B.load()

    if args.offline_select:
        return bench_offline(args, B, W, np, torch)
    if args.config == 5:
        return bench_stack(args, B, W, np, torch)

    sp = W.spec(args.config, args.ratio)
    sh = sp.shape
    log(f"generating {sp.name}: n_ctx={sp.n_ctx} n_sel={sp.n_sel}")
    wl = W.make_workload(sp)
    cfg = B.cfg_from_shape(sh)

    def dev(bits):
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)

    hidden, wqkv = dev(wl.hidden), dev(wl.wqkv)
    rows = None if wl.hidden_rows is None else torch.from_numpy(wl.hidden_rows).cuda()
    sel = torch.from_numpy(wl.sel_idx).cuda()
    host_pool = args.config == 4      # config 4 keeps the cached K/V in pinned host memory
    if host_pool:
        def pin(bits):
            t = torch.empty(bits.shape, dtype=torch.int16, pin_memory=True)
            t.copy_(torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)))
            return t.view(torch.bfloat16)
        k_pool, v_pool = pin(wl.k_cache), pin(wl.v_cache)
    else:
        k_pool, v_pool = dev(wl.k_cache), dev(wl.v_cache)
    k_buf = torch.zeros(k_pool.shape, dtype=torch.bfloat16, device="cuda")
    v_buf = torch.zeros_like(k_buf)
    chunks = B.make_chunks([
        dict(k=k_pool[int(wl.chunk_rows[c]):int(wl.chunk_rows[c + 1])],
             v=v_pool[int(wl.chunk_rows[c]):int(wl.chunk_rows[c + 1])],
             n_tokens=int(wl.chunk_rows[c + 1] - wl.chunk_rows[c]), old_pos_start=int(wl.chunk_old_start[c]),
             new_pos_start=int(wl.chunk_new_start[c]), location=1 if host_pool else 0) for c in range(sp.n_chunks)])
    ws_bytes = B.ct_workspace_bytes(cfg, sp.n_ctx, sp.n_sel)
    if host_pool:   # room for the attention state: the launches follow the chunk groups key range by key range
        ws_bytes += B.ct_attention_state_bytes(cfg, sp.n_ctx, sp.n_sel)
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device="cuda")
    out = torch.zeros((sp.n_sel, sh.n_q_heads, sh.head_dim), dtype=torch.bfloat16, device="cuda")
    compute, copy = torch.cuda.Stream(), torch.cuda.Stream()
    ratio = sp.ratio_pct / 100.0

    def step():
        B.ct_partial_prefill_layer(cfg, chunks, sp.n_chunks, hidden, rows, sel, sp.n_sel, ratio, wqkv, None,
                                   k_buf, v_buf, out, ws, ws_bytes, compute, copy)

    if args.calibration_copy:
        src = torch.empty(512 << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)          # reads 512 MiB, writes 512 MiB
        torch.cuda.synchronize()
        del src, dst
    log(f"warmup {args.warmup}, timing {args.steps} steps")
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # the headline: K steps back to back, nothing but the library's own launches in the streams
    B.ct_set_profiling(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps

    # second pass of the same K steps for the per-kernel split: a pair of HIP events rides on every
    # kernel dispatch (begin and end of that kernel on its launch stream)
    profile = not args.no_profile_events
    kern = {}
    ms_per_step_profiled = None
    if profile:
        B.ct_profile_reset()
        B.ct_set_profiling(True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        ms_per_step_profiled = (time.perf_counter() - t0) * 1e3 / args.steps
        B.ct_set_profiling(False)
        for name in B.KERNEL_CLASSES:
            n, ms = B.ct_profile_read(name)
            if n:
                kern[name] = {"launches_per_step": n / args.steps, "avg_ms": ms / n, "ms_per_step": ms / args.steps}
    B.ct_profile_reset()

    # algorithmic work of one step
    D, Hq, Hkv, E, O_w = sh.head_dim, sh.n_q_heads, sh.n_kv_heads, sh.hidden, sh.qkv_width
    n, N = sp.n_sel, sp.n_ctx
    vis = int((wl.sel_idx.astype(np.int64) + 1).sum())
    attn_flops = 4.0 * D * Hq * vis
    qkv_flops = 2.0 * n * E * O_w
    rerope_bytes = 2.0 * (N - n) * Hkv * D * 2 + 8.0 * (N - n)      # rows that must be rotated: read + write
    scatter_bytes = 2.0 * 2.0 * n * Hkv * D * 2 + 4.0 * n

    # spread of single steps: each of up to 30 further steps between its own pair of events on the
    # launch stream (profiling events off)
    pairs = []
    for _ in range(min(args.steps, 30)):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(compute)
        step()
        e1.record(compute)
        pairs.append((e0, e1))
    torch.cuda.synchronize()
    single = sorted(a.elapsed_time(b) for a, b in pairs)

    extra = {"n_ctx": N, "n_sel": n, "visible_keys": vis, "kernels": kern,
             "ms_per_step_with_kernel_events": ms_per_step_profiled,
             "step_ms_median": single[len(single) // 2], "step_ms_min": single[0]}
    roofline = None
    if "attention" in kern:
        t_attn = (kern["attention"]["ms_per_step"] + kern.get("merge", {}).get("ms_per_step", 0.0)) * 1e-3
        ach = attn_flops / t_attn / 1e12
        # what a kernel of nothing but MFMAs sustains on this device over ~20 ms (power-limited below the peak)
        ceiling = B.ct_measure_mfma_rate(torch.empty(1 << 20, dtype=torch.uint8, device="cuda"), 20000, compute)
        roofline = {"bound": "mfma", "kernel": "selected attention (+ split merge)", "achieved": ach,
                    "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": ach / PEAK_BF16_TFLOPS,
                    "measured_mfma_only_rate": ceiling, "frac_of_measured_rate": ach / ceiling,
                    "traffic": attention_traffic(sp.name)[0],
                    "traffic_unit": "bytes per launch (HBM fetch + write)",
                    "traffic_source": attention_traffic(sp.name)[1],
                    "algorithmic_bytes_per_launch": 2.0 * n * Hq * D * 2 + 2.0 * N * Hkv * D * 2,
                    "algorithmic_flops_per_launch": attn_flops}
        extra["sel_attn_tflops"] = ach
    if "qkv" in kern:
        extra["qkv_tflops"] = qkv_flops / (kern["qkv"]["ms_per_step"] * 1e-3) / 1e12
    if "rerope" in kern:
        gbs = rerope_bytes / (kern["rerope"]["ms_per_step"] * 1e-3) / 1e9
        extra["rerope_gbs_algorithmic"] = gbs
        extra["rerope_frac_of_hbm_peak"] = gbs / PEAK_HBM_GBS
        # the same launch also copies the reused values pool -> buffer: bytes it really moves
        moved = 4.0 * N * Hkv * D * 2
        extra["rerope_plus_vcopy_gbs_moved"] = moved / (kern["rerope"]["ms_per_step"] * 1e-3) / 1e9
    if "scatter" in kern:
        extra["scatter_gbs"] = scatter_bytes / (kern["scatter"]["ms_per_step"] * 1e-3) / 1e9

    if host_pool:
        extra["host_to_device_bytes_per_step"] = 4 * N * Hkv * D
        extra["host_link_gbs_if_transfer_bound"] = 4.0 * N * Hkv * D / (ms_per_step * 1e-3) / 1e9
    if not args.no_cold_cache and not host_pool:
        extra["cold_cache"] = cold_cache_bandwidth(B, cfg, wl, sp, torch, np)

    cpu = None
    if not args.no_cpu_baseline:
        log("timing the CPU oracle on a bounded sample")
        from oracle import ct_oracle as O
        # configs 1, 2 and config 3 up to r = 15 %: the whole oracle, nothing extrapolated (about 40 s at the
        # headline point); beyond that the attention is timed on a sample of rows
        whole = args.cpu_sample_rows == 0 or (args.cpu_sample_rows < 0 and attn_flops <= 1.4e12)
        cpu = cpu_baseline(wl, 0 if whole else (args.cpu_sample_rows if args.cpu_sample_rows > 0 else 96), O, W, np)

    line = {
        "metric": f"ms/layer partial prefill @{N // 1024}K ctx, r={sp.ratio_pct}% (sel-attn TFLOP/s and re-RoPE GB/s in extra)",
        "value": ms_per_step, "unit": "ms/layer", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": sp.name, "n_ctx": N, "n_chunks": sp.n_chunks, "chunk_len": sp.chunk_len,
                   "recompute_ratio": ratio, "n_sel": n, "hidden": E, "heads": f"{Hq}/{Hkv}", "head_dim": D,
                   "kv_pool": "pinned host memory, streamed in and rotated by a kernel on a second stream each step"
                   if host_pool else "device-resident, rotated + copied into the layer buffers each step"},
        "roofline": roofline, "cpu_baseline": cpu, "extra": extra,
    }
    print(json.dumps(line), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
