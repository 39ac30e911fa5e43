#!/usr/bin/env python3
"""Benchmark of the pruned multimodal encoder forward on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C5] [--no-cpu] [--no-extras] [--moe-only]

One "step" is one pass of the whole hot path over one batch of seeded synthetic
input already resident in HBM: gate scores -> keep masks, compaction of the
weights, and the encoder forward (LayerNorm, Q/K/V projection, sparse GQA,
output projection, pruned FFN) of every layer.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "encoder tokens/sec + sparse-GQA TFLOP/s (% of bf16 MFMA peak), 1 MI355X"
PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published
PEAK_HBM_GBS = 8000.0

# kernel behind each of the five GEMM launches of a layer (large shapes; small ones fall back, see gemm_bf16.hip)
GEMM_KERNEL_NAMES = {
    "qkv_proj": "gemm_bf16_ws_kernel<0> (Q/K/V projection, V as the transposed column range)",
    "qk_proj": "gemm_bf16_ws_kernel<0> (Q/K projection)",
    "v_proj": "gemm_bf16_fast_kernel<..., true, 0> (V projection, transposed output)",
    "o_proj": "gemm_bf16_ws_kernel<0> (output projection + residual), or gemm_bf16_fast_kernel on the active rows only",
    "ffn_up": "gemm_bf16_ws_kernel<1> (FFN up-projection + ReLU)",
    "ffn_down": "gemm_bf16_ws_kernel<0> (FFN down-projection + residual)",
}
# HBM-side bytes per launch of the GEMM launches come from the rocprofv3 --pmc summary under profiles/ (FETCH_SIZE /
# WRITE_SIZE, two runs, scaled by the same counters' reading of a plain device copy).  The summary carries a line
#   traffic_bytes_per_launch: {"workload": "C5", "kernel_source_digest": "...", "ffn_up": ..., ...}
# and the figure is used only while the digest of the kernel sources still matches (else `traffic` is null: the
# counters have to be collected again).
TRAFFIC_SUMMARY = os.path.join(ROOT, "profiles", "encoder_C5_hbm_traffic.txt")


def kernel_source_digest():
    """sha256 over the HIP sources and the public header (what the measured traffic depends on)."""
    import glob
    import hashlib
    h = hashlib.sha256()
    files = sorted(glob.glob(os.path.join(ROOT, "paper_2604_08971_amd", "csrc", "*")) +
                   glob.glob(os.path.join(ROOT, "include", "*.h")))
    for f in files:
        h.update(os.path.basename(f).encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()[:16]


def measured_traffic(workload, launch):
    try:
        for line in open(TRAFFIC_SUMMARY):
            if line.startswith("traffic_bytes_per_launch:"):
                rec = json.loads(line.split(":", 1)[1])
                if rec.get("workload") == workload and rec.get("kernel_source_digest") == kernel_source_digest():
                    return rec.get(launch)
    except (OSError, ValueError):
        pass
    return None


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def key_valid_host(dm):
    from paper_2604_08971_amd.device_model import key_valid_host as f
    return f(dm)


def n_allowed_keys(wl, key_valid):
    """Allowed keys per sample from the device's key mask (host copy, or None = every position)."""
    import numpy as np
    B, L = wl.x.shape[0], wl.spec.L
    return np.full(B, L) if key_valid is None else key_valid.sum(axis=1).astype(np.int64)


def algorithmic_flops(wl, masks_host, U, oproj_rows=None, key_valid=None):
    """Flops credited per step: kept heads / kept groups / kept channels only, no padding.  oproj_rows[l]: rows
    per sample that go through the output projection of layer l when the library projects the active rows only
    (the distinct rows that are active in some head, counted from the selection; None: every row)."""
    import numpy as np
    s = wl.spec
    B, L, d, dh = wl.x.shape[0], s.L, s.d, s.dh
    n_allowed = n_allowed_keys(wl, key_valid)
    gemm = score = active = 0
    for l in range(s.n_layers):
        kh, kf = int(wl.k_head[l]), int(wl.k_ffn[l])
        ng = masks_host["n_groups"][l][wl.pattern_id].astype(np.int64)          # per sample
        gemm += int((2 * L * d * dh * (kh + 2 * ng)).sum())                     # Q, K, V projections
        rows_o = B * L if oproj_rows is None or oproj_rows[l] is None else int(oproj_rows[l].sum()) + B
        gemm += 2 * rows_o * kh * dh * d                                        # output projection (+ one context row per sample)
        gemm += B * 4 * L * d * kf                                              # both FFN GEMMs
        if 0 < U < L:
            score += int((kh * 2 * n_allowed * n_allowed * dh).sum())           # QK^T stream of the sparsity score
        active += int((kh * 4 * np.minimum(U, n_allowed) * n_allowed * dh).sum())   # QK^T + PV of the active rows
    return {"gemm": gemm, "score": score, "active": active, "total": gemm + score + active}


def gemm_flops_by_launch(wl, masks_host, oproj_rows=None):
    """Algorithmic flops of the five GEMM launches of a layer, summed over layers."""
    import numpy as np
    s = wl.spec
    B, L, d, dh = wl.x.shape[0], s.L, s.d, s.dh
    out = {"qk_proj": 0, "v_proj": 0, "o_proj": 0, "ffn_up": 0, "ffn_down": 0}
    for l in range(s.n_layers):
        kh, kf = int(wl.k_head[l]), int(wl.k_ffn[l])
        ng = masks_host["n_groups"][l][wl.pattern_id].astype(np.int64)
        out["qk_proj"] += int((2 * L * d * dh * (kh + ng)).sum())
        out["v_proj"] += int((2 * L * d * dh * ng).sum())
        rows_o = B * L if oproj_rows is None or oproj_rows[l] is None else int(oproj_rows[l].sum())
        out["o_proj"] += 2 * rows_o * kh * dh * d
        out["ffn_up"] += B * 2 * L * d * kf
        out["ffn_down"] += B * 2 * L * d * kf
    return out


def time_steps(fn, steps, warmup):
    """W untimed calls, then exactly K calls between two events (and two synchronisations).  The launches are
    issued from Python, so the collector is held off during the timed region (a collection pause would idle
    the GPU on the small workloads, whose steps are launch-bound)."""
    import gc
    import torch
    # the collection runs before the warm-up: between the synchronisation and the first timed launch the GPU must not
    # sit idle for the tens of milliseconds a collection takes (its clocks fall back and the first timed steps pay
    # for the ramp: 1.8 ms per timed region measured, 9 % of 20 steps)
    gc.collect()
    gc_was = gc.isenabled()
    gc.disable()
    try:
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        ev0.record()
        for _ in range(steps):
            fn()
        ev1.record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e3 / steps
    finally:
        if gc_was:
            gc.enable()
    return ev0.elapsed_time(ev1) / steps, wall


def bench_config(name, steps, warmup, extras, cpu, use_graph=False, repeats=1):
    import numpy as np
    import torch
    from paper_2604_08971_amd import binding as sf
    from paper_2604_08971_amd import workloads as W
    from paper_2604_08971_amd.device_model import DeviceModel, to_host

    spec = W.CONFIGS[name]
    t0 = time.perf_counter()
    wl = W.make_workload(spec)
    dm = DeviceModel(wl).build_plan()
    torch.cuda.synchronize()
    log(f"[{name}] inputs generated and uploaded in {time.perf_counter() - t0:.1f} s")
    s = spec
    B, L = wl.x.shape[0], s.L
    U = sf.num_active(dm.desc)
    y = torch.empty_like(dm.x)
    masks_host = {k: to_host(v) for k, v in dm.masks.items()}
    # layers whose output projection runs on the active rows only: count those rows from one forward's selection
    oproj_rows = [None] * s.n_layers
    if any(sf.active_projection_rows(dm.desc, int(k)) > 0 for k in wl.k_head):
        _, sel, _ = dm.forward(want_sel=True)
        sel_h = to_host(sel)
        for l in range(s.n_layers):
            if sf.active_projection_rows(dm.desc, int(wl.k_head[l])) > 0:
                oproj_rows[l] = np.array([len(np.unique(sel_h[l, b][sel_h[l, b] >= 0])) for b in range(B)])
    flops = algorithmic_flops(wl, masks_host, U, oproj_rows, key_valid_host(dm))

    def step():                       # the whole hot path
        dm.build_plan()
        dm.forward(out=y)

    # Optionally the step's launches (about 20 per layer) are recorded once into a HIP graph and replayed: same
    # kernels, same arguments, same stream order.
    launch = "eager"
    run = step
    if use_graph:
        try:
            step()                                        # first call sizes the workspace and sets kernel attributes
            torch.cuda.synchronize()
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                step()
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                step()
            torch.cuda.synchronize()
            y_ref = y.clone()
            y.zero_()
            graph.replay()
            torch.cuda.synchronize()
            if not torch.equal(y, y_ref):
                raise RuntimeError("graph replay differs from the eager step")
            run, launch = graph.replay, "hipGraph"
        except Exception as e:                            # noqa: BLE001 - any capture problem falls back to eager launches
            log(f"[{name}] graph capture not used: {e}")
            torch.cuda.synchronize()
            run, launch = step, "eager"

    ms, wall_ms = time_steps(run, steps, warmup)
    if repeats > 1:
        # context figures (the other workloads): median of `repeats` timings of K steps each
        runs = sorted([(ms, wall_ms)] + [time_steps(run, steps, 1) for _ in range(repeats - 1)])
        ms, wall_ms = runs[len(runs) // 2]
    res = {"workload": name, "ms_per_step": ms, "host_ms_per_step": wall_ms, "tokens_per_s": B * L / (ms * 1e-3),
           "B": B, "L": L, "U": U, "algorithmic_tflop_per_step": flops["total"] / 1e12,
           "tflops_total": flops["total"] / (ms * 1e-3) / 1e12, "launch": launch}
    if launch != "eager":
        ms_eager, _ = time_steps(step, steps, 2)
        res["ms_per_step_eager"] = ms_eager
    if not extras:
        return res, dm, wl, flops

    ms_fwd, _ = time_steps(lambda: dm.forward(out=y), steps, 2)
    ms_plan, _ = time_steps(lambda: dm.build_plan(), steps, 2)
    res.update({"ms_encoder_only": ms_fwd, "ms_plan_only": ms_plan,
                "tokens_per_s_encoder_only": B * L / (ms_fwd * 1e-3)})

    # per-kernel-class timing with HIP events on the launch stream (second pass of the same steps)
    prof = {}
    if s.dtype == "bf16":
        for cls, key in ((sf.SF_KERNEL_GEMM, "gemm"), (sf.SF_KERNEL_SCORE, "score"), (sf.SF_KERNEL_ATTEND, "active")):
            sf.profile_begin(cls, steps * 64 * s.n_layers)
            for _ in range(steps):
                step()
            n, tot_ms, each = sf.profile_end(each=True)
            if n:
                prof[key] = {"launches_per_step": n / steps, "avg_launch_us": tot_ms * 1e3 / n,
                             "ms_per_step": tot_ms / steps,
                             "tflops": flops[key] * steps / (tot_ms * 1e-3) / 1e12 if tot_ms > 0 else None}
                prof[key]["frac_of_bf16_peak"] = prof[key]["tflops"] / PEAK_BF16_TFLOPS if prof[key]["tflops"] else None
                if key == "active" and tot_ms > 0:
                    # the bound that matters for the sparse pattern: K and V of every referenced (sample, group) once
                    kv_bytes = sum(int(masks_host["n_groups"][l][wl.pattern_id].astype(np.int64).sum()) * 2 * L * s.dh * 2
                                   for l in range(s.n_layers))
                    prof[key]["kv_algorithmic_bytes_per_step"] = kv_bytes
                    prof[key]["kv_GBs"] = kv_bytes * steps / (tot_ms * 1e-3) / 1e9
                    prof[key]["kv_frac_of_hbm_peak"] = prof[key]["kv_GBs"] / PEAK_HBM_GBS
            if key == "gemm" and n and n % steps == 0 and n // steps in (4 * s.n_layers, 5 * s.n_layers):
                # the GEMM launches of a layer, in launch order, averaged over steps and layers: four when the
                # Q/K/V projection is one launch (large shapes), five when V is projected separately
                per = n // steps
                nper = per // s.n_layers
                names = (["qkv_proj"] if nper == 4 else ["qk_proj", "v_proj"]) + ["o_proj", "ffn_up", "ffn_down"]
                fl = gemm_flops_by_launch(wl, masks_host, oproj_rows)
                fl["qkv_proj"] = fl["qk_proj"] + fl["v_proj"]
                by = {}
                for j, nm in enumerate(names):
                    d = [each[i] for i in range(n) if (i % per) % nper == j]
                    us = sum(d) * 1e3 / len(d)
                    by[nm] = {"avg_launch_us": us, "launches_per_step": len(d) / steps,
                              "tflops": fl[nm] / s.n_layers / (us * 1e-6) / 1e12}
                prof["gemm"]["by_launch"] = by
    res["kernels"] = prof
    if any(r is not None for r in oproj_rows):
        res["active_row_projection"] = {
            "layers": [l for l in range(s.n_layers) if oproj_rows[l] is not None],
            "rows_projected_per_sample_mean": float(np.mean([r.mean() for r in oproj_rows if r is not None])),
            "rows_per_sample": L,
            "note": "output projection on the rows that are active in some head; the other rows of a sample take the "
                    "projection of its context vectors (computed once); flops are credited for the projected rows only"}
    return res, dm, wl, flops


def bench_ceilings(seconds=0.6):
    """What this machine reaches, measured in this run: a register-only bf16 MFMA loop (constant operands, and rotating
    pseudo-random operands whose switching activity lowers the sustained clock under the power cap) and a plain
    device copy.  Each is run for about `seconds` first, so the clocks have settled, then timed."""
    import torch
    from paper_2604_08971_amd import binding as sf
    out = {}
    sink = torch.zeros(4096, dtype=torch.float32, device="cuda")
    wgs, iters = 1024, 2000
    for tag, rnd in (("mfma_bf16_constant_operands", False), ("mfma_bf16_random_operands", True)):
        fl = sf.ceiling_mfma_launch(wgs, iters, rnd, sink)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(); sf.ceiling_mfma_launch(wgs, iters, rnd, sink); e1.record(); torch.cuda.synchronize()
        n = max(3, int(seconds * 1e3 / max(e0.elapsed_time(e1), 1e-3)))
        for _ in range(n):
            sf.ceiling_mfma_launch(wgs, iters, rnd, sink)
        e0.record()
        for _ in range(n):
            sf.ceiling_mfma_launch(wgs, iters, rnd, sink)
        e1.record(); torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / n
        out[tag] = {"tflops": fl / (ms * 1e-3) / 1e12, "frac_of_published": fl / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}
    nbytes = 1 << 30
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda").random_(0, 255)
    dst = torch.empty_like(src)
    sf.ceiling_copy_launch(src, dst); torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    n = 40
    for _ in range(n):
        sf.ceiling_copy_launch(src, dst)
    e0.record()
    for _ in range(n):
        sf.ceiling_copy_launch(src, dst)
    e1.record(); torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / n
    out["hbm_copy"] = {"GBs_read_plus_write": 2 * nbytes / (ms * 1e-3) / 1e9,
                       "frac_of_published": 2 * nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, "bytes_each_way": nbytes}
    out["note"] = ("measured in this run on this box with sf_ceiling_mfma_launch / sf_ceiling_copy_launch; the "
                   "published peaks (2.5 PFLOP/s bf16, 8 TB/s) stay the denominators of every `frac`")
    del src, dst
    torch.cuda.empty_cache()
    return out


def bench_sparse_gqa(dm, wl, steps):
    """sparse_gqa_forward alone, at the workload's kept shapes, c-sparse and dense pattern."""
    import numpy as np
    import torch
    from paper_2604_08971_amd import binding as sf
    s = wl.spec
    if s.dtype != "bf16":
        return None
    B, L, dh, kh = wl.x.shape[0], s.L, s.dh, int(wl.k_head[0])
    g = torch.Generator(device="cuda").manual_seed(1)
    Q = torch.randn((B, kh, L, dh), generator=g, device="cuda").to(torch.bfloat16)
    K = torch.randn((B, s.Hk, L, dh), generator=g, device="cuda").to(torch.bfloat16)
    V = torch.randn((B, s.Hk, L, dh), generator=g, device="cuda").to(torch.bfloat16)
    hg = dm.masks["head_group"][0][:, :kh].contiguous()
    n_allowed = n_allowed_keys(wl, key_valid_host(dm))
    out = {}
    for tag, Uo in (("c5", -1), ("dense", L)):
        desc = sf.make_desc(B, L, s.d, s.Hq, s.Hk, dh, s.F, dtype=sf.SF_BF16, c_factor=s.c, U_override=Uo)
        U = sf.num_active(desc)
        ws = sf.workspace(sf.sparse_gqa_workspace_bytes(desc, kh, s.Hk))
        fn = lambda: sf.sparse_gqa_forward(desc, Q, K, V, hg, dm.pattern_id, dm.key_valid, want_sel=False, ws=ws)
        ms, _ = time_steps(fn, steps, 2)
        fl = int((kh * 4 * np.minimum(U, n_allowed) * n_allowed * dh).sum())
        if U < L:
            fl += int((kh * 2 * n_allowed * n_allowed * dh).sum())
        out[tag] = {"U": U, "ms": ms, "tflops": fl / (ms * 1e-3) / 1e12,
                    "frac_of_bf16_peak": fl / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}
        # the same call with V handed over key-contiguous ([B, Hk, dh, Lp], the layout the encoder's projection
        # writes): no transposition pass inside the entry point
        Lp = (L + 7) // 8 * 8
        VT = torch.zeros((B, s.Hk, dh, Lp), dtype=torch.bfloat16, device="cuda")
        VT[..., :L] = V.permute(0, 1, 3, 2)
        fn_t = lambda: sf.sparse_gqa_forward(desc, Q, K, VT, hg, dm.pattern_id, dm.key_valid, v_transposed=True,
                                             want_sel=False, ws=ws)
        ms_t, _ = time_steps(fn_t, steps, 2)
        out[tag + "_v_transposed"] = {"U": U, "ms": ms_t, "tflops": fl / (ms_t * 1e-3) / 1e12,
                                      "frac_of_bf16_peak": fl / (ms_t * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}
        del VT
    return out


def bench_sampled_score(wl, steps, warmup, kv_host):
    """The same step with the sampled-key sparsity score: n_sample = U = c*ceil(ln L) allowed keys per sample
    (drawn by the caller, seeded), which replaces the 2*L*L*dh score stream by 2*L*U*dh per head."""
    import numpy as np
    import torch
    from paper_2604_08971_amd import binding as sf
    from paper_2604_08971_amd.device_model import DeviceModel, to_host
    s = wl.spec
    B, L = wl.x.shape[0], s.L
    U = sf.num_active(sf.make_desc(B, L, s.d, s.Hq, s.Hk, s.dh, s.F, c_factor=s.c))
    if not (0 < U < L) or s.dtype != "bf16":
        return None
    rng = np.random.default_rng(7)
    samp = np.full((B, U), -1, np.int32)
    for b in range(B):
        allowed = np.arange(L) if kv_host is None else np.flatnonzero(kv_host[b])
        k = min(U, len(allowed))
        samp[b, :k] = np.sort(rng.choice(allowed, k, replace=False))
    dm = DeviceModel(wl, sample_idx=samp).build_plan()
    y = torch.empty_like(dm.x)

    def step():
        dm.build_plan()
        dm.forward(out=y)

    ms, _ = time_steps(step, steps, warmup)
    masks_host = {k: to_host(v) for k, v in dm.masks.items()}
    fl = algorithmic_flops(wl, masks_host, U, None, kv_host)
    n_allowed = n_allowed_keys(wl, kv_host)
    score = sum(int((int(wl.k_head[l]) * 2 * n_allowed * np.minimum(U, n_allowed) * s.dh).sum()) for l in range(s.n_layers))
    total = fl["gemm"] + fl["active"] + score
    del dm
    torch.cuda.empty_cache()
    return {"n_sample": U, "ms_per_step": ms, "tokens_per_s": B * L / (ms * 1e-3),
            "algorithmic_tflop_per_step": total / 1e12, "tflops": total / (ms * 1e-3) / 1e12,
            "note": "sparsity score over a caller-supplied sample of U allowed keys per sample (sample_idx); "
                    "`value` above is the score over all allowed keys"}


def bench_f16(wl, steps, warmup):
    """The same step with the model in IEEE binary16 (the FP16 build of the library, libsentryfuse_f16.so: same
    sources, same launches, fp16 MFMA at the bf16 rate): same shapes and seeds, values rounded to binary16."""
    import dataclasses
    import torch
    from paper_2604_08971_amd import binding as sf
    from paper_2604_08971_amd import workloads as W
    from paper_2604_08971_amd.device_model import DeviceModel
    if wl.spec.dtype != "bf16":
        return None
    wl16 = W.make_workload(dataclasses.replace(wl.spec, dtype="f16"))
    with sf.use_half("f16"):
        dm = DeviceModel(wl16).build_plan()
        y = torch.empty_like(dm.x)

        def step():
            dm.build_plan()
            dm.forward(out=y)

        ms, _ = time_steps(step, steps, warmup)
        finite = bool(torch.isfinite(y.float()).all())
        del dm
    torch.cuda.empty_cache()
    B, L = wl.x.shape[0], wl.spec.L
    return {"ms_per_step": ms, "tokens_per_s": B * L / (ms * 1e-3), "output_finite": finite,
            "note": "sf_* entry points of libsentryfuse_f16.so (dtype SF_F16) on the same workload; not part of `value`"}


def bench_moe(wl, steps, warmup, E=8, top_k=2):
    """The workload's tokens through one Sparse-MoE FFN block with pruned experts (E experts, Top-k routing,
    every expert keeps its own channel set): masks of the experts -> compaction -> forward."""
    import numpy as np
    import torch
    from paper_2604_08971_amd import binding as sf
    from paper_2604_08971_amd import workloads as W
    from paper_2604_08971_amd.device_model import to_dev, to_host
    s = wl.spec
    if s.dtype != "bf16":
        return None
    B, L, d, F, P = wl.x.shape[0], s.L, s.d, s.F, wl.P
    mb = W.make_moe_block(wl, E, top_k)
    dt = sf.SF_BF16
    dmask = sf.make_desc(B, L, d, 8, 2, 8, F, n_layers=E, P=P, dtype=dt, act=s.act)
    desc = sf.make_desc(B, L, d, 8, 2, 8, F, n_layers=1, P=P, dtype=dt, act=s.act)
    g_head = torch.zeros((E, P, 8), dtype=torch.float32, device="cuda")
    g_ffn = to_dev(mb.g_ffn, "f32")
    dense = {k: to_dev(v, "bf16") for k, v in mb.dense.items()}
    X = to_dev(wl.x, "bf16").view(B * L, d)
    pid = to_dev(wl.pattern_id, "bf16")
    kf = mb.k_ffn.tolist()
    masks = sf.gate_scores_to_masks(dmask, g_head, g_ffn, [1] * E, kf)
    cm = sf.compact_moe_experts(desc, dense, masks["ffn_idx"], top_k, kf)
    ws = sf.workspace(sf.moe_ffn_workspace_bytes(desc, cm))
    Y = torch.empty_like(X)

    def fwd():
        sf.moe_ffn_forward(desc, cm, X, pid, out=Y, ws=ws)

    def step():
        sf.gate_scores_to_masks(dmask, g_head, g_ffn, [1] * E, kf, out=masks)
        sf.compact_moe_experts(desc, dense, masks["ffn_idx"], top_k, kf, out=cm)
        fwd()

    ms, _ = time_steps(step, steps, warmup)
    ms_fwd, _ = time_steps(fwd, steps, warmup)
    _, route, _, _ = sf.moe_ffn_forward(desc, cm, X, pid, want_route=True, ws=ws)
    load = np.bincount(to_host(route).ravel(), minlength=E).astype(np.int64)
    flops = int((load * 4 * d * mb.k_ffn.astype(np.int64)).sum()) + B * L * 2 * d * E
    sf.profile_begin(sf.SF_KERNEL_GEMM, 64)
    fwd()
    _, _, each = sf.profile_end(each=True)
    del cm, ws, dense
    torch.cuda.empty_cache()
    return {"experts": E, "top_k": top_k, "kept_channels": kf, "expert_load": load.tolist(),
            "ms_per_step": ms, "ms_forward_only": ms_fwd, "tokens_per_s": B * L / (ms * 1e-3),
            "algorithmic_tflop_per_step": flops / 1e12, "tflops": flops / (ms * 1e-3) / 1e12,
            "tflops_forward_only": flops / (ms_fwd * 1e-3) / 1e12,
            "gemm_launch_us": [round(x * 1e3, 1) for x in each],
            "note": "Sparse-MoE FFN block with pruned experts on the same tokens; not part of `value`"}


def bench_gate_plan(wl, reps=50):
    """Plan construction from the gating module: Eq. (1) for all layers and patterns in use, then the global
    threshold for a budget of 60 % of the dense cost (a stand-in budget; the paper names none for these shapes)."""
    import numpy as np
    import torch
    from paper_2604_08971_amd import binding as sf
    from paper_2604_08971_amd import workloads as W
    from paper_2604_08971_amd.device_model import to_dev, to_host
    s = wl.spec
    nl, P, Hq, Hk, F = s.n_layers, wl.P, s.Hq, s.Hk, s.F
    desc = sf.make_desc(1, s.L, s.d, Hq, Hk, s.dh, F, nl, P, sf.SF_F32)
    gp = {k: to_dev(v, "f32") for k, v in W.make_gate_params(nl, s.M, Hq, F, 16, s.seed).items()}
    bits = to_dev(wl.pattern_bits.astype(np.int32), "f32")
    U = sf.num_active(sf.make_desc(1, s.L, s.d, Hq, Hk, s.dh, F, c_factor=s.c))
    ch, cg, cf = W.unit_costs(s, U)
    dense = sum(Hq * ch[l] + Hk * cg[l] + F * cf[l] for l in range(nl))
    budget = int(0.6 * dense)
    res = {}

    def plan():
        gh, gf = sf.gate_eval(desc, gp, bits)
        res["out"] = sf.budget_search(desc, gh, gf, P - 1, ch, cg, cf, 0, budget)

    ms, _ = time_steps(plan, reps, 5)
    o = res["out"]
    return {"us_per_plan": ms * 1e3, "hidden": 16, "budget_frac_of_dense": 0.6, "tau": float(to_host(o["tau"])[0]),
            "k_head": to_host(o["k_head"]).tolist(), "k_ffn": to_host(o["k_ffn"]).tolist(),
            "cost_frac_of_dense": int(to_host(o["cost"])[0]) / dense,
            "note": "sf_gate_eval + sf_budget_search (plan construction from the gating module); not part of `value`"}


def bench_fp8_plan(wl, dm, reps=50):
    """Plan construction from FP8-stored weights (OCP E4M3 codes + one scale per matrix): the compaction reads one
    byte per weight and dequantises in the same pass; the forward path is the same."""
    import numpy as np
    import torch
    from paper_2604_08971_amd import binding as sf
    from paper_2604_08971_amd.device_model import to_dev
    s = wl.spec
    names = ("Wq", "Wk", "Wv", "Wo", "W1", "W2")
    d8, sc = [], []
    for l in range(s.n_layers):
        q, c = dict(dm.dense[l]), {}
        for n in names:
            w = dm.dense[l][n].float()
            c[n] = float(w.abs().max() / 448.0)
            q[n] = (w / c[n]).to(torch.float8_e4m3fn).view(torch.uint8).contiguous()
        d8.append(q); sc.append(c)
    layers8 = [sf.compact_heads_channels_fp8(dm.desc, l, d8[l], sc[l], dm.masks, int(wl.k_head[l]), int(wl.k_ffn[l]))
               for l in range(s.n_layers)]

    def plan8():
        for l in range(s.n_layers):
            sf.compact_heads_channels_fp8(dm.desc, l, d8[l], sc[l], dm.masks, int(wl.k_head[l]), int(wl.k_ffn[l]), out=layers8[l])

    def plan16():
        for l in range(s.n_layers):
            sf.compact_heads_channels(dm.desc, l, dm.dense[l], dm.masks, int(wl.k_head[l]), int(wl.k_ffn[l]), out=dm.layers[l])

    ms8, _ = time_steps(plan8, reps, 5)
    ms16, _ = time_steps(plan16, reps, 5)
    nbytes = sum(int(d8[0][n].numel()) for n in names) * s.n_layers
    del layers8
    return {"us_compaction_from_fp8": ms8 * 1e3, "us_compaction_from_16bit": ms16 * 1e3, "weight_bytes_fp8": nbytes,
            "weight_bytes_16bit": 2 * nbytes,
            "note": "sf_compact_heads_channels_fp8 vs sf_compact_heads_channels, all layers; the forward is unchanged"}


def bench_ffn_fp8(wl, dm, steps, warmup):
    """The pruned FFN of layer 0 on the workload's tokens in FP8 arithmetic (E4M3 codes on both operands of the two
    contractions, static per-tensor scales) next to the same block in bf16; per-launch times of the two GEMMs of
    each, FLOP/s of the FP8 launches against the published dense FP8 rate."""
    import torch
    from paper_2604_08971_amd import binding as sf
    from paper_2604_08971_amd.device_model import to_dev
    s = wl.spec
    if s.dtype != "bf16" or s.d % 128 or s.d < 256 or s.L < 192 or int(wl.k_ffn[0]) <= 128:
        return None
    B, L, d = wl.x.shape[0], s.L, s.d
    kf = int(wl.k_ffn[0])
    dense = dm.dense[0]
    d8, sc = dict(dense), {}
    for n in ("W1", "W2"):
        w = dense[n].float()
        sc[n] = float(w.abs().max() / 448.0)
        d8[n] = (w / sc[n]).to(torch.float8_e4m3fn).view(torch.uint8).contiguous()
    X = to_dev(wl.x, "bf16")
    pid = to_dev(wl.pattern_id, "bf16")
    # activation scales as an offline calibration would set them: amax / 448 of LN2(x) and of the hidden
    # activations, here from the bf16 block's own tensors on this batch
    xn = torch.nn.functional.layer_norm(X.float(), (d,), dense["ln2_g"].float(), dense["ln2_b"].float(), 1e-5)
    sx = float(xn.abs().max() / 448.0)
    pm = dm.masks["ffn_idx"][0, int(wl.pattern_id[0]), :kf].long()
    h0 = torch.relu(xn[0] @ dense["W1"].float()[pm].T + dense["b1"].float()[pm])
    sh = float(h0.abs().max() / 448.0) * 1.25          # one sample seen, some headroom
    del xn, h0
    cf = sf.compact_ffn_fp8(dm.desc, 0, d8, sc, dm.masks, kf, sx, sh)
    ws8 = sf.workspace(sf.lib().sf_pruned_ffn_fp8_workspace_bytes(C_byref(dm.desc), kf))
    ws16 = sf.workspace(sf.lib().sf_pruned_ffn_workspace_bytes(C_byref(dm.desc), kf))

    def f8():
        sf.pruned_ffn_fp8_forward(dm.desc, cf, X, pid, ws=ws8)

    def f16():
        sf.pruned_ffn_forward(dm.desc, dm.layers[0], X, pid, ws=ws16)

    ms8, _ = time_steps(f8, steps, warmup)
    ms16, _ = time_steps(f16, steps, warmup)
    each = {}
    for name, fn in (("fp8", f8), ("bf16", f16)):
        sf.profile_begin(sf.SF_KERNEL_GEMM, 8 * steps)
        for _ in range(steps):
            fn()
        _, _, e = sf.profile_end(each=True)
        each[name] = [sum(e[i::2]) / len(e[i::2]) * 1e3 for i in range(2)]      # us: up, down
    # the whole encoder step with the FFN in FP8 arithmetic (single-layer workloads: one calibrated FFN is all it needs)
    enc = None
    if s.n_layers == 1:
        wse = sf.workspace(sf.encoder_workspace_bytes(dm.desc, dm.layers))
        Ye = torch.empty_like(X)

        def e8():
            sf.encoder_forward_fp8ffn(dm.desc, dm.layers, [cf], X, pid, dm.key_valid, dm.final_ln, out=Ye, ws=wse)

        def e16():
            sf.encoder_forward(dm.desc, dm.layers, X, pid, dm.key_valid, dm.final_ln, out=Ye, ws=wse)

        ms_e8, _ = time_steps(e8, steps, warmup)
        ms_e16, _ = time_steps(e16, steps, warmup)
        enc = {"ms_encoder_fp8_ffn": ms_e8, "ms_encoder_bf16": ms_e16, "tokens_per_s_fp8_ffn": B * L / (ms_e8 * 1e-3),
               "tokens_per_s_bf16": B * L / (ms_e16 * 1e-3)}
        kh = int(wl.k_head[0])
        if (kh * s.dh) % 128 == 0 and (kh + 2 * s.Hk) * s.dh >= 192:
            # and with the Q/K/V and output projections in FP8 arithmetic too (static scales: weights amax / 448;
            # LN1(x) amax / 448; the attention output is a convex combination of V rows, so amax |V| / 448 bounds it)
            p8 = {}
            s_qkv = float(max(dense[n].float().abs().max() for n in ("Wq", "Wk", "Wv")) / 448.0)
            so = float(dense["Wo"].float().abs().max() / 448.0)
            for n in ("Wq", "Wk", "Wv", "Wo"):
                p8[n] = (dense[n].float() / (so if n == "Wo" else s_qkv)).to(torch.float8_e4m3fn).view(torch.uint8).contiguous()
            xn1 = torch.nn.functional.layer_norm(X[0].float(), (d,), dense["ln1_g"].float(), dense["ln1_b"].float(), 1e-5)
            sx1 = float(torch.nn.functional.layer_norm(X.float(), (d,), dense["ln1_g"].float(), dense["ln1_b"].float(),
                                                       1e-5).abs().max() / 448.0)
            sa = float((xn1 @ dense["Wv"].float().T + dense["bv"].float()).abs().max() / 448.0) * 1.25
            cp = sf.compact_proj_fp8(dm.desc, 0, p8, s_qkv, so, dm.masks, kh, sx1, sa)
            wsp = sf.workspace(sf.encoder_fp8_workspace_bytes(dm.desc, dm.layers))

            def e8p():
                sf.encoder_forward_fp8(dm.desc, dm.layers, X, ffn8=[cf], proj8=[cp], pattern_id=pid, key_valid=dm.key_valid,
                                       final_ln=dm.final_ln, out=Ye, ws=wsp)

            ms_e8p, _ = time_steps(e8p, steps, warmup)
            e16()
            y16e = Ye.float().clone()
            e8p()
            rel_e = float((Ye.float() - y16e).norm() / (y16e - X.float()).norm())
            enc.update({"ms_encoder_fp8_proj_ffn": ms_e8p, "tokens_per_s_fp8_proj_ffn": B * L / (ms_e8p * 1e-3),
                        "rel_diff_of_layer_update_fp8_proj_ffn_vs_bf16": rel_e,
                        "proj_scales": {"s_qkv": s_qkv, "so": so, "sx1": sx1, "sa": sa}})
            del wsp, cp, p8, y16e
        del wse, Ye
    y8 = sf.pruned_ffn_fp8_forward(dm.desc, cf, X, pid, ws=ws8).float()
    y16 = sf.pruned_ffn_forward(dm.desc, dm.layers[0], X, pid, ws=ws16).float()
    upd8, upd16 = y8 - X.float(), y16 - X.float()
    rel = float((upd8 - upd16).norm() / upd16.norm())
    flop = 2.0 * B * L * d * kf                      # per GEMM, unpadded
    out = {"k_ffn": kf, "ms_block_fp8": ms8, "ms_block_bf16": ms16,
           "gemm_launch_us_fp8": {"ffn_up": each["fp8"][0], "ffn_down": each["fp8"][1]},
           "gemm_launch_us_bf16": {"ffn_up": each["bf16"][0], "ffn_down": each["bf16"][1]},
           "tflops_fp8": {"ffn_up": flop / each["fp8"][0] / 1e6, "ffn_down": flop / each["fp8"][1] / 1e6},
           "frac_of_fp8_peak": {"ffn_up": flop / each["fp8"][0] / 1e6 / 5000.0,
                                "ffn_down": flop / each["fp8"][1] / 1e6 / 5000.0},
           "encoder_step": enc, "rel_diff_of_ffn_update_vs_bf16": rel, "scales": {"sx": sx, "sh": sh, "s1": sc["W1"], "s2": sc["W2"]},
           "note": "sf_pruned_ffn_fp8_forward vs sf_pruned_ffn_forward (LayerNorm + two GEMMs, layer 0), and the encoder "
                   "forward (plan excluded) with that FFN in FP8 arithmetic, sf_encoder_forward_fp8ffn, and with the "
                   "attention projections in FP8 arithmetic as well, sf_encoder_forward_fp8, vs sf_encoder_forward; "
                   "not part of `value`"}
    del cf, ws8, ws16
    torch.cuda.empty_cache()
    return out


def bench_tokens(name, steps, warmup):
    """Token compaction on a dropout workload: the masked encoder step (absent modalities kept in place and masked as
    keys) against dropping their tokens - all samples in one compacted batch padded to the longest sample, and one
    compacted batch per presence pattern (the caller groups samples by pattern, so every group has one length)."""
    import numpy as np
    import torch
    from paper_2604_08971_amd import binding as sf
    from paper_2604_08971_amd import workloads as W
    from paper_2604_08971_amd.device_model import DeviceModel, desc_for
    wl = W.make_workload(W.CONFIGS[name])
    if wl.presence.all():
        return None
    s = wl.spec
    dm = DeviceModel(wl).build_plan()
    B = wl.x.shape[0]
    lens = key_valid_host(dm).sum(axis=1).astype(int)
    u = np.array([min(s.c * int(np.ceil(np.log(t))), t) if t > 0 else 0 for t in lens])

    def masked():
        dm.forward()

    def make_group(idx):
        idx_t = torch.from_numpy(np.asarray(idx)).to("cuda")
        X = dm.x[idx_t].contiguous()
        kv = dm.key_valid[idx_t].contiguous()
        pid = dm.pattern_id[idx_t].contiguous()
        Lc = min(int(-(-lens[idx].max() // 8) * 8), s.L)
        dfull = desc_for(wl, B=len(idx))
        dc = desc_for(wl, B=len(idx), U_override=int(u[idx].max()))
        dc.L = Lc
        ws = sf.workspace(sf.encoder_workspace_bytes(dc, dm.layers))
        return X, kv, pid, Lc, dfull, dc, ws

    def run_group(g):
        X, kv, pid, Lc, dfull, dc, ws = g
        tc = sf.token_compact(dfull, X, kv, Lc)
        Yc, _, _ = sf.encoder_forward_ragged(dc, dm.layers, tc["Xc"], pid, tc["valid_c"], tc["u_active"],
                                             final_ln=dm.final_ln, ws=ws)
        return sf.token_scatter(dfull, Yc, tc["slot_of"])

    one = [make_group(np.arange(B))]
    by_pattern = [make_group(np.nonzero(wl.pattern_id == p)[0]) for p in np.unique(wl.pattern_id)]
    # two length buckets, each padded to its longest sample: samples that fit one 256-row GEMM tile, and the rest
    cut = 256
    short, long_ = np.nonzero(lens <= cut)[0], np.nonzero(lens > cut)[0]
    two = [make_group(ix) for ix in (short, long_) if len(ix)]
    # no padding: the valid tokens of all samples back to back, runs by pattern; the caller knows the presence counts
    # and sizes the packed buffers for them
    Tc = int(sum(-(-int(lens[wl.pattern_id == p].sum()) // 256) * 256 for p in np.unique(wl.pattern_id))
             + -(-s.L // 256) * 256)
    plan = sf.TokenPackPlan(B, s.L, Tc, dm.x.device)
    dp = desc_for(wl, U_override=int(u.max()))
    ws_p = sf.workspace(sf.encoder_packed_workspace_bytes(dp, dm.layers, Tc))
    Xp = torch.empty((Tc, s.d), dtype=dm.x.dtype, device=dm.x.device)
    Yp, Yfull = torch.empty_like(Xp), torch.empty_like(dm.x)

    def packed():
        sf.token_pack(dm.desc, dm.x, dm.key_valid, dm.pattern_id, plan=plan, out=Xp)
        sf.encoder_forward_packed(dp, dm.layers, Xp, plan, dm.pattern_id, final_ln=dm.final_ln, ws=ws_p, out=Yp)
        return sf.token_unpack(dm.desc, Yp, plan, out=Yfull)

    def packed_encoder_only():
        sf.encoder_forward_packed(dp, dm.layers, Xp, plan, dm.pattern_id, final_ln=dm.final_ln, ws=ws_p, out=Yp)

    ms_masked, _ = time_steps(masked, steps, warmup)
    ms_packed, _ = time_steps(packed, steps, warmup)
    ms_packed_enc, _ = time_steps(packed_encoder_only, steps, warmup)
    n_rows = plan.n_rows.cpu().numpy()
    assert n_rows[0] == n_rows[1] == Tc, (n_rows, Tc)
    ms_two, _ = time_steps(lambda: [run_group(g) for g in two], steps, warmup)
    ms_one, _ = time_steps(lambda: [run_group(g) for g in one], steps, warmup)
    ms_grp, _ = time_steps(lambda: [run_group(g) for g in by_pattern], steps, warmup)
    rows_grp = int(sum(g[3] * g[0].shape[0] for g in by_pattern))
    return {"workload": name, "tokens_total": int(B * s.L), "tokens_present": int(lens.sum()),
            "ms_masked": ms_masked, "ms_packed": ms_packed, "ms_packed_encoder_only": ms_packed_enc, "rows_packed": Tc,
            "ms_compacted_one_batch": ms_one, "Lc_one_batch": one[0][3],
            "ms_compacted_two_buckets": ms_two, "rows_two_buckets": int(sum(g[3] * g[0].shape[0] for g in two)),
            "ms_compacted_per_pattern": ms_grp, "pattern_groups": len(by_pattern), "rows_per_pattern_batches": rows_grp,
            "note": "encoder step only (plan excluded); packed: pack + encoder over the packed rows + unpack; compacted: "
                    "compaction + ragged encoder + scatter per padded batch; eager launches; not part of `value`"}


def C_byref(x):
    import ctypes
    return ctypes.byref(x)


def cpu_baseline(wl, flops_total):
    """The CPU oracle, as it stands, on a bounded number of whole samples of the same workload."""
    import numpy as np
    from oracle import cpu_oracle as orc
    from oracle.packs import compact_packs, key_valid_of, oracle_masks
    s = wl.spec
    B, L = wl.x.shape[0], s.L
    threads = orc.max_threads()
    per_sample = flops_total / B
    n = int(max(1, min(B, round(15.0 * threads * 2.2e9 / per_sample))))    # aim at roughly 15 s
    masks = oracle_masks(wl)
    packs = compact_packs(wl, masks)
    U = orc.num_active(L, s.c)
    kv_all = key_valid_of(wl)            # the oracle's own key mask
    kv = None if kv_all is None else kv_all[:n]
    t0 = time.perf_counter()
    orc.encoder_forward(wl.x[:n], packs, U, wl.pattern_id[:n], kv, act=s.act, final_ln=wl.final_ln,
                        bf16=s.dtype == "bf16", want_sel=False)
    dt = time.perf_counter() - t0
    return {"value": n * L / dt, "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": f"{n} of {B} samples of {s.name} (whole encoder forward, fp64 C oracle, OpenMP over rows), {dt:.1f} s",
            "seconds": dt}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="C5", help="workload timed for `value` (C1..C5)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-extras", action="store_true", help="only the headline number")
    ap.add_argument("--graph", action="store_true",
                    help="time a replayed HIP graph of the step instead of eager launches (measured slower on ROCm 7.2: 1.38 vs 1.35 ms)")
    ap.add_argument("--other-configs", default="C2,C3,C4", help="also time these (reported under `other_workloads`)")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="also run one plain device copy of this many MiB (known traffic, for scaling the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    ap.add_argument("--ffn-fp8-only", action="store_true",
                    help="time only the FP8-arithmetic FFN block (and its bf16 twin) on the workload's tokens and "
                         "print its object (for profiling)")
    ap.add_argument("--f16-only", action="store_true",
                    help="time only the step of the FP16 build of the library on the workload and print its object "
                         "(for profiling)")
    ap.add_argument("--tokens-only", action="store_true",
                    help="time only the token-compaction comparison on the dropout workload C3 and print its object")
    ap.add_argument("--sparse-gqa-only", action="store_true",
                    help="time only sf_sparse_gqa_forward at the workload's kept shapes (c-sparse and dense pattern) and "
                         "print its object (for profiling)")
    ap.add_argument("--moe-only", action="store_true",
                    help="time only the Sparse-MoE FFN block on the workload's tokens and print its object (for profiling)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build is single-GPU (one MI355X holds every workload and no step of the path "
                 "crosses samples); run with --gpus 1")

    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    from paper_2604_08971_amd import binding as sf
    from paper_2604_08971_amd import workloads as W
    sf.lib()

    if args.copy_calibration > 0:
        n = args.copy_calibration << 20
        src = torch.ones(n, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        log(f"copy calibration: 3 device copies of {args.copy_calibration} MiB (reads and writes that many bytes each)")
        del src, dst

    if args.moe_only:
        print(json.dumps(bench_moe(W.make_workload(W.CONFIGS[args.config]), args.steps, args.warmup)), flush=True)
        return

    if args.tokens_only:
        print(json.dumps(bench_tokens("C3", args.steps, args.warmup)), flush=True)
        return

    if args.sparse_gqa_only:
        from paper_2604_08971_amd.device_model import DeviceModel
        wl = W.make_workload(W.CONFIGS[args.config])
        dm = DeviceModel(wl).build_plan()
        print(json.dumps(bench_sparse_gqa(dm, wl, args.steps)), flush=True)
        return

    if args.ffn_fp8_only:
        from paper_2604_08971_amd.device_model import DeviceModel
        wl = W.make_workload(W.CONFIGS[args.config])
        dm = DeviceModel(wl).build_plan()
        print(json.dumps(bench_ffn_fp8(wl, dm, args.steps, args.warmup)), flush=True)
        return

    if args.f16_only:
        print(json.dumps(bench_f16(W.make_workload(W.CONFIGS[args.config]), args.steps, args.warmup)), flush=True)
        return

    extras = not args.no_extras
    res, dm, wl, flops = bench_config(args.config, args.steps, args.warmup, extras, not args.no_cpu, args.graph)
    spec = wl.spec
    out = {
        "metric": METRIC, "value": res["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if spec.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{spec.name}: B={res['B']} L={res['L']} d={spec.d} Hq/Hk/dh={spec.Hq}/{spec.Hk}/{spec.dh} "
                               f"F={spec.F} layers={spec.n_layers} kept heads={list(map(int, wl.k_head))} "
                               f"kept channels={int(wl.k_ffn[0])} U={res['U']} patterns={wl.P}",
                   "step": "gate_scores_to_masks + compact_heads_channels + encoder_forward",
                   "launch": res["launch"]},
        "algorithmic_tflop_per_step": res["algorithmic_tflop_per_step"],
        "tflops": res["tflops_total"], "frac_of_bf16_peak": res["tflops_total"] / PEAK_BF16_TFLOPS,
    }
    if extras:
        out["detail"] = {k: res[k] for k in ("ms_encoder_only", "ms_plan_only", "tokens_per_s_encoder_only",
                                             "host_ms_per_step", "ms_per_step_eager") if k in res}
        k = res.get("kernels", {})
        if "gemm" in k and "by_launch" in k["gemm"]:
            # the dominant kernel: the GEMM launch that takes the most time per step
            by = k["gemm"]["by_launch"]
            nm = max(by, key=lambda q: by[q]["avg_launch_us"] * by[q]["launches_per_step"])
            g = by[nm]
            out["roofline"] = {"bound": "mfma", "kernel": GEMM_KERNEL_NAMES[nm], "launch": nm,
                               "achieved": g["tflops"], "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                               "frac": g["tflops"] / PEAK_BF16_TFLOPS,
                               "traffic": measured_traffic(args.config, nm),
                               "avg_launch_us": g["avg_launch_us"], "launches_per_step": g["launches_per_step"],
                               "all_gemm_launches": {"avg_launch_us": k["gemm"]["avg_launch_us"],
                                                     "tflops": k["gemm"]["tflops"],
                                                     "frac": k["gemm"]["tflops"] / PEAK_BF16_TFLOPS}}
        elif "gemm" in k:
            g = k["gemm"]
            out["roofline"] = {"bound": "mfma", "kernel": "bf16 GEMM launches (all projections + FFN)",
                               "achieved": g["tflops"], "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                               "frac": g["tflops"] / PEAK_BF16_TFLOPS, "traffic": None,
                               "avg_launch_us": g["avg_launch_us"], "launches_per_step": g["launches_per_step"]}
        out["kernels"] = k
        out["ceilings"] = bench_ceilings()
        if "roofline" in out and out["roofline"].get("bound") == "mfma":
            out["roofline"]["frac_of_measured_mfma_ceiling_random_operands"] = (
                out["roofline"]["achieved"] / out["ceilings"]["mfma_bf16_random_operands"]["tflops"])
        out["kernel_source_digest"] = kernel_source_digest()
        out["sparse_gqa"] = bench_sparse_gqa(dm, wl, args.steps)
        out["sampled_score"] = bench_sampled_score(wl, args.steps, args.warmup, key_valid_host(dm))
        out["f16_build"] = bench_f16(wl, args.steps, args.warmup)
        out["moe_ffn"] = bench_moe(wl, args.steps, args.warmup)
        out["gate_plan"] = bench_gate_plan(wl)
        out["fp8_weights"] = bench_fp8_plan(wl, dm)
        out["ffn_fp8"] = bench_ffn_fp8(wl, dm, args.steps, args.warmup)
        out["token_compaction"] = bench_tokens("C3", args.steps, args.warmup)
    if not args.no_cpu:
        log("timing the CPU oracle on a bounded sample ...")
        out["cpu_baseline"] = cpu_baseline(wl, flops["total"])
    del dm
    torch.cuda.empty_cache()
    if extras and args.other_configs:
        others = {}
        for name in args.other_configs.split(","):
            name = name.strip()
            if not name or name == args.config:
                continue
            r, dm2, _, _ = bench_config(name, args.steps, args.warmup, True, False, args.graph, repeats=3)
            others[name] = {k: r[k] for k in ("ms_per_step", "tokens_per_s", "tflops_total", "ms_encoder_only",
                                              "ms_plan_only", "host_ms_per_step", "launch", "ms_per_step_eager") if k in r}
            others[name]["kernels"] = r.get("kernels")
            del dm2
            torch.cuda.empty_cache()
        out["other_workloads"] = others
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
