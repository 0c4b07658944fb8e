"""Benchmark of the APOLLO / APOLLO-Mini optimizer step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload llama7b_mini] [--also a,b,...]

A "step" is one pass of the whole hot path (projection, low-rank Adam + factors, limiter, weight
update; plus, on the one step in T = 200 that re-samples P, the generation of its scratch copy, which
here falls into the warm-up) over every matrix of a synthetic LLaMA-shaped parameter set
whose weights, gradients and optimizer state are already resident in HBM.  Prints ONE JSON line:
value = parameters updated per second over exactly K timed steps; "roofline" describes the
kernel phase that takes the most time (algorithmic bytes or flops per step divided by that
phase's HIP-event time, against the MI355X peak); "cpu_baseline" is the fp64 oracle timed on
the host cores on a bounded sample of the same workload; "also" carries the same measurement
for further variants on the same shapes (rank 256, which the benchmark definition asks for as well;
bfloat16 and 8-bit storage) and for the benchmark definition's other configurations (LLaMA-60M shapes at
rank 128; LLaMA-1B shapes at rank 512; LLaMA-13B shapes, Mini and rank 256, five timed steps of which the first re-samples
P); "adamw_rest" the element-wise AdamW launch on the model's non-projected parameters.  Every step
gets freshly drawn gradients (seed = 1000 * config + step); they are generated between the timed
steps, outside the timed region: each step is bracketed by a device synchronisation on both sides,
and the K bracketed times are added.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 matrix cores, published
PHASES = ["projection_fill", "projection", "adam_norms", "limiter", "update"]
KERNEL_OF_PHASE = {"projection_fill": "fill_projection_kernel", "projection": "project_mfma_kernel",
                   "adam_norms": "adam_norms_kernel", "limiter": "finalize_kernel", "update": "update_kernel"}


def measured_traffic(workload, kernel, live_us=None):
    """HBM bytes per step of `kernel` from the committed rocprofv3 FETCH_SIZE + WRITE_SIZE summary of
    this workload (profiles/<workload>_hbm_traffic.txt, counters scaled by the copy-kernel
    calibration), or None when there is no such summary -- or when the summary is stale: it records
    the kernel's time per step in the profiled run ("kernel_us_per_step <kernel>: t"), and if the time
    measured live in this run (live_us) differs from that by more than 15 % the kernel has changed
    since it was profiled and its byte counts are not reported."""
    path = os.path.join(ROOT, "profiles", "%s_hbm_traffic.txt" % workload)
    names = [kernel]
    if "{" in kernel:  # "a_{x,y}_b" names the kernels a_x_b and a_y_b: their bytes add
        head, rest = kernel.split("{", 1)
        alts, tail = rest.split("}", 1)
        names = [head + a + tail for a in alts.split(",")]
    found, prof_us = {}, {}
    try:
        with open(path) as fh:
            for line in fh:
                for nm in names:
                    if line.startswith("traffic_bytes_per_step %s:" % nm):
                        found[nm] = int(line.split(":")[1])
                    if line.startswith("kernel_us_per_step %s:" % nm):
                        prof_us[nm] = float(line.split(":")[1])
    except OSError:
        return None
    if len(found) != len(names):
        return None
    if live_us is not None:
        if len(prof_us) != len(names):
            return None
        t = sum(prof_us.values())
        if abs(t - live_us) > 0.15 * max(t, live_us):
            print("bench: profiles/%s_hbm_traffic.txt is stale for %s (%.0f us per step there, %.0f us now): "
                  "traffic not reported" % (workload, kernel, t, live_us), file=sys.stderr)
            return None
    return sum(found.values())


def make_cfg(A, wl, seed=20241205):
    mode = A.APOLLO_TENSOR if wl.mode == "tensor" else A.APOLLO_CHANNEL
    return A.ApolloConfig(rank=wl.rank, mode=mode, seed=seed, beta1=wl.beta1, beta2=wl.beta2, eps=wl.eps,
                          scale=wl.scale, weight_decay=wl.weight_decay, nl_gamma=wl.nl_gamma,
                          refresh_interval=wl.refresh_interval, bias_correction=1, side=A.APOLLO_SIDE_AUTO,
                          weight_dtype={"torch.bfloat16": A.APOLLO_BF16, "torch.uint8": A.APOLLO_Q8}.get(str(wl.weight_dtype), A.APOLLO_F32),
                          weight_rounding=A.APOLLO_ROUND_STOCHASTIC if wl.weight_rounding == "stochastic" else A.APOLLO_ROUND_NEAREST,
                          state_dtype=A.APOLLO_BF16 if str(wl.state_dtype) == "torch.bfloat16" else A.APOLLO_F32,
                          projection=A.APOLLO_PROJ_IDENTITY if wl.projection == "identity" else A.APOLLO_PROJ_RANDOM)


def algorithmic_work(wl):
    """Per step and per phase: bytes the method itself has to move (and matrix-core flops)."""
    import torch
    gb = 2 if wl.grad_dtype == torch.bfloat16 else 4
    wb = 2 if wl.weight_dtype == torch.bfloat16 else 4     # W is read and written
    if wl.weight_dtype == torch.uint8:
        wb = 1.0 + 8.0 / 128.0                             # 8-bit codes + (scale, zero) per 128 elements
    sb = 2 if wl.state_dtype == torch.bfloat16 else 4      # M and V are read and written
    params = wl.n_params
    chan = sum(max(s) for s in wl.shapes)                 # sum of channel counts n
    if wl.projection == "identity":   # no projection: the moment pass reads G and the full-size M, V
        return {
            "projection": {"bytes": 0.0, "flops": 0.0},
            "adam_norms": {"bytes": (gb + 4.0 * sb) * params, "flops": 0.0},
            "update": {"bytes": (gb + 2.0 * wb) * params, "flops": 0.0},
            "total_bytes": (2 * gb + 2.0 * wb + 4.0 * sb) * params,
        }
    return {
        "projection": {"bytes": gb * params, "flops": 2.0 * wl.rank * params},
        "adam_norms": {"bytes": 4.0 * sb * wl.rank * chan, "flops": 0.0},
        "update": {"bytes": (gb + 2.0 * wb) * params, "flops": 0.0},
        "total_bytes": (2 * gb + 2.0 * wb) * params + 4.0 * sb * wl.rank * chan,
    }


def measure(A, WL, torch, wl, weights, grads, steps, warmup, dev, overlap_leg=True, first_step=1, graph_leg=True,
            phase_pass="auto"):
    """Times `steps` steps after `warmup` untimed ones, step numbers first_step, first_step + 1, ...
    Every step (warm-up and timed) first gets freshly drawn gradients into the same buffers (seed =
    1000 * config + step), generated outside the timed region; a timed step is bracketed by a device
    synchronisation on both sides (host clock) and by events on the stream (device time)."""
    cfg = make_cfg(A, wl)
    metas = None
    if wl.weight_dtype == torch.uint8:
        weights, metas = weights
    st = A.ApolloStepper(cfg, weights, grads, device=dev, metas=metas)
    # does the projection kernel also update the moments (one kernel for Algorithm 1's steps 1-3)?
    fused = all(st.path(i)[0] == A.APOLLO_PATH_MATRIX_CORE for i in range(len(wl.shapes)))
    t = first_step
    for _ in range(warmup):
        WL.make_grads(wl, t, dev, out=grads)
        st.step(t, wl.lr)
        t += 1
    torch.cuda.synchronize()
    # The library's HIP events around its phases cost a few microseconds each: nothing against a step of
    # milliseconds, a fifth of the step of a set that is bound by launch latency.  Such a set is timed
    # without them, as a caller runs it, and stepped the same number of times again for the per-phase times.
    separate = phase_pass == "separate" or (phase_pass == "auto" and wl.n_params < 100e6)
    if not separate:
        A.apollo_profile_enable(st.handle, True)
    e0 = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]   # (the stepper uses torch's current stream)
    e1 = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    wall = 0.0
    for k in range(steps):
        WL.make_grads(wl, t, dev, out=grads)
        torch.cuda.synchronize()
        h0 = time.perf_counter()
        e0[k].record()
        st.step(t, wl.lr)
        e1[k].record()
        torch.cuda.synchronize()
        wall += time.perf_counter() - h0
        t += 1
    per_step = [e0[k].elapsed_time(e1[k]) for k in range(steps)]
    if separate:
        A.apollo_profile_enable(st.handle, True)
        for k in range(steps):
            WL.make_grads(wl, t, dev, out=grads)
            st.step(t, wl.lr)
            t += 1
        torch.cuda.synchronize()
    rc, ms, n = A.apollo_profile_read(st.handle)
    assert rc == 0 and n == steps, (rc, n)
    A.apollo_profile_enable(st.handle, False)
    finite = all(bool(torch.isfinite(w.float()).all()) for w in (metas if metas is not None else weights)[:7])
    state_bytes, ws_bytes = st.state.numel(), st.workspace.numel()
    st.close()
    del st
    torch.cuda.empty_cache()
    sec = wall / steps
    phase_ms = {p: ms[i] / steps for i, p in enumerate(PHASES)}
    work = algorithmic_work(wl)
    if fused:   # the moments are read and written by the projection kernel: their bytes belong to its phase
        work["projection"]["bytes"] += work["adam_norms"]["bytes"]
        work["adam_norms"]["bytes"] = 0.0
    dom = max(("projection", "adam_norms", "update"), key=lambda p: phase_ms[p])
    w = work[dom]
    t_dom = phase_ms[dom] * 1e-3
    hbm_frac = w["bytes"] / t_dom / 1e9 / HBM_PEAK_GBS
    mfma_frac = w["flops"] / t_dom / 1e12 / MFMA_BF16_PEAK_TFLOPS
    if dom == "projection" and mfma_frac > hbm_frac:
        roof = {"bound": "mfma", "achieved": w["flops"] / t_dom / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": mfma_frac, "traffic": None}
    else:
        roof = {"bound": "hbm", "achieved": w["bytes"] / t_dom / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": hbm_frac, "traffic": None}
    roof["kernel"] = KERNEL_OF_PHASE[dom]
    groups = len(set(wl.shapes))
    # sets below 64 M parameters run the update of all shape groups as one launch of update_groups_kernel
    merged_update = wl.weight_dtype != torch.uint8 and groups > 1 and wl.n_params < (64 << 20)
    if dom == "update" and wl.weight_dtype == torch.uint8:
        roof["kernel"] = "update_q8_kernel"
    if dom == "update" and merged_update:
        roof["kernel"] = "update_groups_kernel"
    if dom == "projection" and wl.rank == 1:
        roof["kernel"] = "project_rank1_left_kernel + project_rank1_right_kernel"
    roof["traffic"] = measured_traffic(wl.name, roof["kernel"] if dom == "update" else KERNEL_OF_PHASE[dom]
                                       if not (dom == "projection" and wl.rank == 1) else "project_rank1_{left,right}_kernel",
                                       live_us=phase_ms[dom] * 1e3)
    roof["traffic_note"] = ("HBM bytes read + written per step (all launches of the kernel), rocprofv3 counters, profiles/; "
                            "null when there is no summary or the kernel's time has moved away from the profiled one")
    roof["algorithmic"] = w["bytes"]
    roof["phase"] = dom
    roof["ms_per_step"] = phase_ms[dom]
    # the matrix-core projection covers all shape groups with one launch, and so does the update of small sets
    roof["launches_per_step"] = 1 if (dom == "projection" and fused) or (dom == "update" and merged_update) else groups
    pw = work["projection"]
    t_proj = phase_ms["projection"] * 1e-3
    proj = {"kernel": "project_mfma_kernel" if wl.rank > 1 else "project_rank1_{left,right}_kernel",
            "fused_with_moment_update": fused,
            "ms_per_step": phase_ms["projection"],
            "hbm": {"achieved": pw["bytes"] / t_proj / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": pw["bytes"] / t_proj / 1e9 / HBM_PEAK_GBS},
            "mfma": {"achieved": pw["flops"] / t_proj / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": pw["flops"] / t_proj / 1e12 / MFMA_BF16_PEAK_TFLOPS},
            "traffic": measured_traffic(wl.name, "project_mfma_kernel", live_us=phase_ms["projection"] * 1e3) if wl.rank > 1 else None}
    res = {
        "projection_roofline": proj,
        "value": wl.n_params / sec, "ms_per_step": sec * 1e3, "device_ms_per_step": sum(per_step) / steps,
        "min_ms_per_step": min(per_step), "phase_ms": phase_ms,
        "roofline": roof,
        "whole_step_hbm_frac": work["total_bytes"] / sec / 1e9 / HBM_PEAK_GBS,
        "projection_tflops": work["projection"]["flops"] / (phase_ms["projection"] * 1e-3) / 1e12,
        "finite": finite, "state_gb": state_bytes / 1e9, "workspace_gb": ws_bytes / 1e9,
        "first_timed_step": first_step + warmup,
    }
    if graph_leg and wl.n_params < 100e6 and metas is None:
        # a set this small is bound by launch latency: the same steps replayed from a HIP graph (the kernels of a
        # step captured once; per step one small kernel writes the step's scalars, then the graph is launched)
        st = A.ApolloStepper(cfg, weights, grads, device=dev)
        st.step(first_step, wl.lr)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            st.launch()
        t = first_step + 1
        for _ in range(warmup):
            st.prepare(t, wl.lr)
            graph.replay()
            t += 1
        torch.cuda.synchronize()
        wall_g = 0.0
        g0 = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
        g1 = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
        for k in range(steps):
            WL.make_grads(wl, t, dev, out=grads)
            torch.cuda.synchronize()
            h0 = time.perf_counter()
            g0[k].record()
            st.prepare(t, wl.lr)
            graph.replay()
            g1[k].record()
            torch.cuda.synchronize()
            wall_g += time.perf_counter() - h0
            t += 1
        res["graph_replay_ms_per_step"] = wall_g / steps * 1e3
        res["graph_replay_device_ms_per_step"] = sum(g0[k].elapsed_time(g1[k]) for k in range(steps)) / steps
        del graph
        st.close()
        del st
        torch.cuda.empty_cache()
    if overlap_leg and wl.rank % 32 == 0 and wl.projection != "identity" and wl.grad_dtype == torch.bfloat16:
        # the optional two-stream schedule (shape groups as overlapping chains): the last gradients again
        cfg.schedule = A.APOLLO_SCHEDULE_OVERLAP
        st = A.ApolloStepper(cfg, weights, grads, device=dev, metas=metas)
        for k in range(warmup):
            st.step(first_step + k, wl.lr)
        torch.cuda.synchronize()
        p0 = time.perf_counter()
        for k in range(steps):
            st.step(first_step + warmup + k, wl.lr)
        torch.cuda.synchronize()
        res["overlap_schedule_ms_per_step"] = (time.perf_counter() - p0) / steps * 1e3
        st.close()
        del st
        torch.cuda.empty_cache()
        # the optional schedule that keeps no P between steps (generated chunk by chunk in every step)
        cfg.schedule = A.APOLLO_SCHEDULE_CHUNKED
        st = A.ApolloStepper(cfg, weights, grads, device=dev, metas=metas)
        for k in range(warmup):
            st.step(first_step + k, wl.lr)
        torch.cuda.synchronize()
        p0 = time.perf_counter()
        for k in range(steps):
            st.step(first_step + warmup + k, wl.lr)
        torch.cuda.synchronize()
        res["chunked_schedule_ms_per_step"] = (time.perf_counter() - p0) / steps * 1e3
        res["chunked_schedule_workspace_gb"] = st.workspace.numel() / 1e9
        st.close()
        del st
        torch.cuda.empty_cache()
    return res


def entry_of(wl, r):
    """One workload's measurement as it appears under "also"."""
    return {"workload": describe(wl), "benchmark_config": wl.config_id, "value": r["value"], "unit": "params/s",
            "ms_per_step": r["ms_per_step"], "device_ms_per_step": r["device_ms_per_step"],
            "min_ms_per_step": r["min_ms_per_step"], "first_timed_step": r["first_timed_step"],
            "phase_ms": r["phase_ms"], "overlap_schedule_ms_per_step": r.get("overlap_schedule_ms_per_step"),
            "chunked_schedule_ms_per_step": r.get("chunked_schedule_ms_per_step"),
            "chunked_schedule_workspace_gb": r.get("chunked_schedule_workspace_gb"),
            "graph_replay_ms_per_step": r.get("graph_replay_ms_per_step"),
            "graph_replay_device_ms_per_step": r.get("graph_replay_device_ms_per_step"),
            "roofline": r["roofline"], "whole_step_hbm_frac": r["whole_step_hbm_frac"],
            "projection_roofline": r["projection_roofline"], "state_gb": r["state_gb"], "workspace_gb": r["workspace_gb"],
            "finite": r["finite"]}


def measure_adamw_rest(A, torch, steps, warmup, dev, store_bf16=False, also_bf16=True):
    """The element-wise AdamW launch on the parameters of a LLaMA-7B that APOLLO does not project:
    the 32000 x 4096 embedding and output head and the 65 norm gains; bf16 gradients, W/M/V in fp32
    (or, store_bf16, in bfloat16).  Algorithmic traffic per parameter: W 8 B, M and V 16 B (4 and 8
    in bfloat16), G 2 B."""
    sizes = [32000 * 4096] * 2 + [4096] * 65
    gen = torch.Generator(device=dev).manual_seed(7)
    weights = [torch.randn(n, generator=gen, device=dev) * 0.02 for n in sizes]
    if store_bf16:
        weights = [w.to(torch.bfloat16) for w in weights]
    per_param = 14.0 if store_bf16 else 26.0
    grads = [(torch.randn(n, generator=gen, device=dev) * 1e-3).to(torch.bfloat16) for n in sizes]
    cfg = A.ApolloAdamwConfig(beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, bias_correction=1, reserved=0)
    st = A.AdamwStepper(cfg, weights, grads, device=dev)
    for t in range(1, warmup + 1):
        st.step(t, 1e-3)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]   # the stepper launches on torch's current stream
    torch.cuda.synchronize()
    ev[0].record()
    for t in range(warmup + 1, warmup + steps + 1):
        st.step(t, 1e-3)
    ev[1].record()
    torch.cuda.synchronize()
    ms = ev[0].elapsed_time(ev[1]) / steps
    n = sum(sizes)
    finite = bool(torch.isfinite(weights[0][:4096].float()).all())
    st.close()
    gbs = per_param * n / (ms * 1e-3) / 1e9
    res = {"workload": "llama7b_rest: embedding + output head (32000x4096 each) + 65 norm gains, bf16 gradients, "
                       "%s W/M/V, element-wise AdamW" % ("bf16" if store_bf16 else "fp32"), "params": n, "ms_per_step": ms,
           "value": n / (ms * 1e-3), "unit": "params/s",
           "roofline": {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
                        "traffic": None if store_bf16 else measured_traffic("llama7b_rest", "adamw_kernel"),
                        "kernel": "adamw_kernel", "algorithmic": per_param * n, "launches_per_step": 1},
           "finite": finite}
    del weights, grads, st
    torch.cuda.empty_cache()
    if not store_bf16 and also_bf16:
        b16 = measure_adamw_rest(A, torch, steps, warmup, dev, store_bf16=True)
        res["bf16_storage"] = {k: b16[k] for k in ("ms_per_step", "value", "roofline", "finite")}
    return res


def cpu_baseline(A, WL, torch, wl, weights, grads, budget_s=20.0):
    """The oracle as it stands, timed on the host: one tensor of each distinct shape from the first
    and from the last layer (the tensor index enters the random stream), as many steps as fit the
    budget (at least one)."""
    import numpy as np
    from oracle import apollo as O
    f32 = lambda v: float(np.float32(v))
    ocfg = O.Config(rank=wl.rank, mode=wl.mode, seed=20241205, beta1=f32(wl.beta1), beta2=f32(wl.beta2),
                    eps=f32(wl.eps), scale=f32(wl.scale), nl_gamma=f32(wl.nl_gamma),
                    refresh_interval=wl.refresh_interval)
    ids, seen = [], set()
    for i, s in enumerate(wl.shapes[:7]):
        if s not in seen:
            seen.add(s)
            ids.append(i)
    ids = ids + [len(wl.shapes) - 7 + i for i in ids]
    Ws = [weights[i].cpu().double().numpy() for i in ids]
    Gs = [grads[i].cpu().float().double().numpy() for i in ids]
    sts = [O.init_state(ocfg, *wl.shapes[i]) for i in ids]
    bf16 = wl.grad_dtype == torch.bfloat16
    params = 0
    t0 = time.perf_counter()
    step = 0
    while True:
        step += 1
        for k, i in enumerate(ids):
            O.step(ocfg, sts[k], Ws[k], Gs[k], step, f32(wl.lr), tensor_id=i, grad_is_bf16=bf16)
            params += Ws[k].size
        el = time.perf_counter() - t0
        if el > budget_s or step >= 64 or el * (step + 1) / step > 1.5 * budget_s:
            break
    el = time.perf_counter() - t0
    try:
        import threadpoolctl
        threads = max([p["num_threads"] for p in threadpoolctl.threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count()
    return {"value": params / el, "unit": "params/s", "cores": int(threads), "kind": "oracle",
            "sample": "%d step(s) on %d tensors (one per distinct shape of the first and of the last layer: %s), "
                      "%.1f s, projection generation included" % (step, len(ids), [wl.shapes[i] for i in ids], el)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="llama7b_mini")
    ap.add_argument("--also", default="llama7b_r256,llama7b_mini_bf16,llama7b_r256_bf16,llama7b_mini_q8",
                    help="further variants on the same shapes, comma separated ('' = none)")
    ap.add_argument("--configs", default="llama60m,llama1b,llama13b_mini,llama13b_r256",
                    help="the benchmark definition's other full-size configurations, each on its own weights and "
                         "gradients, reported under 'also' (comma separated, '' = none); the LLaMA-13B ones time five "
                         "steps starting at step 201, which re-samples P (T = 200)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-adamw-rest", action="store_true",
                    help="skip the element-wise AdamW launch on the non-projected parameters")
    ap.add_argument("--no-overlap-leg", action="store_true",
                    help="skip the extra, separately timed run of the optional two-stream schedule (for "
                         "profiles of the default schedule alone)")
    ap.add_argument("--phase-pass", choices=["auto", "same", "separate"], default="auto",
                    help="per-phase times from the timed steps themselves (same) or from as many further steps "
                         "(separate: the timed steps then run without the library's events); auto: separate for "
                         "sets below 100 M parameters")
    ap.add_argument("--no-graph-leg", action="store_true",
                    help="skip the extra run of small sets replayed from a HIP graph (for profiles of the eager step alone)")
    ap.add_argument("--library-gemm-context", type=int, default=0, metavar="RANK",
                    help="also time torch.matmul on the projection's contraction at this rank (context only)")
    ap.add_argument("--only-adamw-rest", action="store_true", help="run only that launch (for profiling it)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run the library's plain copy kernel on 4 GiB a few times (known traffic: "
                         "4 GiB read + 4 GiB written per launch), for scaling rocprofv3 byte counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the optimizer step needs no communication under data "
              "parallelism (every rank repeats it), so --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2412_05270_amd as A
    from paper_2412_05270_amd import workloads as WL
    if not os.path.exists(A.library_path()):
        from paper_2412_05270_amd import build as _b
        _b.build(verbose=False)
    A.load_library()
    dev = "cuda:0"
    if args.copy_calibration:
        nbytes = 4 << 30
        src = torch.zeros(nbytes, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            assert A.apollo_debug_copy(dst.data_ptr(), src.data_ptr(), nbytes,
                                       torch.cuda.current_stream(dev).cuda_stream) == 0
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": {"kernel": "copy_kernel", "launches": 5, "bytes_read": nbytes,
                                               "bytes_written": nbytes}}))
        return
    if args.only_adamw_rest:
        print(json.dumps({"adamw_rest": measure_adamw_rest(A, torch, args.steps, args.warmup, dev, also_bf16=False)}))   # one variant: for profiling
        return
    wl = WL.workload(args.workload)
    weights = WL.make_q8_weights(wl, dev) if wl.weight_dtype == torch.uint8 else WL.make_weights(wl, dev)
    grads = [torch.empty(s, dtype=wl.grad_dtype, device=dev) for s in wl.shapes]
    torch.cuda.synchronize()
    main_res = measure(A, WL, torch, wl, weights, grads, args.steps, args.warmup, dev, not args.no_overlap_leg,
                       graph_leg=not args.no_graph_leg, phase_pass=args.phase_pass)
    cpu = None
    if not args.no_cpu_baseline:      # before `weights` is replaced by another variant's storage type
        cpu = cpu_baseline(A, WL, torch, wl, weights, grads)
    also = []
    cur_wdt = wl.weight_dtype
    for name in [a for a in args.also.split(",") if a]:
        wl2 = WL.workload(name)
        assert wl2.shapes == wl.shapes and wl2.grad_dtype == wl.grad_dtype
        if wl2.weight_dtype != cur_wdt:          # other weight type: the same values, stored in it
            del weights
            torch.cuda.empty_cache()
            weights = WL.make_q8_weights(wl2, dev) if wl2.weight_dtype == torch.uint8 else WL.make_weights(wl2, dev)
            cur_wdt = wl2.weight_dtype
        r2 = measure(A, WL, torch, wl2, weights, grads, args.steps, args.warmup, dev, not args.no_overlap_leg,
                     graph_leg=not args.no_graph_leg, phase_pass=args.phase_pass)
        also.append(entry_of(wl2, r2))
    del weights, grads
    torch.cuda.empty_cache()
    for name in [a for a in args.configs.split(",") if a]:
        wl3 = WL.workload(name)
        w3 = WL.make_weights(wl3, dev)
        g3 = [torch.empty(s, dtype=wl3.grad_dtype, device=dev) for s in wl3.shapes]
        if wl3.config_id == 5:      # "P refreshed on step 1 and every 200 steps, 5 steps timed": the first timed step is 201
            r3 = measure(A, WL, torch, wl3, w3, g3, 5, args.warmup, dev, False, first_step=201 - args.warmup, phase_pass=args.phase_pass)
        else:
            r3 = measure(A, WL, torch, wl3, w3, g3, args.steps, args.warmup, dev, False, phase_pass=args.phase_pass)
        also.append(entry_of(wl3, r3))
        del w3, g3
        torch.cuda.empty_cache()
    rest = None
    if not args.no_adamw_rest:
        rest = measure_adamw_rest(A, torch, args.steps, args.warmup, dev)
    lib = None
    if args.library_gemm_context > 0:
        lib = library_gemm_context(torch, wl, args.library_gemm_context, dev)
    out = {
        "metric": "APOLLO step params/s + % of HBM/MFMA roofline, LLaMA-7B-shaped params",
        "value": main_res["value"], "unit": "params/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": main_res["ms_per_step"], "device_ms_per_step": main_res["device_ms_per_step"],
        "min_ms_per_step": main_res["min_ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": describe(wl), "benchmark_config": wl.config_id, "params": wl.n_params, "tensors": len(wl.shapes),
                   "grad_dtype": str(wl.grad_dtype).replace("torch.", ""), "state_gb": main_res["state_gb"],
                   "workspace_gb": main_res["workspace_gb"]},
        "roofline": main_res["roofline"], "cpu_baseline": cpu, "phase_ms": main_res["phase_ms"],
        "overlap_schedule_ms_per_step": main_res.get("overlap_schedule_ms_per_step"),
        "chunked_schedule_ms_per_step": main_res.get("chunked_schedule_ms_per_step"),
        "chunked_schedule_workspace_gb": main_res.get("chunked_schedule_workspace_gb"),
        "whole_step_hbm_frac": main_res["whole_step_hbm_frac"], "projection_roofline": main_res["projection_roofline"],
        "finite": main_res["finite"], "also": also, "adamw_rest": rest, "library_gemm_context": lib,
    }
    print(json.dumps(out))


def library_gemm_context(torch, wl, rank, dev, reps=20):
    """Context only, never part of `value`: torch.matmul (the vendor GEMM library) on the same
    contraction as the rank-`rank` projection of this workload's shape groups -- bf16 operands, bf16
    output, no column sums, one batched call per group -- timed with events.  It shows what the
    stock library reaches on this skinny shape (r x m by m x n per tensor) on the same chip."""
    groups = {}
    for s in wl.shapes:
        groups[s] = groups.get(s, 0) + 1
    out, total_ms, total_flops = [], 0.0, 0.0
    for (rows, cols), count in sorted(groups.items()):
        G = torch.randn(count, rows, cols, device=dev, dtype=torch.bfloat16) * wl.grad_scale
        m = min(rows, cols)
        P = torch.randn(rank, m, device=dev, dtype=torch.bfloat16) / math.sqrt(rank)
        if rows <= cols:
            R = torch.empty(count, rank, cols, device=dev, dtype=torch.bfloat16)
            f = lambda: torch.matmul(P, G, out=R)
        else:
            Pt = P.t().contiguous()
            R = torch.empty(count * rows, rank, device=dev, dtype=torch.bfloat16)
            G2 = G.view(count * rows, cols)
            f = lambda: torch.mm(G2, Pt, out=R)
        for _ in range(3):
            f()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            f()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        flops = 2.0 * rank * rows * cols * count
        out.append({"shape": "%dx%d x%d" % (rows, cols, count), "ms": ms, "tflops": flops / ms / 1e9})
        total_ms += ms
        total_flops += flops
        del G, R
        torch.cuda.empty_cache()
    return {"kind": "torch.matmul, bf16 in and out, batched per shape group; context, not the product path",
            "rank": rank, "ms": total_ms, "tflops": total_flops / total_ms / 1e9, "groups": out}


def describe(wl):
    short = lambda dt: {"torch.bfloat16": "bf16", "torch.uint8": "8-bit (group 128, %s rounding)" % wl.weight_rounding}.get(str(dt), "fp32")
    return ("%s: %d matrices (%s), %s gradients ~ %s(%g), %s W, %s M/V, %s rank %d, alpha %.4g, T %d"
            % (wl.name, len(wl.shapes), ", ".join("%dx%d" % s for s in sorted(set(wl.shapes))),
               str(wl.grad_dtype).replace("torch.", ""), wl.grad_kind, wl.grad_scale, short(wl.weight_dtype),
               short(wl.state_dtype),
               ("full-rank moments, " if wl.projection == "identity" else "")
               + ("APOLLO-Mini tensor-wise" if wl.mode == "tensor" else "APOLLO channel-wise"), wl.rank, wl.scale,
               wl.refresh_interval))


if __name__ == "__main__":
    main()
