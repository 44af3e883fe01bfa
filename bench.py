#!/usr/bin/env python3
"""Benchmark of the update-undo hot path on one MI355X.

One "step" of this benchmark is one pass of the whole hot path over the workload's state, which is
resident in HBM before the clock starts:

  1. digest of theta, m, v per tensor                       (state at iteration t)
  2. AdamW step on a seeded random half of the tensors      (an update interrupted by a failure)
  3. digest again, 4. per-tensor "updated" mask from the two digest arrays (on the device), copied
     to the host (one byte per tensor: the only synchronisation of the pass)
  5. AdamW undo of exactly the marked tensors               (selective undo, grid sized to them)
  6. full AdamW step + full AdamW undo
  7. full Adam (coupled decay) step + undo
  8. full SGD-momentum step + undo (theta, g, m only)

`value` is the metric's quantity, Adam update-undo throughput: the parameters of the full list
stepped by AdamW plus the parameters undone by its undo (2 x N) over the time of those two launches
(item 6), measured with HIP events on the launching stream inside the timed pass and averaged over
the timed passes.  `ms_per_step` is the wall time of a whole pass; `whole_pass` gives the number of
parameter updates and undos of all optimizers over that wall time (digests and the mask derivation
are in the time, not in the count).  The `roofline` object describes the dominant kernel, AdamW undo
(launched twice per pass: selective and full list): mean algorithmic bytes per launch (28 per
parameter with fp32 gradients: theta, g, m, v in; theta, m, v out) over the mean launch duration,
from the same events.  The state lives in one arena laid out by swift_arena_layout's rule (--layout
padded, the default); `roofline_framework_layout` is the same kernel timed in the same run on a state
allocated the way a training framework allocates (one allocation per buffer, --layout framework).
`cpu_baseline` times the fp64 CPU oracle on a bounded sample of the same workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline] [--no-extras]
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

METRIC = "params/sec and HBM GB/s (% of roofline) for Adam update-undo, 1 MI355X"
HBM_PEAK_GBS = 8000.0                 # MI355X published HBM3E bandwidth
TRAFFIC_NOTE = os.path.join(ROOT, "profiles", "adamw_undo_llama7b_hbm_traffic.txt")


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def measured_traffic(workload: str):
    """HBM bytes per AdamW-undo launch from the committed rocprofv3 counter summary, if it covers
    this workload (the counters cannot be read from inside this process)."""
    try:
        with open(TRAFFIC_NOTE) as fh:
            rec = dict(l.split(":", 1) for l in fh if ":" in l and not l.startswith("#"))
        if rec.get("workload", "").strip() == workload:
            return float(rec["traffic_bytes_per_launch"])
    except (OSError, KeyError, ValueError):
        pass
    return None


def cpu_baseline(w, state, hp_dict, sample_elems: int):
    """The oracle, as it stands, on the first `sample_elems` elements of the list: AdamW step then
    undo (its own fp64 state) plus the digest of theta, m and v; all cores, static split."""
    import concurrent.futures as cf
    import numpy as np
    import oracle

    import torch

    def head(ts):
        """The first sample_elems elements of the list, tensors concatenated in list order."""
        parts, left = [], sample_elems
        for t in ts:
            if left <= 0:
                break
            parts.append(t[:left] if t.dtype == torch.float32 else t[:left].float())   # bf16 -> fp32 is exact
            left -= parts[-1].numel()
        return torch.cat(parts).cpu().numpy()

    cores = min(len(os.sched_getaffinity(0)), 16)
    x32, g32, m32, v32 = head(state.theta), head(state.grad), head(state.m), head(state.v)
    n = x32.size
    x, g, m, v = (oracle.widen(a) for a in (x32, g32, m32, v32))
    oh = oracle.Hyper("adamw", eta=hp_dict["lr"], lam=hp_dict["weight_decay"], beta1=hp_dict["beta1"],
                      beta2=hp_dict["beta2"], eps=hp_dict["eps"], t=hp_dict["step"])
    bounds = [n * k // cores for k in range(cores + 1)]
    stepped = [None] * cores

    def do_step(k):
        lo, hi = bounds[k], bounds[k + 1]
        stepped[k] = oracle.opt_step(oh, x[lo:hi], g[lo:hi], m[lo:hi], v[lo:hi])

    def do_undo(k):
        lo, hi = bounds[k], bounds[k + 1]
        sx, sm, sv = stepped[k]
        oracle.opt_undo(oh, sx, g[lo:hi], sm, sv)

    def do_digest(k):
        lo, hi = bounds[k], bounds[k + 1]
        for a in (x32, m32, v32):
            oracle.digest(a[lo:hi])

    best = {}
    with cf.ThreadPoolExecutor(cores) as pool:
        for _ in range(3):                       # first round also warms the allocator's pages
            for name, fn in (("adamw_step", do_step), ("adamw_undo", do_undo), ("digest", do_digest)):
                t0 = time.perf_counter()
                list(pool.map(fn, range(cores)))
                dt = time.perf_counter() - t0
                best[name] = dt if name not in best else min(best[name], dt)
    n1 = n // cores
    t0 = time.perf_counter()
    sx, sm, sv = oracle.opt_step(oh, x[:n1], g[:n1], m[:n1], v[:n1])
    oracle.opt_undo(oh, sx, g[:n1], sm, sv)
    t1 = time.perf_counter() - t0
    g_bytes = 2 if state.grad[0].dtype == torch.bfloat16 else 4
    per_kernel = {
        "adamw_step": {"gparams_per_s": round(n / best["adamw_step"] / 1e9, 3),
                       "gb_per_s": round((24 + g_bytes) * n / best["adamw_step"] / 1e9, 1)},
        "adamw_undo": {"gparams_per_s": round(n / best["adamw_undo"] / 1e9, 3),
                       "gb_per_s": round((24 + g_bytes) * n / best["adamw_undo"] / 1e9, 1)},
        "digest_theta_m_v": {"gb_per_s": round(12 * n / best["digest"] / 1e9, 1)},
    }
    whole = best["adamw_step"] + best["adamw_undo"] + best["digest"]
    return {"value": 2 * n / whole, "unit": "params/s", "cores": cores, "kind": "oracle",
            "sample": f"AdamW step, undo and 3 digests on the first {n} elements of the {w.name} list, each timed on its own, "
                      f"static split over {cores} threads, best of 3; value = 2 x elements / (step + undo + digest time)",
            "per_kernel": per_kernel,
            "single_thread_value": 2 * n1 / t1}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama7b_adamw")
    ap.add_argument("--layout", default="padded", choices=["padded", "by_tensor", "by_stream", "framework"],
                    help="where the state tensors are allocated (same values either way): one arena with theta, g, m, v "
                         "of a tensor side by side and 4 KiB of skew between buffers (default); the same order in "
                         "separate torch allocations; all theta, then all g, m, v; or as a training framework would")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-second-layout", action="store_true",
                    help="skip the second roofline measurement (the dominant kernel on a framework-style allocation)")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the launches reported under 'extras' (a profile of such a run holds the timed pass only)")
    ap.add_argument("--cpu-sample", type=int, default=256 * 1024 * 1024)
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="BYTES",
                    help="only run swift_stream_copy on BYTES bytes five times (a copy of known size, to "
                         "scale a profiler's HBM byte counters) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU: the update-undo path needs no communication, every replica "
            "undoes its own copy.  Run with --gpus 1.")
        return 2

    import torch
    from paper_2302_06173_amd import build as hip_build
    hip_build.ensure_built()                      # loads what is built; builds only if there is no library
    from paper_2302_06173_amd import binding as B, synth

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        return 2
    torch.cuda.set_device(0)
    if args.copy_calibration:
        n = args.copy_calibration // 16 * 16
        src = torch.empty(n, dtype=torch.uint8, device="cuda").fill_(0x3c)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(5):
            B.swift_stream_copy(dst, src)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / 5
        print(json.dumps({"copy_bytes": n, "launches": 5, "ms_per_launch": 1e3 * dt,
                          "gb_per_s": 2 * n / dt / 1e9}), flush=True)
        return 0
    w = synth.workloads()[args.workload]
    N, n_t = w.n_params, len(w.shapes)
    log(f"[bench] workload {w.name}: {n_t} tensors, {N:,} params; drawing state on the GPU ...")
    t0 = time.perf_counter()
    state = synth.make_state(w, "cuda:0", with_v=True, layout=args.layout)
    torch.cuda.synchronize()
    log(f"[bench] state ready in {time.perf_counter() - t0:.1f} s; "
        f"{torch.cuda.memory_allocated() / 1e9:.1f} GB allocated")

    bf16 = w.grad_bf16
    own = dict(w.hyper)
    t_step = own.get("step", 1)
    hp_dicts = {
        "adamw": dict(lr=6e-4, weight_decay=0.1, beta1=0.9, beta2=0.95, eps=1e-8, step=t_step),
        "adam": dict(lr=1e-3, weight_decay=0.0, beta1=0.9, beta2=0.999, eps=1e-8, step=t_step),
        "sgdm": dict(lr=0.1, weight_decay=1e-4, momentum=0.9, dampening=0.0, step=t_step),
    }
    hp_dicts[w.kind] = {**hp_dicts[w.kind], **own}
    hps = {k: B.hparams(k, grad_bf16=bf16, **d) for k, d in hp_dicts.items()}
    tl_adam = B.TensorList(state.theta, state.grad, state.m, state.v)
    tl_sgdm = B.TensorList(state.theta, state.grad, state.m, None)
    bufs = B.BufferList(state.theta + state.m + state.v)
    frac = w.masked_fraction if w.masked_fraction > 0 else 0.5
    wm = synth.Workload(**{**w.__dict__, "masked_fraction": frac})
    mask = synth.tensor_mask(wm, n_t)
    n_masked = sum(synth.numel(s) for s, b in zip(w.shapes, mask) if b)
    n_digests = B.swift_digest_count([t.numel() for t in bufs._keep], 0)
    d0 = torch.empty(n_digests, dtype=torch.int64, device="cuda")
    d1 = torch.empty_like(d0)
    dmask = torch.empty(n_t, dtype=torch.uint8, device="cuda")

    segs = ["digest_pre", "adamw_step_masked", "digest_post", "mask_from_digests", "adamw_undo_selective",
            "adamw_step", "adamw_undo", "adam_step", "adam_undo", "sgdm_step", "sgdm_undo"]
    g_bytes = 2 if bf16 else 4
    seg_bytes = {"digest_pre": 12 * N, "digest_post": 12 * N, "mask_from_digests": 0,
                 "adamw_step_masked": (24 + g_bytes) * n_masked, "adamw_undo_selective": (24 + g_bytes) * n_masked,
                 "adamw_step": (24 + g_bytes) * N, "adamw_undo": (24 + g_bytes) * N,
                 "adam_step": (24 + g_bytes) * N, "adam_undo": (24 + g_bytes) * N,
                 "sgdm_step": (16 + g_bytes) * N, "sgdm_undo": (16 + g_bytes) * N}
    seg_params = {s: 0 for s in segs}
    seg_params.update({"adamw_step_masked": n_masked, "adamw_undo_selective": n_masked, "adamw_step": N,
                       "adamw_undo": N, "adam_step": N, "adam_undo": N, "sgdm_step": N, "sgdm_undo": N})

    def one_pass(events=None):
        def mark():
            if events is not None:
                e = torch.cuda.Event(enable_timing=True)
                e.record()
                events.append(e)
        mark()
        B.swift_state_digest(bufs, 0, out=d0); mark()
        B.swift_opt_step(tl_adam, hps["adamw"], host_mask=mask); mark()
        B.swift_state_digest(bufs, 0, out=d1); mark()
        B.swift_mask_from_digests(d0, d1, n_t, out=dmask)
        found = dmask.cpu().tolist(); mark()          # n_t bytes to the host: the only synchronisation of the pass
        B.swift_opt_undo(tl_adam, hps["adamw"], host_mask=found); mark()
        B.swift_opt_step(tl_adam, hps["adamw"]); mark()
        B.swift_opt_undo(tl_adam, hps["adamw"]); mark()
        B.swift_opt_step(tl_adam, hps["adam"]); mark()
        B.swift_opt_undo(tl_adam, hps["adam"]); mark()
        B.swift_opt_step(tl_sgdm, hps["sgdm"]); mark()
        B.swift_opt_undo(tl_sgdm, hps["sgdm"]); mark()

    for _ in range(args.warmup):
        one_pass()
    all_events = []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        ev = []
        one_pass(ev)
        all_events.append(ev)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    if dmask.cpu().tolist() != [1 if (b and synth.numel(s)) else 0 for b, s in zip(mask, w.shapes)]:
        log("[bench] ERROR: digest-derived mask differs from the step mask")
        return 1

    # Outside the timed pass and outside `value`, reported under "extras": LAMB step (three launches,
    # 40 bytes per parameter) and its saved-norm undo; step / undo that also return the digests; step /
    # undo that also write a bfloat16 copy of theta; the selective undo with the mask left on the device.
    extras = {}

    def extra(name, fn, bytes_per_param, n_params=N):
        reps = max(3, min(args.steps, 10))
        fn()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
        ev[0].record()
        for k in range(reps):
            fn()
            ev[k + 1].record()
        torch.cuda.synchronize()
        ms = ev[0].elapsed_time(ev[reps]) / reps
        extras[name] = {"ms": round(ms, 4), "gparams_per_s": round(n_params / ms / 1e6, 2),
                        "gb_per_s": round(bytes_per_param * n_params / ms / 1e6, 1), "bytes_per_param": bytes_per_param}
        log(f"[bench] {name:26s} {ms:9.3f} ms  {extras[name]['gparams_per_s']} Gparam/s  {extras[name]['gb_per_s']} GB/s")

    hp_w = hps["adamw"]
    if args.no_extras:
        def extra(*a, **k):
            return None
    if not bf16 and not args.no_extras:
        hp_lamb = B.hparams("lamb", step=t_step, lr=2e-3, weight_decay=0.01, beta1=0.9, beta2=0.999, eps=1e-6)
        norms = torch.zeros(2 * n_t, dtype=torch.float64, device="cuda")
        extra("lamb_step", lambda: B.swift_lamb_step(tl_adam, hp_lamb, norms), 40)
        extra("lamb_undo", lambda: B.swift_lamb_undo(tl_adam, hp_lamb, norms), 28)
    # App. A's plain SGD: no optimizer state, theta and the gradient only
    hp_sgd = B.hparams("sgd", step=t_step, lr=0.1, weight_decay=1e-4, grad_bf16=bf16)
    tl_sgd = None if args.no_extras else B.TensorList(state.theta, state.grad)
    extra("sgd_step", lambda: B.swift_opt_step(tl_sgd, hp_sgd), 8 + g_bytes)
    extra("sgd_undo", lambda: B.swift_opt_undo(tl_sgd, hp_sgd), 8 + g_bytes)
    dig = torch.zeros(3 * n_t, dtype=torch.int64, device="cuda")
    extra("adamw_step_with_digest", lambda: B.swift_opt_step_digest(tl_adam, hp_w, dig), 24 + g_bytes)
    extra("adamw_undo_with_digest", lambda: B.swift_opt_undo_digest(tl_adam, hp_w, dig), 24 + g_bytes)
    xb = [torch.empty(0 if args.no_extras else t.numel(), dtype=torch.bfloat16, device="cuda") for t in state.theta]
    tl_xb = None if args.no_extras else B.TensorList(state.theta, state.grad, state.m, state.v, param_bf16=xb)
    extra("adamw_step_bf16_copy", lambda: B.swift_opt_step(tl_xb, hp_w), 26 + g_bytes)
    extra("adamw_undo_bf16_copy", lambda: B.swift_opt_undo(tl_xb, hp_w), 26 + g_bytes)
    del xb, tl_xb

    # the paper's own bookkeeping: the update launched group by group (here: about nine tensors per group, as
    # gradients of one layer become final), every launch tracked, then the undo of whatever is marked
    per_group = 9
    ids = [list(range(k, min(k + per_group, n_t))) for k in range(0, n_t, per_group)]
    groups = [B.TensorList([state.theta[i] for i in g], [state.grad[i] for i in g], [state.m[i] for i in g],
                           [state.v[i] for i in g]) for g in ids]
    tracker = B.Tracker(n_t)
    id_arrays = [B.Tracker.ids(g) for g in ids]

    hp_a = hps["adam"]       # Adam, not AdamW: the roofline kernel's launches stay those of the timed pass

    def tracked_step_and_undo():
        tracker.begin(t_step)
        for g, tl_g in zip(id_arrays, groups):
            tracker.step(tl_g, g, hp_a)
        tracker.undo(tl_adam, hp_a)
    extra(f"adam_tracked_step_in_{len(groups)}_groups_plus_undo", tracked_step_and_undo, 24 + g_bytes, 2 * N)
    tracker.close()

    def masked_pair():
        B.swift_opt_step_dmask(tl_adam, hp_w, dmask)
        B.swift_opt_undo_dmask(tl_adam, hp_w, dmask)
    extra("adamw_step_undo_device_mask", masked_pair, 24 + g_bytes, 2 * n_masked)

    # The chip's own 1-read/1-write ceiling with the same launch style (a plain copy of 4 GiB), measured here so
    # that the roofline fraction can also be read against what this GPU delivers, not only against the data sheet.
    ceil_src = torch.empty(1 << 32, dtype=torch.uint8, device="cuda").fill_(0x3c)
    ceil_dst = torch.empty_like(ceil_src)
    B.swift_stream_copy(ceil_dst, ceil_src)
    cev = [torch.cuda.Event(enable_timing=True) for _ in range(6)]
    cev[0].record()
    for k in range(5):
        B.swift_stream_copy(ceil_dst, ceil_src)
        cev[k + 1].record()
    torch.cuda.synchronize()
    copy_gbs = 2 * ceil_src.numel() / min(cev[k].elapsed_time(cev[k + 1]) for k in range(5)) / 1e6
    del ceil_src, ceil_dst
    log(f"[bench] copy ceiling (4 GiB, best of 5): {copy_gbs:.0f} GB/s")

    seg_all = {s: sorted(ev[k].elapsed_time(ev[k + 1]) for ev in all_events) for k, s in enumerate(segs)}
    seg_ms = {s: sum(v) / max(len(v), 1) for s, v in seg_all.items()}
    params_per_pass = sum(seg_params.values())
    whole_pass_value = params_per_pass * args.steps / wall
    value = 2 * N / ((seg_ms["adamw_step"] + seg_ms["adamw_undo"]) * 1e-3)     # Adam update-undo: full step + full undo
    kernels = {}
    for s in segs:
        ms = seg_ms[s]
        kernels[s] = {"ms": round(ms, 4), "ms_median": round(seg_all[s][len(seg_all[s]) // 2], 4),
                      "ms_best": round(seg_all[s][0], 4),
                      "gparams_per_s": round(seg_params[s] / ms / 1e6, 2) if ms > 0 else None,
                      "gb_per_s": round(seg_bytes[s] / ms / 1e6, 1) if ms > 0 else None}
        log(f"[bench] {s:22s} {ms:9.3f} ms  {kernels[s]['gparams_per_s']} Gparam/s  {kernels[s]['gb_per_s']} GB/s")
    # The AdamW undo kernel is launched twice per pass (selective undo of the marked half, then the
    # full list); a profiler averages over both, so the roofline figure does too.
    dom = ("adamw_undo_selective", "adamw_undo")
    dom_bytes = sum(seg_bytes[s] for s in dom) / len(dom)
    dom_ms = sum(seg_ms[s] for s in dom) / len(dom)
    dom_params = sum(seg_params[s] for s in dom) / len(dom)
    achieved = dom_bytes / dom_ms / 1e6
    traffic = measured_traffic(w.name)
    out = {
        "metric": METRIC, "value": value, "unit": "params/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": 1e3 * wall / max(args.steps, 1), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": f"{w.name}: {n_t} tensors, {N} params, fp32 theta/m/v, "
                               f"{'bf16' if bf16 else 'fp32'} grads, {torch.cuda.memory_allocated() / 1e9:.1f} GB resident",
                   "pass": "digest, masked AdamW step, digest, mask, selective undo, full AdamW/Adam/SGDM step+undo",
                   "value_is": "2 x params / (full-list AdamW step + full-list AdamW undo launch time), HIP events inside the timed pass",
                   "allocation_layout": args.layout,
                   "storage": "fp32 state, arithmetic in fp64 registers"},
        "whole_pass": {"params_updated_or_undone_per_pass": params_per_pass, "params_per_s": whole_pass_value,
                       "note": "all optimizers' updates and undos over the wall time of the pass, digests and mask included in the time"},
        "roofline": {"bound": "hbm", "kernel": "opt_kernel<AdamW, undo>: mean of its 2 launches per pass "
                                                 "(selective undo of the marked tensors, full list)",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic,
                     "traffic_source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary kept under profiles/ (counters "
                                       "cannot be read from inside this process); null if it does not cover this workload",
                     "algorithmic_bytes_per_launch": dom_bytes, "avg_launch_ms": dom_ms,
                     "measured_copy_gb_per_s": copy_gbs, "frac_of_measured_copy": achieved / copy_gbs,
                     "gparams_per_s": dom_params / dom_ms / 1e6},
        "kernels": kernels,
        "extras": extras,
    }
    if not args.no_cpu_baseline:
        log("[bench] timing the CPU oracle on a bounded sample ...")
        out["cpu_baseline"] = cpu_baseline(w, state, hp_dicts["adamw"], args.cpu_sample)
    if not args.no_second_layout and args.layout != "framework":
        # The same two launches of the dominant kernel on a state allocated as a training framework allocates it:
        # every buffer an allocation of its own (theta at model build, gradients in backward order, m and v at
        # the first optimizer step).  Same values, same kernels; only the addresses differ.
        del tl_adam, tl_sgdm, bufs, groups, state
        B.swift_cache_trim(0)
        torch.cuda.empty_cache()
        log("[bench] second layout: drawing the state in framework-style allocations ...")
        state = synth.make_state(w, "cuda:0", with_v=True, layout="framework")
        tl_fw = B.TensorList(state.theta, state.grad, state.m, state.v)
        names = ("adamw_step_masked", "adamw_undo_selective", "adamw_step", "adamw_undo")

        def fw_pass(events=None):
            def mark():
                if events is not None:
                    e = torch.cuda.Event(enable_timing=True)
                    e.record()
                    events.append(e)
            mark()
            B.swift_opt_step(tl_fw, hp_w, host_mask=mask); mark()
            B.swift_opt_undo(tl_fw, hp_w, host_mask=mask); mark()
            B.swift_opt_step(tl_fw, hp_w); mark()
            B.swift_opt_undo(tl_fw, hp_w); mark()
        for _ in range(max(args.warmup, 2)):
            fw_pass()
        fw_events = []
        for _ in range(max(3, min(args.steps, 10))):
            ev = []
            fw_pass(ev)
            fw_events.append(ev)
        torch.cuda.synchronize()
        fw_ms = {s_: sum(ev[k].elapsed_time(ev[k + 1]) for ev in fw_events) / len(fw_events) for k, s_ in enumerate(names)}
        fw_dom_ms = (fw_ms["adamw_undo_selective"] + fw_ms["adamw_undo"]) / 2
        fw_achieved = dom_bytes / fw_dom_ms / 1e6
        out["roofline_framework_layout"] = {
            "bound": "hbm", "kernel": out["roofline"]["kernel"], "allocation_layout": "framework",
            "achieved": fw_achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": fw_achieved / HBM_PEAK_GBS,
            "traffic": None, "algorithmic_bytes_per_launch": dom_bytes, "avg_launch_ms": fw_dom_ms,
            "value_params_per_s": 2 * N / ((fw_ms["adamw_step"] + fw_ms["adamw_undo"]) * 1e-3),
            "kernels_ms": {k: round(v, 4) for k, v in fw_ms.items()}}
        log(f"[bench] framework layout: AdamW undo {fw_achieved:.0f} GB/s ({fw_achieved / HBM_PEAK_GBS:.3f} of peak), "
            f"step+undo {out['roofline_framework_layout']['value_params_per_s'] / 1e9:.1f} G params/s")
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
