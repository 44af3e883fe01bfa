"""Every element of the two large configurations against the fp64 oracle.

(SGD with momentum on the 1.62 B list and Adam with coupled decay on the 1.56 B list get a full step and
a full undo the same way, at the end of this file.)
The 1.56 B-parameter list (bf16 gradients) and the 6.74 B-parameter list are stepped and undone by ONE
library call each, in the launch configuration the benchmark times (same binding calls, default launch
shape, state in the benchmark's default layout), and then ALL outputs -- theta, m and v of every tensor,
3 x 6.74 B values for the larger list -- are streamed to the host slice by slice and compared with the
oracle evaluated on the bits that were in device memory before the call:

  masked step (a seeded half of the tensors)  -> marked tensors: oracle step; unmarked tensors: bits unchanged
  selective undo of the marked tensors         -> marked: oracle undo of the stepped bits; unmarked: unchanged
  full step, full undo                         -> oracle step / undo, every element

Tolerance as everywhere: |gpu - oracle| <= max(1e-5 |oracle|, 1e-8) plus the one-ulp check of
gpu_util.assert_parity.  Gradients are checked through their digests (a changed word changes the digest).
The pre-call state is kept in a second copy on the device (theta, m, v: 81 GB for the larger list, which
together with the 108 GB state fits the 288 GB of one MI355X); device-to-host copies go through pinned
buffers on a side stream and overlap the oracle, which runs on all host cores the process may use."""
import concurrent.futures as cf
import os
import time

import numpy as np
import pytest
import torch

import oracle
from gpu_util import assert_parity, binding_hparams, digests_np, oracle_hyper

pytestmark = pytest.mark.gpu

SLICE = 1 << 25                      # elements per streamed slice (7 pinned buffers of 128 MiB per set)
WORKERS = max(1, min(16, len(os.sched_getaffinity(0))))
STAGES = ["masked_step", "selective_undo", "full_step", "full_undo"]


@pytest.fixture(scope="module")
def B():
    from paper_2302_06173_amd import binding
    return binding


@pytest.fixture(scope="module")
def synth():
    from paper_2302_06173_amd import synth
    return synth


class Flow:
    """One workload's state on the device, its pre-call copy, and the streaming comparison."""

    def __init__(self, B, synth, name, variant=None):
        self.B, self.synth = B, synth
        w = synth.workloads()[name]
        if variant is not None:                                  # the same shapes and values under another optimizer
            w = synth.Workload(**{**w.__dict__, **variant})
        self.w = w
        self.has_v = w.kind != "sgdm"
        self.sizes = [synth.numel(s) for s in w.shapes]
        self.n_t = len(self.sizes)
        self.N = sum(self.sizes)
        self.off = np.concatenate([[0], np.cumsum(self.sizes)]).astype(np.int64)
        self.s = synth.make_state(w, "cuda")                     # the benchmark's default layout
        self.ns = 3 if self.has_v else 2                         # state streams: theta, m (, v)
        self.snap = [torch.empty(self.N, dtype=torch.float32, device="cuda") for _ in range(self.ns)]
        self.hp = binding_hparams(B, w.kind, w.hyper, w.grad_bf16)
        self.oh = oracle_hyper(w.kind, w.hyper)
        self.tl = B.TensorList(self.s.theta, self.s.grad, self.s.m, self.s.v if self.has_v else None)
        frac = w.masked_fraction or 0.5
        self.mask = synth.tensor_mask(synth.Workload(**{**w.__dict__, "masked_fraction": frac}), self.n_t)
        gwords = [g.view(torch.int32) if g.dtype == torch.bfloat16 else g for g in self.s.grad]
        self.gbufs = B.BufferList(gwords)
        self.sbufs = B.BufferList(sum(self.streams(), []))
        self.g_digest = digests_np(B.swift_state_digest(self.gbufs, 0)).copy()
        self.copy_stream = torch.cuda.Stream()
        gdt = torch.int16 if w.grad_bf16 else torch.float32
        mk = lambda dt: torch.empty(SLICE, dtype=dt, pin_memory=True)
        self.pin = [dict(pre=[mk(torch.float32) for _ in range(self.ns)], g=mk(gdt),
                         post=[mk(torch.float32) for _ in range(self.ns)]) for _ in range(2)]
        self.pool = cf.ThreadPoolExecutor(WORKERS)
        self.done = []                                            # stages already run
        self.worst = 0.0
        self.snapshot()

    def streams(self):
        return [self.s.theta, self.s.m] + ([self.s.v] if self.has_v else [])

    def snapshot(self):
        for k, ts in enumerate(self.streams()):
            for i, t in enumerate(ts):
                self.snap[k][self.off[i]:self.off[i + 1]].copy_(t)

    # -- the library calls, one per stage -------------------------------------------------------
    def call(self, stage):
        B = self.B
        if stage == "masked_step":
            d0 = B.swift_state_digest(self.sbufs, 0)
            B.swift_opt_step(self.tl, self.hp, host_mask=self.mask)
            d1 = B.swift_state_digest(self.sbufs, 0)
            self.found = B.swift_mask_from_digests(d0, d1, self.n_t).cpu().tolist()
            return self.mask, False
        if stage == "selective_undo":
            assert self.found == self.mask, "digest-derived mask differs from the step mask"
            B.swift_opt_undo(self.tl, self.hp, host_mask=self.found)      # as the benchmark does: mask back on the host
            return self.mask, True
        if stage == "full_step":
            B.swift_opt_step(self.tl, self.hp)
            return None, False
        B.swift_opt_undo(self.tl, self.hp)
        return None, True

    # -- slices -------------------------------------------------------------------------------
    def jobs(self, mask):
        """Ranges [a, b) of the flat element space, at most SLICE long, each all marked or all unmarked."""
        out, i = [], 0
        while i < self.n_t:
            marked = True if mask is None else bool(mask[i])
            j = i
            while j < self.n_t and (True if mask is None else bool(mask[j])) == marked:
                j += 1
            a, end = int(self.off[i]), int(self.off[j])
            while a < end:
                b = min(a + SLICE, end)
                out.append((a, b, marked))
                a = b
            i = j
        return out

    def pieces(self, a, b):
        """(tensor, lo, hi, position in the slice) for the tensors that [a, b) covers."""
        i = int(np.searchsorted(self.off, a, side="right") - 1)
        out = []
        while a < b:
            while self.off[i + 1] <= a:
                i += 1
            hi = min(b, int(self.off[i + 1]))
            out.append((i, a - int(self.off[i]), hi - int(self.off[i])))
            a = hi
        return out

    def fetch(self, job, pin):
        a, b, marked = job
        n = b - a
        with torch.cuda.stream(self.copy_stream):
            for k in range(self.ns):
                pin["pre"][k][:n].copy_(self.snap[k][a:b], non_blocking=True)
            pos = 0
            for (i, lo, hi) in self.pieces(a, b):
                m = hi - lo
                if marked:
                    g = self.s.grad[i]
                    g = g.view(torch.int16) if g.dtype == torch.bfloat16 else g
                    pin["g"][pos:pos + m].copy_(g[lo:hi], non_blocking=True)
                for k, ts in enumerate(self.streams()):
                    pin["post"][k][pos:pos + m].copy_(ts[i][lo:hi], non_blocking=True)
                pos += m
            ev = torch.cuda.Event()
            ev.record()
        return ev

    def compare(self, job, pin, undo, what):
        a, b, marked = job
        n = b - a
        pre = [p[:n].numpy() for p in pin["pre"]]
        post = [p[:n].numpy() for p in pin["post"]]
        if not marked:
            for k in range(self.ns):
                assert np.array_equal(pre[k].view(np.uint32), post[k].view(np.uint32)), \
                    f"{what}: an unmarked tensor changed in elements [{a}, {b})"
            return 0.0
        g = pin["g"][:n].numpy()
        g = g.view(np.uint16) if g.dtype == np.int16 else g
        fn = oracle.opt_undo if undo else oracle.opt_step
        bounds = [n * k // WORKERS for k in range(WORKERS + 1)]

        def part(k):
            lo, hi = bounds[k], bounds[k + 1]
            if lo == hi:
                return 0.0
            x, gg, m = pre[0][lo:hi], g[lo:hi], pre[1][lo:hi]
            v = pre[2][lo:hi] if self.has_v else None
            rx, rm, rv = fn(self.oh, x, gg, m, v)
            sc = max(float(np.abs(x).max()), float(np.abs(oracle.widen(gg)).max()), float(np.abs(m).max()),
                     float(np.abs(v).max()) if self.has_v else 0.0)
            tag = f"{what} elements [{a + lo}, {a + hi})"
            assert_parity(post[0][lo:hi], rx, tag + " theta", sc)
            assert_parity(post[1][lo:hi], rm, tag + " m", sc)
            if self.has_v:
                assert_parity(post[2][lo:hi], rv, tag + " v", sc * max(sc, 1.0))
            # what is reported: the largest error in units of the tolerance max(1e-5 |oracle|, 1e-8)
            used = 0.0
            for q, r in ((post[0][lo:hi], rx), (post[1][lo:hi], rm)) + (((post[2][lo:hi], rv),) if self.has_v else ()):
                used = max(used, float(np.max(np.abs(q.astype(np.float64) - r) / np.maximum(1e-5 * np.abs(r), 1e-8))))
            return used
        return max(self.pool.map(part, range(WORKERS)))

    def run(self, stage, check=True):
        mask, undo = self.call(stage)
        torch.cuda.synchronize()
        compared = 0
        if check:
            jobs = self.jobs(mask)
            ev = self.fetch(jobs[0], self.pin[0])
            for j, job in enumerate(jobs):
                ev.synchronize()
                nxt = self.fetch(jobs[j + 1], self.pin[(j + 1) % 2]) if j + 1 < len(jobs) else None
                self.worst = max(self.worst, self.compare(job, self.pin[j % 2], undo, f"{self.w.name} {stage}"))
                compared += job[1] - job[0]
                ev = nxt
            assert compared == self.N
            after = digests_np(self.B.swift_state_digest(self.gbufs, 0))
            assert np.array_equal(after, self.g_digest), f"{stage}: a gradient was written"
        self.snapshot()
        torch.cuda.synchronize()
        self.done.append(stage)
        return compared

    def advance_to(self, stage):
        """Runs (unchecked) whatever stages come before `stage` and have not been run yet."""
        for s in STAGES[:STAGES.index(stage)]:
            if s not in self.done:
                self.run(s, check=False)

    def close(self):
        self.pool.shutdown()


_current = {}


# Other optimizers on the same shapes: Adam with coupled decay (App. A "Adam" / "Undo Adam") on the 1.56 B list.
VARIANTS = {
    "gpt2_xl_adam_l2_bf16g": ("gpt2_xl_adamw_bf16g",
                              dict(name="gpt2_xl_adam_l2_bf16g", kind="adam",
                                   hyper=dict(lr=1e-3, weight_decay=0.01, beta1=0.9, beta2=0.999, eps=1e-8, step=1000))),
}


def _flow(B, synth, name):
    """One large state at a time: switching workloads releases the previous one first."""
    key = name
    variant = None
    if name in VARIANTS:
        name, variant = VARIANTS[name]
    if _current.get("name") != key:
        old = _current.pop("flow", None)
        _current.clear()
        if old is not None:
            old.close()
            del old
        torch.cuda.empty_cache()
        w = synth.workloads()[name]
        need = w.n_params * ((2 if w.grad_bf16 else 4) + 12 + 12) * 1.04 + 4e9         # state, its copy, padding
        free, _ = torch.cuda.mem_get_info()
        if free < need:
            pytest.skip(f"needs about {need / 1e9:.0f} GB of free device memory")
        _current["flow"] = Flow(B, synth, name, variant)
        _current["name"] = key
    return _current["flow"]


@pytest.fixture(scope="module", autouse=True)
def _release_at_the_end():
    yield
    old = _current.pop("flow", None)
    _current.clear()
    if old is not None:
        old.close()
        del old
    torch.cuda.empty_cache()


@pytest.mark.parametrize("stage", STAGES)                                     # varies fastest: one state per workload
@pytest.mark.parametrize("name", ["gpt2_xl_adamw_bf16g", "llama7b_adamw"])
def test_every_element_against_the_oracle(B, synth, name, stage, capsys):
    flow = _flow(B, synth, name)
    flow.advance_to(stage)
    t0 = time.perf_counter()
    compared = flow.run(stage)
    dt = time.perf_counter() - t0
    with capsys.disabled():
        print(f"\n[full coverage] {name} {stage}: {compared:,} elements x (theta, m, v) compared in {dt:.1f} s, "
              f"largest error so far {flow.worst:.3f} of the tolerance", flush=True)


@pytest.mark.parametrize("stage", ["full_step", "full_undo"])
@pytest.mark.parametrize("name", ["vit_128_32_sgdm", "gpt2_xl_adam_l2_bf16g"])
def test_every_element_other_optimizers(B, synth, name, stage, capsys):
    """SGD with momentum (Alg. 1 / Alg. 2) on the 1.62 B-parameter list and Adam with coupled decay on the 1.56 B
    list with bf16 gradients: one full step and one full undo each, every element against the oracle."""
    flow = _flow(B, synth, name)
    if stage == "full_undo" and "full_step" not in flow.done:
        flow.run("full_step", check=False)
    t0 = time.perf_counter()
    compared = flow.run(stage)
    dt = time.perf_counter() - t0
    with capsys.disabled():
        print(f"\n[full coverage] {name} {stage}: {compared:,} elements x {flow.ns} state streams compared in {dt:.1f} s, "
              f"largest error so far {flow.worst:.3f} of the tolerance", flush=True)
