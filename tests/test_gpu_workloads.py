"""GPU parity at the benchmark's real shapes: the five synthetic workloads and the additional SGD-momentum list, launched exactly as
bench.py launches them (same binding calls, default launch shape).

Small workloads are compared with the fp64 oracle element by element over every tensor.  For the
1.5 B and 7 B lists the oracle checks whole sampled tensors plus windows of the largest ones
(starts, chunk boundaries, ragged ends), and properties that hold at any size cover the rest:
gradients and unmarked tensors keep their digests (i.e. their bits), every marked non-empty tensor
changes its digest, and the mask derived from digests on the device equals the step mask."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import assert_parity, binding_hparams, digests_np, oracle_hyper, to_np

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2302_06173_amd import binding
    return binding


@pytest.fixture(scope="module")
def synth():
    from paper_2302_06173_amd import synth
    return synth


def _scale(*arrs):
    s = 0.0
    for a in arrs:
        if a is not None and a.size:
            s = max(s, float(np.abs(oracle.widen(a)).max()))
    return s


def _check_slices(kind, hpd, pre, post, undo, what):
    """pre/post: dicts key -> (x, g, m, v) numpy slices taken around one GPU call."""
    h = oracle_hyper(kind, hpd)
    fn = oracle.opt_undo if undo else oracle.opt_step
    for key in pre:
        x, g, m, v = pre[key]
        qx, qg, qm, qv = post[key]
        assert np.array_equal(g.view(np.uint8), qg.view(np.uint8)), f"{what} {key}: gradient written"
        rx, rm, rv = fn(h, x, g, m, v)
        sc = _scale(x, g, m, v)
        assert_parity(qx, rx, f"{what} theta {key}", sc)
        assert_parity(qm, rm, f"{what} m {key}", sc)
        if v is not None:
            assert_parity(qv, rv, f"{what} v {key}", sc * max(sc, 1.0))


def _grab(state, picks):
    """Host copies of the picked (tensor, lo, hi) ranges of all four streams."""
    out = {}
    for (i, lo, hi) in picks:
        v = None if state.v is None else to_np(state.v[i][lo:hi])
        out[(i, lo, hi)] = (to_np(state.theta[i][lo:hi]), to_np(state.grad[i][lo:hi]), to_np(state.m[i][lo:hi]), v)
    return out


def _all_ranges(shapes, synth):
    return [(i, 0, synth.numel(s)) for i, s in enumerate(shapes)]


def _sample_ranges(shapes, synth, every, window=70001, whole_limit=5_000_000):
    """Whole tensors for a spread of indices; windows (start, a 65,536-element chunk boundary in the
    middle, the ragged end) of tensors too large to check whole."""
    n_t = len(shapes)
    chosen = sorted(set([0, 1, 2, n_t - 2, n_t - 1] + list(range(3, n_t, every))))
    picks = []
    for i in chosen:
        n = synth.numel(shapes[i])
        if n <= whole_limit:
            picks.append((i, 0, n))
        else:
            mid = (n // 2) // 65536 * 65536
            picks += [(i, 0, window), (i, mid - window // 2, mid + window // 2), (i, n - window, n)]
    return picks


# ------------------------------------------------------------------------------------------
def test_sgdm_flat_1m(B, synth):
    """Configuration 1: step, undo, comparison with the originals, one digest per 64 Ki-element shard."""
    w = synth.workloads()["sgdm_flat_1m"]
    s = synth.make_state(w, "cuda")
    tl = B.TensorList(s.theta, s.grad, s.m, None)
    hp = binding_hparams(B, w.kind, w.hyper)
    picks = _all_ranges(w.shapes, synth)
    bufs = B.BufferList([s.theta[0], s.m[0]])
    orig = _grab(s, picks)
    d0 = B.swift_state_digest(bufs, w.digest_shard)
    B.swift_opt_step(tl, hp)
    d1 = B.swift_state_digest(bufs, w.digest_shard)
    torch.cuda.synchronize()
    mid = _grab(s, picks)
    B.swift_opt_undo(tl, hp)
    d2 = B.swift_state_digest(bufs, w.digest_shard)
    torch.cuda.synchronize()
    end = _grab(s, picks)
    _check_slices(w.kind, w.hyper, orig, mid, False, "sgdm step")
    _check_slices(w.kind, w.hyper, mid, end, True, "sgdm undo")
    key = picks[0]
    for k in (0, 2):                                   # theta and m come back within the stated bar
        a, b = end[key][k].astype(np.float64), orig[key][k].astype(np.float64)
        assert (np.abs(a - b) <= np.maximum(1e-5 * np.abs(b), 1e-8)).all()
    assert d0.numel() == 32
    assert np.array_equal(digests_np(d0), oracle.digest_list([orig[key][0], orig[key][2]], w.digest_shard))
    assert np.array_equal(digests_np(d1), oracle.digest_list([mid[key][0], mid[key][2]], w.digest_shard))
    assert np.array_equal(digests_np(d2), oracle.digest_list([end[key][0], end[key][2]], w.digest_shard))
    assert (digests_np(d0) != digests_np(d1)).all()    # every shard saw the step


@pytest.mark.parametrize("name", ["resnet50_adam", "bert_large_adamw"])
def test_full_list_elementwise(B, synth, name):
    """Configurations 2 and 3: every element of every tensor against the oracle, step then undo;
    configuration 3 also checks the per-tensor digests of theta, m and v."""
    w = synth.workloads()[name]
    s = synth.make_state(w, "cuda")
    tl = B.TensorList(s.theta, s.grad, s.m, s.v)
    hp = binding_hparams(B, w.kind, w.hyper)
    picks = _all_ranges(w.shapes, synth)
    orig = _grab(s, picks)
    B.swift_opt_step(tl, hp)
    torch.cuda.synchronize()
    mid = _grab(s, picks)
    _check_slices(w.kind, w.hyper, orig, mid, False, f"{name} step")
    del orig
    if name == "bert_large_adamw":
        d = B.swift_state_digest(s.theta + s.m + s.v, 0)
        torch.cuda.synchronize()
        want = oracle.digest_list([mid[k][0] for k in picks] + [mid[k][2] for k in picks] + [mid[k][3] for k in picks], 0)
        assert np.array_equal(digests_np(d), want)
    B.swift_opt_undo(tl, hp)
    torch.cuda.synchronize()
    end = _grab(s, picks)
    _check_slices(w.kind, w.hyper, mid, end, True, f"{name} undo")


def _selective_flow(B, synth, w, every):
    n_t = len(w.shapes)
    s = synth.make_state(w, "cuda")
    tl = B.TensorList(s.theta, s.grad, s.m, s.v)
    hp = binding_hparams(B, w.kind, w.hyper, w.grad_bf16)
    state_lists = [s.theta, s.m] + ([s.v] if s.v is not None else [])
    ng = len(state_lists)                                          # digest rows that a step changes
    written = (0, 2, 3)[:ng]                                       # their positions in a _grab tuple
    frac = w.masked_fraction or 0.5
    mask = synth.tensor_mask(synth.Workload(**{**w.__dict__, "masked_fraction": frac}), n_t)
    picks = _sample_ranges(w.shapes, synth, every)
    on = [p for p in picks if mask[p[0]]]
    off = [p for p in picks if not mask[p[0]]]
    assert on and off
    # gradients are digested too (as 32-bit words; bf16 tensors have an even element count here)
    gwords = [g.view(torch.int32) if g.dtype == torch.bfloat16 else g for g in s.grad]
    bufs = B.BufferList(sum(state_lists, []) + gwords)
    orig = _grab(s, picks)
    d0 = B.swift_state_digest(bufs, 0)
    B.swift_opt_step(tl, hp, host_mask=mask)                       # the interrupted update
    d1 = B.swift_state_digest(bufs, 0)
    dmask = B.swift_mask_from_digests(d0[:ng * n_t], d1[:ng * n_t], n_t)
    torch.cuda.synchronize()
    mid = _grab(s, picks)
    a, b = digests_np(d0).reshape(ng + 1, n_t), digests_np(d1).reshape(ng + 1, n_t)
    assert np.array_equal(a[ng], b[ng]), "a gradient changed"
    changed = (a[:ng] != b[:ng])
    assert np.array_equal(changed.all(axis=0), np.array(mask, bool)), "theta, m (and v) of exactly the marked tensors change"
    assert np.array_equal(dmask.cpu().numpy(), np.array(mask, np.uint8))
    # the oracle's hash of the sampled whole tensors agrees with the device digests
    for (i, lo, hi) in picks:
        if lo == 0 and hi == synth.numel(w.shapes[i]):
            assert a[0][i] == oracle.digest(orig[(i, lo, hi)][0])[0]
            assert b[1][i] == oracle.digest(mid[(i, lo, hi)][2])[0]
    _check_slices(w.kind, w.hyper, {k: orig[k] for k in on}, {k: mid[k] for k in on}, False, f"{w.name} masked step")
    for k in off:
        for j in written:
            assert np.array_equal(orig[k][j].view(np.uint32), mid[k][j].view(np.uint32)), f"unmarked {k} changed"
    del orig
    B.swift_opt_undo_dmask(tl, hp, dmask)                          # selective undo, mask stays on the device
    d2 = B.swift_state_digest(bufs, 0)
    torch.cuda.synchronize()
    end = _grab(s, picks)
    c = digests_np(d2).reshape(ng + 1, n_t)
    assert np.array_equal(c[ng], a[ng])
    off_idx = ~np.array(mask, bool)
    assert np.array_equal(c[:ng, off_idx], a[:ng, off_idx]), "an unmarked tensor changed during undo"
    _check_slices(w.kind, w.hyper, {k: mid[k] for k in on}, {k: end[k] for k in on}, True, f"{w.name} selective undo")
    for k in off:
        for j in written:
            assert np.array_equal(mid[k][j].view(np.uint32), end[k][j].view(np.uint32))
    # the benchmark's own selective undo: the mask comes back to the host, the grid covers the marked tensors only
    B.swift_opt_step(tl, hp, host_mask=mask)
    torch.cuda.synchronize()
    again = _grab(s, picks)
    B.swift_opt_undo(tl, hp, host_mask=dmask.cpu().tolist())
    torch.cuda.synchronize()
    back = _grab(s, picks)
    _check_slices(w.kind, w.hyper, {k: again[k] for k in on}, {k: back[k] for k in on}, True, f"{w.name} host-mask undo")
    for k in off:
        for j in written:
            assert np.array_equal(end[k][j].view(np.uint32), back[k][j].view(np.uint32))
    end = back
    # and one full-list step + undo in the launch configuration the benchmark times
    B.swift_opt_step(tl, hp)
    torch.cuda.synchronize()
    full = _grab(s, picks)
    _check_slices(w.kind, w.hyper, end, full, False, f"{w.name} full step")
    B.swift_opt_undo(tl, hp)
    torch.cuda.synchronize()
    _check_slices(w.kind, w.hyper, full, _grab(s, picks), True, f"{w.name} full undo")


def test_gpt2_xl_bf16_gradients_sampled(B, synth):
    """Configuration 4 (1.56 B parameters, bf16 gradients widened in the kernel)."""
    _selective_flow(B, synth, synth.workloads()["gpt2_xl_adamw_bf16g"], every=97)


def test_vit_128_32_sgdm_sampled(B, synth):
    """The additional SGD-momentum list (1.62 B parameters, 1,544 tensors; theta, g, m only)."""
    _selective_flow(B, synth, synth.workloads()["vit_128_32_sgdm"], every=131)


def test_llama7b_selective_undo_sampled(B, synth):
    """Configuration 5 (6.74 B parameters, 107.8 GB of state, zeros and outliers in g)."""
    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info()
    if free < 125e9:
        pytest.skip("needs about 110 GB of free device memory")
    _selective_flow(B, synth, synth.workloads()["llama7b_adamw"], every=41)


def test_tensor_beyond_2_pow_32_elements(B, synth):
    """Maximum sizes: one SGDM tensor of 2^32 + 70,003 elements (element offsets need 64 bits) checked
    on windows at the start, across the 2^32 boundary and at the ragged end; and a digest of a buffer of
    2^32 - 4 words in one shard (the largest index that fits the 32-bit index field) against the CPU hash."""
    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info()
    if free < 60e9:
        pytest.skip("needs about 55 GB of free device memory")
    n = (1 << 32) + 70003
    hpd = dict(lr=0.1, momentum=0.9, dampening=0.0, weight_decay=1e-4, step=1)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(99)
    x = torch.empty(n, dtype=torch.float32, device="cuda").normal_(0.0, 0.02, generator=gen)
    g = torch.empty(n, dtype=torch.float32, device="cuda").normal_(0.0, 1e-3, generator=gen)
    m = torch.empty(n, dtype=torch.float32, device="cuda").normal_(0.0, 1e-3, generator=gen)
    s = synth.State([x], [g], [m], None)
    b = 1 << 32
    picks = [(0, 0, 70001), (0, b - 35000, b + 35001), (0, n - 70001, n)]
    tl = B.TensorList(s.theta, s.grad, s.m, None)
    hp = binding_hparams(B, "sgdm", hpd)
    pre = _grab(s, picks)
    B.swift_opt_step(tl, hp)
    torch.cuda.synchronize()
    mid = _grab(s, picks)
    _check_slices("sgdm", hpd, pre, mid, False, "huge step")
    B.swift_opt_undo(tl, hp)
    torch.cuda.synchronize()
    _check_slices("sgdm", hpd, mid, _grab(s, picks), True, "huge undo")
    # digest: whole-buffer shard at the index limit, and fixed shards over the 2^32 boundary
    words = x[: b - 4]
    d = B.swift_state_digest([words], 0)
    torch.cuda.synchronize()
    host = to_np(words)
    assert digests_np(d)[0] == oracle.digest(host)[0]
    del host
    with pytest.raises(B.SwiftError):
        B.swift_state_digest([x], 0)                       # 2^32 words or more need shard_elems
    shard = (1 << 31) + 12345
    d = B.swift_state_digest([x], shard)
    torch.cuda.synchronize()
    assert d.numel() == 3
    tail = to_np(x[2 * shard:])
    assert digests_np(d)[2] == oracle.digest(tail)[0]


def test_ten_thousand_tiny_tensors(B, synth):
    """Many small tensors in one launch: sizes 1..37 elements cycling, every element checked."""
    shapes = [((i % 37) + 1,) for i in range(10000)]
    hpd = dict(lr=1e-3, weight_decay=0.01, beta1=0.9, beta2=0.999, eps=1e-8, step=3)
    w = synth.Workload("tiny", shapes, "adam", hpd, seed=123, zero_frac=0.1, outlier_frac=0.01)
    s = synth.make_state(w, "cuda")
    # one flat copy per stream makes the host snapshots cheap; the tensors stay separate allocations
    tl = B.TensorList(s.theta, s.grad, s.m, s.v)
    hp = binding_hparams(B, "adam", hpd)
    flat = lambda ts: torch.cat(ts).cpu().numpy()
    pre = (flat(s.theta), flat(s.grad), flat(s.m), flat(s.v))
    B.swift_opt_step(tl, hp)
    torch.cuda.synchronize()
    mid = (flat(s.theta), flat(s.grad), flat(s.m), flat(s.v))
    _check_slices("adam", hpd, {"all": pre}, {"all": mid}, False, "tiny step")
    B.swift_opt_undo(tl, hp)
    torch.cuda.synchronize()
    end = (flat(s.theta), flat(s.grad), flat(s.m), flat(s.v))
    _check_slices("adam", hpd, {"all": mid}, {"all": end}, True, "tiny undo")
