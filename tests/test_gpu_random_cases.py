"""Seeded random cases through the C ABI against the fp64 oracle: random tensor counts and sizes
(empty, one element, ragged, several chunks), random placement inside a shared buffer (any 4-byte
alignment, 2-byte for bfloat16 gradients), random admissible hyper-parameters, optimizer, gradient
type, mask form, clamp flag and bfloat16 copy.  Every element of every tensor is compared; the guard
words around every tensor must keep their bits."""
import random

import numpy as np
import pytest
import torch

import oracle
from gpu_util import assert_parity, binding_hparams, oracle_hyper, to_np

pytestmark = pytest.mark.gpu

GUARD = 8          # elements kept free on both sides of every tensor


@pytest.fixture(scope="module")
def B():
    from paper_2302_06173_amd import binding
    return binding


def _sizes(rng):
    n_t = rng.randint(1, 9)
    pool = [0, 1, 2, 3, 5, 63, 64, 255, 256, 257, 1023, 1024, 4095, 4096, 4099, 16384, 16385, 40000, 70001, 131072 + 7]
    return [rng.choice(pool) if rng.random() < 0.7 else rng.randint(0, 90000) for _ in range(n_t)]


def _place(rng, sizes, dtype, gen, std, absval=False):
    """Tensors as views into one buffer at random element offsets, guard words in between."""
    offs, cur = [], rng.randint(0, 7)
    for n in sizes:
        cur += GUARD
        offs.append(cur)
        cur += n + GUARD + rng.randint(0, 7)
    buf = torch.empty(cur + 16, dtype=torch.float32, device="cuda").normal_(0.0, std, generator=gen)
    if absval:
        buf.abs_()
    if dtype == torch.bfloat16:
        buf = buf.to(torch.bfloat16)
    return buf, [buf[o:o + n] for o, n in zip(offs, sizes)], offs


def _hyper(rng, kind):
    if kind == "sgd":
        return dict(lr=10 ** rng.uniform(-4, -0.5), weight_decay=rng.choice([0.0, 1e-4, 0.1]), step=rng.randint(1, 1000))
    if kind == "sgdm":
        return dict(lr=10 ** rng.uniform(-4, -0.5), momentum=rng.choice([0.0, 0.5, 0.9, 0.99]), dampening=rng.choice([0.0, 0.1, 0.5]),
                    weight_decay=rng.choice([0.0, 1e-4, 0.1]), step=rng.randint(1, 1000))
    return dict(lr=10 ** rng.uniform(-5, -2), weight_decay=rng.choice([0.0, 0.01, 0.1]), beta1=rng.choice([0.5, 0.9, 0.95]),
                beta2=rng.choice([0.9, 0.95, 0.999]), eps=rng.choice([1e-8, 1e-6, 1e-3]), step=rng.randint(1, 200000),
                clamp_v=rng.random() < 0.3)


@pytest.mark.parametrize("seed", list(range(32)))
def test_random_case(B, seed):
    rng = random.Random(1000 + seed)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(5000 + seed)
    kind = "sgd" if seed >= 24 else rng.choice(["sgdm", "adam", "adamw"])      # seeds 24-31: App. A's plain SGD
    bf16g = rng.random() < 0.4
    sizes = _sizes(rng)
    n_t = len(sizes)
    hpd = _hyper(rng, kind)
    bx, x, ox = _place(rng, sizes, torch.float32, gen, 0.02)
    bg, g, og = _place(rng, sizes, torch.bfloat16 if bf16g else torch.float32, gen, 1e-3)
    bm, m, om = (None, None, None) if kind == "sgd" else _place(rng, sizes, torch.float32, gen, 1e-3)
    bv, v, ov = (None, None, None) if kind in ("sgd", "sgdm") else _place(rng, sizes, torch.float32, gen, 1e-6, absval=True)
    with_copy = rng.random() < 0.3
    bxb, xb, oxb = _place(rng, sizes, torch.bfloat16, gen, 1.0) if with_copy else (None, None, None)
    tl = B.TensorList(x, g, m, v, param_bf16=xb)
    hp = binding_hparams(B, kind, hpd, bf16g)
    h = oracle_hyper(kind, hpd)
    bufs = [b for b in (bx, bg, bm, bv, bxb) if b is not None]
    for call_no in range(3):
        undo = call_no == 1 or (call_no == 2 and rng.random() < 0.5)
        mask = None if rng.random() < 0.4 else [rng.randint(0, 1) for _ in range(n_t)]
        on_device = mask is not None and rng.random() < 0.5
        before = [to_np(b) for b in bufs]
        pre = [[to_np(t) for t in ts] if ts is not None else None for ts in (x, g, m, v)]
        if on_device:
            dm = torch.tensor(mask, dtype=torch.uint8, device="cuda")
            (B.swift_opt_undo_dmask if undo else B.swift_opt_step_dmask)(tl, hp, dm)
        else:
            (B.swift_opt_undo if undo else B.swift_opt_step)(tl, hp, host_mask=mask)
        torch.cuda.synchronize()
        post = [[to_np(t) for t in ts] if ts is not None else None for ts in (x, g, m, v)]
        what = f"seed {seed} call {call_no} {kind} {'undo' if undo else 'step'} bf16g={bf16g} mask={mask} dev={on_device}"
        fn = oracle.opt_undo if undo else oracle.opt_step
        for i in range(n_t):
            if mask is not None and not mask[i]:
                continue
            vin = None if v is None else pre[3][i]
            min_ = None if m is None else pre[2][i]
            rx, rm, rv = fn(h, pre[0][i], pre[1][i], min_, vin)
            sc = max([float(np.abs(oracle.widen(a)).max()) for a in (pre[0][i], pre[1][i]) + tuple(a for a in (min_, vin) if a is not None) if a.size] + [0.0])
            assert_parity(post[0][i], rx, f"{what} theta[{i}]", sc)
            if m is not None:
                assert_parity(post[2][i], rm, f"{what} m[{i}]", sc)
            if v is not None:
                assert_parity(post[3][i], rv, f"{what} v[{i}]", sc * max(sc, 1.0))
            if with_copy:
                assert np.array_equal(to_np(xb[i]), oracle.bf16_round(post[0][i])), f"{what} bf16 copy[{i}]"
        # everything outside the marked tensors keeps its bits: guards, unmarked tensors, the whole gradient buffer
        after = [to_np(b) for b in bufs]
        layout = [(ox, True), (og, False)] + ([(om, True)] if m is not None else []) + ([(ov, True)] if v is not None else []) + ([(oxb, True)] if with_copy else [])
        assert len(layout) == len(before)
        for b0, b1, (offs, written) in zip(before, after, layout):
            keep = np.ones(b0.size, bool)
            if written:
                for i, (o, n) in enumerate(zip(offs, sizes)):
                    if mask is None or mask[i]:
                        keep[o:o + n] = False
            w0 = b0.view(np.uint16) if b0.dtype == np.uint16 else b0.view(np.uint32)
            w1 = b1.view(np.uint16) if b1.dtype == np.uint16 else b1.view(np.uint32)
            assert np.array_equal(w0[keep], w1[keep]), f"{what}: bits outside the marked tensors changed"
