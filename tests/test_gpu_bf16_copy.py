"""The optional bfloat16 copy of the parameters that step and undo write next to the fp32 master weights:
bit-exact against the oracle's rounding of the GPU's own fp32 result (the rounding decision is taken from the
same binary32 value on both sides), untouched for unmarked tensors, and without effect on theta, m, v."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import binding_hparams, to_np

pytestmark = pytest.mark.gpu

HP = {
    "sgdm": dict(lr=0.1, momentum=0.9, dampening=0.1, weight_decay=1e-4, step=1),
    "adam": dict(lr=1e-3, weight_decay=0.01, beta1=0.9, beta2=0.999, eps=1e-8, step=1000),
    "adamw": dict(lr=6e-4, weight_decay=0.1, beta1=0.9, beta2=0.95, eps=1e-8, step=7),
}
SHAPES = [(5000,), (1,), (0,), (4096,), (33333,), (2051,), (70001,), (7,)]


@pytest.fixture(scope="module")
def B():
    from paper_2302_06173_amd import binding
    return binding


@pytest.fixture(scope="module")
def synth():
    from paper_2302_06173_amd import synth
    return synth


@pytest.mark.parametrize("bf16g", [False, True], ids=["g_f32", "g_bf16"])
@pytest.mark.parametrize("kind", ["sgdm", "adam", "adamw"])
def test_bf16_copy_follows_theta(B, synth, kind, bf16g):
    w = synth.Workload("t", list(SHAPES), kind, HP[kind], seed=91, grad_bf16=bf16g, zero_frac=0.1, outlier_frac=0.01)
    a = synth.make_state(w, "cuda")
    b = a.clone()
    a.theta[3][:5] = torch.tensor([float("nan"), float("inf"), -0.0, 1e-40, 3.4e38], device="cuda")
    b.theta[3][:5] = a.theta[3][:5]
    n = len(SHAPES)
    hp = binding_hparams(B, kind, HP[kind], bf16g)
    sentinel = 0x1234
    xb = [torch.full((s[0],), 0, dtype=torch.int16, device="cuda").fill_(sentinel).view(torch.bfloat16) for s in SHAPES]
    tla = B.TensorList(a.theta, a.grad, a.m, a.v, param_bf16=xb)
    tlb = B.TensorList(b.theta, b.grad, b.m, b.v)
    mask = [1, 1, 1, 0, 1, 0, 1, 1]
    for call, m in ((B.swift_opt_step, mask), (B.swift_opt_undo, mask), (B.swift_opt_step, None), (B.swift_opt_undo, None)):
        call(tla, hp, host_mask=m)
        call(tlb, hp, host_mask=m)
        torch.cuda.synchronize()
        for i in range(n):
            for x, y in ((a.theta[i], b.theta[i]), (a.m[i], b.m[i])) + (() if a.v is None else ((a.v[i], b.v[i]),)):
                assert torch.equal(x.view(torch.int32), y.view(torch.int32)), "the copy changed the arithmetic"
            got = to_np(xb[i])
            if m is None or m[i]:
                assert np.array_equal(got, oracle.bf16_round(to_np(a.theta[i]))), (kind, i)
        if m is mask and call is B.swift_opt_step:
            for i in (3, 5):
                assert (to_np(xb[i]) == sentinel).all(), "copy of an unmarked tensor was written"
    # device-mask form and unaligned copies (2-byte aligned only) give the same bits
    dm = torch.tensor(mask, dtype=torch.uint8, device="cuda")
    xb2 = []
    for s in SHAPES:
        buf = torch.zeros(s[0] + 8, dtype=torch.bfloat16, device="cuda")
        xb2.append(buf[1:1 + s[0]])
    tlc = B.TensorList(b.theta, b.grad, b.m, b.v, param_bf16=xb2)
    B.swift_opt_step_dmask(tla, hp, dm)
    B.swift_opt_step_dmask(tlc, hp, dm)
    torch.cuda.synchronize()
    for i in range(n):
        if mask[i]:
            assert np.array_equal(to_np(xb[i]), to_np(xb2[i]))
            assert np.array_equal(to_np(xb2[i]), oracle.bf16_round(to_np(b.theta[i])))


@pytest.mark.parametrize("bf16g", [False, True], ids=["g_f32", "g_bf16"])
def test_bf16_copy_in_the_lamb_and_fused_digest_calls(B, synth, bf16g):
    """Same contract: the copy is the rounding of the theta the call wrote, marked tensors only, and theta, m, v,
    norms and digests are what the call without the copy gives."""
    hpd = dict(lr=2e-3, weight_decay=0.01, beta1=0.9, beta2=0.999, eps=1e-6, step=12)
    w = synth.Workload("t", list(SHAPES), "lamb", hpd, seed=93, grad_bf16=bf16g, zero_frac=0.1, outlier_frac=0.01)
    a = synth.make_state(w, "cuda", with_v=True)
    b = a.clone()
    n = len(SHAPES)
    sentinel = 0x1234
    xb = [torch.full((s[0],), 0, dtype=torch.int16, device="cuda").fill_(sentinel).view(torch.bfloat16) for s in SHAPES]
    tla = B.TensorList(a.theta, a.grad, a.m, a.v, param_bf16=xb)
    tlb = B.TensorList(b.theta, b.grad, b.m, b.v)
    mask = [1, 1, 1, 0, 1, 0, 1, 1]

    def same_state_and_copy(m, what):
        torch.cuda.synchronize()
        for i in range(n):
            for x, y in ((a.theta[i], b.theta[i]), (a.m[i], b.m[i]), (a.v[i], b.v[i])):
                assert torch.equal(x.view(torch.int32), y.view(torch.int32)), f"{what}: the copy changed the arithmetic"
            if m is None or m[i]:
                assert np.array_equal(to_np(xb[i]), oracle.bf16_round(to_np(a.theta[i]))), (what, i)
            else:
                assert (to_np(xb[i]) == sentinel).all(), f"{what}: copy of an unmarked tensor was written"

    hl = binding_hparams(B, "lamb", hpd, bf16g)
    na = B.swift_lamb_step(tla, hl, host_mask=mask)
    nb = B.swift_lamb_step(tlb, hl, host_mask=mask)
    same_state_and_copy(mask, "lamb step")
    assert torch.equal(na.view(torch.int64), nb.view(torch.int64))
    B.swift_lamb_undo(tla, hl, na, host_mask=mask)
    B.swift_lamb_undo(tlb, hl, nb, host_mask=mask)
    same_state_and_copy(mask, "lamb undo")
    hw = binding_hparams(B, "adamw", HP["adamw"], bf16g)
    for fused in (B.swift_opt_step_digest, B.swift_opt_undo_digest):
        da = fused(tla, hw, host_mask=mask)
        db = fused(tlb, hw, host_mask=mask)
        same_state_and_copy(mask, fused.__name__)
        assert torch.equal(da, db)
    da = B.swift_opt_step_digest(tla, hw)
    db = B.swift_opt_step_digest(tlb, hw)
    same_state_and_copy(None, "fused step, all tensors")
    assert torch.equal(da, db)


def test_bf16_copy_argument_errors(B, synth):
    w = synth.Workload("t", [(100,)], "adamw", HP["adamw"], seed=1)
    s = synth.make_state(w, "cuda")
    xb = [torch.zeros(100, dtype=torch.bfloat16, device="cuda")]
    tl = B.TensorList(s.theta, s.grad, s.m, s.v, param_bf16=xb)
    with pytest.raises(ValueError):
        B.TensorList(s.theta, s.grad, s.m, s.v, param_bf16=[torch.zeros(99, dtype=torch.bfloat16, device="cuda")])
    tl2 = B.TensorList(s.theta, s.grad, s.m, s.v, param_bf16=[s.theta[0].view(torch.bfloat16)[:100]])   # aliases theta
    with pytest.raises(B.SwiftError) as e:
        B.swift_opt_step(tl2, binding_hparams(B, "adamw", HP["adamw"]))
    assert "overlap" in e.value.message
