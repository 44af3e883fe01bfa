"""The path inside a training loop (synthetic regression, a small MLP; torch only supplies the
gradients): an iteration that is interrupted after part of its update, rolled back with the undo
and applied again ends where the failure-free run ends, up to the rounding the paper's "Update-undo"
section calls negligible; and the library's AdamW follows torch.optim.AdamW on the same stream of
gradients."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2302_06173_amd import binding
    return binding


def _model(seed):
    torch.manual_seed(seed)
    return torch.nn.Sequential(torch.nn.Linear(64, 256), torch.nn.Tanh(), torch.nn.Linear(256, 256), torch.nn.Tanh(),
                               torch.nn.Linear(256, 8)).cuda()


def _data(seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    x = torch.randn(512, 64, device="cuda", generator=g)
    y = torch.tanh(x[:, :8] * 2.0) + 0.1 * torch.randn(512, 8, device="cuda", generator=g)
    return x, y


HPD = dict(lr=2e-3, weight_decay=0.01, beta1=0.9, beta2=0.999, eps=1e-8)


def _run(B, iters, fail_at=None, optimizer="library"):
    model = _model(3)
    x, y = _data(4)
    params = [p for p in model.parameters()]
    if optimizer == "torch":
        opt = torch.optim.AdamW(params, lr=HPD["lr"], betas=(HPD["beta1"], HPD["beta2"]), eps=HPD["eps"],
                                weight_decay=HPD["weight_decay"])
    else:
        flat = [p.data.view(-1) for p in params]
        m = [torch.zeros_like(t) for t in flat]
        v = [torch.zeros_like(t) for t in flat]
    losses = []
    for t in range(1, iters + 1):
        loss = torch.nn.functional.mse_loss(model(x), y)
        losses.append(float(loss.detach()))
        for p in params:
            p.grad = None
        loss.backward()
        if optimizer == "torch":
            opt.step()
            continue
        grads = [p.grad.view(-1) for p in params]
        tl = B.TensorList(flat, grads, m, v)
        hp = B.hparams("adamw", step=t, **HPD)
        if t == fail_at:
            # a peer dies after this replica has updated some of its tensors: roll exactly those back
            # (the tracker knows which), then the iteration's update is applied again by everybody
            tracker = B.Tracker(len(flat))
            tracker.begin(t)
            some = [0, 3, 4]
            tracker.step(B.TensorList([flat[i] for i in some], [grads[i] for i in some], [m[i] for i in some],
                                      [v[i] for i in some]), some, hp)
            assert tracker.marks() == [1 if i in some else 0 for i in range(len(flat))]
            tracker.undo(tl, hp)
            tracker.close()
        B.swift_opt_step(tl, hp)
    torch.cuda.synchronize()
    return losses, [p.detach().cpu().numpy().copy() for p in params]


def test_interrupted_iteration_rolled_back_and_redone(B):
    iters = 120
    clean_loss, clean = _run(B, iters)
    fail_loss, failed = _run(B, iters, fail_at=40)
    assert clean_loss[-1] < 0.5 * clean_loss[0], "the loop must actually train"
    assert np.allclose(clean_loss[:40], fail_loss[:40], rtol=1e-6, atol=0)     # the same run until the failure
    scale = max(float(np.abs(a).max()) for a in clean)
    worst = max(float(np.abs(a - b).max()) for a, b in zip(clean, failed))
    assert worst <= 1e-4 * scale, f"parameters drifted by {worst} (scale {scale}) after undo + redo"
    assert abs(clean_loss[-1] - fail_loss[-1]) <= 1e-4 * clean_loss[-1]


def test_library_adamw_follows_torch_adamw(B):
    iters = 60
    lib_loss, lib = _run(B, iters)
    ref_loss, ref = _run(B, iters, optimizer="torch")
    scale = max(float(np.abs(a).max()) for a in ref)
    worst = max(float(np.abs(a - b).max()) for a, b in zip(lib, ref))
    assert worst <= 2e-3 * scale, f"library and torch.optim.AdamW parameters differ by {worst} (scale {scale})"
    assert abs(lib_loss[-1] - ref_loss[-1]) <= 2e-3 * ref_loss[-1]
