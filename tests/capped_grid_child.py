"""Run by test_gpu_capped_grid.py in a process of its own (the library reads SWIFT_MAX_GRID once per process):
every kind of call on a small seeded state, results saved as one .npz file."""
import os
import sys

import numpy as np
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def run(out_path: str) -> None:
    from paper_2302_06173_amd import binding as B
    gen = torch.Generator(device="cuda")
    gen.manual_seed(77)
    sizes = [70001, 0, 5, 4096, 300000, 16384 + 3, 1 << 18]
    new = lambda n, std: torch.empty(n, device="cuda").normal_(0, std, generator=gen)
    res = {}

    def state():
        th = [new(n, 0.02) for n in sizes]
        g = [new(n, 1e-3) for n in sizes]
        m = [new(n, 1e-4) for n in sizes]
        v = [new(n, 1e-6).abs_() for n in sizes]
        return th, g, m, v

    def keep(tag, th, m, v):
        for k, (a, b, c) in enumerate(zip(th, m, v)):
            res[f"{tag}_x{k}"] = a.cpu().numpy()
            res[f"{tag}_m{k}"] = b.cpu().numpy()
            res[f"{tag}_v{k}"] = c.cpu().numpy()

    for kind in ("sgd", "sgdm", "adam", "adamw"):
        th, g, m, v = state()
        hp = B.hparams(kind, step=7, lr=1e-3, weight_decay=0.01, momentum=0.9, beta1=0.9, beta2=0.999)
        tl = B.TensorList(th, g, None if kind == "sgd" else m, v if kind in ("adam", "adamw") else None)
        B.swift_opt_step(tl, hp)
        keep(kind + "_step", th, m, v)
        B.swift_opt_undo(tl, hp)
        keep(kind + "_undo", th, m, v)
    th, g, m, v = state()
    hp = B.hparams("adamw", step=7, lr=1e-3, weight_decay=0.01)
    tl = B.TensorList(th, g, m, v)
    res["fused_step_digests"] = B.swift_opt_step_digest(tl, hp).cpu().numpy()
    keep("fused_step", th, m, v)
    res["fused_undo_digests"] = B.swift_opt_undo_digest(tl, hp).cpu().numpy()
    keep("fused_undo", th, m, v)
    for shard in (0, 4096, 100000):
        res[f"digest_{shard}"] = B.swift_state_digest(th + m + v, shard).cpu().numpy()
    hpl = B.hparams("lamb", step=7, lr=2e-3, weight_decay=0.01, eps=1e-6)
    norms = B.swift_lamb_step(tl, hpl)
    res["lamb_norms"] = norms.cpu().numpy()
    keep("lamb_step", th, m, v)
    B.swift_lamb_undo(tl, hpl, norms)
    keep("lamb_undo", th, m, v)
    dmask = torch.tensor([1, 0, 1, 0, 1, 1, 0], dtype=torch.uint8, device="cuda")
    B.swift_opt_step_dmask(tl, hp, dmask)
    keep("dmask_step", th, m, v)
    B.swift_opt_undo_dmask(tl, hp, dmask)
    keep("dmask_undo", th, m, v)
    dst = torch.empty_like(th[6])
    B.swift_stream_copy(dst, th[6])
    res["copy"] = dst.cpu().numpy()
    torch.cuda.synchronize()
    np.savez(out_path, **res)


if __name__ == "__main__":
    run(sys.argv[1])
