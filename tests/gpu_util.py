"""Helpers shared by the GPU parity tests: marshalling between torch tensors, the HIP binding and
the CPU oracle, and the comparison rules."""
import numpy as np
import torch

import oracle

REL_TOL, ABS_FLOOR = 1e-5, 1e-8     # |gpu - oracle| <= max(REL_TOL * |oracle|, ABS_FLOOR) per element


def to_np(t: torch.Tensor) -> np.ndarray:
    """Bits of a tensor on the host: float32 as float32, bfloat16 as uint16 bit patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def oracle_hyper(kind: str, hp: dict) -> oracle.Hyper:
    return oracle.Hyper(kind=kind, eta=hp["lr"], lam=hp.get("weight_decay", 0.0), mu=hp.get("momentum", 0.0),
                        tau=hp.get("dampening", 0.0), beta1=hp.get("beta1", 0.9), beta2=hp.get("beta2", 0.999),
                        eps=hp.get("eps", 1e-8), t=hp.get("step", 1), clamp_v=bool(hp.get("clamp_v", False)))


def binding_hparams(B, kind: str, hp: dict, grad_bf16: bool = False):
    return B.hparams(kind, step=hp.get("step", 1), lr=hp["lr"], weight_decay=hp.get("weight_decay", 0.0),
                     momentum=hp.get("momentum", 0.0), dampening=hp.get("dampening", 0.0),
                     beta1=hp.get("beta1", 0.9), beta2=hp.get("beta2", 0.999), eps=hp.get("eps", 1e-8),
                     grad_bf16=grad_bf16, clamp_v=bool(hp.get("clamp_v", False)))


def assert_parity(gpu32: np.ndarray, ref64: np.ndarray, what: str, scale: float = None):
    """Two checks per element.
    (1) The stated bar: |gpu - oracle| <= max(1e-5 |oracle|, 1e-8).
    (2) Stricter, what binary64 arithmetic with one final rounding should deliver: the GPU value is
        within one binary32 ulp of the oracle's value, plus 1e-14 * scale for the few-ulp64
        differences in operation order where large terms cancel (scale = largest magnitude that
        entered the element's arithmetic; defaults to the largest |oracle| value)."""
    gpu32 = np.asarray(gpu32).reshape(-1)
    ref64 = np.asarray(ref64, np.float64).reshape(-1)
    assert gpu32.shape == ref64.shape, what
    g64 = gpu32.astype(np.float64)
    with np.errstate(invalid="ignore", over="ignore"):
        ref32 = ref64.astype(np.float32)
        special = (np.isnan(gpu32) & np.isnan(ref64)) | (np.isinf(ref32) & (gpu32 == ref32))
        err = np.abs(g64 - ref64)
        ok = (err <= np.maximum(REL_TOL * np.abs(ref64), ABS_FLOOR)) | special
    if not ok.all():
        i = int(np.nonzero(~ok)[0][0])
        raise AssertionError(f"{what}: {np.count_nonzero(~ok)} of {ok.size} elements out of tolerance; "
                             f"first at {i}: gpu={gpu32[i]!r} oracle={ref64[i]!r}")
    fin = np.isfinite(ref32) & np.isfinite(gpu32)
    if fin.any():
        if scale is None:
            scale = float(np.abs(ref64[fin]).max())
        ulp = np.spacing(np.abs(ref32[fin])).astype(np.float64)
        bad = err[fin] > ulp + 1e-14 * scale
        if bad.any():
            i = int(np.nonzero(bad)[0][0])
            raise AssertionError(f"{what}: {np.count_nonzero(bad)} elements more than one binary32 ulp from the "
                                 f"oracle; first: gpu={gpu32[fin][i]!r} oracle={ref64[fin][i]!r}")
    return float(np.nanmax(np.where(special, 0.0, err / np.maximum(np.abs(ref64), 1e-300)))) if err.size else 0.0


def digests_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().numpy().view(np.uint64)
