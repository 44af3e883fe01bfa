"""CPU oracle (fp64) for optimizer step / update-undo and the state digest.

TEST INFRASTRUCTURE ONLY: the tests, ``__graft_entry__.smoke()`` and the CPU-baseline
leg of ``bench.py`` may import this package; the GPU library and its Python binding
never do, and this package imports nothing from them.

The arithmetic lives in ``swift_oracle.c`` (plain scalar binary64 loops, one function
per algorithm of the paper: Alg. 1, Alg. 2 and the six algorithms of App. A (SGD, Adam, AdamW and their undos); plus LAMB
with the saved-norm undo that the paper's "Update-undo" section sketches in one sentence).
This module only compiles that file with gcc, widens inputs to fp64 and walks tensor lists.

Pins (see ``tests/test_oracle_pins.py``): hand-worked exact-rational examples stored
under ``tests/golden/``, torch.optim's SGD / Adam / AdamW in fp64 (an independent
library routine the step reduces to), closed forms, and brute-force exact-rational
round trips.  The digest has no definition in the paper; it is pinned to stored test
vectors, to an explicit inverse of its mixer and to order / shard invariants, and is
"parity unpinned" with respect to the paper itself.  LAMB: the paper prints no algorithm, so
the step follows the LAMB publication and is "parity unpinned" with respect to the paper; it
is pinned to the AdamW oracle (LAMB = AdamW with the trust ratio folded into the learning
rate), to hand-worked examples, to its zero-norm fallback and to scaling laws.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "swift_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None

SGD, SGDM, ADAM, ADAMW, LAMB = "sgd", "sgdm", "adam", "adamw", "lamb"


def build(force: bool = False) -> str:
    """Compile swift_oracle.c -> liboracle.so (gcc, no contraction, no fast-math)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off",
             "-fno-fast-math", "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        d, p, i64 = ctypes.c_double, ctypes.c_void_p, ctypes.c_int64
        lib.oracle_sgdm_step.argtypes = [i64, p, p, p, d, d, d, d, p, p]
        lib.oracle_sgdm_undo.argtypes = [i64, p, p, p, d, d, d, d, p, p]
        lib.oracle_sgd_step.argtypes = lib.oracle_sgd_undo.argtypes = [i64, p, p, d, d, p]
        lib.oracle_sgd_step.restype = lib.oracle_sgd_undo.restype = None
        for name in ("adam_step", "adam_undo", "adamw_step", "adamw_undo"):
            getattr(lib, "oracle_" + name).argtypes = [i64, p, p, p, p, d, d, d, d, d, i64, p, p, p]
        for name in ("sgdm_step", "sgdm_undo", "adam_step", "adam_undo", "adamw_step", "adamw_undo"):
            getattr(lib, "oracle_" + name).restype = None
        lib.oracle_lamb_step.argtypes = [i64, p, p, p, p, d, d, d, d, d, i64, p, p, p, p]
        lib.oracle_lamb_undo.argtypes = [i64, p, p, p, p, d, d, d, d, d, i64, p, p, p, p]
        lib.oracle_lamb_step.restype = lib.oracle_lamb_undo.restype = None
        lib.oracle_clamp_v.argtypes = [i64, p]
        lib.oracle_clamp_v.restype = None
        lib.oracle_bf16_round.argtypes = [i64, p, p]
        lib.oracle_bf16_round.restype = None
        lib.oracle_digest.argtypes = [p, i64]
        lib.oracle_digest.restype = ctypes.c_uint64
        _lib = lib
    return _lib


@dataclass
class Hyper:
    """Hyper-parameters in the paper's notation (the oracle's own type)."""
    kind: str                 # "sgd" | "sgdm" | "adam" | "adamw"
    eta: float                # learning rate eta_t
    lam: float = 0.0          # weight decay lambda
    mu: float = 0.0           # momentum (SGDM)
    tau: float = 0.0          # dampening (SGDM)
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    t: int = 1                # index of the update applied / undone
    clamp_v: bool = False     # undo only, not in the paper: a recovered v below zero becomes +0


def widen(a) -> np.ndarray:
    """Exact widening of the bit patterns the GPU sees to a contiguous fp64 vector.

    float32 / float64 arrays widen by value; uint16 arrays are bf16 bit patterns
    (value = the fp32 whose upper half they are).
    """
    a = np.asarray(a)
    if a.dtype == np.uint16:
        a = (a.astype(np.uint32) << np.uint32(16)).view(np.float32)
    if a.dtype not in (np.float32, np.float64):
        raise TypeError(f"oracle.widen: unsupported dtype {a.dtype}")
    return np.ascontiguousarray(a.reshape(-1), dtype=np.float64)


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _run(which: str, hp: Hyper, x, g, m, v):
    lib = _load()
    if hp.kind == SGD:                        # App. A "SGD" / "Undo SGD": no optimizer state
        x, g = widen(x), widen(g)
        if g.size != x.size:
            raise ValueError("oracle: x, g differ in size")
        xo = np.empty(x.size)
        getattr(lib, f"oracle_sgd_{which}")(x.size, _ptr(x), _ptr(g), hp.eta, hp.lam, _ptr(xo))
        return xo, None, None
    x, g, m = widen(x), widen(g), widen(m)
    n = x.size
    if g.size != n or m.size != n:
        raise ValueError("oracle: x, g, m differ in size")
    xo, mo = np.empty(n), np.empty(n)
    if hp.kind == SGDM:
        fn = getattr(lib, f"oracle_sgdm_{which}")
        fn(n, _ptr(x), _ptr(g), _ptr(m), hp.eta, hp.lam, hp.mu, hp.tau, _ptr(xo), _ptr(mo))
        return xo, mo, None
    if hp.kind not in (ADAM, ADAMW):
        raise ValueError(f"oracle: unknown optimizer {hp.kind!r}")
    v = widen(v)
    if v.size != n:
        raise ValueError("oracle: v differs in size")
    vo = np.empty(n)
    fn = getattr(lib, f"oracle_{hp.kind}_{which}")
    fn(n, _ptr(x), _ptr(g), _ptr(m), _ptr(v), hp.eta, hp.lam, hp.beta1, hp.beta2, hp.eps,
       int(hp.t), _ptr(xo), _ptr(mo), _ptr(vo))
    return xo, mo, vo


def opt_step(hp: Hyper, x, g, m=None, v=None):
    """(x_t, g_t, m_{t-1}, v_{t-1}) -> (x_{t+1}, m_t, v_t), all fp64 (v is None for SGDM, m and v for SGD)."""
    return _run("step", hp, x, g, m, v)


def opt_undo(hp: Hyper, x_new, g, m_new=None, v_new=None):
    """(x_{t+1}, g_t, m_t, v_t) -> (x_t, m_{t-1}, v_{t-1}), all fp64.

    Raises ZeroDivisionError where the printed inverse divides by zero and no reading
    rescues it (beta1 = 0, beta2 = 0, eta*lambda = 1 for AdamW and plain SGD); mu = 0 is allowed.
    """
    if hp.kind in (ADAM, ADAMW) and (hp.beta1 == 0.0 or hp.beta2 == 0.0):
        raise ZeroDivisionError("undo: beta = 0 is not invertible")
    if hp.kind in (ADAMW, SGD) and 1.0 - hp.eta * hp.lam == 0.0:
        raise ZeroDivisionError("undo: eta*lambda = 1 is not invertible")
    x_old, m_old, v_old = _run("undo", hp, x_new, g, m_new, v_new)
    if hp.clamp_v and v_old is not None:
        _load().oracle_clamp_v(v_old.size, _ptr(v_old))
    return x_old, m_old, v_old


def lamb_step(hp: Hyper, x, g, m, v):
    """LAMB step of ONE tensor: returns (x_{t+1}, m_t, v_t, norms) with norms = [||x_t||, ||u||], the two
    scalars the undo needs (the paper's saved L2 norm)."""
    lib = _load()
    x, g, m, v = widen(x), widen(g), widen(m), widen(v)
    n = x.size
    if not (g.size == m.size == v.size == n):
        raise ValueError("oracle: x, g, m, v differ in size")
    xo, mo, vo, norms = np.empty(n), np.empty(n), np.empty(n), np.zeros(2)
    lib.oracle_lamb_step(n, _ptr(x), _ptr(g), _ptr(m), _ptr(v), hp.eta, hp.lam, hp.beta1, hp.beta2, hp.eps,
                         int(hp.t), _ptr(xo), _ptr(mo), _ptr(vo), _ptr(norms))
    return xo, mo, vo, norms


def lamb_undo(hp: Hyper, x_new, g, m_new, v_new, norms):
    """Undo of lamb_step for ONE tensor, given the norms that step returned."""
    if hp.beta1 == 0.0 or hp.beta2 == 0.0:
        raise ZeroDivisionError("undo: beta = 0 is not invertible")
    lib = _load()
    x, g, m, v = widen(x_new), widen(g), widen(m_new), widen(v_new)
    norms = np.ascontiguousarray(norms, dtype=np.float64)
    n = x.size
    if not (g.size == m.size == v.size == n) or norms.size != 2:
        raise ValueError("oracle: sizes differ")
    xo, mo, vo = np.empty(n), np.empty(n), np.empty(n)
    lib.oracle_lamb_undo(n, _ptr(x), _ptr(g), _ptr(m), _ptr(v), hp.eta, hp.lam, hp.beta1, hp.beta2, hp.eps,
                         int(hp.t), _ptr(norms), _ptr(xo), _ptr(mo), _ptr(vo))
    if hp.clamp_v:
        lib.oracle_clamp_v(n, _ptr(vo))
    return xo, mo, vo


def _walk(fn, hp, xs, gs, ms, vs, mask):
    out = []
    for i in range(len(xs)):
        m = None if ms is None else ms[i]
        v = None if vs is None else vs[i]
        if mask is not None and not mask[i]:
            out.append((widen(xs[i]), None if m is None else widen(m), None if v is None else widen(v)))
        else:
            out.append(fn(hp, xs[i], gs[i], m, v))
    return out


def step_list(hp: Hyper, xs: Sequence, gs: Sequence, ms: Optional[Sequence] = None, vs: Optional[Sequence] = None,
              mask: Optional[Sequence] = None):
    """Step every tensor whose mask entry is non-zero (all if mask is None); the rest pass through."""
    return _walk(opt_step, hp, xs, gs, ms, vs, mask)


def undo_list(hp: Hyper, xs: Sequence, gs: Sequence, ms: Optional[Sequence] = None, vs: Optional[Sequence] = None,
              mask: Optional[Sequence] = None):
    """Undo every tensor marked as updated (the paper's per-parameter flag); the rest pass through."""
    return _walk(opt_undo, hp, xs, gs, ms, vs, mask)


def bf16_round(x32) -> np.ndarray:
    """bfloat16 bit patterns (uint16) of a float32 array: nearest, ties to even, NaN -> 0x7FC0."""
    x = np.ascontiguousarray(np.asarray(x32).reshape(-1))
    if x.dtype != np.float32:
        raise TypeError("oracle.bf16_round: need float32")
    out = np.empty(x.size, dtype=np.uint16)
    _load().oracle_bf16_round(x.size, _ptr(x), _ptr(out))
    return out


def words(a) -> np.ndarray:
    """Raw 32-bit words of a 4-byte-element array (fp32, int32 or uint32), flattened."""
    a = np.ascontiguousarray(np.asarray(a).reshape(-1))
    if a.dtype.itemsize != 4:
        raise TypeError("oracle.words: need 4-byte elements")
    return a.view(np.uint32)


def digest(buf, shard_elems: int = 0) -> np.ndarray:
    """Digests of one buffer: consecutive shards of shard_elems words (last one short);
    shard_elems = 0 means one shard for the whole buffer.  An empty buffer has no shards
    when shard_elems > 0 and one shard (digest 0) when shard_elems = 0."""
    lib = _load()
    w = words(buf)
    n = w.size
    if shard_elems == 0:
        if n >= 1 << 32:
            raise ValueError("oracle.digest: shard of 2^32 words or more")
        return np.array([lib.oracle_digest(_ptr(w), n)], dtype=np.uint64)
    if not 0 < shard_elems < 1 << 32:
        raise ValueError("oracle.digest: shard_elems out of range")
    out = []
    for lo in range(0, n, shard_elems):
        part = w[lo:lo + shard_elems]
        out.append(lib.oracle_digest(_ptr(part), part.size))
    return np.array(out, dtype=np.uint64)


def digest_list(bufs: Sequence, shard_elems: int = 0) -> np.ndarray:
    """Buffer-major concatenation of digest(buf, shard_elems)."""
    parts = [digest(b, shard_elems) for b in bufs]
    return np.concatenate(parts) if parts else np.zeros(0, dtype=np.uint64)
