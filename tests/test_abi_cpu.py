"""Host-only checks of the C ABI: the library loads, exports what the header declares, and rejects
bad arguments before touching any GPU.  No kernel is launched here."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2302_06173_amd import build
    build.build(force=False)
    from paper_2302_06173_amd import binding
    return binding


def test_every_declared_symbol_is_exported(B):
    text = open(os.path.join(ROOT, "include", "swift_undo.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(swift_[a-z_0-9]+)\s*\(", text))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(B._lib, name), name


def test_struct_layouts_match_the_header(B):
    # int32, int32, int64, 7 doubles / int64 + 5 pointers: no padding surprises
    assert ctypes.sizeof(B.SwiftHparams) == 4 + 4 + 8 + 7 * 8 + 4 + 4
    assert ctypes.sizeof(B.SwiftTensorList) == 8 + 6 * 8
    assert B.SwiftHparams.lr.offset == 16 and B.SwiftHparams.eps.offset == 64 and B.SwiftHparams.flags.offset == 72


def test_digest_count_is_host_arithmetic(B):
    assert B.swift_digest_count([], 0) == 0
    assert B.swift_digest_count([10, 0, 3], 0) == 3
    assert B.swift_digest_count([10, 0, 3], 4) == 3 + 0 + 1
    assert B.swift_digest_count([1 << 20], 1 << 16) == 16
    assert B.swift_digest_count([(1 << 32) + 5], 1 << 31) == 3
    with pytest.raises(B.SwiftError) as e:
        B.swift_digest_count([1 << 32], 0)           # one shard of 2^32 words: index would not fit
    assert e.value.code == B.SWIFT_EINVAL and "shard_elems" in e.value.message
    with pytest.raises(B.SwiftError):
        B.swift_digest_count([-1], 0)
    with pytest.raises(B.SwiftError):
        B.swift_digest_count([4], 1 << 32)
    with pytest.raises(B.SwiftError):
        B.swift_digest_count([4], -1)


def _call(B, fn, hp, n=0):
    lst = B.SwiftTensorList(n, None, None, None, None, None, None)
    return getattr(B._lib, fn)(ctypes.byref(lst), ctypes.byref(hp), None, None)


@pytest.mark.parametrize("fn", ["swift_opt_step", "swift_opt_undo"])
def test_hyper_parameter_domain(B, fn):
    ok = B.hparams("adamw", step=5, lr=1e-3, weight_decay=0.01)
    assert _call(B, fn, ok) == B.SWIFT_OK                       # empty list: nothing to do
    bad = [
        B.hparams(7, step=1, lr=0.1),
        B.hparams("adam", step=0, lr=0.1),
        B.hparams("adam", step=1, lr=float("nan")),
        B.hparams("adam", step=1, lr=float("inf")),
        B.hparams("adam", step=1, lr=0.1, weight_decay=-1.0),
        B.hparams("adam", step=1, lr=0.1, beta1=1.0),
        B.hparams("adam", step=1, lr=0.1, beta2=-0.1),
        B.hparams("adamw", step=1, lr=0.1, eps=-1e-8),
        B.hparams("sgdm", step=1, lr=0.1, momentum=1.5),
        B.hparams("sgdm", step=1, lr=0.1, dampening=-0.5),
    ]
    for hp in bad:
        assert _call(B, fn, hp) == B.SWIFT_EINVAL
        assert B.swift_last_error() != ""
    hp = B.hparams("adam", step=1, lr=0.1)
    hp.grad_dtype = 9
    assert _call(B, fn, hp) == B.SWIFT_EINVAL
    assert _call(B, fn, B.hparams("adam", step=1, lr=0.1, clamp_v=True)) == B.SWIFT_OK
    hp = B.hparams("adam", step=1, lr=0.1)
    hp.flags = 2                                                # a bit nobody defined
    assert _call(B, fn, hp) == B.SWIFT_EINVAL and "flag" in B.swift_last_error()
    hp = B.hparams("adam", step=1, lr=0.1)
    hp.reserved = 1
    assert _call(B, fn, hp) == B.SWIFT_EINVAL


def test_not_invertible_is_an_undo_only_error(B):
    for hp in (B.hparams("adam", step=1, lr=0.1, beta1=0.0),
               B.hparams("adamw", step=1, lr=0.1, beta2=0.0),
               B.hparams("adamw", step=1, lr=0.5, weight_decay=2.0),
               B.hparams("sgd", step=1, lr=0.5, weight_decay=2.0)):       # App. A "Undo SGD" divides by 1 - eta lambda
        assert _call(B, "swift_opt_undo", hp) == B.SWIFT_ENOTINVERTIBLE
        assert "divides" in B.swift_last_error()
        assert _call(B, "swift_opt_step", hp) == B.SWIFT_OK
    # momentum 0 is the paper's plain SGD: undo is allowed
    assert _call(B, "swift_opt_undo", B.hparams("sgdm", step=1, lr=0.1, momentum=0.0)) == B.SWIFT_OK


def test_null_and_negative_arguments(B):
    hp = B.hparams("adam", step=1, lr=0.1)
    assert B._lib.swift_opt_step(None, ctypes.byref(hp), None, None) == B.SWIFT_EINVAL
    lst = B.SwiftTensorList(2, None, None, None, None, None, None)
    assert B._lib.swift_opt_step(ctypes.byref(lst), None, None, None) == B.SWIFT_EINVAL
    assert B._lib.swift_opt_step(ctypes.byref(lst), ctypes.byref(hp), None, None) == B.SWIFT_EINVAL
    assert "NULL" in B.swift_last_error()
    lst = B.SwiftTensorList(-1, None, None, None, None, None, None)
    assert B._lib.swift_opt_undo(ctypes.byref(lst), ctypes.byref(hp), None, None) == B.SWIFT_EINVAL
    # numel < 0, missing v for Adam, misaligned pointer: all caught on the host
    n = 1
    ptr = (ctypes.c_void_p * 1)(0x1000)
    odd = (ctypes.c_void_p * 1)(0x1002)
    P = ctypes.POINTER(ctypes.c_void_p)
    neg = (ctypes.c_int64 * 1)(-5)
    four = (ctypes.c_int64 * 1)(4)
    c = lambda a: ctypes.cast(a, P)
    i64 = lambda a: ctypes.cast(a, ctypes.POINTER(ctypes.c_int64))
    lst = B.SwiftTensorList(n, c(ptr), c(ptr), c(ptr), c(ptr), i64(neg), None)
    assert B._lib.swift_opt_step(ctypes.byref(lst), ctypes.byref(hp), None, None) == B.SWIFT_EINVAL
    huge = (ctypes.c_int64 * 1)(1 << 62)                   # 4 * numel would wrap around
    lst = B.SwiftTensorList(n, c(ptr), c(ptr), c(ptr), c(ptr), i64(huge), None)
    assert B._lib.swift_opt_step(ctypes.byref(lst), ctypes.byref(hp), None, None) == B.SWIFT_EINVAL
    assert "2^40" in B.swift_last_error()
    assert B.swift_digest_count([1 << 20], 1 << 16) == 16
    with pytest.raises(B.SwiftError):
        B.swift_digest_count([1 << 62], 1 << 20)
    assert B._lib.swift_stream_copy(ptr, ptr, 1 << 62, None) == B.SWIFT_EINVAL
    lst = B.SwiftTensorList(n, c(ptr), c(ptr), c(ptr), None, i64(four), None)
    assert B._lib.swift_opt_step(ctypes.byref(lst), ctypes.byref(hp), None, None) == B.SWIFT_EINVAL
    assert "v array" in B.swift_last_error()
    lst = B.SwiftTensorList(n, c(odd), c(ptr), c(ptr), c(ptr), i64(four), None)
    assert B._lib.swift_opt_step(ctypes.byref(lst), ctypes.byref(hp), None, None) == B.SWIFT_EINVAL
    assert "aligned" in B.swift_last_error()
    # bf16 gradients may sit on 2-byte boundaries, fp32 gradients may not
    lst = B.SwiftTensorList(n, c(ptr), c(odd), c(ptr), c(ptr), i64(four), None)
    assert B._lib.swift_opt_step(ctypes.byref(lst), ctypes.byref(hp), None, None) == B.SWIFT_EINVAL
    odd1 = (ctypes.c_void_p * 1)(0x1001)
    lst = B.SwiftTensorList(n, c(ptr), c(ptr), c(ptr), c(ptr), i64(four), c(odd1))
    assert B._lib.swift_opt_step(ctypes.byref(lst), ctypes.byref(hp), None, None) == B.SWIFT_EINVAL
    assert "param_bf16" in B.swift_last_error()
    assert B._lib.swift_mask_from_digests(-1, 3, None, None, None, None) == B.SWIFT_EINVAL
    assert B._lib.swift_mask_from_digests(4, 0, None, None, None, None) == B.SWIFT_EINVAL
    assert B._lib.swift_mask_from_digests(4, 3, None, None, None, None) == B.SWIFT_EINVAL
    assert B._lib.swift_mask_from_digests(0, 3, None, None, None, None) == B.SWIFT_OK
    assert B._lib.swift_stream_copy(None, None, 8, None) == B.SWIFT_EINVAL
    assert B._lib.swift_stream_copy(None, None, 16, None) == B.SWIFT_EINVAL
    assert B._lib.swift_stream_copy(None, None, 0, None) == B.SWIFT_OK
    assert B._lib.swift_state_digest(-1, None, None, 0, None, None) == B.SWIFT_EINVAL
    assert B._lib.swift_state_digest(0, None, None, 0, None, None) == B.SWIFT_OK
    assert B._lib.swift_shutdown() == B.SWIFT_OK


def test_synthetic_workloads_have_the_stated_sizes():
    from paper_2302_06173_amd import synth
    w = synth.workloads()
    got = {k: (len(v.shapes), v.n_params) for k, v in w.items()}
    assert got == {
        "sgdm_flat_1m": (1, 1_048_576),
        "resnet50_adam": (161, 25_557_032),
        "bert_large_adamw": (391, 335_141_888),
        "gpt2_xl_adamw_bf16g": (580, 1_557_611_200),
        "llama7b_adamw": (291, 6_738_415_616),
        "vit_128_32_sgdm": (1544, 1_616_542_696),
    }
    # seeded: same seed, same bits; the mask picks the stated fraction
    s1 = synth.make_state(w["sgdm_flat_1m"], "cpu", shapes=[(33,), (5,)])
    s2 = synth.make_state(w["sgdm_flat_1m"], "cpu", shapes=[(33,), (5,)])
    assert all((a == b).all() for a, b in zip(s1.theta + s1.grad + s1.m, s2.theta + s2.grad + s2.m))
    assert s1.v is None
    mask = synth.tensor_mask(w["llama7b_adamw"], 291)
    assert sum(mask) == 146 and mask == synth.tensor_mask(w["llama7b_adamw"], 291)


def test_padded_layout_keeps_values_and_skews_the_buffers():
    import torch
    from paper_2302_06173_amd import synth
    for nbytes in (1 << 20, (1 << 20) + 4, 4 << 20, 30_720_000, 64 << 20, 180_355_072, 524_288_000):
        d = synth.padded_extent(nbytes)
        assert d >= nbytes + 2048 and d % 4096 == 2048          # consecutive buffers: an odd multiple of 2 KiB apart
        assert d - nbytes < 8192 + 2048                           # at most 10 KiB given away per buffer
    assert synth.padded_extent(100) == 256 and synth.padded_extent(0) == 0
    w = synth.workloads()["gpt2_xl_adamw_bf16g"]
    shapes = [(33,), (0,), (5,), (300_000,), (70_001,)]
    ref = synth.make_state(w, "cpu", shapes=shapes, layout="by_tensor")
    for layout in ("padded", "by_stream", "framework"):
        s = synth.make_state(w, "cpu", shapes=shapes, layout=layout)
        for a, b in zip((s.theta, s.grad, s.m, s.v), (ref.theta, ref.grad, ref.m, ref.v)):
            assert all(torch.equal(x, y) and x.dtype == y.dtype for x, y in zip(a, b)), layout
    s = synth.make_state(w, "cpu", shapes=shapes)                 # the default is the padded arena
    assert s.grad[3].data_ptr() - s.theta[3].data_ptr() == synth.padded_extent(300_000 * 4)
    assert all(t.data_ptr() % 16 == 0 for t in s.theta + s.m + s.v if t.numel())


def test_tracker_host_logic_without_a_gpu(B):
    h = ctypes.c_void_p()
    assert B._lib.swift_tracker_create(-1, ctypes.byref(h)) == B.SWIFT_EINVAL
    assert B._lib.swift_tracker_create(3, None) == B.SWIFT_EINVAL
    assert B._lib.swift_tracker_create(3, ctypes.byref(h)) == B.SWIFT_OK and h.value
    hp = B.hparams("adamw", step=5, lr=1e-3)
    lst = B.SwiftTensorList(0, None, None, None, None, None, None)
    ids = (ctypes.c_int64 * 1)(0)
    # no iteration in progress yet
    assert B._lib.swift_tracker_step(h, ctypes.byref(lst), ids, ctypes.byref(hp), None, None) == B.SWIFT_EINVAL
    assert "begin" in B.swift_last_error()
    assert B._lib.swift_tracker_begin(h, 0) == B.SWIFT_EINVAL
    assert B._lib.swift_tracker_begin(h, 4) == B.SWIFT_OK
    # the step of the hyper-parameters must be the iteration in progress
    assert B._lib.swift_tracker_step(h, ctypes.byref(lst), ids, ctypes.byref(hp), None, None) == B.SWIFT_EINVAL
    assert B._lib.swift_tracker_step(h, None, ids, ctypes.byref(hp), None, None) == B.SWIFT_EINVAL
    assert B._lib.swift_tracker_begin(h, 5) == B.SWIFT_OK
    one = B.SwiftTensorList(1, None, None, None, None, None, None)
    bad = (ctypes.c_int64 * 1)(7)
    assert B._lib.swift_tracker_step(h, ctypes.byref(one), bad, ctypes.byref(hp), None, None) == B.SWIFT_EINVAL
    assert "out of range" in B.swift_last_error()
    assert B._lib.swift_tracker_step(h, ctypes.byref(one), None, ctypes.byref(hp), None, None) == B.SWIFT_EINVAL
    # an id named twice in one call is refused before anything is launched, and leaves no mark behind
    two = B.SwiftTensorList(2, None, None, None, None, None, None)
    dup = (ctypes.c_int64 * 2)(1, 1)
    assert B._lib.swift_tracker_step(h, ctypes.byref(two), dup, ctypes.byref(hp), None, None) == B.SWIFT_EINVAL
    assert "twice" in B.swift_last_error()
    mixed = (ctypes.c_int64 * 2)(2, 9)
    assert B._lib.swift_tracker_step(h, ctypes.byref(two), mixed, ctypes.byref(hp), None, None) == B.SWIFT_EINVAL
    marks = (ctypes.c_uint8 * 3)(9, 9, 9)
    assert B._lib.swift_tracker_marks(h, ctypes.cast(marks, ctypes.c_void_p)) == B.SWIFT_OK    # nothing pending
    assert list(marks) == [0, 0, 0]
    assert B._lib.swift_tracker_marks(h, None) == B.SWIFT_EINVAL
    assert B._lib.swift_tracker_undo(h, ctypes.byref(one), ctypes.byref(hp), None) == B.SWIFT_EINVAL   # wrong length
    assert B._lib.swift_tracker_destroy(h) == B.SWIFT_OK
    assert B._lib.swift_tracker_destroy(None) == B.SWIFT_OK


def test_header_is_plain_c(tmp_path):
    # the boundary is a C ABI: the header must compile as C (no C++ or HIP types in the signatures)
    import subprocess
    src = tmp_path / "use.c"
    src.write_text('#include "swift_undo.h"\n'
                   'int probe(void) { swift_hparams hp; swift_tensor_list l; hp.kind = SWIFT_LAMB; l.n = 0;\n'
                   '  return swift_opt_step(&l, &hp, 0, 0) + (int)swift_digest_count(0, 0, 0); }\n')
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only",
                           "-I", os.path.join(ROOT, "include"), str(src)])


def test_arena_layout_is_host_arithmetic_and_matches_the_benchmark_state(B):
    """swift_arena_layout: offsets are 256-byte aligned and disjoint, large buffers start an odd multiple of 2 KiB
    apart, and the rule is the one the synthetic states are laid out with."""
    from paper_2302_06173_amd import synth
    for shapes, bf16, with_v in ((synth.bert_large_shapes(), False, True), (synth.gpt2_xl_shapes(), True, True),
                                 (synth.vit_128_32_shapes(), False, False), ([(0,), (3,), (1 << 18,), (262145,)], False, True)):
        numel = [synth.numel(s) for s in shapes]
        rows, total = B.swift_arena_layout(numel, grad_bf16=bf16, with_v=with_v)
        off = 0
        for n, row in zip(numel, rows):
            assert len(row) == (4 if with_v else 3)
            for k, o in enumerate(row):
                nbytes = n * (2 if (bf16 and k == 1) else 4)
                assert o == off and o % 256 == 0
                off += synth.padded_extent(nbytes)
                if nbytes >= 1 << 20:
                    assert (off - o) % 4096 == 2048            # an odd multiple of 2 KiB to the next buffer
        assert total == off
    rows, total = B.swift_arena_layout([1 << 18, 5], with_v=False, with_m=False)      # plain SGD: theta and g only
    assert [len(r) for r in rows] == [2, 2] and rows[0] == [0, synth.padded_extent(4 << 18)]
    assert total == 2 * synth.padded_extent(4 << 18) + 2 * 256
    assert B.swift_arena_layout([], with_v=True) == ([], 0)
    with pytest.raises(B.SwiftError):
        B.swift_arena_layout([-1])
