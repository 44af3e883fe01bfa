"""The library's per-list tables: they are never freed behind the caller's back (a layer-wise loop over
hundreds of lists keeps hitting), only swift_cache_trim and swift_shutdown free them, tables that a
captured graph uses survive a trim, and a call that would have to build tables under capture is refused."""
import pytest
import torch

from gpu_util import binding_hparams

pytestmark = pytest.mark.gpu

HPD = dict(lr=6e-4, weight_decay=0.1, beta1=0.9, beta2=0.95, eps=1e-8, step=10)


@pytest.fixture(scope="module")
def B():
    from paper_2302_06173_amd import binding
    return binding


def _lists(B, n_lists, numel, seed):
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    flat = [torch.empty(n_lists * numel, dtype=torch.float32, device="cuda").normal_(0.0, s, generator=gen)
            for s in (0.02, 1e-3, 1e-4, 1e-6)]
    flat[3].abs_()
    cut = lambda f, i: [f[i * numel:(i + 1) * numel]]
    return flat, [B.TensorList(cut(flat[0], i), cut(flat[1], i), cut(flat[2], i), cut(flat[3], i)) for i in range(n_lists)]


def test_three_hundred_lists_stay_cached_until_trimmed(B):
    B.swift_cache_trim(0)
    base, _ = B.swift_cache_stats()
    hp = binding_hparams(B, "adamw", HPD)
    flat, lists = _lists(B, 300, 1000, seed=1)
    for tl in lists:
        B.swift_opt_step(tl, hp)
    n1, bytes1 = B.swift_cache_stats()
    assert n1 == base + 300 and bytes1 > 0
    for tl in lists:                                   # the second round builds nothing: same tables
        B.swift_opt_undo(tl, hp)
    n2, bytes2 = B.swift_cache_stats()
    assert (n2, bytes2) == (n1, bytes1)
    torch.cuda.synchronize()
    B.swift_cache_trim(bytes1 // 2)
    n3, bytes3 = B.swift_cache_stats()
    assert bytes3 <= bytes1 // 2 and 0 < n3 < n1
    B.swift_opt_step(lists[0], hp)                     # the least recently used list was trimmed: rebuilt on demand
    B.swift_opt_undo(lists[0], hp)
    assert B.swift_cache_stats()[0] == n3 + 1
    B.swift_cache_trim(0)
    assert B.swift_cache_stats()[0] == base            # nothing pinned was left by this test


def test_tables_used_by_a_graph_survive_new_lists_and_a_trim(B):
    hp = binding_hparams(B, "adamw", HPD)
    flat_a, (tla,) = _lists(B, 1, 70001, seed=2)
    flat_b = [f.clone() for f in flat_a]
    tlb = B.TensorList(*[[f] for f in flat_b])
    dig_a = torch.zeros(3, dtype=torch.int64, device="cuda")
    dig_b = torch.zeros_like(dig_a)
    dmask = torch.ones(1, dtype=torch.uint8, device="cuda")

    def run(tl, dig):
        B.swift_opt_step_digest(tl, hp, dig)
        B.swift_opt_undo_dmask(tl, hp, dmask)
        B.swift_opt_step(tl, hp)
        B.swift_state_digest([tl._keep[0][0], tl._keep[2][0], tl._keep[3][0]], 0, out=dig)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    fresh_flat, (fresh,) = _lists(B, 1, 5000, seed=3)
    with torch.cuda.stream(side):
        run(tla, dig_a)                                # builds the tables of every call of the sequence
    run(tlb, dig_b)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        run(tla, dig_a)
        with pytest.raises(B.SwiftError) as e:         # a list the library has never seen: no tables, no allocation under capture
            B.swift_opt_step(fresh, hp, stream=side)
        assert e.value.code == B.SWIFT_EINVAL and "capturing" in e.value.message
    _, other = _lists(B, 300, 1000, seed=4)            # 300 further lists, then a trim to nothing
    for tl in other:
        B.swift_opt_step(tl, hp)
    torch.cuda.synchronize()
    B.swift_cache_trim(0)
    assert B.swift_cache_stats()[0] >= 1               # what the graph was recorded with is still there
    for k in range(3):
        graph.replay()
        run(tlb, dig_b)
        torch.cuda.synchronize()
        for x, y in zip(flat_a + [dig_a], flat_b + [dig_b]):
            assert torch.equal(x.view(torch.int32) if x.dtype == torch.float32 else x,
                               y.view(torch.int32) if y.dtype == torch.float32 else y), f"replay {k} differs from the eager run"


def test_reallocated_tensors_are_checked_again(B):
    """A list whose first buffer now lies in another allocation gets fresh tables (and fresh pointer checks)."""
    hp = binding_hparams(B, "adamw", HPD)
    n_before = B.swift_cache_stats()[0]
    big = torch.zeros(4 * 4096, dtype=torch.float32, device="cuda")
    parts = [[big[k * 4096:(k + 1) * 4096]] for k in range(4)]
    tl = B.TensorList(*parts)
    B.swift_opt_step(tl, hp)
    assert B.swift_cache_stats()[0] == n_before + 1
    B.swift_opt_undo(tl, hp)                           # same allocation: same tables
    assert B.swift_cache_stats()[0] == n_before + 1
    torch.cuda.synchronize()


def test_a_list_whose_memory_was_freed_is_validated_again(B):
    """The caller frees its tensors (the memory goes back to the runtime, which may hand the address out again for a
    smaller buffer): a later call with the old pointers and sizes must be refused by the pointer checks -- the cached
    tables are dropped and rebuilt, which validates again -- not run on memory that is gone."""
    hp = binding_hparams(B, "adamw", HPD)
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    n = 1 << 22
    big = torch.zeros(4 * n, dtype=torch.float32, device="cuda")            # 64 MiB: an allocation of its own
    base = big.data_ptr()
    parts = [[big[k * n:(k + 1) * n]] for k in range(4)]
    tl = B.TensorList(*parts)
    B.swift_opt_step(tl, hp)
    B.swift_opt_undo(tl, hp)
    torch.cuda.synchronize()
    n_lists = B.swift_cache_stats()[0]
    del parts, big
    tl._keep = None                                                          # the marshalled pointer arrays stay
    torch.cuda.empty_cache()                                                 # the 64 MiB go back to the runtime
    small = torch.zeros(n, dtype=torch.float32, device="cuda")              # 16 MiB, possibly at the freed address
    with pytest.raises(B.SwiftError) as e:
        B.swift_opt_step(tl, hp)         # same pointers, same sizes: unknown to the runtime now, or beyond `small`
    assert e.value.code == B.SWIFT_EINVAL
    assert ("run past the end" in e.value.message) if small.data_ptr() == base else True
    assert B.swift_cache_stats()[0] == n_lists - 1                           # the stale tables are gone
    torch.cuda.synchronize()
    assert float(small.abs().max()) == 0.0                                   # nothing ran


def test_concurrent_callers(B):
    """Four host threads step and undo their own lists (and digest a shared one) at the same time: results equal
    a serial run, the cache ends up with one entry per distinct list."""
    import threading
    hp = binding_hparams(B, "adamw", HPD)
    B.swift_cache_trim(0)
    base = B.swift_cache_stats()[0]
    flats, lists = [], []
    for t in range(4):
        f, ls = _lists(B, 8, 3000 + 17 * t, seed=10 + t)
        flats.append(f)
        lists.append(ls)
    ref = [[x.clone() for x in f] for f in flats]
    ref_lists = []
    for t in range(4):
        numel = 3000 + 17 * t
        cut = lambda f, i: [f[i * numel:(i + 1) * numel]]
        ref_lists.append([B.TensorList(cut(ref[t][0], i), cut(ref[t][1], i), cut(ref[t][2], i), cut(ref[t][3], i)) for i in range(8)])
    shared = torch.arange(100000, dtype=torch.float32, device="cuda")
    want = B.swift_state_digest([shared], 1 << 12)
    torch.cuda.synchronize()
    errors = []

    def work(t):
        try:
            stream = torch.cuda.Stream()
            with torch.cuda.stream(stream):
                for rep in range(20):
                    for tl in lists[t]:
                        B.swift_opt_step(tl, hp, stream=stream)
                    got = B.swift_state_digest([shared], 1 << 12, stream=stream)
                    for tl in reversed(lists[t]):
                        B.swift_opt_undo(tl, hp, stream=stream)
                    for tl in lists[t]:
                        B.swift_opt_step(tl, hp, stream=stream)
                    stream.synchronize()
                    if not torch.equal(got, want):
                        errors.append(f"thread {t}: digest differs")
        except Exception as exc:                                             # noqa: BLE001
            errors.append(f"thread {t}: {exc!r}")

    threads = [threading.Thread(target=work, args=(t,)) for t in range(4)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    assert not errors, errors
    for t in range(4):                                                       # the same 20 rounds, serially
        for rep in range(20):
            for tl in ref_lists[t]:
                B.swift_opt_step(tl, hp)
            for tl in reversed(ref_lists[t]):
                B.swift_opt_undo(tl, hp)
            for tl in ref_lists[t]:
                B.swift_opt_step(tl, hp)
    torch.cuda.synchronize()
    for t in range(4):
        for a, b in zip(flats[t], ref[t]):
            assert torch.equal(a.view(torch.int32), b.view(torch.int32))
    n_now = B.swift_cache_stats()[0]
    assert n_now == base + 4 * 8 * 2 + 1                                    # 64 optimizer lists (two copies) + the digest list
