"""Pins for the caching-allocator model (the oracle of the memory-trace tool):
hand-worked traces, and invariants that hold for any trace."""
import os

import pytest
from hypothesis import given, settings, strategies as st

from oracle import CachingAllocatorModel

HERE = os.path.dirname(os.path.abspath(__file__))


def hand_traces():
    traces, cur = {}, None
    for line in open(os.path.join(HERE, "golden", "alloc_hand_traces.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if line.startswith("trace "):
            cur = traces.setdefault(line.split()[1], [])
            continue
        op, expect = line.split("|")
        cur.append((op.split(), [int(x) for x in expect.split()]))
    return traces


def replay(model_cls, ops):
    """Runs [(op tokens, expected)] through a model; yields (expected, observed)."""
    m = model_cls()
    handles = {}
    n = 0
    for op, expect in ops:
        if op[0] == "m":
            n += 1
            handles[n] = m.malloc(int(op[1]))
        elif op[0] == "f":
            m.free(handles.pop(int(op[1])))
        else:
            m.empty_cache()
        s = m.stats()
        yield expect, [s["reserved_bytes"], s["allocated_bytes"], s["driver_allocations"],
                       s["last_fragmentation_bytes"], s["n_free_blocks"]]


@pytest.mark.parametrize("name", sorted(hand_traces()))
def test_hand_worked_traces(name):
    for step, (expect, got) in enumerate(replay(CachingAllocatorModel, hand_traces()[name])):
        assert got == expect, (name, step)


def test_fragmentation_at_the_peak_is_what_the_pool_could_not_reuse():
    m = CachingAllocatorModel()
    a = m.malloc(8 << 20)
    m.malloc(8 << 20)
    m.free(a)
    m.malloc(9 << 20)           # 12 MiB free in the pool, but not in one piece
    s = m.stats()
    assert s["peak_reserved_bytes"] == 40 << 20
    assert s["fragmentation_at_peak_reserved_bytes"] == 12 << 20
    assert s["peak_reserved_bytes"] - s["fragmentation_at_peak_reserved_bytes"] == 28 << 20


@settings(max_examples=150, deadline=None)
@given(st.lists(st.tuples(st.sampled_from(["m", "m", "f", "e"]), st.integers(1, 30 << 20), st.integers(0, 50)),
                max_size=120))
def test_invariants_on_random_traces(ops):
    m = CachingAllocatorModel()
    live = []
    for op, size, pick in ops:
        before = m.stats()
        if op == "m":
            live.append((m.malloc(size), size))
            s = m.stats()
            assert s["allocated_bytes"] - before["allocated_bytes"] >= size
            if s["driver_allocations"] > before["driver_allocations"]:
                assert s["last_fragmentation_bytes"] == before["reserved_bytes"] - before["allocated_bytes"]
            else:
                assert s["reserved_bytes"] == before["reserved_bytes"]
        elif op == "f" and live:
            h, _ = live.pop(pick % len(live))
            m.free(h)
            assert m.stats()["reserved_bytes"] == before["reserved_bytes"]
        elif op == "e":
            m.empty_cache()
            s = m.stats()
            assert s["allocated_bytes"] == before["allocated_bytes"]
            assert s["reserved_bytes"] <= before["reserved_bytes"]
        s = m.stats()
        assert 0 <= s["allocated_bytes"] <= s["reserved_bytes"] <= s["peak_reserved_bytes"]
        assert s["allocated_bytes"] % 512 == 0 and s["reserved_bytes"] % (2 << 20) == 0
        # blocks tile every segment exactly, and no two free neighbours remain unmerged
        for seg in m.segments:
            if seg is None:
                continue
            off = 0
            for i, b in enumerate(seg["blocks"]):
                assert b["offset"] == off
                off += b["size"]
                if i:
                    assert not (b["free"] and seg["blocks"][i - 1]["free"])
            assert off == seg["size"]
    for h, _ in live:
        m.free(h)
    m.empty_cache()
    s = m.stats()
    assert s["reserved_bytes"] == 0 and s["allocated_bytes"] == 0 and s["n_segments"] == 0
    assert s["driver_frees"] == s["driver_allocations"]


# ---- the library's simulator against the model, counter by counter ----------
def _lib_model():
    from paper_2410_15651_amd import binding as rb
    return rb.AllocSim


@pytest.mark.parametrize("name", sorted(hand_traces()))
def test_library_simulator_on_hand_worked_traces(name):
    for step, (expect, got) in enumerate(replay(_lib_model(), hand_traces()[name])):
        assert got == expect, (name, step)


@settings(max_examples=150, deadline=None)
@given(st.lists(st.tuples(st.sampled_from(["m", "m", "m", "f", "f", "e"]),
                          st.one_of(st.integers(1, 4096), st.integers(1, 3 << 20), st.integers(1, 40 << 20)),
                          st.integers(0, 1000)), max_size=200))
def test_library_simulator_matches_model_on_random_traces(ops):
    from paper_2410_15651_amd import binding as rb
    lib_sim, model = rb.AllocSim(), CachingAllocatorModel()
    live = []
    try:
        for op, size, pick in ops:
            if op == "m":
                live.append((lib_sim.malloc(size), model.malloc(size)))
            elif op == "f" and live:
                a, b = live.pop(pick % len(live))
                lib_sim.free(a)
                model.free(b)
            elif op == "e":
                lib_sim.empty_cache()
                model.empty_cache()
            assert lib_sim.stats() == model.stats()
        with pytest.raises(rb.RlhfError):
            lib_sim.free(10 ** 9)
        with pytest.raises(rb.RlhfError):
            lib_sim.malloc(0)
    finally:
        lib_sim.close()
