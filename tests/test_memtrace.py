"""The allocation-trace replay (library simulator + host-only arena) against an
independent replay through the Python models, and the qualitative findings of
the paper that the trace is meant to show (Sections 3.1 and 3.3)."""
import numpy as np
import pytest

from oracle import ArenaModel, CachingAllocatorModel
from paper_2410_15651_amd import memtrace
from paper_2410_15651_amd import workloads as wl

TINY = wl.TraceShape("tiny", n_layers=3, hidden=512, n_kv_heads=4, head_dim=64, vocab=50272, critic_layers=2,
                     critic_hidden=256, batch=3, prompt_len=40, gen_len=24)


def model_replay(events, shape, use_arena, empty_cache):
    """The same bookkeeping as memtrace.replay, on the oracle-side models."""
    sim = CachingAllocatorModel()
    P = wl.PAGE_TOKENS
    pages_per_seq = (shape.prompt_len + shape.gen_len + P - 1) // P
    arena = ArenaModel(shape.batch, shape.n_kv_heads * shape.n_layers, shape.head_dim, P,
                       shape.batch * pages_per_seq, pages_per_seq) if use_arena else None
    kv_row = shape.n_kv_heads * shape.head_dim * 2
    handles, kv_keys, kv_tokens = {}, set(), 0
    peak_r = peak_a = frag = 0
    for ev in events:
        if ev[0] == "phase":
            if empty_cache:
                sim.empty_cache()
            if arena is not None and kv_tokens and not ev[1].startswith("generation"):
                arena.reset()
                kv_tokens = 0
            continue
        if ev[0] == "free":
            if ev[1] in kv_keys:
                kv_keys.discard(ev[1])
            else:
                sim.free(handles.pop(ev[1]))
            continue
        _, key, nbytes, kind = ev
        grew = False
        if kind == "kv" and arena is not None:
            kv_keys.add(key)
            tokens = nbytes // (shape.batch * kv_row)
            if tokens > kv_tokens:
                arena.append(list(range(shape.batch)), [tokens - kv_tokens] * shape.batch)
                kv_tokens = tokens
            grew = True
        else:
            before = sim.driver_allocations
            handles[key] = sim.malloc(nbytes)
            grew = sim.driver_allocations > before
        r, a = sim.reserved, sim.allocated
        if arena is not None:
            st = arena.stats()
            r += st["reserved_bytes"]
            a += st["allocated_bytes"]
        if grew:
            peak_a = max(peak_a, a)
            if r > peak_r:
                peak_r, frag = r, sim.last_fragmentation
    return dict(peak_reserved_bytes=peak_r, fragmentation_at_peak_reserved_bytes=frag,
                driver_allocations=sim.driver_allocations + (1 if arena is not None else 0),
                driver_frees=sim.driver_frees)


def test_trace_is_balanced_and_deterministic():
    ev = wl.ppo_iteration_trace(TINY, 2)
    assert ev == wl.ppo_iteration_trace(TINY, 2)
    live = {}
    for e in ev:
        if e[0] == "alloc":
            assert e[1] not in live and e[2] > 0 and e[3] in ("kv", "tensor")
            live[e[1]] = e[2]
        elif e[0] == "free":
            live.pop(e[1])
    # what stays alive is the persistent adapter / optimizer state of the set-up phase
    setup = [e for e in ev[:ev.index(("phase", "generation[0]"))] if e[0] == "alloc"]
    assert sorted(live) == sorted(e[1] for e in setup)
    assert [e[1] for e in ev if e[0] == "phase"][:3] == ["setup", "generation[0]", "inference:actor[0]"]


@pytest.mark.parametrize("use_arena", [False, True])
@pytest.mark.parametrize("empty_cache", [False, True])
def test_library_replay_equals_model_replay(use_arena, empty_cache):
    ev = wl.ppo_iteration_trace(TINY, 2)
    got = memtrace.replay(ev, TINY, use_arena, empty_cache)
    want = model_replay(ev, TINY, use_arena, empty_cache)
    for k, v in want.items():
        assert got[k] == v, k


def test_findings_have_the_shape_the_paper_reports():
    shape = wl.TRACE_SHAPES["opt1.3b_b2"]
    ev = wl.ppo_iteration_trace(shape, 2)
    plain = memtrace.replay(ev, shape, False, False)
    cleared = memtrace.replay(ev, shape, False, True)
    arena = memtrace.replay(ev, shape, True, True)
    # Section 3.1: the peak falls in training, and reserved exceeds what live tensors need by the
    # fragmentation accumulated earlier
    assert plain["peak_phase"].startswith("training")
    assert plain["fragmentation_at_peak_reserved_bytes"] > 0.15 * plain["peak_reserved_bytes"]
    assert plain["peak_reserved_bytes"] - plain["fragmentation_at_peak_reserved_bytes"] <= plain["peak_allocated_bytes"] * 1.02
    # Section 3.3: empty_cache() at the phase boundaries removes most of it, at the price of driver calls
    assert cleared["peak_reserved_bytes"] < 0.85 * plain["peak_reserved_bytes"]
    assert cleared["driver_allocations"] > plain["driver_allocations"]
    # the arena takes the cache out of the allocator's pool: one driver allocation for it, ever
    assert arena["arena_reserved_bytes"] > 0
    assert arena["fragmentation_at_peak_reserved_bytes"] <= cleared["fragmentation_at_peak_reserved_bytes"] + (64 << 20)
    big = wl.TRACE_SHAPES["opt1.3b_b32"]
    ev = wl.ppo_iteration_trace(big, 1)
    assert memtrace.replay(ev, big, True, False)["peak_reserved_bytes"] < \
        0.5 * memtrace.replay(ev, big, False, False)["peak_reserved_bytes"]
