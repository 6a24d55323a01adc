"""Replays the allocation trace of a PPO iteration through the library's
caching-allocator simulator, with the generation phase's key/value cache held
either by that allocator too or by the KV arena, and reports the paper's
counters (Section 2.2): reserved, allocated, and the fragmentation present at
the reserved peak (Section 3.1), with and without `empty_cache()` at the phase
boundaries (Section 3.3).

    python -m paper_2410_15651_amd.memtrace [shape] [iterations]

Everything runs on the host: the simulator is host code and the arena is
created with RLHF_ARENA_HOST_ONLY, which drives the same bookkeeping that a
device arena uses.
"""
from __future__ import annotations

import sys
from typing import List

import numpy as np

from . import binding as rb
from . import workloads as wl

PAGE = wl.PAGE_TOKENS


def _arena_for(shape: wl.TraceShape):
    """One arena for all layers: a page holds 16 tokens of every layer's K and V
    heads (the layers are folded into the head count)."""
    tokens = shape.prompt_len + shape.gen_len
    pages_per_seq = (tokens + PAGE - 1) // PAGE
    kw = dict(max_seqs=shape.batch, n_kv_heads=shape.n_kv_heads * shape.n_layers, head_dim=shape.head_dim,
              n_pages=shape.batch * pages_per_seq, max_pages_per_seq=pages_per_seq, kv_dtype=rb.RLHF_BF16,
              flags=rb.RLHF_ARENA_HOST_ONLY)
    return rb.rlhf_kv_arena_create(**kw)


def replay(events: List[tuple], shape: wl.TraceShape, use_arena: bool, empty_cache: bool) -> dict:
    """Returns the summary counters and the curve [(phase, reserved, allocated)]
    sampled at every phase boundary and at every new reserved peak."""
    sim = rb.AllocSim()
    arena = _arena_for(shape) if use_arena else None
    handles = {}
    kv_keys = set()
    curve, phase = [], "setup"
    peak_reserved = peak_allocated = frag_at_peak = 0
    peak_phase = phase
    seq_ids = np.arange(shape.batch, dtype=np.int32)
    kv_tokens = 0            # tokens per sequence the arena currently holds
    kv_row = shape.n_kv_heads * shape.head_dim * 2

    def totals():
        s = sim.stats()
        r, a = s["reserved_bytes"], s["allocated_bytes"]
        if arena is not None:
            st = rb.rlhf_kv_arena_stats(arena)
            r += st["reserved_bytes"]
            a += st["allocated_bytes"]
        return r, a, s

    try:
        for ev in events:
            if ev[0] == "phase":
                if empty_cache:
                    sim.empty_cache()
                if arena is not None and kv_tokens and not ev[1].startswith("generation"):
                    rb.rlhf_kv_arena_reset(arena)              # phase boundary: every page free again
                    kv_tokens = 0
                r, a, _ = totals()
                curve.append((phase, r, a))
                phase = ev[1]
                continue
            if ev[0] == "alloc":
                _, key, nbytes, kind = ev
                if kind == "kv" and arena is not None:
                    # the cache of a layer after t tokens: the arena holds it once, for all layers
                    kv_keys.add(key)
                    tokens = nbytes // (shape.batch * kv_row)
                    if tokens > kv_tokens:
                        grow = np.full(shape.batch, tokens - kv_tokens, dtype=np.int32)
                        rb.rlhf_kv_arena_append(arena, seq_ids, grow)
                        kv_tokens = tokens
                else:
                    before = sim.stats()["driver_allocations"]
                    handles[key] = sim.malloc(nbytes)
                    if sim.stats()["driver_allocations"] == before:
                        continue
            else:
                key = ev[1]
                if key in kv_keys:
                    kv_keys.discard(key)
                else:
                    sim.free(handles.pop(key))
                continue
            r, a, s = totals()
            peak_allocated = max(peak_allocated, a)
            if r > peak_reserved:
                peak_reserved, peak_phase = r, phase
                frag_at_peak = s["last_fragmentation_bytes"]
                curve.append((phase, r, a))
        s = sim.stats()
        arena_reserved = rb.rlhf_kv_arena_stats(arena)["reserved_bytes"] if arena is not None else 0
        return dict(peak_reserved_bytes=peak_reserved, peak_allocated_bytes=max(peak_allocated, s["peak_allocated_bytes"]),
                    fragmentation_at_peak_reserved_bytes=frag_at_peak, peak_phase=peak_phase,
                    driver_allocations=s["driver_allocations"] + (1 if arena is not None else 0),
                    driver_frees=s["driver_frees"], arena_reserved_bytes=arena_reserved, curve=curve)
    finally:
        sim.close()
        if arena is not None:
            rb.rlhf_kv_arena_destroy(arena)


def table(shape_name: str = "opt1.3b_b32", iterations: int = 2) -> str:
    shape = wl.TRACE_SHAPES[shape_name]
    events = wl.ppo_iteration_trace(shape, iterations)
    gib = 1024.0 ** 3
    lines = [f"allocation trace {shape.name}: {iterations} PPO iterations, {len(events)} events; GiB",
             f"{'KV cache held by':18s} {'empty_cache':>11s} {'peak reserved':>13s} {'peak allocated':>14s} "
             f"{'fragmentation at peak':>21s} {'peak in phase':>22s} {'driver allocations':>18s}"]
    for use_arena in (False, True):
        for ec in (False, True):
            r = replay(events, shape, use_arena, ec)
            lines.append(f"{'arena' if use_arena else 'caching allocator':18s} {'yes' if ec else 'no':>11s} "
                         f"{r['peak_reserved_bytes'] / gib:13.3f} {r['peak_allocated_bytes'] / gib:14.3f} "
                         f"{r['fragmentation_at_peak_reserved_bytes'] / gib:21.3f} {r['peak_phase']:>22s} "
                         f"{r['driver_allocations']:18d}")
    return "\n".join(lines)


if __name__ == "__main__":
    name = sys.argv[1] if len(sys.argv) > 1 else "opt1.3b_b32"
    iters = int(sys.argv[2]) if len(sys.argv) > 2 else 2
    print(table(name, iters))
