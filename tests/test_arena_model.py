"""Pins for the Python arena model: the invariants that the paper's counter
definitions (Section 2.2: reserved vs allocated) and a fixed-page free list
imply, checked on hand-written and random traces."""
import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

from oracle import ArenaModel, ArenaModelError

P = 16


def check_invariants(m: ArenaModel):
    held = [p for row in m.pages for p in row]
    assert sorted(held + m.free) == list(range(m.n_pages))          # each page in exactly one place
    for s in range(m.max_seqs):
        assert len(m.pages[s]) == (m.seq_lens[s] + P - 1) // P
        assert len(m.pages[s]) <= m.max_pages_per_seq
    st_ = m.stats()
    assert st_["reserved_bytes"] == 2 * m.n_pages * m.n_kv_heads * P * m.head_dim * m.elem_bytes
    assert st_["allocated_bytes"] == 2 * len(held) * m.n_kv_heads * P * m.head_dim * m.elem_bytes
    assert st_["pages_free"] + st_["pages_in_use"] == m.n_pages
    assert st_["live_token_bytes"] <= st_["allocated_bytes"] <= st_["reserved_bytes"]
    # internal waste below one page per live sequence
    waste_tokens = sum(len(m.pages[s]) * P - m.seq_lens[s] for s in range(m.max_seqs))
    assert waste_tokens <= (P - 1) * st_["live_seqs"]


def test_hand_trace():
    m = ArenaModel(3, 2, 64, P, 6, 3, initial_free_order=[4, 2, 5, 0, 1, 3])
    placed = m.append([1, 0], [17, 1])
    assert m.pages == [[5], [4, 2], []]
    assert m.seq_lens == [1, 17, 0]
    assert placed[0] == (1, 0, 4, 0) and placed[15] == (1, 15, 4, 15) and placed[16] == (1, 16, 2, 0)
    assert placed[17] == (0, 0, 5, 0)
    assert m.free == [0, 1, 3]
    m.append([0], [15])                       # fills page 5 exactly, no new page
    assert m.pages[0] == [5] and m.free == [0, 1, 3]
    m.append([0], [1])
    assert m.pages[0] == [5, 0]
    m.free_seq(1)
    assert m.free == [1, 3, 4, 2] and m.seq_lens[1] == 0
    s = m.stats()
    assert s["pages_in_use"] == 2 and s["peak_pages_in_use"] == 4 and s["live_seqs"] == 1
    assert s["allocated_bytes"] == 2 * 2 * (2 * P * 64 * 2)
    assert s["live_token_bytes"] == 17 * 2 * 2 * 64 * 2
    m.reset()
    assert m.free == [4, 2, 5, 0, 1, 3] and m.seq_lens == [0, 0, 0]
    check_invariants(m)


def test_oom_and_overflow_change_nothing():
    m = ArenaModel(2, 1, 64, P, 3, 2)
    m.append([0], [20])
    before = (list(m.free), list(m.seq_lens), [list(r) for r in m.pages])
    with pytest.raises(ArenaModelError) as e:
        m.append([1, 0], [17, 1])             # needs 2 pages, 1 free
    assert e.value.kind == "oom"
    assert before == (m.free, m.seq_lens, m.pages)
    with pytest.raises(ArenaModelError) as e:
        m.append([0], [13])                   # 33 tokens > 2 pages
    assert e.value.kind == "invalid"
    with pytest.raises(ArenaModelError):
        m.append([0, 0], [1, 1])              # repeated id
    with pytest.raises(ArenaModelError):
        m.append([2], [1])
    assert before == (m.free, m.seq_lens, m.pages)
    m.append([0], [12])                       # exactly to the limit is fine
    assert m.seq_lens[0] == 32


def test_bad_free_order_rejected():
    with pytest.raises(ArenaModelError):
        ArenaModel(1, 1, 64, P, 3, 2, initial_free_order=[0, 1, 1])


@settings(max_examples=150, deadline=None)
@given(st.data())
def test_random_traces_keep_invariants(data):
    n_pages = data.draw(st.integers(1, 12))
    max_seqs = data.draw(st.integers(1, 4))
    mpps = data.draw(st.integers(1, 5))
    order = data.draw(st.permutations(list(range(n_pages))))
    m = ArenaModel(max_seqs, 2, 64, P, n_pages, mpps, initial_free_order=order)
    for _ in range(data.draw(st.integers(1, 25))):
        op = data.draw(st.sampled_from(["append", "append", "append", "free", "reset"]))
        if op == "append":
            ids = data.draw(st.lists(st.integers(0, max_seqs - 1), unique=True, min_size=0, max_size=max_seqs))
            ns = [data.draw(st.integers(0, 40)) for _ in ids]
            snapshot = (list(m.free), list(m.seq_lens), [list(r) for r in m.pages])
            try:
                placed = m.append(ids, ns)
                assert len(placed) == sum(ns)
                for (s, pos, page, slot) in placed:
                    assert m.pages[s][pos // P] == page and slot == pos % P
            except ArenaModelError:
                assert snapshot == (m.free, m.seq_lens, m.pages)
        elif op == "free":
            m.free_seq(data.draw(st.integers(0, max_seqs - 1)))
        else:
            m.reset()
            assert m.free == list(order)
        check_invariants(m)
