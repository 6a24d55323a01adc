"""CPU-only checks of the C-ABI library: it loads, exports every function the
header declares, rejects bad arguments without touching a device, and its host
bookkeeping (a host-only arena) matches the independent Python model bit for
bit on hand-written and random traces."""
import ctypes
import os
import re

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

from oracle import ArenaModel, ArenaModelError
from paper_2410_15651_amd import binding as rb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
P = 16


def _declared_functions():
    text = "".join(open(os.path.join(ROOT, "include", f)).read()
                   for f in sorted(os.listdir(os.path.join(ROOT, "include"))) if f.endswith(".h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rlhf_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_function():
    names = _declared_functions()
    assert len(names) >= 24
    L = ctypes.CDLL(rb.LIB_PATH)
    for n in names:
        assert hasattr(L, n), n
    assert sorted(rb.EXPORTS) == names
    assert rb.rlhf_version() == 1


def test_struct_sizes_match_the_header():
    # computed from the field lists in include/rlhf_rollout.h on an LP64 target
    assert ctypes.sizeof(rb.ArenaDesc) == 8 * 4 + 8 + 8 + 8
    assert ctypes.sizeof(rb.ArenaStats) == 4 * 8 + 4 * 4
    assert ctypes.sizeof(rb.AttnParams) == 10 * 4
    assert ctypes.sizeof(rb.RewardShaping) == 3 * 8 + 2 * 4 + 8


def _host_arena(**kw):
    base = dict(max_seqs=3, n_kv_heads=2, head_dim=64, n_pages=6, max_pages_per_seq=3,
                kv_dtype=rb.RLHF_BF16, flags=rb.RLHF_ARENA_HOST_ONLY)
    base.update(kw)
    return rb.rlhf_kv_arena_create(**base), base


def _state(h, cfg):
    t, l, f = rb.rlhf_kv_arena_host_state(h, cfg["max_seqs"], cfg["max_pages_per_seq"])
    return t.tolist(), l.tolist(), f.tolist()


def _compare(h, cfg, m: ArenaModel):
    t, l, f = _state(h, cfg)
    assert t == m.page_table()
    assert l == m.seq_lens
    assert f == m.free
    s = rb.rlhf_kv_arena_stats(h)
    ms = m.stats()
    for k, v in ms.items():
        assert s[k] == v, k
    assert s["driver_allocations"] == 0


def test_hand_trace_matches_model():
    order = [4, 2, 5, 0, 1, 3]
    h, cfg = _host_arena(initial_free_order=order)
    m = ArenaModel(3, 2, 64, P, 6, 3, initial_free_order=order)
    try:
        _compare(h, cfg, m)
        for ids, ns in (([1, 0], [17, 1]), ([0], [15]), ([0], [1]), ([2, 1], [0, 3])):
            rb.rlhf_kv_arena_append(h, ids, ns)
            m.append(ids, ns)
            _compare(h, cfg, m)
        rb.rlhf_kv_arena_free_seq(h, 1)
        m.free_seq(1)
        _compare(h, cfg, m)
        rb.rlhf_kv_arena_reset(h)
        m.reset()
        _compare(h, cfg, m)
    finally:
        rb.rlhf_kv_arena_destroy(h)


def test_failed_appends_change_nothing():
    h, cfg = _host_arena(max_seqs=2, n_pages=3, max_pages_per_seq=2, n_kv_heads=1)
    try:
        rb.rlhf_kv_arena_append(h, [0], [20])
        before = _state(h, cfg)
        with pytest.raises(rb.RlhfError) as e:
            rb.rlhf_kv_arena_append(h, [1, 0], [17, 1])
        assert e.value.status == rb.RLHF_ERR_OOM
        assert _state(h, cfg) == before
        for ids, ns in (([0], [13]), ([0, 0], [1, 1]), ([2], [1]), ([-1], [1]), ([1], [-1])):
            with pytest.raises(rb.RlhfError) as e:
                rb.rlhf_kv_arena_append(h, ids, ns)
            assert e.value.status == rb.RLHF_ERR_INVALID
            assert _state(h, cfg) == before
        rb.rlhf_kv_arena_append(h, [0], [12])
        assert _state(h, cfg)[1] == [32, 0]
        with pytest.raises(rb.RlhfError):
            rb.rlhf_kv_arena_free_seq(h, 5)
        with pytest.raises(rb.RlhfError):      # no device views on a host-only arena
            rb.rlhf_kv_arena_views(h)
    finally:
        rb.rlhf_kv_arena_destroy(h)


def test_a_refused_submission_takes_the_bookkeeping_back():
    """A device error before anything was enqueued must leave the arena as it was.
    The testing aid makes the next calls take exactly the path a refused kernel
    launch takes (bookkeeping done, then undone); the state is compared with the
    Python model, which never saw the failed calls."""
    order = [4, 2, 5, 0, 1, 3, 7, 6]
    h, cfg = _host_arena(n_pages=8, max_pages_per_seq=4, initial_free_order=order)
    m = ArenaModel(3, 2, 64, P, 8, 4, initial_free_order=order)
    try:
        rb.rlhf_kv_arena_append(h, [1, 0], [17, 1])
        m.append([1, 0], [17, 1])
        _compare(h, cfg, m)
        rb.rlhf_kv_arena_fail_next_submissions(h, 3)
        # new pages for two sequences, a first token for a third: pages, lengths, live_seqs, peak all move
        with pytest.raises(rb.RlhfError) as e:
            rb.rlhf_kv_arena_append(h, [0, 2, 1], [31, 5, 20])
        assert e.value.status == rb.RLHF_ERR_DEVICE
        _compare(h, cfg, m)
        with pytest.raises(rb.RlhfError) as e:
            rb.rlhf_kv_arena_free_seq(h, 1)
        assert e.value.status == rb.RLHF_ERR_DEVICE
        _compare(h, cfg, m)
        with pytest.raises(rb.RlhfError):                     # a call that fails validation does not use one up
            rb.rlhf_kv_arena_append(h, [0], [1000])
        with pytest.raises(rb.RlhfError) as e:
            rb.rlhf_kv_arena_free_seq(h, 2)                   # an empty sequence
        assert e.value.status == rb.RLHF_ERR_DEVICE
        _compare(h, cfg, m)
        # the aid has run out: the same calls now go through, from exactly the state the model is in
        rb.rlhf_kv_arena_append(h, [0, 2, 1], [31, 5, 20])
        m.append([0, 2, 1], [31, 5, 20])
        _compare(h, cfg, m)
        rb.rlhf_kv_arena_free_seq(h, 1)
        m.free_seq(1)
        _compare(h, cfg, m)
    finally:
        rb.rlhf_kv_arena_destroy(h)


def test_create_rejects_bad_descriptions():
    bad = [
        dict(page_tokens=8), dict(head_dim=96), dict(kv_dtype=rb.RLHF_F32), dict(n_pages=0),
        dict(max_seqs=0), dict(initial_free_order=[0, 1, 2, 3, 4, 4]),
    ]
    for kw in bad:
        with pytest.raises(rb.RlhfError) as e:
            _host_arena(**kw)
        assert e.value.status in (rb.RLHF_ERR_INVALID, rb.RLHF_ERR_UNSUPPORTED), kw
        assert rb.rlhf_last_error_string() != ""


def test_bytes_required_is_two_halves_of_pages():
    n = rb.rlhf_kv_arena_bytes_required(max_seqs=4, n_kv_heads=8, head_dim=128, n_pages=100,
                                        max_pages_per_seq=10, kv_dtype=rb.RLHF_BF16)
    assert n == 2 * 100 * 8 * 16 * 128 * 2


def test_compute_entry_points_validate_before_launching():
    p = rb.attn_params(2, 4, 3, 64, 4, rb.RLHF_BF16)            # 3 does not divide 4
    with pytest.raises(rb.RlhfError) as e:
        rb.rlhf_decode_attention_workspace_bytes(p)
    assert e.value.status == rb.RLHF_ERR_INVALID
    p = rb.attn_params(2, 4, 4, 80, 4, rb.RLHF_BF16)
    with pytest.raises(rb.RlhfError) as e:
        rb.rlhf_decode_attention_workspace_bytes(p)
    assert e.value.status == rb.RLHF_ERR_UNSUPPORTED
    p = rb.attn_params(2, 4, 4, 64, 4, rb.RLHF_BF16)
    assert rb.rlhf_decode_attention_workspace_bytes(p) >= 2 * 4 * (64 + 2) * 4
    with pytest.raises(rb.RlhfError) as e:                       # NULL buffers
        rb.rlhf_decode_attention(p, 0, 0, 0, 0, 0, 0, 0, 0)
    assert e.value.status == rb.RLHF_ERR_INVALID
    with pytest.raises(rb.RlhfError) as e:                       # NULL buffers
        rb.rlhf_prefill_attention(p, 0, 0, 8, 0, 0, 0, 0, 0)
    assert e.value.status == rb.RLHF_ERR_INVALID
    rb.rlhf_prefill_attention(p, 0, 0, 0, 0, 0, 0, 0, 0)         # no rows: nothing to do
    for waves in (0, 8, 12):
        rb.rlhf_prefill_attention_wg(p, 0, 0, 0, 0, 0, 0, 0, 0, waves)
    for waves in (-1, 4, 10, 16):                                  # only 0 (auto), 8 and 12 exist
        with pytest.raises(rb.RlhfError) as e:
            rb.rlhf_prefill_attention_wg(p, 16, 16, 8, 16, 16, 16, 16, 16, waves)
        assert e.value.status == rb.RLHF_ERR_INVALID
    with pytest.raises(rb.RlhfError) as e:
        rb.rlhf_prefill_attention(rb.attn_params(2, 4, 3, 64, 4, rb.RLHF_BF16), 16, 16, 8, 16, 16, 16, 16, 16)
    assert e.value.status == rb.RLHF_ERR_INVALID
    with pytest.raises(rb.RlhfError) as e:
        rb.rlhf_token_logprobs_kl(0, 0, 0, 0, 0, n_positions=4, vocab=10, logits_dtype=rb.RLHF_F32)
    assert e.value.status == rb.RLHF_ERR_INVALID
    with pytest.raises(rb.RlhfError) as e:
        rb.rlhf_token_logprobs_kl(16, 16, 16, 16, 16, n_positions=4, vocab=10, row_stride_elems=8,
                                  logits_dtype=rb.RLHF_F32)
    assert e.value.status == rb.RLHF_ERR_INVALID
    with pytest.raises(rb.RlhfError) as e:                       # unknown penalty kind
        rb.rlhf_token_logprobs_kl_rewards(16, 16, 16, 16, 16, 0.1, penalty=7, n_positions=4, vocab=10,
                                          logits_dtype=rb.RLHF_F32)
    assert e.value.status == rb.RLHF_ERR_INVALID


def test_sampling_and_probe_entry_points_validate_before_launching():
    # workspace sizes: 16 bytes per row and segment; segments = min(8, ceil(512 / rows), vocab / 8192), >= 1
    assert rb.rlhf_sample_tokens_workspace_bytes(128, 128256) == 128 * 4 * 16
    assert rb.rlhf_sample_tokens_workspace_bytes(4, 128256) == 4 * 8 * 16
    assert rb.rlhf_sample_tokens_workspace_bytes(4, 50272) == 4 * 6 * 16
    assert rb.rlhf_sample_tokens_workspace_bytes(4, 100) == 4 * 16
    assert rb.rlhf_sample_tokens_workspace_bytes(1000, 128256) == 1000 * 16
    assert rb.rlhf_sample_tokens_workspace_bytes(0, 128256) == 16          # never zero bytes
    with pytest.raises(rb.RlhfError) as e:
        rb.rlhf_sample_tokens_workspace_bytes(-1, 10)
    assert e.value.status == rb.RLHF_ERR_INVALID
    with pytest.raises(rb.RlhfError) as e:                                   # NULL workspace
        rb.rlhf_sample_tokens_split(16, 16, 1.0, 1, 0, n_rows=4, vocab=10, logits_dtype=rb.RLHF_F32,
                                    workspace_bytes=1024)
    assert e.value.status == rb.RLHF_ERR_INVALID
    with pytest.raises(rb.RlhfError) as e:                                   # workspace too small
        rb.rlhf_sample_tokens_split(16, 16, 1.0, 1, 16, n_rows=4, vocab=65536, logits_dtype=rb.RLHF_BF16,
                                    workspace_bytes=4 * 8 * 16 - 1)
    assert e.value.status == rb.RLHF_ERR_INVALID
    with pytest.raises(rb.RlhfError) as e:                                   # negative temperature
        rb.rlhf_sample_tokens(16, 16, -1.0, 1, n_rows=4, vocab=10, logits_dtype=rb.RLHF_F32)
    assert e.value.status == rb.RLHF_ERR_INVALID
    rb.rlhf_sample_tokens_split(16, 16, 1.0, 1, 16, n_rows=0, vocab=10, logits_dtype=rb.RLHF_F32,
                                workspace_bytes=16)                          # no rows: nothing to do
    for bad in (dict(top_k=0), dict(top_k=-3), dict(top_k=5, temperature=-0.5), dict(top_k=5, vocab=0),
                dict(top_k=5, logits_dtype=9), dict(top_k=5, row_stride_elems=7), dict(top_k=5, logits=0),
                dict(top_k=20, logits=0), dict(top_k=5, logits=18, logits_dtype=rb.RLHF_F32)):
        kw = dict(logits=16, tokens_out=16, temperature=1.0, top_k=5, seed=1, n_rows=4, vocab=10,
                  logits_dtype=rb.RLHF_BF16)
        kw.update(bad)
        with pytest.raises(rb.RlhfError) as e:
            rb.rlhf_sample_tokens_topk(**kw)
        assert e.value.status in (rb.RLHF_ERR_INVALID, rb.RLHF_ERR_UNSUPPORTED), bad
    rb.rlhf_sample_tokens_topk(16, 16, 1.0, 5, 1, n_rows=0, vocab=10, logits_dtype=rb.RLHF_F32)   # no rows
    with pytest.raises(rb.RlhfError) as e:                                   # NULL / misaligned probe buffer
        rb.rlhf_probe_stream_read(0, 64)
    assert e.value.status == rb.RLHF_ERR_INVALID
    with pytest.raises(rb.RlhfError) as e:
        rb.rlhf_probe_stream_read(24, 64)
    assert e.value.status == rb.RLHF_ERR_INVALID
    for args in ((0, 10, 1, 64), (24, 10, 1, 64), (16, -1, 1, 64), (16, 10, 0, 64), (16, 10, 1, 0), (16, 10, 1, 68)):
        with pytest.raises(rb.RlhfError) as e:                               # operands, iterations, workgroups, ticks
            rb.rlhf_probe_matrix_rate(args[0], args[1], args[2], args[3], nbytes=64)
        assert e.value.status == rb.RLHF_ERR_INVALID, args


@settings(max_examples=120, deadline=None)
@given(st.data())
def test_random_traces_match_model(data):
    n_pages = data.draw(st.integers(1, 12))
    max_seqs = data.draw(st.integers(1, 4))
    mpps = data.draw(st.integers(1, 5))
    order = data.draw(st.permutations(list(range(n_pages))))
    cfg = dict(max_seqs=max_seqs, n_kv_heads=2, head_dim=128, n_pages=n_pages, max_pages_per_seq=mpps,
               kv_dtype=rb.RLHF_F16, flags=rb.RLHF_ARENA_HOST_ONLY, initial_free_order=order)
    h = rb.rlhf_kv_arena_create(**cfg)
    m = ArenaModel(max_seqs, 2, 128, P, n_pages, mpps, initial_free_order=order)
    try:
        for _ in range(data.draw(st.integers(1, 25))):
            op = data.draw(st.sampled_from(["append", "append", "append", "free", "reset"]))
            if op == "append":
                ids = data.draw(st.lists(st.integers(0, max_seqs - 1), unique=True, max_size=max_seqs))
                ns = [data.draw(st.integers(0, 40)) for _ in ids]
                try:
                    m.append(ids, ns)
                    expect = None
                except ArenaModelError as e:
                    expect = rb.RLHF_ERR_OOM if e.kind == "oom" else rb.RLHF_ERR_INVALID
                if expect is None:
                    rb.rlhf_kv_arena_append(h, ids, ns)
                else:
                    with pytest.raises(rb.RlhfError) as e:
                        rb.rlhf_kv_arena_append(h, ids, ns)
                    assert e.value.status == expect
            elif op == "free":
                s = data.draw(st.integers(0, max_seqs - 1))
                m.free_seq(s)
                rb.rlhf_kv_arena_free_seq(h, s)
            else:
                m.reset()
                rb.rlhf_kv_arena_reset(h)
            _compare(h, cfg, m)
    finally:
        rb.rlhf_kv_arena_destroy(h)
