"""GPU parity: the HIP library, called through its C ABI, against the fp64 CPU
oracle on the same seeded inputs.  Tolerances are fixed in advance:
2e-3 max-abs on attention outputs, 1e-3 on log-probs and KL (fp32
accumulation), bit-exact for every integer / byte result."""
import os

import numpy as np
import pytest
import torch

from paper_2410_15651_amd import binding as rb
from paper_2410_15651_amd import workloads as wl

pytestmark = pytest.mark.gpu

ATTN_TOL = 2e-3
LOGP_TOL = 1e-3
P = wl.PAGE_TOKENS


@pytest.fixture(scope="module")
def gu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_util
    return gpu_util


def _bits_differ(a, b):
    """Number of bytes in which two tensors differ (0: bit-identical)."""
    return int((a.contiguous().view(torch.uint8) != b.contiguous().view(torch.uint8)).sum())


def _say(msg):
    print(msg, flush=True)


# ------------------------------------------------------------------ arena ----
def _decode_block_layout(raw: np.ndarray, n_pages, Hkv, D):
    """Raw arena bytes -> plain pages [n_pages, Hkv, 16, D] for K and V, written
    from the layout formulas documented in include/rlhf_rollout.h."""
    half = raw.size // 2
    k = raw[:half].reshape(n_pages, Hkv, D // 8, P, 8)            # [dseg][slot][8]
    kp = k.transpose(0, 1, 3, 2, 4).reshape(n_pages, Hkv, P, D)
    v = raw[half:].reshape(n_pages, Hkv, P // 4, D, 4)            # [quad][d][4 slots]
    vp = v.transpose(0, 1, 2, 4, 3).reshape(n_pages, Hkv, P, D)
    return kp, vp


@pytest.mark.parametrize("cfg_index,batch", [(1, 4), (4, 6)])
def test_arena_append_gather_and_layout_bit_exact(gu, cfg_index, batch):
    cfg = wl.small_variant(wl.config(cfg_index), batch=batch, len_lo=1, len_hi=150)
    lens = wl.seq_lengths(cfg)
    lens[0] = 1
    lens[-1] = 150
    _say(f"arena cfg{cfg_index} lens={lens.tolist()}")
    q, ks, vs = wl.qkv(cfg, lens, device=gu.DEV)
    A = gu.FilledArena(cfg, lens, ks, vs)
    try:
        table, hl, free = A.host_state()
        assert table.tolist() == A.model.page_table()
        assert hl.tolist() == A.model.seq_lens == lens.tolist()
        assert free.tolist() == A.model.free
        st = rb.rlhf_kv_arena_stats(A.handle)
        for k_, v_ in A.model.stats().items():
            assert st[k_] == v_
        assert st["reserved_bytes"] == A.bytes and st["driver_allocations"] == 0
        # device mirrors
        _, _, d_table, d_lens = A.views()
        dev_table = torch.empty(cfg.batch * A.mpps, dtype=torch.int32, device=gu.DEV)
        dev_lens = torch.empty(cfg.batch, dtype=torch.int32, device=gu.DEV)
        import ctypes
        hip = ctypes.CDLL("libamdhip64.so")
        assert hip.hipMemcpy(ctypes.c_void_p(dev_table.data_ptr()), ctypes.c_void_p(d_table),
                             ctypes.c_size_t(dev_table.numel() * 4), 3) == 0
        assert hip.hipMemcpy(ctypes.c_void_p(dev_lens.data_ptr()), ctypes.c_void_p(d_lens),
                             ctypes.c_size_t(dev_lens.numel() * 4), 3) == 0
        assert dev_table.cpu().numpy().reshape(cfg.batch, A.mpps).tolist() == table.tolist()
        assert dev_lens.cpu().numpy().tolist() == lens.tolist()
        # gather returns exactly what was appended
        for b in range(cfg.batch):
            L = int(lens[b])
            ko = torch.zeros_like(ks[b])
            vo = torch.zeros_like(vs[b])
            rb.rlhf_kv_arena_gather(A.handle, b, 0, L, ko, vo)
            torch.cuda.synchronize()
            assert torch.equal(ko.view(torch.int16), ks[b].view(torch.int16))
            assert torch.equal(vo.view(torch.int16), vs[b].view(torch.int16))
            if L > 3:
                ko2 = torch.zeros_like(ks[b][2:L - 1])
                vo2 = torch.zeros_like(ko2)
                rb.rlhf_kv_arena_gather(A.handle, b, 2, L - 3, ko2, vo2)
                torch.cuda.synchronize()
                assert torch.equal(ko2.view(torch.int16), ks[b][2:L - 1].view(torch.int16))
                assert torch.equal(vo2.view(torch.int16), vs[b][2:L - 1].view(torch.int16))
        # raw bytes follow the documented block layout
        raw = A.buffer.cpu().numpy().view(np.uint16)
        kp, vp = _decode_block_layout(raw, A.n_pages, cfg.n_kv_heads, cfg.head_dim)
        ek, ev = wl.plain_pages([wl.to_storage(k) for k in ks], [wl.to_storage(v) for v in vs], table, A.n_pages)
        for b in range(cfg.batch):
            for lp in range((int(lens[b]) + P - 1) // P):
                n = min(P, int(lens[b]) - lp * P)
                pg = table[b, lp]
                assert np.array_equal(kp[pg, :, :n], ek[pg, :, :n])
                assert np.array_equal(vp[pg, :, :n], ev[pg, :, :n])
        # free + reuse: freed pages go to the tail, device table rows are cleared
        rb.rlhf_kv_arena_free_seq(A.handle, 0)
        A.model.free_seq(0)
        rb.rlhf_kv_arena_append(A.handle, [0], [5], ks[-1][:5].contiguous(), vs[-1][:5].contiguous())
        A.model.append([0], [5])
        torch.cuda.synchronize()
        table2, hl2, free2 = A.host_state()
        assert table2.tolist() == A.model.page_table() and free2.tolist() == A.model.free
        ko = torch.zeros_like(ks[-1][:5])
        vo = torch.zeros_like(ko)
        rb.rlhf_kv_arena_gather(A.handle, 0, 0, 5, ko, vo)
        torch.cuda.synchronize()
        assert torch.equal(ko.view(torch.int16), ks[-1][:5].view(torch.int16))
        assert torch.equal(vo.view(torch.int16), vs[-1][:5].view(torch.int16))
    finally:
        A.close()


def _device_mirrors(gu, A):
    """Device page table and lengths of a filled arena, copied back."""
    import ctypes
    _, _, d_table, d_lens = A.views()
    table = torch.empty(A.cfg.batch * A.mpps, dtype=torch.int32, device=gu.DEV)
    lens = torch.empty(A.cfg.batch, dtype=torch.int32, device=gu.DEV)
    hip = ctypes.CDLL("libamdhip64.so")
    torch.cuda.synchronize()
    assert hip.hipMemcpy(ctypes.c_void_p(table.data_ptr()), ctypes.c_void_p(d_table),
                         ctypes.c_size_t(table.numel() * 4), 3) == 0
    assert hip.hipMemcpy(ctypes.c_void_p(lens.data_ptr()), ctypes.c_void_p(d_lens),
                         ctypes.c_size_t(lens.numel() * 4), 3) == 0
    return table.cpu().numpy().reshape(A.cfg.batch, A.mpps).tolist(), lens.cpu().numpy().tolist()


def test_arena_refused_submission_leaves_host_and_device_mirrors_alone(gu):
    """A device error before any of a call's work is enqueued: the call returns
    RLHF_ERR_DEVICE and host and device bookkeeping are what they were, so the
    same call then goes through and the read-back is exact.  The refusal is the
    library's testing aid, which takes the path a refused first launch takes.
    Twelve appends in a row without a synchronisation also run through the four
    command slots three times (a call waits for the fourth-previous one)."""
    cfg = wl.small_variant(wl.config(4), batch=5, n_q_heads=4, n_kv_heads=4, len_lo=20, len_hi=90)
    lens = wl.seq_lengths(cfg)
    q, ks, vs = wl.qkv(cfg, lens, device=gu.DEV)
    A = gu.FilledArena(cfg, lens, ks, vs, slack_pages=12, extra_tokens=40)
    try:
        before = ([x.tolist() for x in A.host_state()], rb.rlhf_kv_arena_stats(A.handle), _device_mirrors(gu, A))
        extra_k = [torch.randn(30, cfg.n_kv_heads, cfg.head_dim, device=gu.DEV).to(ks[0].dtype) for _ in range(cfg.batch)]
        extra_v = [torch.randn(30, cfg.n_kv_heads, cfg.head_dim, device=gu.DEV).to(ks[0].dtype) for _ in range(cfg.batch)]
        ids = [3, 0, 4]
        k_new = torch.cat([extra_k[b][:n] for b, n in zip(ids, (30, 1, 17))]).contiguous()
        v_new = torch.cat([extra_v[b][:n] for b, n in zip(ids, (30, 1, 17))]).contiguous()
        rb.rlhf_kv_arena_fail_next_submissions(A.handle, 2)
        with pytest.raises(rb.RlhfError) as e:
            rb.rlhf_kv_arena_append(A.handle, ids, [30, 1, 17], k_new, v_new)
        assert e.value.status == rb.RLHF_ERR_DEVICE
        with pytest.raises(rb.RlhfError) as e:
            rb.rlhf_kv_arena_free_seq(A.handle, 1)
        assert e.value.status == rb.RLHF_ERR_DEVICE
        after = ([x.tolist() for x in A.host_state()], rb.rlhf_kv_arena_stats(A.handle), _device_mirrors(gu, A))
        assert after == before
        # the same calls now succeed, from the unchanged state
        rb.rlhf_kv_arena_append(A.handle, ids, [30, 1, 17], k_new, v_new)
        A.model.append(ids, [30, 1, 17])
        rb.rlhf_kv_arena_free_seq(A.handle, 1)
        A.model.free_seq(1)
        for step in range(12):                              # decode steps back to back, no synchronisation
            rb.rlhf_kv_arena_append(A.handle, [2], [1], extra_k[2][step:step + 1].contiguous(),
                                    extra_v[2][step:step + 1].contiguous())
            A.model.append([2], [1])
        table, hl, free = A.host_state()
        assert table.tolist() == A.model.page_table() and hl.tolist() == A.model.seq_lens
        assert free.tolist() == A.model.free
        d_table, d_lens = _device_mirrors(gu, A)
        assert d_table == table.tolist() and d_lens == hl.tolist()
        for b, n in zip(ids, (30, 1, 17)):
            L = int(lens[b])
            ko = torch.zeros(n, cfg.n_kv_heads, cfg.head_dim, dtype=ks[0].dtype, device=gu.DEV)
            vo = torch.zeros_like(ko)
            rb.rlhf_kv_arena_gather(A.handle, b, L, n, ko, vo)
            torch.cuda.synchronize()
            assert _bits_differ(ko, extra_k[b][:n]) == 0 and _bits_differ(vo, extra_v[b][:n]) == 0
        ko = torch.zeros(12, cfg.n_kv_heads, cfg.head_dim, dtype=ks[0].dtype, device=gu.DEV)
        vo = torch.zeros_like(ko)
        rb.rlhf_kv_arena_gather(A.handle, 2, int(lens[2]), 12, ko, vo)
        torch.cuda.synchronize()
        assert _bits_differ(ko, extra_k[2][:12]) == 0 and _bits_differ(vo, extra_v[2][:12]) == 0
    finally:
        A.close()


@pytest.mark.parametrize("dtype,head_dim", [("bf16", 128), ("f16", 64)])
def test_arena_appends_that_mix_edge_tokens_and_whole_pages(gu, dtype, head_dim):
    """Calls whose tokens start or end inside a page and cover whole pages in
    between (the append writes whole pages and edge tokens with different
    kernels): every row read back must be the row that went in."""
    cfg = wl.small_variant(wl.config(3), batch=4, n_q_heads=6, n_kv_heads=3, head_dim=head_dim, kv_dtype=dtype)
    calls = [([0, 1, 2, 3], [5, 16, 0, 33]), ([1, 0, 3], [40, 59, 15]), ([2, 0], [100, 1]), ([3, 2, 1], [16, 12, 7])]
    total = np.zeros(4, dtype=np.int64)
    for ids, ns in calls:
        total[ids] += ns
    _, ks, vs = wl.qkv(cfg, total, device=gu.DEV)
    n_pages = int(((total + P - 1) // P).sum()) + 5
    order = np.random.default_rng(7).permutation(n_pages).astype(np.int32)
    mpps = int((total.max() + P - 1) // P)
    arena = rb.rlhf_kv_arena_create(max_seqs=4, n_kv_heads=3, head_dim=head_dim, n_pages=n_pages,
                                    max_pages_per_seq=mpps, kv_dtype=wl.DTYPE_CODE[dtype], initial_free_order=order)
    try:
        done = np.zeros(4, dtype=np.int64)
        for ids, ns in calls:
            k_new = torch.cat([ks[b][done[b]:done[b] + n] for b, n in zip(ids, ns)]).contiguous()
            v_new = torch.cat([vs[b][done[b]:done[b] + n] for b, n in zip(ids, ns)]).contiguous()
            rb.rlhf_kv_arena_append(arena, ids, ns, k_new, v_new)
            for b, n in zip(ids, ns):
                done[b] += n
        for b in range(4):
            ko, vo = torch.zeros_like(ks[b]), torch.zeros_like(vs[b])
            rb.rlhf_kv_arena_gather(arena, b, 0, int(total[b]), ko, vo)
            torch.cuda.synchronize()
            assert torch.equal(ko.view(torch.int16), ks[b].view(torch.int16)), b
            assert torch.equal(vo.view(torch.int16), vs[b].view(torch.int16)), b
    finally:
        rb.rlhf_kv_arena_destroy(arena)


def test_arena_reset_between_two_generations(gu, oracle):
    """The phase boundary of the paper's pipeline: a generation fills the arena,
    reset returns every page in the initial order, and the next generation's
    sequences (other lengths) see none of the old state on the device."""
    cfg = wl.small_variant(wl.config(5), batch=5, n_q_heads=8, n_kv_heads=2, len_lo=20, len_hi=200)
    lens1 = wl.seq_lengths(cfg)
    q, ks, vs = wl.qkv(cfg, lens1, device=gu.DEV)
    A = gu.FilledArena(cfg, lens1, ks, vs, slack_pages=9)
    try:
        reserved = rb.rlhf_kv_arena_stats(A.handle)["reserved_bytes"]
        rb.rlhf_kv_arena_reset(A.handle)
        A.model.reset()
        st = rb.rlhf_kv_arena_stats(A.handle)
        assert st["pages_in_use"] == 0 and st["allocated_bytes"] == 0 and st["reserved_bytes"] == reserved
        table, hl, free = A.host_state()
        assert (table == -1).all() and not hl.any() and free.tolist() == A.model.free == A.order.tolist()
        lens2 = np.array([33, 0, 150, 16, 1], dtype=np.int32)       # fits: every sequence shorter than len_hi
        q2, ks2, vs2 = wl.qkv(cfg, lens2, device=gu.DEV, seed=cfg.seed + 1)
        ids = [4, 2, 0, 3]
        rb.rlhf_kv_arena_append(A.handle, ids, [int(lens2[b]) for b in ids],
                                torch.cat([ks2[b] for b in ids]).contiguous(), torch.cat([vs2[b] for b in ids]).contiguous())
        A.model.append(ids, [int(lens2[b]) for b in ids])
        torch.cuda.synchronize()
        table, hl, free = A.host_state()
        assert table.tolist() == A.model.page_table() and hl.tolist() == lens2.tolist() and free.tolist() == A.model.free
        _, _, d_table, d_lens = A.views()
        import ctypes
        hip = ctypes.CDLL("libamdhip64.so")
        dev_table = torch.empty(cfg.batch * A.mpps, dtype=torch.int32, device=gu.DEV)
        dev_lens = torch.empty(cfg.batch, dtype=torch.int32, device=gu.DEV)
        assert hip.hipMemcpy(ctypes.c_void_p(dev_table.data_ptr()), ctypes.c_void_p(d_table),
                             ctypes.c_size_t(dev_table.numel() * 4), 3) == 0
        assert hip.hipMemcpy(ctypes.c_void_p(dev_lens.data_ptr()), ctypes.c_void_p(d_lens),
                             ctypes.c_size_t(dev_lens.numel() * 4), 3) == 0
        assert np.array_equal(dev_table.cpu().numpy().reshape(cfg.batch, A.mpps), table)
        assert np.array_equal(dev_lens.cpu().numpy(), lens2)
        expect = gu.oracle_attention(oracle, cfg, q2, ks2, vs2, table, lens2, A.n_pages)
        out = gu.run_attention(cfg, A, q2, out_dtype=rb.RLHF_F32).cpu().numpy().astype(np.float64)
        assert np.abs(out - expect).max() <= ATTN_TOL
        assert not out[1].any()                                      # the empty sequence
    finally:
        A.close()


def test_arena_with_a_hundred_thousand_sequences(gu):
    """Descriptor lists of 100,000 entries through the one-launch decode step,
    through the general path (edge tokens and whole pages in one call) and
    through a step again; bookkeeping against the Python model, rows read back
    from sampled sequences and the device mirrors against the host's."""
    from oracle import ArenaModel
    S, H, D = 100_000, 2, 64
    rng = np.random.default_rng(99)
    grow = rng.integers(0, 40, S).astype(np.int32)          # tokens of the middle call; a third stay away
    grow[rng.random(S) < 0.33] = 0
    n_pages = int(((2 + grow.astype(np.int64) + P - 1) // P).sum()) + 7
    mpps = 3
    order = rng.permutation(n_pages).astype(np.int32)
    arena = rb.rlhf_kv_arena_create(max_seqs=S, n_kv_heads=H, head_dim=D, n_pages=n_pages, max_pages_per_seq=mpps,
                                    kv_dtype=wl.DTYPE_CODE["f16"], initial_free_order=order)
    model = ArenaModel(S, H, D, P, n_pages, mpps, initial_free_order=order)
    try:
        g = torch.Generator(device=gu.DEV)
        g.manual_seed(5)
        calls = [(np.arange(S, dtype=np.int32), np.ones(S, dtype=np.int32)),
                 (np.nonzero(grow)[0].astype(np.int32)[::-1].copy(), grow[np.nonzero(grow)[0]][::-1].copy()),
                 (np.arange(S, dtype=np.int32), np.ones(S, dtype=np.int32))]
        rows_k = [[] for _ in range(S)]
        rows_v = [[] for _ in range(S)]
        watch = set(rng.choice(S, 60, replace=False).tolist()) | {0, S - 1}
        for ids, cnt in calls:
            total = int(cnt.sum())
            _say(f"append of {total} tokens to {len(ids)} sequences")
            k_new = torch.randn(total, H, D, generator=g, device=gu.DEV).to(torch.float16)
            v_new = torch.randn(total, H, D, generator=g, device=gu.DEV).to(torch.float16)
            rb.rlhf_kv_arena_append(arena, ids, cnt, k_new, v_new)
            model.append(ids.tolist(), cnt.tolist())
            off = np.concatenate([[0], np.cumsum(cnt)])
            for i, b in enumerate(ids.tolist()):
                if b in watch:
                    rows_k[b].append(k_new[off[i]:off[i + 1]])
                    rows_v[b].append(v_new[off[i]:off[i + 1]])
        torch.cuda.synchronize()
        table, hl, free = rb.rlhf_kv_arena_host_state(arena, S, mpps)
        assert hl.tolist() == model.seq_lens == (2 + grow).tolist()
        assert table.tolist() == model.page_table() and free.tolist() == model.free
        _, _, d_table, d_lens = rb.rlhf_kv_arena_views(arena)
        import ctypes
        hip = ctypes.CDLL("libamdhip64.so")
        dev_table = torch.empty(S * mpps, dtype=torch.int32, device=gu.DEV)
        dev_lens = torch.empty(S, dtype=torch.int32, device=gu.DEV)
        assert hip.hipMemcpy(ctypes.c_void_p(dev_table.data_ptr()), ctypes.c_void_p(d_table),
                             ctypes.c_size_t(S * mpps * 4), 3) == 0
        assert hip.hipMemcpy(ctypes.c_void_p(dev_lens.data_ptr()), ctypes.c_void_p(d_lens), ctypes.c_size_t(S * 4), 3) == 0
        assert np.array_equal(dev_table.cpu().numpy().reshape(S, mpps), table)
        assert np.array_equal(dev_lens.cpu().numpy(), hl)
        for b in sorted(watch):
            ek, ev = torch.cat(rows_k[b]), torch.cat(rows_v[b])
            ko, vo = torch.zeros_like(ek), torch.zeros_like(ev)
            rb.rlhf_kv_arena_gather(arena, b, 0, int(hl[b]), ko, vo)
            torch.cuda.synchronize()
            assert torch.equal(ko.view(torch.int16), ek.view(torch.int16)), b
            assert torch.equal(vo.view(torch.int16), ev.view(torch.int16)), b
    finally:
        rb.rlhf_kv_arena_destroy(arena)


def test_arena_append_too_large_for_one_launch_is_refused(gu):
    """The copy kernels take one wavefront per (token, head), four to a
    workgroup of 256 lanes; past 2^32 lanes a launch's size no longer fits the
    runtime's 32 bits.  Such a call is refused before the bookkeeping moves."""
    heads = 32
    arena = rb.rlhf_kv_arena_create(max_seqs=2, n_kv_heads=heads, head_dim=64, n_pages=8, max_pages_per_seq=4,
                                    kv_dtype=wl.DTYPE_CODE["bf16"])
    try:
        dummy = torch.zeros(P, heads, 64, dtype=torch.bfloat16, device=gu.DEV)
        rb.rlhf_kv_arena_append(arena, [1], [P], dummy, dummy)
        before = rb.rlhf_kv_arena_stats(arena)
        with pytest.raises(rb.RlhfError) as e:
            rb.rlhf_kv_arena_append(arena, [0], [1 << 21], dummy, dummy)     # 2^21 tokens x 32 heads / 4 = 2^24
        assert e.value.status == rb.RLHF_ERR_UNSUPPORTED
        assert rb.rlhf_kv_arena_stats(arena) == before
        rb.rlhf_kv_arena_append(arena, [0], [3], dummy, dummy)              # the arena still works
        ko, vo = torch.ones_like(dummy[:3]), torch.ones_like(dummy[:3])
        rb.rlhf_kv_arena_gather(arena, 0, 0, 3, ko, vo)
        torch.cuda.synchronize()
        assert not ko.any() and not vo.any()
    finally:
        rb.rlhf_kv_arena_destroy(arena)


# -------------------------------------------------------------- attention ----
SMALL_ATTN = [
    # (config index, overrides) -- shapes span several pages, chunks and a ragged tail
    (1, dict()),                                                        # full config 1
    (2, dict(batch=3)),
    (3, dict(batch=2, len_lo=500, len_hi=1024)),
    (4, dict(batch=2, n_q_heads=4, n_kv_heads=4, len_lo=1000, len_hi=2048)),
    (5, dict(batch=2, n_q_heads=16, n_kv_heads=2, len_lo=2000, len_hi=4096)),
    (5, dict(batch=3, n_q_heads=8, n_kv_heads=2, head_dim=64, len_lo=1, len_hi=300)),
    (1, dict(batch=3, n_q_heads=6, n_kv_heads=2, head_dim=128, len_lo=1, len_hi=70)),
    (2, dict(batch=3, n_q_heads=8, n_kv_heads=4, len_lo=100, len_hi=400)),            # group of 2
    (3, dict(batch=2, n_q_heads=48, n_kv_heads=2, len_lo=30, len_hi=900)),            # group of 24 > 16
    (1, dict(batch=2, n_q_heads=32, n_kv_heads=2, len_lo=200, len_hi=700)),           # f16, group of 16
    # long contexts: tens of thousands of pages per sequence, far more page steps than wavefronts
    (2, dict(batch=2, n_q_heads=2, n_kv_heads=2, len_lo=150000, len_hi=300000)),
    (5, dict(batch=1, n_q_heads=8, n_kv_heads=1, len_lo=200003, len_hi=200003)),
]


@pytest.mark.parametrize("cfg_index,over", SMALL_ATTN)
def test_attention_matches_oracle(gu, oracle, cfg_index, over):
    cfg = wl.small_variant(wl.config(cfg_index), **over)
    lens = wl.seq_lengths(cfg)
    _say(f"attention cfg{cfg_index} {over} lens={lens.tolist()}")
    q, ks, vs = wl.qkv(cfg, lens, device=gu.DEV)
    A = gu.FilledArena(cfg, lens, ks, vs)
    try:
        table, hl, _ = A.host_state()
        assert table.tolist() == A.model.page_table() and hl.tolist() == lens.tolist()
        expect = gu.oracle_attention(oracle, cfg, q, ks, vs, table, lens, A.n_pages)
        dev32 = gu.run_attention(cfg, A, q, out_dtype=rb.RLHF_F32)
        dev16 = gu.run_attention(cfg, A, q)
        # the 16-bit output is the fp32 output rounded to nearest even, element for element
        assert torch.equal(dev32.to(dev16.dtype).view(torch.int16), dev16.view(torch.int16))
        out32 = dev32.cpu().numpy().astype(np.float64)
        err32 = np.abs(out32 - expect).max()
        out16 = dev16.float().cpu().numpy().astype(np.float64)
        err16 = np.abs(out16 - expect).max()
        _say(f"  max-abs err: f32 out {err32:.3e}, {cfg.kv_dtype} out {err16:.3e}")
        assert err32 <= ATTN_TOL
        if cfg.len_lo >= 256 or cfg.kv_dtype == "f16":
            assert err16 <= ATTN_TOL
        else:   # short caches with unit-variance values: half an ulp of the 16-bit output itself
            ulp = np.abs(expect).max() * 2.0 ** -8
            assert err16 <= ATTN_TOL + ulp
        # a tighter launch bound must not change anything
        out_b = gu.run_attention(cfg, A, q, out_dtype=rb.RLHF_F32, max_seq_len=int(lens.max()))
        assert np.abs(out_b.cpu().numpy() - expect).max() <= ATTN_TOL
    finally:
        A.close()


def test_attention_degenerate_lengths_and_scale(gu, oracle):
    cfg = wl.small_variant(wl.config(3), batch=6, n_q_heads=4, n_kv_heads=2, len_lo=0, len_hi=40)
    lens = np.array([1, 0, 16, 17, 2, 40], dtype=np.int32)
    q, ks, vs = wl.qkv(cfg, lens, device=gu.DEV)
    A = gu.FilledArena(cfg, lens, ks, vs)
    try:
        table, _, _ = A.host_state()
        expect = gu.oracle_attention(oracle, cfg, q, ks, vs, table, lens, A.n_pages)
        out = gu.run_attention(cfg, A, q, out_dtype=rb.RLHF_F32).cpu().numpy().astype(np.float64)
        assert np.isfinite(out).all()
        assert (out[1] == 0).all()                                   # empty cache -> zeros
        for h in range(4):                                           # one cached token -> its V row exactly
            assert np.array_equal(out[0, h], vs[0][0, h // 2].double().cpu().numpy())
        assert np.abs(out - expect).max() <= ATTN_TOL
        out16 = gu.run_attention(cfg, A, q)
        assert torch.equal(out16[0, 3].view(torch.int16), vs[0][0, 1].view(torch.int16))
        # explicit softmax scale
        expect_s = gu.oracle_attention(oracle, cfg, q, ks, vs, table, lens, A.n_pages, scale=0.31)
        out_s = gu.run_attention(cfg, A, q, out_dtype=rb.RLHF_F32, scale=0.31).cpu().numpy()
        assert np.abs(out_s - expect_s).max() <= ATTN_TOL
        assert np.abs(expect_s - expect).max() > 10 * ATTN_TOL       # the scale really matters here
    finally:
        A.close()


@pytest.mark.parametrize("heads", [(2, 2), (8, 2)])
def test_attention_many_sequences_most_of_them_empty(gu, oracle, heads):
    """More sequences than a workgroup has lanes (several lengths per lane in the
    page-count prefix), two thirds of them without a single cached token, runs of
    empty ones at both ends."""
    hq, hkv = heads
    cfg = wl.small_variant(wl.config(2), batch=700, n_q_heads=hq, n_kv_heads=hkv, len_lo=0, len_hi=40)
    rng = np.random.default_rng(700 + hq)
    lens = rng.integers(1, 41, cfg.batch).astype(np.int32)
    lens[rng.random(cfg.batch) < 0.66] = 0
    lens[:9] = 0
    lens[-5:] = 0
    q, ks, vs = wl.qkv(cfg, lens, device=gu.DEV)
    A = gu.FilledArena(cfg, lens, ks, vs)
    try:
        table, hl, _ = A.host_state()
        assert hl.tolist() == lens.tolist()
        expect = gu.oracle_attention(oracle, cfg, q, ks, vs, table, lens, A.n_pages)
        out = gu.run_attention(cfg, A, q, out_dtype=rb.RLHF_F32).cpu().numpy().astype(np.float64)
        assert np.isfinite(out).all()
        assert (out[lens == 0] == 0).all()
        assert np.abs(out - expect).max() <= ATTN_TOL
    finally:
        A.close()


def test_attention_at_the_largest_batch_one_call_takes(gu, oracle):
    """8192 sequences (the page-count prefix of a call lives in LDS and is sized
    for that many), short ragged caches, grouped heads; one more is refused."""
    cfg = wl.small_variant(wl.config(2), batch=8192, n_q_heads=2, n_kv_heads=1, len_lo=0, len_hi=20)
    rng = np.random.default_rng(8192)
    lens = rng.integers(0, 21, cfg.batch).astype(np.int32)
    q, ks, vs = wl.qkv(cfg, lens, device=gu.DEV)
    A = gu.FilledArena(cfg, lens, ks, vs)
    try:
        table, hl, _ = A.host_state()
        assert hl.tolist() == lens.tolist()
        expect = gu.oracle_attention(oracle, cfg, q, ks, vs, table, lens, A.n_pages)
        out = gu.run_attention(cfg, A, q, out_dtype=rb.RLHF_F32).cpu().numpy().astype(np.float64)
        assert (out[lens == 0] == 0).all()
        assert np.abs(out - expect).max() <= ATTN_TOL
    finally:
        A.close()
    too_many = rb.attn_params(8193, 2, 1, 64, 2, rb.RLHF_BF16)
    with pytest.raises(rb.RlhfError) as e:
        rb.rlhf_decode_attention_workspace_bytes(too_many)
    assert e.value.status == rb.RLHF_ERR_UNSUPPORTED


def test_attention_is_bit_identical_under_page_permutation(gu):
    base = wl.small_variant(wl.config(3), batch=4, n_q_heads=8, n_kv_heads=8, len_lo=100, len_hi=700)
    lens = wl.seq_lengths(base)
    q, ks, vs = wl.qkv(base, lens, device=gu.DEV)
    outs = []
    for shuffled in (False, True):
        cfg = wl.small_variant(base, shuffled_pages=shuffled)
        A = gu.FilledArena(cfg, lens, ks, vs, slack_pages=11)
        try:
            outs.append(gu.run_attention(cfg, A, q, out_dtype=rb.RLHF_F32))
            if shuffled:
                table, _, _ = A.host_state()
                assert table[0, :3].tolist() != [0, 1, 2]
        finally:
            A.close()
    assert torch.equal(outs[0].view(torch.int32), outs[1].view(torch.int32))


@pytest.mark.parametrize("cfg_index", [1, 2, 3, 4, 5])
def test_attention_full_size_every_element(gu, oracle, cfg_index):
    """The benchmark's launch configuration at the full shape; the oracle
    computes every sequence and the maximum error is taken over all elements."""
    cfg = wl.config(cfg_index)
    lens = wl.seq_lengths(cfg)
    _say(f"attention full cfg{cfg_index}: B={cfg.batch} tokens={int(lens.sum())}")
    q, ks, vs = wl.qkv(cfg, lens, device=gu.DEV)
    A = gu.FilledArena(cfg, lens, ks, vs)
    try:
        table, hl, free = A.host_state()
        assert table.tolist() == A.model.page_table()
        assert hl.tolist() == lens.tolist() and free.tolist() == A.model.free
        expect = gu.oracle_attention(oracle, cfg, q, ks, vs, table, lens, A.n_pages)
        assert expect.shape == (cfg.batch, cfg.n_q_heads, cfg.head_dim)
        out = gu.run_attention(cfg, A, q, out_dtype=rb.RLHF_F32, max_seq_len=cfg.len_hi)
        assert torch.isfinite(out).all()
        err = np.abs(out.cpu().numpy().astype(np.float64) - expect).max()
        out16 = gu.run_attention(cfg, A, q, max_seq_len=cfg.len_hi)
        err16 = np.abs(out16.float().cpu().numpy().astype(np.float64) - expect).max()
        _say(f"  all {expect.size} elements: max-abs err f32 out {err:.3e}, 16-bit out {err16:.3e}")
        assert err <= ATTN_TOL
        if cfg.len_lo >= 256 or cfg.kv_dtype == "f16":
            assert err16 <= ATTN_TOL
        else:   # caches of a few tokens: half an ulp of the 16-bit output itself
            assert err16 <= ATTN_TOL + np.abs(expect).max() * 2.0 ** -8
        # property that holds at any size: every output inside the range of the values
        G = cfg.n_q_heads // cfg.n_kv_heads
        for b in (int(lens.argmin()), int(lens.argmax())):
            vmin = vs[b].float().amin(0)
            vmax = vs[b].float().amax(0)
            o = out[b].view(cfg.n_kv_heads, G, cfg.head_dim)
            assert (o >= vmin[:, None, :] - 1e-5).all() and (o <= vmax[:, None, :] + 1e-5).all()
    finally:
        A.close()


ONE_LAUNCH_SHAPES = [
    # one head per KV head and enough (sequence, head) units: a single launch when run eagerly
    (2, dict(batch=8, len_lo=0, len_hi=700)),                                   # D=64
    (3, dict(batch=8, n_q_heads=40, n_kv_heads=40, len_lo=1, len_hi=300)),      # D=128
    (1, dict(batch=30, n_q_heads=12, n_kv_heads=12, len_lo=0, len_hi=500)),     # f16
    (1, dict(batch=4, n_q_heads=12, n_kv_heads=12, len_lo=1, len_hi=512)),      # 48 units of at most 6 MB in all:
                                                                                # cut into few ranges, one launch
    # grouped heads: always the split kernel and the merge kernel
    (5, dict(batch=32, n_q_heads=16, n_kv_heads=8, len_lo=0, len_hi=900)),      # groups of 2
    (5, dict(batch=24, n_q_heads=64, n_kv_heads=8, len_lo=100, len_hi=1300)),   # groups of 8
    (1, dict(batch=40, n_q_heads=96, n_kv_heads=4, head_dim=128, len_lo=1, len_hi=200)),   # f16, groups of 24
]


@pytest.mark.parametrize("cfg_index,over", ONE_LAUNCH_SHAPES)
def test_attention_in_one_launch_and_in_two_is_the_same_bit_for_bit(gu, oracle, cfg_index, over):
    """Run eagerly, a call with one query head per KV head is one kernel launch (the
    wavefront that completes a unit merges it); recorded into a graph, and with
    grouped heads, it is the split kernel and the merge kernel.  Both merge a
    unit's partials in range order through the same arithmetic, so the outputs
    must be identical bit for bit, and both must match the oracle.  Which form
    ran is read off the workspace: only the two-launch form leaves the page-count
    prefix for its merge kernel there."""
    cfg = wl.small_variant(wl.config(cfg_index), **over)
    lens = wl.seq_lengths(cfg)
    if cfg.len_lo == 0:
        lens[1] = 0
        lens[-1] = 0
    _say(f"one/two launches cfg{cfg_index} {over} lens={lens.tolist()[:12]}...")
    q, ks, vs = wl.qkv(cfg, lens, device=gu.DEV)
    A = gu.FilledArena(cfg, lens, ks, vs)
    try:
        k, v, table, dl = A.views()
        host_table, _, _ = A.host_state()
        expect = gu.oracle_attention(oracle, cfg, q, ks, vs, host_table, lens, A.n_pages)
        for out_dtype in (rb.RLHF_F32, None):
            params = rb.attn_params(cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, A.mpps,
                                    wl.DTYPE_CODE[cfg.kv_dtype], out_dtype=out_dtype)
            nws = rb.rlhf_decode_attention_workspace_bytes(params)
            odt = torch.float32 if out_dtype == rb.RLHF_F32 else q.dtype
            prefix_words = cfg.batch + 1

            def fresh():
                ws = torch.full((nws,), 0xFF, dtype=torch.uint8, device=gu.DEV)
                out = torch.full((cfg.batch, cfg.n_q_heads, cfg.head_dim), float("nan"), dtype=odt, device=gu.DEV)
                return ws, out

            ws1, out1 = fresh()
            rb.rlhf_decode_attention(params, q, k, v, table, dl, out1, ws1)
            torch.cuda.synchronize()
            if cfg.n_q_heads == cfg.n_kv_heads:
                assert (ws1[:4 * prefix_words] == 0xFF).all(), "the eager call was expected to be one launch"
            else:
                assert not (ws1[:4 * prefix_words] == 0xFF).all(), "grouped heads were expected to take two launches"
            ws2, out2 = fresh()
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                rb.rlhf_decode_attention(params, q, k, v, table, dl, out2, ws2, stream=side)
            for rep in range(2):
                out2.fill_(float("nan"))
                torch.cuda.synchronize()
                graph.replay()
                torch.cuda.synchronize()
                pages = ws2[:4 * prefix_words].view(torch.int32)
                assert int(pages[-1]) == int(((lens.astype(np.int64) + 15) // 16).sum()), "two launches expected"
                assert _bits_differ(out1, out2) == 0, rep
            err = np.abs(out1.float().cpu().numpy().astype(np.float64) - expect).max()
            _say(f"  out {odt}: max-abs err {err:.3e}")
            assert (out1[lens == 0] == 0).all()
            if out_dtype == rb.RLHF_F32:
                assert err <= ATTN_TOL
            else:
                assert err <= ATTN_TOL + np.abs(expect).max() * 2.0 ** -8
    finally:
        A.close()


def test_attention_calls_in_one_launch_from_several_streams_at_once(gu):
    """The one-launch form keeps arrival counters in device memory of the
    library's, a set per calling stream.  Four host threads, each on a stream of
    its own with its own outputs and workspace, call twenty times each at the
    same time, cycling through four queries; every result must equal the one the
    same query gives alone."""
    import threading
    cfg = wl.small_variant(wl.config(2), batch=16, len_lo=100, len_hi=900)
    lens = wl.seq_lengths(cfg)
    q, ks, vs = wl.qkv(cfg, lens, device=gu.DEV)
    A = gu.FilledArena(cfg, lens, ks, vs)
    try:
        k, v, table, dl = A.views()
        params = rb.attn_params(cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, A.mpps,
                                wl.DTYPE_CODE[cfg.kv_dtype], out_dtype=rb.RLHF_F32)
        nws = rb.rlhf_decode_attention_workspace_bytes(params)
        qs = [(q.float() * (1.0 - 0.2 * i) + 0.05 * i).to(q.dtype) for i in range(4)]
        alone = []
        for qi in qs:
            ws = torch.full((nws,), 0xFF, dtype=torch.uint8, device=gu.DEV)
            out = torch.empty(cfg.batch, cfg.n_q_heads, cfg.head_dim, dtype=torch.float32, device=gu.DEV)
            rb.rlhf_decode_attention(params, qi, k, v, table, dl, out, ws)
            torch.cuda.synchronize()
            assert (ws[:4 * (cfg.batch + 1)] == 0xFF).all(), "expected the one-launch form"
            alone.append(out)
        assert not torch.equal(alone[0], alone[1])
        results, errors = {}, []

        def worker(i):
            try:
                stream = torch.cuda.Stream()
                ws = torch.full((nws,), 0xFF, dtype=torch.uint8, device=gu.DEV)
                outs = [torch.empty_like(alone[0]) for _ in range(20)]
                torch.cuda.synchronize()
                for j, o in enumerate(outs):    # two queries in turn through one workspace: a partial
                    rb.rlhf_decode_attention(params, qs[(i + j) % 4], k, v, table, dl, o, ws, stream=stream)
                stream.synchronize()            # left over from the call before must never be read
                results[i] = outs
            except Exception as e:      # reported by the main thread
                errors.append(e)

        threads = [threading.Thread(target=worker, args=(i,)) for i in range(4)]
        for t in threads:
            t.start()
        for t in threads:
            t.join()
        assert not errors, errors
        for i in range(4):
            for j, o in enumerate(results[i]):
                assert _bits_differ(o, alone[(i + j) % 4]) == 0, (i, j)
    finally:
        A.close()


# ------------------------------------------------------------- logprob/KL ----
SMALL_LOGITS = [
    (1, 96), (2, 64), (3, 64), (5, 24),
]


@pytest.mark.parametrize("cfg_index,n", SMALL_LOGITS)
def test_logprobs_kl_match_oracle(gu, oracle, cfg_index, n):
    cfg = wl.config(cfg_index)
    actor, ref = wl.logits(cfg, n_positions=n, device=gu.DEV)
    tok = wl.tokens(cfg, n_positions=n)
    _say(f"logprob cfg{cfg_index} n={n} V={cfg.vocab} {cfg.logits_dtype}")
    logp, kl = gu.run_logprobs(actor, ref, tok)
    el, ek = oracle.token_logprobs_kl(wl.to_storage(actor), wl.to_storage(ref), tok,
                                      wl.DTYPE_CODE[cfg.logits_dtype])
    _say(f"  max-abs err logp {np.abs(logp - el).max():.3e} kl {np.abs(kl - ek).max():.3e}")
    assert np.abs(logp - el).max() <= LOGP_TOL
    assert np.abs(kl - ek).max() <= LOGP_TOL
    assert (kl > -1e-5).all()


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("vocab,stride,offset", [(1003, 1003, 0), (4099, 4104, 0), (7, 8, 0), (2048, 2048, 1),
                                                  (1, 1, 0), (50272, 50272, 0)])
def test_logprobs_ragged_vocab_strides_and_alignment(gu, oracle, dtype, vocab, stride, offset):
    """Tail elements past the last 16-byte vector, padded rows, rows that do not
    start 16-byte aligned (element-wise path), one-element vocabularies."""
    tdt = wl.torch_dtype(dtype)
    n = 9
    g = torch.Generator(device=gu.DEV)
    g.manual_seed(vocab * 31 + stride)
    buf_a = (torch.randn(n * stride + 8, generator=g, device=gu.DEV) * 3).to(tdt)
    buf_r = (torch.randn(n * stride + 8, generator=g, device=gu.DEV) * 3).to(tdt)
    actor = buf_a[offset:offset + n * stride].view(n, stride)
    ref = buf_r[offset:offset + n * stride].view(n, stride)
    tok = np.random.default_rng(vocab).integers(0, vocab, n).astype(np.int32)
    logp, kl = gu.run_logprobs(actor, ref, tok, vocab=vocab, stride=stride)
    el, ek = oracle.token_logprobs_kl(wl.to_storage(actor), wl.to_storage(ref), tok, wl.DTYPE_CODE[dtype],
                                      vocab=vocab)
    assert np.abs(logp - el).max() <= LOGP_TOL
    assert np.abs(kl - ek).max() <= LOGP_TOL


def test_logprobs_special_rows(gu, oracle):
    """Identical rows (KL exactly 0), padded positions, -inf logits, a late
    maximum far above the running reference, large common offsets."""
    V, n = 5000, 8
    g = torch.Generator(device=gu.DEV)
    g.manual_seed(7)
    actor = (torch.randn(n, V, generator=g, device=gu.DEV) * 3).to(torch.bfloat16)
    ref = (torch.randn(n, V, generator=g, device=gu.DEV) * 3).to(torch.bfloat16)
    ref[0] = actor[0]                                   # identical
    actor[1, 100:2000] = float("-inf")                  # masked actor logits
    ref[2, 5:50] = float("-inf")                        # reference forbids tokens the actor allows
    actor[3, 4000] = 90.0                               # late spike, > lift threshold above the rest
    ref[3, 17] = 70.0
    actor[4] += 300.0                                   # large common offset
    ref[4] -= 300.0
    actor[5, :] = float("-inf")
    actor[5, 7] = 0.0                                   # one-hot actor
    tok = np.array([3, 5, 1000, 4000, 9, 7, -1, V], dtype=np.int32)
    logp, kl = gu.run_logprobs(actor, ref, tok)
    el, ek = oracle.token_logprobs_kl(wl.to_storage(actor), wl.to_storage(ref), tok, rb.RLHF_BF16)
    assert kl[0] == 0.0
    assert logp[6] == 0 and kl[6] == 0 and logp[7] == 0 and kl[7] == 0
    assert np.isinf(ek[2]) and np.isinf(kl[2]) and kl[2] > 0
    fin = [0, 1, 3, 4, 5, 6, 7]
    assert np.isfinite(kl[fin]).all() and np.isfinite(logp).all()
    assert np.abs(logp - el).max() <= LOGP_TOL
    assert np.abs(kl[fin] - ek[fin]).max() <= LOGP_TOL * max(1.0, np.abs(ek[fin]).max() / 100)
    assert abs(logp[5]) <= 1e-6 and abs(logp[3]) <= 1e-3


def test_logprobs_of_large_constant_rows_and_a_nan_row(gu, oracle):
    """Logits of magnitude 1000 (the absolute error grows with the magnitude,
    fp32 rounding of the logits themselves: 1e-3 still holds here); a NaN logit
    marks its row."""
    V = 3001
    for tdt, big in ((torch.float32, 1000.0), (torch.bfloat16, 1024.0)):
        actor = torch.zeros(5, V, dtype=torch.float32, device=gu.DEV)
        actor[0] = -big                                     # constant, hugely negative: uniform
        actor[1] = big                                      # constant, hugely positive
        actor[2] = -big
        actor[2, 11] = big                                  # one entry towers over the rest
        actor[3] = torch.linspace(-1.0, 1.0, V, device=gu.DEV)
        actor[3, 5] = float("nan")
        actor[4] = torch.linspace(-5.0, 5.0, V, device=gu.DEV)
        actor = actor.to(tdt)
        ref = torch.zeros_like(actor)
        tok = np.array([7, 8, 11, 9, 3000], dtype=np.int32)
        logp, kl = gu.run_logprobs(actor, ref, tok)
        el, _ = oracle.token_logprobs_kl(wl.to_storage(actor), wl.to_storage(ref), tok, rb.dtype_code(tdt))
        assert np.isnan(logp[3]) and np.isnan(kl[3])
        ok = [0, 1, 2, 4]
        assert np.abs(logp[ok] - el[ok]).max() <= LOGP_TOL
        assert abs(logp[0] + np.log(V)) <= LOGP_TOL and abs(logp[2]) <= LOGP_TOL


def _full_size_rows(cfg):
    """Rows the oracle checks at the full shape: all of them, except for the
    largest configuration (67 GB of logits), where it is the first 256, the last
    256 and 1536 seeded rows in between."""
    n = cfg.n_positions
    if cfg.index != 5:
        return np.arange(n)
    rng = np.random.default_rng(cfg.seed)
    mid = 256 + rng.choice(n - 512, size=1536, replace=False)
    return np.sort(np.concatenate([np.arange(256), mid, np.arange(n - 256, n)]))


@pytest.mark.parametrize("cfg_index", [1, 2, 3, 4, 5])
def test_logprobs_full_size_every_row(gu, oracle, cfg_index):
    """The benchmark's launch at the full shape.  The oracle scores every row of
    configurations 1-4 (logits copied back in chunks of rows) and a fixed
    2048-row sample of configuration 5; the maximum error is over all of them."""
    cfg = wl.config(cfg_index)
    n = cfg.n_positions
    eb = 4 if cfg.logits_dtype == "f32" else 2
    _say(f"logprob full cfg{cfg_index}: N={n} V={cfg.vocab} bytes={2 * n * cfg.vocab * eb / 1e9:.1f} GB")
    actor, ref = wl.logits(cfg, device=gu.DEV)
    tok = wl.tokens(cfg)
    logp, kl = gu.run_logprobs(actor, ref, tok)
    assert np.isfinite(logp).all() and np.isfinite(kl).all()
    assert (logp < 0).all() and (kl > -1e-5).all()
    rows = _full_size_rows(cfg)
    assert rows.size == (2048 if cfg_index == 5 else n) and np.unique(rows).size == rows.size
    err_l = err_k = 0.0
    for c0 in range(0, rows.size, 2048):
        r = rows[c0:c0 + 2048]
        idx = torch.from_numpy(r).to(gu.DEV)
        el, ek = oracle.token_logprobs_kl(wl.to_storage(actor[idx]), wl.to_storage(ref[idx]), tok[r],
                                          wl.DTYPE_CODE[cfg.logits_dtype])
        err_l = max(err_l, np.abs(logp[r] - el).max())
        err_k = max(err_k, np.abs(kl[r] - ek).max())
    _say(f"  {rows.size} of {n} rows: max-abs err logp {err_l:.3e} kl {err_k:.3e}")
    assert err_l <= LOGP_TOL
    assert err_k <= LOGP_TOL


@pytest.mark.parametrize("cfg_index,n", [(1, 64), (3, 48), (5, 16)])
@pytest.mark.parametrize("penalty", [rb.RLHF_PENALTY_FULL_KL, rb.RLHF_PENALTY_SAMPLED])
def test_reward_shaping_matches_oracle(gu, oracle, cfg_index, n, penalty):
    """Reference log-prob and KL-penalised per-token reward from the same single
    pass; padded positions and terminal scores included."""
    cfg = wl.config(cfg_index)
    actor, ref = wl.logits(cfg, n_positions=n, device=gu.DEV)
    tok = wl.tokens(cfg, n_positions=n)
    tok[5] = -1
    rng = np.random.default_rng(cfg.seed)
    term = np.zeros(n, dtype=np.float32)
    term[[5, n // 2, n - 1]] = rng.standard_normal(3).astype(np.float32)
    d = lambda a: torch.from_numpy(a).to(gu.DEV)
    outs = [torch.full((n,), float("nan"), dtype=torch.float32, device=gu.DEV) for _ in range(4)]
    logp, kl, ref_logp, reward = outs
    rb.rlhf_token_logprobs_kl_rewards(actor, ref, d(tok), logp, kl, 0.15, penalty=penalty, ref_logp_out=ref_logp,
                                      reward_out=reward, terminal_scores=d(term))
    torch.cuda.synchronize()
    code = wl.DTYPE_CODE[cfg.logits_dtype]
    el, ek = oracle.token_logprobs_kl(wl.to_storage(actor), wl.to_storage(ref), tok, code)
    erl, erw = oracle.token_rewards(wl.to_storage(actor), wl.to_storage(ref), tok, code, 0.15,
                                    penalty == rb.RLHF_PENALTY_SAMPLED, terminal=term.astype(np.float64))
    got = [t.cpu().numpy().astype(np.float64) for t in outs]
    for name, g, e in zip(("logp", "kl", "ref_logp", "reward"), got, (el, ek, erl, erw)):
        err = np.abs(g - e).max()
        _say(f"  {name}: max-abs err {err:.3e}")
        assert err <= LOGP_TOL, name
    assert got[2][5] == 0 and got[3][5] == 0          # padded position: zeros, terminal score ignored
    # outputs that were not asked for are simply skipped
    logp2 = torch.empty_like(logp)
    kl2 = torch.empty_like(kl)
    rb.rlhf_token_logprobs_kl_rewards(actor, ref, d(tok), logp2, kl2, 0.15, penalty=penalty)
    torch.cuda.synchronize()
    assert torch.equal(logp2, logp) and torch.equal(kl2, kl)


def test_token_error_flag_tells_an_out_of_range_id_from_padding(gu):
    """A token id at or above the vocabulary is scored like padding (zeros), and
    the optional device flag becomes 1 and stays 1; negative ids (the padding
    convention) never set it.  Integer result: exact."""
    V, n = 3000, 6
    g = torch.Generator(device=gu.DEV)
    g.manual_seed(3)
    actor = (torch.randn(n, V, generator=g, device=gu.DEV) * 3).to(torch.bfloat16)
    ref = (torch.randn(n, V, generator=g, device=gu.DEV) * 3).to(torch.bfloat16)
    flag = torch.zeros(1, dtype=torch.int32, device=gu.DEV)
    logp = torch.empty(n, dtype=torch.float32, device=gu.DEV)
    kl = torch.empty_like(logp)

    def run(tok):
        t = torch.tensor(tok, dtype=torch.int32, device=gu.DEV)
        logp.fill_(float("nan"))
        rb.rlhf_token_logprobs_kl_rewards(actor, ref, t, logp, kl, 0.1, token_error_flag=flag)
        torch.cuda.synchronize()
        return int(flag.item())

    assert run([0, 5, -1, V - 1, -7, 17]) == 0                 # valid ids and padding only
    assert logp[2] == 0 and logp[4] == 0 and (logp[[0, 1, 3, 5]] < 0).all()
    assert run([0, 5, V, 2, 3, 4]) == 1                        # one id just past the vocabulary
    assert logp[2] == 0 and kl[2] == 0
    assert run([1, 2, 3, 4, 5, 6]) == 1                        # sticky: a clean call does not clear it
    flag.zero_()
    assert run([1, 2, 2 ** 31 - 1, 4, 5, 6]) == 1
    flag.zero_()
    assert run([1, 2, 3, 4, 5, 6]) == 0


# ---------------------------------------------------------------- sampling ----
def _check_sampling(gu, oracle, logits, temperature, seed, offset, vocab=None, stride=0, split=False):
    """The sampled decision is an argmax of fp32 scores on the GPU and of fp64
    scores in the oracle, so a near-tie may legitimately resolve differently: the
    GPU's token must reach the oracle's maximum perturbed score within 1e-3, and
    rows whose top two scores are further apart than that must agree exactly."""
    n = logits.shape[0]
    tok = torch.full((n,), -7, dtype=torch.int32, device=gu.DEV)
    logp = torch.full((n,), float("nan"), dtype=torch.float32, device=gu.DEV)
    if split:   # rows cut into segments; scratch poisoned so that a stale record shows
        v_eff = logits.shape[1] if vocab is None else vocab
        ws = torch.full((rb.rlhf_sample_tokens_workspace_bytes(n, v_eff),), 0xFF, dtype=torch.uint8,
                        device=gu.DEV)
        if vocab is None:
            rb.rlhf_sample_tokens_split(logits, tok, temperature, seed, ws, offset, logp_out=logp)
        else:
            rb.rlhf_sample_tokens_split(logits, tok, temperature, seed, ws, offset, logp_out=logp, n_rows=n,
                                        vocab=vocab, row_stride_elems=stride,
                                        logits_dtype=rb.dtype_code(logits.dtype))
    elif vocab is None:
        rb.rlhf_sample_tokens(logits, tok, temperature, seed, offset, logp_out=logp)
    else:
        rb.rlhf_sample_tokens(logits, tok, temperature, seed, offset, logp_out=logp, n_rows=n, vocab=vocab,
                              row_stride_elems=stride, logits_dtype=rb.dtype_code(logits.dtype))
    torch.cuda.synchronize()
    code = rb.dtype_code(logits.dtype)
    et, el, pert = oracle.sample_tokens(wl.to_storage(logits), code, temperature, seed, offset, vocab=vocab,
                                        return_perturbed=True)
    got = tok.cpu().numpy()
    V = pert.shape[1]
    assert ((got >= 0) & (got < V)).all()
    rows = np.arange(n)
    top = pert.max(axis=1)
    assert (pert[rows, got] >= top - 1e-3).all()
    second = np.partition(pert, V - 2, axis=1)[:, V - 2] if V > 1 else top - 1
    clear = top - second > 1e-3
    assert (got[clear] == et[clear]).all()
    agree = got == et
    x = logits.double().cpu().numpy()[:, :V] * (1.0 / temperature if temperature > 0 else 1.0)
    import scipy.special
    ref_logp = scipy.special.log_softmax(x, axis=1)[rows, got]       # log-prob of the token the GPU chose
    assert np.abs(logp.cpu().numpy() - ref_logp).max() <= LOGP_TOL
    assert np.abs(el[agree] - ref_logp[agree]).max() <= 1e-9
    return got, agree.mean(), clear.mean()


@pytest.mark.parametrize("cfg_index,n", [(1, 48), (2, 32), (5, 128), (3, 1100)])   # 1100 rows: the 256-lane variant
@pytest.mark.parametrize("temperature", [1.0, 0.7, 0.0])
def test_sampling_matches_oracle(gu, oracle, cfg_index, n, temperature):
    cfg = wl.config(cfg_index)
    actor, _ = wl.logits(cfg, n_positions=n, device=gu.DEV)
    got, agree, clear = _check_sampling(gu, oracle, actor, temperature, 0xC0FFEE1234, 17)
    _say(f"sampling cfg{cfg_index} T={temperature}: identical tokens {agree:.3f}, clear rows {clear:.3f}")
    assert agree >= 0.98
    if temperature > 0:
        got2, _, _ = _check_sampling(gu, oracle, actor, temperature, 0xC0FFEE1234, 18)
        assert (got != got2).mean() > 0.5                     # a new offset gives a new draw


@pytest.mark.parametrize("cfg_index,n", [(1, 4), (2, 16), (5, 128), (3, 300), (3, 600)])   # 600 rows: no split left
@pytest.mark.parametrize("temperature", [1.0, 0.0])
def test_sampling_split_rows_matches_oracle_and_the_unsplit_draw(gu, oracle, cfg_index, n, temperature):
    """Rows cut into segments (a decode step's few rows): same bar against the
    oracle, and token for token the draw of the unsplit call."""
    cfg = wl.config(cfg_index)
    actor, _ = wl.logits(cfg, n_positions=n, device=gu.DEV)
    got, agree, _ = _check_sampling(gu, oracle, actor, temperature, 0xC0FFEE1234, 17, split=True)
    assert agree >= 0.98
    tok = torch.empty(n, dtype=torch.int32, device=gu.DEV)
    logp = torch.empty(n, dtype=torch.float32, device=gu.DEV)
    rb.rlhf_sample_tokens(actor, tok, temperature, 0xC0FFEE1234, 17, logp_out=logp)
    torch.cuda.synchronize()
    assert (tok.cpu().numpy() == got).all()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("vocab,stride,offset_elems", [(70001, 70001, 0), (16384, 16392, 0), (65543, 65544, 1),
                                                        (5, 8, 0)])
def test_sampling_split_rows_ragged_vocab_strides_and_alignment(gu, oracle, dtype, vocab, stride, offset_elems):
    tdt = wl.torch_dtype(dtype)
    n = 3
    g = torch.Generator(device=gu.DEV)
    g.manual_seed(vocab * 17 + stride)
    buf = (torch.randn(n * stride + 8, generator=g, device=gu.DEV) * 3).to(tdt)
    logits = buf[offset_elems:offset_elems + n * stride].view(n, stride)
    for T in (0.0, 1.3):
        _check_sampling(gu, oracle, logits, T, 5, 2 ** 33 + 9, vocab=vocab, stride=stride, split=True)


@pytest.mark.parametrize("temperature", [1.0, 0.0])
def test_sampling_without_a_log_probability_draws_the_same_tokens(gu, temperature):
    """With logp_out NULL the kernels leave the sum of exponentials out; the
    draw itself must not change (plain, split and ragged scalar paths)."""
    cfg = wl.config(2)
    actor, _ = wl.logits(cfg, n_positions=40, device=gu.DEV)
    ws = torch.empty(rb.rlhf_sample_tokens_workspace_bytes(40, cfg.vocab), dtype=torch.uint8, device=gu.DEV)
    a, b, c, d = (torch.empty(40, dtype=torch.int32, device=gu.DEV) for _ in range(4))
    lp = torch.empty(40, dtype=torch.float32, device=gu.DEV)
    rb.rlhf_sample_tokens(actor, a, temperature, 99, 4, logp_out=lp)
    rb.rlhf_sample_tokens(actor, b, temperature, 99, 4)
    rb.rlhf_sample_tokens_split(actor, c, temperature, 99, ws, 4)
    ragged = actor[:, 3:3 + 30001]                      # misaligned rows: the scalar path
    rb.rlhf_sample_tokens(ragged, d, temperature, 99, 4, n_rows=40, vocab=30001, row_stride_elems=actor.stride(0),
                          logits_dtype=rb.dtype_code(actor.dtype))
    e = torch.empty_like(d)
    rb.rlhf_sample_tokens(ragged, e, temperature, 99, 4, logp_out=lp, n_rows=40, vocab=30001,
                          row_stride_elems=actor.stride(0), logits_dtype=rb.dtype_code(actor.dtype))
    torch.cuda.synchronize()
    assert torch.equal(a, b) and torch.equal(a, c) and torch.equal(d, e)


def test_sampling_split_rejects_a_short_workspace(gu):
    logits = torch.zeros(4, 65536, dtype=torch.bfloat16, device=gu.DEV)
    tok = torch.empty(4, dtype=torch.int32, device=gu.DEV)
    need = rb.rlhf_sample_tokens_workspace_bytes(4, 65536)
    assert need == 4 * 8 * 16
    ws = torch.empty(need - 16, dtype=torch.uint8, device=gu.DEV)
    with pytest.raises(rb.RlhfError):
        rb.rlhf_sample_tokens_split(logits, tok, 1.0, 1, ws)


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("vocab,stride,offset_elems", [(1003, 1003, 0), (4099, 4104, 0), (5, 8, 0), (2048, 2048, 1),
                                                        (1, 1, 0)])
def test_sampling_ragged_vocab_strides_and_alignment(gu, oracle, dtype, vocab, stride, offset_elems):
    tdt = wl.torch_dtype(dtype)
    n = 12
    g = torch.Generator(device=gu.DEV)
    g.manual_seed(vocab * 17 + stride)
    buf = (torch.randn(n * stride + 8, generator=g, device=gu.DEV) * 3).to(tdt)
    logits = buf[offset_elems:offset_elems + n * stride].view(n, stride)
    for T in (0.0, 1.3):
        _check_sampling(gu, oracle, logits, T, 5, 2 ** 33 + 9, vocab=vocab, stride=stride)


def _check_topk(gu, oracle, logits, temperature, top_k, seed, offset, vocab=None, stride=0):
    """Same bar as the plain draw, restricted to the oracle's survivors: the
    survivor set is decided by exact comparisons on both sides, so a token
    outside it is an error whatever the noise."""
    import scipy.special
    n = logits.shape[0]
    tok = torch.full((n,), -7, dtype=torch.int32, device=gu.DEV)
    logp = torch.full((n,), float("nan"), dtype=torch.float32, device=gu.DEV)
    if vocab is None:
        rb.rlhf_sample_tokens_topk(logits, tok, temperature, top_k, seed, offset, logp_out=logp)
    else:
        rb.rlhf_sample_tokens_topk(logits, tok, temperature, top_k, seed, offset, logp_out=logp, n_rows=n,
                                   vocab=vocab, row_stride_elems=stride, logits_dtype=rb.dtype_code(logits.dtype))
    torch.cuda.synchronize()
    code = rb.dtype_code(logits.dtype)
    et, el, tau, count, pert = oracle.sample_tokens_topk(wl.to_storage(logits), code, temperature, top_k, seed,
                                                         offset, vocab=vocab, return_perturbed=True)
    got = tok.cpu().numpy()
    V = pert.shape[1]
    assert ((got >= 0) & (got < V)).all()
    rows = np.arange(n)
    x = logits.double().cpu().numpy()[:, :V]
    assert (x[rows, got] >= tau).all(), "a removed entry was drawn"
    assert (count >= min(top_k, V)).all()
    top = pert.max(axis=1)
    assert (pert[rows, got] >= top - 1e-3).all()
    second = np.partition(pert, V - 2, axis=1)[:, V - 2] if V > 1 else top - 1
    clear = top - second > 1e-3
    assert (got[clear] == et[clear]).all()
    y = np.where(x >= tau[:, None], x * (1.0 / temperature if temperature > 0 else 1.0), -np.inf)
    ref_logp = scipy.special.log_softmax(y, axis=1)[rows, got]       # over the survivors, at the GPU's token
    assert np.abs(logp.cpu().numpy() - ref_logp).max() <= LOGP_TOL
    agree = got == et
    assert np.abs(logp.cpu().numpy()[agree] - el[agree]).max() <= LOGP_TOL
    return got, float(agree.mean()), count


@pytest.mark.parametrize("cfg_index,n", [(1, 16), (2, 64), (5, 128)])
@pytest.mark.parametrize("top_k", [1, 2, 50, 1000, 1024, 1025, 5000, 40000])
@pytest.mark.parametrize("temperature", [1.0, 0.7, 0.0])
def test_topk_sampling_matches_oracle(gu, oracle, cfg_index, n, top_k, temperature):
    """k from the argmax, through lists that fit the kernel's on-chip candidate
    store, to k beyond it (the search then ends on the row itself)."""
    cfg = wl.config(cfg_index)
    actor, _ = wl.logits(cfg, n_positions=n, device=gu.DEV)
    got, agree, count = _check_topk(gu, oracle, actor, temperature, top_k, 0xC0FFEE1234, 17)
    _say(f"top-{top_k} cfg{cfg_index} T={temperature}: identical tokens {agree:.3f}, survivors "
         f"{count.min()}..{count.max()}")
    assert agree >= 0.97
    x = actor.float().cpu().numpy()
    if top_k == 1:                         # only the row maximum (and what ties with it) is left
        assert (x[np.arange(n), got] == x.max(axis=1)).all()
    if temperature == 0.0:                 # greedy: the first index of the maximum
        assert (got == x.argmax(axis=1)).all()


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("vocab,stride,offset_elems", [(1003, 1003, 0), (4099, 4104, 0), (5, 8, 0), (2048, 2048, 1),
                                                        (1, 1, 0), (70001, 70001, 0), (65543, 65544, 1)])
def test_topk_sampling_ragged_vocab_strides_and_alignment(gu, oracle, dtype, vocab, stride, offset_elems):
    tdt = wl.torch_dtype(dtype)
    n = 6
    g = torch.Generator(device=gu.DEV)
    g.manual_seed(vocab * 17 + stride)
    buf = (torch.randn(n * stride + 8, generator=g, device=gu.DEV) * 3).to(tdt)
    logits = buf[offset_elems:offset_elems + n * stride].view(n, stride)
    for T, k in ((0.0, 3), (1.3, 1), (1.3, 7), (0.6, 900), (1.0, max(1, vocab - 1)), (1.0, vocab), (1.0, vocab + 5)):
        _check_topk(gu, oracle, logits, T, k, 5, 2 ** 33 + 9, vocab=vocab, stride=stride)


def test_topk_at_or_above_vocab_is_the_plain_draw(gu):
    cfg = wl.config(2)
    actor, _ = wl.logits(cfg, n_positions=32, device=gu.DEV)
    a = torch.empty(32, dtype=torch.int32, device=gu.DEV)
    b = torch.empty_like(a)
    la = torch.empty(32, dtype=torch.float32, device=gu.DEV)
    lb = torch.empty_like(la)
    rb.rlhf_sample_tokens(actor, a, 0.9, 77, 3, logp_out=la)
    for k in (cfg.vocab, cfg.vocab + 1, 2 ** 31 - 1):
        rb.rlhf_sample_tokens_topk(actor, b, 0.9, k, 77, 3, logp_out=lb)
        torch.cuda.synchronize()
        assert torch.equal(a, b) and torch.equal(la, lb)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_topk_ties_at_the_threshold_all_survive(gu, oracle, dtype):
    """Rows made of a few distinct values, so the k-th largest is tied many
    times over: a handful of ties, more ties than the kernel keeps on chip, a
    constant row, -0 against +0, and rows with -inf entries."""
    tdt = wl.torch_dtype(dtype)
    V = 30011
    g = torch.Generator(device=gu.DEV)
    g.manual_seed(99)
    levels = torch.tensor([-2.0, -0.5, 0.0, 0.25, 1.5, 3.0], device=gu.DEV)
    rows = []
    rows.append(levels[torch.randint(0, 6, (V,), generator=g, device=gu.DEV)])                 # ~5000 per level
    r = torch.randn(V, generator=g, device=gu.DEV)
    r[torch.randperm(V, generator=g, device=gu.DEV)[:40]] = 5.0                                   # 40 tied at the top
    rows.append(r)
    rows.append(torch.full((V,), 0.75, device=gu.DEV))                                          # everything tied
    z = torch.zeros(V, device=gu.DEV)
    z[::2] = -0.0
    z[5] = 1.0
    rows.append(z)                                                                               # +-0 are one value
    m = torch.randn(V, generator=g, device=gu.DEV)
    m[torch.rand(V, generator=g, device=gu.DEV) < 0.9] = float("-inf")                           # a masked row
    rows.append(m)
    logits = torch.stack(rows).to(tdt).contiguous()
    for k in (1, 2, 39, 40, 41, 1024, 1025, 3000, 6000, 20000, V - 1):
        for T in (1.0, 0.0):
            got, _, count = _check_topk(gu, oracle, logits, T, k, 31337, k)
    # the all-tied row keeps every entry whatever k is
    _, _, count = _check_topk(gu, oracle, logits, 1.0, 3, 1, 0)
    assert count[2] == V and count[3] == V


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_draws_on_rows_of_nan_and_infinities_end_and_stay_in_range(gu, dtype):
    """Rows a draw has no defined answer for (all NaN, all +inf, all -inf, a few
    numbers among NaN): every kernel loop has a bound that does not depend on the
    data, so the calls return, and the tokens they leave are valid indices.
    Rows next to them keep their normal result."""
    tdt = wl.torch_dtype(dtype)
    V = 9001
    g = torch.Generator(device=gu.DEV)
    g.manual_seed(5)
    good = (torch.randn(V, generator=g, device=gu.DEV) * 2).to(tdt)
    few = torch.full((V,), float("nan"), device=gu.DEV)
    few[[3, 77, 4000]] = torch.tensor([0.5, 2.0, -1.0], device=gu.DEV)
    rows = torch.stack([good.float(), torch.full((V,), float("nan"), device=gu.DEV),
                        torch.full((V,), float("inf"), device=gu.DEV),
                        torch.full((V,), float("-inf"), device=gu.DEV), few, good.float()]).to(tdt).contiguous()
    n = rows.shape[0]
    ref_tok = torch.empty(2, dtype=torch.int32, device=gu.DEV)
    for k in (None, 1, 5, 1500, 5000):
        tok = torch.full((n,), -7, dtype=torch.int32, device=gu.DEV)
        both = torch.stack([good, good]).contiguous()
        if k is None:
            rb.rlhf_sample_tokens(rows, tok, 1.0, 9, 2)
            rb.rlhf_sample_tokens(both, ref_tok, 1.0, 9, 2)
        else:
            rb.rlhf_sample_tokens_topk(rows, tok, 1.0, k, 9, 2)
            rb.rlhf_sample_tokens_topk(both, ref_tok, 1.0, k, 9, 2)
        torch.cuda.synchronize()
        t = tok.cpu().numpy()
        assert ((t >= 0) & (t < V)).all(), (k, t)
        assert t[0] == ref_tok.cpu().numpy()[0]          # row 0 is row 0 of the clean call
        if k is not None and k <= 3:
            assert t[4] in (3, 77, 4000)                  # the numbers among the NaN


@pytest.mark.parametrize("cfg_index,n", [(2, 64), (5, 128)])
def test_topk_draw_is_the_plain_draw_whenever_its_winner_survives(gu, cfg_index, n):
    """No oracle needed: both kernels score an entry with the same noise and the
    same fp32 arithmetic, so removing entries can only change the result by
    removing the plain draw's winner."""
    cfg = wl.config(cfg_index)
    actor, _ = wl.logits(cfg, n_positions=n, device=gu.DEV)
    plain = torch.empty(n, dtype=torch.int32, device=gu.DEV)
    rb.rlhf_sample_tokens(actor, plain, 1.0, 4711, 9)
    x = actor.float()
    rows = torch.arange(n, device=gu.DEV)
    for k in (1, 7, 50, 700, 3000, 20000):
        tok = torch.empty(n, dtype=torch.int32, device=gu.DEV)
        rb.rlhf_sample_tokens_topk(actor, tok, 1.0, k, 4711, 9)
        torch.cuda.synchronize()
        tau = torch.topk(x, k, dim=1).values[:, -1]
        survives = x[rows, plain.long()] >= tau
        assert torch.equal(tok[survives], plain[survives])
        assert (tok[~survives] != plain[~survives]).all()
        assert (x[rows, tok.long()] >= tau).all()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_topk_many_short_rows(gu, oracle, dtype):
    """Thousands of rows of a small vocabulary (a scoring-sized call): one
    workgroup per row, most lanes without an entry of their own."""
    tdt = wl.torch_dtype(dtype)
    g = torch.Generator(device=gu.DEV)
    g.manual_seed(321)
    logits = (torch.randn(3000, 777, generator=g, device=gu.DEV) * 2.5).to(tdt)
    for k, T in ((5, 1.0), (300, 0.6), (776, 0.0)):
        _check_topk(gu, oracle, logits, T, k, 8, 1)


@pytest.mark.parametrize("dtype,vocab,stride", [("bf16", 3000017, 3000024), ("f32", 2500003, 2500003)])
def test_rows_of_millions_of_entries(gu, oracle, dtype, vocab, stride):
    """Rows far longer than any vocabulary of the paper's models (vector path
    with a ragged tail, and the element-wise path of an odd stride): scoring,
    the plain draw whole and in segments, top-k with an on-chip list, with a
    list too long for it, and with half the row surviving."""
    n = 3
    g = torch.Generator(device=gu.DEV)
    g.manual_seed(vocab)
    tdt = wl.torch_dtype(dtype)
    actor = (torch.randn(n, stride, generator=g, device=gu.DEV) * 3.0).to(tdt)
    ref = (torch.randn(n, stride, generator=g, device=gu.DEV) * 3.0).to(tdt)
    tok = np.array([0, vocab - 1, vocab // 2], dtype=np.int32)
    _say(f"logprob V={vocab} stride={stride} {dtype}")
    logp, kl = gu.run_logprobs(actor, ref, tok, vocab=vocab, stride=stride)
    el, ek = oracle.token_logprobs_kl(wl.to_storage(actor), wl.to_storage(ref), tok, wl.DTYPE_CODE[dtype],
                                      vocab=vocab)
    assert np.abs(logp - el).max() <= LOGP_TOL
    assert np.abs(kl - ek).max() <= LOGP_TOL
    del ref
    _say("  plain draw")
    _check_sampling(gu, oracle, actor, 1.0, 5, 9, vocab=vocab, stride=stride)
    _check_sampling(gu, oracle, actor, 0.8, 5, 9, vocab=vocab, stride=stride, split=True)
    for k in (50, 70000, vocab // 2):
        _say(f"  top-{k}")
        _check_topk(gu, oracle, actor, 1.0, k, 6, 2, vocab=vocab, stride=stride)


@pytest.mark.parametrize("n", [(1 << 20) + 5, (1 << 24) + 3])
def test_row_counts_past_one_grid_dimension(gu, oracle, n):
    """One workgroup per row.  2^20 rows fill the grid's first dimension, and
    2^24 workgroups of 256 lanes are where the size of a one-dimensional launch
    no longer fits 32 bits: every row must still be scored and drawn, with the
    noise of its own row index."""
    V = 4
    g = torch.Generator(device=gu.DEV)
    g.manual_seed(n)
    actor = torch.randn(n, V, generator=g, device=gu.DEV) * 2.0
    ref = torch.randn(n, V, generator=g, device=gu.DEV) * 2.0
    tok = torch.randint(0, V, (n,), generator=g, device=gu.DEV, dtype=torch.int32).cpu().numpy()
    _say(f"logprob n={n} V={V} f32")
    logp, kl = gu.run_logprobs(actor, ref, tok)
    el, ek = oracle.token_logprobs_kl(wl.to_storage(actor), wl.to_storage(ref), tok, wl.DTYPE_CODE["f32"])
    assert np.abs(logp - el).max() <= LOGP_TOL
    assert np.abs(kl - ek).max() <= LOGP_TOL
    del ref
    _say(f"plain draw n={n}")
    got, agree, clear = _check_sampling(gu, oracle, actor, 1.0, 77, 3)
    assert agree > 0.999


@pytest.mark.parametrize("n", [(1 << 20) + 5, (1 << 22) + 3])
def test_topk_row_counts_past_one_grid_dimension(gu, oracle, n):
    """As above for the 1024-lane top-k kernel, whose one-dimensional launch
    would stop fitting 32 bits at 2^22 rows."""
    g = torch.Generator(device=gu.DEV)
    g.manual_seed(n)
    logits = torch.randn(n, 4, generator=g, device=gu.DEV) * 2.0
    _say(f"top-2 draw n={n}")
    got, agree, count = _check_topk(gu, oracle, logits, 1.0, 2, 78, 5)
    assert agree > 0.999


def test_topk_frequencies_on_the_gpu_follow_the_truncated_softmax(gu):
    import scipy.special
    import scipy.stats
    base = np.array([0.0, 1.0, -1.0, 2.5, 0.3, -3.0, 0.9, -0.2])
    logits = torch.tensor(base, dtype=torch.float32, device=gu.DEV)
    N, T, k = 80000, 0.8, 3
    tok = torch.empty(N, dtype=torch.int32, device=gu.DEV)
    rb.rlhf_sample_tokens_topk(logits.repeat(N, 1).contiguous(), tok, T, k, 4242, 1)
    torch.cuda.synchronize()
    keep = np.argsort(-base)[:k]
    p = np.zeros(8)
    p[keep] = scipy.special.softmax(base[keep] / T)
    counts = np.bincount(tok.cpu().numpy(), minlength=8)
    assert counts[p == 0].sum() == 0
    chi2 = ((counts[keep] - N * p[keep]) ** 2 / (N * p[keep])).sum()
    assert chi2 < scipy.stats.chi2.ppf(1 - 1e-6, k - 1), chi2


def test_sampling_frequencies_on_the_gpu_follow_softmax(gu):
    """Property that needs no oracle: the empirical distribution of many draws
    from one fixed row is softmax(logits / T)."""
    import scipy.special
    import scipy.stats
    logits = torch.tensor([0.0, 1.0, -1.0, 2.5, 0.3, -3.0, 0.9, -0.2], device=gu.DEV)
    N, T = 80000, 0.8
    tok = torch.empty(N, dtype=torch.int32, device=gu.DEV)
    rb.rlhf_sample_tokens(logits.repeat(N, 1).contiguous(), tok, T, 4242, 1)
    torch.cuda.synchronize()
    p = scipy.special.softmax(logits.double().cpu().numpy() / T)
    counts = np.bincount(tok.cpu().numpy(), minlength=8)
    chi2 = ((counts - N * p) ** 2 / (N * p)).sum()
    assert chi2 < scipy.stats.chi2.ppf(1 - 1e-6, 7), chi2


# ------------------------------------------------- streams, measurement aid ----
def test_calls_on_a_side_stream_give_the_same_results(gu):
    """Every entry point takes the caller's stream: the same work issued on a
    second stream (default priority) must give bit-identical outputs."""
    cfg = wl.small_variant(wl.config(5), batch=4, n_q_heads=16, n_kv_heads=2, len_lo=100, len_hi=900,
                           gen_len=8, vocab=32000)
    lens = wl.seq_lengths(cfg)
    q, ks, vs = wl.qkv(cfg, lens, device=gu.DEV)
    actor, ref = wl.logits(cfg, device=gu.DEV)
    tok = torch.from_numpy(wl.tokens(cfg)).to(gu.DEV)
    A = gu.FilledArena(cfg, lens, ks, vs)
    try:
        k, v, table, dl = A.views()
        params = rb.attn_params(cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, A.mpps,
                                wl.DTYPE_CODE[cfg.kv_dtype])
        nws = rb.rlhf_decode_attention_workspace_bytes(params)
        sws = rb.rlhf_sample_tokens_workspace_bytes(cfg.batch, cfg.vocab)

        def run(stream):
            ws = torch.empty(nws, dtype=torch.uint8, device=gu.DEV)
            out = torch.empty(cfg.batch, cfg.n_q_heads, cfg.head_dim, dtype=q.dtype, device=gu.DEV)
            logp = torch.empty(cfg.n_positions, dtype=torch.float32, device=gu.DEV)
            kl = torch.empty_like(logp)
            draw = torch.empty(cfg.batch, dtype=torch.int32, device=gu.DEV)
            sw = torch.empty(sws, dtype=torch.uint8, device=gu.DEV)
            torch.cuda.synchronize()
            rb.rlhf_decode_attention(params, q, k, v, table, dl, out, ws, stream=stream)
            rb.rlhf_token_logprobs_kl(actor, ref, tok, logp, kl, stream=stream)
            rb.rlhf_sample_tokens_split(actor[:cfg.batch], draw, 0.9, 77, sw, 3, stream=stream)
            torch.cuda.synchronize()
            return out, logp, kl, draw

        base = run(None)
        side = run(torch.cuda.Stream())
        for a, b in zip(base, side):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))

        # four host threads at once, each on a stream of its own with buffers of its own:
        # the compute entry points share no state that one caller could disturb for another
        import threading
        results, errors = {}, []

        def worker(i):
            try:
                stream = torch.cuda.Stream()
                ws = torch.empty(nws, dtype=torch.uint8, device=gu.DEV)
                sw = torch.empty(sws, dtype=torch.uint8, device=gu.DEV)
                out = torch.empty(cfg.batch, cfg.n_q_heads, cfg.head_dim, dtype=q.dtype, device=gu.DEV)
                logp = torch.empty(cfg.n_positions, dtype=torch.float32, device=gu.DEV)
                kl = torch.empty_like(logp)
                draw = torch.empty(cfg.batch, dtype=torch.int32, device=gu.DEV)
                for _ in range(10):
                    rb.rlhf_decode_attention(params, q, k, v, table, dl, out, ws, stream=stream)
                    rb.rlhf_token_logprobs_kl(actor, ref, tok, logp, kl, stream=stream)
                    rb.rlhf_sample_tokens_split(actor[:cfg.batch], draw, 0.9, 77, sw, 3, stream=stream)
                stream.synchronize()
                results[i] = (out, logp, kl, draw)
            except Exception as e:      # reported by the main thread
                errors.append(e)

        torch.cuda.synchronize()
        threads = [threading.Thread(target=worker, args=(i,)) for i in range(4)]
        for t in threads:
            t.start()
        for t in threads:
            t.join()
        assert not errors, errors
        for i in range(4):
            for a, b in zip(base, results[i]):
                assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), i
    finally:
        A.close()


@pytest.mark.parametrize("nbytes", [0, 16, 4096 + 16, 256 * 4 * 16 * 3 + 48, 1 << 22])
def test_read_probe_accepts_any_size(gu, nbytes):
    buf = torch.zeros(max(nbytes, 16) + 16, dtype=torch.uint8, device=gu.DEV)
    sink = torch.zeros(1, dtype=torch.int32, device=gu.DEV)
    rb.rlhf_probe_stream_read(buf, nbytes, sink)
    torch.cuda.synchronize()
    assert int(sink.item()) == 0
    with pytest.raises(rb.RlhfError):
        rb.rlhf_probe_stream_read(buf.data_ptr() + 8, 64)


def test_matrix_probe_reports_a_duration_and_a_clock(gu):
    """The probe's loop of matrix instructions runs to the end on any operand buffer (read modulo its length), and
    its two counters give a shader clock inside what the device can hold."""
    ticks = torch.zeros(3, dtype=torch.int64, device=gu.DEV)
    for ops in (torch.zeros(8, dtype=torch.bfloat16, device=gu.DEV),            # 16 bytes: every lane reads them
                torch.randn(4096 + 8, device=gu.DEV).to(torch.bfloat16)):       # not a multiple of a lane's share
        rb.rlhf_probe_matrix_rate(ops, 2000, 8, ticks)
        torch.cuda.synchronize()
        wall, cycles, _ = ticks.cpu().tolist()
        assert wall > 0 and 500 <= cycles / wall * 100 <= 3000, (wall, cycles)  # MHz
    rb.rlhf_probe_matrix_rate(ops, 0, 1, ticks)                                 # no iterations: nothing to do
    torch.cuda.synchronize()
    with pytest.raises(rb.RlhfError):
        rb.rlhf_probe_matrix_rate(ops.data_ptr() + 8, 10, 1, ticks, nbytes=64)
    with pytest.raises(rb.RlhfError):
        rb.rlhf_probe_matrix_rate(ops, 10, 0, ticks)
    with pytest.raises(rb.RlhfError):
        rb.rlhf_probe_matrix_rate(ops, 10, 1, 0)


@pytest.mark.parametrize("cfg_index,batch", [(1, 4), (2, 5), (5, 3)])
def test_rollout_demo_runs_the_whole_path(gu, cfg_index, batch):
    """The demo script composes every entry point in the order a rollout uses
    them and checks its own invariants (lengths, finite outputs, KL >= 0, the
    arena empty after the reset)."""
    from paper_2410_15651_amd import rollout_demo
    r = rollout_demo.run(cfg_index, gen_len=3, batch=batch, verbose=False)
    assert r["generated"] == 3 * batch and r["mean_kl"] >= 0
    assert r["arena_allocated_bytes"] <= r["arena_reserved_bytes"]
    r = rollout_demo.run(cfg_index, gen_len=2, batch=batch, verbose=False, top_k=20)     # the truncated draw
    assert r["generated"] == 2 * batch and r["mean_logp"] <= 0


def test_a_process_may_record_its_first_decode_attention_call_into_a_graph(gu):
    """The header lets the compute calls be recorded into a HIP graph with no eager
    call before.  Checked where it can be: in a fresh process
    (tests/cold_capture_check.py) whose first decode-attention call happens
    during capture; its replays must equal a later eager call bit for bit."""
    import subprocess
    import sys
    script = os.path.join(os.path.dirname(os.path.abspath(__file__)), "cold_capture_check.py")
    res = subprocess.run([sys.executable, script], capture_output=True, text=True, timeout=240)
    assert res.returncode == 0 and "OK" in res.stdout, (res.stdout + res.stderr)[-3000:]


def test_compute_entry_points_replay_from_a_hip_graph(gu):
    """The compute calls allocate nothing, clear nothing with memsets and never
    synchronise, so a caller may record them into a HIP graph.  A step's worth of
    them (decode attention, the plain, split and top-k draws, log-prob/KL with
    rewards, prefill attention) is captured once and replayed several times with
    eager work and synchronisations in between; every replay must reproduce the
    eager results bit for bit, and must follow the inputs' current contents."""
    cfg = wl.small_variant(wl.config(5), batch=4, n_q_heads=16, n_kv_heads=2, len_lo=90, len_hi=400, vocab=40000)
    lens = wl.seq_lengths(cfg)
    q, ks, vs = wl.qkv(cfg, lens, device=gu.DEV)
    A = gu.FilledArena(cfg, lens, ks, vs)
    try:
        k, v, table, sl = A.views()
        code = wl.DTYPE_CODE[cfg.kv_dtype]
        params = rb.attn_params(cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, A.mpps, code)
        ws = torch.empty(rb.rlhf_decode_attention_workspace_bytes(params), dtype=torch.uint8, device=gu.DEV)
        out = torch.empty_like(q)
        actor, ref = wl.logits(cfg, n_positions=64, device=gu.DEV)
        tok = torch.from_numpy(wl.tokens(cfg)[:64].copy()).to(gu.DEV)
        logp, kl, reward = (torch.empty(64, dtype=torch.float32, device=gu.DEV) for _ in range(3))
        d_plain, d_split, d_topk = (torch.empty(64, dtype=torch.int32, device=gu.DEV) for _ in range(3))
        sws = torch.empty(rb.rlhf_sample_tokens_workspace_bytes(64, cfg.vocab), dtype=torch.uint8, device=gu.DEV)
        cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        cu_d = torch.from_numpy(cu).to(gu.DEV)
        qp = wl.query_rows(cfg, int(cu[-1]), device=gu.DEV)
        outp = torch.empty_like(qp)
        results = [out, logp, kl, reward, d_plain, d_split, d_topk, outp]

        def step():
            rb.rlhf_decode_attention(params, q, k, v, table, sl, out, ws)
            rb.rlhf_sample_tokens(actor, d_plain, 0.8, 11, 3)
            rb.rlhf_sample_tokens_split(actor, d_split, 0.8, 11, sws, 3)
            rb.rlhf_sample_tokens_topk(actor, d_topk, 0.8, 30, 11, 3)
            rb.rlhf_token_logprobs_kl_rewards(actor, ref, tok, logp, kl, 0.1, reward_out=reward)
            rb.rlhf_prefill_attention(params, qp, cu_d, int(lens.max()), k, v, table, sl, outp)

        def eager():
            for r in results:
                r.view(torch.uint8).fill_(0x5A)
            step()
            torch.cuda.synchronize()
            return [r.clone() for r in results]

        expect = eager()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()                                      # warm-up on the capture stream
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        q2 = (q.float() * -0.5 + 0.25).to(q.dtype)
        for rep in range(4):
            if rep == 2:                                # new input contents in the recorded buffers
                q.copy_(q2)
                expect = eager()
            for r in results:
                r.view(torch.uint8).fill_(0xA5)         # eager work between replays; outputs poisoned
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            for r, e in zip(results, expect):
                assert torch.equal(r.view(torch.uint8), e.view(torch.uint8)), rep
    finally:
        A.close()
