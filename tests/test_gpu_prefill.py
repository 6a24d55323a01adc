"""GPU parity of the prefill (causal block) attention, called through the C ABI,
against the fp64 CPU oracle on the same seeded inputs: 2e-3 max-abs, the
attention tolerance."""
import numpy as np
import pytest
import torch

from paper_2410_15651_amd import binding as rb
from paper_2410_15651_amd import workloads as wl

pytestmark = pytest.mark.gpu

ATTN_TOL = 2e-3
P = wl.PAGE_TOKENS


@pytest.fixture(scope="module")
def gu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_util
    return gpu_util


def _say(msg):
    print(msg, flush=True)


_WAVES = 0


@pytest.fixture(autouse=True, params=[0, 8, 12], ids=["auto", "wg8", "wg12"])
def _workgroup_size(request):
    """Every test of this file runs with the library's own choice of workgroup
    size and with each of the two sizes forced (rlhf_prefill_attention_wg)."""
    global _WAVES
    _WAVES = request.param
    yield
    _WAVES = 0


def _run(gu, cfg, A, q, cu, max_q_len, out_dtype=None, scale=0.0, max_seq_len=0):
    k, v, table, lens = A.views()
    params = rb.attn_params(cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, A.mpps,
                            wl.DTYPE_CODE[cfg.kv_dtype], out_dtype=out_dtype, softmax_scale=scale,
                            max_seq_len=max_seq_len)
    odt = torch.float32 if out_dtype == rb.RLHF_F32 else wl.torch_dtype(cfg.kv_dtype)
    out = torch.full(tuple(q.shape), float("nan"), dtype=odt, device=gu.DEV)
    cu_d = torch.from_numpy(cu).to(gu.DEV)
    if _WAVES:
        rb.rlhf_prefill_attention_wg(params, q, cu_d, max_q_len, k, v, table, lens, out, _WAVES)
    else:
        rb.rlhf_prefill_attention(params, q, cu_d, max_q_len, k, v, table, lens, out)
    torch.cuda.synchronize()
    return out


def _oracle(oracle, cfg, q, cu, ks, vs, table, lens, n_pages, scale=None):
    kp, vp = wl.plain_pages([wl.to_storage(k) for k in ks], [wl.to_storage(v) for v in vs], table, n_pages)
    return oracle.prefill_attention(wl.to_storage(q), cu, kp, vp, table, lens, wl.DTYPE_CODE[cfg.kv_dtype],
                                    scale=scale)


def _rows(cfg, lens, how):
    """New rows per sequence: the whole cache ('full'), a trailing chunk
    ('chunk'), or a mix with an empty and a one-row sequence ('mix')."""
    rng = np.random.default_rng(cfg.seed + 77)
    if how == "full":
        n = lens.copy()
    elif how == "chunk":
        n = np.array([int(rng.integers(1, L + 1)) for L in lens], dtype=np.int32)
    else:
        n = lens.copy()
        n[0] = 0
        n[-1] = 1
        if len(n) > 2:
            n[1] = min(int(lens[1]), 17)
    return n.astype(np.int32)


SMALL = [
    # (config index, overrides, rows) -- several position blocks, pages and a ragged tail
    (1, dict(batch=3, len_lo=1, len_hi=300), "full"),                                  # f16 MHA, D=64
    (2, dict(batch=2, n_q_heads=4, n_kv_heads=4, len_lo=200, len_hi=600), "full"),     # bf16 MHA, D=64: 3 blocks
    (3, dict(batch=2, n_q_heads=4, n_kv_heads=4, len_lo=100, len_hi=700), "chunk"),    # D=128
    (5, dict(batch=3, n_q_heads=16, n_kv_heads=2, len_lo=20, len_hi=260), "full"),     # group of 8
    (5, dict(batch=3, n_q_heads=16, n_kv_heads=2, len_lo=20, len_hi=400), "mix"),
    (4, dict(batch=2, n_q_heads=6, n_kv_heads=2, len_lo=90, len_hi=200), "full"),      # group of 3: idle columns
    (3, dict(batch=2, n_q_heads=48, n_kv_heads=2, len_lo=30, len_hi=120), "chunk"),    # group of 24
    (1, dict(batch=2, n_q_heads=32, n_kv_heads=2, head_dim=128, len_lo=33, len_hi=90), "full"),   # f16, group of 16
    (2, dict(batch=1, n_q_heads=4, n_kv_heads=4, len_lo=3001, len_hi=3001), "full"),   # a long prompt: 8+ blocks of rows
    (5, dict(batch=2, n_q_heads=8, n_kv_heads=2, head_dim=64, len_lo=1, len_hi=50), "full"),
]


@pytest.mark.parametrize("cfg_index,over,how", SMALL)
def test_prefill_matches_oracle(gu, oracle, cfg_index, over, how):
    cfg = wl.small_variant(wl.config(cfg_index), **over)
    lens = wl.seq_lengths(cfg)
    n_new = _rows(cfg, lens, how)
    cu = np.concatenate([[0], np.cumsum(n_new)]).astype(np.int32)
    _say(f"prefill cfg{cfg_index} {over} lens={lens.tolist()} rows={n_new.tolist()}")
    _, ks, vs = wl.qkv(cfg, lens, device=gu.DEV)
    q = wl.query_rows(cfg, int(cu[-1]), device=gu.DEV)
    A = gu.FilledArena(cfg, lens, ks, vs)
    try:
        table, _, _ = A.host_state()
        expect = _oracle(oracle, cfg, q, cu, ks, vs, table, lens, A.n_pages)
        out32 = _run(gu, cfg, A, q, cu, int(n_new.max()), out_dtype=rb.RLHF_F32)
        assert torch.isfinite(out32).all()
        err32 = np.abs(out32.cpu().numpy().astype(np.float64) - expect).max()
        out16 = _run(gu, cfg, A, q, cu, int(n_new.max()) + 5)
        err16 = np.abs(out16.float().cpu().numpy().astype(np.float64) - expect).max()
        ulp = np.abs(expect).max() * (2.0 ** -8 if cfg.kv_dtype == "bf16" else 2.0 ** -11)
        _say(f"  max-abs err: f32 out {err32:.3e}, {cfg.kv_dtype} out {err16:.3e}")
        assert err32 <= ATTN_TOL
        assert err16 <= ATTN_TOL + ulp        # plus half an ulp of the 16-bit output itself
        # the 16-bit output is the fp32 output rounded to nearest even, element for element
        assert torch.equal(out32.to(out16.dtype).view(torch.int16), out16.view(torch.int16))
    finally:
        A.close()


def test_prefill_first_row_is_its_value_row_and_skipped_sequences_stay_untouched(gu, oracle):
    cfg = wl.small_variant(wl.config(3), batch=4, n_q_heads=4, n_kv_heads=2, len_lo=0, len_hi=64)
    lens = np.array([40, 16, 1, 33], dtype=np.int32)
    n_new = np.array([40, 17, 1, 2], dtype=np.int32)        # sequence 1 claims more rows than it has tokens
    cu = np.concatenate([[0], np.cumsum(n_new)]).astype(np.int32)
    _, ks, vs = wl.qkv(cfg, lens, device=gu.DEV)
    q = wl.query_rows(cfg, int(cu[-1]), device=gu.DEV)
    A = gu.FilledArena(cfg, lens, ks, vs)
    try:
        out = _run(gu, cfg, A, q, cu, 40, out_dtype=rb.RLHF_F32)
        assert torch.isnan(out[cu[1]:cu[2]]).all()                       # skipped, as documented
        out16 = _run(gu, cfg, A, q, cu, 40)
        for h in range(4):                        # position 0 sees one key: V_0 (to the rounding of the weights)
            for row, b in ((0, 0), (int(cu[2]), 2)):
                v0 = vs[b][0, h // 2]
                assert (out[row, h] - v0.float()).abs().max().item() <= 1e-4
                assert torch.equal(out16[row, h].view(torch.int16), v0.view(torch.int16))
        keep = [0, 2, 3]
        table, _, _ = A.host_state()
        cu_k = np.concatenate([[0], np.cumsum(n_new[keep])]).astype(np.int32)
        qk = torch.cat([q[cu[b]:cu[b + 1]] for b in keep])
        expect = _oracle(oracle, cfg, qk, cu_k, [ks[b] for b in keep], [vs[b] for b in keep], table[keep],
                         lens[keep], A.n_pages)
        got = torch.cat([out[cu[b]:cu[b + 1]] for b in keep]).cpu().numpy().astype(np.float64)
        assert np.abs(got - expect).max() <= ATTN_TOL
        # explicit softmax scale, and a launch bound below the longest block: rows beyond it are not computed
        expect_s = _oracle(oracle, cfg, qk, cu_k, [ks[b] for b in keep], [vs[b] for b in keep], table[keep],
                           lens[keep], A.n_pages, scale=0.31)
        out_s = _run(gu, cfg, A, q, cu, 40, out_dtype=rb.RLHF_F32, scale=0.31)
        got_s = torch.cat([out_s[cu[b]:cu[b + 1]] for b in keep]).cpu().numpy().astype(np.float64)
        assert np.abs(got_s - expect_s).max() <= ATTN_TOL
        assert np.abs(expect_s - expect).max() > 10 * ATTN_TOL
    finally:
        A.close()


def test_prefill_rows_equal_decode_steps(gu):
    """A prefill row at position p and a decode step over the first p+1 tokens
    are the same computation: the two kernels must agree to rounding.  The
    prefill kernel feeds its weights to the matrix cores as fp16 (relative
    rounding at most 2^-11 each), so an output element may differ by
    2^-11 * sum_j w_j |v_j|; that sum is the decode kernel's own output on |V|,
    and the bound below is that plus fp32 accumulation noise."""
    cfg = wl.small_variant(wl.config(5), batch=2, n_q_heads=16, n_kv_heads=2, len_lo=150, len_hi=300)
    lens = wl.seq_lengths(cfg)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    _, ks, vs = wl.qkv(cfg, lens, device=gu.DEV)
    q = wl.query_rows(cfg, int(cu[-1]), device=gu.DEV)
    A = gu.FilledArena(cfg, lens, ks, vs)
    A_abs = gu.FilledArena(cfg, lens, ks, [v.abs() for v in vs])
    try:
        out = _run(gu, cfg, A, q, cu, int(lens.max()), out_dtype=rb.RLHF_F32)
        last = torch.stack([q[cu[b + 1] - 1] for b in range(cfg.batch)]).contiguous()
        dec = gu.run_attention(cfg, A, last, out_dtype=rb.RLHF_F32)
        weight_abs = gu.run_attention(cfg, A_abs, last, out_dtype=rb.RLHF_F32)
        bound = 2.0 ** -11 * weight_abs + 1e-5
        assert bound.max().item() < 0.5 * ATTN_TOL
        for b in range(cfg.batch):
            assert ((out[cu[b + 1] - 1] - dec[b]).abs() <= bound[b]).all()
    finally:
        A.close()
        A_abs.close()


def test_prefill_is_bit_identical_under_page_permutation(gu):
    base = wl.small_variant(wl.config(3), batch=3, n_q_heads=8, n_kv_heads=4, len_lo=100, len_hi=500)
    lens = wl.seq_lengths(base)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    _, ks, vs = wl.qkv(base, lens, device=gu.DEV)
    q = wl.query_rows(base, int(cu[-1]), device=gu.DEV)
    outs = []
    for shuffled in (False, True):
        cfg = wl.small_variant(base, shuffled_pages=shuffled)
        A = gu.FilledArena(cfg, lens, ks, vs, slack_pages=11)
        try:
            outs.append(_run(gu, cfg, A, q, cu, int(lens.max()), out_dtype=rb.RLHF_F32))
        finally:
            A.close()
    assert torch.equal(outs[0].view(torch.int32), outs[1].view(torch.int32))


_FULL_EXPECT = {}   # configuration -> (sequences, oracle rows): the three workgroup sizes share one oracle run


@pytest.mark.parametrize("cfg_index", [1, 2, 3, 4, 5])
def test_prefill_full_size(gu, oracle, cfg_index):
    """The benchmark's prefill launch at the full shape.  The oracle computes
    every row of configurations 1-3; for 4 and 5 (10^11 .. 10^13 fp64 operations
    for all rows) every row of the shortest, the longest and two seeded
    sequences.  The maximum error is over all elements of those rows."""
    cfg = wl.config(cfg_index)
    lens = wl.prompt_lengths(cfg)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    _say(f"prefill full cfg{cfg_index}: B={cfg.batch} rows={int(cu[-1])}")
    _, ks, vs = wl.qkv(cfg, lens, device=gu.DEV)
    q = wl.query_rows(cfg, int(cu[-1]), device=gu.DEV)
    A = gu.FilledArena(cfg, lens, ks, vs)
    try:
        table, _, _ = A.host_state()
        out = _run(gu, cfg, A, q, cu, int(lens.max()), out_dtype=rb.RLHF_F32)
        assert torch.isfinite(out).all()
        if cfg_index not in _FULL_EXPECT:
            if cfg_index <= 3:
                seqs = list(range(cfg.batch))
            else:
                rng = np.random.default_rng(cfg.seed)
                seqs = sorted({int(lens.argmin()), int(lens.argmax()), *rng.integers(0, cfg.batch, 2).tolist()})
            sub_cu = np.concatenate([[0], np.cumsum(lens[seqs])]).astype(np.int32)
            sub_q = torch.cat([q[cu[b]:cu[b + 1]] for b in seqs])
            expect = _oracle(oracle, cfg, sub_q, sub_cu, [ks[b] for b in seqs], [vs[b] for b in seqs],
                             table[seqs], lens[seqs], A.n_pages)
            _FULL_EXPECT[cfg_index] = (seqs, expect)
        seqs, expect = _FULL_EXPECT[cfg_index]
        got = torch.cat([out[cu[b]:cu[b + 1]] for b in seqs]).cpu().numpy().astype(np.float64)
        assert got.shape == expect.shape
        worst = np.abs(got - expect).max()
        _say(f"  {len(seqs)} of {cfg.batch} sequences, {expect.shape[0]} rows, every element: max-abs err {worst:.3e}")
        assert worst <= ATTN_TOL
        # holds at any size: every output lies inside the range of its head's values
        b = seqs[0]
        G = cfg.n_q_heads // cfg.n_kv_heads
        vmin, vmax = vs[b].float().amin(0), vs[b].float().amax(0)
        o = out[cu[b]:cu[b + 1]].view(-1, cfg.n_kv_heads, G, cfg.head_dim)
        assert (o >= vmin[None, :, None, :] - 1e-5).all() and (o <= vmax[None, :, None, :] + 1e-5).all()
    finally:
        A.close()


def test_pages_beyond_4_gib_of_an_arena_half(gu, oracle):
    """K and V halves of 4.6 GiB each, the sequences' pages scattered over all of
    them by the shuffled free list: block offsets inside a half need more than
    32 bits in the append, the read-back, decode attention and prefill."""
    cfg = wl.small_variant(wl.config(5), batch=3, n_q_heads=16, n_kv_heads=8, len_lo=100, len_hi=600)
    lens = wl.seq_lengths(cfg)
    q1, ks, vs = wl.qkv(cfg, lens, device=gu.DEV)
    _say(f"large arena: lens={lens.tolist()}")
    A = gu.FilledArena(cfg, lens, ks, vs, slack_pages=150000)
    try:
        table, _, _ = A.host_state()
        half_page_bytes = cfg.n_kv_heads * P * cfg.head_dim * 2
        beyond = int((table.astype(np.int64) * half_page_bytes >= 2 ** 32).sum())
        _say(f"  {beyond} of {int((table >= 0).sum())} pages start beyond 4 GiB")
        assert beyond >= 3
        # the oracle gets the same pages under compact numbers (the arena's own run to 150,000)
        used = np.unique(table[table >= 0])
        compact = np.where(table >= 0, np.searchsorted(used, table), -1).astype(np.int32)
        for b in range(cfg.batch):
            ko, vo = torch.zeros_like(ks[b]), torch.zeros_like(vs[b])
            rb.rlhf_kv_arena_gather(A.handle, b, 0, int(lens[b]), ko, vo)
            torch.cuda.synchronize()
            assert torch.equal(ko.view(torch.int16), ks[b].view(torch.int16))
            assert torch.equal(vo.view(torch.int16), vs[b].view(torch.int16))
        expect = gu.oracle_attention(oracle, cfg, q1, ks, vs, compact, lens, len(used))
        out = gu.run_attention(cfg, A, q1, out_dtype=rb.RLHF_F32).cpu().numpy().astype(np.float64)
        assert np.abs(out - expect).max() <= ATTN_TOL
        cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        q = wl.query_rows(cfg, int(cu[-1]), device=gu.DEV)
        expect = _oracle(oracle, cfg, q, cu, ks, vs, compact, lens, len(used))
        outp = _run(gu, cfg, A, q, cu, int(lens.max()), out_dtype=rb.RLHF_F32).cpu().numpy().astype(np.float64)
        assert np.abs(outp - expect).max() <= ATTN_TOL
    finally:
        A.close()


def test_prefill_of_thousands_of_short_prompts(gu, oracle):
    """A scoring-sized batch: 3,001 sequences of 0 to 40 tokens, three KV heads
    (units per launch not a multiple of the chip's eight dies), one position
    block each, most of it empty."""
    cfg = wl.small_variant(wl.config(2), batch=3001, n_q_heads=6, n_kv_heads=3, len_lo=0, len_hi=40)
    lens = wl.seq_lengths(cfg)
    lens[0] = 0
    lens[-1] = 40
    n_new = lens.copy()
    n_new[5::7] = np.minimum(n_new[5::7], 3)            # some sequences score only their last tokens
    cu = np.concatenate([[0], np.cumsum(n_new)]).astype(np.int32)
    _, ks, vs = wl.qkv(cfg, lens, device=gu.DEV)
    q = wl.query_rows(cfg, int(cu[-1]), device=gu.DEV)
    A = gu.FilledArena(cfg, lens, ks, vs)
    try:
        table, _, _ = A.host_state()
        expect = _oracle(oracle, cfg, q, cu, ks, vs, table, lens, A.n_pages)
        out = _run(gu, cfg, A, q, cu, int(n_new.max()), out_dtype=rb.RLHF_F32)
        assert torch.isfinite(out).all()
        assert np.abs(out.cpu().numpy().astype(np.float64) - expect).max() <= ATTN_TOL
    finally:
        A.close()


def test_lengths_above_max_seq_len_count_as_max_seq_len(gu, oracle):
    """The documented clamp, for the decode step and for prefill: a sequence
    longer than params.max_seq_len is attended as if it ended there."""
    cfg = wl.small_variant(wl.config(3), batch=5, n_q_heads=4, n_kv_heads=2, len_lo=0, len_hi=130)
    lens = np.array([130, 37, 48, 49, 5], dtype=np.int32)
    cap = 48
    clipped = np.minimum(lens, cap).astype(np.int32)
    q1, ks, vs = wl.qkv(cfg, lens, device=gu.DEV)
    A = gu.FilledArena(cfg, lens, ks, vs)
    try:
        table, _, _ = A.host_state()
        expect = gu.oracle_attention(oracle, cfg, q1, ks, vs, table, clipped, A.n_pages)
        out = gu.run_attention(cfg, A, q1, out_dtype=rb.RLHF_F32, max_seq_len=cap).cpu().numpy().astype(np.float64)
        assert np.abs(out - expect).max() <= ATTN_TOL
        n_new = np.array([48, 7, 20, 1, 5], dtype=np.int32)       # rows are the last ones of the clamped cache
        cu = np.concatenate([[0], np.cumsum(n_new)]).astype(np.int32)
        q = wl.query_rows(cfg, int(cu[-1]), device=gu.DEV)
        expect = _oracle(oracle, cfg, q, cu, ks, vs, table, clipped, A.n_pages)
        outp = _run(gu, cfg, A, q, cu, 48, out_dtype=rb.RLHF_F32, max_seq_len=cap)
        assert np.abs(outp.cpu().numpy().astype(np.float64) - expect).max() <= ATTN_TOL
    finally:
        A.close()


def test_rows_past_max_q_len_are_correct_or_untouched(gu, oracle):
    """max_q_len sizes the launch.  A sequence with more rows than that gets its
    first max_q_len rows; each later row is either computed (the last block of
    positions reaches it) or left as it was, never anything else."""
    cfg = wl.small_variant(wl.config(3), batch=2, n_q_heads=4, n_kv_heads=2, len_lo=0, len_hi=1500)
    lens = np.array([1500, 30], dtype=np.int32)
    n_new = np.array([1400, 30], dtype=np.int32)
    cu = np.concatenate([[0], np.cumsum(n_new)]).astype(np.int32)
    _, ks, vs = wl.qkv(cfg, lens, device=gu.DEV)
    q = wl.query_rows(cfg, int(cu[-1]), device=gu.DEV)
    A = gu.FilledArena(cfg, lens, ks, vs)
    try:
        table, _, _ = A.host_state()
        expect = _oracle(oracle, cfg, q, cu, ks, vs, table, lens, A.n_pages)
        bound = 100
        out = _run(gu, cfg, A, q, cu, bound, out_dtype=rb.RLHF_F32).cpu().numpy().astype(np.float64)
        done = ~np.isnan(out).any(axis=(1, 2))
        assert done[:bound].all() and done[cu[1]:].all()
        assert not done[cu[1] - 1]                       # 1,400 rows are more than one block past 100
        assert not np.isnan(out[done]).any()
        assert (np.isnan(out[~done])).all()              # untouched rows hold the NaN fill in every element
        assert np.abs(out[done] - expect[done]).max() <= ATTN_TOL
    finally:
        A.close()
