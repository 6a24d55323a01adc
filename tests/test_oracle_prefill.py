"""Pins for the prefill (causal block) attention oracle: it must agree, query by
query, with the separately pinned decode oracle run on a truncated cache; with
torch's fp64 causal scaled-dot-product attention on a dense case; the first
token of a sequence sees only itself; later keys never leak backwards."""
import numpy as np
import torch

from paper_2410_15651_amd import workloads as wl

P = wl.PAGE_TOKENS
F32 = 2


def _case(rng, lens, n_new, Hq, Hkv, D, shuffle=False):
    B = len(lens)
    ks = [rng.standard_normal((L, Hkv, D)).astype(np.float32) for L in lens]
    vs = [rng.standard_normal((L, Hkv, D)).astype(np.float32) for L in lens]
    need = [(L + P - 1) // P for L in lens]
    n_pages = sum(need) + 2
    order = rng.permutation(n_pages) if shuffle else np.arange(n_pages)
    table = np.full((B, max(need)), -1, dtype=np.int32)
    it = iter(order)
    for b in range(B):
        for lp in range(need[b]):
            table[b, lp] = next(it)
    kp, vp = wl.plain_pages(ks, vs, table, n_pages)
    cu = np.concatenate([[0], np.cumsum(n_new)]).astype(np.int32)
    q = rng.standard_normal((cu[-1], Hq, D)).astype(np.float32)
    return q, cu, ks, vs, kp, vp, table, np.array(lens, dtype=np.int32)


def test_each_query_equals_decode_attention_on_the_truncated_cache(oracle):
    rng = np.random.default_rng(0)
    lens, n_new = [37, 5, 64], [20, 5, 1]
    q, cu, ks, vs, kp, vp, table, L = _case(rng, lens, n_new, 4, 2, 8, shuffle=True)
    out = oracle.prefill_attention(q, cu, kp, vp, table, L, F32)
    for b in range(3):
        for i in range(n_new[b]):
            pos = lens[b] - n_new[b] + i
            one = oracle.decode_attention(q[cu[b] + i][None], kp, vp, table[b][None],
                                          np.array([pos + 1], dtype=np.int32), F32)
            np.testing.assert_allclose(out[cu[b] + i], one[0], rtol=1e-13, atol=1e-15)


def test_against_torch_causal_sdpa_fp64(oracle):
    rng = np.random.default_rng(1)
    B, H, D, Lq = 2, 3, 16, 40
    q, cu, ks, vs, kp, vp, table, L = _case(rng, [Lq] * B, [Lq] * B, H, H, D)
    out = oracle.prefill_attention(q, cu, kp, vp, table, L, F32)
    tq = torch.from_numpy(q).double().view(B, Lq, H, D).permute(0, 2, 1, 3)
    tk = torch.stack([torch.from_numpy(k) for k in ks]).double().permute(0, 2, 1, 3)
    tv = torch.stack([torch.from_numpy(v) for v in vs]).double().permute(0, 2, 1, 3)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)
    np.testing.assert_allclose(out.reshape(B, Lq, H, D), ref.permute(0, 2, 1, 3).numpy(), rtol=1e-11, atol=1e-13)


def test_first_token_sees_only_itself_and_the_future_never_leaks(oracle):
    rng = np.random.default_rng(2)
    q, cu, ks, vs, kp, vp, table, L = _case(rng, [33], [33], 2, 1, 4)
    out = oracle.prefill_attention(q, cu, kp, vp, table, L, F32)
    assert np.array_equal(out[0, 0], vs[0][0, 0].astype(np.float64))
    assert np.array_equal(out[0, 1], vs[0][0, 0].astype(np.float64))
    # changing keys/values at positions >= 20 must leave the first 20 outputs untouched
    ks2 = [ks[0].copy()]
    vs2 = [vs[0].copy()]
    ks2[0][20:] += 3.0
    vs2[0][20:] -= 5.0
    kp2, vp2 = wl.plain_pages(ks2, vs2, table, kp.shape[0])
    out2 = oracle.prefill_attention(q, cu, kp2, vp2, table, L, F32)
    assert np.array_equal(out[:20], out2[:20]) and not np.array_equal(out[20:], out2[20:])


def test_chunked_prefill_equals_full_prefill(oracle):
    """Queries for the last 7 tokens only (an earlier chunk already cached) give
    the same rows as the full prefill."""
    rng = np.random.default_rng(3)
    q, cu, ks, vs, kp, vp, table, L = _case(rng, [50], [50], 2, 2, 8)
    full = oracle.prefill_attention(q, cu, kp, vp, table, L, F32)
    part = oracle.prefill_attention(q[43:], np.array([0, 7], dtype=np.int32), kp, vp, table, L, F32)
    assert np.array_equal(part, full[43:])


def test_custom_scale_and_grouped_heads(oracle):
    rng = np.random.default_rng(4)
    q, cu, ks, vs, kp, vp, table, L = _case(rng, [19, 30], [19, 4], 6, 2, 8)
    out = oracle.prefill_attention(q, cu, kp, vp, table, L, F32, scale=0.4)
    import scipy.special
    b, i, hq = 1, 2, 5
    pos = 30 - 4 + i
    s = 0.4 * (ks[b][:pos + 1, hq // 3].astype(np.float64) @ q[cu[b] + i, hq].astype(np.float64))
    np.testing.assert_allclose(out[cu[b] + i, hq],
                               scipy.special.softmax(s) @ vs[b][:pos + 1, hq // 3].astype(np.float64), rtol=1e-12)


def test_bad_block_lengths_are_rejected(oracle):
    import pytest
    rng = np.random.default_rng(5)
    q, cu, ks, vs, kp, vp, table, L = _case(rng, [10], [10], 1, 1, 4)
    with pytest.raises(ValueError):
        oracle.prefill_attention(q, cu, kp, vp, table, np.array([9], dtype=np.int32), F32)   # more queries than tokens
