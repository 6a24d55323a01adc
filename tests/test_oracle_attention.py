"""Pins for the attention oracle: closed forms, invariants, library routines and
brute force.  None of these re-types the oracle's own loop; each would fail for
a plausible slip in it (dropped scale, wrong head mapping, wrong page or slot
index, transposed operand, unnormalised weights)."""
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.special
import torch

from paper_2410_15651_amd import workloads as wl

P = wl.PAGE_TOKENS
F16, BF16, F32 = 0, 1, 2
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _paged(ks, vs, n_pages=None, perm=None):
    """Per-sequence rows -> plain pages + page table (identity or permuted)."""
    B = len(ks)
    need = [(k.shape[0] + P - 1) // P for k in ks]
    max_pages = max(1, max(need))
    total = sum(need)
    n_pages = total if n_pages is None else n_pages
    order = np.arange(n_pages) if perm is None else np.asarray(perm)
    table = np.full((B, max_pages), -1, dtype=np.int32)
    it = iter(order)
    for b in range(B):
        for lp in range(need[b]):
            table[b, lp] = next(it)
    kp, vp = wl.plain_pages(ks, vs, table, max(n_pages, 1))
    return kp, vp, table


def _rand_case(rng, B, Hq, Hkv, D, lens, dtype=np.float32):
    q = rng.standard_normal((B, Hq, D)).astype(dtype)
    ks = [rng.standard_normal((L, Hkv, D)).astype(dtype) for L in lens]
    vs = [rng.standard_normal((L, Hkv, D)).astype(dtype) for L in lens]
    return q, ks, vs


def _run(oracle, q, ks, vs, dtype=F32, scale=None, perm=None, n_pages=None, weights=False):
    kp, vp, table = _paged(ks, vs, n_pages=n_pages, perm=perm)
    lens = np.array([k.shape[0] for k in ks], dtype=np.int32)
    return oracle.decode_attention(q, kp, vp, table, lens, dtype, scale=scale,
                                   return_weights=weights)


def test_golden_rational_weights(oracle):
    """D = 1, q = 1, scale = 1, keys = ln(n_j): weights are n_j / sum n."""
    for line in open(os.path.join(GOLDEN, "attention_closed_forms.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, ns, vals, expect = [f.strip() for f in line.split("|")]
        n = np.array([float(x) for x in ns.split()])
        v = np.array([float(x) for x in vals.split()], dtype=np.float32)
        q = np.ones((1, 1, 1), dtype=np.float32)
        ks = [np.log(n).astype(np.float32).reshape(-1, 1, 1)]
        vs = [v.reshape(-1, 1, 1)]
        out = _run(oracle, q, ks, vs, scale=1.0)
        assert out.shape == (1, 1, 1)
        assert abs(out[0, 0, 0] - float(Fraction(expect))) < 2e-6, name


def test_single_token_returns_value_row_exactly(oracle):
    rng = np.random.default_rng(0)
    for dtype_code, tdt in ((F16, torch.float16), (BF16, torch.bfloat16)):
        q = wl.to_storage(torch.from_numpy(rng.standard_normal((3, 4, 8)).astype(np.float32)).to(tdt))
        ks = [wl.to_storage(torch.from_numpy(rng.standard_normal((1, 2, 8)).astype(np.float32)).to(tdt))
              for _ in range(3)]
        vs_t = [torch.from_numpy(rng.standard_normal((1, 2, 8)).astype(np.float32)).to(tdt)
                for _ in range(3)]
        vs = [wl.to_storage(v) for v in vs_t]
        out = _run(oracle, q, ks, vs, dtype=dtype_code)
        for b in range(3):
            for hq in range(4):
                expect = vs_t[b][0, hq // 2].double().numpy()
                assert np.array_equal(out[b, hq], expect)


def test_widening_of_every_16bit_pattern(oracle):
    """L = 1, q = k = 0 makes out equal the stored V exactly, so V can carry all
    65536 bit patterns; torch's own conversions are the independent reference."""
    bits = np.arange(65536, dtype=np.uint16)
    for dtype_code, tdt in ((F16, torch.float16), (BF16, torch.bfloat16)):
        expect = torch.from_numpy(bits.view(np.int16).copy()).view(tdt).double().numpy()
        D = 65536
        q = np.zeros((1, 1, D), dtype=np.uint16)
        ks = [np.zeros((1, 1, D), dtype=np.uint16)]
        vs = [bits.reshape(1, 1, D).copy()]
        out = _run(oracle, q, ks, vs, dtype=dtype_code)[0, 0]
        assert np.array_equal(out, expect, equal_nan=True)


def test_zero_query_gives_mean_of_values(oracle):
    rng = np.random.default_rng(1)
    q, ks, vs = _rand_case(rng, 2, 2, 2, 4, [37, 5])
    q[:] = 0
    out = _run(oracle, q, ks, vs)
    for b in range(2):
        for h in range(2):
            np.testing.assert_allclose(out[b, h], vs[b][:, h].astype(np.float64).mean(0), rtol=1e-13)


def test_equal_keys_give_mean_of_values(oracle):
    rng = np.random.default_rng(2)
    q, ks, vs = _rand_case(rng, 1, 1, 1, 8, [50])
    ks[0][:] = ks[0][0]
    out = _run(oracle, q, ks, vs)
    np.testing.assert_allclose(out[0, 0], vs[0][:, 0].astype(np.float64).mean(0), rtol=1e-12)


def test_dominant_key_selects_its_value(oracle):
    rng = np.random.default_rng(3)
    q, ks, vs = _rand_case(rng, 1, 1, 1, 4, [20])
    q[0, 0] = [1, 0, 0, 0]
    ks[0][:, 0, 0] = 0
    ks[0][7, 0, 0] = 200.0   # scale 1/2 -> score 100 above everything else
    out = _run(oracle, q, ks, vs)
    np.testing.assert_allclose(out[0, 0], vs[0][7, 0].astype(np.float64), atol=1e-30, rtol=1e-12)


def test_weights_are_a_distribution_and_match_scipy(oracle):
    rng = np.random.default_rng(4)
    lens = [33, 1, 16, 47]
    q, ks, vs = _rand_case(rng, 4, 4, 2, 8, lens)
    out, w = _run(oracle, q, ks, vs, weights=True)
    scale = 1 / np.sqrt(8)
    for b, L in enumerate(lens):
        for hq in range(4):
            ww = w[b, hq, :L]
            assert abs(ww.sum() - 1) < 1e-13
            assert (ww > 0).all() and (ww <= 1).all()
            scores = scale * (ks[b][:, hq // 2].astype(np.float64) @ q[b, hq].astype(np.float64))
            np.testing.assert_allclose(ww, scipy.special.softmax(scores), rtol=1e-12)
            np.testing.assert_allclose(out[b, hq], ww @ vs[b][:, hq // 2].astype(np.float64), rtol=1e-12,
                                       atol=1e-14)


def test_against_torch_sdpa_fp64_dense_case(oracle):
    rng = np.random.default_rng(5)
    B, H, D, L = 3, 5, 16, 48
    q, ks, vs = _rand_case(rng, B, H, H, D, [L] * B)
    out = _run(oracle, q, ks, vs)
    tq = torch.from_numpy(q).double().unsqueeze(2)                      # [B,H,1,D]
    tk = torch.stack([torch.from_numpy(k) for k in ks]).double().permute(0, 2, 1, 3)  # [B,H,L,D]
    tv = torch.stack([torch.from_numpy(v) for v in vs]).double().permute(0, 2, 1, 3)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv).squeeze(2).numpy()
    np.testing.assert_allclose(out, ref, rtol=1e-11, atol=1e-13)


def test_custom_scale_is_applied_to_scores(oracle):
    rng = np.random.default_rng(6)
    q, ks, vs = _rand_case(rng, 1, 2, 2, 8, [19])
    out = _run(oracle, q, ks, vs, scale=0.3)
    for h in range(2):
        s = 0.3 * (ks[0][:, h].astype(np.float64) @ q[0, h].astype(np.float64))
        np.testing.assert_allclose(out[0, h], scipy.special.softmax(s) @ vs[0][:, h].astype(np.float64),
                                   rtol=1e-12)


def test_shift_of_all_keys_changes_nothing(oracle):
    rng = np.random.default_rng(7)
    q, ks, vs = _rand_case(rng, 2, 2, 2, 8, [21, 40], dtype=np.float32)
    # dyadic values so the shift is exact in float32
    ks = [np.round(k * 8) / 8 for k in ks]
    delta = (np.round(rng.standard_normal(8) * 8) / 8).astype(np.float32)
    out0 = _run(oracle, q, ks, vs)
    out1 = _run(oracle, q, [k + delta for k in ks], vs)
    np.testing.assert_allclose(out0, out1, rtol=1e-11, atol=1e-13)


def test_affine_in_values_and_inside_their_range(oracle):
    rng = np.random.default_rng(8)
    q, ks, vs = _rand_case(rng, 2, 4, 4, 8, [29, 64])
    vs = [np.round(v * 16) / 16 for v in vs]
    out0 = _run(oracle, q, ks, vs)
    out1 = _run(oracle, q, ks, [v * 4 + 0.5 for v in vs])
    np.testing.assert_allclose(out1, 4 * out0 + 0.5, rtol=1e-12, atol=1e-13)
    for b in range(2):
        for h in range(4):
            col = vs[b][:, h].astype(np.float64)
            assert (out0[b, h] >= col.min(0) - 1e-14).all()
            assert (out0[b, h] <= col.max(0) + 1e-14).all()


def test_physical_page_permutation_is_bit_identical(oracle):
    rng = np.random.default_rng(9)
    lens = [70, 3, 16, 33]
    q, ks, vs = _rand_case(rng, 4, 4, 2, 8, lens)
    total = sum((L + P - 1) // P for L in lens)
    out0 = _run(oracle, q, ks, vs, n_pages=total + 3)
    perm = rng.permutation(total + 3)
    out1 = _run(oracle, q, ks, vs, n_pages=total + 3, perm=perm)
    assert np.array_equal(out0, out1)


def test_logical_token_permutation_only_reorders_the_sum(oracle):
    rng = np.random.default_rng(10)
    q, ks, vs = _rand_case(rng, 1, 2, 2, 8, [45])
    perm = rng.permutation(45)
    out0 = _run(oracle, q, ks, vs)
    out1 = _run(oracle, q, [ks[0][perm]], [vs[0][perm]])
    np.testing.assert_allclose(out0, out1, rtol=1e-12, atol=1e-14)


def test_grouped_query_heads_equal_repeated_kv_heads(oracle):
    rng = np.random.default_rng(11)
    lens = [18, 40]
    q, ks, vs = _rand_case(rng, 2, 8, 2, 8, lens)
    out_gqa = _run(oracle, q, ks, vs)
    ks_rep = [np.repeat(k, 4, axis=1) for k in ks]
    vs_rep = [np.repeat(v, 4, axis=1) for v in vs]
    out_mha = _run(oracle, q, ks_rep, vs_rep)
    assert np.array_equal(out_gqa, out_mha)


def test_brute_force_without_max_subtraction(oracle):
    rng = np.random.default_rng(12)
    q, ks, vs = _rand_case(rng, 1, 1, 1, 2, [5])
    out = _run(oracle, q, ks, vs, scale=1.0)
    num = np.zeros(2)
    den = 0.0
    for j in range(5):
        e = np.exp(float(q[0, 0, 0]) * float(ks[0][j, 0, 0]) + float(q[0, 0, 1]) * float(ks[0][j, 0, 1]))
        num += e * vs[0][j, 0].astype(np.float64)
        den += e
    np.testing.assert_allclose(out[0, 0], num / den, rtol=1e-13)


def test_empty_sequence_gives_zeros(oracle):
    rng = np.random.default_rng(13)
    q = rng.standard_normal((2, 2, 4)).astype(np.float32)
    kp = rng.standard_normal((2, 2, P, 4)).astype(np.float32)
    vp = rng.standard_normal((2, 2, P, 4)).astype(np.float32)
    table = np.array([[0], [1]], dtype=np.int32)
    out = oracle.decode_attention(q, kp, vp, table, np.array([0, 5], dtype=np.int32), F32)
    assert (out[0] == 0).all() and np.isfinite(out).all() and (out[1] != 0).any()


def test_slots_past_the_length_are_ignored(oracle):
    rng = np.random.default_rng(14)
    q, ks, vs = _rand_case(rng, 1, 1, 1, 4, [21])
    kp, vp, table = _paged(ks, vs)
    lens = np.array([21], dtype=np.int32)
    out0 = oracle.decode_attention(q, kp, vp, table, lens, F32)
    kp[table[0, 1], :, 5:, :] = 1e6   # garbage in the unused tail of the last page
    vp[table[0, 1], :, 5:, :] = -1e6
    out1 = oracle.decode_attention(q, kp, vp, table, lens, F32)
    assert np.array_equal(out0, out1)


def test_bad_page_table_is_rejected(oracle):
    q = np.zeros((1, 1, 4), dtype=np.float32)
    kp = np.zeros((1, 1, P, 4), dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.decode_attention(q, kp, kp, np.array([[3]], dtype=np.int32),
                                np.array([2], dtype=np.int32), F32)
