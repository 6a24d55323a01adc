"""Pins for the sampling oracle: Philox known-answer vectors, the counter
convention, greedy = argmax, Gumbel-max frequencies against softmax, noise
moments, log-prob via scipy, determinism."""
import math
import os

import numpy as np
import scipy.special
import scipy.stats

F32 = 2
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_philox_known_answers(oracle):
    n = 0
    for line in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        ctr, key, out = [[int(w, 16) for w in part.split()] for part in line.split("|")]
        assert oracle.philox4x32_10(ctr, key).tolist() == out
        n += 1
    assert n == 3


def test_counter_convention_and_gumbel_transform(oracle):
    """Zero logits, T = 1: the perturbed score is the noise itself, and entry v
    of row i uses word v%4 of Philox(counter (v/4, i, offset lo, offset hi), key = seed)."""
    V, N = 11, 3
    seed, offset = 0x1234567890ABCDEF, (7 << 32) | 5
    _, _, pert = oracle.sample_tokens(np.zeros((N, V), dtype=np.float32), F32, 1.0, seed, offset,
                                      return_perturbed=True)
    for i in range(N):
        for v in range(V):
            r = oracle.philox4x32_10([v // 4, i, offset & 0xffffffff, offset >> 32],
                                     [seed & 0xffffffff, seed >> 32])
            u = ((int(r[v % 4]) >> 9) + 0.5) / 2 ** 23
            assert abs(pert[i, v] - (-math.log(-math.log(u)))) < 1e-12


def test_greedy_is_argmax_with_lowest_index_ties(oracle):
    rng = np.random.default_rng(0)
    a = (rng.standard_normal((20, 300)) * 3).astype(np.float32)
    a[3, 17] = a[3, 200] = 50.0
    tok, logp = oracle.sample_tokens(a, F32, 0.0, 1)
    assert tok.tolist() == a.argmax(axis=1).tolist() and tok[3] == 17
    np.testing.assert_allclose(logp, scipy.special.log_softmax(a.astype(np.float64), axis=1)[np.arange(20), tok],
                               rtol=1e-12)


def test_gumbel_max_frequencies_follow_softmax(oracle):
    logits = np.array([0.0, 1.0, -1.0, 2.5, 0.3, -3.0], dtype=np.float32)
    N = 60000
    for T in (1.0, 0.7, 2.0):
        tok, logp = oracle.sample_tokens(np.tile(logits, (N, 1)), F32, T, 99, 3)
        p = scipy.special.softmax(logits.astype(np.float64) / T)
        counts = np.bincount(tok, minlength=6)
        chi2 = ((counts - N * p) ** 2 / (N * p)).sum()
        assert chi2 < scipy.stats.chi2.ppf(1 - 1e-6, 5), (T, chi2)
        np.testing.assert_allclose(logp, np.log(p)[tok], rtol=1e-12)


def test_noise_is_independent_of_the_logits_and_has_gumbel_moments(oracle):
    rng = np.random.default_rng(1)
    a = rng.standard_normal((40, 500)).astype(np.float32)
    b = rng.standard_normal((40, 500)).astype(np.float32)
    ta, _, pa = oracle.sample_tokens(a, F32, 0.5, 5, 11, return_perturbed=True)
    tb, _, pb = oracle.sample_tokens(b, F32, 0.5, 5, 11, return_perturbed=True)
    noise = pa - a.astype(np.float64) / 0.5
    np.testing.assert_allclose(noise, pb - b.astype(np.float64) / 0.5, atol=1e-12)
    assert ta.tolist() == pa.argmax(axis=1).tolist()
    assert abs(noise.mean() - 0.5772156649) < 0.02 and abs(noise.var() - math.pi ** 2 / 6) < 0.05
    assert np.isfinite(noise).all()


def test_seed_offset_row_and_temperature_matter(oracle):
    a = np.zeros((64, 1000), dtype=np.float32)
    t0, _ = oracle.sample_tokens(a, F32, 1.0, 1, 0)
    t1, _ = oracle.sample_tokens(a, F32, 1.0, 1, 0)
    assert t0.tolist() == t1.tolist()                       # deterministic
    assert len(set(t0.tolist())) > 40                       # rows get different noise
    assert t0.tolist() != oracle.sample_tokens(a, F32, 1.0, 2, 0)[0].tolist()
    assert t0.tolist() != oracle.sample_tokens(a, F32, 1.0, 1, 1)[0].tolist()
    rng = np.random.default_rng(2)
    b = (rng.standard_normal((200, 50)) * 2).astype(np.float32)
    cold, _ = oracle.sample_tokens(b, F32, 0.01, 3)
    assert (cold == b.argmax(axis=1)).mean() > 0.97         # T -> 0 approaches greedy
    hot, _ = oracle.sample_tokens(b, F32, 100.0, 3)
    assert (hot == b.argmax(axis=1)).mean() < 0.2           # T -> inf approaches uniform


def test_strides_and_16bit_inputs(oracle):
    import torch
    from paper_2410_15651_amd import workloads as wl
    rng = np.random.default_rng(3)
    t = torch.from_numpy(rng.standard_normal((6, 24)).astype(np.float32) * 3).to(torch.bfloat16)
    tok, logp, pert = oracle.sample_tokens(wl.to_storage(t), 1, 0.8, 4, 0, vocab=20, return_perturbed=True)
    x = t.double().numpy()[:, :20] / 0.8
    assert pert.shape == (6, 20) and tok.tolist() == pert.argmax(axis=1).tolist()
    np.testing.assert_allclose(logp, scipy.special.log_softmax(x, axis=1)[np.arange(6), tok], rtol=1e-12)


# ------------------------------------------------------------------ top-k ----
HAND_ROW = np.array([[0.0, 1.0, -1.0, 2.5, 0.3, -3.0, 2.5, 0.9]], dtype=np.float32)


def test_topk_hand_cases(oracle):
    n = 0
    for line in open(os.path.join(GOLDEN, "topk_hand_cases.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, tau, count, token, logp = [x.strip() for x in line.split("|")]
        t, lp, th, c = oracle.sample_tokens_topk(HAND_ROW, F32, 0.0, int(k), 1)
        assert th[0] == float(np.float32(tau)) and c[0] == int(count) and t[0] == int(token), line
        assert abs(lp[0] - float(logp)) < 1e-7, line      # the row is stored in binary32 (0.3, 0.9 are rounded)
        n += 1
    assert n == 6


def test_topk_threshold_and_survivors_against_numpy(oracle):
    rng = np.random.default_rng(7)
    a = np.round(rng.standard_normal((30, 400)) * 3, 1).astype(np.float32)      # one decimal: plenty of ties
    for k in (1, 2, 7, 50, 399, 400, 1000):
        tok, logp, tau, count, pert = oracle.sample_tokens_topk(a, F32, 0.9, k, 11, 2, return_perturbed=True)
        kth = np.sort(a.astype(np.float64), axis=1)[:, ::-1][:, min(k, 400) - 1]
        assert np.array_equal(tau, kth)
        kept = a.astype(np.float64) >= kth[:, None]
        assert np.array_equal(count, kept.sum(axis=1)) and (count >= min(k, 400)).all()
        assert np.array_equal(np.isfinite(pert), kept)                           # removed entries: -inf
        assert tok.tolist() == pert.argmax(axis=1).tolist() and kept[np.arange(30), tok].all()
        x = np.where(kept, a.astype(np.float64) / 0.9, -np.inf)
        np.testing.assert_allclose(logp, scipy.special.log_softmax(x, axis=1)[np.arange(30), tok], rtol=1e-12)


def test_topk_with_everything_kept_is_the_plain_draw(oracle):
    rng = np.random.default_rng(8)
    a = (rng.standard_normal((25, 333)) * 2).astype(np.float32)
    for T in (0.0, 0.6, 1.5):
        t0, l0, p0 = oracle.sample_tokens(a, F32, T, 99, 5, return_perturbed=True)
        t1, l1, _, c1, p1 = oracle.sample_tokens_topk(a, F32, T, 333, 99, 5, return_perturbed=True)
        assert t0.tolist() == t1.tolist() and (c1 == 333).all()
        np.testing.assert_allclose(l1, l0, rtol=1e-12)
        np.testing.assert_array_equal(p1, p0)
        # and the survivors of a smaller k carry the same noise as in the plain draw
        _, _, _, _, p2 = oracle.sample_tokens_topk(a, F32, T, 10, 99, 5, return_perturbed=True)
        kept = np.isfinite(p2)
        np.testing.assert_array_equal(p2[kept], p0[kept])


def test_topk_of_one_is_the_argmax_whatever_the_noise(oracle):
    rng = np.random.default_rng(9)
    a = rng.permuted(np.tile(np.arange(200, dtype=np.float32) * 0.01, (40, 1)), axis=1)   # distinct values
    for T in (0.0, 1.0, 50.0):
        tok, logp, _, count = oracle.sample_tokens_topk(a, F32, T, 1, 3, 4)
        assert tok.tolist() == a.argmax(axis=1).tolist() and (count == 1).all()
        np.testing.assert_allclose(logp, 0.0, atol=1e-15)


def test_topk_frequencies_follow_the_survivors_softmax(oracle):
    logits = np.array([0.0, 1.0, -1.0, 2.5, 0.3, -3.0, 2.0, 0.9], dtype=np.float32)
    N, T, k = 60000, 0.8, 4
    tok, logp, tau, count = oracle.sample_tokens_topk(np.tile(logits, (N, 1)), F32, T, k, 1234, 6)
    kept = logits >= np.sort(logits)[::-1][k - 1]
    assert kept.sum() == 4 and (count == 4).all()
    p = scipy.special.softmax(np.where(kept, logits.astype(np.float64) / T, -np.inf))
    counts = np.bincount(tok, minlength=8)
    assert (counts[~kept] == 0).all()
    chi2 = ((counts[kept] - N * p[kept]) ** 2 / (N * p[kept])).sum()
    assert chi2 < scipy.stats.chi2.ppf(1 - 1e-6, 3), chi2
    np.testing.assert_allclose(logp, np.log(p[tok]), rtol=1e-12)


def test_topk_strides_16bit_inputs_and_bad_k(oracle):
    import torch
    from paper_2410_15651_amd import workloads as wl
    rng = np.random.default_rng(10)
    t = torch.from_numpy(rng.standard_normal((6, 24)).astype(np.float32) * 3).to(torch.bfloat16)
    tok, logp, tau, count, pert = oracle.sample_tokens_topk(wl.to_storage(t), 1, 0.8, 5, 4, 0, vocab=20,
                                                            return_perturbed=True)
    x = t.double().numpy()[:, :20]
    kth = np.sort(x, axis=1)[:, ::-1][:, 4]
    assert np.array_equal(tau, kth) and pert.shape == (6, 20)
    xm = np.where(x >= kth[:, None], x / 0.8, -np.inf)
    np.testing.assert_allclose(logp, scipy.special.log_softmax(xm, axis=1)[np.arange(6), tok], rtol=1e-12)
    import pytest
    with pytest.raises(ValueError):
        oracle.sample_tokens_topk(np.zeros((2, 4), dtype=np.float32), F32, 1.0, 0, 1)


def test_topk_survivor_sets_are_nested_and_the_draw_is_the_plain_one_when_it_survives(oracle):
    """Properties that hold for any logits: the threshold falls (weakly) and the
    survivor count grows with k and is at least k; removed entries can only
    remove the plain draw's winner, so whenever that winner is among the
    survivors the top-k draw is the same token (same noise, smaller contest),
    and otherwise it differs.  Checked over random rows with many ties."""
    rng = np.random.default_rng(2024)
    for trial in range(30):
        V = int(rng.integers(3, 400))
        levels = rng.normal(0, 2, size=int(rng.integers(2, 40)))
        x = rng.choice(levels, size=(5, V)).astype(np.float32)          # few distinct values: ties everywhere
        T = float(rng.choice([0.5, 1.0, 2.0]))
        plain, _, pert = oracle.sample_tokens(x, 2, T, 77, trial, return_perturbed=True)
        prev_tau, prev_cnt = None, None
        for k in sorted(set(int(v) for v in rng.integers(1, V + 1, size=6)) | {1, V}):
            tok, logp, tau, cnt = oracle.sample_tokens_topk(x, 2, T, k, 77, trial)
            assert (cnt >= k).all() and (cnt == (x >= tau[:, None]).sum(axis=1)).all()
            kth = -np.sort(-x, axis=1)[:, k - 1]
            assert (tau == kth).all()
            if prev_tau is not None:
                assert (tau <= prev_tau).all() and (cnt >= prev_cnt).all()
            prev_tau, prev_cnt = tau, cnt
            survives = x[np.arange(5), plain] >= tau
            assert (tok[survives] == plain[survives]).all()
            assert (tok[~survives] != plain[~survives]).all()
            assert (x[np.arange(5), tok] >= tau).all() and (logp <= 1e-12).all()
