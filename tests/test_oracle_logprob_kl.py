"""Pins for the log-prob / KL oracle: hand-reduced closed forms, brute force on
tiny vocabularies, scipy's routines and invariants.  A dropped lse term, a
swapped KL direction, a wrong sign or a gather at the wrong index fails at
least one of them."""
import math
import os
import re
from fractions import Fraction

import numpy as np
import pytest
import scipy.special
import torch

from paper_2410_15651_amd import workloads as wl

F16, BF16, F32 = 0, 1, 2
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _eval_expr(expr: str) -> float:
    total = 0.0
    for term in expr.split("+"):
        m = re.fullmatch(r"\s*([-\d/]+)\*ln\(([\d/]+)\)\s*", term)
        assert m, term
        total += float(Fraction(m.group(1))) * math.log(float(Fraction(m.group(2))))
    return total


def test_golden_rational_distributions(oracle):
    for line in open(os.path.join(GOLDEN, "kl_closed_forms.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, a, r, tok, logp_e, kl_e = [f.strip() for f in line.split("|")]
        al = np.log(np.array([float(x) for x in a.split()])).astype(np.float32)[None]
        rl = np.log(np.array([float(x) for x in r.split()])).astype(np.float32)[None]
        logp, kl = oracle.token_logprobs_kl(al, rl, np.array([int(tok)], dtype=np.int32), F32)
        assert abs(logp[0] - _eval_expr(logp_e)) < 1e-6, name
        assert abs(kl[0] - _eval_expr(kl_e)) < 1e-6, name


def test_probabilities_sum_to_one(oracle):
    rng = np.random.default_rng(0)
    V = 11
    a = (rng.standard_normal((1, V)) * 3).astype(np.float32)
    r = (rng.standard_normal((1, V)) * 3).astype(np.float32)
    A = np.repeat(a, V, axis=0)
    R = np.repeat(r, V, axis=0)
    logp, _ = oracle.token_logprobs_kl(A, R, np.arange(V, dtype=np.int32), F32)
    assert abs(np.exp(logp).sum() - 1.0) < 1e-13


def test_brute_force_on_tiny_vocabularies(oracle):
    rng = np.random.default_rng(1)
    for V in (1, 2, 3, 5, 8):
        a = rng.uniform(-5, 5, size=(6, V)).astype(np.float32)
        r = rng.uniform(-5, 5, size=(6, V)).astype(np.float32)
        tok = rng.integers(0, V, size=6).astype(np.int32)
        logp, kl = oracle.token_logprobs_kl(a, r, tok, F32)
        for i in range(6):
            ea = [math.exp(float(x)) for x in a[i]]
            er = [math.exp(float(x)) for x in r[i]]
            p = [x / sum(ea) for x in ea]
            qd = [x / sum(er) for x in er]
            assert abs(logp[i] - math.log(p[tok[i]])) < 1e-13
            assert abs(kl[i] - sum(pi * math.log(pi / qi) for pi, qi in zip(p, qd))) < 1e-13


def test_scipy_logsumexp_log_softmax_rel_entr(oracle):
    rng = np.random.default_rng(2)
    N, V = 7, 1000
    a = (rng.standard_normal((N, V)) * 3).astype(np.float32)
    r = (rng.standard_normal((N, V)) * 3).astype(np.float32)
    tok = rng.integers(0, V, size=N).astype(np.int32)
    logp, kl = oracle.token_logprobs_kl(a, r, tok, F32)
    a64, r64 = a.astype(np.float64), r.astype(np.float64)
    np.testing.assert_allclose(logp, a64[np.arange(N), tok] - scipy.special.logsumexp(a64, axis=1), rtol=1e-12)
    lsa = scipy.special.log_softmax(a64, axis=1)
    np.testing.assert_allclose(logp, lsa[np.arange(N), tok], rtol=1e-12)
    p = scipy.special.softmax(a64, axis=1)
    qd = scipy.special.softmax(r64, axis=1)
    np.testing.assert_allclose(kl, scipy.special.rel_entr(p, qd).sum(axis=1), rtol=1e-10)


def test_uniform_logits(oracle):
    V = 37
    a = np.full((2, V), 1.25, dtype=np.float32)
    r = np.full((2, V), -3.0, dtype=np.float32)
    logp, kl = oracle.token_logprobs_kl(a, r, np.array([0, V - 1], dtype=np.int32), F32)
    np.testing.assert_allclose(logp, -math.log(V), rtol=1e-14)
    assert np.abs(kl).max() < 1e-15


def test_two_way_closed_form(oracle):
    for x in (-4.0, -0.5, 0.0, 2.0, 9.0):
        a = np.array([[x, 0.0]], dtype=np.float32)
        logp, _ = oracle.token_logprobs_kl(a, a, np.array([0], dtype=np.int32), F32)
        assert abs(logp[0] + math.log1p(math.exp(-x))) < 1e-14


def test_uniform_actor_kl_closed_form(oracle):
    rng = np.random.default_rng(3)
    V = 64
    a = np.zeros((1, V), dtype=np.float32)
    r = (rng.standard_normal((1, V)) * 2).astype(np.float32)
    _, kl = oracle.token_logprobs_kl(a, r, np.array([0], dtype=np.int32), F32)
    log_q = scipy.special.log_softmax(r.astype(np.float64), axis=1)
    assert abs(kl[0] - (-math.log(V) - log_q.mean())) < 1e-13


def test_kl_of_identical_rows_is_exactly_zero_and_kl_is_nonnegative(oracle):
    rng = np.random.default_rng(4)
    a = (rng.standard_normal((5, 501)) * 3).astype(np.float32)
    r = (rng.standard_normal((5, 501)) * 3).astype(np.float32)
    tok = np.zeros(5, dtype=np.int32)
    _, kl_same = oracle.token_logprobs_kl(a, a.copy(), tok, F32)
    assert (kl_same == 0.0).all()
    _, kl = oracle.token_logprobs_kl(a, r, tok, F32)
    assert (kl > 0).all()


def test_direction_is_actor_relative_to_reference(oracle):
    # p = (1/2, 1/2), q = (1/10, 9/10): KL(p||q) = ln(5/3), KL(q||p) is different.
    a = np.log(np.array([[1.0, 1.0]])).astype(np.float32)
    r = np.log(np.array([[1.0, 9.0]])).astype(np.float32)
    _, kl = oracle.token_logprobs_kl(a, r, np.array([0], dtype=np.int32), F32)
    assert abs(kl[0] - math.log(5 / 3)) < 1e-6
    _, kl_rev = oracle.token_logprobs_kl(r, a, np.array([0], dtype=np.int32), F32)
    assert abs(kl_rev[0] - (0.1 * math.log(0.2) + 0.9 * math.log(1.8))) < 1e-6


def test_independent_shifts_change_nothing(oracle):
    rng = np.random.default_rng(5)
    a = np.round(rng.standard_normal((3, 200)) * 24) / 8
    r = np.round(rng.standard_normal((3, 200)) * 24) / 8
    tok = rng.integers(0, 200, size=3).astype(np.int32)
    l0, k0 = oracle.token_logprobs_kl(a.astype(np.float32), r.astype(np.float32), tok, F32)
    l1, k1 = oracle.token_logprobs_kl((a + 7.5).astype(np.float32), (r - 11.25).astype(np.float32), tok, F32)
    np.testing.assert_allclose(l0, l1, rtol=0, atol=1e-12)
    np.testing.assert_allclose(k0, k1, rtol=0, atol=1e-12)


def test_padding_tokens_give_zeros(oracle):
    rng = np.random.default_rng(6)
    a = rng.standard_normal((4, 9)).astype(np.float32)
    r = rng.standard_normal((4, 9)).astype(np.float32)
    logp, kl = oracle.token_logprobs_kl(a, r, np.array([-1, 3, 9, -100], dtype=np.int32), F32)
    assert logp[0] == 0 and kl[0] == 0 and logp[2] == 0 and kl[2] == 0 and logp[3] == 0
    assert logp[1] < 0 and kl[1] > 0


def test_minus_infinity_logits(oracle):
    ninf = -np.inf
    a = np.array([[0.0, ninf, 0.0]], dtype=np.float32)
    r = np.array([[0.0, 0.0, 0.0]], dtype=np.float32)
    logp, kl = oracle.token_logprobs_kl(a, r, np.array([0], dtype=np.int32), F32)
    assert abs(logp[0] + math.log(2)) < 1e-15
    assert abs(kl[0] - math.log(1.5)) < 1e-15          # p=(1/2,0,1/2), q uniform
    logp, kl = oracle.token_logprobs_kl(r, a, np.array([1], dtype=np.int32), F32)
    assert kl[0] == np.inf                               # reference forbids a token the actor allows
    logp, _ = oracle.token_logprobs_kl(a, r, np.array([1], dtype=np.int32), F32)
    assert logp[0] == ninf


def test_row_stride_and_16bit_inputs(oracle):
    rng = np.random.default_rng(7)
    N, V, stride = 5, 40, 48
    for code, tdt in ((BF16, torch.bfloat16), (F16, torch.float16)):
        at = torch.from_numpy(rng.standard_normal((N, stride)).astype(np.float32) * 3).to(tdt)
        rt = torch.from_numpy(rng.standard_normal((N, stride)).astype(np.float32) * 3).to(tdt)
        tok = rng.integers(0, V, size=N).astype(np.int32)
        logp, kl = oracle.token_logprobs_kl(wl.to_storage(at), wl.to_storage(rt), tok, code, vocab=V)
        a64 = at.double().numpy()[:, :V]
        r64 = rt.double().numpy()[:, :V]
        np.testing.assert_allclose(logp, scipy.special.log_softmax(a64, axis=1)[np.arange(N), tok], rtol=1e-12)
        np.testing.assert_allclose(
            kl, scipy.special.rel_entr(scipy.special.softmax(a64, axis=1),
                                       scipy.special.softmax(r64, axis=1)).sum(axis=1), rtol=1e-10)


def test_fused_single_pass_identity_holds(oracle):
    """The GPU kernel evaluates KL as sum p (a - r) - lse_a + lse_r; the oracle
    sums the definition term by term.  Check here, on the CPU, that the two are
    the same number, so that a GPU/oracle mismatch cannot be blamed on algebra."""
    rng = np.random.default_rng(8)
    a = (rng.standard_normal((4, 3000)) * 3).astype(np.float32)
    r = (a + rng.standard_normal((4, 3000)).astype(np.float32) * 0.1).astype(np.float32)
    _, kl = oracle.token_logprobs_kl(a, r, np.zeros(4, dtype=np.int32), F32)
    a64, r64 = a.astype(np.float64), r.astype(np.float64)
    p = scipy.special.softmax(a64, axis=1)
    fused = (p * (a64 - r64)).sum(1) - scipy.special.logsumexp(a64, axis=1) + scipy.special.logsumexp(r64, axis=1)
    np.testing.assert_allclose(kl, fused, rtol=1e-9, atol=1e-15)


def test_bad_arguments_are_rejected(oracle):
    a = np.zeros((2, 4), dtype=np.float32)
    with pytest.raises(TypeError):
        oracle.token_logprobs_kl(a.astype(np.float64), a, np.zeros(2, dtype=np.int32), F32)
    with pytest.raises(ValueError):
        oracle.token_logprobs_kl(a, a, np.zeros(2, dtype=np.int32), F32, vocab=5)


# ------------------------------------------------------------ reward shaping ----
def test_reference_logprob_closed_form_and_scipy(oracle):
    """Logits = ln(integers): log p_ref(tok) = ln(r_tok / sum r)."""
    for line in open(os.path.join(GOLDEN, "kl_closed_forms.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, a, r, tok, _, _ = [f.strip() for f in line.split("|")]
        ai = [int(x) for x in a.split()]
        ri = [int(x) for x in r.split()]
        al = np.log(np.array(ai, dtype=np.float64)).astype(np.float32)[None]
        rl = np.log(np.array(ri, dtype=np.float64)).astype(np.float32)[None]
        ref_logp, _ = oracle.token_rewards(al, rl, np.array([int(tok)], dtype=np.int32), F32, 0.0, False)
        assert abs(ref_logp[0] - math.log(Fraction(ri[int(tok)], sum(ri)))) < 1e-6, name
    rng = np.random.default_rng(20)
    a = (rng.standard_normal((6, 300)) * 3).astype(np.float32)
    r = (rng.standard_normal((6, 300)) * 3).astype(np.float32)
    tok = rng.integers(0, 300, 6).astype(np.int32)
    ref_logp, _ = oracle.token_rewards(a, r, tok, F32, 0.0, False)
    np.testing.assert_allclose(ref_logp, scipy.special.log_softmax(r.astype(np.float64), axis=1)[np.arange(6), tok],
                               rtol=1e-12)


def test_sampled_penalty_averages_to_the_full_kl(oracle):
    """E_{tok ~ actor}[log p_a(tok) - log p_r(tok)] is the KL of the row: run every
    token of a small vocabulary through the sampled-penalty reward and average
    with the actor's probabilities (from scipy)."""
    rng = np.random.default_rng(21)
    V = 13
    a = (rng.standard_normal((1, V)) * 2).astype(np.float32)
    r = (rng.standard_normal((1, V)) * 2).astype(np.float32)
    A, R = np.repeat(a, V, axis=0), np.repeat(r, V, axis=0)
    toks = np.arange(V, dtype=np.int32)
    _, reward = oracle.token_rewards(A, R, toks, F32, 1.0, True)        # reward = -penalty
    p = scipy.special.softmax(a.astype(np.float64)[0])
    _, kl = oracle.token_logprobs_kl(a, r, np.zeros(1, dtype=np.int32), F32)
    assert abs(-(p * reward).sum() - kl[0]) < 1e-13
    # and each sampled penalty is the difference of the two log-probabilities
    logp, _ = oracle.token_logprobs_kl(A, R, toks, F32)
    ref_logp, _ = oracle.token_rewards(A, R, toks, F32, 0.0, False)
    np.testing.assert_allclose(-reward, logp - ref_logp, rtol=0, atol=1e-14)


def test_reward_is_affine_in_coefficient_and_terminal_score(oracle):
    rng = np.random.default_rng(22)
    N, V = 9, 50
    a = (rng.standard_normal((N, V)) * 2).astype(np.float32)
    r = (rng.standard_normal((N, V)) * 2).astype(np.float32)
    tok = rng.integers(0, V, N).astype(np.int32)
    term = np.zeros(N)
    term[[2, 8]] = [1.75, -0.5]
    _, kl = oracle.token_logprobs_kl(a, r, tok, F32)
    for sampled in (False, True):
        _, r0 = oracle.token_rewards(a, r, tok, F32, 0.0, sampled, terminal=term)
        assert np.array_equal(r0, term)                                   # no penalty: the terminal score alone
        _, r1 = oracle.token_rewards(a, r, tok, F32, 0.1, sampled, terminal=term)
        _, r2 = oracle.token_rewards(a, r, tok, F32, 0.3, sampled, terminal=term)
        _, r1n = oracle.token_rewards(a, r, tok, F32, 0.1, sampled)
        np.testing.assert_allclose(r1 - r1n, term, atol=1e-15)
        np.testing.assert_allclose((r1 - r2) / 0.2, (r0 - r1) / 0.1, rtol=1e-9, atol=1e-12)
        if not sampled:
            np.testing.assert_allclose(r1, term - 0.1 * kl, rtol=1e-13, atol=1e-15)
            assert (r1n <= 0).all()                                       # full KL is non-negative


def test_reward_padding_and_strides(oracle):
    rng = np.random.default_rng(23)
    N, V, stride = 4, 20, 24
    at = torch.from_numpy(rng.standard_normal((N, stride)).astype(np.float32) * 3).to(torch.bfloat16)
    rt = torch.from_numpy(rng.standard_normal((N, stride)).astype(np.float32) * 3).to(torch.bfloat16)
    tok = np.array([3, -1, 19, V], dtype=np.int32)
    term = np.array([0.0, 5.0, 2.0, 5.0])
    ref_logp, reward = oracle.token_rewards(wl.to_storage(at), wl.to_storage(rt), tok, BF16, 0.2, True,
                                            terminal=term, vocab=V)
    assert ref_logp[1] == 0 and reward[1] == 0 and ref_logp[3] == 0 and reward[3] == 0
    a64, r64 = at.double().numpy()[:, :V], rt.double().numpy()[:, :V]
    la = scipy.special.log_softmax(a64, axis=1)
    lr = scipy.special.log_softmax(r64, axis=1)
    for i in (0, 2):
        assert abs(ref_logp[i] - lr[i, tok[i]]) < 1e-12
        assert abs(reward[i] - (term[i] - 0.2 * (la[i, tok[i]] - lr[i, tok[i]]))) < 1e-12
