"""Pins for the float64 oracle: closed forms, special cases that reduce to
library routines, invariants and brute force on tiny vocabularies.

None of these re-types the oracle's own formulas around its own output; each
compares against something fixed by the paper or by the mathematics:
  * log-softmax against scipy's routine,
  * the ratio rule (Eq. 7) at S_ctx == S_noctx, lambda = 1 against the textbook
    speculative-sampling test min(1, p/q),
  * the recovery distribution (Eq. 8) at beta = 1, T = 1 against the target
    distribution of Eq. 4 built from probabilities, not logits,
  * the closed form solution (Eq. 2) against random points of the simplex under
    the objective of Eq. 1,
  * first-rejection and whole-step output laws against exhaustive grids,
  * hand-derived rational worked examples stored under tests/golden/.
"""
import json
import os

import numpy as np
import pytest
from scipy.special import log_softmax, softmax

HERE = os.path.dirname(os.path.abspath(__file__))


def rand_block(rng, B, K, V, scale=2.0):
    G = (rng.normal(size=(B, K + 1, V)) * scale).astype(np.float32)
    Sp = (rng.normal(size=(B, K + 1, V)) * scale).astype(np.float32)
    Sm = (rng.normal(size=(B, K + 1, V)) * scale).astype(np.float32)
    d = rng.integers(0, V, (B, K)).astype(np.int32)
    u = rng.random((B, K + 1)).astype(np.float32)
    return G, Sp, Sm, d, u


def to_bf16_bits(x):
    """Round-to-nearest-even fp32 -> bf16 bit patterns (uint16), numpy only."""
    b = np.ascontiguousarray(x, np.float32).view(np.uint32).astype(np.uint64)
    r = (b + 0x7FFF + ((b >> 16) & 1)) >> 16
    return r.astype(np.uint16)


def bf16_bits_to_f64(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


# ---------------------------------------------------------------- log-softmax

@pytest.mark.parametrize("T", [1.0, 0.7, 2.5])
def test_draft_logprobs_match_scipy_log_softmax(oracle, T):
    rng = np.random.default_rng(1)
    G, Sp, Sm, d, u = rand_block(rng, 3, 5, 97)
    r = oracle.verify_block(G, Sp, Sm, d, u, lam=0.5, beta=1.0, temperature=T)
    Tf = float(np.float32(T))
    lg = log_softmax(G.astype(np.float64) / Tf, axis=-1)
    ls = log_softmax(Sm.astype(np.float64) / Tf, axis=-1)
    for b in range(3):
        for t in range(5):
            assert r["draft_logprobs"][b, t, 0] == pytest.approx(lg[b, t, d[b, t]], abs=1e-12)
            assert r["draft_logprobs"][b, t, 1] == pytest.approx(ls[b, t, d[b, t]], abs=1e-12)


def test_recovery_logprobs_normalise_and_shift_invariant(oracle):
    rng = np.random.default_rng(2)
    G, Sp, Sm, d, u = rand_block(rng, 4, 3, 211, scale=4.0)
    r0 = oracle.verify_block(G, Sp, Sm, d, u, beta=1.3, temperature=0.9)
    assert np.allclose(np.exp(r0["recovery_logprobs"]).sum(-1), 1.0, atol=1e-12)
    # adding a per-row constant to any logits row changes no probability.  The shifts are
    # dyadic so the shifted float32 logits stay exact for this scale.
    shift = rng.integers(-8, 8, size=(3, 4, 4, 1)).astype(np.float32) * 0.5
    q = lambda x: (np.round(x * 1024) / 1024).astype(np.float32)
    G, Sp, Sm = q(G), q(Sp), q(Sm)
    r0 = oracle.verify_block(G, Sp, Sm, d, u, beta=1.3, temperature=0.9)
    r1 = oracle.verify_block(G + shift[0], Sp + shift[1], Sm + shift[2], d, u, beta=1.3, temperature=0.9)
    assert np.array_equal(r0["accepted_len"], r1["accepted_len"])
    assert np.array_equal(r0["next_token"], r1["next_token"])
    assert np.allclose(r0["recovery_logprobs"], r1["recovery_logprobs"], atol=1e-10)
    assert np.allclose(r0["draft_logprobs"], r1["draft_logprobs"], atol=1e-10, equal_nan=True)


def test_large_offsets_and_peaked_rows_are_stable(oracle):
    rng = np.random.default_rng(3)
    G, Sp, Sm, d, u = rand_block(rng, 3, 4, 300, scale=8.0)
    q = lambda x: (np.round(x * 64) / 64).astype(np.float32)
    G, Sp, Sm = q(G), q(Sp), q(Sm)
    r0 = oracle.verify_block(G, Sp, Sm, d, u, beta=1.5)
    for off in (80.0, -80.0):
        o = np.float32(off)
        r1 = oracle.verify_block(G + o, Sp + o, Sm + o, d, u, beta=1.5)
        assert np.array_equal(r0["accepted_len"], r1["accepted_len"])
        assert np.array_equal(r0["next_token"], r1["next_token"])
        assert np.allclose(r0["recovery_logprobs"], r1["recovery_logprobs"], atol=1e-9)
        assert np.all(np.isfinite(r1["recovery_logprobs"]))


# ---------------------------------------------------------------- acceptance rule (Eq. 7)

def test_ratio_rule_reduces_to_standard_speculative_sampling(oracle):
    """S_ctx == S_noctx, lambda = 1, T = 1: alpha_t = min(1, p(y)/q(y)) with p the
    generalist's and q the drafter's distribution -- the textbook acceptance test."""
    rng = np.random.default_rng(4)
    B, K, V = 64, 6, 50
    G, _, Sm, d, u = rand_block(rng, B, K, V, scale=1.0)
    r = oracle.verify_block(G, Sm, Sm, d, u, lam=1.0, beta=1.0, temperature=1.0)
    p = softmax(G.astype(np.float64), axis=-1)
    q = softmax(Sm.astype(np.float64), axis=-1)
    seen_reject = seen_full = False
    for b in range(B):
        n = K
        for t in range(K):
            a = min(1.0, p[b, t, d[b, t]] / q[b, t, d[b, t]])
            assert r["alpha"][b, t] == pytest.approx(a, rel=1e-12)
            if u[b, t] > a:
                n = t
                break
        assert r["accepted_len"][b] == n
        assert np.all(np.isnan(r["alpha"][b, n + 1:]))
        seen_reject |= n < K
        seen_full |= n == K
    assert seen_reject and seen_full


def test_threshold_lambda_scales_the_ratio(oracle):
    rng = np.random.default_rng(5)
    G, Sp, Sm, d, u = rand_block(rng, 8, 1, 40, scale=1.0)
    u[:, 0] = 0.0  # always accept, so alpha is reported for every sequence
    p = softmax(G.astype(np.float64), axis=-1)[:, 0]
    q = softmax(Sm.astype(np.float64), axis=-1)[:, 0]
    for lam in (1.0, 0.5, 0.1, 0.01, 3.0):
        r = oracle.verify_block(G, Sp, Sm, d, u, lam=lam)
        lamf = float(np.float32(lam))
        want = np.minimum(1.0, p[np.arange(8), d[:, 0]] / (lamf * q[np.arange(8), d[:, 0]]))
        assert np.allclose(r["alpha"][:, 0], want, rtol=1e-12)


def test_acceptance_ignores_the_private_distribution(oracle):
    """P_SLM^+ cancels from the acceptance ratio: accepted_len cannot depend on S_ctx."""
    rng = np.random.default_rng(6)
    G, Sp, Sm, d, u = rand_block(rng, 32, 5, 60)
    r0 = oracle.verify_block(G, Sp, Sm, d, u)
    Sp2 = (rng.normal(size=Sp.shape) * 5).astype(np.float32)
    r1 = oracle.verify_block(G, Sp2, Sm, d, u)
    assert np.array_equal(r0["accepted_len"], r1["accepted_len"])
    assert np.array_equal(r0["alpha"], r1["alpha"], equal_nan=True)
    assert not np.allclose(r0["recovery_logprobs"], r1["recovery_logprobs"])


def test_accepted_len_monotone_in_lambda_and_limits(oracle):
    rng = np.random.default_rng(7)
    G, Sp, Sm, d, u = rand_block(rng, 64, 6, 80)
    u = np.maximum(u, np.float32(1e-3))
    prev = None
    for lam in (1e-30, 0.01, 0.1, 0.5, 1.0, 4.0, 1e30):
        n = oracle.verify_block(G, Sp, Sm, d, u, lam=lam)["accepted_len"]
        if prev is not None:
            assert np.all(n <= prev)  # a larger lambda is a stricter gate
        prev = n
        if lam == 1e-30:
            assert np.all(n == 6)
        if lam == 1e30:
            assert np.all(n == 0)


def test_equality_accepts(oracle):
    """Algorithm 1 accepts when the uniform is <= alpha: u = 0 always passes and so does
    a uniform exactly equal to an alpha that float32 represents."""
    V = 4
    G = np.zeros((1, 2, V), np.float32)
    Sm = np.zeros((1, 2, V), np.float32)
    d = np.zeros((1, 1), np.int32)
    # P_LLM = P_SLM^- = 1/4, lambda = 2 -> alpha = 0.5 exactly
    for uval, want in ((0.5, 1), (np.nextafter(np.float32(0.5), np.float32(1)), 0), (0.0, 1)):
        u = np.array([[uval, 0.3]], np.float32)
        r = oracle.verify_block(G, G, Sm, d, u, lam=2.0)
        assert r["alpha"][0, 0] == 0.5
        assert r["accepted_len"][0] == want


# ---------------------------------------------------------------- first rejection (Alg. 1 loop)

def test_first_rejection_law_on_uniform_grid(oracle):
    """For fixed drafts Pr[n = t] = (prod_{i<t} alpha_i)(1 - alpha_t), Pr[n = K] = prod alpha_i.
    Exhaustive midpoint grid over the K uniforms; alpha from the independent formula."""
    rng = np.random.default_rng(8)
    K, V, M = 3, 6, 40
    G1, _, Sm1, d1, _ = rand_block(rng, 1, K, V, scale=1.0)
    lam = 0.8
    p = softmax(G1.astype(np.float64), axis=-1)[0]
    q = softmax(Sm1.astype(np.float64), axis=-1)[0]
    alpha = np.array([min(1.0, p[t, d1[0, t]] / (float(np.float32(lam)) * q[t, d1[0, t]])) for t in range(K)])
    assert np.any(alpha < 1) and np.all(alpha > 0.02)
    grid = (np.arange(M) + 0.5) / M
    uu = np.stack(np.meshgrid(grid, grid, grid, indexing="ij"), -1).reshape(-1, K)
    B = uu.shape[0]
    u = np.concatenate([uu, np.full((B, 1), 0.5)], 1).astype(np.float32)
    rep = lambda x: np.ascontiguousarray(np.broadcast_to(x, (B,) + x.shape[1:]))
    r = oracle.verify_block(rep(G1), rep(G1), rep(Sm1), rep(d1), u, lam=lam)
    freq = np.bincount(r["accepted_len"], minlength=K + 1) / B
    want = [np.prod(alpha[:t]) * (1 - alpha[t]) for t in range(K)] + [np.prod(alpha)]
    assert np.allclose(freq, want, atol=1.5 * K / M)
    assert abs(freq.sum() - 1) < 1e-12


# ---------------------------------------------------------------- recovery distribution (Eq. 8)

def test_recovery_beta_zero_or_no_context_gain_is_the_generalist(oracle):
    rng = np.random.default_rng(9)
    G, Sp, Sm, d, u = rand_block(rng, 6, 3, 120)
    T = 0.8
    Tf = float(np.float32(T))
    r = oracle.verify_block(G, Sp, Sm, d, u, beta=0.0, temperature=T)
    n = r["accepted_len"]
    want = log_softmax(G[np.arange(6), n].astype(np.float64) / Tf, axis=-1)
    assert np.allclose(r["recovery_logprobs"], want, atol=1e-12)
    r = oracle.verify_block(G, Sm, Sm, d, u, beta=1.7, temperature=T)
    want = log_softmax(G[np.arange(6), r["accepted_len"]].astype(np.float64) / Tf, axis=-1)
    assert np.allclose(r["recovery_logprobs"], want, atol=1e-12)


def test_recovery_beta_one_equals_bayesian_target(oracle):
    """beta = 1, T = 1: Softmax(h_rec) must equal the target of Eq. 4,
    P* = P_LLM * P_SLM^+ / P_SLM^- renormalised, built from probabilities."""
    rng = np.random.default_rng(10)
    G, Sp, Sm, d, u = rand_block(rng, 8, 4, 77)
    r = oracle.verify_block(G, Sp, Sm, d, u, beta=1.0, temperature=1.0)
    n = r["accepted_len"]
    ar = np.arange(8)
    pl = softmax(G[ar, n].astype(np.float64), -1)
    pp = softmax(Sp[ar, n].astype(np.float64), -1)
    pm = softmax(Sm[ar, n].astype(np.float64), -1)
    star = pl * pp / pm
    star /= star.sum(-1, keepdims=True)
    assert np.allclose(np.exp(r["recovery_logprobs"]), star, rtol=1e-10, atol=1e-15)


def test_recovery_general_beta_is_tilted_generalist(oracle):
    """General beta: probabilities are P_LLM * (P^+/P^-)^beta renormalised (log of Eq. 4
    with the reward scaled by beta), again from probabilities rather than logits."""
    rng = np.random.default_rng(11)
    G, Sp, Sm, d, u = rand_block(rng, 5, 2, 33)
    for beta, T in ((0.5, 1.0), (1.5, 1.0), (2.5, 1.0), (-0.5, 1.0), (0.8, 0.7), (1.5, 2.0)):
        r = oracle.verify_block(G, Sp, Sm, d, u, beta=beta, temperature=T)
        n = r["accepted_len"]
        ar = np.arange(5)
        Tf = float(np.float32(T))
        # every distribution is tempered the same way: P_x = softmax(h_x / T)
        w = softmax(G[ar, n].astype(np.float64) / Tf, -1) * (
            softmax(Sp[ar, n].astype(np.float64) / Tf, -1) / softmax(Sm[ar, n].astype(np.float64) / Tf, -1)
        ) ** float(np.float32(beta))
        w /= w.sum(-1, keepdims=True)
        assert np.allclose(np.exp(r["recovery_logprobs"]), w, rtol=1e-10, atol=1e-15)


def test_recovery_distribution_maximises_the_fusion_objective(oracle):
    """Eq. 1 / Eq. 2 on V <= 8: with r = log P^+ - log P^-, the recovery distribution at
    beta = 1 maximises E_pi[r] - KL(pi || P_LLM) against random simplex points."""
    rng = np.random.default_rng(12)
    V = 7
    G, Sp, Sm, d, u = rand_block(rng, 1, 0, V, scale=1.0)
    r = oracle.verify_block(G, Sp, Sm, np.zeros((1, 0), np.int32), u, beta=1.0)
    pi = np.exp(r["recovery_logprobs"][0])
    pl = softmax(G[0, 0].astype(np.float64))
    rew = log_softmax(Sp[0, 0].astype(np.float64)) - log_softmax(Sm[0, 0].astype(np.float64))
    J = lambda x: float(np.sum(x * rew) - np.sum(x * np.log(x / pl)))
    best = J(pi)
    for _ in range(2000):
        x = rng.dirichlet(np.ones(V) * rng.choice([0.3, 1.0, 5.0]))
        x = np.clip(x, 1e-300, None)
        assert J(x) <= best + 1e-12
    # closed form: the optimum equals log of the partition function
    assert best == pytest.approx(np.log(np.sum(pl * np.exp(rew))), abs=1e-12)


# ---------------------------------------------------------------- sampling

def test_sampling_intervals_small_vocab(oracle):
    """Token j is returned exactly for u_s in [CDF[j-1], CDF[j]): probe both sides of every edge."""
    rng = np.random.default_rng(13)
    for V in (1, 2, 5, 8):
        G, Sp, Sm, _, _ = rand_block(rng, 1, 0, V, scale=1.0)
        pr = softmax(G[0, 0].astype(np.float64) + 0.5 * (Sp[0, 0].astype(np.float64) - Sm[0, 0].astype(np.float64)))
        cdf = np.cumsum(pr)
        probes = [(0.0, 0)]
        for j in range(V - 1):
            lo = np.nextafter(np.float32(cdf[j]), np.float32(0))
            if float(lo) >= cdf[j]:
                lo = np.nextafter(lo, np.float32(0))
            hi = np.nextafter(np.float32(cdf[j]), np.float32(1))
            if float(hi) <= cdf[j]:
                hi = np.nextafter(hi, np.float32(1))
            probes += [(float(lo), j), (float(hi), j + 1)]
        probes.append((float(np.nextafter(np.float32(1), np.float32(0))), V - 1))
        for us, want in probes:
            u = np.array([[us]], np.float32)
            r = oracle.verify_block(G, Sp, Sm, np.zeros((1, 0), np.int32), u, beta=0.5)
            assert r["accepted_len"][0] == 0
            assert r["next_token"][0] == want, (V, us, cdf)
            assert r["next_token_logprob"][0] == pytest.approx(np.log(pr[want]), abs=1e-12)
            assert r["sample_margin"][0] == pytest.approx(np.min(np.abs(cdf - us)), abs=1e-12)


def test_zero_probability_tokens_are_never_returned(oracle):
    V = 6
    G = np.array([[[0, -2000, 0, -2000, 0, -2000]]], np.float32)  # p = 1/3 at 0, 2, 4; exact 0 elsewhere
    z = np.zeros_like(G)
    for us in np.linspace(0, 0.9999, 97):
        r = oracle.verify_block(G, z, z, np.zeros((1, 0), np.int32), np.array([[us]], np.float32))
        assert r["next_token"][0] in (0, 2, 4)
    r = oracle.verify_block(G, z, z, np.zeros((1, 0), np.int32),
                            np.array([[np.nextafter(np.float32(1), np.float32(0))]], np.float32))
    assert r["next_token"][0] == 4
    # u_s = 0 with a zero-probability token at index 0: the comparison is strict (CDF > u_s)
    G = np.array([[[-2000, 0, -2000, 0]]], np.float32)
    z = np.zeros_like(G)
    r = oracle.verify_block(G, z, z, np.zeros((1, 0), np.int32), np.array([[0.0]], np.float32))
    assert r["next_token"][0] == 1


def test_whole_step_output_law_brute_force(oracle):
    """One drafted position, V = 6.  Drafts come from P^+ = softmax(S_ctx); enumerating every
    draft token over a fine grid of (u, u_s) the emitted token follows
        Pr[y] = P^+(y) alpha(y) + (1 - sum_y' P^+(y') alpha(y')) R(y),
    R = Softmax(h_rec) -- Algorithm 1 resamples from R itself, not from a residual."""
    rng = np.random.default_rng(14)
    V, M = 6, 96
    lam, beta = 0.9, 1.2
    G1, Sp1, Sm1, _, _ = rand_block(rng, 1, 1, V, scale=1.0)
    pl = softmax(G1[0, 0].astype(np.float64))
    pp = softmax(Sp1[0, 0].astype(np.float64))
    pm = softmax(Sm1[0, 0].astype(np.float64))
    alpha = np.minimum(1.0, pl / (float(np.float32(lam)) * pm))
    R = pl * (pp / pm) ** float(np.float32(beta))
    R /= R.sum()
    want = pp * alpha + (1 - np.sum(pp * alpha)) * R
    grid = (np.arange(M) + 0.5) / M
    uu = np.stack(np.meshgrid(grid, grid, indexing="ij"), -1).reshape(-1, 2).astype(np.float32)
    Bg = uu.shape[0]
    rep = lambda x: np.ascontiguousarray(np.broadcast_to(x, (Bg,) + x.shape[1:]))
    got = np.zeros(V)
    for y in range(V):
        d = np.full((Bg, 1), y, np.int32)
        r = oracle.verify_block(rep(G1), rep(Sp1), rep(Sm1), d, uu, lam=lam, beta=beta)
        emitted = np.where(r["accepted_len"] == 1, y, r["next_token"])
        got += pp[y] * np.bincount(emitted, minlength=V) / Bg
    assert abs(got.sum() - 1) < 1e-12
    assert np.allclose(got, want, atol=3.0 / M)
    # and it is NOT the Bayesian target in general (documented consequence of the paper's recovery rule)
    star = pl * pp / pm
    star /= star.sum()
    assert not np.allclose(want, star, atol=1e-3)


def test_bonus_token_when_all_accepted(oracle):
    rng = np.random.default_rng(15)
    G, Sp, Sm, d, u = rand_block(rng, 4, 3, 30)
    u[:, :3] = 0.0
    r = oracle.verify_block(G, Sp, Sm, d, u, beta=0.7)
    assert np.all(r["accepted_len"] == 3)
    h = G[:, 3].astype(np.float64) + float(np.float32(0.7)) * (Sp[:, 3].astype(np.float64) - Sm[:, 3].astype(np.float64))
    assert np.allclose(r["recovery_logprobs"], log_softmax(h, -1), atol=1e-12)
    cdf = np.cumsum(softmax(h, -1), -1)
    for b in range(4):
        assert r["next_token"][b] == int(np.searchsorted(cdf[b], u[b, 3], side="right"))


# ---------------------------------------------------------------- ragged lengths, padding, bad input

def test_padding_is_never_read(oracle):
    rng = np.random.default_rng(16)
    B, K, V = 6, 5, 64
    G, Sp, Sm, d, u = rand_block(rng, B, K, V)
    u[:, :K] = np.minimum(u[:, :K], np.float32(0.2))  # long accepted prefixes
    lens = np.array([0, 1, 3, 5, 2, 4], np.int32)
    r0 = oracle.verify_block(G, Sp, Sm, d, u, draft_len=lens)
    G2, Sp2, Sm2, d2, u2 = G.copy(), Sp.copy(), Sm.copy(), d.copy(), u.copy()
    for b in range(B):
        G2[b, lens[b] + 1:] = np.nan
        Sp2[b, lens[b] + 1:] = np.nan
        Sm2[b, lens[b] + 1:] = np.nan
        d2[b, lens[b]:] = -7
        u2[b, lens[b]:K] = np.nan
    r1 = oracle.verify_block(G2, Sp2, Sm2, d2, u2, draft_len=lens)
    for k in ("accepted_len", "next_token", "next_token_logprob", "recovery_logprobs", "draft_logprobs", "alpha"):
        assert np.array_equal(r0[k], r1[k], equal_nan=True), k
    assert np.all(r0["accepted_len"] <= lens)
    assert r0["accepted_len"][0] == 0
    # a ragged call equals the dense call on the truncated sequence
    for b in range(B):
        k = int(lens[b])
        rb = oracle.verify_block(G[b:b + 1, :k + 1], Sp[b:b + 1, :k + 1], Sm[b:b + 1, :k + 1], d[b:b + 1, :k],
                                 np.concatenate([u[b:b + 1, :k], u[b:b + 1, K:]], 1))
        assert rb["accepted_len"][0] == r0["accepted_len"][b]
        assert rb["next_token"][0] == r0["next_token"][b]


def test_bad_sequences_are_flagged_not_fatal(oracle):
    rng = np.random.default_rng(17)
    G, Sp, Sm, d, u = rand_block(rng, 4, 3, 20)
    lens = np.array([3, 4, -1, 2], np.int32)  # 4 > k_max, -1 < 0
    d[3, 1] = 20  # out of vocabulary inside the valid prefix
    d[0, 2] = 19
    r = oracle.verify_block(G, Sp, Sm, d, u, draft_len=lens)
    assert list(r["accepted_len"][1:]) == [-1, -1, -1]
    assert list(r["next_token"][1:]) == [-1, -1, -1]
    assert r["accepted_len"][0] >= 0 and np.isnan(r["next_token_logprob"][1])


def test_bf16_inputs_are_widened_exactly(oracle):
    rng = np.random.default_rng(18)
    G, Sp, Sm, d, u = rand_block(rng, 3, 4, 130, scale=3.0)
    gb, pb, mb = to_bf16_bits(G), to_bf16_bits(Sp), to_bf16_bits(Sm)
    r16 = oracle.verify_block(gb, pb, mb, d, u, beta=0.8, temperature=0.7)
    f = lambda bits: bf16_bits_to_f64(bits).astype(np.float32)  # bf16 values are exact in fp32
    r32 = oracle.verify_block(f(gb), f(pb), f(mb), d, u, beta=0.8, temperature=0.7)
    for k in r16:
        assert np.array_equal(r16[k], r32[k], equal_nan=True), k
    # rounding helper itself: 1 + 2^-8 is a tie and goes to even (1.0); 1 + 3*2^-9 rounds up
    assert bf16_bits_to_f64(to_bf16_bits(np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -9], np.float32))).tolist() == [1.0, 1 + 2.0 ** -7]


def test_threads_do_not_change_results(oracle):
    rng = np.random.default_rng(19)
    G, Sp, Sm, d, u = rand_block(rng, 16, 4, 200)
    r1 = oracle.verify_block(G, Sp, Sm, d, u, num_threads=1)
    r4 = oracle.verify_block(G, Sp, Sm, d, u, num_threads=4)
    for k in r1:
        assert np.array_equal(r1[k], r4[k], equal_nan=True)


# ---------------------------------------------------------------- hand-derived worked examples

def test_golden_rational_examples(oracle):
    """tests/golden/rational_examples.json: logits are logs of small integers, so every
    probability, alpha and CDF edge is a hand-computed rational (derivations in the file)."""
    with open(os.path.join(HERE, "golden", "rational_examples.json")) as f:
        cases = json.load(f)["cases"]
    assert len(cases) >= 4
    for c in cases:
        lg = lambda w: np.log(np.array(w, np.float64)).astype(np.float32)[None]
        G, Sp, Sm = lg(c["w_llm"]), lg(c["w_slm_ctx"]), lg(c["w_slm_noctx"])
        d = np.array([c["draft"]], np.int32)
        u = np.array([c["uniforms"]], np.float32)
        r = oracle.verify_block(G, Sp, Sm, d, u, lam=c["lambda"], beta=c["beta"], temperature=1.0)
        assert r["accepted_len"][0] == c["accepted_len"], c["name"]
        assert r["next_token"][0] == c["next_token"], c["name"]
        for t, a in enumerate(c["alpha"]):
            assert r["alpha"][0, t] == pytest.approx(a, rel=1e-6), c["name"]  # float32 logs of integers
        assert np.allclose(np.exp(r["recovery_logprobs"][0]), c["recovery_probs"], rtol=1e-6), c["name"]


# ---------------------------------------------------------------- greedy decoding (the paper's evaluation setting)

def test_greedy_takes_argmax_of_recovery_logits(oracle):
    """The paper decodes greedily in its experiments; the deterministic form of the sampling step of Algorithm 1, phase 3,
    is the mode of that distribution: argmax of Eq. 8, independent of temperature and of the sampling uniform."""
    rng = np.random.default_rng(21)
    G, Sp, Sm, d, u = rand_block(rng, 16, 3, 90)
    for beta, T in ((1.0, 1.0), (0.5, 0.7), (2.0, 3.0), (0.0, 1.0)):
        r = oracle.verify_block(G, Sp, Sm, d, u, beta=beta, temperature=T, greedy=True)
        rs = oracle.verify_block(G, Sp, Sm, d, u, beta=beta, temperature=T, greedy=False)
        assert np.array_equal(r["accepted_len"], rs["accepted_len"])  # the ratio test is untouched
        assert np.array_equal(r["recovery_logprobs"], rs["recovery_logprobs"])
        n = r["accepted_len"]
        ar = np.arange(16)
        # mode of the recovery distribution, from the independently pinned log-probs
        assert np.array_equal(r["next_token"], np.argmax(rs["recovery_logprobs"], axis=-1))
        h = G[ar, n].astype(np.float64) + float(np.float32(beta)) * (Sp[ar, n].astype(np.float64) - Sm[ar, n].astype(np.float64))
        assert np.array_equal(r["next_token"], np.argmax(h, axis=-1))
        assert np.allclose(r["next_token_logprob"], rs["recovery_logprobs"][ar, r["next_token"]], atol=0)
        u2 = u.copy()
        u2[:, -1] = rng.random(16).astype(np.float32)
        assert np.array_equal(r["next_token"], oracle.verify_block(G, Sp, Sm, d, u2, beta=beta, temperature=T, greedy=True)["next_token"])


def test_greedy_ties_go_to_the_lowest_index(oracle):
    G = np.array([[[1.0, 3.0, 3.0, -1.0, 3.0]]], np.float32)
    z = np.zeros_like(G)
    r = oracle.verify_block(G, z, z, np.zeros((1, 0), np.int32), np.array([[0.99]], np.float32), greedy=True)
    assert r["next_token"][0] == 1
    # steering breaks the tie: beta * (S_ctx - S_noctx) lifts index 4
    Sp = np.array([[[0, 0, 0, 0, 0.5]]], np.float32)
    r = oracle.verify_block(G, Sp, z, np.zeros((1, 0), np.int32), np.array([[0.0]], np.float32), greedy=True, beta=1.0)
    assert r["next_token"][0] == 4


# ---------------------------------------------------------------- deployment split: cloud top-k, edge resample

def test_cloud_topk_matches_a_library_sort(oracle):
    rng = np.random.default_rng(31)
    G, Sp, Sm, d, u = rand_block(rng, 5, 2, 300)
    G[0, 1, 7] = G[0, 1, 3] = G[0, 1, 250] = 9.0  # ties inside the top-k
    Sm[0, 1, [3, 7, 250]] = 0.0
    row = np.array([1, 0, 2, 1, -1], np.int32)
    beta = 0.8
    idx, val = oracle.cloud_topk(G, Sm, row, beta=beta, topk=32)
    for b in range(4):
        h = G[b, row[b]].astype(np.float64) - float(np.float32(beta)) * Sm[b, row[b]].astype(np.float64)
        order = np.lexsort((np.arange(300), -h))[:32]  # by decreasing value, then increasing id
        assert np.array_equal(idx[b], order)
        assert np.array_equal(val[b], h[order].astype(np.float32))
    assert list(idx[0][:3]) == [3, 7, 250]
    assert np.all(idx[4] == -1) and np.all(np.isneginf(val[4]))
    # fewer tokens than slots
    idx, val = oracle.cloud_topk(G[:, :, :5].copy(), Sm[:, :, :5].copy(), row, beta=beta, topk=8)
    assert np.all(idx[0, 5:] == -1) and np.all(idx[0, :5] >= 0) and sorted(idx[0, :5]) == [0, 1, 2, 3, 4]


def test_split_recovery_with_full_payload_equals_eq8(oracle):
    """h_cloud + beta*h^+ = h_LLM + beta*(h^+ - h^-): with k = V nothing is truncated, so the edge's
    distribution must be the recovery distribution of the one-GPU block (up to the fp32 payload)."""
    rng = np.random.default_rng(32)
    B, V = 6, 40
    G, Sp, Sm, d, u = rand_block(rng, B, 2, V, scale=1.5)
    u[:, :2] = 0.0
    ref = oracle.verify_block(G, Sp, Sm, d, u, beta=1.3, temperature=0.8)  # all accepted: row 2
    row = ref["accepted_len"]
    idx, val = oracle.cloud_topk(G, Sm, row, beta=1.3, topk=V)
    e = oracle.edge_resample(idx, val, Sp, row, u[:, 2], beta=1.3, temperature=0.8)
    for b in range(B):
        assert np.allclose(e["cand_logprobs"][b], ref["recovery_logprobs"][b, idx[b]], atol=5e-6)
        assert np.isclose(np.exp(e["cand_logprobs"][b]).sum(), 1.0, atol=1e-12)


def test_edge_resample_law_and_truncation(oracle):
    """Tokens outside the payload are never drawn; inside it the draw follows softmax over the k candidates:
    every CDF interval is probed from both sides."""
    rng = np.random.default_rng(33)
    V, k = 50, 6
    G, Sp, Sm, _, _ = rand_block(rng, 1, 0, V, scale=1.0)
    row = np.zeros(1, np.int32)
    idx, val = oracle.cloud_topk(G, Sm, row, beta=0.7, topk=k)
    h = val[0].astype(np.float64) + float(np.float32(0.7)) * Sp[0, 0, idx[0]].astype(np.float64)
    pr = softmax(h / float(np.float32(1.5)))
    cdf = np.cumsum(pr)
    probes = [(0.0, 0)] + [(float(np.float32(cdf[j] - 1e-5)), j) for j in range(k)] + \
             [(float(np.float32(cdf[j] + 1e-5)), j + 1) for j in range(k - 1)]
    for us, want in probes:
        e = oracle.edge_resample(idx, val, Sp, row, np.array([us], np.float32), beta=0.7, temperature=1.5)
        assert e["next_token"][0] == idx[0, want]
        assert e["next_token_logprob"][0] == pytest.approx(np.log(pr[want]), abs=1e-12)
    e = oracle.edge_resample(idx, val, Sp, row, np.array([0.3], np.float32), beta=0.7, temperature=1.5, greedy=True)
    assert e["next_token"][0] == idx[0, int(np.argmax(h))]
    # flagged sequence
    e = oracle.edge_resample(idx, val, Sp, np.array([-1], np.int32), np.array([0.3], np.float32))
    assert e["next_token"][0] == -1 and np.isnan(e["next_token_logprob"][0])


def test_edge_resample_on_an_exact_cdf_edge(oracle):
    """Equal candidates make the k-way CDF exactly 1/k, 2/k, ... (k a power of two): a uniform that sits exactly
    on an edge belongs to the NEXT candidate, because the draw takes the first inclusive cumulative
    probability that exceeds it -- the same strict rule as the full-vocabulary draw."""
    V = 16
    G = np.full((1, 1, V), -30.0, np.float32)
    G[0, 0, [3, 7, 9, 12]] = 0.0          # four equal leaders at 0, so that log-sum-exp is exactly log 4
    Z = np.zeros_like(G)
    row = np.zeros(1, np.int32)
    idx, val = oracle.cloud_topk(G, Z, row, beta=1.0, topk=4)
    assert idx[0].tolist() == [3, 7, 9, 12]
    for us, want in [(0.0, 3), (0.25, 7), (0.5, 9), (0.75, 12), (0.24999999, 3), (0.4999999, 7)]:
        e = oracle.edge_resample(idx, val, Z, row, np.array([us], np.float32), beta=1.0, temperature=1.0)
        assert e["next_token"][0] == want, (us, e["next_token"][0])
        assert e["next_token_logprob"][0] == pytest.approx(np.log(0.25), abs=1e-15)


def test_edge_resample_with_a_uniform_of_one(oracle):
    """Same fallback on the edge side: the last payload entry that has any probability."""
    V = 12
    G = np.full((1, 1, V), -3.0e4, np.float32)
    G[0, 0, [2, 9]] = 0.0
    G[0, 0, [4, 5]] = -1.0e4          # in the payload, but with no probability next to the leaders
    Z = np.zeros_like(G)
    row = np.zeros(1, np.int32)
    idx, val = oracle.cloud_topk(G, Z, row, beta=1.0, topk=4)
    assert idx[0].tolist() == [2, 9, 4, 5]
    for us, want in [(1.0, 9), (0.5, 9), (0.25, 2)]:
        e = oracle.edge_resample(idx, val, Z, row, np.array([us], np.float32), beta=1.0, temperature=1.0)
        assert e["next_token"][0] == want, (us, e["next_token"][0])


def test_a_uniform_of_one_returns_the_last_token_with_probability(oracle):
    """uniforms are promised in [0, 1); a value of exactly 1 is not below any cumulative probability, and the
    draw then falls back to the last token that has any probability at all (never to one with none)."""
    V = 6
    G = np.full((1, 1, V), -1.0e4, np.float32)
    G[0, 0, 1] = G[0, 0, 3] = 0.0  # p = (0, 1/2, 0, 1/2, 0, 0) exactly: the CDF ends at exactly 1
    Z = np.zeros_like(G)
    d = np.zeros((1, 0), np.int32)
    for us, want in [(1.0, 3), (0.5, 3), (0.49999997, 1), (0.0, 1)]:
        r = oracle.verify_block(G, Z, Z, d, np.array([[us]], np.float32))
        assert r["next_token"][0] == want, (us, r["next_token"][0])
        assert r["next_token_logprob"][0] == pytest.approx(np.log(0.5), abs=1e-15)


def test_a_uniform_of_zero_returns_the_first_token_with_probability(oracle):
    """u = 0 with the head of the row ~300 nats under its maximum and a few masked tokens in front: the
    inverse CDF's strict comparison returns the first token whose probability is positive in double
    precision, with that token's own (very negative) log-prob -- checked against scipy's log-softmax."""
    V = 5000
    G = np.full((1, 1, V), -300.0, np.float32)
    G[0, 0, :3] = -np.inf
    G[0, 0, 2048:] = np.random.default_rng(2).normal(0, 1, V - 2048).astype(np.float32)
    Z = np.zeros_like(G)
    r = oracle.verify_block(G, Z, Z, np.zeros((1, 0), np.int32), np.zeros((1, 1), np.float32), beta=1.0)
    lp = log_softmax(G[0, 0].astype(np.float64))
    assert r["next_token"][0] == 3 == int(np.nonzero(np.exp(lp) > 0)[0][0])
    assert r["next_token_logprob"][0] == pytest.approx(lp[3], abs=1e-9) and lp[3] < -300


def test_tokens_masked_by_the_generalist_have_no_probability(oracle):
    """-inf in G: the token has probability zero under P_LLM, so it is rejected when drafted, and the recovery
    distribution is the softmax of Eq. 8 over the tokens that are left (scipy's softmax treats -inf the same way)."""
    rng = np.random.default_rng(51)
    B, K, V = 6, 3, 40
    G, Sp, Sm, d, u = rand_block(rng, B, K, V)
    mask = rng.random(G.shape) < 0.3
    G[mask] = -np.inf
    u = np.maximum(u, np.float32(1e-3))
    r = oracle.verify_block(G, Sp, Sm, d, u, lam=0.5, beta=0.8, temperature=0.9)
    beta, T = float(np.float32(0.8)), float(np.float32(0.9))
    for b in range(B):
        n = r["accepted_len"][b]
        for t in range(min(n + 1, K)):
            if mask[b, t, d[b, t]]:
                assert n == t                      # a masked draft token stops the block right there
        want = log_softmax((G[b, n].astype(np.float64) + beta * (Sp[b, n].astype(np.float64) - Sm[b, n])) / T)
        got = r["recovery_logprobs"][b]
        assert np.all(np.isneginf(got[mask[b, n]]))
        assert np.allclose(got[~mask[b, n]], want[~mask[b, n]], atol=1e-12)
        assert not mask[b, n, r["next_token"][b]]


def test_tokens_masked_in_every_model(oracle):
    """A vocabulary mask shared by the three models (-inf in G, S_ctx and S_noctx at the same ids): those tokens
    have no probability anywhere, the rest of the row is untouched -- the steering term of a masked token is
    nothing, not inf - inf.  A token masked for the specialist only (with and without context) keeps the
    generalist's logit."""
    rng = np.random.default_rng(52)
    B, K, V = 5, 2, 30
    G, Sp, Sm, d, u = rand_block(rng, B, K, V)
    common = rng.random((B, K + 1, V)) < 0.25
    spec_only = (rng.random((B, K + 1, V)) < 0.15) & ~common
    for b in range(B):
        for t in range(K):
            common[b, t, d[b, t]] = spec_only[b, t, d[b, t]] = False   # the drafted tokens stay ordinary
    G[common] = -np.inf
    Sp[common | spec_only] = -np.inf
    Sm[common | spec_only] = -np.inf
    r = oracle.verify_block(G, Sp, Sm, d, u, lam=0.5, beta=1.3, temperature=0.8)
    beta, T = float(np.float32(1.3)), float(np.float32(0.8))
    for b in range(B):
        n = r["accepted_len"][b]
        hl, hp, hm = (x[b, n].astype(np.float64) for x in (G, Sp, Sm))
        steer = np.where(np.isneginf(hp) & np.isneginf(hm), 0.0, np.where(np.isneginf(hp), 0.0, hp) - np.where(np.isneginf(hm), 0.0, hm))
        want = log_softmax((hl + beta * steer) / T)
        got = r["recovery_logprobs"][b]
        assert np.all(np.isneginf(got[common[b, n]])) and np.all(np.isfinite(got[~common[b, n]]))
        assert np.allclose(got[~common[b, n]], want[~common[b, n]], atol=1e-12)
        assert np.isclose(np.exp(got).sum(), 1.0, atol=1e-12)
    # greedy: never a masked token, and a specialist-only mask leaves the generalist's logit in the race
    g = oracle.verify_block(G, Sp, Sm, d, u, lam=0.5, beta=1.3, temperature=0.8, greedy=True)
    for b in range(B):
        n = g["accepted_len"][b]
        assert g["next_token"][b] == int(np.argmax(g["recovery_logprobs"][b])) and not common[b, n, g["next_token"][b]]


def test_cloud_topk_keeps_masked_tokens_masked(oracle):
    rng = np.random.default_rng(53)
    V, k = 40, 8
    G, _, Sm, _, _ = rand_block(rng, 2, 0, V)
    masked = np.zeros(V, bool)
    masked[[1, 5, 6, 30]] = True
    G[0, 0, masked] = -np.inf
    Sm[0, 0, masked] = -np.inf         # -inf - beta * (-inf) must not come back as a candidate
    G[1, 0, 6:] = -np.inf              # second row: fewer finite logits than payload slots
    Sm[1, 0, 6:] = -np.inf
    row = np.zeros(2, np.int32)
    idx, val = oracle.cloud_topk(G, Sm, row, beta=0.9, topk=k)
    h0 = G[0, 0].astype(np.float64) - float(np.float32(0.9)) * np.where(masked, 0.0, Sm[0, 0].astype(np.float64))
    want0 = np.lexsort((np.arange(V), -h0))[:k]
    assert idx[0].tolist() == want0.tolist() and not masked[idx[0]].any()
    assert np.array_equal(val[0], h0[want0].astype(np.float32))
    assert sorted(idx[1, :6].tolist()) == [0, 1, 2, 3, 4, 5] and idx[1, 6:].tolist() == [6, 7]
    assert np.all(np.isneginf(val[1, 6:]))


# ---------------------------------------------------------------- structure of the loop (Algorithm 1)

def test_a_block_equals_its_two_halves_verified_in_turn(oracle):
    """Algorithm 1 walks the positions in order and stops at the first rejection, so verifying K drafted
    tokens at once must agree with verifying the first K1 and, only if all of them pass, the remaining
    K - K1 on the rows that follow (row t scores draft token t; the row after the last accepted token
    yields the correction or bonus token)."""
    rng = np.random.default_rng(41)
    B, K, K1, V = 48, 7, 3, 23
    G, Sp, Sm, d, u = rand_block(rng, B, K, V, scale=1.2)
    whole = oracle.verify_block(G, Sp, Sm, d, u, lam=0.6, beta=0.9, temperature=1.1)
    # first half: rows 0..K1 (K1 draft rows + the row after them), same sampling uniform
    u1 = np.concatenate([u[:, :K1], u[:, -1:]], axis=1)
    first = oracle.verify_block(G[:, :K1 + 1], Sp[:, :K1 + 1], Sm[:, :K1 + 1], d[:, :K1], u1, lam=0.6, beta=0.9,
                                temperature=1.1)
    u2 = np.concatenate([u[:, K1:K], u[:, -1:]], axis=1)
    second = oracle.verify_block(G[:, K1:], Sp[:, K1:], Sm[:, K1:], d[:, K1:], u2, lam=0.6, beta=0.9, temperature=1.1)
    seen = set()
    for b in range(B):
        if first["accepted_len"][b] < K1:
            n, tok = first["accepted_len"][b], first["next_token"][b]
            seen.add("early")
        else:
            n, tok = K1 + second["accepted_len"][b], second["next_token"][b]
            seen.add("late")
        assert whole["accepted_len"][b] == n and whole["next_token"][b] == tok
    assert seen == {"early", "late"}


def test_sequences_do_not_interact(oracle):
    rng = np.random.default_rng(42)
    G, Sp, Sm, d, u = rand_block(rng, 9, 4, 31)
    dl = rng.integers(0, 5, 9).astype(np.int32)
    ref = oracle.verify_block(G, Sp, Sm, d, u, draft_len=dl, beta=1.4)
    perm = rng.permutation(9)
    got = oracle.verify_block(G[perm], Sp[perm], Sm[perm], d[perm], u[perm], draft_len=dl[perm], beta=1.4)
    for k in ("accepted_len", "next_token", "next_token_logprob", "recovery_logprobs"):
        assert np.array_equal(ref[k][perm], got[k]), k


# ---------------------------------------------------------------- frozen outputs

def test_oracle_reproduces_its_frozen_block():
    """tests/golden/oracle_block_fixture.json was written by tests/golden/make_oracle_fixture.py (numpy + oracle
    only).  It pins nothing to the paper by itself; it makes any later drift of the oracle's arithmetic visible."""
    import importlib.util

    spec = importlib.util.spec_from_file_location("make_oracle_fixture", os.path.join(HERE, "golden", "make_oracle_fixture.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    want = json.load(open(os.path.join(HERE, "golden", "oracle_block_fixture.json")))["outputs"]
    got = mod.run_all(*mod.build_inputs())
    assert got.keys() == want.keys()

    def same(a, b):
        if isinstance(a, list):
            return len(a) == len(b) and all(same(x, y) for x, y in zip(a, b))
        if isinstance(a, float) and isinstance(b, float):
            return a == b or abs(a - b) <= 1e-14 * max(1.0, abs(b))
        return a == b

    for case in want:
        for key in want[case]:
            assert same(got[case][key], want[case][key]), (case, key)
