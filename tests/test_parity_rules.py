"""CPU tests of the comparison rules themselves (tests/parity.py): what a near-threshold statistic may
excuse, and that the excused outcome must be the other admissible one.  The "GPU" outputs here are
fabricated from oracle runs; no kernel is involved."""
import numpy as np
import pytest

import parity


def _block(seed=0, B=4, K=3, V=6):
    rng = np.random.default_rng(seed)
    G = rng.normal(0, 1.5, (B, K + 1, V)).astype(np.float32)
    Sp = (G + rng.normal(0, 0.7, G.shape)).astype(np.float32)
    Sm = (G + rng.normal(0, 0.7, G.shape)).astype(np.float32)
    draft = rng.integers(0, V, (B, K)).astype(np.int32)
    u = rng.uniform(0.05, 0.95, (B, K + 1)).astype(np.float32)
    return G, Sp, Sm, draft, u


HP = dict(lam=0.5, beta=0.8, temperature=0.9)


def _run(oracle, G, Sp, Sm, draft, u):
    ora = oracle.verify_block(G, Sp, Sm, draft, u, **HP)
    return parity.attach_recheck(ora, oracle, G, Sp, Sm, draft, None, **HP)


def _as_gpu(ora):
    return {"accepted_len": ora["accepted_len"].copy(), "next_token": ora["next_token"].copy(),
            "next_token_logprob": ora["next_token_logprob"].astype(np.float32)}


def test_identical_outputs_pass_with_nothing_excused(oracle):
    G, Sp, Sm, draft, u = _block()
    ora = _run(oracle, G, Sp, Sm, draft, u)
    rep = parity.compare(_as_gpu(ora), ora, u)
    assert rep["excused_mismatches"] == 0 and rep["excused_outcomes"] == []


def test_a_wrong_token_far_from_any_edge_fails(oracle):
    G, Sp, Sm, draft, u = _block()
    ora = _run(oracle, G, Sp, Sm, draft, u)
    assert ora["sample_margin"][1] > 1e-4
    gpu = _as_gpu(ora)
    gpu["next_token"][1] = (gpu["next_token"][1] + 1) % G.shape[2]
    with pytest.raises(AssertionError, match="unexcused"):
        parity.compare(gpu, ora, u)


def _edge_case(oracle):
    """Sequence 0's sampling uniform is put 3e-7 above a CDF edge of its recovery row."""
    G, Sp, Sm, draft, u = _block(seed=3)
    ora = _run(oracle, G, Sp, Sm, draft, u)
    cdf = np.cumsum(np.exp(ora["recovery_logprobs"][0]))
    j = 2
    u[0, -1] = np.float32(cdf[j] + 3e-7)
    ora = _run(oracle, G, Sp, Sm, draft, u)
    assert ora["sample_margin"][0] < parity.NEAR
    return G, Sp, Sm, draft, u, ora


def test_near_cdf_edge_admits_the_neighbour_and_nothing_else(oracle):
    G, Sp, Sm, draft, u, ora = _edge_case(oracle)
    t = int(ora["next_token"][0])
    lp = ora["recovery_logprobs"][0]
    # the neighbour on the other side of the edge, with its own log-prob: admissible
    nb = t - 1 if float(u[0, -1]) >= np.cumsum(np.exp(lp))[t - 1] and t > 0 else t + 1
    gpu = _as_gpu(ora)
    gpu["next_token"][0] = nb
    gpu["next_token_logprob"][0] = np.float32(lp[nb])
    rep = parity.compare(gpu, ora, u)
    assert rep["excused_mismatches"] == 1 and rep["excused_outcomes"][0]["sample"]["gpu"] == nb
    assert set(rep["excused_outcomes"][0]["sample"]["admissible"]) == {t, nb}
    # the neighbour with the wrong log-prob: not admissible
    gpu["next_token_logprob"][0] = np.float32(lp[t] + 1e-3) if abs(lp[t] - lp[nb]) < 1e-3 else np.float32(lp[t])
    with pytest.raises(AssertionError, match="next_token_logprob"):
        parity.compare(gpu, ora, u)
    # a token two places away: not admissible although the sequence is near an edge
    far = (max(t, nb) + 1) % G.shape[2]
    if far in (t, nb):
        far = (far + 1) % G.shape[2]
    gpu["next_token"][0] = far
    gpu["next_token_logprob"][0] = np.float32(lp[far])
    with pytest.raises(AssertionError, match="not admissible"):
        parity.compare(gpu, ora, u)


def test_near_edge_does_not_excuse_a_different_accepted_len(oracle):
    G, Sp, Sm, draft, u, ora = _edge_case(oracle)
    gpu = _as_gpu(ora)
    gpu["accepted_len"][0] = (gpu["accepted_len"][0] + 1) % (draft.shape[1] + 1)
    with pytest.raises(AssertionError, match="unexcused"):
        parity.compare(gpu, ora, u)


@pytest.mark.parametrize("side", [+1, -1])
def test_near_threshold_accept_admits_exactly_the_flipped_continuation(oracle, side):
    G, Sp, Sm, draft, u = _block(seed=5, B=3, K=4, V=8)
    u[:, :-1] = 0.0                                   # everything accepted ...
    ora = _run(oracle, G, Sp, Sm, draft, u)
    cand = np.argwhere((ora["alpha"][:, :3] < 0.999) & (ora["alpha"][:, :3] > 1e-3))
    assert len(cand), "the seeded block should hold a position that is not accepted outright"
    s0, t = (int(x) for x in cand[0])
    a = ora["alpha"][s0, t]
    u[s0, t] = np.float32(a + side * 4e-7)            # ... except a coin toss at one position of one sequence
    ora = _run(oracle, G, Sp, Sm, draft, u)
    assert abs(ora["alpha"][s0, t] - float(u[s0, t])) < parity.NEAR
    # the other admissible outcome: the oracle with that one decision forced the other way
    oracle_accepts = ora["accepted_len"][s0] > t
    u2 = u.copy()
    u2[s0, t] = 1.0 if oracle_accepts else 0.0
    other = oracle.verify_block(G, Sp, Sm, draft, u2, **HP)
    assert other["accepted_len"][s0] != ora["accepted_len"][s0]
    gpu = _as_gpu(ora)
    for k in gpu:
        gpu[k][s0] = other[k][s0]
    rep = parity.compare(gpu, ora, u)
    assert rep["excused_mismatches"] == 1
    f = rep["excused_outcomes"][0]["forced"][0]
    assert f["position"] == t and f["gpu"] == ("reject" if oracle_accepts else "accept")
    # right accepted_len but the token of the oracle's original row: inadmissible unless the rows happen to agree
    if other["next_token"][s0] != ora["next_token"][s0]:
        gpu["next_token"][s0] = ora["next_token"][s0]
        with pytest.raises(AssertionError):
            parity.compare(gpu, ora, u)
    # an accepted_len that no flip of that decision produces
    gpu = _as_gpu(ora)
    gpu["accepted_len"][s0] = next(n for n in range(draft.shape[1] + 1)
                                   if n not in (ora["accepted_len"][s0], other["accepted_len"][s0]))
    with pytest.raises(AssertionError):
        parity.compare(gpu, ora, u)


def test_tolerance_is_plain_1e5_in_the_benchmark_range():
    assert np.all(parity.logprob_tol(np.array([0.0, -1.0, -17.0, -36.0, -40.0])) == 1e-5)
    assert parity.logprob_tol(-1000.0) > 1e-5
