"""Shared comparison of the HIP path against the float64 oracle (used by the GPU tests,
the smoke check and the benchmark's parity line).

Bar: log-probs within 1e-5 absolute; accepted_len and next_token bit-exact, except where a
test statistic lies within 1e-6 of its threshold.  There exactly two outcomes are admissible
and the check says which two:
  * an acceptance test with |alpha_t - u_t| < 1e-6 (and alpha_t < 1) may go either way.  The
    GPU's accepted_len must then be what the oracle gives with exactly that decision forced
    the GPU's way (the oracle is run again on that sequence with u_t replaced by 0 or 1), and
    token and log-prob are compared with that second oracle run;
  * a sampling uniform within 1e-6 of a CDF edge may fall on either side of it: the GPU's
    token must be one the inverse CDF returns for some uniform in [u - 1e-6, u + 1e-6], i.e.
    the oracle's token or its neighbour across that edge (zero-probability tokens skipped),
    and its log-prob must be the oracle's log-prob of that token.
Such outcomes are counted and listed in the report, never silently dropped; anything else is
an unexcused mismatch and fails.

Log-prob tolerance: 1e-5 absolute wherever |oracle log-prob| <= 40 (every value on the five
benchmark configurations).  Beyond that the float32 output itself cannot carry 1e-5 (half an
ulp at -100 is 3.8e-6, at -1000 3e-5), so only there half an fp32 ulp of the value is added.
"""
from __future__ import annotations

import numpy as np

LOGPROB_ATOL = 1e-5
FP32_HALF_ULP = 2.0 ** -24
LOGPROB_PLAIN_RANGE = 40.0
NEAR = 1e-6
MAX_FLIPS = 4  # near-threshold decisions one sequence may need forced before the outcomes agree


def logprob_tol(want):
    want = np.abs(np.asarray(want, dtype=np.float64))
    with np.errstate(invalid="ignore"):
        return np.where(want <= LOGPROB_PLAIN_RANGE, LOGPROB_ATOL, LOGPROB_ATOL + FP32_HALF_ULP * want)


def _np(x):
    if x is None or isinstance(x, np.ndarray):
        return x
    return x.detach().cpu().numpy()


def attach_recheck(ora, oracle, G, S_ctx, S_noctx, draft, draft_len, *, lam, beta, temperature, greedy=False):
    """Give an oracle result the means to run the oracle again on one of its sequences with a changed
    row of uniforms (host tensors, already restricted to the sequences of ``ora``)."""

    def recheck(i, u_row):
        return oracle.verify_block(G[i:i + 1], S_ctx[i:i + 1], S_noctx[i:i + 1], draft[i:i + 1],
                                   np.asarray(u_row, dtype=np.float32)[None, :], lam=lam, beta=beta,
                                   temperature=temperature,
                                   draft_len=None if draft_len is None else draft_len[i:i + 1],
                                   want_recovery_logprobs=True, num_threads=1, greedy=greedy)

    ora["_recheck"] = recheck
    return ora


def oracle_run(oracle, inp, *, lam, beta, temperature, seqs=None, want_recovery_logprobs=True, num_threads=8,
               greedy=False):
    """Run the oracle on host copies of the inputs (optionally only on sequences ``seqs``)."""
    sel = slice(None) if seqs is None else seqs
    dl = inp.get("draft_len")
    host = {k: inp[k][sel].cpu() for k in ("G", "S_ctx", "S_noctx", "draft", "uniforms")}
    hdl = None if dl is None else dl[sel].cpu()
    ora = oracle.verify_block(host["G"], host["S_ctx"], host["S_noctx"], host["draft"], host["uniforms"], lam=lam,
                              beta=beta, temperature=temperature, draft_len=hdl,
                              want_recovery_logprobs=want_recovery_logprobs, num_threads=num_threads, greedy=greedy)
    return attach_recheck(ora, oracle, host["G"], host["S_ctx"], host["S_noctx"], host["draft"], hdl, lam=lam,
                          beta=beta, temperature=temperature, greedy=greedy)


def _admissible_tokens(lp_row, us):
    """Tokens the inverse CDF returns for some uniform in [us - NEAR, us + NEAR]."""
    p = np.exp(lp_row)
    cdf = np.cumsum(p)
    pos = np.nonzero(p > 0)[0]

    def draw(x):
        j = int(np.searchsorted(cdf, x, side="right"))  # first j with cdf[j] > x
        return j if j < len(cdf) else int(pos[-1])

    lo, hi = draw(us - NEAR), draw(us + NEAR)
    return [int(j) for j in pos[(pos >= lo) & (pos <= hi)]]


def _validate_excused(i, n_g, tok_g, lp_g, ora, u_row, kmax, greedy_ok):
    """Sequence i (index into ``ora``) disagrees with the oracle.  Show that the GPU's outcome is the other
    admissible one, or raise.  Returns a description of both outcomes."""
    recheck = ora.get("_recheck")
    assert recheck is not None, "an excused mismatch needs a second oracle run to be validated"
    u_row = np.array(u_row, dtype=np.float32)
    cur = {k: (None if ora[k] is None else ora[k][i]) for k in
           ("accepted_len", "next_token", "next_token_logprob", "alpha", "recovery_logprobs")}
    what = {"sequence": int(i), "oracle": {"accepted_len": int(cur["accepted_len"]), "next_token": int(cur["next_token"])},
            "gpu": {"accepted_len": int(n_g), "next_token": int(tok_g)}, "forced": []}
    rerun = False
    for _ in range(MAX_FLIPS):
        n_o = int(cur["accepted_len"])
        if n_g == n_o:
            break
        t = min(n_g, n_o)  # the first position the two sides decide differently
        assert t < kmax, "accepted lengths differ beyond the last position"
        a, ut = float(cur["alpha"][t]), float(u_row[t])
        assert a < 1.0 and abs(a - ut) < NEAR, (
            f"sequence {i}: accepted_len gpu/oracle {n_g}/{n_o} but position {t} is not near its threshold "
            f"(alpha {a!r}, u {ut!r})")
        gpu_accepts = n_g > t
        what["forced"].append({"position": int(t), "alpha": a, "u": ut,
                               "admissible": [f"accept (u <= alpha): go on to position {t + 1}",
                                              f"reject: accepted_len = {t}"],
                               "gpu": "accept" if gpu_accepts else "reject"})
        u_row[t] = 0.0 if gpu_accepts else 1.0  # u = 0 always accepts; u = 1 rejects since alpha < 1
        r = recheck(i, u_row)
        cur = {k: (None if r[k] is None else r[k][0]) for k in cur}
        rerun = True
    assert n_g == int(cur["accepted_len"]), f"sequence {i}: accepted_len {n_g} is not reachable by flipping near-threshold tests"
    if cur["recovery_logprobs"] is None:
        r = recheck(i, u_row)
        cur = {k: (None if r[k] is None else r[k][0]) for k in cur}
    if tok_g != int(cur["next_token"]):
        assert greedy_ok, f"sequence {i}: greedy token gpu/oracle {tok_g}/{int(cur['next_token'])}"
        us = float(u_row[kmax])
        adm = _admissible_tokens(cur["recovery_logprobs"], us)
        assert tok_g in adm, (f"sequence {i}: token {tok_g} is not admissible for u = {us!r}: the inverse CDF gives "
                              f"{adm} over [u - 1e-6, u + 1e-6] (oracle {int(cur['next_token'])})")
        what["sample"] = {"u": us, "admissible": adm, "gpu": int(tok_g)}
    if lp_g is not None:
        want = float(cur["recovery_logprobs"][tok_g])
        assert abs(float(lp_g) - want) <= float(logprob_tol(want)), (
            f"sequence {i}: next_token_logprob {lp_g!r} vs oracle {want!r} for the admissible token {tok_g}")
    what["second_oracle_run"] = rerun
    return what


def compare(gpu_out, ora, uniforms, draft_len=None, seqs=None):
    """Element-by-element comparison.  Returns a report dict; raises AssertionError on any
    unexcused mismatch, inadmissible excused outcome, or log-prob outside tolerance."""
    sel = slice(None) if seqs is None else (seqs.cpu().numpy() if hasattr(seqs, "cpu") else seqs)
    n_g = _np(gpu_out["accepted_len"])[sel]
    tok_g = _np(gpu_out["next_token"])[sel]
    n_o, tok_o = ora["accepted_len"], ora["next_token"]
    u32 = _np(uniforms)[sel].astype(np.float32)
    u = u32.astype(np.float64)
    B, kmax = ora["alpha"].shape
    valid = n_o >= 0
    lp_tok_g = None if gpu_out.get("next_token_logprob") is None else _np(gpu_out["next_token_logprob"])[sel]

    # flagged sequences must be flagged identically
    assert np.array_equal(n_g[~valid], n_o[~valid]) and np.array_equal(tok_g[~valid], tok_o[~valid])

    alpha = ora["alpha"]
    with np.errstate(invalid="ignore"):
        near_acc = (np.abs(alpha - u[:, :kmax]) < NEAR) & (alpha < 1.0)  # NaN (untested) compares False
        near_samp = ora["sample_margin"] < NEAR
    mismatch = ((n_g != n_o) | (tok_g != tok_o)) & valid
    # what can excuse what: a different accepted_len needs a near-threshold acceptance test, a different
    # token alone a uniform near a CDF edge; which outcome the GPU took is validated below
    n_diff = (n_g != n_o) & valid
    tok_only = (tok_g != tok_o) & ~n_diff & valid
    bad = (n_diff & ~near_acc.any(axis=1)) | (tok_only & ~near_samp)
    assert not bad.any(), (
        f"unexcused mismatches at sequences {np.nonzero(bad)[0][:8]}: "
        f"n gpu/oracle {n_g[bad][:8]}/{n_o[bad][:8]}, token gpu/oracle {tok_g[bad][:8]}/{tok_o[bad][:8]}")
    greedy_ok = bool(np.isfinite(ora["sample_margin"][valid]).all()) if valid.any() else True
    outcomes = []
    for i in np.nonzero(mismatch)[0]:
        outcomes.append(_validate_excused(int(i), int(n_g[i]), int(tok_g[i]),
                                          None if lp_tok_g is None else lp_tok_g[i], ora, u32[i], kmax, greedy_ok))

    report = {
        "sequences": int(B),
        "near_threshold_accepts": int(near_acc.sum()),
        "near_threshold_samples": int(near_samp[valid].sum()),
        "excused_sequences": int(((near_acc.any(axis=1) | near_samp) & valid).sum()),
        "excused_mismatches": int(mismatch.sum()),
        "excused_outcomes_validated": len(outcomes),
        "excused_outcomes": outcomes[:8],
        "unexcused_mismatches": 0,
        "mean_accepted_len": float(n_o[valid].mean()) if valid.any() else 0.0,
    }
    same = valid & ~mismatch

    def check_lp(name, got, want, mask):
        with np.errstate(invalid="ignore"):  # rows of flagged sequences are never written and may hold any bits
            got = got.astype(np.float64)
        with np.errstate(invalid="ignore"):  # a masked token's log-prob is -inf on both sides
            err = np.abs(got - want)
        tol = logprob_tol(want)
        m = mask & np.isfinite(want)
        worst = float(err[m].max()) if m.any() else 0.0
        report["max_abs_err_" + name] = worst
        assert np.all(err[m] <= tol[m]), f"{name}: max |gpu - oracle| = {worst:.3e}"
        assert np.all(np.isfinite(got[m]))

    if lp_tok_g is not None:
        check_lp("next_token_logprob", lp_tok_g, ora["next_token_logprob"], same)
        assert np.all(np.isnan(lp_tok_g[~valid]))
    if gpu_out.get("draft_logprobs") is not None:
        got = _np(gpu_out["draft_logprobs"])[sel]
        want = ora["draft_logprobs"]
        K = np.full(B, kmax) if draft_len is None else _np(draft_len)[sel]
        pos = np.arange(kmax)[None, :, None] < K[:, None, None]
        mask = np.broadcast_to(pos & valid[:, None, None], want.shape)
        check_lp("draft_logprobs", got, want, mask)
        pad = np.broadcast_to(~pos & valid[:, None, None], want.shape)
        assert np.all(got[pad] == 0.0)
        assert np.all(np.isnan(got[~valid]))
    if gpu_out.get("recovery_logprobs") is not None and ora.get("recovery_logprobs") is not None:
        got = _np(gpu_out["recovery_logprobs"])[sel]
        want = ora["recovery_logprobs"]
        rows = (n_g == n_o) & valid  # same row => same distribution, whichever token was drawn
        check_lp("recovery_logprobs", got, want, np.broadcast_to(rows[:, None], want.shape))
    return report
