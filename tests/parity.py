"""Shared comparison of the HIP path against the float64 oracle (used by the GPU tests,
the smoke check and the benchmark's parity line).

Bar: log-probs within 1e-5 absolute (plus half an fp32 ulp of the stored value, which is
what writing the result as float32 costs); accepted_len and next_token bit-exact, except
for sequences touching a position whose test statistic lies within 1e-6 of its threshold.
Those are counted and reported, never silently dropped.
"""
from __future__ import annotations

import numpy as np

LOGPROB_ATOL = 1e-5
FP32_HALF_ULP = 2.0 ** -24
NEAR = 1e-6


def _np(x):
    if x is None or isinstance(x, np.ndarray):
        return x
    return x.detach().cpu().numpy()


def oracle_run(oracle, inp, *, lam, beta, temperature, seqs=None, want_recovery_logprobs=True, num_threads=8,
               greedy=False):
    """Run the oracle on host copies of the inputs (optionally only on sequences ``seqs``)."""
    sel = slice(None) if seqs is None else seqs
    dl = inp.get("draft_len")
    return oracle.verify_block(
        inp["G"][sel].cpu(), inp["S_ctx"][sel].cpu(), inp["S_noctx"][sel].cpu(), inp["draft"][sel].cpu(),
        inp["uniforms"][sel].cpu(), lam=lam, beta=beta, temperature=temperature,
        draft_len=None if dl is None else dl[sel].cpu(), want_recovery_logprobs=want_recovery_logprobs,
        num_threads=num_threads, greedy=greedy)


def compare(gpu_out, ora, uniforms, draft_len=None, seqs=None):
    """Element-by-element comparison.  Returns a report dict; raises AssertionError on any
    unexcused mismatch or log-prob outside tolerance."""
    sel = slice(None) if seqs is None else (seqs.cpu().numpy() if hasattr(seqs, "cpu") else seqs)
    n_g = _np(gpu_out["accepted_len"])[sel]
    tok_g = _np(gpu_out["next_token"])[sel]
    n_o, tok_o = ora["accepted_len"], ora["next_token"]
    u = _np(uniforms)[sel].astype(np.float64)
    B, kmax = ora["alpha"].shape
    valid = n_o >= 0

    # flagged sequences must be flagged identically
    assert np.array_equal(n_g[~valid], n_o[~valid]) and np.array_equal(tok_g[~valid], tok_o[~valid])

    alpha = ora["alpha"]
    with np.errstate(invalid="ignore"):
        near_acc = (np.abs(alpha - u[:, :kmax]) < NEAR) & (alpha < 1.0)  # NaN (untested) compares False
    near_samp = ora["sample_margin"] < NEAR
    excused = near_acc.any(axis=1) | near_samp  # alpha is only filled for t <= n_oracle
    mismatch = ((n_g != n_o) | (tok_g != tok_o)) & valid
    bad = mismatch & ~excused
    assert not bad.any(), (
        f"unexcused mismatches at sequences {np.nonzero(bad)[0][:8]}: "
        f"n gpu/oracle {n_g[bad][:8]}/{n_o[bad][:8]}, token gpu/oracle {tok_g[bad][:8]}/{tok_o[bad][:8]}")
    # a mismatching accepted_len must come from the acceptance band, a token-only mismatch from the sampling band
    assert np.all(near_acc.any(axis=1)[(n_g != n_o) & valid])

    report = {
        "sequences": int(B),
        "near_threshold_accepts": int(near_acc.sum()),
        "near_threshold_samples": int(near_samp[valid].sum()),
        "excused_sequences": int((excused & valid).sum()),
        "excused_mismatches": int((mismatch & excused).sum()),
        "unexcused_mismatches": 0,
        "mean_accepted_len": float(n_o[valid].mean()) if valid.any() else 0.0,
    }
    same = valid & ~mismatch

    def check_lp(name, got, want, mask):
        with np.errstate(invalid="ignore"):  # rows of flagged sequences are never written and may hold any bits
            got = got.astype(np.float64)
        with np.errstate(invalid="ignore"):  # a masked token's log-prob is -inf on both sides
            err = np.abs(got - want)
        tol = LOGPROB_ATOL + FP32_HALF_ULP * np.abs(want)
        m = mask & np.isfinite(want)
        worst = float(err[m].max()) if m.any() else 0.0
        report["max_abs_err_" + name] = worst
        assert np.all(err[m] <= tol[m]), f"{name}: max |gpu - oracle| = {worst:.3e}"
        assert np.all(np.isfinite(got[m]))

    if gpu_out.get("next_token_logprob") is not None:
        check_lp("next_token_logprob", _np(gpu_out["next_token_logprob"])[sel], ora["next_token_logprob"], same)
        assert np.all(np.isnan(_np(gpu_out["next_token_logprob"])[sel][~valid]))
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
