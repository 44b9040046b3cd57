"""Writes tests/golden/oracle_block_fixture.json: one small seeded block and what the float64 oracle returns
for it (sampled and greedy, fp32 and bf16 logits, one masked token, one flagged sequence).

It calls nothing but numpy and oracle/.  The fixture freezes the oracle's arithmetic: a change to
oracle/specsteer_oracle.c that moves any of these numbers has to be a deliberate one (the readings
of Algorithm 1, Eq. 7 and Eq. 8 it implements are listed in the design notes), and this script is
then re-run.

    python tests/golden/make_oracle_fixture.py
"""
import json
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))
import oracle  # noqa: E402


def bf16_bits(x):
    b = np.ascontiguousarray(x, np.float32).view(np.uint32).astype(np.uint64)
    return ((b + 0x7FFF + ((b >> 16) & 1)) >> 16).astype(np.uint16)


def build_inputs():
    rng = np.random.default_rng(16219)
    B, K, V = 5, 3, 19
    q = lambda a: (np.round(a * 64) / 64).astype(np.float32)  # dyadic, exact in bf16-free fp32 and short in JSON
    G, Sp, Sm = (q(rng.normal(size=(B, K + 1, V)) * 2.0) for _ in range(3))
    G[1, :, 4] = -np.inf                                    # a token the generalist masks
    draft = rng.integers(0, V, (B, K)).astype(np.int32)
    draft_len = np.array([3, 2, 0, 3, 5], np.int32)         # the last one is out of range: flagged
    u = (rng.integers(1, 1 << 20, (B, K + 1)) / float(1 << 20)).astype(np.float32)
    return G, Sp, Sm, draft, draft_len, u


def run_all(G, Sp, Sm, draft, draft_len, u):
    out = {}
    for dtype in ("f32", "bf16"):
        g, sp, sm = (G, Sp, Sm) if dtype == "f32" else (bf16_bits(G), bf16_bits(Sp), bf16_bits(Sm))
        for greedy in (False, True):
            r = oracle.verify_block(g, sp, sm, draft, u, lam=0.5, beta=0.75, temperature=0.8, draft_len=draft_len,
                                    greedy=greedy)
            out[f"{dtype}{'-greedy' if greedy else ''}"] = {
                "accepted_len": r["accepted_len"].tolist(),
                "next_token": r["next_token"].tolist(),
                "next_token_logprob": [None if np.isnan(x) else float(x) for x in r["next_token_logprob"]],
                "alpha": [[None if np.isnan(x) else float(x) for x in row] for row in r["alpha"]],
            }
    row = np.array([0, 1, 3, 2, 1], np.int32)
    idx, val = oracle.cloud_topk(G, Sm, row, beta=0.75, topk=4)
    e = oracle.edge_resample(idx, val, Sp, row, u[:, -1].copy(), beta=0.75, temperature=0.8)
    out["split"] = {"row": row.tolist(), "index": idx.tolist(), "value": [[float(x) for x in r] for r in val.tolist()],
                    "next_token": e["next_token"].tolist(), "next_token_logprob": [float(x) for x in e["next_token_logprob"]]}
    return out


def main():
    G, Sp, Sm, draft, draft_len, u = build_inputs()
    fixture = {
        "about": "oracle outputs for the block built by make_oracle_fixture.build_inputs() "
                 "(lambda 0.5, beta 0.75, T 0.8): Algorithm 1 phases 2-3, Eq. 7, Eq. 8; deployment split with k = 4",
        "outputs": run_all(G, Sp, Sm, draft, draft_len, u),
    }
    with open(os.path.join(HERE, "oracle_block_fixture.json"), "w") as f:
        json.dump(fixture, f, indent=1)
        f.write("\n")


if __name__ == "__main__":
    main()
