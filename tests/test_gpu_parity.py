"""GPU parity: the HIP path, called through the C ABI, against the float64 oracle on the
same seeded inputs.  Needs a real MI355X (pytest -m gpu)."""
import numpy as np
import pytest
import torch

import parity
from paper_2603_16219_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def binding():
    from paper_2603_16219_amd import binding as b

    assert torch.cuda.is_available(), "GPU tests need a device"
    b.library()
    return b


def run_both(binding, oracle, w, inp, seqs=None, rec=True):
    out = binding.verify_block(inp["G"], inp["S_ctx"], inp["S_noctx"], inp["draft"], inp["uniforms"],
                               lam=w.lam, beta=w.beta, temperature=w.temperature, draft_len=inp["draft_len"],
                               want_recovery_logprobs=rec, want_draft_logprobs=True)
    torch.cuda.synchronize()
    ora = parity.oracle_run(oracle, inp, lam=w.lam, beta=w.beta, temperature=w.temperature, seqs=seqs,
                            want_recovery_logprobs=rec, num_threads=16)
    rep = parity.compare(out, ora, inp["uniforms"], inp["draft_len"], seqs=seqs)
    print(f"\n[{w.name}] {rep}", flush=True)
    return out, ora, rep


# ------------------------------------------------------------------ the five configs

@pytest.mark.parametrize("name", ["c1", "c2", "c3"])
def test_config_full_size(binding, oracle, name):
    w = W.WORKLOADS[name]
    inp = W.generate(w, "cuda")
    out, ora, rep = run_both(binding, oracle, w, inp)
    assert 0 < rep["mean_accepted_len"] <= w.k_max


def test_config_c4_ragged_full_size(binding, oracle):
    w = W.WORKLOADS["c4"]
    inp = W.generate(w, "cuda")
    out, ora, rep = run_both(binding, oracle, w, inp)
    n = out["accepted_len"].cpu()
    assert torch.all(n <= inp["draft_len"].cpu()) and torch.all(n >= 0)


def test_config_c5_full_size(binding, oracle):
    """All 512 sequences through the oracle (per-position log-probs and the full recovery rows included)."""
    w = W.WORKLOADS["c5"]
    inp = W.generate(w, "cuda")
    out, ora, rep = run_both(binding, oracle, w, inp, rec=True)
    # and properties that hold for every sequence at any size
    n = out["accepted_len"].cpu().numpy()
    tok = out["next_token"].cpu().numpy()
    assert np.all((n >= 0) & (n <= w.k_max)) and np.all((tok >= 0) & (tok < w.vocab))
    lp = out["recovery_logprobs"]
    assert torch.allclose(torch.exp(lp.double()).sum(-1), torch.ones(w.batch, dtype=torch.float64, device="cuda"),
                          atol=1e-5)
    assert torch.allclose(lp.cpu()[torch.arange(w.batch), torch.from_numpy(tok).long()],
                          out["next_token_logprob"].cpu(), atol=1e-5)


# ------------------------------------------------------------------ shapes that stress tiling

@pytest.mark.parametrize("vocab,pad", [(20011, 0), (20011, 5), (20008, 0), (2048, 0), (2049, 7), (777, 0),
                                       (8, 0), (5, 3), (1, 0), (1, 7), (65, 0), (512 * 4 * 3 + 8, 0)])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_ragged_tails_and_alignment(binding, oracle, vocab, pad, dtype):
    """pad > 0 stores rows with a padded stride (aligned rows with a partial last vector when the
    stride is a multiple of 16 bytes); pad == 0 with an odd vocabulary makes most rows start off
    16-byte boundaries, which the 16-byte loads tolerate."""
    base = W.scaled(W.WORKLOADS["c4"], batch=7, vocab=vocab + pad, k_max=5, name=f"tail{vocab}+{pad}{dtype}")
    import dataclasses
    base = dataclasses.replace(base, dtype=dtype)
    inp = W.generate(base, "cuda")
    if pad:
        for k in ("G", "S_ctx", "S_noctx"):
            inp[k][..., vocab:] = float("nan")  # the padding must never be read
            inp[k] = inp[k][..., :vocab]
        inp["draft"] = inp["draft"].clamp(max=vocab - 1)
    inp["draft_len"] = torch.tensor([0, 1, 5, 3, 5, 2, 4], dtype=torch.int32, device="cuda")
    w = dataclasses.replace(base, vocab=vocab)
    run_both(binding, oracle, w, inp)


def test_unaligned_base_pointers(binding, oracle):
    w = W.scaled(W.WORKLOADS["c2"], batch=3, vocab=4096, k_max=4, name="unaligned")
    inp = W.generate(w, "cuda")
    for k in ("G", "S_ctx", "S_noctx"):
        flat = torch.empty(inp[k].numel() + 3, dtype=inp[k].dtype, device="cuda")
        view = flat[3:].view_as(inp[k])  # 6 bytes off a 16-byte boundary
        view.copy_(inp[k])
        inp[k] = view
        assert inp[k].data_ptr() % 16 != 0
    run_both(binding, oracle, w, inp)


def test_no_drafts_and_single_sequence(binding, oracle):
    w = W.scaled(W.WORKLOADS["c1"], batch=1, vocab=32000, k_max=0, name="k0")
    inp = W.generate(w, "cuda")
    out, ora, _ = run_both(binding, oracle, w, inp)
    assert out["accepted_len"].item() == 0
    w = W.scaled(W.WORKLOADS["c4"], batch=5, vocab=3000, k_max=3, name="allzero")
    inp = W.generate(w, "cuda")
    inp["draft_len"] = torch.zeros(5, dtype=torch.int32, device="cuda")
    run_both(binding, oracle, w, inp)


def test_long_draft_blocks_use_more_than_one_ballot(binding, oracle):
    w = W.scaled(W.WORKLOADS["c4"], batch=3, vocab=1024, k_max=150, name="k150")
    inp = W.generate(w, "cuda")
    inp["draft_len"] = torch.tensor([150, 70, 129], dtype=torch.int32, device="cuda")
    inp["uniforms"][:, :150] *= 0.02  # long accepted prefixes so the first rejection falls in a late ballot
    out, ora, rep = run_both(binding, oracle, w, inp)
    assert rep["mean_accepted_len"] > 20


def test_padding_rows_and_slots_are_never_read(binding, oracle):
    w = W.scaled(W.WORKLOADS["c4"], batch=16, vocab=8192, k_max=8, name="poison")
    inp = W.generate(w, "cuda")
    ref = binding.verify_block(inp["G"], inp["S_ctx"], inp["S_noctx"], inp["draft"], inp["uniforms"], lam=w.lam,
                               beta=w.beta, temperature=w.temperature, draft_len=inp["draft_len"],
                               want_recovery_logprobs=True, want_draft_logprobs=True)
    L = inp["draft_len"].cpu()
    n = ref["accepted_len"].cpu()
    for b in range(w.batch):
        for k in ("G", "S_noctx"):
            inp[k][b, L[b] + 1:] = float("nan")
        inp["S_ctx"][b, : n[b]] = float("nan")  # only the recovery row of S_ctx is ever touched
        inp["S_ctx"][b, n[b] + 1:] = float("nan")
        inp["draft"][b, L[b]:] = -123456
        inp["uniforms"][b, L[b]: w.k_max] = float("nan")
    got = binding.verify_block(inp["G"], inp["S_ctx"], inp["S_noctx"], inp["draft"], inp["uniforms"], lam=w.lam,
                               beta=w.beta, temperature=w.temperature, draft_len=inp["draft_len"],
                               want_recovery_logprobs=True, want_draft_logprobs=True)
    for k in ref:
        assert torch.equal(ref[k], got[k]), k
    run_both(binding, oracle, w, inp)


def test_bad_sequences_are_flagged(binding, oracle):
    w = W.scaled(W.WORKLOADS["c4"], batch=6, vocab=4000, k_max=4, name="bad")
    inp = W.generate(w, "cuda")
    inp["draft_len"] = torch.tensor([4, 5, -1, 2, 3, 0], dtype=torch.int32, device="cuda")
    inp["draft"][3, 1] = 4000
    inp["draft"][4, 0] = -1
    inp["draft"][0, 3] = 3999
    out, ora, _ = run_both(binding, oracle, w, inp)
    assert out["accepted_len"].cpu().tolist()[1:5] == [-1, -1, -1, -1]
    assert out["accepted_len"][0].item() >= 0 and out["accepted_len"][5].item() == 0


def test_extreme_logits_and_peaked_rows(binding, oracle):
    import dataclasses
    w = dataclasses.replace(W.scaled(W.WORKLOADS["c5"], batch=6, vocab=30000, k_max=4, name="peaked"), beta=2.5)
    inp = W.generate(w, "cuda")
    inp["G"][0:2] += 80.0
    inp["S_ctx"][2:4] -= 80.0
    inp["S_noctx"][1:3] += 64.0
    run_both(binding, oracle, w, inp)
    w2 = dataclasses.replace(w, dtype="f32", temperature=0.3, name="peaked32")
    run_both(binding, oracle, w2, W.generate(w2, "cuda"))


def test_strided_batch_view(binding, oracle):
    w = W.scaled(W.WORKLOADS["c2"], batch=6, vocab=4096, k_max=5, name="strided")
    inp = W.generate(w, "cuda")
    for k in ("G", "S_ctx", "S_noctx"):
        inp[k] = inp[k][::2, :4]  # every other sequence, first 4 rows: stride_b and stride_t both non-dense
    inp["draft"] = inp["draft"][::2, :3].contiguous()
    inp["uniforms"] = inp["uniforms"][::2, :4].contiguous()
    w = W.scaled(w, batch=3, k_max=3)
    run_both(binding, oracle, w, inp)


def test_run_twice_bit_identical(binding):
    w = W.scaled(W.WORKLOADS["c4"], batch=32, vocab=50000, k_max=8, name="twice")
    inp = W.generate(w, "cuda")
    outs = []
    for _ in range(2):
        outs.append(binding.verify_block(inp["G"], inp["S_ctx"], inp["S_noctx"], inp["draft"], inp["uniforms"],
                                         lam=w.lam, beta=w.beta, temperature=w.temperature,
                                         draft_len=inp["draft_len"], want_recovery_logprobs=True,
                                         want_draft_logprobs=True))
    torch.cuda.synchronize()
    for k in outs[0]:
        assert torch.equal(outs[0][k], outs[1][k]), k


def test_lambda_sweep_matches_oracle(binding, oracle):
    """The threshold values of the paper's sensitivity study."""
    import dataclasses
    base = W.scaled(W.WORKLOADS["c4"], batch=24, vocab=16384, k_max=8, name="lam")
    inp = W.generate(base, "cuda")
    prev = None
    for lam in (1.0, 0.5, 0.1, 0.01):
        w = dataclasses.replace(base, lam=lam, name=f"lam{lam}")
        out, ora, rep = run_both(binding, oracle, w, inp)
        if prev is not None:
            assert rep["mean_accepted_len"] >= prev  # a smaller threshold accepts more
        prev = rep["mean_accepted_len"]


def test_sampling_edges_on_gpu(binding, oracle):
    """Uniforms placed just inside both ends of every CDF interval of a 6-token row."""
    V = 6
    G = torch.tensor([[[0.5, -1.0, 2.0, 0.0, 1.5, -0.5]]], dtype=torch.float32, device="cuda")
    z = torch.zeros_like(G)
    p = torch.softmax(G[0, 0].double(), -1).cpu().numpy()
    cdf = np.cumsum(p)
    us, want = [0.0], [0]
    for j in range(V - 1):
        us += [float(np.float32(cdf[j] - 3e-6)), float(np.float32(cdf[j] + 3e-6))]
        want += [j, j + 1]
    us.append(float(np.nextafter(np.float32(1), np.float32(0))))
    want.append(V - 1)
    B = len(us)
    Gb = G.expand(B, 1, V).contiguous()
    out = binding.verify_block(Gb, torch.zeros_like(Gb), torch.zeros_like(Gb),
                               torch.zeros(B, 0, dtype=torch.int32, device="cuda"),
                               torch.tensor(us, dtype=torch.float32, device="cuda").view(B, 1))
    assert out["next_token"].cpu().tolist() == want


# ------------------------------------------------------------------ greedy decoding and the comparison modes

@pytest.mark.parametrize("name,batch,vocab", [("c2", 8, 151936), ("c4", 48, 50000), ("c5", 16, 64000), ("c1", 3, 32000)])
def test_greedy_mode(binding, oracle, name, batch, vocab):
    w = W.scaled(W.WORKLOADS[name], batch=batch, vocab=vocab, name=f"greedy-{name}")
    inp = W.generate(w, "cuda")
    out = binding.verify_block(inp["G"], inp["S_ctx"], inp["S_noctx"], inp["draft"], inp["uniforms"], lam=w.lam,
                               beta=w.beta, temperature=w.temperature, draft_len=inp["draft_len"],
                               want_recovery_logprobs=True, want_draft_logprobs=True, greedy=True)
    ora = parity.oracle_run(oracle, inp, lam=w.lam, beta=w.beta, temperature=w.temperature, greedy=True, num_threads=16)
    rep = parity.compare(out, ora, inp["uniforms"], inp["draft_len"])
    print(f"\n[{w.name}] {rep}", flush=True)
    assert rep["near_threshold_samples"] == 0  # no uniform is involved in the pick: nothing is excused there
    # and the pick does not depend on the sampling uniform
    inp["uniforms"][:, -1] = 0.123
    again = binding.verify_block(inp["G"], inp["S_ctx"], inp["S_noctx"], inp["draft"], inp["uniforms"], lam=w.lam,
                                 beta=w.beta, temperature=w.temperature, draft_len=inp["draft_len"], greedy=True)
    assert torch.equal(out["next_token"], again["next_token"])


def test_greedy_ties_take_the_lowest_index_on_gpu(binding):
    V = 5000
    G = torch.zeros(4, 1, V, dtype=torch.bfloat16, device="cuda")
    G[0, 0, [17, 4000, 4999]] = 2.0
    G[1, 0, [4095, 4096]] = 1.0       # a tie across two lanes / chunks
    G[2, 0, :] = -3.0                 # everything ties: index 0
    G[3, 0, 4999] = 0.5
    z = torch.zeros_like(G)
    out = binding.verify_block(G, z, z, torch.zeros(4, 0, dtype=torch.int32, device="cuda"),
                               torch.full((4, 1), 0.9, device="cuda"), greedy=True)
    assert out["next_token"].cpu().tolist() == [17, 4095, 0, 4999]


def test_beta_zero_never_reads_the_context_rows(binding, oracle):
    w = W.scaled(W.WORKLOADS["c4"], batch=12, vocab=30000, k_max=6, name="beta0")
    import dataclasses
    w = dataclasses.replace(w, beta=0.0)
    inp = W.generate(w, "cuda")
    ora = parity.oracle_run(oracle, inp, lam=w.lam, beta=0.0, temperature=w.temperature)
    inp["S_ctx"].fill_(float("nan"))
    out = binding.verify_block(inp["G"], inp["S_ctx"], inp["S_noctx"], inp["draft"], inp["uniforms"], lam=w.lam,
                               beta=0.0, temperature=w.temperature, draft_len=inp["draft_len"],
                               want_recovery_logprobs=True, want_draft_logprobs=True)
    parity.compare(out, ora, inp["uniforms"], inp["draft_len"])


def test_standard_speculative_acceptance_mode(binding, oracle):
    """The baseline the paper compares with: alpha = min(1, P_LLM / P_SLM^+), no steering.  It is this block
    with the drafter's own logits in the S_noctx slot, lambda = 1 and beta = 0."""
    w = W.scaled(W.WORKLOADS["c2"], batch=16, vocab=40000, k_max=8, name="stdspec")
    inp = W.generate(w, "cuda")
    out = binding.verify_block(inp["G"], inp["S_ctx"], inp["S_ctx"], inp["draft"], inp["uniforms"], lam=1.0, beta=0.0,
                               temperature=1.0, want_recovery_logprobs=True, want_draft_logprobs=True)
    host = [inp[k].cpu() for k in ("G", "S_ctx", "S_ctx", "draft")]
    ora = oracle.verify_block(*host, inp["uniforms"].cpu(), lam=1.0, beta=0.0, temperature=1.0, num_threads=16)
    parity.attach_recheck(ora, oracle, *host, None, lam=1.0, beta=0.0, temperature=1.0)
    parity.compare(out, ora, inp["uniforms"], None)
    # independent check of the rule itself on the GPU's own log-probs
    lp = out["draft_logprobs"].double().cpu()
    alpha = torch.exp(lp[..., 0] - lp[..., 1]).clamp(max=1.0)
    acc = inp["uniforms"].cpu()[:, :8].double() <= alpha
    n = torch.where(acc.all(1), torch.tensor(8), (~acc).int().argmax(1))
    assert torch.equal(n.int(), out["accepted_len"].cpu())


def test_always_on_steering_rows(binding, oracle):
    """Eq. 8 and one draw on EVERY row (the per-token fusion baseline): k_max = 0 on flattened rows."""
    w = W.scaled(W.WORKLOADS["c3"], batch=6, vocab=30000, k_max=7, name="steer-rows")
    inp = W.generate(w, "cuda")
    rows = lambda t: t.reshape(-1, w.vocab)
    G, Sp, Sm = rows(inp["G"]), rows(inp["S_ctx"]), rows(inp["S_noctx"])
    u = torch.rand(G.shape[0], generator=torch.Generator("cuda").manual_seed(5), device="cuda")
    out = binding.steer_rows(G, Sp, Sm, u, beta=w.beta, temperature=w.temperature, want_logprobs=True)
    N = G.shape[0]
    host = [G.view(N, 1, -1).cpu(), Sp.view(N, 1, -1).cpu(), Sm.view(N, 1, -1).cpu(), torch.zeros(N, 0, dtype=torch.int32)]
    ora = oracle.verify_block(*host, u.view(N, 1).cpu(), beta=w.beta, temperature=w.temperature, num_threads=16)
    parity.attach_recheck(ora, oracle, *host, None, lam=0.5, beta=w.beta, temperature=w.temperature)
    rep = parity.compare({"accepted_len": torch.zeros(N, dtype=torch.int32), "next_token": out["token"],
                          "next_token_logprob": out["token_logprob"], "recovery_logprobs": out["logprobs"]},
                         ora, u.view(N, 1), None)
    assert rep["unexcused_mismatches"] == 0


def test_draft_sampler_reproduces_the_harness_drafts(binding):
    """Eq. 5: y ~ softmax(S_ctx / T).  The workload generator draws its drafts with torch (float64 softmax,
    cumsum, searchsorted); the block with k_max = 0 and beta = 0, fed the same uniforms, must pick the same
    tokens wherever the uniform is not within 1e-6 of a CDF edge."""
    w = W.scaled(W.WORKLOADS["c4"], batch=8, vocab=128256, k_max=8, name="drafts")
    dev = torch.device("cuda")
    S = (torch.randn(w.batch * w.k_max, w.vocab, generator=torch.Generator(dev).manual_seed(7), device=dev) * 3).to(torch.bfloat16)
    u64 = torch.rand(S.shape[0], 1, generator=torch.Generator(dev).manual_seed(8), device=dev, dtype=torch.float64)
    u = u64.float()
    cdf = torch.cumsum(torch.softmax(S.double() / w.temperature, -1), -1)
    want = torch.searchsorted(cdf, u.double(), right=True).squeeze(-1).clamp(max=w.vocab - 1)
    got = binding.sample_rows(S, u.squeeze(-1), temperature=w.temperature)["token"].long()
    edge = (cdf - u.double()).abs().min(-1).values < 1e-6
    assert torch.equal(got[~edge], want[~edge])
    assert (~edge).sum() > 0.8 * len(edge)


# ------------------------------------------------------------------ deployment split: cloud top-k, edge resample

def _split_case(binding, oracle, w, topk, greedy=False, pad=0):
    inp = W.generate(w, "cuda")
    if pad:
        for k in ("G", "S_ctx", "S_noctx"):
            inp[k][..., w.vocab - pad:] = float("nan")
            inp[k] = inp[k][..., : w.vocab - pad]
    B = w.batch
    row = torch.randint(0, w.k_max + 1, (B,), generator=torch.Generator("cuda").manual_seed(3), device="cuda",
                        dtype=torch.int32)
    if B > 2:
        row[1] = -1  # a flagged sequence
    idx, val = binding.cloud_topk(inp["G"], inp["S_noctx"], row, beta=w.beta, topk=topk)
    oidx, oval = oracle.cloud_topk(inp["G"].cpu(), inp["S_noctx"].cpu(), row.cpu(), beta=w.beta, topk=topk)
    assert np.array_equal(idx.cpu().numpy(), oidx), "payload ids differ"
    assert np.array_equal(val.cpu().numpy(), oval), "payload values differ"
    u = inp["uniforms"][:, -1].contiguous()
    out = binding.edge_resample(idx, val, inp["S_ctx"], row, u, beta=w.beta, temperature=w.temperature, greedy=greedy)
    ora = oracle.edge_resample(oidx, oval, inp["S_ctx"].cpu(), row.cpu(), u.cpu(), beta=w.beta,
                               temperature=w.temperature, greedy=greedy)
    tok = out["next_token"].cpu().numpy()
    lp = out["next_token_logprob"].cpu().numpy().astype(np.float64)
    excused = ora["sample_margin"] < parity.NEAR
    mism = tok != ora["next_token"]
    assert not np.any(mism & ~excused), (tok, ora["next_token"])
    ok = ~mism & (ora["next_token"] >= 0)
    assert np.all(np.abs(lp[ok] - ora["next_token_logprob"][ok]) <= parity.logprob_tol(ora["next_token_logprob"][ok]))
    assert np.all(np.isnan(lp[ora["next_token"] < 0]))
    print(f"\n[{w.name}] split ok: {int(excused.sum())} near-threshold, {int((mism & excused).sum())} excused mismatches", flush=True)


@pytest.mark.parametrize("name,batch,vocab,topk", [("c4", 24, 128256, 32), ("c2", 8, 151936, 32), ("c5", 8, 50000, 64),
                                                    ("c3", 6, 20011, 32), ("c1", 2, 32000, 32), ("c4", 5, 777, 5),
                                                    ("c4", 4, 20, 32), ("c4", 3, 1, 1)])
def test_cloud_topk_and_edge_resample(binding, oracle, name, batch, vocab, topk):
    w = W.scaled(W.WORKLOADS[name], batch=batch, vocab=vocab, k_max=min(W.WORKLOADS[name].k_max, 4),
                 name=f"split-{name}-{vocab}-{topk}")
    _split_case(binding, oracle, w, topk)
    _split_case(binding, oracle, w, topk, greedy=True)


def test_cloud_topk_with_ties_and_padded_rows(binding, oracle):
    w = W.scaled(W.WORKLOADS["c4"], batch=4, vocab=4103 + 9, k_max=2, name="split-pad")
    _split_case(binding, oracle, w, 32, pad=9)  # stride 4112 (aligned rows), V = 4103: partial last vector
    # many exact ties: quantised logits
    inp = W.generate(W.scaled(W.WORKLOADS["c4"], batch=3, vocab=9000, k_max=1, name="ties"), "cuda")
    for k in ("G", "S_noctx"):
        inp[k] = (inp[k].float().round() * 0.5).to(torch.bfloat16)
    row = torch.zeros(3, dtype=torch.int32, device="cuda")
    idx, val = binding.cloud_topk(inp["G"], inp["S_noctx"], row, beta=0.5, topk=32)
    oidx, oval = oracle.cloud_topk(inp["G"].cpu(), inp["S_noctx"].cpu(), row.cpu(), beta=0.5, topk=32)
    assert np.array_equal(idx.cpu().numpy(), oidx) and np.array_equal(val.cpu().numpy(), oval)


def test_full_payload_reproduces_the_one_gpu_recovery(binding):
    """k = V (tiny vocabulary): the split loses nothing, so its token must be the block's token."""
    w = W.scaled(W.WORKLOADS["c2"], batch=32, vocab=48, k_max=3, name="split-full")
    inp = W.generate(w, "cuda")
    ref = binding.verify_block(inp["G"], inp["S_ctx"], inp["S_noctx"], inp["draft"], inp["uniforms"], lam=w.lam,
                               beta=w.beta, temperature=w.temperature, greedy=True)
    idx, val = binding.cloud_topk(inp["G"], inp["S_noctx"], ref["accepted_len"], beta=w.beta, topk=48)
    out = binding.edge_resample(idx, val, inp["S_ctx"], ref["accepted_len"], inp["uniforms"][:, -1].contiguous(),
                                beta=w.beta, temperature=w.temperature, greedy=True)
    assert torch.equal(out["next_token"], ref["next_token"])


# ------------------------------------------------------------------ two-pass schedule (stop scoring after a rejection)

@pytest.mark.parametrize("name,batch,vocab,dtype", [("c4", 96, 100000, "bf16"), ("c5", 160, 110000, "bf16"),
                                                     ("c3", 128, 151936, "bf16"), ("c4", 64, 70000, "f32")])
def test_two_pass_schedule_matches_one_pass_and_oracle(binding, oracle, name, batch, vocab, dtype):
    """Large enough for the library to split the row pass in two windows: outputs must equal those of the
    one-pass schedule bit for bit (same arithmetic, fewer rows read) and match the oracle."""
    import dataclasses
    w = dataclasses.replace(W.scaled(W.WORKLOADS[name], batch=batch, vocab=vocab, name=f"twopass-{name}-{dtype}"), dtype=dtype)
    inp = W.generate(w, "cuda")
    p = binding.make_params(w.batch, w.k_max, w.vocab, inp["G"].dtype, lam=w.lam, beta=w.beta, temperature=w.temperature)
    assert binding.first_window(p) == w.k_max // 4, "this case is meant to take the two-pass schedule"
    kw = dict(lam=w.lam, beta=w.beta, temperature=w.temperature, draft_len=inp["draft_len"], want_recovery_logprobs=True)
    two = binding.verify_block(inp["G"], inp["S_ctx"], inp["S_noctx"], inp["draft"], inp["uniforms"], **kw)
    one = binding.verify_block(inp["G"], inp["S_ctx"], inp["S_noctx"], inp["draft"], inp["uniforms"], full_rows=True, **kw)
    for k in ("accepted_len", "next_token", "next_token_logprob", "recovery_logprobs"):
        assert torch.equal(two[k], one[k]), k
    ora = parity.oracle_run(oracle, inp, lam=w.lam, beta=w.beta, temperature=w.temperature, num_threads=16)
    rep = parity.compare(two, ora, inp["uniforms"], inp["draft_len"])
    print(f"\n[{w.name}] {rep}", flush=True)
    n = two["accepted_len"].cpu()
    t1 = w.k_max // 4
    assert (n < t1).any() and (n >= t1).any(), "both kinds of sequences should occur"


def test_two_pass_schedule_never_reads_rows_after_an_early_rejection(binding):
    w = W.scaled(W.WORKLOADS["c4"], batch=96, vocab=100000, name="twopass-poison")
    inp = W.generate(w, "cuda")
    assert binding.first_window(binding.make_params(w.batch, w.k_max, w.vocab, inp["G"].dtype, lam=w.lam, beta=w.beta,
                                                    temperature=w.temperature)) == w.k_max // 4
    kw = dict(lam=w.lam, beta=w.beta, temperature=w.temperature, draft_len=inp["draft_len"])
    ref = binding.verify_block(inp["G"], inp["S_ctx"], inp["S_noctx"], inp["draft"], inp["uniforms"], **kw)
    n = ref["accepted_len"].cpu()
    L = inp["draft_len"].cpu()
    t1 = w.k_max // 4
    poisoned = 0
    for b in range(w.batch):
        if n[b] < t1 and L[b] > t1:  # rejected inside the first window: rows t1.. are dead weight
            for k in ("G", "S_noctx"):
                inp[k][b, t1:] = float("nan")
            poisoned += 1
    assert poisoned > 5
    got = binding.verify_block(inp["G"], inp["S_ctx"], inp["S_noctx"], inp["draft"], inp["uniforms"], **kw)
    for k in ("accepted_len", "next_token", "next_token_logprob"):
        assert torch.equal(ref[k], got[k]), k


def test_two_pass_schedule_flags_bad_sequences_like_one_pass(binding, oracle):
    w = W.scaled(W.WORKLOADS["c4"], batch=96, vocab=100000, name="twopass-bad")
    inp = W.generate(w, "cuda")
    assert binding.first_window(binding.make_params(w.batch, w.k_max, w.vocab, inp["G"].dtype, lam=w.lam, beta=w.beta,
                                                    temperature=w.temperature)) == w.k_max // 4
    inp["draft_len"][3] = 17
    inp["draft_len"][4] = -2
    inp["draft_len"][5] = 16
    inp["draft"][5, 15] = 100000    # out of vocabulary far behind any likely rejection
    inp["draft_len"][6] = 2
    inp["draft"][6, 1] = -1
    inp["draft_len"][7] = 0
    out = binding.verify_block(inp["G"], inp["S_ctx"], inp["S_noctx"], inp["draft"], inp["uniforms"], lam=w.lam,
                               beta=w.beta, temperature=w.temperature, draft_len=inp["draft_len"])
    ora = parity.oracle_run(oracle, inp, lam=w.lam, beta=w.beta, temperature=w.temperature, want_recovery_logprobs=False,
                            num_threads=16)
    parity.compare(out, ora, inp["uniforms"], inp["draft_len"])
    assert out["accepted_len"].cpu().tolist()[3:7] == [-1, -1, -1, -1] and out["accepted_len"][7].item() == 0


# ------------------------------------------------------------------ limits of the interface

def test_batch_beyond_the_in_kernel_row_list(binding, oracle):
    """More than 8192 sequences: the row list no longer fits LDS and is built by its own kernel."""
    w = W.scaled(W.WORKLOADS["c4"], batch=9000, vocab=96, k_max=3, name="bigbatch")
    inp = W.generate(w, "cuda", seq_chunk=512)
    inp["draft_len"] = torch.randint(0, 4, (9000,), generator=torch.Generator("cuda").manual_seed(1), device="cuda",
                                     dtype=torch.int32)
    run_both(binding, oracle, w, inp)


def test_big_batch_two_pass_with_global_row_lists(binding, oracle):
    w = W.scaled(W.WORKLOADS["c4"], batch=9000, vocab=8192, k_max=4, name="bigbatch-twopass")
    inp = W.generate(w, "cuda", seq_chunk=256)
    p = binding.make_params(w.batch, w.k_max, w.vocab, inp["G"].dtype, lam=w.lam, beta=w.beta, temperature=w.temperature)
    assert binding.first_window(p) == 1
    out = binding.verify_block(inp["G"], inp["S_ctx"], inp["S_noctx"], inp["draft"], inp["uniforms"], lam=w.lam,
                               beta=w.beta, temperature=w.temperature, draft_len=inp["draft_len"])
    one = binding.verify_block(inp["G"], inp["S_ctx"], inp["S_noctx"], inp["draft"], inp["uniforms"], lam=w.lam,
                               beta=w.beta, temperature=w.temperature, draft_len=inp["draft_len"], full_rows=True)
    for k in ("accepted_len", "next_token", "next_token_logprob"):
        assert torch.equal(out[k], one[k]), k
    seqs = torch.arange(0, 9000, 9, device="cuda")
    ora = parity.oracle_run(oracle, inp, lam=w.lam, beta=w.beta, temperature=w.temperature, seqs=seqs,
                            want_recovery_logprobs=False, num_threads=16)
    parity.compare(out, ora, inp["uniforms"], inp["draft_len"], seqs=seqs)


def test_longest_draft_block(binding, oracle):
    w = W.scaled(W.WORKLOADS["c2"], batch=2, vocab=200, k_max=1024, name="kmax1024")
    inp = W.generate(w, "cuda")
    inp["uniforms"][:, :1024] *= 0.001  # accept almost everything: the first rejection is far down the block
    out, ora, rep = run_both(binding, oracle, w, inp)
    assert rep["mean_accepted_len"] > 100


@pytest.mark.parametrize("dtype,shift", [("bf16", 0), ("f32", 0), ("bf16", 1)])
def test_largest_vocabulary(binding, oracle, dtype, shift):
    """V = 2^20, the interface's maximum; shift = 1 moves the rows off 16-byte alignment."""
    import dataclasses
    V = (1 << 20) - shift
    w = dataclasses.replace(W.scaled(W.WORKLOADS["c2"], batch=2, vocab=V, k_max=2, name=f"vmax-{dtype}-{shift}"), dtype=dtype)
    inp = W.generate(w, "cuda", seq_chunk=1)
    run_both(binding, oracle, w, inp)


# ------------------------------------------------------------------ small batches: recovery row shared by several workgroups

@pytest.mark.parametrize("name,batch,vocab,dtype", [
    ("c2", 1, 151936, "bf16"),    # the on-device case: one sequence, 5 parts
    ("c2", 17, 151936, "bf16"),   # 256 // 17 = 15 parts wanted, 5 available
    ("c4", 128, 32776, "bf16"),   # 2 parts, the second holds a single chunk
    ("c4", 100, 70000, "bf16"),   # 2 parts of 3 wanted by the chunks
    ("c1", 1, 32000, "f32"),
    ("c5", 33, 65544, "f32"),     # 7 parts
    ("c3", 16, 151937, "bf16"),   # odd vocabulary: rows off 16-byte boundaries
])
def test_split_recovery_shapes(binding, oracle, name, batch, vocab, dtype):
    import dataclasses
    w = dataclasses.replace(W.scaled(W.WORKLOADS[name], batch=batch, vocab=vocab, name=f"split-{name}-{batch}"),
                            dtype=dtype)
    inp = W.generate(w, "cuda")
    run_both(binding, oracle, w, inp)
    out = binding.verify_block(inp["G"], inp["S_ctx"], inp["S_noctx"], inp["draft"], inp["uniforms"], lam=w.lam,
                               beta=w.beta, temperature=w.temperature, draft_len=inp["draft_len"], greedy=True)
    ora = parity.oracle_run(oracle, inp, lam=w.lam, beta=w.beta, temperature=w.temperature, greedy=True,
                            want_recovery_logprobs=False, num_threads=16)
    rep = parity.compare(out, ora, inp["uniforms"], inp["draft_len"])
    assert rep["near_threshold_samples"] == 0


def test_split_recovery_reuses_one_workspace(binding, oracle):
    """Back-to-back calls on one workspace, the arrival counters of the parts start from zero
    every time; sampled, greedy and draft-free calls interleaved, with flagged sequences."""
    w = W.scaled(W.WORKLOADS["c4"], batch=12, vocab=128256, name="split-ws")
    p = binding.make_params(w.batch, w.k_max, w.vocab, torch.bfloat16, lam=w.lam, beta=w.beta, temperature=w.temperature)
    ws = torch.empty(binding.workspace_bytes(p), dtype=torch.uint8, device="cuda")
    ws.fill_(0xAB)
    for rnd in range(4):
        inp = W.generate(w, "cuda", seed_shift=rnd)
        greedy = rnd == 2
        if rnd == 1:
            inp["draft_len"][3] = w.k_max + 1
            inp["draft"][7, 0] = w.vocab
        out = binding.verify_block(inp["G"], inp["S_ctx"], inp["S_noctx"], inp["draft"], inp["uniforms"], lam=w.lam,
                                   beta=w.beta, temperature=w.temperature, draft_len=inp["draft_len"],
                                   want_recovery_logprobs=True, greedy=greedy, workspace=ws)
        ora = parity.oracle_run(oracle, inp, lam=w.lam, beta=w.beta, temperature=w.temperature, greedy=greedy,
                                num_threads=16)
        rep = parity.compare(out, ora, inp["uniforms"], inp["draft_len"])
        print(f"\n[split-ws {rnd}] {rep}", flush=True)
        if rnd == 1:
            assert out["accepted_len"][3].item() == -1 and out["accepted_len"][7].item() == -1
    # rows without drafts (k_max = 0) have no row pass in front of the recovery
    w0 = W.scaled(W.WORKLOADS["c2"], batch=5, vocab=100000, k_max=0, name="split-k0")
    p0 = binding.make_params(w0.batch, 0, w0.vocab, torch.bfloat16, lam=w0.lam, beta=w0.beta, temperature=w0.temperature)
    ws0 = torch.full((binding.workspace_bytes(p0),), 0xCD, dtype=torch.uint8, device="cuda")
    for rnd in range(2):
        inp = W.generate(w0, "cuda", seed_shift=rnd)
        out = binding.verify_block(inp["G"], inp["S_ctx"], inp["S_noctx"], inp["draft"], inp["uniforms"], lam=w0.lam,
                                   beta=w0.beta, temperature=w0.temperature, want_recovery_logprobs=True, workspace=ws0)
        ora = parity.oracle_run(oracle, inp, lam=w0.lam, beta=w0.beta, temperature=w0.temperature, num_threads=16)
        parity.compare(out, ora, inp["uniforms"], inp["draft_len"])


# ------------------------------------------------------------------ every benchmark mode at the size and launch shape bench.py times

@pytest.fixture(scope="module")
def c4_inputs():
    w = W.WORKLOADS["c4"]
    return w, W.generate(w, "cuda")


def test_c4_timed_schedule_full_size(binding, oracle, c4_inputs):
    """The call bench.py times: no per-position log-probs, hence the two-pass schedule, all 256 sequences."""
    w, inp = c4_inputs
    p = binding.make_params(w.batch, w.k_max, w.vocab, torch.bfloat16, lam=w.lam, beta=w.beta, temperature=w.temperature)
    assert binding.first_window(p) == 4
    out = binding.verify_block(inp["G"], inp["S_ctx"], inp["S_noctx"], inp["draft"], inp["uniforms"], lam=w.lam,
                               beta=w.beta, temperature=w.temperature, draft_len=inp["draft_len"])
    ora = parity.oracle_run(oracle, inp, lam=w.lam, beta=w.beta, temperature=w.temperature,
                            want_recovery_logprobs=False, num_threads=16)
    rep = parity.compare(out, ora, inp["uniforms"], inp["draft_len"])
    print(f"\n[c4 timed schedule] {rep}", flush=True)


def test_c5_timed_schedule_full_size(binding, oracle):
    """The call bench.py times on c5, all 512 sequences against the oracle."""
    w = W.WORKLOADS["c5"]
    inp = W.generate(w, "cuda")
    out = binding.verify_block(inp["G"], inp["S_ctx"], inp["S_noctx"], inp["draft"], inp["uniforms"], lam=w.lam,
                               beta=w.beta, temperature=w.temperature, draft_len=inp["draft_len"])
    ora = parity.oracle_run(oracle, inp, lam=w.lam, beta=w.beta, temperature=w.temperature,
                            want_recovery_logprobs=False, num_threads=16)
    rep = parity.compare(out, ora, inp["uniforms"], inp["draft_len"])
    print(f"\n[c5 timed schedule] {rep}", flush=True)
    one = binding.verify_block(inp["G"], inp["S_ctx"], inp["S_noctx"], inp["draft"], inp["uniforms"], lam=w.lam,
                               beta=w.beta, temperature=w.temperature, draft_len=inp["draft_len"], full_rows=True)
    for k in ("accepted_len", "next_token", "next_token_logprob"):
        assert torch.equal(out[k], one[k]), k  # every sequence: both schedules, bit for bit


def test_c4_greedy_full_size(binding, oracle, c4_inputs):
    w, inp = c4_inputs
    out = binding.verify_block(inp["G"], inp["S_ctx"], inp["S_noctx"], inp["draft"], inp["uniforms"], lam=w.lam,
                               beta=w.beta, temperature=w.temperature, draft_len=inp["draft_len"], greedy=True)
    ora = parity.oracle_run(oracle, inp, lam=w.lam, beta=w.beta, temperature=w.temperature, greedy=True,
                            want_recovery_logprobs=False, num_threads=16)
    rep = parity.compare(out, ora, inp["uniforms"], inp["draft_len"])
    assert rep["near_threshold_samples"] == 0


def test_c4_cloud_topk_full_size(binding, oracle, c4_inputs):
    w, inp = c4_inputs
    row = torch.randint(0, w.k_max + 1, (w.batch,), generator=torch.Generator("cuda").manual_seed(11), device="cuda",
                        dtype=torch.int32)
    idx, val = binding.cloud_topk(inp["G"], inp["S_noctx"], row, beta=w.beta, topk=32)
    sel = torch.arange(0, w.batch, 4, device="cuda")  # 64 of the 256 rows through the oracle's full sort
    oidx, oval = oracle.cloud_topk(inp["G"][sel].cpu(), inp["S_noctx"][sel].cpu(), row[sel].cpu(), beta=w.beta, topk=32)
    assert np.array_equal(idx[sel].cpu().numpy(), oidx) and np.array_equal(val[sel].cpu().numpy(), oval)
    # every row: ordered payload of distinct in-range ids whose values are the exact double logits, rounded
    assert torch.all((idx >= 0) & (idx < w.vocab))
    assert torch.all(val[:, :-1] >= val[:, 1:])
    assert all(len(set(r)) == 32 for r in idx.cpu().tolist())
    b = torch.arange(w.batch, device="cuda").view(-1, 1).expand(-1, 32)
    r = row.long().view(-1, 1).expand(-1, 32)
    g = inp["G"][b, r, idx.long()].double()
    s = inp["S_noctx"][b, r, idx.long()].double()
    assert torch.equal((g - float(np.float32(w.beta)) * s).float(), val)


@pytest.mark.parametrize("mode", ["steer_rows", "draft_sample"])
def test_c4_row_modes_full_size_sampled_rows(binding, oracle, c4_inputs, mode):
    """All 4352 rows of the workload as one-row sequences, as bench.py --mode steer_rows / draft_sample runs them."""
    w, inp = c4_inputs
    n = w.batch * (w.k_max + 1)
    G, Sp, Sm = (inp[k].view(n, w.vocab) for k in ("G", "S_ctx", "S_noctx"))
    u = inp["uniforms"].reshape(n)
    if mode == "steer_rows":
        out = binding.steer_rows(G, Sp, Sm, u, beta=w.beta, temperature=w.temperature)
        beta = w.beta
    else:
        out = binding.sample_rows(Sp, u, temperature=w.temperature)
        G = Sm = Sp
        beta = 0.0
    sel = torch.arange(7, n, 29, device="cuda")  # 150 rows through the oracle
    m = len(sel)
    host = [G[sel].view(m, 1, -1).cpu(), Sp[sel].view(m, 1, -1).cpu(), Sm[sel].view(m, 1, -1).cpu(),
            torch.zeros(m, 0, dtype=torch.int32)]
    ora = oracle.verify_block(*host, u[sel].view(m, 1).cpu(), beta=beta, temperature=w.temperature,
                              want_recovery_logprobs=False, num_threads=16)
    parity.attach_recheck(ora, oracle, *host, None, lam=0.5, beta=beta, temperature=w.temperature)
    rep = parity.compare({"accepted_len": torch.zeros(m, dtype=torch.int32), "next_token": out["token"][sel],
                          "next_token_logprob": out["token_logprob"][sel]}, ora, u[sel].view(m, 1), None)
    print(f"\n[c4 {mode}] {rep}", flush=True)
    tok = out["token"]
    assert torch.all((tok >= 0) & (tok < w.vocab))


# ------------------------------------------------------------------ the block inside a HIP graph

@pytest.mark.parametrize("name,batch", [("c2", 8), ("c4", 40)])
def test_graph_capture_replays_match_direct_launches(binding, name, batch):
    """The library enqueues kernels only, so a caller may capture the block in a HIP graph.  Replays with new
    contents in the same buffers, interleaved with direct launches and synchronisations, must reproduce the
    direct results bit for bit (the split recovery's arrival counters are cleared inside the graph)."""
    w = W.scaled(W.WORKLOADS[name], batch=batch, name=f"graph-{name}")
    inp = W.generate(w, "cuda")
    p = binding.make_params(w.batch, w.k_max, w.vocab, W.torch_dtype(w.dtype), lam=w.lam, beta=w.beta,
                            temperature=w.temperature)
    ws = torch.empty(binding.workspace_bytes(p), dtype=torch.uint8, device="cuda")
    mk = lambda dt: torch.empty(w.batch, dtype=dt, device="cuda")
    acc, tok, lp = mk(torch.int32), mk(torch.int32), mk(torch.float32)
    call = lambda a, t, l, wsp: binding.verify_block_raw(inp["G"], inp["S_ctx"], inp["S_noctx"], inp["draft"],
                                                         inp["draft_len"], inp["uniforms"], p, a, t, l, None, None, wsp)
    call(acc, tok, lp, ws)  # warm-up outside the capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        call(acc, tok, lp, ws)
    ws2 = torch.empty_like(ws)
    acc2, tok2, lp2 = mk(torch.int32), mk(torch.int32), mk(torch.float32)
    for rnd in range(4):
        fresh = W.generate(w, "cuda", seed_shift=rnd + 1)
        for k in ("G", "S_ctx", "S_noctx", "draft", "uniforms"):
            inp[k].copy_(fresh[k])
        if inp["draft_len"] is not None:
            inp["draft_len"].copy_(fresh["draft_len"])
        acc.fill_(-7)
        tok.fill_(-7)
        g.replay()
        torch.cuda.synchronize()
        call(acc2, tok2, lp2, ws2)
        torch.cuda.synchronize()
        assert torch.equal(acc, acc2) and torch.equal(tok, tok2) and torch.equal(lp, lp2), rnd


@pytest.mark.parametrize("temperature,beta", [(0.05, 1.0), (0.01, -0.7), (25.0, 3.0), (1e-3, 0.5)])
def test_temperature_and_beta_extremes(binding, oracle, temperature, beta):
    """Near-deterministic rows (tiny T: exponents in the thousands, one token carries the row), nearly flat rows
    (large T: every token matters, the CDF walk crosses many chunks) and a negative steering strength."""
    import dataclasses
    w = dataclasses.replace(W.scaled(W.WORKLOADS["c4"], batch=20, vocab=40000, k_max=6, name=f"T{temperature}"),
                            temperature=temperature, beta=beta)
    inp = W.generate(w, "cuda")
    run_both(binding, oracle, w, inp)


@pytest.mark.parametrize("greedy", [False, True])
@pytest.mark.parametrize("beta", [0.0, 1.2])
@pytest.mark.parametrize("dtype,vocab", [("bf16", 9000), ("f32", 5003)])
def test_many_sequences_use_half_size_workgroups(binding, oracle, greedy, beta, dtype, vocab):
    """B >= 512 runs the recovery with two 8-wave workgroups per compute unit: every variant of that kernel
    (sampled / greedy, steered / beta = 0, aligned / unaligned rows), with flagged sequences in the batch."""
    import dataclasses
    w = dataclasses.replace(W.scaled(W.WORKLOADS["c4"], batch=600, vocab=vocab, k_max=5, name=f"half-{dtype}-{beta}-{greedy}"),
                            dtype=dtype, beta=beta)
    inp = W.generate(w, "cuda")
    inp["draft_len"][17] = 6
    inp["draft"][300, 0] = vocab
    inp["draft_len"][300] = max(1, int(inp["draft_len"][300]))
    out = binding.verify_block(inp["G"], inp["S_ctx"], inp["S_noctx"], inp["draft"], inp["uniforms"], lam=w.lam,
                               beta=w.beta, temperature=w.temperature, draft_len=inp["draft_len"],
                               want_recovery_logprobs=True, want_draft_logprobs=True, greedy=greedy)
    ora = parity.oracle_run(oracle, inp, lam=w.lam, beta=w.beta, temperature=w.temperature, greedy=greedy, num_threads=16)
    rep = parity.compare(out, ora, inp["uniforms"], inp["draft_len"])
    assert out["accepted_len"][17].item() == -1 and out["accepted_len"][300].item() == -1
    assert rep["unexcused_mismatches"] == 0


# ------------------------------------------------------------------ properties that hold at any size

@pytest.mark.parametrize("name", ["c2", "c4"])
def test_sequences_are_independent_of_their_place_in_the_batch(binding, name):
    """Every sequence is verified on its own: shuffling the batch shuffles the outputs, bit for bit (nothing a
    sequence produces may depend on which workgroups, slices or passes its neighbours happened to get)."""
    w = W.WORKLOADS[name]
    inp = W.generate(w, "cuda")
    call = lambda d: binding.verify_block(d["G"], d["S_ctx"], d["S_noctx"], d["draft"], d["uniforms"], lam=w.lam,
                                          beta=w.beta, temperature=w.temperature, draft_len=d["draft_len"],
                                          want_recovery_logprobs=(name == "c2"))
    ref = call(inp)
    perm = torch.randperm(w.batch, generator=torch.Generator("cuda").manual_seed(99), device="cuda")
    shuf = {k: (None if v is None else v[perm].contiguous()) for k, v in inp.items()}
    del inp
    got = call(shuf)
    for k in ("accepted_len", "next_token", "next_token_logprob", "recovery_logprobs"):
        if ref[k] is not None:
            assert torch.equal(ref[k][perm], got[k]), k
    # and a sequence alone gives what it gave inside the batch
    one = {k: (None if v is None else v[3:4].contiguous()) for k, v in shuf.items()}
    solo = call(one)
    for k in ("accepted_len", "next_token"):
        assert torch.equal(solo[k], got[k][3:4]), k
    assert abs(solo["next_token_logprob"].item() - got["next_token_logprob"][3].item()) <= 2e-6


@pytest.mark.parametrize("lam", [1e-30, 1e30, 3.0])
def test_threshold_extremes(binding, oracle, lam):
    """A vanishing threshold accepts every draft token (exp overflows to inf before the min), a huge one rejects at
    the first position; both sides must still agree on the recovery token."""
    import dataclasses
    w = dataclasses.replace(W.scaled(W.WORKLOADS["c4"], batch=24, vocab=20000, k_max=6, name=f"lam{lam}"), lam=lam)
    inp = W.generate(w, "cuda")
    inp["uniforms"].clamp_(min=1e-3)
    out, ora, rep = run_both(binding, oracle, w, inp)
    n = out["accepted_len"].cpu()
    if lam == 1e-30:
        assert torch.equal(n, inp["draft_len"].cpu())
    if lam == 1e30:
        assert torch.all(n[inp["draft_len"].cpu() > 0] == 0)


# ------------------------------------------------------------------ the boundary from plain C

def test_plain_c_caller_without_python_or_torch(binding, oracle, tmp_path):
    """A C99 program (tests/abi_client) stages one block with hipMalloc / hipMemcpy, calls the library and
    writes the outputs to a file: they must be what the oracle says, and bit-identical to the binding's."""
    import subprocess
    import sys

    sys.path.insert(0, str(__import__("pathlib").Path(__file__).parent))
    import abi_client

    exe = abi_client.build()
    w = W.scaled(W.WORKLOADS["c4"], batch=9, vocab=50000, k_max=6, name="c-client")
    inp = W.generate(w, "cuda")
    blob = tmp_path / "in.bin"
    with open(blob, "wb") as f:
        f.write(np.array([w.batch, w.k_max, w.vocab, 1, 1], np.int32).tobytes())
        f.write(np.array([w.lam, w.beta, w.temperature], np.float32).tobytes())
        for k in ("G", "S_ctx", "S_noctx"):
            f.write(inp[k].contiguous().view(torch.int16).cpu().numpy().tobytes())
        f.write(inp["draft"].cpu().numpy().astype(np.int32).tobytes())
        f.write(inp["draft_len"].cpu().numpy().astype(np.int32).tobytes())
        f.write(inp["uniforms"].cpu().numpy().astype(np.float32).tobytes())
    outp = tmp_path / "out.bin"
    r = subprocess.run([exe, str(blob), str(outp)], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stderr
    raw = np.fromfile(outp, dtype=np.int32)
    B = w.batch
    got = {"accepted_len": raw[:B], "next_token": raw[B:2 * B], "next_token_logprob": raw[2 * B:3 * B].view(np.float32)}
    ora = parity.oracle_run(oracle, inp, lam=w.lam, beta=w.beta, temperature=w.temperature, want_recovery_logprobs=False)
    parity.compare(got, ora, inp["uniforms"], inp["draft_len"])
    ref = binding.verify_block(inp["G"], inp["S_ctx"], inp["S_noctx"], inp["draft"], inp["uniforms"], lam=w.lam,
                               beta=w.beta, temperature=w.temperature, draft_len=inp["draft_len"])
    for k in got:
        assert np.array_equal(ref[k].cpu().numpy().view(np.int32), np.asarray(got[k]).view(np.int32)), k


def test_a_uniform_of_one_on_gpu(binding, oracle):
    """Out of contract (uniforms are promised below 1) but harmless: the draw falls back to the last token that has
    any probability, on a row whose tail has none, in the first chunk and across chunks."""
    for V, hot in ((6, [1, 3]), (5000, [17, 4100]), (70000, [5, 65000])):
        G = torch.full((1, 1, V), -1.0e4, dtype=torch.float32, device="cuda")
        G[0, 0, hot] = 0.0
        Z = torch.zeros_like(G)
        d = torch.zeros(1, 0, dtype=torch.int32, device="cuda")
        for us in (1.0, 0.0):
            u = torch.tensor([[us]], dtype=torch.float32, device="cuda")
            out = binding.verify_block(G, Z, Z, d, u)
            ora = oracle.verify_block(G.cpu(), Z.cpu(), Z.cpu(), d.cpu(), u.cpu())
            assert out["next_token"].item() == ora["next_token"][0] == (hot[1] if us == 1.0 else hot[0])
            assert abs(out["next_token_logprob"].item() - np.log(0.5)) < 1e-6


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_a_uniform_of_zero_on_a_row_whose_head_is_far_below_its_maximum(binding, oracle, dtype):
    """The chunk the draw lands in sits ~300 nats under the row's maximum and starts with masked tokens: the pick
    works relative to that chunk's own exponent reference, so token and log-prob are the oracle's."""
    V = 5000
    G = torch.full((2, 1, V), -300.0, dtype=torch.float32, device="cuda")
    G[:, 0, :3] = float("-inf")
    G[:, 0, 2048:] = torch.randn(V - 2048, generator=torch.Generator("cuda").manual_seed(2), device="cuda")
    G[1, 0, :70] = float("-inf")  # more masked tokens than one lane holds: the first live token is another lane's
    G = G.to(dtype)
    Z = torch.zeros_like(G)
    d = torch.zeros(2, 0, dtype=torch.int32, device="cuda")
    u = torch.zeros(2, 1, dtype=torch.float32, device="cuda")
    out = binding.verify_block(G, Z, Z, d, u, want_recovery_logprobs=True)
    ora = oracle.verify_block(G.cpu(), Z.cpu(), Z.cpu(), d.cpu(), u.cpu())
    assert out["next_token"].cpu().tolist() == ora["next_token"].tolist() == [3, 70]
    got = out["next_token_logprob"].double().cpu().numpy()
    assert np.all(np.abs(got - ora["next_token_logprob"]) <= parity.logprob_tol(ora["next_token_logprob"]))
    assert np.all(got < -290)


def test_edge_resample_with_a_uniform_of_one_on_gpu(binding, oracle):
    V = 12
    G = torch.full((1, 1, V), -3.0e4, dtype=torch.float32, device="cuda")
    G[0, 0, [2, 9]] = 0.0
    G[0, 0, [4, 5]] = -1.0e4
    Z = torch.zeros_like(G)
    row = torch.zeros(1, dtype=torch.int32, device="cuda")
    idx, val = binding.cloud_topk(G, Z, row, beta=1.0, topk=4)
    assert idx[0].cpu().tolist() == [2, 9, 4, 5]
    for us, want in [(1.0, 9), (0.75, 9), (0.25, 2)]:
        out = binding.edge_resample(idx, val, Z, row, torch.tensor([us], dtype=torch.float32, device="cuda"), beta=1.0,
                                    temperature=1.0)
        assert out["next_token"].item() == want, (us, out["next_token"].item())


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_tokens_masked_by_the_generalist(binding, oracle, dtype):
    """-inf in G (a logits processor masked the token for the verifier) is probability zero: such a draft token
    is rejected, such a token is never drawn or picked, and everything else is as usual."""
    import dataclasses
    w = dataclasses.replace(W.scaled(W.WORKLOADS["c4"], batch=24, vocab=30000, k_max=6, name=f"masked-{dtype}"), dtype=dtype)
    inp = W.generate(w, "cuda")
    mask = torch.rand(inp["G"].shape, device="cuda", generator=torch.Generator("cuda").manual_seed(4)) < 0.3
    mask[:, :, 1000:1100] = True            # whole 16-byte vectors and a whole stretch masked
    inp["G"][mask] = float("-inf")
    out, ora, rep = run_both(binding, oracle, w, inp)
    tok = out["next_token"].long()
    n = out["accepted_len"].long()
    b = torch.arange(w.batch, device="cuda")
    assert torch.all(torch.isfinite(inp["G"][b, n, tok].float()))          # never a masked token
    lp = out["recovery_logprobs"]
    assert torch.all(lp[mask[b, n]] == float("-inf"))
    assert torch.allclose(torch.exp(lp.double()).sum(-1), torch.ones(w.batch, dtype=torch.float64, device="cuda"), atol=1e-5)
    # a masked draft token is rejected on the spot (its uniform is positive)
    d0 = inp["draft"][:, 0].long()
    masked_first = mask[b, 0, d0] & (inp["draft_len"] > 0) & (inp["uniforms"][:, 0] > 0)
    assert torch.all(n[masked_first] == 0) and masked_first.any()
    g = binding.verify_block(inp["G"], inp["S_ctx"], inp["S_noctx"], inp["draft"], inp["uniforms"], lam=w.lam,
                             beta=w.beta, temperature=w.temperature, draft_len=inp["draft_len"], greedy=True)
    og = parity.oracle_run(oracle, inp, lam=w.lam, beta=w.beta, temperature=w.temperature, greedy=True,
                           want_recovery_logprobs=False)
    parity.compare(g, og, inp["uniforms"], inp["draft_len"])


def test_cloud_topk_with_masked_tokens(binding, oracle):
    w = W.scaled(W.WORKLOADS["c4"], batch=6, vocab=40000, k_max=2, name="topk-masked")
    inp = W.generate(w, "cuda")
    mask = torch.rand(inp["G"].shape, device="cuda", generator=torch.Generator("cuda").manual_seed(6)) < 0.5
    mask[0, :, 40:] = True          # fewer finite logits than the payload holds: the rest of it is -inf entries, lowest ids first
    inp["G"][mask] = float("-inf")
    row = torch.tensor([0, 1, 2, 0, 1, 2], dtype=torch.int32, device="cuda")
    idx, val = binding.cloud_topk(inp["G"], inp["S_noctx"], row, beta=w.beta, topk=32)
    oidx, oval = oracle.cloud_topk(inp["G"].cpu(), inp["S_noctx"].cpu(), row.cpu(), beta=w.beta, topk=32)
    assert np.array_equal(idx.cpu().numpy(), oidx) and np.array_equal(val.cpu().numpy(), oval)


@pytest.mark.parametrize("dtype,batch", [("bf16", 24), ("f32", 24), ("bf16", 600)])
def test_tokens_masked_in_every_model(binding, oracle, dtype, batch):
    """A vocabulary mask shared by the three models, plus tokens masked for the specialist only (with and without
    context): no inf - inf anywhere, masked tokens have no probability, the rest of the row is as usual."""
    import dataclasses
    w = dataclasses.replace(W.scaled(W.WORKLOADS["c4"], batch=batch, vocab=20000, k_max=5, name=f"mask3-{dtype}-{batch}"),
                            dtype=dtype)
    inp = W.generate(w, "cuda")
    gen = torch.Generator("cuda").manual_seed(8)
    common = torch.rand(inp["G"].shape, device="cuda", generator=gen) < 0.25
    common[:, :, 4096:4200] = True
    spec_only = (torch.rand(inp["G"].shape, device="cuda", generator=gen) < 0.1) & ~common
    b = torch.arange(w.batch, device="cuda").view(-1, 1).expand(-1, w.k_max)
    t = torch.arange(w.k_max, device="cuda").view(1, -1).expand(w.batch, -1)
    common[b, t, inp["draft"].long()] = False        # drafted tokens stay ordinary
    spec_only[b, t, inp["draft"].long()] = False
    inp["G"][common] = float("-inf")
    inp["S_ctx"][common | spec_only] = float("-inf")
    inp["S_noctx"][common | spec_only] = float("-inf")
    out, ora, rep = run_both(binding, oracle, w, inp)
    n, tok = out["accepted_len"].long(), out["next_token"].long()
    bb = torch.arange(w.batch, device="cuda")
    assert not common[bb, n, tok].any()
    lp = out["recovery_logprobs"]
    assert torch.all(lp[common[bb, n]] == float("-inf")) and torch.all(torch.isfinite(lp[~common[bb, n]]))
    g = binding.verify_block(inp["G"], inp["S_ctx"], inp["S_noctx"], inp["draft"], inp["uniforms"], lam=w.lam,
                             beta=w.beta, temperature=w.temperature, draft_len=inp["draft_len"], greedy=True)
    og = parity.oracle_run(oracle, inp, lam=w.lam, beta=w.beta, temperature=w.temperature, greedy=True,
                           want_recovery_logprobs=False, num_threads=16)
    parity.compare(g, og, inp["uniforms"], inp["draft_len"])
    # the deployment split on the same rows
    row = out["accepted_len"].clamp(min=0)
    idx, val = binding.cloud_topk(inp["G"], inp["S_noctx"], row, beta=w.beta, topk=32)
    sel = torch.arange(0, w.batch, max(1, w.batch // 24), device="cuda")
    oidx, oval = oracle.cloud_topk(inp["G"][sel].cpu(), inp["S_noctx"][sel].cpu(), row[sel].cpu(), beta=w.beta, topk=32)
    assert np.array_equal(idx[sel].cpu().numpy(), oidx) and np.array_equal(val[sel].cpu().numpy(), oval)


def test_gpu_against_the_frozen_oracle_block(binding):
    """The stored expected values were written by tests/golden/make_oracle_fixture.py, which calls only the oracle."""
    import importlib.util
    import json
    import os

    here = os.path.dirname(os.path.abspath(__file__))
    spec = importlib.util.spec_from_file_location("make_oracle_fixture", os.path.join(here, "golden", "make_oracle_fixture.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    want = json.load(open(os.path.join(here, "golden", "oracle_block_fixture.json")))["outputs"]
    G, Sp, Sm, draft, draft_len, u = mod.build_inputs()
    dev = "cuda"
    t = lambda a, dt=None: torch.from_numpy(np.ascontiguousarray(a)).to(dev) if dt is None else torch.from_numpy(np.ascontiguousarray(a)).to(dev).to(dt)
    for dtype, tdt in (("f32", torch.float32), ("bf16", torch.bfloat16)):
        for greedy in (False, True):
            w = want[f"{dtype}{'-greedy' if greedy else ''}"]
            out = binding.verify_block(t(G, tdt), t(Sp, tdt), t(Sm, tdt), t(draft), t(u), lam=0.5, beta=0.75,
                                       temperature=0.8, draft_len=t(draft_len), greedy=greedy)
            assert out["accepted_len"].cpu().tolist() == w["accepted_len"]
            assert out["next_token"].cpu().tolist() == w["next_token"]
            for got, exp in zip(out["next_token_logprob"].cpu().tolist(), w["next_token_logprob"]):
                assert (exp is None and got != got) or abs(got - exp) <= 1e-5
    s = want["split"]
    idx, val = binding.cloud_topk(t(G), t(Sm), t(np.array(s["row"], np.int32)), beta=0.75, topk=4)
    assert idx.cpu().tolist() == s["index"]
    assert np.array_equal(val.cpu().numpy(), np.array(s["value"], np.float32))
    e = binding.edge_resample(idx, val, t(Sp), t(np.array(s["row"], np.int32)), t(u[:, -1].copy()), beta=0.75, temperature=0.8)
    assert e["next_token"].cpu().tolist() == s["next_token"]
    assert np.allclose(e["next_token_logprob"].cpu().numpy(), np.array(s["next_token_logprob"]), atol=1e-5)


@pytest.mark.parametrize("name,batch", [("c2", 8), ("c4", 160)])
def test_timed_entry_point_gives_the_same_outputs_and_sane_times(binding, name, batch):
    """specsteer_verify_block_timed is the same operation bracketed with events: identical outputs, one
    non-negative time per stage, stages that do not run report (close to) nothing."""
    w = W.scaled(W.WORKLOADS[name], batch=batch, name=f"timed-{name}")
    inp = W.generate(w, "cuda")
    p = binding.make_params(w.batch, w.k_max, w.vocab, W.torch_dtype(w.dtype), lam=w.lam, beta=w.beta,
                            temperature=w.temperature)
    ws = torch.empty(binding.workspace_bytes(p), dtype=torch.uint8, device="cuda")
    mk = lambda dt: torch.empty(w.batch, dtype=dt, device="cuda")
    a1, t1, l1, a2, t2, l2 = mk(torch.int32), mk(torch.int32), mk(torch.float32), mk(torch.int32), mk(torch.int32), mk(torch.float32)
    args = (inp["G"], inp["S_ctx"], inp["S_noctx"], inp["draft"], inp["draft_len"], inp["uniforms"], p)
    binding.verify_block_raw(*args, a1, t1, l1, None, None, ws)
    ms = binding.verify_block_raw(*args, a2, t2, l2, None, None, ws, timed=True)
    torch.cuda.synchronize()
    assert torch.equal(a1, a2) and torch.equal(t1, t2) and torch.equal(l1, l2)
    assert set(ms) == set(binding.STAGES) and all(0.0 <= v < 50.0 for v in ms.values())
    two_pass = binding.first_window(p) < w.k_max
    assert ms["row_pass1"] > 0 and ms["recover"] > 0
    if not two_pass:
        assert ms["verdict"] < 0.02 and ms["row_pass2"] < 0.02


def test_concurrent_calls_from_several_threads_and_streams(binding):
    """The header promises re-entrancy across streams given distinct workspaces: four host threads, each on its
    own stream with its own workspace and outputs, repeatedly verify different blocks at once; every result must
    be what the same block gives when verified alone."""
    import threading

    w = W.scaled(W.WORKLOADS["c4"], batch=40, vocab=60000, k_max=8, name="threads")
    jobs = []
    for i in range(4):
        inp = W.generate(w, "cuda", seed_shift=i)
        ref = binding.verify_block(inp["G"], inp["S_ctx"], inp["S_noctx"], inp["draft"], inp["uniforms"], lam=w.lam,
                                   beta=w.beta, temperature=w.temperature, draft_len=inp["draft_len"])
        jobs.append((inp, ref))
    torch.cuda.synchronize()
    errors = []

    def work(i):
        try:
            inp, ref = jobs[i]
            stream = torch.cuda.Stream()
            with torch.cuda.stream(stream):
                for _ in range(25):
                    out = binding.verify_block(inp["G"], inp["S_ctx"], inp["S_noctx"], inp["draft"], inp["uniforms"],
                                               lam=w.lam, beta=w.beta, temperature=w.temperature,
                                               draft_len=inp["draft_len"])
                    stream.synchronize()
                    for k in ("accepted_len", "next_token", "next_token_logprob"):
                        if not torch.equal(out[k], ref[k]):
                            errors.append((i, k))
        except Exception as e:  # surfaced in the main thread below
            errors.append((i, repr(e)))

    threads = [threading.Thread(target=work, args=(i,)) for i in range(4)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=100)
    assert not any(t.is_alive() for t in threads)
    assert not errors, errors[:5]


# ------------------------------------------------------------------ random configurations

def random_case(seed):
    """One seeded configuration inside the documented limits: shapes, dtype, hyper-parameters, raggedness,
    row padding, decoding mode and requested outputs all drawn at random."""
    import dataclasses
    rng = np.random.default_rng(1000 + seed)
    B = int(rng.choice([1, 2, 3, 5, 8, 17, 33, 64, 100, 129, 200, 300, 520]))
    K = int(rng.choice([0, 1, 2, 3, 4, 5, 8, 13, 16, 20]))
    V = int(rng.choice([1, 7, 64, 777, 2048, 4099, 20000, 32776, 50001, 70000]))
    while B * (K + 1) * V > 120_000_000:       # keep the oracle's share of the test short
        B = max(1, B // 2)
    pad = int(rng.choice([0, 0, 8 - V % 8 if V % 8 else 8, 3]))
    w = dataclasses.replace(
        W.scaled(W.WORKLOADS[str(rng.choice(["c2", "c3", "c4", "c5"]))], batch=B, vocab=V + pad, k_max=K, name=f"rand{seed}"),
        dtype=str(rng.choice(["bf16", "f32"])), beta=float(rng.choice([0.0, 0.5, 1.0, 1.5, -0.5])),
        lam=float(rng.choice([0.5, 1.0, 0.1, 2.0])), temperature=float(rng.choice([1.0, 0.7, 1.6, 0.2])))
    return w, V, pad, bool(rng.integers(2)), bool(rng.integers(2)), bool(rng.integers(2)), rng


@pytest.mark.parametrize("seed", range(24))
def test_random_configurations(binding, oracle, seed):
    import dataclasses
    w, V, pad, greedy, want_rec, want_dlp, rng = random_case(seed)
    inp = W.generate(w, "cuda")
    if pad:
        for k in ("G", "S_ctx", "S_noctx"):
            inp[k][..., V:] = float("nan")
            inp[k] = inp[k][..., :V]
        inp["draft"] = inp["draft"].clamp(max=V - 1)
    if inp["draft_len"] is None and w.k_max > 0 and rng.integers(2):
        inp["draft_len"] = torch.from_numpy(rng.integers(0, w.k_max + 1, w.batch).astype(np.int32)).cuda()
    w = dataclasses.replace(w, vocab=V)
    out = binding.verify_block(inp["G"], inp["S_ctx"], inp["S_noctx"], inp["draft"], inp["uniforms"], lam=w.lam,
                               beta=w.beta, temperature=w.temperature, draft_len=inp["draft_len"], greedy=greedy,
                               want_recovery_logprobs=want_rec, want_draft_logprobs=want_dlp)
    ora = parity.oracle_run(oracle, inp, lam=w.lam, beta=w.beta, temperature=w.temperature, greedy=greedy,
                            want_recovery_logprobs=want_rec, num_threads=16)
    rep = parity.compare(out, ora, inp["uniforms"], inp["draft_len"])
    assert rep["unexcused_mismatches"] == 0
