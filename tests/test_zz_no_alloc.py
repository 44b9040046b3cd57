"""GPU test of specsteer_verify_block_static, the entry point for callers that cannot allocate: the block on
the library's own scratch array must give what specsteer_verify_block gives on a caller's workspace, on two
calls in a row, the second on a smaller block (stale contents of the shared array must not matter)."""
import ctypes

import pytest
import torch

from paper_2603_16219_amd import workloads as W

pytestmark = pytest.mark.gpu


def _both(binding, w, greedy=False, want_rows=False):
    inp = W.generate(w, "cuda")
    B, K, V = w.batch, w.k_max, w.vocab
    p = binding.make_params(B, K, V, W.torch_dtype(w.dtype), lam=w.lam, beta=w.beta, temperature=w.temperature,
                            flags=binding.SS_FLAG_GREEDY if greedy else 0)
    assert binding.workspace_bytes(p) <= binding.STATIC_SCRATCH_BYTES
    ws = torch.empty(binding.workspace_bytes(p), dtype=torch.uint8, device="cuda")
    mk = lambda dt, *shape: torch.full(shape, -7, dtype=dt, device="cuda")
    ref = [mk(torch.int32, B), mk(torch.int32, B), mk(torch.float32, B),
           mk(torch.float32, B, V) if want_rows else None, mk(torch.float32, B, K, 2) if want_rows else None]
    got = [None if t is None else t.clone() for t in ref]
    args = (inp["G"], inp["S_ctx"], inp["S_noctx"], inp["draft"] if K else None, inp["draft_len"], inp["uniforms"], p)
    binding.verify_block_raw(*args, *ref, ws)
    binding.verify_block_static_raw(*args, *got)
    torch.cuda.synchronize()
    for r, g, name in zip(ref, got, ("accepted_len", "next_token", "next_token_logprob", "recovery_logprobs", "draft_logprobs")):
        if r is not None:
            assert torch.equal(r, g), (w.name, name)   # same kernels, same arithmetic: bit for bit
    assert torch.all(ref[0] >= 0)


def test_static_scratch_entry_point_matches_the_workspace_one(binding_mod):
    binding = binding_mod
    # a block with ragged lengths that takes the early-exit schedule, then a smaller one on the same array,
    # then a small batch (recovery rows shared between workgroups: arrival counters live in the scratch)
    _both(binding, W.scaled(W.WORKLOADS["c4"], batch=96, vocab=100000, name="static-big"))
    _both(binding, W.scaled(W.WORKLOADS["c4"], batch=20, vocab=30000, k_max=5, name="static-small"), want_rows=True)
    _both(binding, W.scaled(W.WORKLOADS["c2"], batch=3, vocab=151936, name="static-split"), greedy=True)
    _both(binding, W.scaled(W.WORKLOADS["c2"], batch=3, vocab=151936, name="static-split-again"))
    _both(binding, W.scaled(W.WORKLOADS["c1"], batch=9, vocab=4000, k_max=0, name="static-rows"))


def test_static_scratch_entry_point_refuses_blocks_beyond_its_limit(binding_mod):
    binding = binding_mod
    p = binding.make_params(4096, 64, 1 << 20, torch.bfloat16, lam=0.5, beta=1.0, temperature=1.0)
    assert binding.workspace_bytes(p) > binding.STATIC_SCRATCH_BYTES
    x = torch.zeros(8, device="cuda")
    with pytest.raises(binding.SpecSteerError) as e:
        binding.verify_block_static_raw(x, x, x, x, None, x, p, x, x, x, None, None)
    assert e.value.status == 6


@pytest.fixture(scope="module")
def binding_mod():
    from paper_2603_16219_amd import binding as b

    assert torch.cuda.is_available(), "GPU tests need a device"
    b.library()
    return b


def test_static_scratch_entry_point_inside_a_hip_graph(binding_mod):
    """The callers this entry point is for: the block captured in a HIP graph (no allocation, no workspace argument),
    replayed on new contents of the same buffers, with eager work and synchronisations between the replays; every replay
    must equal the workspace entry point's direct result bit for bit."""
    binding = binding_mod
    w = W.scaled(W.WORKLOADS["c4"], batch=48, vocab=60000, name="static-graph")
    inp = W.generate(w, "cuda")
    B, K, V = w.batch, w.k_max, w.vocab
    p = binding.make_params(B, K, V, torch.bfloat16, lam=w.lam, beta=w.beta, temperature=w.temperature)
    mk = lambda dt: torch.full((B,), -7, dtype=dt, device="cuda")
    acc, tok, lp = mk(torch.int32), mk(torch.int32), mk(torch.float32)
    args = (inp["G"], inp["S_ctx"], inp["S_noctx"], inp["draft"], inp["draft_len"], inp["uniforms"], p)
    binding.verify_block_static_raw(*args, acc, tok, lp, None, None)   # first call on the device: outside any capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        binding.verify_block_static_raw(*args, acc, tok, lp, None, None)
    ws = torch.empty(binding.workspace_bytes(p), dtype=torch.uint8, device="cuda")
    acc2, tok2, lp2 = mk(torch.int32), mk(torch.int32), mk(torch.float32)
    for rnd in range(4):
        fresh = W.generate(w, "cuda", seed_shift=rnd + 1)
        for k in ("G", "S_ctx", "S_noctx", "draft", "uniforms", "draft_len"):
            inp[k].copy_(fresh[k])
        acc.fill_(-7)
        tok.fill_(-7)
        g.replay()
        torch.cuda.synchronize()
        binding.verify_block_raw(*args, acc2, tok2, lp2, None, None, ws)
        torch.cuda.synchronize()
        assert torch.equal(acc, acc2) and torch.equal(tok, tok2) and torch.equal(lp, lp2), rnd
        assert torch.all(acc >= 0)
