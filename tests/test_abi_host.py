"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares,
and rejects bad arguments on the host before anything is enqueued (no GPU work happens in
any of these calls: argument errors return first, and batch == 0 is a no-op)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2603_16219_amd import binding

    return binding.library()


@pytest.fixture(scope="module")
def B():
    from paper_2603_16219_amd import binding

    return binding


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "specsteer.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(specsteer_\w+)\s*\(", text)))


def test_library_exports_every_declared_symbol(lib):
    names = declared_symbols()
    assert names == ["specsteer_cloud_topk", "specsteer_edge_resample", "specsteer_first_window",
                     "specsteer_status_string",
                     "specsteer_verify_block", "specsteer_verify_block_static", "specsteer_verify_block_timed", "specsteer_version",
                     "specsteer_workspace_bytes"]
    for n in names:
        assert getattr(lib, n) is not None


def test_version_and_status_strings(B):
    assert B.version() >= 100
    seen = {B.status_string(i) for i in range(8)}
    assert len(seen) == 8 and B.status_string(0) == "ok" and B.status_string(99) == "unknown status"


def test_params_struct_matches_header_layout(B):
    # int32 x4, int64 x2, float x3, uint32: 48 bytes, strides 8-byte aligned at offset 16
    assert ctypes.sizeof(B.SSParams) == 48
    assert B.SSParams.stride_b.offset == 16 and B.SSParams.lambda_.offset == 32 and B.SSParams.flags.offset == 44


def test_workspace_bytes(B):
    import torch

    p = B.make_params(256, 16, 128256, torch.bfloat16, lam=0.5, beta=0.8, temperature=0.7)
    n = B.workspace_bytes(p)
    assert n % 256 == 0 and 0 < n < 64 << 20
    assert B.workspace_bytes(B.make_params(0, 0, 1, torch.float32, lam=0.5, beta=1.0, temperature=1.0)) > 0
    for bad in (dict(batch=-1), dict(k_max=-1), dict(vocab=0), dict(vocab=(1 << 20) + 1), dict(k_max=1025)):
        kw = dict(batch=4, k_max=4, vocab=100)
        kw.update(bad)
        assert B.workspace_bytes(B.make_params(kw["batch"], kw["k_max"], kw["vocab"], torch.float32, lam=0.5,
                                               beta=1.0, temperature=1.0)) == 0
    p.dtype = 7
    assert B.workspace_bytes(p) == 0
    assert B.library().specsteer_workspace_bytes(None) == 0


def call(B, params, *, null=None, ws=256, ws_bytes=1 << 30, nudge=None):
    """Invoke the entry point with fake, never-dereferenced device addresses."""
    fake = {k: 4096 * (i + 1) for i, k in enumerate(
        ["G", "S_ctx", "S_noctx", "draft", "draft_len", "uniforms", "accepted_len", "next_token", "ntl", "rec",
         "dlp"])}
    if null:
        fake[null] = 0
    if nudge:
        fake[nudge[0]] += nudge[1]
    v = lambda k: ctypes.c_void_p(fake[k])
    return B.library().specsteer_verify_block(
        v("G"), v("S_ctx"), v("S_noctx"), v("draft"), v("draft_len"), v("uniforms"),
        ctypes.byref(params) if params is not None else None, v("accepted_len"), v("next_token"), v("ntl"),
        v("rec"), v("dlp"), ctypes.c_void_p(ws), ctypes.c_size_t(ws_bytes), None)


def test_argument_errors_are_reported_on_the_host(B):
    import torch

    def P(**kw):
        base = dict(batch=0, k_max=4, vocab=1000, lam=0.5, beta=1.0, temperature=1.0, stride_b=0, stride_t=0, flags=0)
        base.update(kw)
        return B.make_params(base["batch"], base["k_max"], base["vocab"], torch.bfloat16, lam=base["lam"],
                             beta=base["beta"], temperature=base["temperature"], stride_b=base["stride_b"],
                             stride_t=base["stride_t"], flags=base["flags"])

    OK, NULL, SHAPE, DTYPE, PARAM, STRIDE, WS = 0, 1, 2, 3, 4, 5, 6
    assert call(B, P()) == OK  # batch == 0: validated, nothing launched
    assert call(B, None) == NULL
    for k in ("G", "S_ctx", "S_noctx", "draft", "uniforms", "accepted_len", "next_token"):
        assert call(B, P(), null=k) == NULL, k
    for k in ("draft_len", "ntl", "rec", "dlp"):  # optional pointers
        assert call(B, P(), null=k) == OK, k
    assert call(B, P(k_max=0), null="draft") == OK
    assert call(B, P(batch=-1)) == SHAPE
    assert call(B, P(vocab=0)) == SHAPE
    assert call(B, P(k_max=2000)) == SHAPE
    p = P()
    p.dtype = 2
    assert call(B, p) == DTYPE
    for kw in (dict(lam=0.0), dict(lam=-1.0), dict(lam=float("inf")), dict(lam=float("nan")),
               dict(temperature=0.0), dict(temperature=float("nan")), dict(beta=float("inf")), dict(flags=4), dict(flags=0x80000001)):
        assert call(B, P(**kw)) == PARAM, kw
    assert call(B, P(stride_t=999)) == STRIDE       # rows would overlap
    assert call(B, P(stride_t=1000, stride_b=4999)) == STRIDE
    assert call(B, P(stride_t=-8)) == STRIDE
    assert call(B, P(stride_t=1008, stride_b=5 * 1008)) == OK
    for k in ("G", "S_ctx", "S_noctx"):             # bf16 logits must sit on 2-byte boundaries, nothing more
        assert call(B, P(), nudge=(k, 1)) == STRIDE, k
        assert call(B, P(), nudge=(k, 2)) == OK, k
    assert call(B, P(), ws=0) == WS
    assert call(B, P(), ws=128) == WS               # not 256-byte aligned
    assert call(B, P(batch=4), ws_bytes=16) == WS   # too small; rejected before any launch


def test_python_wrapper_refuses_cpu_tensors(B):
    import torch

    x = torch.zeros(1, 2, 8)
    with pytest.raises(ValueError):
        B.verify_block(x, x, x, torch.zeros(1, 1, dtype=torch.int32), torch.zeros(1, 2))


def test_python_wrappers_refuse_misshapen_arguments_before_any_launch(B):
    """The kernels index draft, uniforms, draft_len, row, uniform, index and value by the batch and block
    shape alone, so the wrappers refuse anything else (shape checks come before the device check, which is
    what lets them run here without a GPU)."""
    import torch

    Bn, K, V = 3, 4, 16
    x = torch.zeros(Bn, K + 1, V)
    d, u, dl = torch.zeros(Bn, K, dtype=torch.int32), torch.zeros(Bn, K + 1), torch.zeros(Bn, dtype=torch.int32)
    for bad in (dict(draft=torch.zeros(Bn, K - 1, dtype=torch.int32)), dict(uniforms=torch.zeros(Bn, K)),
                dict(uniforms=torch.zeros(Bn * (K + 1))), dict(draft_len=torch.zeros(Bn - 1, dtype=torch.int32)),
                dict(draft=torch.zeros(Bn - 1, K, dtype=torch.int32))):
        kw = dict(draft=d, uniforms=u, draft_len=dl)
        kw.update(bad)
        with pytest.raises(ValueError, match="must be"):
            B.verify_block(x, x, x, kw["draft"], kw["uniforms"], draft_len=kw["draft_len"])
    with pytest.raises(ValueError, match="no CPU path"):       # well-shaped, but not on a device
        B.verify_block(x, x, x, d, u, draft_len=dl)
    with pytest.raises(ValueError, match="row must be"):
        B.cloud_topk(x, x, torch.zeros(Bn + 1, dtype=torch.int32))
    idx, val = torch.zeros(Bn, 32, dtype=torch.int32), torch.zeros(Bn, 32)
    row, un = torch.zeros(Bn, dtype=torch.int32), torch.zeros(Bn)
    with pytest.raises(ValueError, match="index and value"):
        B.edge_resample(idx, val[:, :16], x, row, un)
    with pytest.raises(ValueError, match="index and value"):
        B.edge_resample(idx[:2], val[:2], x, row, un)
    with pytest.raises(ValueError, match="row and uniform"):
        B.edge_resample(idx, val, x, row, un[:2])
    with pytest.raises(ValueError, match="int32"):
        B.edge_resample(idx.long(), val, x, row, un)
    with pytest.raises(ValueError, match="one uniform per row"):
        B.steer_rows(x[0], x[0], x[0], torch.zeros(K))


def test_split_entry_points_reject_bad_arguments_on_the_host(B):
    import torch

    lib = B.library()
    P = lambda **kw: B.make_params(kw.get("batch", 0), 4, kw.get("vocab", 1000), torch.bfloat16, lam=0.5,
                                   beta=kw.get("beta", 1.0), temperature=kw.get("temperature", 1.0),
                                   flags=kw.get("flags", 0))
    f = lambda x: ctypes.c_void_p(x)
    cloud = lambda p, topk=32, g=4096: lib.specsteer_cloud_topk(f(g), f(8192), f(12288), ctypes.byref(p), topk,
                                                                f(16384), f(20480), None)
    edge = lambda p, topk=32, u=4096: lib.specsteer_edge_resample(f(4096), f(8192), f(12288), f(16384), f(u),
                                                                  ctypes.byref(p), topk, f(20480), f(24576), None)
    assert cloud(P()) == 0 and edge(P()) == 0               # batch == 0: validated, nothing launched
    assert cloud(P(), topk=0) == 2 and cloud(P(), topk=65) == 2 and edge(P(), topk=0) == 2
    assert cloud(P(), g=0) == 1 and edge(P(), u=0) == 1
    assert edge(P(flags=1), u=0) == 0                       # greedy needs no uniform
    assert cloud(P(beta=float("nan"))) == 4 and edge(P(temperature=0.0)) == 4 and cloud(P(flags=8)) == 4
    assert cloud(P(vocab=0)) == 2
    assert lib.specsteer_cloud_topk(f(1), f(1), f(1), None, 32, f(1), f(1), None) == 1


def test_static_scratch_entry_point_checks_its_limit_on_the_host(B):
    import torch

    lib = B.library()
    f = lambda x: ctypes.c_void_p(x)
    call = lambda p: lib.specsteer_verify_block_static(f(4096), f(4096), f(4096), f(4096), None, f(4096), ctypes.byref(p),
                                                       f(4096), f(4096), None, None, None, None)
    big = B.make_params(4096, 64, 1 << 20, torch.bfloat16, lam=0.5, beta=1.0, temperature=1.0)
    assert B.workspace_bytes(big) > B.STATIC_SCRATCH_BYTES and call(big) == 6   # refused before any GPU call
    assert call(B.make_params(1, 2000, 100, torch.bfloat16, lam=0.5, beta=1.0, temperature=1.0)) == 2
    assert lib.specsteer_verify_block_static(None, None, None, None, None, None, None, None, None, None, None, None, None) == 1
    hdr = open(os.path.join(ROOT, "include", "specsteer.h")).read()
    assert re.search(r"#define SS_STATIC_SCRATCH_BYTES \(8u << 20\)", hdr) and B.STATIC_SCRATCH_BYTES == 8 << 20


def test_first_window(B):
    import torch

    big = B.make_params(256, 16, 128256, torch.bfloat16, lam=0.5, beta=0.8, temperature=0.7)
    assert B.first_window(big) == 4
    big.flags = B.SS_FLAG_FULL_ROWS
    assert B.first_window(big) == 16
    assert B.first_window(B.make_params(8, 8, 151936, torch.bfloat16, lam=0.5, beta=1.0, temperature=1.0)) == 8   # small batch
    assert B.first_window(B.make_params(512, 3, 256000, torch.bfloat16, lam=0.5, beta=1.0, temperature=1.0)) == 3  # short block
    assert B.first_window(B.make_params(-1, 3, 10, torch.bfloat16, lam=0.5, beta=1.0, temperature=1.0)) == -1


def test_header_is_plain_c():
    """The boundary is a C ABI: the header must compile as C99 and as C++ on its own."""
    import subprocess

    hdr = os.path.join(ROOT, "include", "specsteer.h")
    for lang, std in (("c", "-std=c99"), ("c++", "-std=c++11")):
        r = subprocess.run(["gcc", "-x", lang, std, "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", hdr],
                           capture_output=True, text=True)
        assert r.returncode == 0, r.stderr


def test_plain_c_client_builds_against_the_library(lib):
    import sys

    sys.path.insert(0, os.path.join(ROOT, "tests"))
    import abi_client

    assert os.path.exists(abi_client.build())
