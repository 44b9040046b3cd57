"""Float64 CPU oracle for SpecSteer's verify-and-recover block (Algorithm 1, Eq. 7, Eq. 8).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
benchmark's cpu_baseline leg.  Nothing in the product package imports it and
it imports nothing from the product package.

The arithmetic lives in ``specsteer_oracle.c`` (plain C, double precision);
this module compiles it with gcc on first use and marshals numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "specsteer_oracle.c")
_LIB = os.path.join(_HERE, "libspecsteer_oracle.so")

F32, BF16 = 0, 1


class _Params(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32),
        ("k_max", ctypes.c_int32),
        ("vocab", ctypes.c_int32),
        ("dtype", ctypes.c_int32),
        ("stride_b", ctypes.c_int64),
        ("stride_t", ctypes.c_int64),
        ("lambda_", ctypes.c_float),
        ("beta", ctypes.c_float),
        ("temperature", ctypes.c_float),
        ("num_threads", ctypes.c_int32),
        ("greedy", ctypes.c_int32),
    ]


# The pin suite's mutation test points this at deliberately wrong builds of the oracle to show that
# the pins notice; nothing else sets it.
_LIB_OVERRIDE = os.environ.get("SPECSTEER_ORACLE_LIBRARY")


def build(force: bool = False) -> str:
    """Compile the C oracle into a shared library next to its source."""
    if _LIB_OVERRIDE:
        return _LIB_OVERRIDE
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.specsteer_oracle_verify_block.restype = ctypes.c_int
        lib.specsteer_oracle_verify_block.argtypes = [ctypes.c_void_p] * 14
        lib.specsteer_oracle_max_threads.restype = ctypes.c_int
        lib.specsteer_oracle_cloud_topk.restype = ctypes.c_int
        lib.specsteer_oracle_cloud_topk.argtypes = [ctypes.c_void_p] * 4 + [ctypes.c_int32] + [ctypes.c_void_p] * 2
        lib.specsteer_oracle_edge_resample.restype = ctypes.c_int
        lib.specsteer_oracle_edge_resample.argtypes = [ctypes.c_void_p] * 6 + [ctypes.c_int32] + [ctypes.c_void_p] * 4
        _lib = lib
    return _lib


def max_threads() -> int:
    return int(_load().specsteer_oracle_max_threads())


def _logits_array(x):
    """Accept a numpy float32 array, a numpy uint16 array of bf16 bit patterns,
    or a CPU torch tensor (float32 / bfloat16).  Returns (contiguous ndarray, dtype code)."""
    if hasattr(x, "detach"):  # torch tensor, without importing torch here
        t = x.detach().cpu().contiguous()
        if str(t.dtype) == "torch.bfloat16":
            import torch

            return t.view(torch.int16).numpy().view(np.uint16), BF16
        if str(t.dtype) == "torch.float32":
            return t.numpy(), F32
        raise TypeError(f"unsupported logits dtype {t.dtype}")
    a = np.ascontiguousarray(x)
    if a.dtype == np.float32:
        return a, F32
    if a.dtype == np.uint16:
        return a, BF16
    raise TypeError(f"unsupported logits dtype {a.dtype}")


def _int32(x):
    if hasattr(x, "detach"):
        x = x.detach().cpu().numpy()
    return np.ascontiguousarray(x, dtype=np.int32)


def verify_block(G, S_ctx, S_noctx, draft, uniforms, *, lam=0.5, beta=1.0, temperature=1.0,
                 draft_len=None, want_recovery_logprobs=True, num_threads=1, greedy=False):
    """Run the oracle on host arrays shaped [B, k_max+1, V] (logits), [B, k_max]
    (draft), [B, k_max+1] (uniforms).  Returns a dict of numpy arrays."""
    g, dt = _logits_array(G)
    sp, dt2 = _logits_array(S_ctx)
    sm, dt3 = _logits_array(S_noctx)
    if not (dt == dt2 == dt3) or not (g.shape == sp.shape == sm.shape) or g.ndim != 3:
        raise ValueError("logit tensors must share dtype and [B, k_max+1, V] shape")
    B, k1, V = g.shape
    kmax = k1 - 1
    # a zero-length draft still needs a non-null pointer for the C side
    d = _int32(draft).reshape(B, kmax) if B * kmax > 0 else np.zeros(1, np.int32)
    if hasattr(uniforms, "detach"):
        uniforms = uniforms.detach().cpu().numpy()
    u = np.ascontiguousarray(uniforms, dtype=np.float32).reshape(B, k1)
    dl = None if draft_len is None else _int32(draft_len).reshape(B)

    p = _Params(B, kmax, V, dt, 0, 0, float(lam), float(beta), float(temperature), int(num_threads),
                1 if greedy else 0)
    acc = np.empty(B, np.int32)
    tok = np.empty(B, np.int32)
    tok_lp = np.empty(B, np.float64)
    rec = np.empty((B, V), np.float64) if want_recovery_logprobs else None
    dlp = np.empty((B, kmax, 2), np.float64)
    alpha = np.empty((B, kmax), np.float64)
    margin = np.empty(B, np.float64)

    def ptr(a):
        return None if a is None else a.ctypes.data_as(ctypes.c_void_p)

    rc = _load().specsteer_oracle_verify_block(
        ptr(g), ptr(sp), ptr(sm), ptr(d),
        ptr(dl), ptr(u), ctypes.cast(ctypes.byref(p), ctypes.c_void_p),
        ptr(acc), ptr(tok), ptr(tok_lp), ptr(rec), ptr(dlp), ptr(alpha), ptr(margin))
    if rc != 0:
        raise ValueError("oracle rejected its arguments")
    return {
        "accepted_len": acc,
        "next_token": tok,
        "next_token_logprob": tok_lp,
        "recovery_logprobs": rec,
        "draft_logprobs": dlp,
        "alpha": alpha,
        "sample_margin": margin,
    }


def _cptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def cloud_topk(G, S_noctx, row, *, beta=1.0, topk=32):
    """Cloud side of the deployment split: top-k of h_LLM - beta*h_SLM^- at row[b] of every sequence.
    Returns (index [B, topk] int32, value [B, topk] float32), ordered by decreasing value, ties by id."""
    g, dt = _logits_array(G)
    sm, dt2 = _logits_array(S_noctx)
    if dt != dt2 or g.shape != sm.shape or g.ndim != 3:
        raise ValueError("logit tensors must share dtype and [B, k_max+1, V] shape")
    B, k1, V = g.shape
    r = _int32(row).reshape(B)
    p = _Params(B, k1 - 1, V, dt, 0, 0, 0.5, float(beta), 1.0, 1, 0)
    idx = np.empty((B, topk), np.int32)
    val = np.empty((B, topk), np.float32)
    rc = _load().specsteer_oracle_cloud_topk(_cptr(g), _cptr(sm), _cptr(r), ctypes.cast(ctypes.byref(p), ctypes.c_void_p),
                                             int(topk), _cptr(idx), _cptr(val))
    if rc != 0:
        raise ValueError("oracle rejected its arguments")
    return idx, val


def edge_resample(index, value, S_ctx, row, uniform, *, beta=1.0, temperature=1.0, greedy=False):
    """Edge side: add beta*h_SLM^+ on the top-k entries and resample among them."""
    sp, dt = _logits_array(S_ctx)
    B, k1, V = sp.shape
    idx = np.ascontiguousarray(index, np.int32)
    val = np.ascontiguousarray(value, np.float32)
    topk = idx.shape[1]
    r = _int32(row).reshape(B)
    if hasattr(uniform, "detach"):
        uniform = uniform.detach().cpu().numpy()
    u = np.ascontiguousarray(uniform, np.float32).reshape(B)
    p = _Params(B, k1 - 1, V, dt, 0, 0, 0.5, float(beta), float(temperature), 1, 1 if greedy else 0)
    tok = np.empty(B, np.int32)
    lp = np.empty(B, np.float64)
    cand = np.empty((B, topk), np.float64)
    margin = np.empty(B, np.float64)
    rc = _load().specsteer_oracle_edge_resample(_cptr(idx), _cptr(val), _cptr(sp), _cptr(r), _cptr(u),
                                                ctypes.cast(ctypes.byref(p), ctypes.c_void_p), int(topk), _cptr(tok),
                                                _cptr(lp), _cptr(cand), _cptr(margin))
    if rc != 0:
        raise ValueError("oracle rejected its arguments")
    return {"next_token": tok, "next_token_logprob": lp, "cand_logprobs": cand, "sample_margin": margin}
