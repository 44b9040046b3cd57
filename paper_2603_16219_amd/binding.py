"""ctypes binding of the C-ABI library: argument marshalling only.

Every step of the block runs inside ``libspecsteer.so`` (hand-written HIP for
gfx950); PyTorch supplies device memory and the stream.  There is no CPU or
PyTorch fallback: if the library cannot be loaded or a call fails, this raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch  # imported before the library so both share one HIP runtime

from . import build as _build

SS_F32, SS_BF16 = 0, 1
SS_FLAG_GREEDY = 1
SS_FLAG_FULL_ROWS = 2
_STATUS_OK = 0


class SSParams(ctypes.Structure):
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
        ("flags", ctypes.c_uint32),
    ]


class SpecSteerError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"specsteer status {status}: {message}")
        self.status = status


_lib = None


def library() -> ctypes.CDLL:
    """Load libspecsteer.so from the package directory (building it only if absent)."""
    global _lib
    if _lib is None:
        path = _build.LIBRARY
        if not os.path.exists(path):
            _build.build()
        lib = ctypes.CDLL(path)
        lib.specsteer_workspace_bytes.restype = ctypes.c_size_t
        lib.specsteer_workspace_bytes.argtypes = [ctypes.POINTER(SSParams)]
        lib.specsteer_verify_block.restype = ctypes.c_int
        lib.specsteer_verify_block.argtypes = (
            [ctypes.c_void_p] * 6 + [ctypes.POINTER(SSParams)] + [ctypes.c_void_p] * 6
            + [ctypes.c_size_t, ctypes.c_void_p])
        lib.specsteer_verify_block_timed.restype = ctypes.c_int
        lib.specsteer_verify_block_timed.argtypes = lib.specsteer_verify_block.argtypes + [ctypes.c_void_p]
        lib.specsteer_verify_block_static.restype = ctypes.c_int
        lib.specsteer_verify_block_static.argtypes = (
            [ctypes.c_void_p] * 6 + [ctypes.POINTER(SSParams)] + [ctypes.c_void_p] * 6)
        lib.specsteer_cloud_topk.restype = ctypes.c_int
        lib.specsteer_cloud_topk.argtypes = ([ctypes.c_void_p] * 3 + [ctypes.POINTER(SSParams), ctypes.c_int32]
                                             + [ctypes.c_void_p] * 3)
        lib.specsteer_edge_resample.restype = ctypes.c_int
        lib.specsteer_edge_resample.argtypes = ([ctypes.c_void_p] * 5 + [ctypes.POINTER(SSParams), ctypes.c_int32]
                                                + [ctypes.c_void_p] * 3)
        lib.specsteer_first_window.restype = ctypes.c_int
        lib.specsteer_first_window.argtypes = [ctypes.POINTER(SSParams)]
        lib.specsteer_status_string.restype = ctypes.c_char_p
        lib.specsteer_status_string.argtypes = [ctypes.c_int]
        lib.specsteer_version.restype = ctypes.c_int
        _lib = lib
    return _lib


def status_string(status: int) -> str:
    return library().specsteer_status_string(int(status)).decode()


def version() -> int:
    return int(library().specsteer_version())


def make_params(batch: int, k_max: int, vocab: int, dtype: torch.dtype, *, lam: float, beta: float,
                temperature: float, stride_b: int = 0, stride_t: int = 0, flags: int = 0) -> SSParams:
    code = {torch.float32: SS_F32, torch.bfloat16: SS_BF16}.get(dtype)
    if code is None:
        raise TypeError(f"logits must be float32 or bfloat16, got {dtype}")
    return SSParams(batch, k_max, vocab, code, stride_b, stride_t, lam, beta, temperature, flags)


def first_window(params: SSParams) -> int:
    return int(library().specsteer_first_window(ctypes.byref(params)))


def workspace_bytes(params: SSParams) -> int:
    return int(library().specsteer_workspace_bytes(ctypes.byref(params)))


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


STAGES = ("row_pass1", "verdict", "row_pass2", "recover")


def verify_block_raw(G, S_ctx, S_noctx, draft, draft_len, uniforms, params: SSParams, accepted_len,
                     next_token, next_token_logprob, recovery_logprobs, draft_logprobs, workspace,
                     stream: Optional[int] = None, timed: bool = False):
    """Thin call: every tensor is passed by its device pointer, nothing is checked or copied here.
    With ``timed`` it calls specsteer_verify_block_timed (which waits for the stream) and returns
    the per-stage milliseconds as a dict."""
    if stream is None:
        stream = torch.cuda.current_stream(G.device).cuda_stream
    args = [
        _ptr(G), _ptr(S_ctx), _ptr(S_noctx), _ptr(draft), _ptr(draft_len), _ptr(uniforms),
        ctypes.byref(params), _ptr(accepted_len), _ptr(next_token), _ptr(next_token_logprob),
        _ptr(recovery_logprobs), _ptr(draft_logprobs), _ptr(workspace),
        0 if workspace is None else workspace.numel() * workspace.element_size(),
        ctypes.c_void_p(stream)]
    if timed:
        ms = (ctypes.c_float * len(STAGES))()
        rc = library().specsteer_verify_block_timed(*args, ctypes.cast(ms, ctypes.c_void_p))
    else:
        rc = library().specsteer_verify_block(*args)
    if rc != _STATUS_OK:
        raise SpecSteerError(rc, status_string(rc))
    return dict(zip(STAGES, (float(x) for x in ms))) if timed else None


STATIC_SCRATCH_BYTES = 8 << 20


def verify_block_static_raw(G, S_ctx, S_noctx, draft, draft_len, uniforms, params: SSParams, accepted_len,
                            next_token, next_token_logprob, recovery_logprobs, draft_logprobs,
                            stream: Optional[int] = None) -> None:
    """Thin call of specsteer_verify_block_static: the block on the library's own scratch array, no
    workspace argument and no allocation anywhere in the call."""
    if stream is None:
        stream = torch.cuda.current_stream(G.device).cuda_stream
    rc = library().specsteer_verify_block_static(
        _ptr(G), _ptr(S_ctx), _ptr(S_noctx), _ptr(draft), _ptr(draft_len), _ptr(uniforms), ctypes.byref(params),
        _ptr(accepted_len), _ptr(next_token), _ptr(next_token_logprob), _ptr(recovery_logprobs),
        _ptr(draft_logprobs), ctypes.c_void_p(stream))
    if rc != _STATUS_OK:
        raise SpecSteerError(rc, status_string(rc))


def verify_block(G: torch.Tensor, S_ctx: torch.Tensor, S_noctx: torch.Tensor, draft: torch.Tensor,
                 uniforms: torch.Tensor, *, lam: float = 0.5, beta: float = 1.0, temperature: float = 1.0,
                 draft_len: Optional[torch.Tensor] = None, want_recovery_logprobs: bool = False,
                 want_draft_logprobs: bool = False, workspace: Optional[torch.Tensor] = None,
                 greedy: bool = False, full_rows: bool = False) -> dict:
    """specsteer_verify_block on device tensors G/S_ctx/S_noctx [B, k_max+1, V] (vocab stride 1),
    draft [B, k_max] int32, uniforms [B, k_max+1] float32.  Allocates the outputs (and a workspace
    unless one is given) with torch and returns them in a dict; runs on torch's current stream."""
    if not (G.shape == S_ctx.shape == S_noctx.shape) or G.dim() != 3:
        raise ValueError("logit tensors must share a [B, k_max+1, V] shape")
    if not (G.dtype == S_ctx.dtype == S_noctx.dtype):
        raise ValueError("logit tensors must share a dtype")
    if not (G.stride() == S_ctx.stride() == S_noctx.stride()) or G.stride(2) != 1:
        raise ValueError("logit tensors must share strides, with the vocabulary contiguous")
    B, k1, V = G.shape
    k_max = k1 - 1
    dev = G.device
    # the kernels index these three by the batch and block shape alone: a short one would be read out of bounds
    if tuple(draft.shape) != (B, k_max):
        raise ValueError(f"draft must be [B, k_max] = [{B}, {k_max}], got {tuple(draft.shape)}")
    if tuple(uniforms.shape) != (B, k_max + 1):
        raise ValueError(f"uniforms must be [B, k_max+1] = [{B}, {k_max + 1}], got {tuple(uniforms.shape)}")
    if draft_len is not None and tuple(draft_len.shape) != (B,):
        raise ValueError(f"draft_len must be [B] = [{B}], got {tuple(draft_len.shape)}")
    if not (G.is_cuda and S_ctx.is_cuda and S_noctx.is_cuda):
        raise ValueError("specsteer_verify_block needs device tensors; there is no CPU path")
    if workspace is not None and (not workspace.is_cuda or not workspace.is_contiguous()):
        raise ValueError("workspace must be a contiguous device tensor")
    draft = draft.to(device=dev, dtype=torch.int32).contiguous()
    uniforms = uniforms.to(device=dev, dtype=torch.float32).contiguous()
    if draft_len is not None:
        draft_len = draft_len.to(device=dev, dtype=torch.int32).contiguous()
    params = make_params(B, k_max, V, G.dtype, lam=lam, beta=beta, temperature=temperature,
                         stride_b=G.stride(0) if B > 1 else 0, stride_t=G.stride(1) if k1 > 1 else 0,
                         flags=(SS_FLAG_GREEDY if greedy else 0) | (SS_FLAG_FULL_ROWS if full_rows else 0))
    need = workspace_bytes(params)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    out = {
        "accepted_len": torch.empty(B, dtype=torch.int32, device=dev),
        "next_token": torch.empty(B, dtype=torch.int32, device=dev),
        "next_token_logprob": torch.empty(B, dtype=torch.float32, device=dev),
        "recovery_logprobs": torch.empty(B, V, dtype=torch.float32, device=dev) if want_recovery_logprobs else None,
        "draft_logprobs": torch.empty(B, k_max, 2, dtype=torch.float32, device=dev) if want_draft_logprobs else None,
    }
    verify_block_raw(G, S_ctx, S_noctx, draft if k_max > 0 else None, draft_len, uniforms, params,
                     out["accepted_len"], out["next_token"], out["next_token_logprob"],
                     out["recovery_logprobs"], out["draft_logprobs"], workspace)
    return out


def steer_rows(G: torch.Tensor, S_ctx: torch.Tensor, S_noctx: torch.Tensor, uniforms: torch.Tensor, *,
               beta: float = 1.0, temperature: float = 1.0, greedy: bool = False,
               want_logprobs: bool = False) -> dict:
    """Always-on steering: the recovery distribution of Eq. 8 applied to EVERY row ([N, V] logits,
    one uniform per row) -- the per-token fusion the paper compares against.  This is the same entry
    point with no drafted positions (k_max = 0): each row is a one-row sequence whose bonus token is
    drawn from softmax((G + beta (S_ctx - S_noctx)) / T)."""
    if G.dim() != 2 or uniforms.numel() != G.shape[0]:
        raise ValueError("rows must be [N, V] with one uniform per row")
    n, v = G.shape
    out = verify_block(G.view(n, 1, v), S_ctx.view(n, 1, v), S_noctx.view(n, 1, v),
                       torch.empty(n, 0, dtype=torch.int32, device=G.device), uniforms.reshape(n, 1),
                       beta=beta, temperature=temperature, want_recovery_logprobs=want_logprobs, greedy=greedy)
    return {"token": out["next_token"], "token_logprob": out["next_token_logprob"],
            "logprobs": out["recovery_logprobs"]}


def sample_rows(logits: torch.Tensor, uniforms: torch.Tensor, *, temperature: float = 1.0,
                greedy: bool = False) -> dict:
    """Plain softmax sampling of [N, V] rows by inverse CDF (Eq. 5, the drafting step, when the rows are
    the specialist's): the block with k_max = 0 and beta = 0, which reads each row once."""
    return steer_rows(logits, logits, logits, uniforms, beta=0.0, temperature=temperature, greedy=greedy)


def _split_params(T: torch.Tensor, beta: float, temperature: float, greedy: bool) -> SSParams:
    B, k1, V = T.shape
    return make_params(B, k1 - 1, V, T.dtype, lam=0.5, beta=beta, temperature=temperature,
                       stride_b=T.stride(0) if B > 1 else 0, stride_t=T.stride(1) if k1 > 1 else 0,
                       flags=SS_FLAG_GREEDY if greedy else 0)


def cloud_topk(G: torch.Tensor, S_noctx: torch.Tensor, row: torch.Tensor, *, beta: float = 1.0,
               topk: int = 32):
    """specsteer_cloud_topk on device tensors: returns (index [B, topk] int32, value [B, topk] float32)."""
    if G.dim() != 3 or G.shape != S_noctx.shape or G.stride() != S_noctx.stride() or G.stride(2) != 1:
        raise ValueError("G and S_noctx must share one [B, k_max+1, V] shape and stride, vocabulary contiguous")
    B = G.shape[0]
    if tuple(row.shape) != (B,):
        raise ValueError(f"row must be [B] = [{B}], got {tuple(row.shape)}")
    if not (G.is_cuda and S_noctx.is_cuda):
        raise ValueError("specsteer_cloud_topk needs device tensors; there is no CPU path")
    row = row.to(device=G.device, dtype=torch.int32).contiguous()
    idx = torch.empty(B, topk, dtype=torch.int32, device=G.device)
    val = torch.empty(B, topk, dtype=torch.float32, device=G.device)
    p = _split_params(G, beta, 1.0, False)
    rc = library().specsteer_cloud_topk(_ptr(G), _ptr(S_noctx), _ptr(row), ctypes.byref(p), topk, _ptr(idx), _ptr(val),
                                        ctypes.c_void_p(torch.cuda.current_stream(G.device).cuda_stream))
    if rc != _STATUS_OK:
        raise SpecSteerError(rc, status_string(rc))
    return idx, val


def edge_resample(index: torch.Tensor, value: torch.Tensor, S_ctx: torch.Tensor, row: torch.Tensor,
                  uniform: torch.Tensor, *, beta: float = 1.0, temperature: float = 1.0,
                  greedy: bool = False) -> dict:
    """specsteer_edge_resample on device tensors."""
    if S_ctx.dim() != 3 or S_ctx.stride(2) != 1:
        raise ValueError("S_ctx must be [B, k_max+1, V] with the vocabulary contiguous")
    B = S_ctx.shape[0]
    dev = S_ctx.device
    if index.dim() != 2 or index.shape[0] != B or index.shape != value.shape:
        raise ValueError("index and value must both be [B, topk] for S_ctx [B, k_max+1, V]")
    if index.dtype != torch.int32 or value.dtype != torch.float32:
        raise ValueError("index must be int32 and value float32")
    if tuple(row.shape) != (B,) or (not greedy and (uniform is None or tuple(uniform.shape) != (B,))):
        raise ValueError(f"row and uniform must be [B] = [{B}]")
    if not (S_ctx.is_cuda and index.is_cuda and value.is_cuda):
        raise ValueError("specsteer_edge_resample needs device tensors; there is no CPU path")
    row = row.to(device=dev, dtype=torch.int32).contiguous()
    uniform = None if uniform is None else uniform.to(device=dev, dtype=torch.float32).contiguous()
    tok = torch.empty(B, dtype=torch.int32, device=dev)
    lp = torch.empty(B, dtype=torch.float32, device=dev)
    p = _split_params(S_ctx, beta, temperature, greedy)
    rc = library().specsteer_edge_resample(_ptr(index.contiguous()), _ptr(value.contiguous()), _ptr(S_ctx), _ptr(row),
                                           _ptr(uniform), ctypes.byref(p), index.shape[1], _ptr(tok), _ptr(lp),
                                           ctypes.c_void_p(torch.cuda.current_stream(dev).cuda_stream))
    if rc != _STATUS_OK:
        raise SpecSteerError(rc, status_string(rc))
    return {"next_token": tok, "next_token_logprob": lp}
