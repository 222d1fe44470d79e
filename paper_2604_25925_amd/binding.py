"""ctypes binding of libspecgbv.so: same names as the C ABI, argument marshalling only.

PyTorch appears here for device memory and the current HIP stream; every step of the
verification runs inside the library's kernels.  There is no fallback: if the library
cannot be loaded the import of a symbol raises.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, c_char_p, c_double, c_float, c_int, c_int32, c_size_t, c_uint64, c_void_p
from typing import Dict, Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libspecgbv.so")

F32, BF16 = 0, 1
ALGO_AUTO, ALGO_SPLIT, ALGO_CHAIN = 0, 1, 2
_ALGO = {"auto": ALGO_AUTO, "split": ALGO_SPLIT, "chain": ALGO_CHAIN}

EXPORTS = ("specgbv_workspace_bytes", "specgbv_verify", "specgbv_verify_static", "specgbv_verify_ex", "specgbv_verify_kseq", "specgbv_read_kseq_intermediates", "specgbv_read_intermediates",
           "specgbv_workspace_carry", "specgbv_modify_target", "specgbv_modify_workspace_bytes", "specgbv_sample_tokens", "specgbv_sample_workspace_bytes",
           "specgbv_read_sample_intermediates", "specgbv_carry_advance", "specgbv_carry_workspace_bytes", "specgbv_pending_state_bytes", "specgbv_last_error", "specgbv_version")


class SpecGBVError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("specgbv status %d: %s" % (status, message))
        self.status = status


class _Options(ctypes.Structure):
    _fields_ = [("algo", c_int32), ("pending_levels", c_int32), ("ev_main_start", c_void_p), ("ev_main_stop", c_void_p),
                ("pending_carry_log_nu", c_void_p), ("pending_count", c_void_p), ("pending_state", c_void_p),
                ("shared_row0", c_int32), ("reserved", c_int32)]


class _KseqIntermediates(ctypes.Structure):
    _fields_ = [("rho_all", POINTER(c_double)), ("beta_all", POINTER(c_double)), ("accept", POINTER(c_double)),
                ("eta", POINTER(c_double)), ("state", POINTER(c_int32)), ("retained", POINTER(c_int32)),
                ("lead", POINTER(c_int32)), ("res_norm", POINTER(c_double)), ("u_final", POINTER(c_double)),
                ("margin", POINTER(c_double))]


class _Intermediates(ctypes.Structure):
    _fields_ = [("lse_q", POINTER(c_double)), ("lse_p", POINTER(c_double)), ("log_nu", POINTER(c_double)),
                ("log_P", POINTER(c_double)), ("s", POINTER(c_double)), ("h", POINTER(c_double)),
                ("eta", POINTER(c_double)), ("state", POINTER(c_int32)), ("res_norm", POINTER(c_double)),
                ("u_final", POINTER(c_double)), ("margin", POINTER(c_double)), ("fallback", POINTER(c_int32)),
                ("carry_log_nu", POINTER(c_double)), ("modify_count", POINTER(c_int32))]


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libspecgbv.so (building it with hipcc only if no built library exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        from .build import build
        build()
    L = ctypes.CDLL(_LIB_PATH)
    L.specgbv_workspace_bytes.argtypes = [c_int, c_int, c_int, c_int, c_int]
    L.specgbv_workspace_bytes.restype = c_size_t
    verify_args = [c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_int, c_float, c_uint64, c_uint64,
                   c_void_p, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
    L.specgbv_verify.argtypes = verify_args
    L.specgbv_verify.restype = c_int
    L.specgbv_verify_static.argtypes = verify_args[:14] + [c_void_p]
    L.specgbv_verify_static.restype = c_int
    L.specgbv_verify_kseq.argtypes = verify_args[:11] + [c_int] + verify_args[11:]
    L.specgbv_verify_kseq.restype = c_int
    L.specgbv_read_kseq_intermediates.argtypes = [c_void_p, c_size_t, c_int, c_int, c_int, c_int,
                                                  POINTER(_KseqIntermediates), c_void_p]
    L.specgbv_read_kseq_intermediates.restype = c_int
    L.specgbv_verify_ex.argtypes = verify_args + [POINTER(_Options)]
    L.specgbv_verify_ex.restype = c_int
    L.specgbv_pending_state_bytes.argtypes = [c_int]
    L.specgbv_pending_state_bytes.restype = c_size_t
    L.specgbv_read_intermediates.argtypes = [c_void_p, c_size_t, c_int, c_int, c_int, c_int, c_int,
                                             POINTER(_Intermediates), c_void_p]
    L.specgbv_read_intermediates.restype = c_int
    L.specgbv_workspace_carry.argtypes = [c_void_p, c_size_t, c_int, c_int, c_int, c_int, POINTER(c_void_p),
                                          POINTER(c_void_p)]
    L.specgbv_workspace_carry.restype = c_int
    L.specgbv_modify_target.argtypes = [c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_int, c_int, c_float,
                                        c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_size_t,
                                        c_void_p]
    L.specgbv_modify_target.restype = c_int
    L.specgbv_modify_workspace_bytes.argtypes = [c_int, c_int, c_int, c_int]
    L.specgbv_modify_workspace_bytes.restype = c_size_t
    L.specgbv_sample_tokens.argtypes = [c_void_p, c_int, c_int, c_int, c_float, c_uint64, c_uint64, ctypes.c_uint32,
                                        c_void_p, c_void_p, c_size_t, c_void_p]
    L.specgbv_sample_tokens.restype = c_int
    L.specgbv_sample_workspace_bytes.argtypes = [c_int, c_int]
    L.specgbv_sample_workspace_bytes.restype = c_size_t
    L.specgbv_read_sample_intermediates.argtypes = [c_void_p, c_size_t, c_int, c_int, POINTER(c_double),
                                                    POINTER(c_double), c_void_p]
    L.specgbv_read_sample_intermediates.restype = c_int
    L.specgbv_carry_advance.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_int, c_int, c_int,
                                        c_int, c_int, c_int, c_float, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
    L.specgbv_carry_advance.restype = c_int
    L.specgbv_carry_workspace_bytes.argtypes = [c_int, c_int]
    L.specgbv_carry_workspace_bytes.restype = c_size_t
    L.specgbv_last_error.argtypes = []
    L.specgbv_last_error.restype = c_char_p
    L.specgbv_version.argtypes = []
    L.specgbv_version.restype = c_char_p
    _lib = L
    return L


def specgbv_last_error() -> str:
    return load_library().specgbv_last_error().decode()


def specgbv_version() -> str:
    return load_library().specgbv_version().decode()


def _check(status: int):
    if status != 0:
        raise SpecGBVError(status, specgbv_last_error())


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError("logits must be float32 or bfloat16, got %s" % t.dtype)


def specgbv_workspace_bytes(batch: int, K: int, L: int, V: int, dtype: int) -> int:
    return int(load_library().specgbv_workspace_bytes(batch, K, L, V, dtype))


def _shapes(target_logits, draft_logits, draft_tokens):
    import torch
    if target_logits.dim() != 4 or draft_logits.dim() != 4 or draft_tokens.dim() != 3:
        raise ValueError("expected target [B,K,L+1,V], draft [B,K,L,V], tokens [B,K,L]")
    B, K, L1, V = target_logits.shape
    L = L1 - 1
    if tuple(draft_logits.shape) != (B, K, L, V) or tuple(draft_tokens.shape) != (B, K, L):
        raise ValueError("inconsistent shapes: target %s draft %s tokens %s" %
                         (tuple(target_logits.shape), tuple(draft_logits.shape), tuple(draft_tokens.shape)))
    if target_logits.dtype != draft_logits.dtype:
        raise TypeError("target and draft logits must share a dtype")
    if draft_tokens.dtype != torch.int32:
        raise TypeError("draft_tokens must be int32")
    for t in (target_logits, draft_logits, draft_tokens):
        if not t.is_cuda:
            raise ValueError("all tensors must live on the GPU")
        if not t.is_contiguous():
            raise ValueError("all tensors must be contiguous")
    return B, K, L, V


def specgbv_verify_ex(target_logits, draft_logits, draft_tokens, temperature: float, rng_seed: int,
                      rng_offset: int, *, workspace=None, out: Optional[Tuple] = None, algo="auto",
                      events: Optional[Tuple[int, int]] = None, stream: Optional[int] = None, pending=None,
                      pending_state=None, shared_row0: bool = False):
    """Enqueue one verification on the current (or given) HIP stream.

    Returns (accepted_len [B], accepted_draft_idx [B], out_tokens [B, L+1], workspace), all
    device tensors; nothing is synchronised.  `events` is a pair of raw hipEvent_t handles
    recorded around the vocabulary-streaming kernels.  `pending` is a pair (carry_log_nu, count)
    of [B] (one level) or [levels, B] float64 / int32 device tensors, or raw device addresses of
    one level: pending distribution modifications (Algorithm 2) applied on the fly, innermost
    first.  `pending_state` (instead) is a zero-initialised uint8 device tensor of
    specgbv_pending_state_bytes(B) bytes that the call reads and updates in place: the whole
    bookkeeping of Algorithm 3's modifications.  `shared_row0` states that rows 0 of a prefix's K drafts
    are copies of one another (Algorithm 3: position 0 is conditioned on the prefix alone), which lets the
    chain schedule read them once per prefix.
    """
    import torch
    lib = load_library()
    B, K, L, V = _shapes(target_logits, draft_logits, draft_tokens)
    dt = _dtype_code(target_logits)
    dev = target_logits.device
    need = specgbv_workspace_bytes(B, K, L, V, dt)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    if out is None:
        out = (torch.empty(B, dtype=torch.int32, device=dev), torch.empty(B, dtype=torch.int32, device=dev),
               torch.empty((B, L + 1), dtype=torch.int32, device=dev))
    acc_len, acc_idx, out_tokens = out
    if stream is None:
        stream = torch.cuda.current_stream(dev).cuda_stream
    levels = 0
    if pending is not None:
        for t, dtp in ((pending[0], torch.float64), (pending[1], torch.int32)):
            if isinstance(t, int):
                continue
            if t.dtype != dtp or not t.is_cuda or not t.is_contiguous() or t.shape[-1] != B or t.dim() not in (1, 2):
                raise ValueError("pending must be ([B] or [levels, B] float64, int32) contiguous GPU tensors or raw device addresses")
            lv = 1 if t.dim() == 1 else int(t.shape[0])
            if levels not in (0, lv):
                raise ValueError("pending carry and count disagree on the number of levels")
            levels = lv
    if pending_state is not None:
        if not pending_state.is_cuda or not pending_state.is_contiguous() or \
                pending_state.numel() * pending_state.element_size() < specgbv_pending_state_bytes(B):
            raise ValueError("pending_state must be a contiguous GPU tensor of specgbv_pending_state_bytes(B) bytes")
    opt = _Options(_ALGO[algo] if isinstance(algo, str) else int(algo), levels,
                   events[0] if events else None, events[1] if events else None,
                   _dev_ptr(pending[0]) if pending is not None else None,
                   _dev_ptr(pending[1]) if pending is not None else None,
                   pending_state.data_ptr() if pending_state is not None else None,
                   1 if shared_row0 else 0, 0)
    st = lib.specgbv_verify_ex(target_logits.data_ptr(), draft_logits.data_ptr(), draft_tokens.data_ptr(), K, L, V,
                               B, dt, c_float(temperature), rng_seed, rng_offset, acc_len.data_ptr(),
                               acc_idx.data_ptr(), out_tokens.data_ptr(), workspace.data_ptr(),
                               workspace.numel() * workspace.element_size(), stream, ctypes.byref(opt))
    _check(st)
    return acc_len, acc_idx, out_tokens, workspace


MAX_PENDING = 16          # SPECGBV_MAX_PENDING of the C header


def specgbv_pending_state_bytes(batch: int) -> int:
    return int(load_library().specgbv_pending_state_bytes(batch))


def pending_state_views(buf: np.ndarray, batch: int):
    """(carry_log_nu [MAX_PENDING, batch] float64, count [MAX_PENDING, batch] int32) views of a host copy of a
    pending_state buffer (uint8 numpy array): the layout specgbv_pending_state_bytes describes."""
    n = MAX_PENDING * batch
    return buf[:n * 8].view(np.float64).reshape(MAX_PENDING, batch), buf[n * 8:n * 12].view(np.int32).reshape(MAX_PENDING, batch)


def specgbv_verify(target_logits, draft_logits, draft_tokens, temperature: float, rng_seed: int, rng_offset: int,
                   *, workspace=None, out: Optional[Tuple] = None, stream: Optional[int] = None):
    """specgbv_verify of the C ABI: default schedule, no instrumentation."""
    import torch
    lib = load_library()
    B, K, L, V = _shapes(target_logits, draft_logits, draft_tokens)
    dt = _dtype_code(target_logits)
    dev = target_logits.device
    if workspace is None:
        workspace = torch.empty(max(specgbv_workspace_bytes(B, K, L, V, dt), 256), dtype=torch.uint8, device=dev)
    if out is None:
        out = (torch.empty(B, dtype=torch.int32, device=dev), torch.empty(B, dtype=torch.int32, device=dev),
               torch.empty((B, L + 1), dtype=torch.int32, device=dev))
    if stream is None:
        stream = torch.cuda.current_stream(dev).cuda_stream
    st = lib.specgbv_verify(target_logits.data_ptr(), draft_logits.data_ptr(), draft_tokens.data_ptr(), K, L, V, B,
                            dt, c_float(temperature), rng_seed, rng_offset, out[0].data_ptr(), out[1].data_ptr(),
                            out[2].data_ptr(), workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                            stream)
    _check(st)
    return out[0], out[1], out[2], workspace


def specgbv_verify_kseq(target_logits, draft_logits, draft_tokens, temperature: float, rng_seed: int, rng_offset: int,
                        ndrafts: Optional[int] = None, *, workspace=None, out: Optional[Tuple] = None,
                        stream: Optional[int] = None):
    """specgbv_verify_kseq of the C ABI: the comparison verifier (SpecTr's K-SEQ rule; ndrafts = 1 is token-level
    speculative decoding) on the inputs of specgbv_verify.  Returns (accepted_len, accepted_draft_idx, out_tokens,
    workspace)."""
    import torch
    lib = load_library()
    B, K, L, V = _shapes(target_logits, draft_logits, draft_tokens)
    dt = _dtype_code(target_logits)
    dev = target_logits.device
    if workspace is None:
        workspace = torch.empty(max(specgbv_workspace_bytes(B, K, L, V, dt), 256), dtype=torch.uint8, device=dev)
    if out is None:
        out = (torch.empty(B, dtype=torch.int32, device=dev), torch.empty(B, dtype=torch.int32, device=dev),
               torch.empty((B, L + 1), dtype=torch.int32, device=dev))
    if stream is None:
        stream = torch.cuda.current_stream(dev).cuda_stream
    st = lib.specgbv_verify_kseq(target_logits.data_ptr(), draft_logits.data_ptr(), draft_tokens.data_ptr(), K, L, V, B, dt,
                                 c_float(temperature), rng_seed, rng_offset, K if ndrafts is None else int(ndrafts),
                                 out[0].data_ptr(), out[1].data_ptr(), out[2].data_ptr(), workspace.data_ptr(),
                                 workspace.numel() * workspace.element_size(), stream)
    _check(st)
    return out[0], out[1], out[2], workspace


def specgbv_read_kseq_intermediates(workspace, batch: int, K: int, L: int, V: int,
                                    stream: Optional[int] = None) -> Dict[str, np.ndarray]:
    """Copy the intermediates of the last specgbv_verify_kseq call out of `workspace` (synchronises the stream)."""
    import torch
    lib = load_library()
    if stream is None:
        stream = torch.cuda.current_stream(workspace.device).cuda_stream
    res = {"rho_all": np.full((batch, K, L), np.nan), "beta_all": np.full((batch, K, L), np.nan),
           "accept": np.full((batch, K, L), np.nan), "eta": np.full((batch, K, L), np.nan),
           "state": np.zeros((batch, K, L), np.int32), "retained": np.zeros((batch, L), np.int32),
           "lead": np.zeros((batch, L), np.int32), "res_norm": np.full(batch, np.nan), "u_final": np.full(batch, np.nan),
           "margin": np.full(batch, np.nan)}
    dp = lambda a: a.ctypes.data_as(POINTER(c_double))
    ip = lambda a: a.ctypes.data_as(POINTER(c_int32))
    out = _KseqIntermediates(dp(res["rho_all"]), dp(res["beta_all"]), dp(res["accept"]), dp(res["eta"]), ip(res["state"]),
                             ip(res["retained"]), ip(res["lead"]), dp(res["res_norm"]), dp(res["u_final"]), dp(res["margin"]))
    _check(lib.specgbv_read_kseq_intermediates(workspace.data_ptr(), workspace.numel() * workspace.element_size(), batch,
                                               K, L, V, ctypes.byref(out), stream))
    return res


STATIC_SCRATCH_BYTES = 8 << 20      # SPECGBV_STATIC_SCRATCH_BYTES of the C header


def specgbv_verify_static(target_logits, draft_logits, draft_tokens, temperature: float, rng_seed: int, rng_offset: int,
                          *, out: Tuple, stream: Optional[int] = None):
    """specgbv_verify_static of the C ABI: the verification on the library's built-in scratch buffer.  The
    caller passes the three output tensors; nothing is allocated here or in the library."""
    import torch
    lib = load_library()
    B, K, L, V = _shapes(target_logits, draft_logits, draft_tokens)
    dt = _dtype_code(target_logits)
    if stream is None:
        stream = torch.cuda.current_stream(target_logits.device).cuda_stream
    st = lib.specgbv_verify_static(target_logits.data_ptr(), draft_logits.data_ptr(), draft_tokens.data_ptr(), K, L, V, B,
                                   dt, c_float(temperature), rng_seed, rng_offset, out[0].data_ptr(), out[1].data_ptr(),
                                   out[2].data_ptr(), stream)
    _check(st)
    return out


def specgbv_read_intermediates(workspace, batch: int, K: int, L: int, V: int, dtype: int,
                               stream: Optional[int] = None) -> Dict[str, np.ndarray]:
    """Copy the intermediates of the last call out of `workspace` (synchronises the stream)."""
    import torch
    lib = load_library()
    if stream is None:
        stream = torch.cuda.current_stream(workspace.device).cuda_stream
    n = (batch, K, L)
    res = {k: np.empty(n, np.float64) for k in ("lse_q", "lse_p", "log_nu", "log_P", "s", "h", "eta")}
    res["state"] = np.empty(n, np.int32)
    for k in ("res_norm", "u_final", "margin"):
        res[k] = np.empty(batch, np.float64)
    res["fallback"] = np.empty(batch, np.int32)
    res["carry_log_nu"] = np.empty(batch, np.float64)
    res["modify_count"] = np.empty(batch, np.int32)
    dp = lambda a: a.ctypes.data_as(POINTER(c_double))
    ip = lambda a: a.ctypes.data_as(POINTER(c_int32))
    im = _Intermediates(dp(res["lse_q"]), dp(res["lse_p"]), dp(res["log_nu"]), dp(res["log_P"]), dp(res["s"]),
                        dp(res["h"]), dp(res["eta"]), ip(res["state"]), dp(res["res_norm"]), dp(res["u_final"]),
                        dp(res["margin"]), ip(res["fallback"]), dp(res["carry_log_nu"]), ip(res["modify_count"]))
    st = lib.specgbv_read_intermediates(workspace.data_ptr(), workspace.numel() * workspace.element_size(), batch,
                                        K, L, V, dtype, ctypes.byref(im), stream)
    _check(st)
    return res


def specgbv_workspace_carry(workspace, batch: int, K: int, L: int, V: int) -> Tuple[int, int]:
    """Raw device addresses (carry_log_nu [batch] float64, modify_count [batch] int32) inside
    `workspace`, as left by the last verification of this shape."""
    lib = load_library()
    a, b = c_void_p(), c_void_p()
    st = lib.specgbv_workspace_carry(workspace.data_ptr(), workspace.numel() * workspace.element_size(), batch, K, L,
                                     V, ctypes.byref(a), ctypes.byref(b))
    _check(st)
    return int(a.value), int(b.value)


def specgbv_modify_workspace_bytes(batch: int, K: int, M: int, bonus_row: int) -> int:
    return int(load_library().specgbv_modify_workspace_bytes(batch, K, M, bonus_row))


def _dev_ptr(x) -> Optional[int]:
    if x is None:
        return None
    return x if isinstance(x, int) else x.data_ptr()


def specgbv_modify_target(target_logits, draft_logits, draft_tokens, temperature: float, carry_log_nu, modify_count,
                          *, want_logp: bool = False, want_norm: bool = False, out=None, workspace=None,
                          stream: Optional[int] = None):
    """Enqueue Algorithm 2 for the drafts of the next iteration.

    draft_logits [B, K, M, V]; target_logits [B, K, M, V] or [B, K, M+1, V] (with the bonus row);
    draft_tokens [B, K, M]; carry_log_nu / modify_count are device tensors ([B] float64 / int32) or
    the raw addresses returned by specgbv_workspace_carry.  Returns a dict of device tensors: logq
    (float32, shape of target_logits) and, on request, logp [B, K, M, V], norm, fallback [B, K, M],
    plus the workspace used (pass the dict back as `out` to reuse every buffer).
    """
    import torch
    lib = load_library()
    if target_logits.dim() != 4 or draft_logits.dim() != 4:
        raise ValueError("expected draft logits [B, K, M, V] and target logits [B, K, M or M+1, V]")
    B, K, M, V = draft_logits.shape
    bonus = target_logits.shape[2] - M
    if bonus not in (0, 1) or tuple(target_logits.shape) != (B, K, M + bonus, V):
        raise ValueError("expected draft logits [B, K, M, V] and target logits [B, K, M or M+1, V]")
    if tuple(draft_tokens.shape) != (B, K, M) or draft_tokens.dtype != torch.int32:
        raise ValueError("draft_tokens must be int32 [B, K, M]")
    if target_logits.dtype != draft_logits.dtype:
        raise TypeError("target and draft logits must share a dtype")
    for t in (target_logits, draft_logits, draft_tokens):
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError("all tensors must be contiguous GPU tensors")
    for t, dt in ((carry_log_nu, torch.float64), (modify_count, torch.int32)):
        if not isinstance(t, int) and (t.dtype != dt or tuple(t.shape) != (B,) or not t.is_cuda):
            raise ValueError("carry_log_nu / modify_count must be [B] float64 / int32 GPU tensors")
    dev = target_logits.device
    res = dict(out) if out else {}
    if "logq" not in res:
        res["logq"] = torch.empty((B, K, M + bonus, V), dtype=torch.float32, device=dev)
    if want_logp and "logp" not in res:
        res["logp"] = torch.empty((B, K, M, V), dtype=torch.float32, device=dev)
    if want_norm:
        res.setdefault("norm", torch.empty((B, K, M), dtype=torch.float64, device=dev))
        res.setdefault("fallback", torch.empty((B, K, M), dtype=torch.int32, device=dev))
    if workspace is None:
        workspace = res.get("workspace")
    if workspace is None:
        workspace = torch.empty(max(specgbv_modify_workspace_bytes(B, K, M, bonus), 256), dtype=torch.uint8, device=dev)
    res["workspace"] = workspace
    if stream is None:
        stream = torch.cuda.current_stream(dev).cuda_stream
    st = lib.specgbv_modify_target(target_logits.data_ptr(), draft_logits.data_ptr(), draft_tokens.data_ptr(), K, M, bonus,
                                   V, B, _dtype_code(target_logits), c_float(temperature), _dev_ptr(carry_log_nu),
                                   _dev_ptr(modify_count), res["logq"].data_ptr(), _dev_ptr(res.get("logp")),
                                   _dev_ptr(res.get("norm")), _dev_ptr(res.get("fallback")), workspace.data_ptr(),
                                   workspace.numel() * workspace.element_size(), stream)
    _check(st)
    return res


def specgbv_sample_workspace_bytes(rows: int, V: int) -> int:
    return int(load_library().specgbv_sample_workspace_bytes(rows, V))


def specgbv_sample_tokens(logits, temperature: float, rng_seed: int, rng_offset: int, position: int, *, out=None,
                          workspace=None, stream: Optional[int] = None):
    """Enqueue the draw of one token per row of logits [rows, V] (or [..., V], flattened);
    returns (tokens [rows] int32, workspace)."""
    import torch
    lib = load_library()
    if not logits.is_cuda or not logits.is_contiguous() or logits.dim() < 2:
        raise ValueError("logits must be a contiguous GPU tensor [rows, V]")
    V = logits.shape[-1]
    rows = logits.numel() // V if V else 0
    dev = logits.device
    if out is None:
        out = torch.empty(rows, dtype=torch.int32, device=dev)
    if workspace is None:
        workspace = torch.empty(max(specgbv_sample_workspace_bytes(rows, V), 256), dtype=torch.uint8, device=dev)
    if stream is None:
        stream = torch.cuda.current_stream(dev).cuda_stream
    st = lib.specgbv_sample_tokens(logits.data_ptr(), rows, V, _dtype_code(logits), c_float(temperature), rng_seed,
                                   rng_offset, position, out.data_ptr(), workspace.data_ptr(),
                                   workspace.numel() * workspace.element_size(), stream)
    _check(st)
    return out, workspace


def specgbv_read_sample_intermediates(workspace, rows: int, V: int, stream: Optional[int] = None) -> Dict[str, np.ndarray]:
    import torch
    lib = load_library()
    if stream is None:
        stream = torch.cuda.current_stream(workspace.device).cuda_stream
    u, m = np.empty(rows, np.float64), np.empty(rows, np.float64)
    st = lib.specgbv_read_sample_intermediates(workspace.data_ptr(), workspace.numel() * workspace.element_size(), rows,
                                               V, u.ctypes.data_as(POINTER(c_double)), m.ctypes.data_as(POINTER(c_double)),
                                               stream)
    _check(st)
    return {"u": u, "margin": m}


def specgbv_carry_workspace_bytes(batch: int, M: int) -> int:
    return int(load_library().specgbv_carry_workspace_bytes(batch, M))


def specgbv_carry_advance(rows_q, rows_p, draft_tokens, accepted_len, accepted_draft_idx, out_tokens,
                          temperature: float, carry_log_nu, modify_count, *, workspace=None,
                          stream: Optional[int] = None):
    """Advance one pending modification (carry_log_nu [B] float64, modify_count [B] int32, both updated in
    place) along the tokens the last verification emitted; rows_q [B, K, M or M+1, V] are the rows that
    modification modifies, rows_p [B, K, M, V] the draft rows."""
    import torch
    lib = load_library()
    B, K, M, V = rows_p.shape
    bonus = rows_q.shape[2] - M
    if bonus not in (0, 1) or tuple(rows_q.shape) != (B, K, M + bonus, V) or rows_q.dtype != rows_p.dtype:
        raise ValueError("expected rows_p [B, K, M, V] and rows_q [B, K, M or M+1, V] of one dtype")
    if tuple(draft_tokens.shape) != (B, K, M) or tuple(out_tokens.shape) != (B, M + 1):
        raise ValueError("draft_tokens must be [B, K, M] and out_tokens [B, M+1]")
    for t, dt in ((draft_tokens, torch.int32), (accepted_len, torch.int32), (accepted_draft_idx, torch.int32),
                  (out_tokens, torch.int32), (carry_log_nu, torch.float64), (modify_count, torch.int32)):
        if t.dtype != dt or not t.is_cuda or not t.is_contiguous():
            raise ValueError("integer tensors must be int32, carry_log_nu float64, all contiguous on the GPU")
    if not (rows_q.is_cuda and rows_p.is_cuda and rows_q.is_contiguous() and rows_p.is_contiguous()):
        raise ValueError("rows must be contiguous GPU tensors")
    if workspace is None:
        workspace = torch.empty(max(specgbv_carry_workspace_bytes(B, M), 256), dtype=torch.uint8, device=rows_q.device)
    if stream is None:
        stream = torch.cuda.current_stream(rows_q.device).cuda_stream
    st = lib.specgbv_carry_advance(rows_q.data_ptr(), rows_p.data_ptr(), draft_tokens.data_ptr(), accepted_len.data_ptr(),
                                   accepted_draft_idx.data_ptr(), out_tokens.data_ptr(), K, M, bonus, V, B,
                                   _dtype_code(rows_q), c_float(temperature), carry_log_nu.data_ptr(),
                                   modify_count.data_ptr(), workspace.data_ptr(),
                                   workspace.numel() * workspace.element_size(), stream)
    _check(st)
    return workspace
