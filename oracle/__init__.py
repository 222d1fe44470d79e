"""ctypes loader for the CPU float64 oracle (oracle/specgbv_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by ``__graft_entry__.smoke()`` and
by the ``cpu_baseline`` leg of ``bench.py``.  The product package never imports
this module, and this module never imports the product package.

Every wrapper only marshals numpy arrays to the C functions; the arithmetic
(paper Section 4.2: Algorithm 1, Eq. (hik), Eq. (hLk), Eq. (pres)) lives in the
C file.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from ctypes import POINTER, c_double, c_float, c_int, c_int32, c_uint32, c_uint64, c_void_p

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "specgbv_oracle.c")
_LIB = os.path.join(_HERE, "libspecgbv_oracle.so")

F32, BF16, F64 = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP only for the prefix loop)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Debug(ctypes.Structure):
    _fields_ = [
        ("lse_q", POINTER(c_double)), ("lse_p", POINTER(c_double)),
        ("log_nu", POINTER(c_double)), ("log_P", POINTER(c_double)),
        ("s", POINTER(c_double)), ("h", POINTER(c_double)), ("eta", POINTER(c_double)),
        ("state", POINTER(c_int32)), ("res_norm", POINTER(c_double)),
        ("u_final", POINTER(c_double)), ("margin", POINTER(c_double)),
        ("fallback", POINTER(c_int32)),
        ("carry_log_nu", POINTER(c_double)), ("modify_count", POINTER(c_int32)),
    ]


class _KseqDebug(ctypes.Structure):
    _fields_ = [("rho", POINTER(c_double)), ("beta", POINTER(c_double)), ("retained", POINTER(c_int32)),
                ("lead", POINTER(c_int32)), ("accept", POINTER(c_double)), ("eta", POINTER(c_double)),
                ("state", POINTER(c_int32)), ("res_norm", POINTER(c_double)), ("u_final", POINTER(c_double)),
                ("margin", POINTER(c_double)), ("rho_all", POINTER(c_double)), ("beta_all", POINTER(c_double))]


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        L.specgbv_oracle_philox4x32_10.argtypes = [POINTER(c_uint32)] * 3
        L.specgbv_oracle_philox4x32_10.restype = None
        L.specgbv_oracle_uniform.argtypes = [c_uint64, c_uint64, c_uint32, c_uint32]
        L.specgbv_oracle_uniform.restype = c_double
        L.specgbv_oracle_log_softmax.argtypes = [POINTER(c_double), c_int, c_double, POINTER(c_double)]
        L.specgbv_oracle_log_softmax.restype = c_double
        L.specgbv_oracle_ot_sum.argtypes = [POINTER(c_double), POINTER(c_double), c_int, c_double, c_int]
        L.specgbv_oracle_ot_sum.restype = c_double
        L.specgbv_oracle_h_sub.argtypes = [c_double, c_double, c_double, c_int]
        L.specgbv_oracle_h_sub.restype = c_double
        L.specgbv_oracle_ot_excess.argtypes = [POINTER(c_double), POINTER(c_double), c_int, c_double, c_int]
        L.specgbv_oracle_ot_excess.restype = c_double
        L.specgbv_oracle_h_sub_excess.argtypes = [c_double, c_double, c_double, c_int]
        L.specgbv_oracle_h_sub_excess.restype = c_double
        L.specgbv_oracle_h_full.argtypes = [c_double, c_double, c_int]
        L.specgbv_oracle_h_full.restype = c_double
        L.specgbv_oracle_decision_scan.argtypes = [POINTER(c_double), POINTER(c_double), POINTER(c_int32),
                                                   c_int, c_int, POINTER(c_int32), POINTER(c_int32),
                                                   POINTER(c_int32)]
        L.specgbv_oracle_decision_scan.restype = None
        L.specgbv_oracle_sample_cdf.argtypes = [POINTER(c_double), c_int, c_double, POINTER(c_double),
                                                POINTER(c_double)]
        L.specgbv_oracle_sample_cdf.restype = c_int32
        L.specgbv_oracle_verify.argtypes = [c_void_p, c_void_p, POINTER(c_int32), c_int, c_int, c_int, c_int,
                                            c_int, c_float, c_uint64, c_uint64, POINTER(c_int32),
                                            POINTER(c_int32), POINTER(c_int32), POINTER(_Debug), POINTER(c_int32), c_int]
        L.specgbv_oracle_verify.restype = c_int
        L.specgbv_oracle_modify.argtypes = [c_void_p, c_void_p, POINTER(c_int32), c_int, c_int, c_int, c_int, c_int,
                                            c_float, POINTER(c_double), POINTER(c_int32), POINTER(c_double),
                                            POINTER(c_double), POINTER(c_int32)]
        L.specgbv_oracle_modify.restype = c_int
        L.specgbv_oracle_sample_rows.argtypes = [c_void_p, c_int, c_int, c_int, c_float, c_uint64, c_uint64, c_uint32,
                                                 POINTER(c_int32), POINTER(c_double), POINTER(c_double)]
        L.specgbv_oracle_sample_rows.restype = c_int
        L.specgbv_oracle_carry_advance.argtypes = [c_void_p, c_void_p, POINTER(c_int32), POINTER(c_int32), POINTER(c_int32),
                                                   POINTER(c_int32), c_int, c_int, c_int, c_int, c_int, c_int, c_float,
                                                   POINTER(c_double), POINTER(c_int32)]
        L.specgbv_oracle_carry_advance.restype = c_int
        L.specgbv_oracle_kseq_beta.argtypes = [POINTER(c_double), POINTER(c_double), c_int, c_double]
        L.specgbv_oracle_kseq_beta.restype = c_double
        L.specgbv_oracle_kseq_rho.argtypes = [POINTER(c_double), POINTER(c_double), c_int, c_int]
        L.specgbv_oracle_kseq_rho.restype = c_double
        L.specgbv_oracle_verify_kseq.argtypes = [c_void_p, c_void_p, POINTER(c_int32), c_int, c_int, c_int, c_int, c_int,
                                                 c_float, c_uint64, c_uint64, c_int, POINTER(c_int32), POINTER(c_int32),
                                                 POINTER(c_int32), POINTER(_KseqDebug), POINTER(c_int32), c_int]
        L.specgbv_oracle_verify_kseq.restype = c_int
        L.specgbv_oracle_verify_token_sd.argtypes = [c_void_p, c_void_p, POINTER(c_int32), c_int, c_int, c_int, c_int,
                                                     c_int, c_float, c_uint64, c_uint64, POINTER(c_int32), POINTER(c_int32)]
        L.specgbv_oracle_verify_token_sd.restype = c_int
        L.specgbv_oracle_num_procs.argtypes = []
        L.specgbv_oracle_num_procs.restype = c_int
        _lib = L
    return _lib


def _dp(a: np.ndarray):
    return a.ctypes.data_as(POINTER(c_double))


def _ip(a: np.ndarray):
    return a.ctypes.data_as(POINTER(c_int32))


def philox4x32_10(counter, key) -> tuple:
    c = (c_uint32 * 4)(*[int(v) & 0xFFFFFFFF for v in counter])
    k = (c_uint32 * 2)(*[int(v) & 0xFFFFFFFF for v in key])
    out = (c_uint32 * 4)()
    lib().specgbv_oracle_philox4x32_10(c, k, out)
    return tuple(int(v) for v in out)


def uniform(seed: int, offset: int, prefix: int, slot: int) -> float:
    return float(lib().specgbv_oracle_uniform(seed, offset, prefix, slot))


def log_softmax(z, T: float = 1.0):
    z = np.ascontiguousarray(z, dtype=np.float64)
    out = np.empty_like(z)
    lse = lib().specgbv_oracle_log_softmax(_dp(z), z.size, float(T), _dp(out))
    return out, float(lse)


def ot_sum(lq, lp, log_nu: float, K: int) -> float:
    lq = np.ascontiguousarray(lq, dtype=np.float64)
    lp = np.ascontiguousarray(lp, dtype=np.float64)
    assert lq.shape == lp.shape
    return float(lib().specgbv_oracle_ot_sum(_dp(lq), _dp(lp), lq.size, float(log_nu), int(K)))


def ot_excess(lq, lp, log_nu: float, K: int) -> float:
    """nu^2 (s - g) of Eq. (hik) for nu > 1 as a sum of non-negative terms (no cancellation)."""
    lq = np.ascontiguousarray(lq, dtype=np.float64)
    lp = np.ascontiguousarray(lp, dtype=np.float64)
    assert lq.shape == lp.shape and lq.ndim == 1
    return float(lib().specgbv_oracle_ot_excess(_dp(lq), _dp(lp), lq.size, float(log_nu), int(K)))


def h_sub_excess(log_nu: float, log_P: float, E: float, K: int) -> float:
    """Eq. (hik) for nu > 1 from E = ot_excess(...)."""
    return float(lib().specgbv_oracle_h_sub_excess(float(log_nu), float(log_P), float(E), int(K)))


def h_sub(log_nu: float, log_P: float, s: float, K: int) -> float:
    return float(lib().specgbv_oracle_h_sub(float(log_nu), float(log_P), float(s), int(K)))


def h_full(log_nu: float, log_P: float, K: int) -> float:
    return float(lib().specgbv_oracle_h_full(float(log_nu), float(log_P), int(K)))


def decision_scan(h, eta, tokens):
    """Algorithm 1's loop for one prefix.  h, eta: [K, L]; tokens: [K, L]."""
    h = np.ascontiguousarray(h, dtype=np.float64)
    eta = np.ascontiguousarray(eta, dtype=np.float64)
    tokens = np.ascontiguousarray(tokens, dtype=np.int32)
    K, L = tokens.shape
    assert h.shape == (K, L) and eta.shape == (K, L)
    tau, f = c_int32(), c_int32()
    state = np.zeros((K, L), dtype=np.int32)
    lib().specgbv_oracle_decision_scan(_dp(h), _dp(eta), _ip(tokens), K, L, ctypes.byref(tau),
                                       ctypes.byref(f), _ip(state))
    return int(tau.value), int(f.value), state


def sample_cdf(w, u: float):
    w = np.ascontiguousarray(w, dtype=np.float64)
    W, margin = c_double(), c_double()
    y = lib().specgbv_oracle_sample_cdf(_dp(w), w.size, float(u), ctypes.byref(W), ctypes.byref(margin))
    return int(y), float(W.value), float(margin.value)


def to_raw(logits: np.ndarray):
    """(contiguous array, dtype code) for float32 arrays, uint16 bfloat16 bit patterns, or float64
    arrays (one oracle result fed to another oracle function without rounding)."""
    if logits.dtype == np.float32:
        return np.ascontiguousarray(logits), F32
    if logits.dtype == np.float64:
        return np.ascontiguousarray(logits), F64
    if logits.dtype == np.uint16:
        return np.ascontiguousarray(logits), BF16
    raise TypeError("logits must be float32, float64 or uint16 (bfloat16 bits), got %s" % logits.dtype)


def verify(target_logits: np.ndarray, draft_logits: np.ndarray, draft_tokens: np.ndarray,
           temperature: float, rng_seed: int, rng_offset: int, debug: bool = False, nthreads: int = 1,
           prefix_ids=None):
    """Run the oracle on host arrays.

    target_logits [B, K, L+1, V], draft_logits [B, K, L, V] (float32, or uint16 holding
    bfloat16 bits), draft_tokens [B, K, L] int32.  Returns a dict with accepted_len [B],
    accepted_draft_idx [B], out_tokens [B, L+1] and, with debug=True, the intermediates.
    prefix_ids [B] (optional) are the Philox prefix counters of the batch entries.
    """
    tl, dt = to_raw(target_logits)
    dl, dt2 = to_raw(draft_logits)
    assert dt == dt2
    B, K, L1, V = tl.shape
    L = L1 - 1
    assert dl.shape == (B, K, L, V), (dl.shape, (B, K, L, V))
    tok = np.ascontiguousarray(draft_tokens, dtype=np.int32)
    assert tok.shape == (B, K, L)
    res = {
        "accepted_len": np.full(B, -9, np.int32),
        "accepted_draft_idx": np.full(B, -9, np.int32),
        "out_tokens": np.full((B, L + 1), -9, np.int32),
    }
    pids = None
    if prefix_ids is not None:
        pids = np.ascontiguousarray(prefix_ids, dtype=np.int32)
        assert pids.shape == (B,)
    dbg = None
    if debug:
        nan = np.nan
        res.update(
            lse_q=np.full((B, K, L + 1), nan), lse_p=np.full((B, K, L), nan),
            log_nu=np.full((B, K, L), nan), log_P=np.full((B, K, L), nan),
            s=np.full((B, K, L), nan), h=np.full((B, K, L), nan), eta=np.full((B, K, L), nan),
            state=np.zeros((B, K, L), np.int32), res_norm=np.full(B, nan), u_final=np.full(B, nan),
            margin=np.full(B, nan), fallback=np.zeros(B, np.int32),
            carry_log_nu=np.full(B, nan), modify_count=np.zeros(B, np.int32))
        dbg = _Debug(_dp(res["lse_q"]), _dp(res["lse_p"]), _dp(res["log_nu"]), _dp(res["log_P"]),
                     _dp(res["s"]), _dp(res["h"]), _dp(res["eta"]), _ip(res["state"]),
                     _dp(res["res_norm"]), _dp(res["u_final"]), _dp(res["margin"]), _ip(res["fallback"]),
                     _dp(res["carry_log_nu"]), _ip(res["modify_count"]))
    rc = lib().specgbv_oracle_verify(
        tl.ctypes.data_as(c_void_p), dl.ctypes.data_as(c_void_p), _ip(tok), K, L, V, B, dt,
        c_float(temperature), rng_seed, rng_offset, _ip(res["accepted_len"]),
        _ip(res["accepted_draft_idx"]), _ip(res["out_tokens"]),
        ctypes.byref(dbg) if dbg is not None else None,
        _ip(pids) if pids is not None else None, int(nthreads))
    if rc != 0:
        raise ValueError("specgbv_oracle_verify rejected its arguments (code %d)" % rc)
    return res


def kseq_beta(lq, lp, rho: float) -> float:
    """beta(rho) = sum_x min{p[x], q[x]/rho} (Section 3.2) from log-probability rows."""
    lq = np.ascontiguousarray(lq, dtype=np.float64)
    lp = np.ascontiguousarray(lp, dtype=np.float64)
    assert lq.shape == lp.shape and lq.ndim == 1
    return float(lib().specgbv_oracle_kseq_beta(_dp(lq), _dp(lp), lq.size, float(rho)))


def kseq_rho(lq, lp, k: int) -> float:
    """The root of 1 - (1 - beta(rho))^k = rho beta(rho) in [1, k] (Section 3.2)."""
    lq = np.ascontiguousarray(lq, dtype=np.float64)
    lp = np.ascontiguousarray(lp, dtype=np.float64)
    assert lq.shape == lp.shape and lq.ndim == 1
    return float(lib().specgbv_oracle_kseq_rho(_dp(lq), _dp(lp), lq.size, int(k)))


def verify_kseq(target_logits: np.ndarray, draft_logits: np.ndarray, draft_tokens: np.ndarray, temperature: float,
                rng_seed: int, rng_offset: int, ndrafts=None, debug: bool = False, eager: bool = False,
                nthreads: int = 1, prefix_ids=None):
    """SpecTr K-SEQ verification (Section 3.2) with the first `ndrafts` drafts (default all K; 1 = token-level
    speculative decoding) on the inputs of verify().  eager=True also fills rho_all / beta_all [B, K, L]."""
    tl, dt = to_raw(target_logits)
    dl, dt2 = to_raw(draft_logits)
    assert dt == dt2
    B, K, L1, V = tl.shape
    L = L1 - 1
    assert dl.shape == (B, K, L, V)
    tok = np.ascontiguousarray(draft_tokens, dtype=np.int32)
    assert tok.shape == (B, K, L)
    nd = K if ndrafts is None else int(ndrafts)
    res = {"accepted_len": np.full(B, -9, np.int32), "accepted_draft_idx": np.full(B, -9, np.int32),
           "out_tokens": np.full((B, L + 1), -9, np.int32)}
    pids = None
    if prefix_ids is not None:
        pids = np.ascontiguousarray(prefix_ids, dtype=np.int32)
        assert pids.shape == (B,)
    dbg = None
    if debug or eager:
        nan = np.nan
        res.update(rho=np.full((B, L), nan), beta=np.full((B, L), nan), retained=np.zeros((B, L), np.int32),
                   lead=np.full((B, L), -1, np.int32), accept=np.full((B, K, L), nan), eta=np.full((B, K, L), nan),
                   state=np.zeros((B, K, L), np.int32), res_norm=np.full(B, nan), u_final=np.full(B, nan),
                   margin=np.full(B, nan))
        if eager:
            res.update(rho_all=np.full((B, K, L), nan), beta_all=np.full((B, K, L), nan))
        null_d = ctypes.cast(None, POINTER(c_double))
        dbg = _KseqDebug(_dp(res["rho"]), _dp(res["beta"]), _ip(res["retained"]), _ip(res["lead"]), _dp(res["accept"]),
                         _dp(res["eta"]), _ip(res["state"]), _dp(res["res_norm"]), _dp(res["u_final"]),
                         _dp(res["margin"]), _dp(res["rho_all"]) if eager else null_d,
                         _dp(res["beta_all"]) if eager else null_d)
    rc = lib().specgbv_oracle_verify_kseq(tl.ctypes.data_as(c_void_p), dl.ctypes.data_as(c_void_p), _ip(tok), K, L, V, B,
                                          dt, c_float(temperature), rng_seed, rng_offset, nd, _ip(res["accepted_len"]),
                                          _ip(res["accepted_draft_idx"]), _ip(res["out_tokens"]),
                                          ctypes.byref(dbg) if dbg is not None else None,
                                          _ip(pids) if pids is not None else None, int(nthreads))
    if rc != 0:
        raise ValueError("specgbv_oracle_verify_kseq rejected its arguments (code %d)" % rc)
    return res


def verify_token_sd(target_logits: np.ndarray, draft_logits: np.ndarray, draft_tokens: np.ndarray, temperature: float,
                    rng_seed: int, rng_offset: int):
    """Token-level speculative decoding (Section 3.1) on draft 0 of the inputs of verify()."""
    tl, dt = to_raw(target_logits)
    dl, dt2 = to_raw(draft_logits)
    assert dt == dt2
    B, K, L1, V = tl.shape
    L = L1 - 1
    tok = np.ascontiguousarray(draft_tokens, dtype=np.int32)
    res = {"accepted_len": np.full(B, -9, np.int32), "out_tokens": np.full((B, L + 1), -9, np.int32)}
    rc = lib().specgbv_oracle_verify_token_sd(tl.ctypes.data_as(c_void_p), dl.ctypes.data_as(c_void_p), _ip(tok), K, L, V,
                                              B, dt, c_float(temperature), rng_seed, rng_offset,
                                              _ip(res["accepted_len"]), _ip(res["out_tokens"]))
    if rc != 0:
        raise ValueError("specgbv_oracle_verify_token_sd rejected its arguments (code %d)" % rc)
    return res


def modify(target_logits: np.ndarray, draft_logits: np.ndarray, tokens: np.ndarray, temperature: float,
           carry_log_nu, count):
    """Algorithm 2 on host arrays: the distribution to use for the first rows of the next iteration.

    target_logits, draft_logits [B, K, M, V]; tokens [B, K, M]; carry_log_nu [B] and count [B] come
    from the previous iteration (verify(..., debug=True)).  Returns a dict with logq [B, K, M, V]
    (natural log of q_new for rows < count, of q otherwise), norm [B, K, M], fallback [B, K, M].
    """
    tl, dt = to_raw(target_logits)
    dl, dt2 = to_raw(draft_logits)
    assert dt == dt2 and tl.shape == dl.shape
    B, K, M, V = tl.shape
    tok = np.ascontiguousarray(tokens, dtype=np.int32)
    assert tok.shape == (B, K, M)
    carry = np.ascontiguousarray(carry_log_nu, dtype=np.float64)
    cnt = np.ascontiguousarray(count, dtype=np.int32)
    assert carry.shape == (B,) and cnt.shape == (B,)
    res = {"logq": np.full((B, K, M, V), np.nan), "norm": np.full((B, K, M), np.nan),
           "fallback": np.zeros((B, K, M), np.int32)}
    rc = lib().specgbv_oracle_modify(tl.ctypes.data_as(c_void_p), dl.ctypes.data_as(c_void_p), _ip(tok), K, M, V, B,
                                     dt, c_float(temperature), _dp(carry), _ip(cnt), _dp(res["logq"]),
                                     _dp(res["norm"]), _ip(res["fallback"]))
    if rc != 0:
        raise ValueError("specgbv_oracle_modify rejected its arguments (code %d)" % rc)
    return res


def sample_rows(logits: np.ndarray, temperature: float, rng_seed: int, rng_offset: int, position: int):
    """The drafting step of Algorithm 3 on host arrays: one token per row of logits [rows, V]
    (float32, or uint16 holding bfloat16 bits).  Returns tokens, the uniforms and the margins."""
    lg, dt = to_raw(logits)
    assert lg.ndim == 2
    rows, V = lg.shape
    res = {"tokens": np.full(rows, -9, np.int32), "u": np.full(rows, np.nan), "margin": np.full(rows, np.nan)}
    rc = lib().specgbv_oracle_sample_rows(lg.ctypes.data_as(c_void_p), rows, V, dt, c_float(temperature), rng_seed,
                                          rng_offset, position, _ip(res["tokens"]), _dp(res["u"]), _dp(res["margin"]))
    if rc != 0:
        raise ValueError("specgbv_oracle_sample_rows rejected its arguments (code %d)" % rc)
    return res


def carry_advance(rows_q: np.ndarray, rows_p: np.ndarray, tokens, accepted_len, accepted_idx, out_tokens,
                  temperature: float, carry_log_nu, count):
    """Advance one pending modification along the emitted tokens (see the C function).
    Returns new (carry_log_nu, count) arrays; the inputs are not changed."""
    rq, dt = to_raw(rows_q)
    rp, dt2 = to_raw(rows_p)
    assert dt == dt2
    B, K, M, V = rp.shape
    bonus = rq.shape[2] - M
    assert rq.shape == (B, K, M + bonus, V) and bonus in (0, 1)
    tok = np.ascontiguousarray(tokens, dtype=np.int32)
    al = np.ascontiguousarray(accepted_len, dtype=np.int32)
    ai = np.ascontiguousarray(accepted_idx, dtype=np.int32)
    ot = np.ascontiguousarray(out_tokens, dtype=np.int32)
    assert tok.shape == (B, K, M) and al.shape == (B,) and ai.shape == (B,) and ot.shape == (B, M + 1)
    carry = np.array(carry_log_nu, dtype=np.float64)
    cnt = np.array(count, dtype=np.int32)
    rc = lib().specgbv_oracle_carry_advance(rq.ctypes.data_as(c_void_p), rp.ctypes.data_as(c_void_p), _ip(tok), _ip(al),
                                            _ip(ai), _ip(ot), K, M, bonus, V, B, dt, c_float(temperature), _dp(carry),
                                            _ip(cnt))
    if rc != 0:
        raise ValueError("specgbv_oracle_carry_advance rejected its arguments (code %d)" % rc)
    return carry, cnt


def num_procs() -> int:
    return int(lib().specgbv_oracle_num_procs())
