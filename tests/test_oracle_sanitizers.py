"""The oracle's C code under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU).

oracle/sanitizer_driver.c calls every whole-call entry point of specgbv_oracle.c (verification with its debug
outputs, Algorithm 2, the ratio's advance, K-SEQ with 1..K drafts, token-level speculative decoding, the drafting
step) on inputs from a small linear congruential generator; built with -fsanitize=address,undefined and
-fno-sanitize-recover, any out-of-bounds access, use after free, signed overflow or misaligned access aborts the run.
What it prints is compared with the ordinary build's results on the same inputs, so the sanitized run also has to
compute the same thing.
"""
import math
import os
import subprocess

import numpy as np
import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _lcg(n, state):
    out = np.empty(n)
    for i in range(n):
        state = (state * 6364136223846793005 + 1442695040888963407) & 0xFFFFFFFFFFFFFFFF
        out[i] = (state >> 11) / 9007199254740992.0
    return out, state


def test_oracle_runs_clean_under_sanitizers_and_computes_the_same(tmp_path):
    exe = str(tmp_path / "oracle_sanitized")
    cmd = ["gcc", "-std=c99", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-fopenmp", os.path.join(ROOT, "oracle", "specgbv_oracle.c"),
           os.path.join(ROOT, "oracle", "sanitizer_driver.c"), "-lm", "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0 and "asan" in (r.stderr or "").lower() and "cannot find" in r.stderr.lower():
        pytest.skip("the sanitizer runtime is not installed with this compiler")
    assert r.returncode == 0, r.stderr
    # (verify_asan_link_order=0: the environment may preload libraries of its own ahead of the sanitizer runtime)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1", OMP_NUM_THREADS="2")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0, "sanitized run failed:\n" + r.stderr[-3000:]
    assert "ERROR" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-3000:]
    lines = {ln.split(":", 1)[0]: ln.split(":", 1)[1].split() for ln in r.stdout.strip().splitlines()}

    B, K, L, V = 5, 3, 4, 37
    u, st = _lcg(B * K * (L + 1) * V, 12345)
    t = (6.0 * u - 3.0).astype(np.float32).reshape(B, K, L + 1, V)
    u, st = _lcg(B * K * L * V, st)
    d = (6.0 * u - 3.0).astype(np.float32).reshape(B, K, L, V)
    u, st = _lcg(B * K * L, st)
    tok = (u * V).astype(np.int32).reshape(B, K, L)
    t.reshape(-1)[7] = -np.inf
    T = float(np.float32(0.9))
    res = None
    for off in range(3):
        res = oracle.verify(t, d, tok, T, 77, off, debug=True)
        got = lines["verify %d" % off]
        want = [v for b in range(B) for v in (res["accepted_len"][b], res["accepted_draft_idx"][b])] + list(res["out_tokens"].reshape(-1))
        assert [int(v) for v in got[:-1]] == [int(v) for v in want]
        assert math.isclose(float(got[-1]), float(res["h"].sum()), rel_tol=1e-10)
    # the driver hands Algorithm 2 the target buffer as a dense [B, K, L, V] tensor: its first B K L V values
    t_dense = np.ascontiguousarray(t.reshape(-1)[:B * K * L * V].reshape(B, K, L, V))
    mod = oracle.modify(t_dense, d, tok, T, res["carry_log_nu"], res["modify_count"])
    assert math.isclose(float(lines["modify"][0]), float(mod["norm"].sum()), rel_tol=1e-10)
    carry, cnt = oracle.carry_advance(t, d, tok, res["accepted_len"], res["accepted_draft_idx"], res["out_tokens"], T,
                                      res["carry_log_nu"], res["modify_count"])
    adv = lines["advance"]
    for b in range(B):
        assert math.isclose(float(adv[2 * b]), float(carry[b]), rel_tol=1e-10, abs_tol=1e-12) and int(adv[2 * b + 1]) == int(cnt[b])
    for nd in range(1, K + 1):
        ks = oracle.verify_kseq(t, d, tok, T, 78, 1, ndrafts=nd, eager=True)
        got = lines["kseq %d" % nd]
        want = [v for b in range(B) for v in (ks["accepted_len"][b], ks["accepted_draft_idx"][b])] + list(ks["out_tokens"].reshape(-1))
        assert [int(v) for v in got[:-1]] == [int(v) for v in want]
        assert math.isclose(float(got[-1]), float(ks["rho_all"][:, :nd].sum()), rel_tol=1e-10)
    sd = oracle.verify_token_sd(t, d, tok, T, 78, 1)
    assert [int(v) for v in lines["sd"]] == [int(v) for v in list(sd["accepted_len"]) + list(sd["out_tokens"].reshape(-1))]
    # the driver passes the first B*K rows of the draft tensor as they lie in memory
    sm = oracle.sample_rows(d.reshape(-1, V)[:B * K].copy(), T, 5, 6, 2)
    assert [int(v) for v in lines["sample"]] == [int(v) for v in sm["tokens"]]
