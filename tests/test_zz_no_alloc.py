"""specgbv_verify_static (the entry point for callers that cannot allocate device memory) against
specgbv_verify through the C ABI (needs an MI355X: run with -m gpu).

Both run the same kernels, one on the library's built-in scratch buffer, the other on a caller-owned workspace,
so every output must be bit-identical: accepted lengths, draft indices and tokens.  Two calls in a row, the
second with a smaller input (the buffer keeps the first call's contents), then a larger one again, and a shape
beyond the buffer, which must be refused on the host.
"""
import numpy as np
import pytest

from parity_util import to_torch
from specgbv_synth import WORKLOADS, Workload, make_inputs, with_batch

pytestmark = pytest.mark.gpu


def _both(w, seed, offset):
    import torch
    import paper_2604_25925_amd as sg
    t, d, tok = make_inputs(w, seed=seed)
    tl, dl, tk = to_torch(t), to_torch(d), to_torch(tok)
    B, L = w.batch, w.L
    dev = tl.device
    out = (torch.full((B,), -7, dtype=torch.int32, device=dev), torch.full((B,), -7, dtype=torch.int32, device=dev),
           torch.full((B, L + 1), -7, dtype=torch.int32, device=dev))
    sg.specgbv_verify_static(tl, dl, tk, w.temperature, 5, offset, out=out)
    ref = sg.specgbv_verify(tl, dl, tk, w.temperature, 5, offset)
    torch.cuda.synchronize()
    for name, a, b in zip(("accepted_len", "accepted_draft_idx", "out_tokens"), out, ref[:3]):
        assert np.array_equal(a.cpu().numpy(), b.cpu().numpy()), "%s differs (%s, offset %d)" % (name, w.name, offset)
    tau = out[0].cpu().numpy()
    assert np.all((tau >= 0) & (tau <= L))
    return tau


def test_static_scratch_matches_workspace_on_consecutive_calls():
    big = Workload("static_big", 40, 8, 4, 32768, "bf16", 3.0, 1.0, head=20, temperature=1.0)       # chain schedule
    small = Workload("static_small", 3, 2, 3, 1000, "f32", 2.0, 0.5, temperature=0.8)               # two-pass schedule
    mid = with_batch(WORKLOADS["cfg2"], 5)
    seen = []
    for w, off in ((big, 0), (small, 1), (mid, 2), (big, 3), (small, 4)):
        seen.append(_both(w, 11, off))
    assert any(np.any(t > 0) for t in seen) and any(np.any(t == 0) for t in seen)


def test_static_scratch_refuses_what_does_not_fit_and_bad_arguments():
    import torch
    import paper_2604_25925_amd as sg
    w = WORKLOADS["cfg5"]
    assert sg.specgbv_workspace_bytes(w.batch, w.K, w.L, w.V, 1) > sg.binding.STATIC_SCRATCH_BYTES
    lib = sg.load_library()
    import ctypes
    P = 1 << 20                                     # never dereferenced: refused in the host checks
    st = lib.specgbv_verify_static(P, P, P, w.K, w.L, w.V, w.batch, 1, ctypes.c_float(0.7), 0, 0, P, P, P, None)
    assert st == 2 and "SPECGBV_STATIC_SCRATCH_BYTES" in sg.specgbv_last_error()
    assert lib.specgbv_verify_static(P, P, P, 0, 4, 1000, 1, 0, ctypes.c_float(1.0), 0, 0, P, P, P, None) == 1
    assert lib.specgbv_verify_static(None, P, P, 2, 4, 1000, 1, 0, ctypes.c_float(1.0), 0, 0, P, P, P, None) == 1
    assert lib.specgbv_verify_static(P, P, P, 2, 4, 1000, 1, 0, ctypes.c_float(-1.0), 0, 0, P, P, P, None) == 1
    assert lib.specgbv_verify_static(P, P, P, 2, 4, 1000, 0, 0, ctypes.c_float(1.0), 0, 0, P, P, P, None) == 0
    torch.cuda.synchronize()
