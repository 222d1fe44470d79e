"""The entry points under HIP graph capture: a serving loop records one decoding iteration's
library calls once and replays them.  Every call is asynchronous on the caller's stream,
allocates nothing and records no memset, so it can be captured; each replay (with eager work
and synchronisations in between, and new inputs copied into the captured buffers) must
reproduce the eager result bit for bit."""
import numpy as np
import pytest

from parity_util import to_torch
from specgbv_synth import Workload, make_inputs

pytestmark = pytest.mark.gpu


def test_verify_modify_sample_replay_under_graph_capture():
    import torch
    import paper_2604_25925_amd as sg
    w = Workload("graph", 6, 4, 4, 8192, "bf16", 2.5, 0.9, head=20, temperature=0.9)
    sets = [make_inputs(w, seed=s) for s in (41, 42, 43)]
    T, B, K, L, V = w.temperature, w.batch, w.K, w.L, w.V
    dev = torch.device("cuda")
    # static buffers of the captured iteration
    tl, dl, tk = (to_torch(a) for a in sets[0])
    ws = torch.empty(sg.specgbv_workspace_bytes(B, K, L, V, 1), dtype=torch.uint8, device=dev)
    out = (torch.empty(B, dtype=torch.int32, device=dev), torch.empty(B, dtype=torch.int32, device=dev),
           torch.empty((B, L + 1), dtype=torch.int32, device=dev))
    carry_ptr, count_ptr = sg.specgbv_workspace_carry(ws, B, K, L, V)
    ws2 = torch.empty_like(ws)
    out2 = tuple(torch.empty_like(t) for t in out)
    ws3 = torch.empty_like(ws)
    out3 = tuple(torch.empty_like(t) for t in out)
    rng = np.random.default_rng(5)
    state0 = np.zeros(sg.specgbv_pending_state_bytes(B), np.uint8)        # two levels pending for every prefix
    c0, n0 = sg.pending_state_views(state0, B)
    c0[:2] = rng.normal(2.0, 0.5, (2, B))
    n0[:2] = [[1] * B, [3] * B]
    state0 = torch.from_numpy(state0).to(dev)
    state = torch.empty_like(state0)
    mod = {"logq": torch.empty((B, K, L + 1, V), dtype=torch.float32, device=dev),
           "logp": torch.empty((B, K, L, V), dtype=torch.float32, device=dev),
           "workspace": torch.empty(sg.specgbv_modify_workspace_bytes(B, K, L, 1), dtype=torch.uint8, device=dev)}
    rows = dl[:, :, 0].contiguous().view(B * K, V)
    stok = torch.empty(B * K, dtype=torch.int32, device=dev)
    sws = torch.empty(sg.specgbv_sample_workspace_bytes(B * K, V), dtype=torch.uint8, device=dev)

    def iteration():
        sg.specgbv_verify_ex(tl, dl, tk, T, 5, 2, workspace=ws, out=out)
        sg.specgbv_modify_target(tl, dl, tk, T, carry_ptr, count_ptr, want_logp=True, out=mod)
        sg.specgbv_sample_tokens(rows, T, 5, 2, 0, out=stok, workspace=sws)
        # the same modification applied on the fly by a second verification (its own workspace and outputs)
        sg.specgbv_verify_ex(tl, dl, tk, T, 5, 3, workspace=ws2, out=out2, pending=(carry_ptr, count_ptr))
        # and a verification that reads and updates a pending state (reset first, so that every replay starts alike)
        state.copy_(state0)
        sg.specgbv_verify_ex(tl, dl, tk, T, 5, 4, workspace=ws3, out=out3, pending_state=state)

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in (*out, mod["logq"], mod["logp"], stok, *out2, *out3, state)]

    def load(inputs):
        a, b, c = (to_torch(x) for x in inputs)
        tl.copy_(a); dl.copy_(b); tk.copy_(c)
        rows.copy_(dl[:, :, 0].reshape(B * K, V))

    eager = []
    for inputs in sets:
        load(inputs)
        iteration()
        eager.append(snapshot())

    load(sets[0])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        iteration()                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        iteration()
    for rep, inputs in enumerate(sets + sets[:1]):
        load(inputs)
        for t in (*out, stok, *out2, *out3):
            t.fill_(-7)                               # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot()
        want = eager[rep % len(sets)]
        for g, e in zip(got, want):
            assert torch.equal(g, e) or (g.dtype.is_floating_point and
                                         torch.equal(torch.nan_to_num(g, neginf=-1e30), torch.nan_to_num(e, neginf=-1e30))), \
                "replay %d differs from the eager result" % rep


def test_chain_schedule_with_shared_rows_0_under_graph_capture():
    # two kernels in the streaming part (the reduction of the shared rows 0, then the chains): both are captured
    import torch
    import paper_2604_25925_amd as sg
    w = Workload("graph", 5, 4, 3, 32768, "bf16", 2.5, 0.9, head=20, temperature=1.1)
    sets = [make_inputs(w, seed=s) for s in (51, 52)]
    T, B, K, L, V = w.temperature, w.batch, w.K, w.L, w.V
    dev = torch.device("cuda")
    tl, dl, tk = (to_torch(a) for a in sets[0])
    ws = torch.empty(sg.specgbv_workspace_bytes(B, K, L, V, 1), dtype=torch.uint8, device=dev)
    out = (torch.empty(B, dtype=torch.int32, device=dev), torch.empty(B, dtype=torch.int32, device=dev),
           torch.empty((B, L + 1), dtype=torch.int32, device=dev))

    def iteration():
        sg.specgbv_verify_ex(tl, dl, tk, T, 9, 1, workspace=ws, out=out, algo="chain", shared_row0=True)

    def load(inputs):
        a, b, c = (to_torch(x) for x in inputs)
        tl.copy_(a); dl.copy_(b); tk.copy_(c)

    eager = []
    for inputs in sets:
        load(inputs)
        iteration()
        torch.cuda.synchronize()
        eager.append([t.clone() for t in out])
    load(sets[0])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        iteration()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        iteration()
    for rep, inputs in enumerate(sets + sets):
        load(inputs)
        for t in out:
            t.fill_(-7)
        ws.fill_(rep)                                 # the workspace carries nothing from one call to the next
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for g, e in zip(out, eager[rep % len(sets)]):
            assert torch.equal(g, e), "replay %d differs from the eager result" % rep
