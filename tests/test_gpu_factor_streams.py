"""The factor's helper stream: nodes of the largest tile class run one GEMM beside the rest on a stream the
library keeps per device, forked from and joined back into the caller's stream with events.  A factor wide
enough to take that path (6016 columns) is held to the oracle, then called from two host threads at once on
two streams (the library serialises the enqueueing, the events are reused call after call), and captured
into a graph and replayed with changed input."""
import threading

import numpy as np
import pytest
import torch

import paper_2601_19675_amd as ptq
from paper_2601_19675_amd import binding
from oracle import ptq_oracle as orc

pytestmark = pytest.mark.gpu

N = 6016        # 47 leaves; the top node's halves are 2944 and 3072 wide: 128 x 128 tiles, helper stream
DAMP = 0.01


def _hessian(seed):
    g = torch.Generator(device="cuda").manual_seed(seed)
    X = torch.randn((N + 64, N), device="cuda", generator=g, dtype=torch.float64)
    X *= torch.exp(0.5 * torch.randn(N, device="cuda", generator=g, dtype=torch.float64))
    return X.T @ X


def _buffers():
    U = torch.full((N, N), float("nan"), dtype=torch.float64, device="cuda")
    dead = torch.zeros(N, dtype=torch.uint8, device="cuda")
    info = torch.full((2,), -1, dtype=torch.int32, device="cuda")
    ws = torch.empty(ptq.ptq_workspace_bytes(binding.OP_CHOLESKY_INV, 0, N), dtype=torch.uint8, device="cuda")
    return U, dead, info, ws


def _factor(H):
    U, dead, info, ws = _buffers()
    ptq.ptq_damped_cholesky_inv(H, DAMP, U, dead, info, ws)
    torch.cuda.synchronize()
    assert info.cpu().tolist() == [0, 0]
    return U


def test_wide_factor_matches_oracle_and_concurrent_callers_agree():
    H1, H2 = _hessian(11), _hessian(12)
    U1, U2 = _factor(H1), _factor(H2)
    Hd, _ = orc.damp(np.triu(H1.cpu().numpy()) + np.triu(H1.cpu().numpy(), 1).T, DAMP)
    Uref = orc.inverse_cholesky_upper(Hd)
    assert np.max(np.abs(U1.cpu().numpy() - Uref)) <= 1e-9 * np.max(np.abs(Uref))
    del Hd, Uref
    results, errors = {}, []

    def worker(name, H, ref):
        try:
            st = torch.cuda.Stream()
            U, dead, info, ws = _buffers()
            with torch.cuda.stream(st):
                for _ in range(3):
                    U.fill_(float("nan"))
                    ptq.ptq_damped_cholesky_inv(H, DAMP, U, dead, info, ws)
                    st.synchronize()
                    if info.cpu().tolist() != [0, 0] or not torch.equal(U, ref):
                        errors.append(name)
            results[name] = True
        except Exception as e:   # noqa: BLE001 - reported below
            errors.append(f"{name}: {e!r}")

    ts = [threading.Thread(target=worker, args=("a", H1, U1)), threading.Thread(target=worker, args=("b", H2, U2))]
    for t in ts:
        t.start()
    for t in ts:
        t.join()
    torch.cuda.synchronize()
    assert not errors and results == {"a": True, "b": True}, errors


def test_wide_factor_replays_from_a_captured_graph():
    H = _hessian(13)
    U, dead, info, ws = _buffers()
    ptq.ptq_damped_cholesky_inv(H, DAMP, U, dead, info, ws)   # first call outside the capture: creates the helper stream
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=torch.cuda.Stream()):
        ptq.ptq_damped_cholesky_inv(H, DAMP, U, dead, info, ws)
    for k in range(3):
        # eager work between the replays: a new input in place, and its result by an ordinary call
        H.diagonal().add_(float(k + 1))
        ref = _factor(H)
        U.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert info.cpu().tolist() == [0, 0] and torch.equal(U, ref), f"replay {k}"
