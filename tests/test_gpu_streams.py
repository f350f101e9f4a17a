"""GPU tests of the launch contract: everything is enqueued on the caller's stream, nothing is
allocated or synchronised inside the library, so a call can run on a side stream and can be
captured into a HIP graph and replayed."""
import numpy as np
import pytest
import torch

import paper_2605_02568_amd as P

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _problem(seed, S, T, k, H=64, D=128):
    g = torch.Generator(device="cpu").manual_seed(seed)
    q = torch.randn((1, S, H, D), generator=g).to(torch.bfloat16).to(DEV)
    K = torch.randn((1, T, D), generator=g).to(torch.bfloat16).to(DEV)
    w = (torch.randn((1, S, H), generator=g) / np.sqrt(H)).to(DEV)
    return q, K, w


def _outputs(S, k):
    return (torch.full((1, S, k), -7, dtype=torch.int32, device=DEV),
            torch.full((1, S, k), 123.0, dtype=torch.float32, device=DEV))


def _same(a, b):
    return torch.equal(a[0], b[0]) and torch.equal(a[1].view(torch.int32), b[1].view(torch.int32))


@pytest.mark.parametrize("schedule", ["tiled", "single_pass", "single_pass_wide", "static"])
@pytest.mark.parametrize("S,T,m,k", [(2048, 512, 4, 64), (1536, 1536, 1, 1024)])
def test_side_stream_and_graph_replay(S, T, m, k, schedule):
    print(f"streams S={S} T={T} m={m} k={k} {schedule}", flush=True)
    q, K, w = _problem(11, S, T, k)
    c_S, c_T = 512, 384
    if schedule == "tiled":
        ws = torch.empty(P.si_workspace_bytes(1, S, 64, 128, T, k, c_S, c_T), dtype=torch.uint8, device=DEV)
        call = lambda oi, os_, stream=None: P.si_indexer_topk_tiled(  # noqa: E731
            q, K, w, m, k, P.SI_MASK_CAUSAL_BLOCK, c_S, c_T, oi, os_, ws, stream=stream)
    elif schedule == "static":  # scratch inside the library; its address is looked up by the eager call below
        ws = torch.empty(256, dtype=torch.uint8, device=DEV)
        call = lambda oi, os_, stream=None: P.si_indexer_topk_static(  # noqa: E731
            q, K, w, m, k, P.SI_MASK_CAUSAL_BLOCK, oi, os_, stream=stream)
    else:  # the library's choice of workgroup shape (narrow at these key ranges), or the wide one
        shape = 8 if schedule == "single_pass_wide" else 0
        ws = torch.empty(P.si_fused_workspace_bytes(1, S, 64, 128, T, k, c_S), dtype=torch.uint8, device=DEV)
        call = lambda oi, os_, stream=None: P.si_indexer_topk_fused_shape(  # noqa: E731
            q, K, w, m, k, P.SI_MASK_CAUSAL_BLOCK, c_S, shape, oi, os_, ws, stream=stream)

    eager = _outputs(S, k)
    call(eager[0], eager[1])
    torch.cuda.synchronize()

    # a side stream (default priority): the result is there once that stream is synchronised
    side = torch.cuda.Stream()
    on_side = _outputs(S, k)
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        call(on_side[0], on_side[1], stream=side)
    side.synchronize()
    assert _same(eager, on_side)

    # graph capture of the whole call; every replay is checked, with eager work and
    # synchronisations of the program's own in between
    captured = _outputs(S, k)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call(captured[0], captured[1])
    for replay in range(3):
        captured[0].fill_(-9)
        captured[1].fill_(-1.0)
        ws.random_(0, 255)  # the workspace carries nothing from call to call
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert _same(eager, captured), f"replay {replay}"
        again = _outputs(S, k)
        call(again[0], again[1])
        torch.cuda.synchronize()
        assert _same(eager, again)


def test_consumer_under_graph_replay():
    """si_sparse_attention launches one kernel and allocates nothing: capture and replay."""
    S, T, m, k, H, D = 512, 128, 4, 32, 64, 128
    q, K, w = _problem(12, S, T, k)
    g = torch.Generator(device="cpu").manual_seed(13)
    qa = torch.randn((1, S, H, D), generator=g).to(torch.bfloat16).to(DEV)
    idx, score = _outputs(S, k)
    ws = torch.empty(P.si_fused_workspace_bytes(1, S, H, D, T, k), dtype=torch.uint8, device=DEV)
    P.si_indexer_topk(q, K, w, m, k, P.SI_MASK_CAUSAL_BLOCK, idx, score, ws)
    eager = torch.empty((1, S, H, D), dtype=torch.float32, device=DEV)
    P.si_sparse_attention(qa, K, idx, m, P.SI_MASK_CAUSAL_BLOCK, 8, 0.1, eager)
    torch.cuda.synchronize()
    captured = torch.empty_like(eager)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        P.si_sparse_attention(qa, K, idx, m, P.SI_MASK_CAUSAL_BLOCK, 8, 0.1, captured)
    for replay in range(3):
        captured.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(eager.view(torch.int32), captured.view(torch.int32)), f"replay {replay}"
