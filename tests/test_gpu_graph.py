"""dart_reduce under HIP graph capture: the library only enqueues kernels (no allocation, no
synchronisation, no memset nodes), so a caller may capture a step once and replay it.  Every
replay is checked against the eager result on the same input, with eager work and
synchronisations between the replays."""
import numpy as np
import pytest
import torch

import paper_2502_11494_amd as D
from paper_2502_11494_amd import workloads as W

import gpu_util as G

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("make", [
    lambda seed: W.multicrop_batch(seed=seed, B=3, N=700, D=1024, P=16, K=120, n_centroids=64),
    lambda seed: W.ragged_batch(seed=seed, B=4, n_lo=200, n_hi=900, D=512, P=8),
])
def test_captured_step_replays_like_eager(make):
    ws_list = [make(seed) for seed in (11, 12, 13, 14)]
    w0 = ws_list[0]
    if w0.ragged:  # the captured step has fixed shapes: same lengths, different contents
        ws_list = [W.ragged_batch(seed=s, B=w0.B, D=w0.D, P=w0.P, lengths=w0.lengths.tolist())
                   for s in (11, 12, 13, 14)]
        w0 = ws_list[0]
    cu_dev = torch.from_numpy(w0.cu).cuda() if w0.ragged else None
    desc = G.desc_of(w0, cu_dev)
    ws = D.alloc_workspace(desc)
    total_keep = sum(w0.budget(b) for b in range(w0.B))
    Xs = G.to_device(w0).clone()                       # static input buffer of the graph
    pos = torch.from_numpy(w0.pos).cuda()
    Y = torch.zeros((total_keep, w0.D), dtype=Xs.dtype, device="cuda")
    keep = torch.zeros(total_keep, dtype=torch.int32, device="cuda")
    pos_out = torch.zeros(total_keep, dtype=torch.int64, device="cuda")

    def step():
        D.dart_reduce(desc, Xs, Y, keep, ws, pos=pos, pos_out=pos_out)

    step()  # warm-up outside the capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for rep, w in enumerate(ws_list):
        Xs.copy_(G.to_device(w))
        # eager reference on separate outputs (and eager work between the replays)
        ws2 = D.alloc_workspace(desc)
        Y2, keep2, pos2 = torch.zeros_like(Y), torch.zeros_like(keep), torch.zeros_like(pos_out)
        D.dart_reduce(desc, Xs, Y2, keep2, ws2, pos=pos, pos_out=pos2)
        torch.cuda.synchronize()
        Y.zero_(); keep.zero_(); pos_out.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(keep, keep2), f"replay {rep}"
        assert torch.equal(pos_out, pos2), f"replay {rep}"
        assert G.bits(Y).tobytes() == G.bits(Y2).tobytes(), f"replay {rep}"
        assert int(keep2.max()) > 0
        if w0.ragged:
            assert D.dart_device_status(desc, ws) == D.DART_OK


def test_captured_steps_with_drawn_pivots_and_with_callers_norms():
    """The two variants that skip the norm pass, captured once and replayed on new contents
    of the input buffer (the norms follow the contents: they sit in a buffer the caller
    refreshes before each replay)."""
    import oracle
    ws_list = [W.multicrop_batch(seed=s, B=3, N=700, D=1024, P=16, K=120, n_centroids=64)
               for s in (21, 22, 23)]
    w0 = ws_list[0]
    total_keep = w0.B * w0.K
    Xs = G.to_device(w0).clone()
    l1 = torch.zeros(w0.B * 700, dtype=torch.float32, device="cuda")
    outs = {}
    graphs = {}
    descs = {"drawn": G.desc_of(w0, None, mode=D.DART_PIVOT_RANDOM, seed=5),
             "norms": G.desc_of(w0, None)}
    wss = {k: D.alloc_workspace(d) for k, d in descs.items()}
    for kind in descs:
        outs[kind] = (torch.zeros((total_keep, w0.D), dtype=Xs.dtype, device="cuda"),
                      torch.zeros(total_keep, dtype=torch.int32, device="cuda"))

    def step(kind):
        Y, keep = outs[kind]
        if kind == "drawn":
            D.dart_reduce(descs[kind], Xs, Y, keep, wss[kind])
        else:
            D.dart_reduce_with_norms(descs[kind], Xs, Y, keep, wss[kind], l1, 1e-6)

    l1.copy_(torch.from_numpy(oracle.l1_norms(w0.X, w0.dtype).astype(np.float32)).cuda())
    for kind in descs:
        step(kind)  # warm-up outside the capture
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        graphs[kind] = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graphs[kind], stream=side):
                step(kind)
        torch.cuda.synchronize()
    for rep, w in enumerate(ws_list):
        Xs.copy_(G.to_device(w))
        l1.copy_(torch.from_numpy(oracle.l1_norms(w.X, w.dtype).astype(np.float32)).cuda())
        drawn = [oracle.reduce_given(w.sample(b), w.dtype, oracle.random_pivots(5, b, 700, w.P), w.K)
                 for b in range(w.B)]
        ranked = G.oracle_samples(w)
        for kind, refs in (("drawn", drawn), ("norms", ranked)):
            if not all(oracle.admissible(w.sample(b), r) for b, r in enumerate(refs)):
                continue
            Y, keep = outs[kind]
            Y.zero_(); keep.zero_()
            torch.cuda.synchronize()
            graphs[kind].replay()
            torch.cuda.synchronize()
            want = np.concatenate([r.keep for r in refs])
            np.testing.assert_array_equal(keep.cpu().numpy(), want, err_msg=f"{kind} replay {rep}")
            assert G.bits(Y).tobytes() == b"".join(r.Y.tobytes() for r in refs), (kind, rep)
