"""The one-launch form of the step (a persistent kernel that runs norms, pivot selection,
scores, ordering, retained set and compaction as work items with per-sample dependencies;
opt-in through DART_FUSED=1) against the oracle, and against the default kernel-per-step path."""
import os

import numpy as np
import pytest

import paper_2502_11494_amd as D
from paper_2502_11494_amd import workloads as W

import gpu_util as G

pytestmark = pytest.mark.gpu


@pytest.fixture()
def fused():
    os.environ["DART_FUSED"] = "1"
    yield
    os.environ.pop("DART_FUSED", None)


CASES = [
    lambda: W.image_batch(B=3, N=200, D=1024, P=8, K=64, n_centroids=32),
    lambda: W.multicrop_batch(B=2, N=700, D=2048, P=16, K=80, n_centroids=64),   # exact copies
    lambda: W.multicrop_batch(B=1, N=1000, D=520, P=20, K=111, n_centroids=64),  # ragged D-chunk
    lambda: W.ragged_batch(B=5, n_lo=200, n_hi=900, D=1024, P=16),
    lambda: W.video_batch(B=2, frames=8, per_frame=60, D=1024, P=32, K=96, n_centroids=8),
    lambda: W.video_batch(B=1, frames=6, per_frame=50, D=512, P=40, K=100, n_centroids=8),
    lambda: W.image_batch(B=1, N=200, D=2048, P=64, K=80, n_centroids=16),
    lambda: W.image_batch(B=2, N=300, D=512, P=16, K=20, n_centroids=16),        # empty stages
    lambda: W.image_batch(B=1, N=64, D=8, P=64, K=64, n_centroids=4),            # one D-chunk
    lambda: W.image_batch(B=40, N=130, D=256, P=8, K=30, n_centroids=8),         # many samples
    lambda: W.ragged_batch(B=2, D=256, P=64, lengths=[16384, 4100], keep_num=1, keep_den=8),
    lambda: W.image_batch(B=3000, N=24, D=64, P=2, K=6, n_centroids=6),          # thousands of chains
]


@pytest.mark.parametrize("make", CASES)
def test_one_launch_path_matches_the_oracle(make, fused):
    w = make()
    print(f"[case] fused {w.name} B={w.B} D={w.D} P={w.P} K={w.K}", flush=True)
    g = G.run_reduce(w)
    G.compare(w, g, G.oracle_samples(w))


@pytest.mark.parametrize("index", [1, 2, 4])
def test_one_launch_path_on_benchmark_shapes(index, fused):
    w = W.by_index(index)
    print(f"[case] fused configs[{index}]", flush=True)
    g = G.run_reduce(w)
    G.compare(w, g, G.oracle_samples(w))
    again = G.run_reduce(w)
    for f in ("piv", "keep", "S", "Y", "pos_out"):
        np.testing.assert_array_equal(getattr(g, f), getattr(again, f), err_msg=f)
    # the default path picks the same pivots, retained tokens and rows
    os.environ.pop("DART_FUSED", None)
    staged = G.run_reduce(w)
    for f in ("piv", "keep", "cu_keep", "Y", "pos_out"):
        np.testing.assert_array_equal(getattr(g, f), getattr(staged, f), err_msg=f)
    assert np.abs(g.S.astype(np.float64) - staged.S).max() <= 2 * D.score_tolerance(w.dtype)


def test_one_launch_path_with_rejected_and_empty_samples(fused):
    import torch
    w = W.ragged_batch(B=5, D=512, P=16, lengths=[300, 1, 200, 10, 400])
    lens = [300, 0, 200, 10, 400]
    cu = np.zeros(6, dtype=np.int32)
    cu[1:] = np.cumsum(lens)
    X = np.concatenate([w.sample(0), w.sample(2), w.sample(3), w.sample(4)])
    Xd = torch.from_numpy(X.view(np.int16)).view(torch.bfloat16).cuda()
    cu_dev = torch.from_numpy(cu).cuda()
    desc = D.make_desc(5, 512, 16, D.DART_BF16, keep_num=111, keep_den=1000, cu_seqlens=cu_dev,
                       total_N=int(cu[-1]), max_N=400)
    ws = D.alloc_workspace(desc)
    budgets = [33, 0, 22, 0, 44]
    tot = sum(budgets)
    Y = torch.zeros((tot, 512), dtype=torch.bfloat16, device="cuda")
    keep = torch.full((tot,), -1, dtype=torch.int32, device="cuda")
    cu_keep = torch.full((6,), -1, dtype=torch.int32, device="cuda")
    D.dart_reduce(desc, Xd, Y, keep, ws, cu_keep=cu_keep)
    assert D.dart_device_status(desc, ws) == D.DART_ERR_DEVICE  # sample 3 is shorter than P
    np.testing.assert_array_equal(cu_keep.cpu().numpy(), np.concatenate([[0], np.cumsum(budgets)]))
    import oracle
    keep_h, k0 = keep.cpu().numpy(), 0
    for b, kb in enumerate(budgets):
        if kb:
            r = oracle.reduce(X[cu[b]:cu[b + 1]], oracle.BF16, 16, kb)
            np.testing.assert_array_equal(keep_h[k0:k0 + kb], r.keep)
            k0 += kb
