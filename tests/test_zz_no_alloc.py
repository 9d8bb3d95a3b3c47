"""The entry point that allocates nothing (dart_reduce_static: scratch in a buffer built into
the library) against dart_reduce with a caller workspace: every output bit for bit, on two
calls in a row, the second on a smaller input."""
import numpy as np
import pytest
import torch

import paper_2502_11494_amd as D
from paper_2502_11494_amd import workloads as W

import gpu_util as G

pytestmark = pytest.mark.gpu


def run_both(w, mode=D.DART_PIVOT_MAX_L1, seed=0):
    Xd = G.to_device(w)
    cu_dev = torch.from_numpy(w.cu).cuda() if w.ragged else None
    desc = G.desc_of(w, cu_dev, mode=mode, seed=seed)
    assert D.dart_workspace_bytes(desc) <= D.dart_static_scratch_bytes()
    total_keep = sum(w.budget(b) for b in range(w.B))
    total_N = int(w.cu[-1])
    pos = torch.from_numpy(w.pos).cuda()

    def outputs():
        return dict(Y=torch.full((total_keep, w.D), 7, dtype=Xd.dtype, device="cuda"),
                    keep=torch.full((total_keep,), -1, dtype=torch.int32, device="cuda"),
                    pos_out=torch.full((total_keep,), -1, dtype=torch.int64, device="cuda"),
                    cu_keep=torch.full((w.B + 1,), -1, dtype=torch.int32, device="cuda"),
                    piv=torch.full((w.B * w.P,), -1, dtype=torch.int32, device="cuda"),
                    S=torch.full((w.P * total_N,), float("nan"), dtype=torch.float32,
                                 device="cuda"))

    ref, got = outputs(), outputs()
    ws = D.alloc_workspace(desc)
    D.dart_reduce(desc, Xd, ref["Y"], ref["keep"], ws, pos=pos, pos_out=ref["pos_out"],
                  cu_keep=ref["cu_keep"], piv_out=ref["piv"], S_out=ref["S"])
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    D.dart_reduce_static(desc, Xd, got["Y"], got["keep"], pos=pos, pos_out=got["pos_out"],
                         cu_keep=got["cu_keep"], piv_out=got["piv"], S_out=got["S"])
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    if w.ragged:
        assert D.dart_device_status_static(desc) == D.dart_device_status(desc, ws) == D.DART_OK
    for name in ref:
        assert torch.equal(ref[name].view(torch.uint8), got[name].view(torch.uint8)), name
    assert int(ref["keep"].min()) >= 0


def test_static_scratch_entry_matches_dart_reduce_twice_in_a_row():
    print("[case] static entry: video batch, then a smaller ragged batch", flush=True)
    run_both(W.video_batch(B=2, frames=16, per_frame=144, D=1024, P=32, K=256, n_centroids=16))
    run_both(W.ragged_batch(B=3, n_lo=200, n_hi=600, D=512, P=16))
    run_both(W.single_image(N=300, D=512, P=8, K=64, n_centroids=16))
    # pivots drawn at random on the device
    run_both(W.image_batch(B=4, N=333, D=520, P=5, K=64, n_centroids=32),
             mode=D.DART_PIVOT_RANDOM, seed=77)


def test_static_scratch_entry_refuses_oversized_problems():
    w = W.image_batch(B=1, N=64, D=64, P=4, K=8, n_centroids=4)
    Xd = G.to_device(w)
    desc = D.make_desc(60, 64, 64, D.DART_BF16, N=16384, K=64)  # 63 M scores: far over 32 MiB
    assert D.dart_workspace_bytes(desc) > D.dart_static_scratch_bytes()
    keep = torch.empty(8, dtype=torch.int32, device="cuda")
    with pytest.raises(D.DartError) as e:
        D.dart_reduce_static(desc, Xd, None, keep)
    assert e.value.status == D.DART_ERR_STATIC_LIMIT
