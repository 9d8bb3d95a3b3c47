"""dart_reduce_with_norms: the criterion norms come from the caller (an epilogue of the
projection that made the criterion rows), good to a stated relative error; the step skips its
norm pass and must still pick the pivots of the exact norms, hence the oracle's sets."""
import numpy as np
import pytest
import torch

import oracle
import paper_2502_11494_amd as D
from paper_2502_11494_amd import workloads as W

import gpu_util as G

pytestmark = pytest.mark.gpu


def run_with_norms(w, l1, rel_err, crit=None, mode=D.DART_PIVOT_MAX_L1):
    Xd = G.to_device(w)
    cu_dev = torch.from_numpy(w.cu).cuda() if w.ragged else None
    desc = G.desc_of(w, cu_dev, mode=mode)
    ws = D.alloc_workspace(desc)
    total_keep = sum(w.budget(b) for b in range(w.B))
    total_N = int(w.cu[-1])
    pos = torch.from_numpy(w.pos).cuda()
    Y = torch.full((total_keep, w.D), 7, dtype=Xd.dtype, device="cuda")
    pos_out = torch.full((total_keep,), -1, dtype=torch.int64, device="cuda")
    keep = torch.full((total_keep,), -1, dtype=torch.int32, device="cuda")
    cu_keep = torch.full((w.B + 1,), -1, dtype=torch.int32, device="cuda")
    piv = torch.full((w.B * w.P,), -1, dtype=torch.int32, device="cuda")
    S = torch.full((w.P * total_N,), float("nan"), dtype=torch.float32, device="cuda")
    kw = {}
    if crit is not None:
        kw = dict(crit=crit, crit_D=crit.shape[1], crit_ld=crit.stride(0))
    D.dart_reduce_with_norms(desc, Xd, Y, keep, ws, torch.from_numpy(l1).cuda(), rel_err, pos=pos,
                             pos_out=pos_out, cu_keep=cu_keep, piv_out=piv, S_out=S, **kw)
    torch.cuda.synchronize()
    if w.ragged:
        assert D.dart_device_status(desc, ws) == D.DART_OK
    return G.GpuResult(piv.cpu().numpy().reshape(w.B, w.P), keep.cpu().numpy(), cu_keep.cpu().numpy(),
                       S.cpu().numpy(), G.bits(Y), pos_out.cpu().numpy())


def noisy_norms(exact, err, seed):
    """fp32 norms within a relative error of err of the exact ones (the rounding to fp32 comes
    on top: the library allows for it)."""
    u = np.random.default_rng(seed).uniform(-1.0, 1.0, size=exact.shape)
    return (exact * (1.0 + err * u)).astype(np.float32), err


CASES = [
    lambda: W.multicrop_batch(B=3, N=700, D=1024, P=16, K=120, n_centroids=64),   # exact copies
    lambda: W.image_batch(B=2, N=333, D=520, P=5, K=64, n_centroids=32),
    lambda: W.single_image(N=300, D=256, P=8, K=50, n_centroids=16),              # fp32
    lambda: W.ragged_batch(B=4, n_lo=300, n_hi=1200, D=512, P=16),
    lambda: W.video_batch(B=2, frames=8, per_frame=60, D=1024, P=32, K=96, n_centroids=8),
]


@pytest.mark.parametrize("err", [0.0, 1e-5, 2e-3])
@pytest.mark.parametrize("mode", [D.DART_PIVOT_MAX_L1, D.DART_PIVOT_MIN_L1])
def test_callers_norms_give_the_pivots_of_the_exact_norms(err, mode):
    omode = oracle.MAX_L1 if mode == D.DART_PIVOT_MAX_L1 else oracle.MIN_L1
    compared = 0
    for ci, make in enumerate(CASES):
        w = make()
        print(f"[case] norms given err={err} mode={mode} {w.name} B={w.B} P={w.P}", flush=True)
        refs = G.oracle_samples(w, mode=omode)
        if not all(oracle.admissible(w.sample(b), r) for b, r in enumerate(refs)):
            continue
        l1, bound = noisy_norms(oracle.l1_norms(w.X, w.dtype), err, 100 + ci)
        G.compare(w, run_with_norms(w, l1, bound, mode=mode), refs)
        compared += 1
    assert compared >= len(CASES) - 1


def test_callers_norms_of_separate_key_rows():
    """The K-norm use: key rows as the criterion, their norms from the caller."""
    w = W.multicrop_batch(B=3, N=700, D=1024, P=16, K=120, n_centroids=64)
    crit_bits = W.key_states(w, 128, seed=5)
    refs = G.oracle_samples(w, crit=crit_bits)
    assert all(oracle.admissible(w.sample(b), r) for b, r in enumerate(refs))
    crit_dev = torch.from_numpy(crit_bits.view(np.int16)).view(torch.bfloat16).cuda()
    l1, bound = noisy_norms(oracle.l1_norms(crit_bits, w.dtype), 1e-4, 9)
    G.compare(w, run_with_norms(w, l1, bound, crit=crit_dev), refs)


def test_callers_norms_at_full_size_and_refusals():
    w = W.by_index(2)
    refs = G.oracle_samples(w)
    l1, bound = noisy_norms(oracle.l1_norms(w.X, w.dtype), 1e-5, 3)
    g = run_with_norms(w, l1, bound)
    G.compare(w, g, refs)
    # the plain call picks the same pivots, tokens and rows
    plain = G.run_reduce(w)
    for f in ("piv", "keep", "Y", "pos_out"):
        np.testing.assert_array_equal(getattr(g, f), getattr(plain, f), err_msg=f)
    # refused on the host: no norms, a bound that is no bound, pivot modes that rank nothing
    small = W.image_batch(B=2, N=100, D=64, P=4, K=16, n_centroids=8)
    Xd = G.to_device(small)
    keep = torch.empty(32, dtype=torch.int32, device="cuda")
    l1d = torch.ones(200, dtype=torch.float32, device="cuda")
    desc = G.desc_of(small, None)
    ws = D.alloc_workspace(desc)
    for bad_err in (-1e-3, 0.11, float("nan")):
        with pytest.raises(D.DartError) as e:
            D.dart_reduce_with_norms(desc, Xd, None, keep, ws, l1d, bad_err)
        assert e.value.status == D.DART_ERR_SHAPE
    with pytest.raises(D.DartError) as e:
        D.dart_reduce_with_norms(desc, Xd, None, keep, ws, None, 1e-6)
    assert e.value.status == D.DART_ERR_NULL
    for mode in (D.DART_PIVOT_GIVEN, D.DART_PIVOT_RANDOM):
        with pytest.raises(D.DartError) as e:
            D.dart_reduce_with_norms(G.desc_of(small, None, mode=mode), Xd, None, keep, ws, l1d, 1e-6)
        assert e.value.status == D.DART_ERR_DTYPE
