"""Parity of the four stage entry points of the C ABI with the oracle's steps."""
import os

import numpy as np
import pytest
import torch

import oracle
import paper_2502_11494_amd as D
from paper_2502_11494_amd import workloads as W

import gpu_util as G

pytestmark = pytest.mark.gpu


def setup(w, ld=None):
    Xd = G.to_device(w, ld)
    cu_dev = torch.from_numpy(w.cu).cuda() if w.ragged else None
    desc = G.desc_of(w, cu_dev, ld)
    return Xd, cu_dev, desc, D.alloc_workspace(desc)


CASES = [
    lambda: W.single_image(N=300, D=512, P=8, K=64, n_centroids=16),
    lambda: W.multicrop_batch(B=3, N=450, D=1024, P=16, K=100, n_centroids=32),
    lambda: W.ragged_batch(B=4, n_lo=80, n_hi=700, D=768, P=12),
]


@pytest.mark.parametrize("make", CASES)
def test_select_pivots_and_norms(make):
    w = make()
    Xd, cu_dev, desc, ws = setup(w)
    piv = torch.full((w.B * w.P,), -1, dtype=torch.int32, device="cuda")
    l1 = torch.zeros(int(w.cu[-1]), dtype=torch.float32, device="cuda")
    D.dart_select_pivots(desc, Xd, piv, ws, l1_out=l1)
    torch.cuda.synchronize()
    piv_h, l1_h = piv.cpu().numpy().reshape(w.B, w.P), l1.cpu().numpy().astype(np.float64)
    for b in range(w.B):
        lo, hi = int(w.cu[b]), int(w.cu[b + 1])
        c = oracle.l1_norms(w.X[lo:hi], w.dtype)
        np.testing.assert_allclose(l1_h[lo:hi], c, rtol=2e-6, atol=0)
        np.testing.assert_array_equal(piv_h[b], oracle.select_pivots(c, w.P))


@pytest.mark.parametrize("make", CASES)
def test_duplication_scores(make):
    w = make()
    Xd, cu_dev, desc, ws = setup(w)
    rng = np.random.default_rng(1)
    # any pivots will do for this entry point: take random distinct tokens
    piv_h = np.stack([rng.permutation(int(n))[:w.P] for n in w.lengths]).astype(np.int32)
    piv = torch.from_numpy(piv_h).cuda()
    S = torch.full((w.P * int(w.cu[-1]),), float("nan"), dtype=torch.float32, device="cuda")
    D.dart_duplication_scores(desc, Xd, piv, S, ws)
    torch.cuda.synchronize()
    S_h = S.cpu().numpy().astype(np.float64)
    tau = D.score_tolerance(w.dtype)
    for b in range(w.B):
        lo, hi = int(w.cu[b]), int(w.cu[b + 1])
        ref = oracle.scores(w.X[lo:hi], w.dtype, piv_h[b])
        got = S_h[w.P * lo:w.P * hi].reshape(w.P, hi - lo)
        err = np.abs(got - ref)
        assert np.all(err <= G.RTOL[w.dtype] * np.abs(ref) + G.ATOL)
        assert err.max() <= tau
        for i, p in enumerate(piv_h[b]):
            assert abs(got[i, p] - 1.0) <= tau  # self-similarity


def test_topk_keep_on_given_scores_is_exact_integer_work():
    # X = NULL: the fp32 scores are the truth, so the oracle's retain step on the
    # same numbers must give the same indices, ties included
    rng = np.random.default_rng(2)
    for N, P, K, grid in [(500, 8, 64, None), (333, 5, 47, 0.25), (64, 16, 64, 0.5),
                          (2000, 32, 999, None), (100, 1, 100, 1.0)]:
        B = 3
        S_h = rng.standard_normal((B, P, N)).astype(np.float32) * 0.1
        if grid:
            S_h = (np.round(S_h / (grid * 0.1)) * (grid * 0.1)).astype(np.float32)  # many ties
        S_h[0, 0, :5] = -0.0
        S_h[0, 0, 5:9] = 0.0
        piv_h = np.stack([rng.permutation(N)[:P] for _ in range(B)]).astype(np.int32)
        desc = D.make_desc(B, 64, P, D.DART_BF16, N=N, K=K)
        ws = D.alloc_workspace(desc)
        keep = torch.full((B * K,), -1, dtype=torch.int32, device="cuda")
        cu_keep = torch.full((B + 1,), -1, dtype=torch.int32, device="cuda")
        D.dart_topk_keep(desc, torch.from_numpy(S_h).cuda(), torch.from_numpy(piv_h).cuda(), keep,
                         ws, cu_keep=cu_keep)
        torch.cuda.synchronize()
        keep_h = keep.cpu().numpy().reshape(B, K)
        np.testing.assert_array_equal(cu_keep.cpu().numpy(), np.arange(B + 1) * K)
        for b in range(B):
            np.testing.assert_array_equal(keep_h[b], oracle.retain(S_h[b], piv_h[b], K))


def test_topk_keep_ragged_with_certification():
    w = W.ragged_batch(B=4, n_lo=80, n_hi=700, D=768, P=12)
    Xd, cu_dev, desc, ws = setup(w)
    refs = G.oracle_samples(w)
    total = int(w.cu[-1])
    # feed the oracle's own scores, rounded to fp32: decisions that fp32 cannot
    # separate must be recovered from the rows
    S_h = np.concatenate([r.S.astype(np.float32).ravel() for r in refs])
    piv_h = np.concatenate([r.piv for r in refs]).astype(np.int32)
    tk = sum(w.budget(b) for b in range(w.B))
    keep = torch.full((tk,), -1, dtype=torch.int32, device="cuda")
    D.dart_topk_keep(desc, torch.from_numpy(S_h).cuda(), torch.from_numpy(piv_h).cuda(), keep, ws,
                     X=Xd)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(keep.cpu().numpy(), np.concatenate([r.keep for r in refs]))
    assert total == S_h.shape[0] // w.P


@pytest.mark.parametrize("make", CASES)
def test_gather_compact(make):
    w = make()
    ld = w.D + (32 if w.dtype == W.BF16 else 16)
    Xd, cu_dev, desc, ws = setup(w, ld)
    rng = np.random.default_rng(3)
    keeps = [np.sort(rng.permutation(int(n))[:w.budget(b)]).astype(np.int32)
             for b, n in enumerate(w.lengths)]
    keep = torch.from_numpy(np.concatenate(keeps)).cuda()
    tk = keep.numel()
    pos_h = rng.integers(-2**40, 2**40, size=int(w.cu[-1])).astype(np.int64)
    Y = torch.zeros((tk, w.D), dtype=Xd.dtype, device="cuda")
    pos_out = torch.zeros(tk, dtype=torch.int64, device="cuda")
    D.dart_gather_compact(desc, Xd, keep, Y, ws, pos=torch.from_numpy(pos_h).cuda(),
                          pos_out=pos_out)
    torch.cuda.synchronize()
    Yh, k0 = G.bits(Y), 0
    for b, kp in enumerate(keeps):
        lo, hi = int(w.cu[b]), int(w.cu[b + 1])
        Yr, pr = oracle.gather(w.X[lo:hi], w.dtype, pos_h[lo:hi], kp)
        assert Yh[k0:k0 + len(kp)].tobytes() == Yr.tobytes()
        np.testing.assert_array_equal(pos_out.cpu().numpy()[k0:k0 + len(kp)], pr)
        k0 += len(kp)


@pytest.mark.parametrize("drift,frames,per_frame,K", [(1e-3, 100, 16, 48), (2e-3, 40, 24, 40)])
def test_topk_keep_recovers_from_misleading_scores(drift, frames, per_frame, K):
    # Near-duplicate frames: many scores sit within the certified bound of each
    # other.  The scores handed in are the oracle's, nudged by up to half the bound,
    # so their fp32 order is wrong at many stage boundaries; with X given, the fp64
    # re-evaluation must still reproduce the oracle's retained sets (this drives the
    # correction / walk-again path).
    w = W.video_batch(B=2, frames=frames, per_frame=per_frame, D=512, P=8, K=K, n_centroids=4,
                      drift=drift)
    Xd, cu_dev, desc, ws = setup(w)
    refs = G.oracle_samples(w)
    for b, r in enumerate(refs):
        assert oracle.admissible(w.sample(b), r)
    tau = D.score_tolerance(w.dtype)
    rng = np.random.default_rng(11)
    S_h = np.concatenate([(r.S + rng.uniform(-0.5 * tau, 0.5 * tau, size=r.S.shape))
                          .astype(np.float32).ravel() for r in refs])
    piv_h = np.concatenate([r.piv for r in refs]).astype(np.int32)
    close = sum(int((r.stage_gap < 2 * tau).sum()) for r in refs)
    assert close >= 4, "the case is meant to have many boundaries inside the bound"
    keep = torch.full((w.B * w.K,), -1, dtype=torch.int32, device="cuda")
    D.dart_topk_keep(desc, torch.from_numpy(S_h).cuda(), torch.from_numpy(piv_h).cuda(), keep, ws,
                     X=Xd)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(keep.cpu().numpy(), np.concatenate([r.keep for r in refs]))


def test_stage_entry_points_with_pivots_from_outside():
    """The stage entry points chained by hand with P_ext pivot rows that are no tokens of the
    samples: selection picks P - P_ext pivots and marks the others, scores cover all P,
    the retained set spends K - (P - P_ext) slots over the P stages."""
    for w, P_ext in ((W.multicrop_batch(B=2, N=450, D=1024, P=8, K=100, n_centroids=32), 4),
                     (W.ragged_batch(B=3, n_lo=200, n_hi=700, D=768, P=12), 12),
                     (W.single_image(N=300, D=512, P=8, K=64, n_centroids=16), 2)):
        E = W.text_pivot_rows(w, P_ext, seed=3)
        flat = np.ascontiguousarray(E.reshape(-1, w.D))
        Ed = (torch.from_numpy(flat.view(np.int16)).view(torch.bfloat16) if w.dtype == W.BF16
              else torch.from_numpy(flat)).cuda()
        Xd = G.to_device(w)
        cu_dev = torch.from_numpy(w.cu).cuda() if w.ragged else None
        desc = G.desc_of(w, cu_dev, ext=Ed, P_ext=P_ext)
        ws = D.alloc_workspace(desc)
        total, total_keep = int(w.cu[-1]), sum(w.budget(b) for b in range(w.B))
        piv = torch.full((w.B * w.P,), 777, dtype=torch.int32, device="cuda")
        S = torch.full((w.P * total,), float("nan"), dtype=torch.float32, device="cuda")
        keep = torch.full((total_keep,), -1, dtype=torch.int32, device="cuda")
        cu_keep = torch.full((w.B + 1,), -1, dtype=torch.int32, device="cuda")
        Y = torch.zeros((total_keep, w.D), dtype=Xd.dtype, device="cuda")
        D.dart_select_pivots(desc, Xd, piv, ws)
        D.dart_duplication_scores(desc, Xd, piv, S, ws)
        D.dart_topk_keep(desc, S, piv, keep, ws, X=Xd, cu_keep=cu_keep)
        D.dart_gather_compact(desc, Xd, keep, Y, ws)
        torch.cuda.synchronize()
        assert D.dart_device_status(desc, ws) == D.DART_OK
        piv_h, keep_h = piv.cpu().numpy().reshape(w.B, w.P), keep.cpu().numpy()
        S_h, Y_h = S.cpu().numpy().astype(np.float64), G.bits(Y)
        tau = D.score_tolerance(w.dtype)
        k0 = 0
        for b in range(w.B):
            lo, hi = int(w.cu[b]), int(w.cu[b + 1])
            r = oracle.reduce_mixed(w.sample(b), w.dtype, E[b], w.P - P_ext, w.budget(b))
            assert oracle.admissible(w.sample(b), r)
            np.testing.assert_array_equal(piv_h[b], r.piv)
            got = S_h[w.P * lo:w.P * hi].reshape(w.P, hi - lo)
            assert np.abs(got - r.S).max() <= tau
            np.testing.assert_array_equal(keep_h[k0:k0 + w.budget(b)], r.keep)
            assert Y_h[k0:k0 + w.budget(b)].tobytes() == r.Y.tobytes()
            k0 += w.budget(b)


def test_matrix_core_sum_stays_inside_the_assumed_rounding_bound():
    """The certified score bound assumes that one bf16 matrix-core instruction returns the sum
    of its 32 exact products with an error of at most 16 * 2^-24 * sum|products| (the
    instruction's internal rounding is not documented).  Checked here on the GPU the tests run
    on, against exact fp64 sums, for unit-normal, wide-dynamic-range, all-positive, one-huge-
    term and cancelling inputs (8.4 million sums)."""
    rng = np.random.default_rng(0xDA31)
    tiles = 4096
    worst = {}
    for mode in ("normal", "wide", "positive", "huge_term", "cancel"):
        a = rng.standard_normal((tiles, 16, 32))
        b = rng.standard_normal((tiles, 16, 32))
        if mode == "wide":
            a *= np.exp2(rng.integers(-8, 8, a.shape))
            b *= np.exp2(rng.integers(-8, 8, b.shape))
        elif mode == "positive":
            a, b = np.abs(a), np.abs(b)
        elif mode == "huge_term":
            a *= 0.01
            b *= 0.01
            a[..., 0] = 4096.0
            b[..., 0] = 4096.0
        elif mode == "cancel":
            a[..., 0] = a[..., 1] = 256.0
            b[..., 0], b[..., 1] = 256.0, -256.0
        A = W.f32_to_bf16_bits(a.astype(np.float32))
        B = W.f32_to_bf16_bits(b.astype(np.float32))
        dev = lambda bits: torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()
        out = torch.empty((tiles, 16, 16), dtype=torch.float32, device="cuda")
        D.dart_probe_mfma_dot32(dev(A), dev(B), out)
        torch.cuda.synchronize()
        Af = (A.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        Bf = (B.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        # products of two bf16 values are exact in fp64; sums of 32 of them to ~1e-16 relative
        exact = np.einsum("tik,tjk->tij", Af, Bf)
        mags = np.einsum("tik,tjk->tij", np.abs(Af), np.abs(Bf))
        err = np.abs(out.cpu().numpy().astype(np.float64) - exact)
        units = err / (mags * 2.0 ** -24)
        worst[mode] = float(units.max())
        assert np.all(err <= 16.0 * 2.0 ** -24 * mags), (mode, worst[mode])
        # the layout the score kernel relies on: out[t][i][j] pairs row i of A with row j of B
        assert np.all(err <= 1e-3 * mags + 1e-30)
    print("worst error in units of 2^-24 * sum|products|:", worst, flush=True)


def test_stage_entry_points_leave_the_pivot_flag_defined():
    """With a caller-supplied-pivots descriptor every entry point that takes the workspace
    leaves the flag dart_device_status reads in a defined state, whatever the workspace held."""
    w = W.image_batch(B=2, N=200, D=256, P=8, K=40, n_centroids=8)
    Xd = G.to_device(w)
    desc = G.desc_of(w, None, mode=D.DART_PIVOT_GIVEN)
    ws = D.alloc_workspace(desc)
    rng = np.random.default_rng(2)
    piv_h = np.stack([rng.permutation(200)[:w.P] for _ in range(w.B)]).astype(np.int32)
    piv = torch.from_numpy(piv_h).cuda()
    S = torch.empty(w.P * 400, dtype=torch.float32, device="cuda")
    keep = torch.empty(w.B * w.K, dtype=torch.int32, device="cuda")
    Y = torch.empty((w.B * w.K, w.D), dtype=torch.bfloat16, device="cuda")
    ws.fill_(0xFF)  # stale flags
    D.dart_duplication_scores(desc, Xd, piv, S, ws)
    assert D.dart_device_status(desc, ws) == D.DART_OK
    ws[:256].fill_(0xFF)
    D.dart_topk_keep(desc, S, piv, keep, ws, X=Xd)
    assert D.dart_device_status(desc, ws) == D.DART_OK
    ws[:256].fill_(0xFF)
    D.dart_gather_compact(desc, Xd, keep, Y, ws)
    assert D.dart_device_status(desc, ws) == D.DART_OK
    # a list with a repeated pivot is reported by the entry points that read it
    bad = piv_h.copy()
    bad[1, 3] = bad[1, 2]
    D.dart_duplication_scores(desc, Xd, torch.from_numpy(bad).cuda(), S, ws)
    assert D.dart_device_status(desc, ws) == D.DART_ERR_DEVICE
    D.dart_gather_compact(desc, Xd, keep, Y, ws)  # reads no pivots: clears the flag
    assert D.dart_device_status(desc, ws) == D.DART_OK


def test_profiled_call_matches_the_plain_call_and_times_every_stage():
    """dart_reduce_profiled: the same outputs as dart_reduce, and for every stage that launches
    a kernel a positive duration between its two events; a stage without a kernel (the
    ordering under the single-threshold rule) leaves its events unrecorded."""
    import sys
    sys.path.insert(0, os.path.join(os.path.dirname(os.path.abspath(__file__)), ".."))
    from bench import HipEvents
    w = W.multicrop_batch(B=3, N=700, D=1024, P=16, K=120, n_centroids=64)
    base = G.run_reduce(w)
    Xd = G.to_device(w)
    tot = w.B * w.K
    for score_mode in (D.DART_SCORE_PER_PIVOT, D.DART_SCORE_MIN):
        desc = G.desc_of(w, None, score_mode=score_mode)
        ws = D.alloc_workspace(desc)
        Y = torch.zeros((tot, w.D), dtype=Xd.dtype, device="cuda")
        keep = torch.full((tot,), -1, dtype=torch.int32, device="cuda")
        evs = HipEvents(12)
        for _ in range(2):  # the second call re-stamps the same events
            D.dart_reduce_profiled(desc, Xd, Y, keep, ws, evs.handles(0, 12))
        torch.cuda.synchronize()
        times = [evs.ms(2 * s, 2 * s + 1, missing=-1.0) for s in range(6)]
        evs.close()
        print(f"[case] profiled score_mode={score_mode} stage ms {times}", flush=True)
        for s, t in enumerate(times):
            if s == 3 and score_mode != D.DART_SCORE_PER_PIVOT:
                assert t == -1.0
            else:
                assert 0.0 < t < 5.0, (s, t)
        if score_mode == D.DART_SCORE_PER_PIVOT:
            np.testing.assert_array_equal(keep.cpu().numpy(), base.keep)
            assert G.bits(Y).tobytes() == base.Y.tobytes()
