"""Parity of the fused HIP path (dart_reduce through the C ABI) with the CPU
oracle: pivots, retained indices, gathered rows and position ids bit for bit,
scores within tolerance."""
import os

import numpy as np
import pytest
import torch

import oracle
import paper_2502_11494_amd as D
from paper_2502_11494_amd import workloads as W

import gpu_util as G

pytestmark = pytest.mark.gpu


def check(w, **kw):
    print(f"[case] {w.name} B={w.B} D={w.D} P={w.P} K={w.K} lens={w.lengths[:6].tolist()}",
          flush=True)
    g = G.run_reduce(w, **kw)
    frac = G.compare(w, g, G.oracle_samples(w))
    print(f"       worst score error = {frac:.3f} of the certified bound", flush=True)
    return g


# ---- sizes the oracle finishes in seconds; several tiles and a ragged tail --------

SMALL = [
    lambda: W.single_image(N=200, D=1024, P=8, K=40, n_centroids=16),          # fp32
    lambda: W.single_image(N=577, D=1000, P=5, K=64, n_centroids=32),          # fp32, odd sizes
    lambda: W.image_batch(B=3, N=200, D=1024, P=8, K=64, n_centroids=32),      # N % 64 != 0
    lambda: W.image_batch(B=2, N=333, D=3584, P=8, K=129, n_centroids=32),     # remainder rule
    lambda: W.multicrop_batch(B=2, N=700, D=2048, P=16, K=80, n_centroids=64),  # exact copies
    lambda: W.multicrop_batch(B=1, N=1000, D=520, P=20, K=111, n_centroids=64),  # D % 256 != 0
    lambda: W.ragged_batch(B=5, n_lo=200, n_hi=900, D=1024, P=16),
    lambda: W.video_batch(B=2, frames=8, per_frame=60, D=1024, P=32, K=96, n_centroids=8),
    lambda: W.video_batch(B=1, frames=6, per_frame=50, D=512, P=40, K=100, n_centroids=8),
    # fewer free slots than pivots: most stages take nothing
    lambda: W.image_batch(B=2, N=300, D=512, P=16, K=20, n_centroids=16),
    # stage lists longer than one 1024-entry step of the walk, long scans (near-duplicate frames)
    lambda: W.video_batch(B=1, frames=40, per_frame=64, D=256, P=8, K=1500, n_centroids=8),
    # lists that need several LDS staging groups (32 lists of up to 2049 entries)
    lambda: W.video_batch(B=2, frames=32, per_frame=128, D=128, P=32, K=2048, n_centroids=8),
    # small batches with long rows: groups of waves share a score tile and split D
    # (2, 3 and 4 pivot column blocks; row lengths that leave a ragged last chunk)
    lambda: W.image_batch(B=2, N=300, D=2048, P=20, K=64, n_centroids=16),
    lambda: W.video_batch(B=1, frames=6, per_frame=50, D=2048, P=40, K=100, n_centroids=8),
    lambda: W.image_batch(B=1, N=200, D=2048, P=64, K=80, n_centroids=16),
    lambda: W.image_batch(B=2, N=150, D=2120, P=20, K=40, n_centroids=16),
    lambda: W.image_batch(B=2, N=150, D=4104, P=8, K=40, n_centroids=16),
    lambda: W.ragged_batch(B=3, n_lo=200, n_hi=500, D=4096, P=16),
]


@pytest.mark.parametrize("make", SMALL)
def test_small_cases(make):
    check(make())


def test_padded_row_stride():
    w = W.image_batch(B=2, N=150, D=1024, P=8, K=32, n_centroids=16)
    check(w, ld=1024 + 64)


def test_min_norm_pivots():
    w = W.image_batch(B=2, N=150, D=1024, P=8, K=32, n_centroids=16)
    g = G.run_reduce(w, mode=D.DART_PIVOT_MIN_L1)
    G.compare(w, g, G.oracle_samples(w, mode=oracle.MIN_L1))


def test_separate_criterion_tensor():
    w = W.image_batch(B=2, N=150, D=1024, P=8, K=32, n_centroids=16)
    rng = np.random.default_rng(5)
    crit_f = rng.standard_normal((int(w.cu[-1]), 128)).astype(np.float32)
    crit_bits = W.f32_to_bf16_bits(crit_f)
    crit_dev = torch.from_numpy(crit_bits.view(np.int16)).view(torch.bfloat16).cuda()
    g = G.run_reduce(w, crit=crit_dev)
    G.compare(w, g, G.oracle_samples(w, crit=crit_bits))


# ---- edge cases -----------------------------------------------------------------------

def test_keep_only_the_pivots_and_keep_everything():
    for K in (8, 150):
        w = W.image_batch(B=2, N=150, D=512, P=8, K=K, n_centroids=16)
        check(w)


def test_tiny_samples():
    check(W.single_image(N=1, D=256, P=1, K=1, n_centroids=1))
    check(W.image_batch(B=3, N=5, D=64, P=2, K=3, n_centroids=2))
    check(W.image_batch(B=1, N=64, D=8, P=64, K=64, n_centroids=4))


def test_identical_rows_everywhere():
    # every decision is an exact tie: only the index rule can decide, and the
    # fp64 re-evaluation paths handle whole samples
    w = W.image_batch(B=2, N=300, D=512, P=4, K=37, n_centroids=1, sigma=0.0)
    assert len(np.unique(w.sample(0), axis=0)) == 1
    g = check(w)
    np.testing.assert_array_equal(g.piv[0], [0, 1, 2, 3])
    np.testing.assert_array_equal(g.keep[:37], np.arange(37))
    # the same with more ties than the re-scoring queue holds, plus a few distinct rows
    w = W.image_batch(B=1, N=3000, D=256, P=4, K=100, n_centroids=1, sigma=0.0)
    rng = np.random.default_rng(3)
    w.X[rng.permutation(3000)[:40]] = W.f32_to_bf16_bits(
        rng.standard_normal((40, 256)).astype(np.float32))
    check(w)


def test_zero_rows_score_zero():
    w = W.image_batch(B=1, N=130, D=512, P=4, K=30, n_centroids=8)
    w.X[5] = 0
    w.X[77] = 0
    w.X[100] = 0x8000  # every element -0.0
    g = check(w)
    S = g.S.reshape(w.P, 130)
    assert np.all(S[:, [5, 77, 100]] == 0.0) and not np.any(np.signbit(S[:, [5, 77, 100]]))


@pytest.mark.parametrize("make", [
    lambda: W.image_batch(B=2, N=150, D=8, P=4, K=30, n_centroids=8),       # one 16-byte piece
    lambda: W.image_batch(B=2, N=150, D=16, P=4, K=30, n_centroids=8),
    lambda: W.single_image(N=150, D=4, P=4, K=30, n_centroids=8),           # fp32, one piece
    lambda: W.image_batch(B=2, N=90, D=65536, P=8, K=24, n_centroids=8),    # the widest rows
    lambda: W.single_image(N=70, D=65536, P=8, K=20, n_centroids=8),        # fp32, widest
], ids=["bf16-D8", "bf16-D16", "f32-D4", "bf16-D65536", "f32-D65536"])
def test_narrowest_and_widest_rows(make):
    check(make())


def test_thousands_of_tiny_samples():
    """Grids of thousands of workgroups with almost no work each: 3000 dense samples of 24
    tokens, and 2500 packed samples of 10 to 59 tokens."""
    check(W.image_batch(B=3000, N=24, D=64, P=2, K=6, n_centroids=6))
    lengths = [int(x) for x in np.random.default_rng(1).integers(10, 60, 2500)]
    check(W.ragged_batch(seed=101, B=2500, D=64, P=3, keep_num=300, keep_den=1000,
                         lengths=lengths))


def test_many_pivots_and_longest_sample():
    w = W.ragged_batch(B=2, D=256, P=64, lengths=[16384, 4100], keep_num=1, keep_den=8)
    check(w)


def test_ragged_with_empty_and_rejected_samples():
    # sample 1 is empty (valid, keeps nothing); sample 3 is shorter than P (rejected)
    w = W.ragged_batch(B=5, D=512, P=16, lengths=[300, 1, 200, 10, 400])
    # drop the one-row sample and rebuild the offsets so that sample 1 is truly empty
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
    assert D.dart_device_status(desc, ws) == D.DART_ERR_DEVICE
    np.testing.assert_array_equal(cu_keep.cpu().numpy(), np.concatenate([[0], np.cumsum(budgets)]))
    keep_h, Yh, k0 = keep.cpu().numpy(), G.bits(Y), 0
    for b, kb in enumerate(budgets):
        if kb == 0:
            continue
        xs = X[cu[b]:cu[b + 1]]
        r = oracle.reduce(xs, oracle.BF16, 16, kb)
        np.testing.assert_array_equal(keep_h[k0:k0 + kb], r.keep)
        assert Yh[k0:k0 + kb].tobytes() == r.Y.tobytes()
        k0 += kb
    # a max_N that a sample exceeds is reported, not overrun
    desc2 = D.make_desc(5, 512, 16, D.DART_BF16, keep_num=111, keep_den=1000, cu_seqlens=cu_dev,
                        total_N=int(cu[-1]), max_N=256)
    ws2 = D.alloc_workspace(desc2)
    D.dart_reduce(desc2, Xd, Y, keep, ws2, cu_keep=cu_keep)
    assert D.dart_device_status(desc2, ws2) == D.DART_ERR_DEVICE
    np.testing.assert_array_equal(cu_keep.cpu().numpy(), [0, 0, 0, 22, 22, 22])


def test_empty_batch_is_a_noop():
    desc = D.make_desc(0, 512, 4, D.DART_BF16, N=100, K=10)
    ws = torch.empty(max(D.dart_workspace_bytes(desc), 256), dtype=torch.uint8, device="cuda")
    X = torch.zeros((1, 512), dtype=torch.bfloat16, device="cuda")
    keep = torch.full((4,), -5, dtype=torch.int32, device="cuda")
    D.dart_reduce(desc, X, X, keep, ws)
    torch.cuda.synchronize()
    assert keep.cpu().tolist() == [-5] * 4


def test_runs_are_bit_identical_and_position_independent():
    w = W.multicrop_batch(B=3, N=500, D=1024, P=16, K=96, n_centroids=32)
    a = G.run_reduce(w)
    b = G.run_reduce(w)
    for f in ("piv", "keep", "S", "Y", "pos_out"):
        np.testing.assert_array_equal(getattr(a, f), getattr(b, f))
    # the same sample placed elsewhere in a batch gives the same bits
    solo = W.multicrop_batch(B=3, N=500, D=1024, P=16, K=96, n_centroids=32)
    solo.X, solo.pos, solo.cu, solo.B = w.sample(2).copy(), w.pos[:500].copy(), w.cu[:2].copy(), 1
    c = G.run_reduce(solo)
    np.testing.assert_array_equal(c.S, a.S[16 * 1000:])
    np.testing.assert_array_equal(c.keep, a.keep[2 * 96:])
    # bit-identical rows get bit-identical scores
    X0 = w.sample(0)
    S0 = a.S[:16 * 500].reshape(16, 500)
    _, inv, cnt = np.unique(X0, axis=0, return_inverse=True, return_counts=True)
    for grp in np.flatnonzero(cnt > 1)[:20]:
        m = np.flatnonzero(inv == grp)
        assert np.all(S0[:, m] == S0[:, m[:1]])


def test_random_shapes_sweep():
    """Forty seeded random shapes (token counts, hidden sizes, pivots, budgets, recipes,
    dtypes) against the oracle: whatever path a shape takes must agree bit for bit."""
    rng = np.random.default_rng(0xDA27)
    done = 0
    while done < 40:
        kind = int(rng.integers(0, 4))
        P = int(rng.choice([1, 2, 3, 7, 8, 16, 17, 24, 32, 48, 64]))
        N = int(rng.integers(max(P, 8), 1400))
        K = int(rng.integers(P, N + 1)) if rng.random() < 0.3 else int(
            rng.integers(P, max(P + 1, N // 3)))
        D_ = int(rng.choice([8, 64, 200, 256, 520, 1024, 1536]))
        B = int(rng.integers(1, 4))
        seed = int(rng.integers(1, 1 << 30))
        if kind == 0:
            w = W.single_image(seed=seed, N=N, D=(D_ + 3) // 4 * 4, P=P, K=K, n_centroids=16)
        elif kind == 1:
            w = W.image_batch(seed=seed, B=B, N=N, D=D_, P=P, K=K, n_centroids=24)
        elif kind == 2:
            w = W.multicrop_batch(seed=seed, B=B, N=N, D=D_, P=P, K=K, n_centroids=32)
        else:
            frames = int(rng.integers(2, 12))
            per = max(N // frames, P // frames + 1)
            if frames * per < max(P, K):
                continue
            w = W.video_batch(seed=seed, B=B, frames=frames, per_frame=per, D=D_, P=P,
                              K=min(K, frames * per), n_centroids=8)
        refs = G.oracle_samples(w)
        if not all(oracle.admissible(w.sample(b), r) for b, r in enumerate(refs)):
            continue  # a margin below the oracle's own resolution: not a parity case
        check(w)
        done += 1


def test_random_everything_sweep():
    """Seeded random draws over all batch recipes (fp32 and bf16, dense and packed, with and
    without separate criterion rows, pivots ranked by norm -- the library's or the caller's
    norms -- or drawn at random), hidden sizes with and without partial chunks and 1 to 64
    pivots, each compared bit for bit.  DART_SWEEP_CASES / DART_SWEEP_SEED in the environment
    make it as long as wanted (3000 cases take about three minutes)."""
    cases = int(os.environ.get("DART_SWEEP_CASES", "80"))
    rng = np.random.default_rng(int(os.environ.get("DART_SWEEP_SEED", "20261128")))
    done = skipped = 0
    while done < cases:
        kind = int(rng.integers(0, 5))
        P = int(rng.choice([1, 2, 5, 8, 13, 16, 17, 24, 32, 33, 48, 49, 64]))
        N = int(rng.integers(max(P, 8), 4000))
        K = int(rng.integers(P, N + 1)) if rng.random() < 0.2 else int(
            rng.integers(P, max(P + 1, N // 3)))
        D_ = int(rng.choice([8, 64, 136, 256, 520, 1024, 1096, 2048, 3584, 4096]))
        B = int(rng.integers(1, 6))
        if B * N * D_ > 3e7:
            continue
        seed = int(rng.integers(1, 1 << 30))
        if kind == 0:
            w = W.single_image(seed=seed, N=N, D=(D_ + 3) // 4 * 4, P=P, K=K, n_centroids=16)
        elif kind == 1:
            w = W.image_batch(seed=seed, B=B, N=N, D=D_, P=P, K=K, n_centroids=24)
        elif kind == 2:
            w = W.multicrop_batch(seed=seed, B=B, N=N, D=D_, P=P, K=K, n_centroids=32)
        elif kind == 3:
            frames = int(rng.integers(2, 12))
            per = max(N // frames, P // frames + 1)
            if frames * per < max(P, K):
                continue
            w = W.video_batch(seed=seed, B=B, frames=frames, per_frame=per, D=D_, P=P,
                              K=min(K, frames * per), n_centroids=8)
        else:
            num = int(rng.integers(60, 600))
            n_min = -(-P * 1000 // num) + 1
            lengths = [int(rng.integers(n_min, n_min + 2500)) for _ in range(B)]
            if sum(lengths) * D_ > 3e7:
                continue
            w = W.ragged_batch(seed=seed, B=B, D=D_, P=P, keep_num=num, keep_den=1000,
                               lengths=lengths)
        use_crit = w.dtype == W.BF16 and rng.random() < 0.35
        drawn = rng.random() < 0.12  # pivots drawn at random on the device instead of ranked
        draw_seed = int(rng.integers(0, 2**63))
        with_norms = not drawn and rng.random() < 0.12
        norm_err = float(rng.choice([0.0, 1e-6, 1e-4]))
        crit_bits = (W.key_states(w, int(rng.choice([64, 128, 512])), seed=seed & 0xffff)
                     if use_crit else None)
        if drawn:
            refs = [oracle.reduce_given(
                w.sample(b), w.dtype, oracle.random_pivots(draw_seed, b, int(w.lengths[b]), w.P),
                w.budget(b), pos=w.pos[int(w.cu[b]):int(w.cu[b + 1])]) for b in range(w.B)]
        else:
            refs = G.oracle_samples(w, crit=crit_bits)
        if not all(oracle.admissible(w.sample(b), r) for b, r in enumerate(refs)):
            skipped += 1
            continue  # a margin below the oracle's own resolution: not a parity case
        print(f"[case {done}] {w.name} B={w.B} D={w.D} P={w.P} K={w.K} "
              f"lens={w.lengths[:5].tolist()} crit={use_crit} drawn={drawn} norms={with_norms}",
              flush=True)
        crit_dev = (None if crit_bits is None else
                    torch.from_numpy(crit_bits.view(np.int16)).view(torch.bfloat16).cuda())
        if drawn:  # (a criterion tensor, if passed, is ignored)
            g = G.run_reduce(w, crit=crit_dev, mode=D.DART_PIVOT_RANDOM, seed=draw_seed)
        elif with_norms:  # the caller's norms, off by up to err: no norm pass
            exact = oracle.l1_norms(w.X if crit_bits is None else crit_bits, w.dtype)
            noisy = exact * (1.0 + norm_err * np.random.default_rng(draw_seed).uniform(
                -1.0, 1.0, size=exact.shape))
            g = G.run_reduce(w, crit=crit_dev, norms=(noisy.astype(np.float32), norm_err))
        else:
            g = G.run_reduce(w, crit=crit_dev)
        G.compare(w, g, refs)
        done += 1
    assert skipped <= cases // 4, f"{skipped} inadmissible draws for {cases} cases"


def test_caller_supplied_pivots():
    """DART_PIVOT_GIVEN: random distinct pivots per sample (the random rows of the pivot
    ablation), dense and ragged; scores, retained sets and rows match the oracle run with
    the same pivots.  An invalid list is reported and nothing is overrun."""
    rng = np.random.default_rng(0xDA29)
    for w in (W.multicrop_batch(B=3, N=700, D=1024, P=16, K=120, n_centroids=64),
              W.image_batch(B=2, N=333, D=520, P=5, K=64, n_centroids=32),
              W.single_image(N=300, D=256, P=8, K=50, n_centroids=16),
              W.ragged_batch(B=4, n_lo=300, n_hi=1200, D=512, P=16)):
        piv = np.stack([rng.permutation(int(w.lengths[b]))[:w.P] for b in range(w.B)]).astype(np.int32)
        refs = [oracle.reduce_given(w.sample(b), w.dtype, piv[b], w.budget(b),
                                    pos=w.pos[int(w.cu[b]):int(w.cu[b + 1])]) for b in range(w.B)]
        assert all(oracle.admissible(w.sample(b), r) for b, r in enumerate(refs))
        g = G.run_reduce(w, mode=D.DART_PIVOT_GIVEN, given_piv=piv)
        G.compare(w, g, refs)
    # the oracle's own pivots give back the default result
    w = W.multicrop_batch(B=2, N=500, D=1024, P=16, K=96, n_centroids=32)
    base = G.run_reduce(w)
    again = G.run_reduce(w, mode=D.DART_PIVOT_GIVEN, given_piv=base.piv)
    for f in ("keep", "Y", "pos_out"):
        np.testing.assert_array_equal(getattr(again, f), getattr(base, f))
    # (the scores agree within the certified bound, not bit for bit: with given pivots there is
    # no norm pass, so the token norms come from the score kernel's own Gram products)
    assert np.abs(again.S.astype(np.float64) - base.S).max() <= 2 * D.score_tolerance(w.dtype)
    # a duplicated and an out-of-range pivot are reported
    bad = base.piv.copy()
    bad[1, 3] = bad[1, 2]
    G.run_reduce(w, mode=D.DART_PIVOT_GIVEN, given_piv=bad, expect_status=D.DART_ERR_DEVICE)
    bad = base.piv.copy()
    bad[0, 0] = 500
    G.run_reduce(w, mode=D.DART_PIVOT_GIVEN, given_piv=bad, expect_status=D.DART_ERR_DEVICE)


@pytest.mark.parametrize("agg", [oracle.AGG_MIN, oracle.AGG_MAX])
def test_single_threshold_rule(agg):
    """DART_SCORE_MIN / DART_SCORE_MAX: one threshold for all pivots.  Exact copies put the
    boundary on ties (the fp64 band path), near-duplicate frames on near-ties."""
    mode = D.DART_SCORE_MIN if agg == oracle.AGG_MIN else D.DART_SCORE_MAX
    cases = [W.multicrop_batch(B=3, N=700, D=1024, P=16, K=120, n_centroids=64),
             W.image_batch(B=2, N=333, D=520, P=5, K=64, n_centroids=32),
             W.single_image(N=300, D=256, P=8, K=50, n_centroids=16),
             W.video_batch(B=2, frames=8, per_frame=60, D=512, P=8, K=96, n_centroids=8),
             W.image_batch(B=2, N=150, D=256, P=8, K=8, n_centroids=16),     # pivots only
             W.image_batch(B=2, N=150, D=256, P=8, K=150, n_centroids=16),   # keep everything
             W.image_batch(B=1, N=300, D=256, P=4, K=37, n_centroids=1, sigma=0.0),  # all ties
             W.ragged_batch(B=4, n_lo=300, n_hi=2500, D=512, P=16)]
    compared = 0
    for w in cases:
        refs = [oracle.reduce_single(w.sample(b), w.dtype, w.P, w.budget(b), agg,
                                     pos=w.pos[int(w.cu[b]):int(w.cu[b + 1])]) for b in range(w.B)]
        if not all(oracle.admissible(w.sample(b), r) for b, r in enumerate(refs)):
            continue  # a margin below the oracle's own resolution: not a parity case
        print(f"[case] {w.name} agg={agg} B={w.B} P={w.P}", flush=True)
        g = G.run_reduce(w, score_mode=mode)
        G.compare(w, g, refs)
        compared += 1
    assert compared >= 6, f"only {compared} of {len(cases)} cases were admissible"


def _mixed_refs(w, E, P_ext, agg=0, given=None):
    return [oracle.reduce_mixed(w.sample(b), w.dtype, E[b], w.P - P_ext, w.budget(b),
                                pos=w.pos[int(w.cu[b]):int(w.cu[b + 1])], agg=agg,
                                given=None if given is None else given[b][:w.P - P_ext])
            for b in range(w.B)]


def test_pivots_from_outside_the_samples():
    """The last P_ext pivots are rows that are no tokens of the sample (text-token pivots of
    the pivot ablation): scored against, staged after the inside pivots, never retained, no
    slot of the budget.  Mixed 4 + 4, all pivots from outside, budgets between P_in and P,
    ragged batches, fp32, a padded stride of the outside rows."""
    cases = [(W.multicrop_batch(B=3, N=700, D=1024, P=8, K=128, n_centroids=64), 4),
             (W.image_batch(B=2, N=333, D=520, P=8, K=64, n_centroids=32), 4),
             (W.image_batch(B=2, N=333, D=520, P=6, K=61, n_centroids=32), 6),   # none inside
             (W.single_image(N=300, D=256, P=8, K=50, n_centroids=16), 3),       # fp32
             (W.image_batch(B=2, N=200, D=256, P=16, K=16, n_centroids=16), 12),  # K < P
             (W.image_batch(B=2, N=200, D=256, P=16, K=200, n_centroids=16), 5),  # keep all
             (W.video_batch(B=2, frames=8, per_frame=60, D=512, P=40, K=120, n_centroids=8), 8),
             (W.ragged_batch(B=4, n_lo=300, n_hi=1500, D=512, P=16), 8)]
    for ci, (w, P_ext) in enumerate(cases):
        if w.K == 16 and P_ext == 12:
            w.K = 7  # P_in = 4 <= K < P
        E = W.text_pivot_rows(w, P_ext, seed=ci + 1)
        refs = _mixed_refs(w, E, P_ext)
        assert all(oracle.admissible(w.sample(b), r) for b, r in enumerate(refs)), ci
        print(f"[case] {w.name} B={w.B} P={w.P} P_ext={P_ext} K={w.K}", flush=True)
        g = G.run_reduce(w, ext=E, ext_ld=w.D + 8 * (ci % 2))
        G.compare(w, g, refs)


@pytest.mark.parametrize("agg", [oracle.AGG_MIN, oracle.AGG_MAX])
def test_pivots_from_outside_single_threshold_and_given(agg):
    """Outside pivots with the single-threshold rule, and with caller-supplied inside pivots."""
    mode = D.DART_SCORE_MIN if agg == oracle.AGG_MIN else D.DART_SCORE_MAX
    rng = np.random.default_rng(0xDA30 + agg)
    compared = 0
    for ci, (w, P_ext) in enumerate(
            [(W.multicrop_batch(B=2, N=700, D=1024, P=8, K=128, n_centroids=64), 4),
             (W.image_batch(B=2, N=333, D=520, P=6, K=61, n_centroids=32), 6),
             (W.ragged_batch(B=3, n_lo=300, n_hi=1500, D=512, P=16), 8)]):
        E = W.text_pivot_rows(w, P_ext, seed=10 + ci)
        refs = _mixed_refs(w, E, P_ext, agg=agg)
        if all(oracle.admissible(w.sample(b), r) for b, r in enumerate(refs)):
            G.compare(w, G.run_reduce(w, ext=E, score_mode=mode), refs)
            compared += 1
        piv = np.stack([np.concatenate([rng.permutation(int(w.lengths[b]))[:w.P - P_ext],
                                        np.full(P_ext, 12345)]) for b in range(w.B)]).astype(np.int32)
        refs = _mixed_refs(w, E, P_ext, given=piv)
        assert all(oracle.admissible(w.sample(b), r) for b, r in enumerate(refs))
        G.compare(w, G.run_reduce(w, ext=E, mode=D.DART_PIVOT_GIVEN, given_piv=piv), refs)
    assert compared >= 2, f"only {compared} of 3 single-threshold cases were admissible"


def test_random_ragged_sweep():
    """Twelve seeded random packed batches (lengths, ratios, pivots) against the oracle."""
    rng = np.random.default_rng(0xDA28)
    compared = 0
    for _ in range(12):
        P = int(rng.choice([1, 4, 8, 16, 32, 64]))
        num, den = int(rng.integers(60, 600)), 1000
        n_min = -(-P * den // num) + 1  # the shortest sample still keeps >= P tokens
        B = int(rng.integers(1, 7))
        lengths = [int(rng.integers(n_min, n_min + 1500)) for _ in range(B)]
        D_ = int(rng.choice([64, 256, 520, 1024]))
        w = W.ragged_batch(seed=int(rng.integers(1, 1 << 30)), B=B, D=D_, P=P, keep_num=num,
                           keep_den=den, lengths=lengths)
        refs = G.oracle_samples(w)
        if not all(oracle.admissible(w.sample(b), r) for b, r in enumerate(refs)):
            continue  # a margin below the oracle's own resolution: not a parity case
        check(w)
        compared += 1
    assert compared >= 10, f"only {compared} of 12 random batches were admissible"


# ---- the five benchmark configurations at full size --------------------------------

def test_config0_single_image_fp32():
    check(W.by_index(0))


@pytest.mark.parametrize("K", [64, 128, 192])
def test_config1_image_batch(K):
    check(W.by_index(1, K=K))


def test_config1_pivot_ablation_four_visual_four_text():
    """The pivot ablation's setting at full size: B=16 images of 576 tokens, 4 visual + 4 text
    pivots, 128 retained tokens (Table 8 caption)."""
    w = W.by_index(1, K=128)
    assert w.P == 8
    E = W.text_pivot_rows(w, 4, seed=8)
    refs = _mixed_refs(w, E, 4)
    assert all(oracle.admissible(w.sample(b), r) for b, r in enumerate(refs))
    G.compare(w, G.run_reduce(w, ext=E), refs)


@pytest.mark.parametrize("Dc", [1024, 512])
def test_config2_key_norm_criterion(Dc):
    """The K-norm criterion at full size with grouped-query shapes: the pivots come from the
    L1 norms of separate key-state rows (8 or 4 kv heads of 128), the hidden states are read
    by the score pass only."""
    w = W.by_index(2)
    crit_bits = W.key_states(w, Dc, seed=Dc)
    crit_dev = torch.from_numpy(crit_bits.view(np.int16)).view(torch.bfloat16).cuda()
    refs = G.oracle_samples(w, crit=crit_bits)
    assert all(oracle.admissible(w.sample(b), r) for b, r in enumerate(refs))
    g = G.run_reduce(w, crit=crit_dev)
    G.compare(w, g, refs)
    # the pivots differ from those of the hidden-state norms
    assert not np.array_equal(g.piv, np.stack([r.piv for r in G.oracle_samples(w)]))


def test_config2_multicrop_batch():
    check(W.by_index(2))


@pytest.mark.parametrize("agg", [oracle.AGG_MIN, oracle.AGG_MAX])
def test_config2_single_threshold(agg):
    w = W.by_index(2)
    refs = [oracle.reduce_single(w.sample(b), w.dtype, w.P, w.budget(b), agg,
                                 pos=w.pos[int(w.cu[b]):int(w.cu[b + 1])]) for b in range(w.B)]
    assert all(oracle.admissible(w.sample(b), r) for b, r in enumerate(refs))
    g = G.run_reduce(w, score_mode=D.DART_SCORE_MIN if agg == oracle.AGG_MIN else D.DART_SCORE_MAX)
    G.compare(w, g, refs)


def test_config4_video_batch():
    check(W.by_index(4))


def test_config3_ragged_batch():
    check(W.by_index(3))


@pytest.mark.parametrize("index", [2, 4])
def test_full_size_runs_are_bit_identical(index):
    """The headline and the video batch at full size, twice: every output bit for bit the
    same (no result may depend on which workgroup finished first)."""
    w = W.by_index(index)
    a = G.run_reduce(w)
    b = G.run_reduce(w)
    for f in ("piv", "keep", "cu_keep", "S", "Y", "pos_out"):
        np.testing.assert_array_equal(getattr(a, f), getattr(b, f), err_msg=f)


# ---- other modalities and model sizes the paper reports on ----------------------------------

@pytest.mark.parametrize("name,kw", [
    ("audio", dict(keep_num=800)), ("audio", dict(keep_num=700)), ("audio", dict(keep_num=500)),
    ("action", {}), ("wide13b", {}), ("wide72b", {}), ("wide72b", dict(K=64, P=16)),
])
def test_other_modalities_and_hidden_sizes(name, kw):
    """Audio tokens pruned by 20/30/50 % with 8 pivots (packed utterances), 256 -> 56 tokens of
    a vision-language-action model, and the hidden sizes of 13B and 72B language models."""
    check(W.by_name(name, **kw))


def test_audio_with_key_norm_criterion_on_spans():
    """The audio study's setting end to end: K-norm pivots from separate key rows, the audio
    tokens sitting inside whole sequences, 30 % pruned."""
    w = W.by_name("audio", B=6)
    sq = W.sequences_around(w, seed=9)
    crit_rows = W.key_states(w, 1024, seed=4)
    crit_full = np.zeros((sq.H.shape[0], 1024), dtype=crit_rows.dtype)
    for b in range(w.B):  # key rows exist for every row of the sequence; only the span's count
        crit_full[sq.span_start[b]:sq.span_start[b] + int(w.lengths[b])] = \
            crit_rows[int(w.cu[b]):int(w.cu[b + 1])]
    dev = lambda a: torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).cuda()
    Hd, Cd = dev(sq.H), dev(crit_full)
    cu_dev, span_dev = torch.from_numpy(w.cu).cuda(), torch.from_numpy(sq.span_start).cuda()
    desc = D.make_desc(w.B, w.D, w.P, w.dtype, keep_num=w.keep_num, keep_den=w.keep_den,
                       cu_seqlens=cu_dev, total_N=int(w.cu[-1]), max_N=int(w.lengths.max()),
                       span_start=span_dev, X_rows=sq.H.shape[0])
    ws = D.alloc_workspace(desc)
    total_keep = sum(w.budget(b) for b in range(w.B))
    keep = torch.empty(total_keep, dtype=torch.int32, device="cuda")
    piv = torch.empty(w.B * w.P, dtype=torch.int32, device="cuda")
    D.dart_reduce(desc, Hd, None, keep, ws, crit=Cd, crit_D=1024, crit_ld=1024, piv_out=piv)
    torch.cuda.synchronize()
    assert D.dart_device_status(desc, ws) == D.DART_OK
    k0 = 0
    for b, r in enumerate(G.oracle_samples(w, crit=crit_rows)):
        assert oracle.admissible(w.sample(b), r)
        np.testing.assert_array_equal(piv.cpu().numpy()[b * w.P:(b + 1) * w.P], r.piv)
        np.testing.assert_array_equal(keep.cpu().numpy()[k0:k0 + w.budget(b)], r.keep)
        k0 += w.budget(b)


# ---- value range ------------------------------------------------------------------------------

@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_power_of_two_scales_change_no_output_bit(dtype):
    """Inside the documented value range (2^-55 <= |x| <= 2^55) a common power-of-two factor is
    exact in every fp32 and fp64 step of the path: pivots, scores, retained set are
    bit-identical to the unscaled run and equal to the oracle's."""
    if dtype == "bf16":
        w = W.multicrop_batch(B=2, N=700, D=1024, P=16, K=80, n_centroids=64)
    else:
        w = W.single_image(N=300, D=512, P=8, K=64, n_centroids=16)
    refs = G.oracle_samples(w)
    base = G.run_reduce(w)
    G.compare(w, base, refs)
    orig = w.X.copy()
    for e in (-50, -30, 30, 50):
        if dtype == "bf16":  # exponent field of a bf16: bits 7..14
            scaled = orig.copy()
            nz = (orig & 0x7FFF) != 0
            scaled[nz] = (orig[nz].astype(np.int32) + (e << 7)).astype(np.uint16)
        else:
            scaled = (orig.astype(np.float64) * 2.0 ** e).astype(np.float32)
        w.X = scaled
        g = G.run_reduce(w)
        for f in ("piv", "keep", "S", "pos_out"):
            np.testing.assert_array_equal(getattr(g, f), getattr(base, f), err_msg=f"2^{e}: {f}")
        scaled_refs = G.oracle_samples(w)
        for b, r in enumerate(scaled_refs):
            np.testing.assert_array_equal(r.keep, refs[b].keep)
        G.compare(w, g, scaled_refs)
    w.X = orig


def test_rows_of_very_different_magnitudes():
    """Every row carries its own power-of-two factor (2^-20 .. 2^20): cosines do not change, the
    norms (and with them the pivots) do; the result must follow the oracle on the scaled rows.
    (No exact copies in this input: copies with different factors would tie exactly as
    different rows, which the oracle cannot decide either.)"""
    w = W.image_batch(B=2, N=600, D=1024, P=16, K=80, n_centroids=64)
    rng = np.random.default_rng(11)
    e = rng.integers(-20, 21, size=w.X.shape[0])
    nz = (w.X & 0x7FFF) != 0
    w.X = np.where(nz, (w.X.astype(np.int32) + (e[:, None] << 7)), w.X).astype(np.uint16)
    check(w)
