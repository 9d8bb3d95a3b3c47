"""Vision tokens as spans of whole sequences (text before and after), and the compaction of
the whole sequences: hidden states, cached key/value rows, multi-plane position ids and the
new sequence offsets, against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2502_11494_amd as D
from paper_2502_11494_amd import workloads as W

import gpu_util as G

pytestmark = pytest.mark.gpu


def dev(a, dtype):
    if dtype == W.BF16 and a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(a).cuda()


def run(w, sq, seq_cu=None, span=None, expect=D.DART_OK, X_rows=None):
    """dart_reduce on the spans (no gather), then dart_compact_sequences."""
    rows = sq.H.shape[0]
    Hd = dev(sq.H, w.dtype)
    cu_dev = torch.from_numpy(w.cu).cuda()
    span_dev = torch.from_numpy(sq.span_start if span is None else span).cuda()
    seq_dev = torch.from_numpy(sq.seq_cu if seq_cu is None else seq_cu).cuda()
    lens = w.lengths
    desc = D.make_desc(w.B, w.D, w.P, w.dtype, K=w.K, keep_num=w.keep_num, keep_den=w.keep_den,
                       cu_seqlens=cu_dev, total_N=int(w.cu[-1]), max_N=int(lens.max()),
                       span_start=span_dev, X_rows=rows if X_rows is None else X_rows)
    ws = D.alloc_workspace(desc)
    total_keep = sum(w.budget(b) for b in range(w.B))
    total_N = int(w.cu[-1])
    keep = torch.full((max(total_keep, 1),), -1, dtype=torch.int32, device="cuda")
    cu_keep = torch.full((w.B + 1,), -1, dtype=torch.int32, device="cuda")
    piv = torch.full((w.B * w.P,), -1, dtype=torch.int32, device="cuda")
    S = torch.full((w.P * total_N,), float("nan"), dtype=torch.float32, device="cuda")
    D.dart_reduce(desc, Hd, None, keep, ws, cu_keep=cu_keep, piv_out=piv, S_out=S)
    out_rows = rows - total_N + total_keep
    row_map = torch.full((max(out_rows, 1),), -7, dtype=torch.int32, device="cuda")
    seq_out = torch.full((w.B + 1,), -1, dtype=torch.int32, device="cuda")
    srcs = [Hd] + [dev(t, w.dtype) for t in sq.kv]
    dsts = [torch.zeros((max(out_rows, 1), s.shape[1]), dtype=s.dtype, device="cuda") for s in srcs]
    posd = torch.from_numpy(sq.pos).cuda()
    pos_out = torch.full((3, max(out_rows, 1)), -1, dtype=torch.int64, device="cuda")
    D.dart_compact_sequences(desc, seq_dev, keep, list(zip(srcs, dsts)), seq_out, row_map, ws,
                             pos=posd, pos_out=pos_out)
    torch.cuda.synchronize()
    assert D.dart_device_status(desc, ws) == expect
    return dict(keep=keep.cpu().numpy()[:total_keep], cu_keep=cu_keep.cpu().numpy(),
                piv=piv.cpu().numpy().reshape(w.B, w.P), S=S.cpu().numpy(),
                row_map=row_map.cpu().numpy(), seq_out=seq_out.cpu().numpy(),
                dsts=[G.bits(d) for d in dsts], pos_out=pos_out.cpu().numpy(), out_rows=out_rows)


CASES = [
    lambda: W.ragged_batch(B=5, n_lo=200, n_hi=900, D=1024, P=16),
    lambda: W.multicrop_batch(B=3, N=700, D=1024, P=8, K=128, n_centroids=64),
    lambda: W.single_image(N=300, D=256, P=8, K=50, n_centroids=16),            # fp32
    lambda: W.video_batch(B=2, frames=8, per_frame=60, D=512, P=32, K=96, n_centroids=8),
    lambda: W.image_batch(B=4, N=150, D=520, P=4, K=150, n_centroids=16),       # keep everything
]


@pytest.mark.parametrize("make", CASES)
def test_spans_and_sequence_compaction(make):
    w = make()
    sq = W.sequences_around(w, seed=3, kv_width=264)
    print(f"[case] {w.name} B={w.B} rows={sq.H.shape[0]} seq_cu={sq.seq_cu.tolist()}", flush=True)
    g = run(w, sq)
    refs = G.oracle_samples(w)
    tau = D.score_tolerance(w.dtype)
    k0, keeps = 0, []
    for b, r in enumerate(refs):
        lo, hi = int(w.cu[b]), int(w.cu[b + 1])
        kb = w.budget(b)
        assert oracle.admissible(w.sample(b), r)
        np.testing.assert_array_equal(g["piv"][b], r.piv)
        got = g["S"][w.P * lo:w.P * hi].reshape(w.P, hi - lo).astype(np.float64)
        assert np.abs(got - r.S).max() <= tau
        np.testing.assert_array_equal(g["keep"][k0:k0 + kb], r.keep)
        assert g["cu_keep"][b] == k0
        keeps.append(r.keep)
        k0 += kb
    row_map, cu_out = oracle.compact_sequences(sq.seq_cu, sq.span_start, w.lengths, keeps)
    assert cu_out[-1] == g["out_rows"]
    np.testing.assert_array_equal(g["seq_out"], cu_out)
    np.testing.assert_array_equal(g["row_map"][:g["out_rows"]], row_map)
    for src, dst in zip([sq.H] + sq.kv, g["dsts"]):
        assert dst[:g["out_rows"]].tobytes() == oracle.gather_rows(src, row_map).tobytes()
    for p in range(3):
        want = oracle.gather_rows(sq.pos[p].reshape(-1, 1), row_map)[:, 0]
        np.testing.assert_array_equal(g["pos_out"][p, :g["out_rows"]], want)


def test_reduce_on_spans_gathers_rows_and_positions_of_X():
    """dart_reduce with Y on spans: rows and position ids are taken at the span's rows of X."""
    w = W.ragged_batch(B=4, n_lo=200, n_hi=700, D=512, P=8)
    sq = W.sequences_around(w, seed=5)
    Hd = dev(sq.H, w.dtype)
    cu_dev = torch.from_numpy(w.cu).cuda()  # named by the descriptor: must outlive the calls
    span_dev = torch.from_numpy(sq.span_start).cuda()
    desc = D.make_desc(w.B, w.D, w.P, w.dtype, keep_num=w.keep_num, keep_den=w.keep_den,
                       cu_seqlens=cu_dev, total_N=int(w.cu[-1]), max_N=int(w.lengths.max()),
                       span_start=span_dev, X_rows=sq.H.shape[0])
    ws = D.alloc_workspace(desc)
    total_keep = sum(w.budget(b) for b in range(w.B))
    keep = torch.empty(total_keep, dtype=torch.int32, device="cuda")
    Y = torch.zeros((total_keep, w.D), dtype=Hd.dtype, device="cuda")
    posd = torch.from_numpy(np.ascontiguousarray(sq.pos[1])).cuda()
    pos_out = torch.empty(total_keep, dtype=torch.int64, device="cuda")
    D.dart_reduce(desc, Hd, Y, keep, ws, pos=posd, pos_out=pos_out)
    torch.cuda.synchronize()
    assert D.dart_device_status(desc, ws) == D.DART_OK
    k0 = 0
    for b, r in enumerate(G.oracle_samples(w)):
        kb = w.budget(b)
        np.testing.assert_array_equal(keep.cpu().numpy()[k0:k0 + kb], r.keep)
        assert G.bits(Y)[k0:k0 + kb].tobytes() == r.Y.tobytes()
        np.testing.assert_array_equal(pos_out.cpu().numpy()[k0:k0 + kb],
                                      sq.pos[1][sq.span_start[b] + r.keep])
        k0 += kb


def test_invalid_spans_and_sequences_are_reported():
    w = W.ragged_batch(B=4, n_lo=200, n_hi=700, D=256, P=8)
    sq = W.sequences_around(w, seed=6)
    rows = sq.H.shape[0]
    # a span that leaves X: the sample is skipped and reported, the others are unaffected
    span = sq.span_start.copy()
    span[2] = rows - 5
    g = run(w, sq, span=span, expect=D.DART_ERR_DEVICE)
    refs = G.oracle_samples(w)
    np.testing.assert_array_equal(g["keep"][:w.budget(0)], refs[0].keep)
    assert g["cu_keep"][3] - g["cu_keep"][2] == 0
    # (the moved span is also outside its sequence, so nothing is compacted)
    assert not g["seq_out"].any()
    # a span inside X but outside its sequence
    span = sq.span_start.copy()
    span[1] = sq.seq_cu[2]
    g = run(w, sq, span=span, expect=D.DART_ERR_DEVICE)
    assert not g["seq_out"].any() and (g["row_map"] == -7).all()
    # sequence offsets that do not end at the last row
    bad = sq.seq_cu.copy()
    bad[-1] -= 1
    g = run(w, sq, seq_cu=bad, expect=D.DART_ERR_DEVICE)
    assert not g["seq_out"].any()
    # decreasing sequence offsets
    bad = sq.seq_cu.copy()
    bad[2] = bad[1] - 1
    g = run(w, sq, seq_cu=bad, expect=D.DART_ERR_DEVICE)
    assert not g["seq_out"].any()


def test_random_combinations_of_the_variants():
    """Sixteen seeded random batches mixing everything the descriptor offers: spans inside
    whole sequences, pivots from outside, either retained-set rule, largest / smallest /
    caller-supplied pivots, a separate criterion tensor, fixed or proportional budgets."""
    rng = np.random.default_rng(0xDA31)
    done = 0
    while done < 16:
        P = int(rng.choice([2, 4, 8, 16, 24]))
        P_ext = int(rng.integers(0, P + 1)) if rng.random() < 0.6 else 0
        P_in = P - P_ext
        B = int(rng.integers(1, 5))
        D_ = int(rng.choice([64, 256, 520, 1024]))
        lengths = [int(rng.integers(max(P, 40), 900)) for _ in range(B)]
        seed = int(rng.integers(1, 1 << 30))
        w = W.ragged_batch(seed=seed, B=B, D=D_, P=P, keep_num=int(rng.integers(80, 500)),
                           keep_den=1000, lengths=lengths)
        if rng.random() < 0.4:
            w.K, w.keep_num = int(rng.integers(max(P_in, 1), min(lengths) + 1)), 0
        if any(w.budget(b) < max(P_in, 1) for b in range(B)):
            continue
        agg = int(rng.choice([0, 0, oracle.AGG_MIN, oracle.AGG_MAX]))
        pmode = int(rng.choice([D.DART_PIVOT_MAX_L1, D.DART_PIVOT_MIN_L1, D.DART_PIVOT_GIVEN]))
        use_crit = pmode != D.DART_PIVOT_GIVEN and rng.random() < 0.5
        sq = W.sequences_around(w, seed=seed ^ 5, n_kv=1, kv_width=64)
        rows = sq.H.shape[0]
        E = W.text_pivot_rows(w, P_ext, seed=seed ^ 7) if P_ext else None
        crit_rows = W.key_states(w, 128, seed=seed ^ 9) if use_crit else None
        given = None
        if pmode == D.DART_PIVOT_GIVEN:
            given = np.stack([np.concatenate([rng.permutation(lengths[b])[:P_in],
                                              np.full(P_ext, -99)]) for b in range(B)]).astype(np.int32)
        refs = []
        for b in range(B):
            lo, hi = int(w.cu[b]), int(w.cu[b + 1])
            X = w.X[lo:hi]
            Eb = E[b] if P_ext else np.empty((0, w.D), dtype=X.dtype)
            if given is not None:
                r = oracle.reduce_mixed(X, w.dtype, Eb, P_in, w.budget(b), agg=agg,
                                        given=given[b][:P_in])
            elif use_crit:
                # pivots by the criterion rows: rank them with the oracle's own steps
                c = oracle.l1_norms(crit_rows[lo:hi], w.dtype)
                ranked = oracle.select_pivots(c, min(hi - lo, P_in + 1), pmode) if P_in else \
                    np.empty(0, dtype=np.int32)
                r = oracle.reduce_mixed(X, w.dtype, Eb, P_in, w.budget(b), agg=agg,
                                        given=ranked[:P_in])
                r.c = c
                r.piv_gap = np.array([abs(c[ranked[i]] - c[ranked[i + 1]]) if i + 1 < len(ranked)
                                      else np.inf for i in range(P_in)])
            else:
                r = oracle.reduce_mixed(X, w.dtype, Eb, P_in, w.budget(b), mode=pmode, agg=agg)
            refs.append(r)
        if not all(oracle.admissible(w.sample(b), r) for b, r in enumerate(refs)):
            continue
        print(f"[case {done}] B={B} P={P} P_ext={P_ext} D={D_} K={w.K or (w.keep_num, 1000)} "
              f"agg={agg} pivots={pmode} crit={use_crit} lens={lengths}", flush=True)
        # ---- GPU
        Hd = dev(sq.H, w.dtype)
        cu_dev, span_dev = torch.from_numpy(w.cu).cuda(), torch.from_numpy(sq.span_start).cuda()
        Ed = dev(np.ascontiguousarray(E.reshape(-1, w.D)), w.dtype) if P_ext else None
        desc = D.make_desc(B, w.D, P, w.dtype, K=w.K, keep_num=w.keep_num, keep_den=w.keep_den,
                           cu_seqlens=cu_dev, total_N=int(w.cu[-1]), max_N=max(lengths),
                           pivot_mode=pmode, score_mode=agg, ext_pivots=Ed, P_ext=P_ext,
                           span_start=span_dev, X_rows=rows)
        ws = D.alloc_workspace(desc)
        total_keep = sum(w.budget(b) for b in range(B))
        keep = torch.full((max(total_keep, 1),), -1, dtype=torch.int32, device="cuda")
        piv = (torch.from_numpy(given.reshape(-1)).cuda() if given is not None
               else torch.full((B * P,), -5, dtype=torch.int32, device="cuda"))
        kw = {}
        if use_crit:
            full = np.zeros((rows, 128), dtype=crit_rows.dtype)
            for b in range(B):
                full[sq.span_start[b]:sq.span_start[b] + lengths[b]] = \
                    crit_rows[int(w.cu[b]):int(w.cu[b + 1])]
            Cd = dev(full, w.dtype)
            kw = dict(crit=Cd, crit_D=128, crit_ld=128)
        D.dart_reduce(desc, Hd, None, keep, ws, piv_out=piv, **kw)
        out_rows = rows - int(w.cu[-1]) + total_keep
        row_map = torch.full((max(out_rows, 1),), -7, dtype=torch.int32, device="cuda")
        seq_out = torch.full((B + 1,), -1, dtype=torch.int32, device="cuda")
        Hout = torch.zeros((max(out_rows, 1), w.D), dtype=Hd.dtype, device="cuda")
        D.dart_compact_sequences(desc, torch.from_numpy(sq.seq_cu).cuda(), keep, [(Hd, Hout)],
                                 seq_out, row_map, ws)
        torch.cuda.synchronize()
        assert D.dart_device_status(desc, ws) == D.DART_OK
        k0, keeps = 0, []
        for b, r in enumerate(refs):
            kb = w.budget(b)
            np.testing.assert_array_equal(piv.cpu().numpy()[b * P:(b + 1) * P], r.piv)
            np.testing.assert_array_equal(keep.cpu().numpy()[k0:k0 + kb], r.keep)
            keeps.append(r.keep)
            k0 += kb
        want_map, cu_out = oracle.compact_sequences(sq.seq_cu, sq.span_start, w.lengths, keeps)
        np.testing.assert_array_equal(seq_out.cpu().numpy(), cu_out)
        np.testing.assert_array_equal(row_map.cpu().numpy()[:out_rows], want_map)
        assert G.bits(Hout)[:out_rows].tobytes() == oracle.gather_rows(sq.H, want_map).tobytes()
        done += 1
