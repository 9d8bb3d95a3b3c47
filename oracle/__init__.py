"""ctypes front end of the CPU oracle (oracle/dart_oracle.cpp).

TEST INFRASTRUCTURE ONLY: the test-suite, the smoke check and the benchmark's
CPU-baseline leg may import this package; the product never does.  Nothing here
touches the GPU library.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dart_oracle.cpp")
_LIB = os.path.join(_HERE, "libdart_oracle.so")
_lib = None

F32, BF16 = 0, 1
MAX_L1, MIN_L1 = 0, 1


def build(force: bool = True) -> str:
    """Compile the oracle with the host compiler (plain -O2, OpenMP on)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O2", "-std=c++17", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
               _SRC, "-o", _LIB]
        subprocess.run(cmd, check=True)
    return _LIB


def build_sanitized() -> str:
    """Compile the oracle together with oracle/sanitize_check.cpp under AddressSanitizer and
    UndefinedBehaviorSanitizer (no recovery: the first finding aborts) and return the path of
    the executable, which runs every oracle function on exactly sized buffers."""
    exe = os.path.join(_HERE, "sanitize_check")
    cmd = ["g++", "-O1", "-g", "-std=c++17", "-fopenmp", "-Wall", "-Wextra",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           _SRC, os.path.join(_HERE, "sanitize_check.cpp"), "-o", exe]
    subprocess.run(cmd, check=True)
    return exe


def lib():
    global _lib
    if _lib is None:
        build(force=False)
        L = C.CDLL(_LIB)
        vp, i32, i64, dp = C.c_void_p, C.c_int, C.c_int64, C.c_void_p
        L.oracle_set_threads.argtypes = [i32]
        L.oracle_set_threads.restype = i32
        L.oracle_l1_norms.argtypes = [vp, i32, i64, i64, i64, dp]
        L.oracle_l1_norms.restype = None
        L.oracle_select_pivots.argtypes = [dp, i64, i32, i32, vp]
        L.oracle_select_pivots.restype = None
        L.oracle_scores.argtypes = [vp, i32, i64, i64, i64, vp, i32, dp]
        L.oracle_scores.restype = None
        L.oracle_scores_rows.argtypes = [vp, i32, i64, i64, i64, vp, i32, i64, dp]
        L.oracle_scores_rows.restype = None
        L.oracle_retain.argtypes = [dp, i64, vp, i32, i32, vp, vp, vp, dp]
        L.oracle_retain.restype = i32
        L.oracle_retain_single.argtypes = [dp, i64, vp, i32, i32, i32, vp, vp, vp, dp]
        L.oracle_retain_single.restype = i32
        L.oracle_gather.argtypes = [vp, i32, i64, i64, vp, vp, i32, vp, vp]
        L.oracle_gather.restype = None
        L.oracle_sequence_map.argtypes = [i64, i64, i64, vp, i32, vp]
        L.oracle_sequence_map.restype = i64
        L.oracle_gather_rows.argtypes = [vp, i64, i64, vp, i64, vp, i64]
        L.oracle_gather_rows.restype = None
        L.oracle_reduce.argtypes = [vp, i32, i64, i64, i64, vp, i64, i64, vp, i32, i32, i32,
                                    vp, vp, dp, dp, vp, vp, dp, vp, vp, dp]
        L.oracle_reduce.restype = i32
        L.oracle_philox4x32_10.argtypes = [vp, vp, vp]
        L.oracle_philox4x32_10.restype = None
        L.oracle_random_pivots.argtypes = [C.c_uint64, i64, i64, i32, vp]
        L.oracle_random_pivots.restype = i32
        L.oracle_random_pivots_limited.argtypes = [C.c_uint64, i64, i64, i32, i32, vp]
        L.oracle_random_pivots_limited.restype = i32
        _lib = L
    return _lib


def set_threads(n: int) -> int:
    return int(lib().oracle_set_threads(int(n)))


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _check_rows(X: np.ndarray, dtype: int):
    want = np.uint16 if dtype == BF16 else np.float32
    assert X.dtype == want and X.ndim == 2 and X.strides[1] == X.itemsize, (X.dtype, X.shape)
    return X.shape[0], X.shape[1], X.strides[0] // X.itemsize


def l1_norms(Cm: np.ndarray, dtype: int) -> np.ndarray:
    n, d, ld = _check_rows(Cm, dtype)
    out = np.empty(n, dtype=np.float64)
    lib().oracle_l1_norms(_p(Cm), dtype, n, d, ld, _p(out))
    return out


def select_pivots(c: np.ndarray, P: int, mode: int = MAX_L1) -> np.ndarray:
    c = np.ascontiguousarray(c, dtype=np.float64)
    piv = np.empty(P, dtype=np.int32)
    lib().oracle_select_pivots(_p(c), c.shape[0], P, mode, _p(piv))
    return piv


def scores(X: np.ndarray, dtype: int, piv: np.ndarray) -> np.ndarray:
    n, d, ld = _check_rows(X, dtype)
    piv = np.ascontiguousarray(piv, dtype=np.int32)
    S = np.empty((piv.shape[0], n), dtype=np.float64)
    lib().oracle_scores(_p(X), dtype, n, d, ld, _p(piv), piv.shape[0], _p(S))
    return S


def scores_rows(X: np.ndarray, dtype: int, E: np.ndarray) -> np.ndarray:
    """Scores of every token of X against rows E that are not tokens of X."""
    n, d, ld = _check_rows(X, dtype)
    pe, de, lde = _check_rows(E, dtype)
    assert de == d
    S = np.empty((pe, n), dtype=np.float64)
    lib().oracle_scores_rows(_p(X), dtype, n, d, ld, _p(E), pe, lde, _p(S))
    return S


def retain(S: np.ndarray, piv: np.ndarray, K: int, diagnostics: bool = False):
    S = np.ascontiguousarray(S, dtype=np.float64)
    P, n = S.shape
    piv = np.ascontiguousarray(piv, dtype=np.int32)
    keep = np.empty(K, dtype=np.int32)
    last = np.empty(P, dtype=np.int32)
    nxt = np.empty(P, dtype=np.int32)
    gap = np.empty(P, dtype=np.float64)
    rc = lib().oracle_retain(_p(S), n, _p(piv), P, K, _p(keep), _p(last), _p(nxt), _p(gap))
    if rc != 0:
        raise ValueError(f"oracle_retain failed rc={rc} (P={P}, K={K}, N={n})")
    return (keep, last, nxt, gap) if diagnostics else keep


AGG_MIN, AGG_MAX = 1, 2


def retain_single(S: np.ndarray, piv: np.ndarray, K: int, agg: int, diagnostics: bool = False):
    """Retained set under one threshold common to all pivots (aggregate = min or max of a
    token's scores over the pivots)."""
    S = np.ascontiguousarray(S, dtype=np.float64)
    P, n = S.shape
    piv = np.ascontiguousarray(piv, dtype=np.int32)
    keep = np.empty(K, dtype=np.int32)
    last = np.empty(1, dtype=np.int32)
    nxt = np.empty(1, dtype=np.int32)
    gap = np.empty(1, dtype=np.float64)
    rc = lib().oracle_retain_single(_p(S), n, _p(piv), P, K, agg, _p(keep), _p(last), _p(nxt),
                                    _p(gap))
    if rc != 0:
        raise ValueError(f"oracle_retain_single failed rc={rc} (P={P}, K={K}, N={n})")
    return (keep, last, nxt, gap) if diagnostics else keep


def gather(X: np.ndarray, dtype: int, pos: Optional[np.ndarray], keep: np.ndarray):
    n, d, ld = _check_rows(X, dtype)
    keep = np.ascontiguousarray(keep, dtype=np.int32)
    K = keep.shape[0]
    Y = np.empty((K, d), dtype=X.dtype)
    pos_out = None
    if pos is not None:
        pos = np.ascontiguousarray(pos, dtype=np.int64)
        pos_out = np.empty(K, dtype=np.int64)
    lib().oracle_gather(_p(X), dtype, d, ld, _p(pos), _p(keep), K, _p(Y), _p(pos_out))
    return Y, pos_out


def sequence_map(T: int, vs: int, N: int, keep: np.ndarray) -> np.ndarray:
    """Rows of the original sequence (T rows, vision span [vs, vs+N)) that make up the
    shortened one: text before, retained vision tokens, text after."""
    keep = np.ascontiguousarray(keep, dtype=np.int32)
    out = np.empty(T - N + keep.shape[0], dtype=np.int32)
    n = lib().oracle_sequence_map(T, vs, N, _p(keep), keep.shape[0], _p(out))
    if n != out.shape[0]:
        raise ValueError(f"oracle_sequence_map failed (T={T}, vs={vs}, N={N}, K={keep.shape[0]})")
    return out


def gather_rows(src: np.ndarray, row_map: np.ndarray) -> np.ndarray:
    """dst[r] = src[row_map[r]] as a byte copy; src is 2-D with contiguous rows (any stride)."""
    assert src.ndim == 2 and src.strides[1] == src.itemsize
    row_map = np.ascontiguousarray(row_map, dtype=np.int32)
    dst = np.empty((row_map.shape[0], src.shape[1]), dtype=src.dtype)
    lib().oracle_gather_rows(_p(src), src.shape[1] * src.itemsize, src.strides[0], _p(row_map),
                             row_map.shape[0], _p(dst), dst.strides[0] if dst.size else 0)
    return dst


def compact_sequences(seq_cu: np.ndarray, span_start: np.ndarray, lengths: np.ndarray, keeps):
    """A packed batch: sequence b is rows [seq_cu[b], seq_cu[b+1]) and its vision span starts
    at row span_start[b] (a row of the packed tensor) with lengths[b] tokens; keeps[b] are
    its retained tokens.  Returns (row_map over the packed tensor, new seq_cu)."""
    maps, cu = [], [0]
    for b in range(len(lengths)):
        lo, hi = int(seq_cu[b]), int(seq_cu[b + 1])
        m = sequence_map(hi - lo, int(span_start[b]) - lo, int(lengths[b]), keeps[b]) + lo
        maps.append(m.astype(np.int32))
        cu.append(cu[-1] + m.shape[0])
    row_map = np.concatenate(maps) if maps else np.empty(0, dtype=np.int32)
    return row_map, np.asarray(cu, dtype=np.int32)


class Reduced:
    """Everything oracle_reduce reports for one sample."""
    __slots__ = ("piv", "keep", "c", "S", "Y", "pos_out", "piv_gap", "stage_last",
                 "stage_next", "stage_gap")


def reduce(X: np.ndarray, dtype: int, P: int, K: int, pos: Optional[np.ndarray] = None,
           crit: Optional[np.ndarray] = None, mode: int = MAX_L1, want_scores: bool = True,
           want_rows: bool = True) -> Reduced:
    n, d, ld = _check_rows(X, dtype)
    cd = cld = 0
    if crit is not None:
        cn, cd, cld = _check_rows(crit, dtype)
        assert cn == n
    r = Reduced()
    r.piv = np.empty(P, dtype=np.int32)
    r.keep = np.empty(K, dtype=np.int32)
    r.c = np.empty(n, dtype=np.float64)
    r.S = np.empty((P, n), dtype=np.float64) if want_scores else None
    r.Y = np.empty((K, d), dtype=X.dtype) if want_rows else None
    r.pos_out = None
    if pos is not None:
        pos = np.ascontiguousarray(pos, dtype=np.int64)
        if want_rows:
            r.pos_out = np.empty(K, dtype=np.int64)
    r.piv_gap = np.empty(P, dtype=np.float64)
    r.stage_last = np.empty(P, dtype=np.int32)
    r.stage_next = np.empty(P, dtype=np.int32)
    r.stage_gap = np.empty(P, dtype=np.float64)
    rc = lib().oracle_reduce(_p(X), dtype, n, d, ld, _p(crit), cd, cld, _p(pos), P, K, mode,
                             _p(r.piv), _p(r.keep), _p(r.c), _p(r.S), _p(r.Y), _p(r.pos_out),
                             _p(r.piv_gap), _p(r.stage_last), _p(r.stage_next), _p(r.stage_gap))
    if rc != 0:
        raise ValueError(f"oracle_reduce failed rc={rc} (P={P}, K={K}, N={n})")
    return r


def reduce_given(X: np.ndarray, dtype: int, piv: np.ndarray, K: int,
                 pos: Optional[np.ndarray] = None) -> Reduced:
    """Steps 3-5 with caller-supplied pivots (the random rows of the pivot ablation):
    scores against the given pivots in the given stage order, retained set, gather."""
    r = Reduced()
    r.piv = np.ascontiguousarray(piv, dtype=np.int32)
    r.c = l1_norms(X, dtype)
    r.S = scores(X, dtype, r.piv)
    r.keep, r.stage_last, r.stage_next, r.stage_gap = retain(r.S, r.piv, K, diagnostics=True)
    r.Y, r.pos_out = gather(X, dtype, pos, r.keep)
    r.piv_gap = np.full(r.piv.shape[0], np.inf)  # no ranking decision was taken
    return r


def philox4x32_10(counter, key) -> np.ndarray:
    """One Philox4x32-10 block: counter (4 words), key (2 words) -> 4 words."""
    c = np.ascontiguousarray(counter, dtype=np.uint32)
    k = np.ascontiguousarray(key, dtype=np.uint32)
    assert c.shape == (4,) and k.shape == (2,)
    out = np.empty(4, dtype=np.uint32)
    lib().oracle_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def random_pivots(seed: int, b: int, n: int, P: int, want_draws: bool = False,
                  max_draws: Optional[int] = None):
    """The P pivots sample b of n tokens draws at random from `seed` (see
    oracle_random_pivots); with want_draws also the number of draws it took.  max_draws
    replaces the rule's limit of 4096 draws (for tests of the fill that follows it)."""
    piv = np.empty(P, dtype=np.int32)
    if max_draws is None:
        t = int(lib().oracle_random_pivots(C.c_uint64(seed & (2**64 - 1)), b, n, P, _p(piv)))
    else:
        t = int(lib().oracle_random_pivots_limited(C.c_uint64(seed & (2**64 - 1)), b, n, P,
                                                   max_draws, _p(piv)))
    assert t >= 0
    return (piv, t) if want_draws else piv


def reduce_mixed(X: np.ndarray, dtype: int, E: np.ndarray, P_in: int, K: int,
                 pos: Optional[np.ndarray] = None, mode: int = MAX_L1, agg: int = 0,
                 given: Optional[np.ndarray] = None) -> Reduced:
    """The step with pivots of two sources (the 4 visual + 4 text pivots of the pivot
    ablation): P_in pivots chosen among the tokens of X (by norm, or `given`), then the
    rows of E, which are scored against but are no tokens of X.  piv marks them -1-e.
    agg = 0: the staged rule; AGG_MIN / AGG_MAX: the single-threshold rule."""
    n = X.shape[0]
    r = Reduced()
    r.c = l1_norms(X, dtype)
    if given is not None:
        inside = np.ascontiguousarray(given, dtype=np.int32)
        assert inside.shape[0] == P_in
        r.piv_gap = np.full(P_in, np.inf)
    elif P_in > 0:
        ranked = select_pivots(r.c, min(n, P_in + 1), mode)
        inside = ranked[:P_in]
        r.piv_gap = np.array([abs(r.c[ranked[i]] - r.c[ranked[i + 1]]) if i + 1 < len(ranked)
                              else np.inf for i in range(P_in)])
    else:
        inside = np.empty(0, dtype=np.int32)
        r.piv_gap = np.empty(0)
    pe = E.shape[0]
    r.piv = np.concatenate([inside, -1 - np.arange(pe, dtype=np.int32)]).astype(np.int32)
    parts = []
    if P_in > 0:
        parts.append(scores(X, dtype, inside))
    if pe > 0:
        parts.append(scores_rows(X, dtype, E))
    r.S = np.concatenate(parts, axis=0)
    if agg == 0:
        r.keep, r.stage_last, r.stage_next, r.stage_gap = retain(r.S, r.piv, K, diagnostics=True)
    else:
        r.keep, r.stage_last, r.stage_next, r.stage_gap = retain_single(r.S, r.piv, K, agg,
                                                                        diagnostics=True)
    r.Y, r.pos_out = gather(X, dtype, pos, r.keep)
    return r


def reduce_single(X: np.ndarray, dtype: int, P: int, K: int, agg: int,
                  pos: Optional[np.ndarray] = None, mode: int = MAX_L1) -> Reduced:
    """The whole step with the single-threshold retained set: pivots and scores as in
    reduce(), then retain_single."""
    base = reduce(X, dtype, P, P, mode=mode, want_rows=False)  # pivots, norms, scores
    r = Reduced()
    r.piv, r.c, r.S, r.piv_gap = base.piv, base.c, base.S, base.piv_gap
    r.keep, r.stage_last, r.stage_next, r.stage_gap = retain_single(r.S, r.piv, K, agg,
                                                                    diagnostics=True)
    r.Y, r.pos_out = gather(X, dtype, pos, r.keep)
    return r


def admissible(X: np.ndarray, r: Reduced, rel: float = 1e-9) -> bool:
    """True if every decision the oracle took is safe from fp64 rounding: each
    margin (between consecutive pivots' norms, and between the last token taken
    and the first one refused at every stage) is either clearly non-zero, or an
    exact tie between two rows that are bit-identical (then the lowest index is
    the true answer)."""
    ranked = [p for p in r.piv if p >= 0]  # pivots from outside the sample took no decision
    P = len(ranked)
    for i in range(P):
        g = r.piv_gap[i]
        if np.isinf(g) or g > rel * abs(r.c[ranked[i]]):
            continue
        if g == 0.0 and i + 1 < P and np.array_equal(X[ranked[i]], X[ranked[i + 1]]):
            continue
        if g == 0.0 and i + 1 == P:
            # the rival is not a pivot: find it by its norm and compare rows
            rivals = [j for j in np.flatnonzero(r.c == r.c[ranked[i]]) if j not in ranked]
            if rivals and all(np.array_equal(X[ranked[i]], X[j]) for j in rivals):
                continue
        return False
    for i in range(len(r.stage_gap)):
        g = r.stage_gap[i]
        if np.isinf(g) or g > rel:
            continue
        if g == 0.0 and np.array_equal(X[r.stage_last[i]], X[r.stage_next[i]]):
            continue
        return False
    return True
