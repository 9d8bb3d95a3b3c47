"""Seeded synthetic inputs with the shapes of the paper's workloads.

The paper's inputs (LLaVA-1.5 images with 576 vision tokens, LLaVA-Next
multi-crop images with 2880, dynamic-resolution Qwen2-VL images, multi-frame
video; Section 4 and Tables 1-6) need model weights and datasets.  These
generators stand in for them: hidden states are clustered Gaussians, so that
near-duplicate tokens abound the way they do after an early decoder layer.

This module holds no arithmetic of the reduction method itself.  It only draws
numbers; both the CPU oracle's tests and the GPU path's tests consume its
arrays.  numpy only.

bf16 tensors are returned as uint16 bit patterns (round-to-nearest-even of the
fp32 value).
"""
from __future__ import annotations

import dataclasses
from typing import List, Optional

import numpy as np

F32 = 0
BF16 = 1


@dataclasses.dataclass
class Workload:
    """One batch for the reduction step.

    X        [total_N, D] float32, or uint16 bit patterns when dtype == BF16
    pos      [total_N] int64 position ids (0..N_b-1 inside every sample)
    cu       [B+1] int32 row offsets of the samples (also given for dense)
    ragged   True if the per-sample lengths differ (packed layout)
    K        per-sample keep budget, or 0 when the ratio keep_num/keep_den rules
    """
    name: str
    X: np.ndarray
    pos: np.ndarray
    cu: np.ndarray
    dtype: int
    B: int
    D: int
    P: int
    K: int
    keep_num: int
    keep_den: int
    ragged: bool

    @property
    def lengths(self) -> np.ndarray:
        return np.diff(self.cu).astype(np.int64)

    def budget(self, b: int) -> int:
        n = int(self.cu[b + 1] - self.cu[b])
        return self.K if self.K > 0 else (n * self.keep_num) // self.keep_den

    def sample(self, b: int) -> np.ndarray:
        return self.X[self.cu[b]:self.cu[b + 1]]


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rng(seed: int, *stream: int) -> np.random.Generator:
    return np.random.default_rng(np.random.SeedSequence([seed, *stream]))


def clustered_tokens(rng: np.random.Generator, n: int, d: int, n_centroids: int,
                     sigma: float) -> np.ndarray:
    """n rows = unit-normal centroid (drawn uniformly among n_centroids) plus
    N(0, sigma^2) noise; float32."""
    cent = rng.standard_normal((n_centroids, d), dtype=np.float32)
    which = rng.integers(0, n_centroids, size=n)
    out = cent[which]
    chunk = max(1, (1 << 24) // d)
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        out[s:e] += np.float32(sigma) * rng.standard_normal((e - s, d), dtype=np.float32)
    return out


def _finish(name, rows: List[np.ndarray], dtype, P, K, keep_num=0, keep_den=1,
            ragged=False) -> Workload:
    lens = [r.shape[0] for r in rows]
    cu = np.zeros(len(rows) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(lens)
    D = rows[0].shape[1]
    if dtype == BF16:
        X = np.empty((int(cu[-1]), D), dtype=np.uint16)
        for b, r in enumerate(rows):
            X[cu[b]:cu[b + 1]] = f32_to_bf16_bits(r)
    else:
        X = np.ascontiguousarray(np.concatenate(rows, axis=0), dtype=np.float32)
    pos = np.concatenate([np.arange(n, dtype=np.int64) for n in lens])
    return Workload(name, X, pos, cu, dtype, len(rows), D, P, K, keep_num, keep_den, ragged)


def single_image(seed: int = 0xDA270000, N: int = 576, D: int = 4096, P: int = 8,
                 K: int = 64, n_centroids: int = 64, sigma: float = 0.05) -> Workload:
    """One 576-token image, fp32 (LLaVA-1.5 token count, Table 1)."""
    rows = [clustered_tokens(_rng(seed, 0), N, D, n_centroids, sigma)]
    return _finish("single_image", rows, F32, P, K)


def image_batch(seed: int = 0xDA270001, B: int = 16, N: int = 576, D: int = 4096, P: int = 8,
                K: int = 64, n_centroids: int = 128, sigma: float = 0.1) -> Workload:
    """Batch of 576-token images, bf16; budgets 64/128/192 are those of Table 1."""
    rows = [clustered_tokens(_rng(seed, b), N, D, n_centroids, sigma) for b in range(B)]
    return _finish("image_batch", rows, BF16, P, K)


def multicrop_batch(seed: int = 0xDA270002, B: int = 8, N: int = 2880, D: int = 4096,
                    P: int = 16, K: int = 320, n_centroids: int = 256, sigma: float = 0.1,
                    copy_frac: float = 0.10) -> Workload:
    """High-resolution multi-crop images (2880 tokens kept down to 320, Tables 2-3),
    bf16, with a tenth of the tokens overwritten by bit-exact copies of others."""
    rows = []
    for b in range(B):
        rng = _rng(seed, b)
        x = clustered_tokens(rng, N, D, n_centroids, sigma)
        n_copy = int(N * copy_frac)
        perm = rng.permutation(N)
        dst, pool = perm[:n_copy], perm[n_copy:]
        src = pool[rng.integers(0, pool.shape[0], size=n_copy)]
        x[dst] = x[src]
        rows.append(x)
    return _finish("multicrop_batch", rows, BF16, P, K)


def ragged_batch(seed: int = 0xDA270003, B: int = 32, n_lo: int = 1024, n_hi: int = 16384,
                 D: int = 3584, P: int = 16, keep_num: int = 111, keep_den: int = 1000,
                 sigma: float = 0.1, lengths: Optional[List[int]] = None) -> Workload:
    """Dynamic-resolution images of different token counts packed back to back
    (Table 4's model family); N_b uniform in [n_lo, n_hi], N_b/16 centroids,
    each sample keeps floor(11.1 %) of its tokens."""
    if lengths is None:
        lengths = [int(v) for v in _rng(seed, 1 << 20).integers(n_lo, n_hi + 1, size=B)]
    rows = [clustered_tokens(_rng(seed, b), n, D, max(1, n // 16), sigma)
            for b, n in enumerate(lengths)]
    return _finish("ragged_batch", rows, BF16, P, 0, keep_num, keep_den, ragged=True)


def video_batch(seed: int = 0xDA270004, B: int = 4, frames: int = 64, per_frame: int = 144,
                D: int = 3584, P: int = 32, K: int = 1024, n_centroids: int = 16,
                sigma: float = 0.1, drift: float = 0.02) -> Workload:
    """Video: frame f = frame f-1 + N(0, drift^2), accumulated in fp32, so tokens
    duplicate heavily across frames (Table 6's setting); token index f*per_frame+t."""
    rows = []
    for b in range(B):
        rng = _rng(seed, b)
        x = np.empty((frames * per_frame, D), dtype=np.float32)
        cur = clustered_tokens(rng, per_frame, D, n_centroids, sigma)
        x[:per_frame] = cur
        for f in range(1, frames):
            cur = cur + np.float32(drift) * rng.standard_normal((per_frame, D), dtype=np.float32)
            x[f * per_frame:(f + 1) * per_frame] = cur
        rows.append(x)
    return _finish("video_batch", rows, BF16, P, K)


def by_index(i: int, **kw) -> Workload:
    """The five benchmark configurations, 0..4, at their full sizes by default."""
    return [single_image, image_batch, multicrop_batch, ragged_batch, video_batch][i](**kw)


def text_pivot_rows(w: Workload, P_ext: int, seed: int = 1, mix: float = 0.5) -> np.ndarray:
    """[B, P_ext, D] rows standing in for the hidden states of text tokens used as pivots
    (the pivot ablation mixes 4 visual with 4 text pivots): a different distribution from
    the vision tokens -- unit-normal rows -- each blended with one vision token of its
    sample (weight `mix`) so that the vision tokens' scores against it are spread out
    rather than all near zero.  Same element type as w.X."""
    out = np.empty((w.B, P_ext, w.D), dtype=np.float32)
    for b in range(w.B):
        rng = _rng(seed, 77, b)
        rows = rng.standard_normal((P_ext, w.D)).astype(np.float32)
        n = int(w.cu[b + 1] - w.cu[b])
        if n > 0:
            pick = rng.integers(0, n, size=P_ext)
            xs = w.sample(b)[pick]
            xs = bf16_bits_to_f32(xs) if w.dtype == BF16 else xs
            rows = (1.0 - mix) * rows + mix * xs
        out[b] = rows
    return f32_to_bf16_bits(out) if w.dtype == BF16 else out


@dataclasses.dataclass
class SequenceBatch:
    """Whole sequences around the vision tokens of a Workload, packed row after row.

    H           [rows, D] hidden states: per sequence text rows, the sample's vision rows
                (bit-identical to the Workload's), text rows
    seq_cu      [B+1] int32 offsets of the sequences in H
    span_start  [B] int32 row of H where sequence b's vision tokens start
    pos         [3, rows] int64 position ids in three planes (temporal, height, width: text
                rows carry their index in all three, vision rows a grid), the layout
                multimodal rotary embeddings use
    kv          list of [rows, W] per-token tensors standing in for the cached key and value
                rows of the layers before the step (same element type as H)
    """
    H: np.ndarray
    seq_cu: np.ndarray
    span_start: np.ndarray
    pos: np.ndarray
    kv: List[np.ndarray]


def sequences_around(w: Workload, seed: int = 1, before=(3, 40), after=(0, 60), n_kv: int = 2,
                     kv_width: int = 256) -> SequenceBatch:
    """Wraps every sample of `w` in text rows: U{before} rows ahead of the vision span and
    U{after} rows behind it (unit-normal rows; a system prompt and a question)."""
    rng = _rng(seed, 88)
    pre = rng.integers(before[0], before[1] + 1, size=w.B)
    post = rng.integers(after[0], after[1] + 1, size=w.B)
    lens = w.lengths
    seq_cu = np.zeros(w.B + 1, dtype=np.int32)
    seq_cu[1:] = np.cumsum(pre + lens + post)
    rows = int(seq_cu[-1])
    text = rng.standard_normal((rows, w.D)).astype(np.float32)
    H = f32_to_bf16_bits(text) if w.dtype == BF16 else text
    span = (seq_cu[:-1] + pre).astype(np.int32)
    pos = np.zeros((3, rows), dtype=np.int64)
    for b in range(w.B):
        lo, n = int(seq_cu[b]), int(lens[b])
        H[span[b]:span[b] + n] = w.sample(b)
        T = int(seq_cu[b + 1]) - lo
        pos[:, lo:lo + T] = np.arange(T)
        side = max(1, int(np.sqrt(max(n, 1))))
        j = np.arange(n)
        pos[0, span[b]:span[b] + n] = pre[b]
        pos[1, span[b]:span[b] + n] = pre[b] + j // side
        pos[2, span[b]:span[b] + n] = pre[b] + j % side
    kv = []
    for i in range(n_kv):
        t = rng.standard_normal((rows, kv_width)).astype(np.float32)
        kv.append(f32_to_bf16_bits(t) if w.dtype == BF16 else t)
    return SequenceBatch(H, seq_cu, span, pos, kv)


def key_states(w: Workload, Dc: int, seed: int = 1, heavy: float = 0.02) -> np.ndarray:
    """[total_N, Dc] rows standing in for a layer's key states, the pivot criterion the paper
    uses (K-norm): with grouped-query attention Dc = kv_heads * head_dim is much smaller than
    the hidden size.  Unit-normal rows; a fraction `heavy` of the tokens is scaled up (the
    massive-norm tokens early decoder layers are known for), so the top of the norm ranking
    is not a near-tie.  Same element type as w.X."""
    rng = _rng(seed, 99)
    total = int(w.cu[-1])
    c = rng.standard_normal((total, Dc)).astype(np.float32)
    big = rng.random(total) < heavy
    c[big] *= rng.uniform(1.5, 4.0, size=(int(big.sum()), 1)).astype(np.float32)
    return f32_to_bf16_bits(c) if w.dtype == BF16 else c


def audio_batch(seed: int = 0xDA270005, B: int = 16, n_lo: int = 300, n_hi: int = 1500,
                D: int = 3072, P: int = 8, keep_num: int = 700, keep_den: int = 1000,
                n_centroids: int = 64, sigma: float = 0.1,
                lengths: Optional[List[int]] = None) -> Workload:
    """Audio tokens of utterances of different lengths, packed (the speech-recognition study
    prunes 20-50 % of the audio tokens with 8 pivots): runs of 3-12 consecutive frames share
    a centroid (a held sound), so neighbouring tokens duplicate each other; bf16."""
    if lengths is None:
        lengths = [int(v) for v in _rng(seed, 1 << 20).integers(n_lo, n_hi + 1, size=B)]
    rows = []
    for b, n in enumerate(lengths):
        rng = _rng(seed, b)
        cent = rng.standard_normal((n_centroids, D), dtype=np.float32)
        which = np.empty(n, dtype=np.int64)
        t = 0
        while t < n:
            run = int(rng.integers(3, 13))
            which[t:t + run] = int(rng.integers(0, n_centroids))
            t += run
        x = cent[which] + np.float32(sigma) * rng.standard_normal((n, D), dtype=np.float32)
        rows.append(x)
    return _finish("audio_batch", rows, BF16, P, 0, keep_num, keep_den, ragged=True)


def action_batch(seed: int = 0xDA270006, B: int = 32, N: int = 256, D: int = 4096, P: int = 8,
                 K: int = 56, n_centroids: int = 32, sigma: float = 0.1) -> Workload:
    """Camera frames of a vision-language-action model: 256 vision tokens kept down to 56
    (the robot-manipulation study); bf16."""
    rows = [clustered_tokens(_rng(seed, b), N, D, n_centroids, sigma) for b in range(B)]
    return _finish("action_batch", rows, BF16, P, K)


def wide_image_batch(seed: int = 0xDA270007, B: int = 16, N: int = 576, D: int = 5120,
                     P: int = 8, K: int = 128, n_centroids: int = 128,
                     sigma: float = 0.1) -> Workload:
    """576-token images at the hidden size of a 13B language model (5120); D=8192 gives the
    72B size.  bf16."""
    rows = [clustered_tokens(_rng(seed, b), N, D, n_centroids, sigma) for b in range(B)]
    return _finish("wide_image_batch", rows, BF16, P, K)


EXTRA = {"audio": audio_batch, "action": action_batch, "wide13b": wide_image_batch,
         "wide72b": lambda **kw: wide_image_batch(**{"D": 8192, "B": 8, **kw})}


def by_name(name: str, **kw) -> Workload:
    """Workloads beyond the five benchmark configurations: other modalities and model sizes
    the paper reports on."""
    return EXTRA[name](**kw)
