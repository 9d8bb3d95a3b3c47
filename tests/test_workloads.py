"""The synthetic input generators: deterministic, and shaped as documented."""
import numpy as np

from paper_2502_11494_amd import workloads as W


def test_bf16_rounding_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 0.0, 3.140625], dtype=np.float32)
    # 1.00390625 = 1 + 2^-8 is a tie between 1.0 and 1.0078125 -> even mantissa (1.0);
    # 1.01171875 = 1 + 3*2^-8 is a tie between 1.0078125 and 1.015625 -> even (1.015625)
    got = W.bf16_bits_to_f32(W.f32_to_bf16_bits(x))
    np.testing.assert_array_equal(got, np.array([1.0, 1.0, 1.015625, -2.5, 0.0, 3.140625],
                                                dtype=np.float32))


def test_generators_are_deterministic_and_shaped():
    a = W.multicrop_batch(B=2, N=200, D=64, P=4, K=20, n_centroids=16)
    b = W.multicrop_batch(B=2, N=200, D=64, P=4, K=20, n_centroids=16)
    np.testing.assert_array_equal(a.X, b.X)
    assert a.X.shape == (400, 64) and a.X.dtype == np.uint16
    np.testing.assert_array_equal(a.cu, [0, 200, 400])
    np.testing.assert_array_equal(a.pos[:3], [0, 1, 2])
    assert a.pos[200] == 0
    # a tenth of the rows are exact copies of other rows
    for s in range(2):
        uniq = np.unique(a.sample(s), axis=0).shape[0]
        assert uniq <= 200 - 20 + 1 and uniq >= 200 - 20 - 2
    c = W.multicrop_batch(seed=1, B=2, N=200, D=64, P=4, K=20, n_centroids=16)
    assert not np.array_equal(a.X, c.X)


def test_ragged_budget_rule():
    w = W.ragged_batch(B=5, n_lo=100, n_hi=400, D=32, P=4)
    assert w.ragged and w.K == 0
    lens = w.lengths
    assert lens.min() >= 100 and lens.max() <= 400 and len(set(lens.tolist())) > 1
    for b in range(5):
        assert w.budget(b) == (int(lens[b]) * 111) // 1000
    w2 = W.ragged_batch(D=32, lengths=[1024, 16384])
    assert (w2.budget(0), w2.budget(1)) == (113, 1818)


def test_video_frames_drift_slowly():
    w = W.video_batch(B=1, frames=6, per_frame=10, D=256, P=2, K=8, n_centroids=3)
    x = W.bf16_bits_to_f32(w.X).astype(np.float64)
    f0, f1, f5 = x[:10], x[10:20], x[50:60]
    cos = lambda a, b: (a * b).sum(1) / np.linalg.norm(a, axis=1) / np.linalg.norm(b, axis=1)
    assert np.all(cos(f0, f1) > 0.995) and np.all(cos(f0, f5) > 0.98)
    assert np.all(cos(f0, f5) < cos(f0, f1))


def test_full_size_shapes_of_the_headline_configuration():
    w = W.by_index(2, B=1)
    assert (w.X.shape, w.P, w.K, w.dtype) == ((2880, 4096), 16, 320, W.BF16)


def test_text_pivot_rows_are_seeded_and_typed():
    w = W.image_batch(B=2, N=100, D=64, P=8, K=20, n_centroids=8)
    a, b = W.text_pivot_rows(w, 4, seed=3), W.text_pivot_rows(w, 4, seed=3)
    assert a.shape == (2, 4, 64) and a.dtype == w.X.dtype
    np.testing.assert_array_equal(a, b)
    assert not np.array_equal(a, W.text_pivot_rows(w, 4, seed=4))
    assert not np.array_equal(a[0], a[1])
