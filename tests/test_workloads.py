"""The seeded input generators: shapes, determinism and the structure they promise."""
import numpy as np

from paper_1810_07354_amd import workloads as wl


def test_k_of_fraction_is_a_ceiling():
    assert wl.k_of_fraction(0.25, 1000) == 250
    assert wl.k_of_fraction(0.10, 165_000) == 16_500
    assert wl.k_of_fraction(0.05, 100_000) == 5_000
    assert [wl.k_of_fraction(r, 6104) for r in (0.01, 0.10, 0.50)] == [62, 611, 3052]
    assert wl.k_of_fraction(0.10, 1 << 20) == 104_858
    assert wl.k_of_fraction(1.0, 7) == 7


def test_bf16_rounding_is_nearest_even():
    f = np.array([1.0, 1.00390625, 1.01171875, -2.5, 0.0, np.inf], dtype=np.float32)
    # 1.00390625 = 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7 -> even (1.0);
    # 1.01171875 = 1 + 3*2^-8 is a tie between 1+2^-7 (odd) and 1+2^-6 (even) -> 1+2^-6
    b = wl.f32_to_bf16_bits(f)
    back = wl.bf16_bits_to_f32(b)
    np.testing.assert_array_equal(back, np.array([1.0, 1.0, 1.015625, -2.5, 0.0, np.inf], dtype=np.float32))
    r = np.random.default_rng(0).normal(size=10000).astype(np.float32)
    err = np.abs(wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(r)).astype(np.float64) - r)
    assert np.all(err <= np.abs(r) * 2.0 ** -8)
    assert np.isnan(wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(np.array([np.nan], dtype=np.float32))))[0]


def test_mlr_like_full_shape_and_determinism():
    a, b = wl.mlr_like(), wl.mlr_like()
    assert a.n_elems == 784_000 and a.block_len == 784 and a.n_blocks == 1000
    assert a.k == 250 and a.lost.size == 500 and a.dtype == wl.F32
    np.testing.assert_array_equal(a.x, b.x)
    np.testing.assert_array_equal(a.lost, b.lost)
    assert np.all(np.diff(a.lost.astype(np.int64)) > 0)
    assert abs(float(a.c.std()) - 0.1) < 0.002
    assert not np.array_equal(a.x, wl.mlr_like(seed=5).x)


def test_mf_like_small_has_a_heavy_tailed_row_scale():
    w = wl.mf_like(u_rows=4000, v_rows=1000, rank=100)
    assert w.n_blocks == 5000 and w.k == 500 and w.lost.size == 1000
    np.testing.assert_array_equal(w.lost, np.arange(1000))
    d = (w.x.astype(np.float64) - w.c).reshape(5000, 100)
    rms = np.sqrt((d * d).mean(axis=1))
    assert rms.max() / np.median(rms) > 100


def test_lda_like_small_preserves_row_sums_and_moves_few_entries():
    w = wl.lda_like(words=2000, topics=100)
    x, c = w.x.reshape(2000, 100), w.c.reshape(2000, 100)
    assert w.dtype == wl.I32 and x.dtype == np.int32
    np.testing.assert_array_equal(x.sum(1, dtype=np.int64), c.sum(1, dtype=np.int64))
    assert x.min() >= 0
    frac = np.mean(x != c)
    assert 0.002 < frac < 0.04
    assert w.k == 100 and w.lost.size == 250


def test_cnn_like_small_has_a_ragged_tail():
    w = wl.cnn_like(n_elems=100_000, block_len=4096, fraction=0.5)
    assert w.n_blocks == 25 and w.n_elems % 4096 == 1696
    assert w.k == 13 and 3 <= w.lost.size <= 6
    assert len(set(w.lost.tolist())) == w.lost.size


def test_flat_like_small_and_bf16_copy():
    w = wl.flat_like(n_elems=1 << 16)
    assert w.n_blocks == 64 and w.k == 7 and w.lost.size == 8
    d = (w.x.astype(np.float64) - w.c) / 1e-3
    assert 1.2 < d.std() < 3.0 and np.abs(d).max() > 8       # heavy tails
    h = wl.flat_like(n_elems=1 << 16, dtype=wl.BF16)
    assert h.x.dtype == np.uint16
    np.testing.assert_array_equal(h.x, wl.f32_to_bf16_bits(w.x))


def test_flat_like_torch_cpu_is_seeded():
    import torch
    x1, c1 = wl.flat_like_torch("cpu", n_elems=1 << 14, chunk=1 << 12)
    x2, c2 = wl.flat_like_torch("cpu", n_elems=1 << 14, chunk=1 << 12)
    assert torch.equal(x1, x2) and torch.equal(c1, c2)
    assert abs(float(c1.std()) - 0.02) < 0.002
    x0 = x1.clone()
    wl.drift_torch(x1, seed=7, fraction=0.25, block_len=1024)
    changed = (x1 != x0).reshape(16, 1024).any(dim=1)
    assert int(changed.sum()) == 4


def test_by_layer_generators():
    w = wl.layers_like()
    assert w.n_blocks == 10 and int(w.offsets[-1]) == w.x.size == sum(wl.CNN_LAYER_SIZES)
    assert w.k == 3 and w.lost.size == 3
    sizes = wl.mixed_layer_sizes(200, 6_000_000)
    assert sizes.size == 200 and (sizes == 0).sum() >= 1 and sizes.max() > 1000 * max(1, np.median(sizes)) / 50
    assert 0.5 * 6_000_000 < sizes.sum() < 1.1 * 6_000_000
    v = wl.layers_like(sizes, seed=9, dtype=wl.I32)
    assert v.x.dtype == np.int32 and np.all(np.diff(v.offsets.astype(np.int64)) == sizes)


def test_doc_topic_rows_are_distributions_with_lengths():
    w = wl.doc_topic_like(docs=300, topics=20)
    x, c = w.x.reshape(-1, 20), w.c.reshape(-1, 20)
    np.testing.assert_allclose(x.sum(1), 1.0, atol=1e-5)
    np.testing.assert_allclose(c.sum(1), 1.0, atol=1e-5)
    assert np.all(x >= 0) and np.all(c >= 0)
    n = w.extra["lengths"]
    assert n.dtype == np.float32 and n.shape == (300,) and np.all(n >= 5)
    # rows are whole token counts over the document's length
    np.testing.assert_allclose(c * n[:, None], np.round(c * n[:, None]), atol=1e-3)
    assert np.any(x != c) and w.k == 38 and w.lost.size == 75
    w2 = wl.doc_topic_like(docs=300, topics=20)
    np.testing.assert_array_equal(w.x, w2.x)
