"""The synthetic input recipe: determinism, ranges, and the Zipf law it claims to draw from."""

import numpy as np

from paper_1808_02621_amd import inputs


def test_deterministic_and_in_range():
    w = inputs.TINY
    a, b = inputs.sparse_ids(w), inputs.sparse_ids(w)
    assert all(np.array_equal(x, y) for x, y in zip(a, b))
    assert len(a) == w.n_workers and all(x.dtype == np.int64 and x.size == w.n_per_worker for x in a)
    assert all(x.min() >= 0 and x.max() < w.vocab for x in a)
    v = inputs.sparse_values(w)
    assert all(x.shape == (w.n_per_worker, w.dim) and x.dtype == np.float32 for x in v)
    assert not np.array_equal(v[0], v[1])
    t = inputs.table_init(w)
    assert t.shape == (w.vocab, w.dim) and abs(float(t.std()) - 0.02) < 1e-3


def test_zipf_head_probability():
    # p(1) = 1 / H(V, s); for V = 10,000, s = 1 that is 1 / 9.7876 = 0.1022
    cdf = inputs.zipf_cdf(10_000, 1.0)
    assert abs(cdf[0] - 1.0 / np.sum(1.0 / np.arange(1, 10_001))) < 1e-12
    assert abs(cdf[0] - 0.1022) < 1e-4 and cdf[-1] == 1.0
    ids = inputs.draw_ids(np.random.default_rng(0), 10_000, 1.0, 200_000)
    freq = np.bincount(ids, minlength=10_000) / ids.size
    assert abs(freq[0] - cdf[0]) < 5e-3
    assert abs(freq[1] - cdf[0] / 2) < 5e-3 and abs(freq[9] - cdf[0] / 10) < 2e-3


def test_tiny_statistics():
    w = inputs.TINY
    m, u, longest, alpha = inputs.id_statistics(inputs.sparse_ids(w), w.vocab)
    assert m == 1024 and 440 <= u <= 600 and 70 <= longest <= 150 and 0 < alpha < 0.03


def test_permuted_ids_keep_the_multiset_shape():
    w = inputs.TINY
    plain, perm = inputs.sparse_ids(w), inputs.sparse_ids(w, permute=True)
    p = inputs.id_permutation(w)
    assert np.array_equal(np.sort(p), np.arange(w.vocab))
    assert all(np.array_equal(p[a], b) for a, b in zip(plain, perm))


def test_bf16_round_trip():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 0.0, 3.140625], dtype=np.float32)
    bits = inputs.f32_to_bf16_bits(x)
    back = inputs.bf16_bits_to_f32(bits)
    # 1 + 2^-8 is a tie -> even (1.0); 1 + 3*2^-8 is a tie -> even (1 + 2^-6)
    assert back.tolist() == [1.0, 1.0, 1.015625, -2.5, 0.0, 3.140625]


def test_bf16_rounding_agrees_with_pytorch_including_nan_and_inf():
    import torch
    rng = np.random.default_rng(3)
    x = rng.standard_normal(100_000).astype(np.float32) * np.float32(10.0) ** rng.integers(-20, 20, 100_000).astype(np.float32)
    special = np.array([np.inf, -np.inf, 0.0, -0.0, 3.3895314e38, -3.3895314e38], dtype=np.float32)
    nans = np.array([0x7F800001, 0xFFFFFFFF, 0x7FC00000, 0x7F80FFFF, 0xFF800001, 0x7FFFFFFF], dtype=np.uint32).view(np.float32)
    x = np.concatenate([x, special, nans])
    bits = inputs.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    finite = ~np.isnan(x)
    assert np.array_equal(bits[finite], ref[finite])              # round to nearest even, overflow to infinity
    back = inputs.bf16_bits_to_f32(bits)
    assert np.isnan(back[~finite]).all() and not np.isnan(back[finite]).any()
    assert np.array_equal(np.signbit(back[~finite]), np.signbit(x[~finite]))
