"""The seeded input generators: determinism, shapes, dtype rounding."""
import numpy as np
import torch

from paper_2510_22049_amd import inputs as I


def test_bf16_rounding_matches_torch():
    x = np.random.default_rng(0).normal(size=4096).astype(np.float32)
    x[:4] = [1.00390625, 1.01171875, -0.0, 3.0e38]     # two ties, signed zero, near max
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(I.round_to(x, "bf16"), want)
    assert np.array_equal(I.from_bf16_bits(I.to_bf16_bits(want)), want)


def test_lengths_follow_the_stated_rules():
    l2 = I.lengths(I.CONFIGS[2])
    assert l2.shape == (64,) and l2.min() >= 1000 and l2.max() <= 100000
    assert 4000 < np.median(l2) < 16000
    l5 = I.lengths(I.CONFIGS[5])
    assert l5.shape == (256,) and l5.min() >= 10000 and l5.max() <= 100000
    assert np.all(I.lengths(I.CONFIGS[3]) == 1_000_000)
    off = I.offsets_from_lengths(l2)
    assert off[0] == 0 and off[-1] == l2.sum() and off.dtype == np.int64


def test_streams_are_reproducible_and_distinct():
    c = I.CONFIGS[2]
    a, b = I.history_user(c, 3, 50), I.history_user(c, 3, 50)
    assert np.array_equal(a, b)
    assert not np.array_equal(a, I.history_user(c, 4, 50))
    assert np.array_equal(I.round_to(a, "bf16"), a)                 # already bf16-representable
    assert abs(I.projection(c, "W_k").std() - 128 ** -0.5) < 0.01
    assert not np.array_equal(I.projection(c, "W_k"), I.projection(c, "W_v"))
    X = I.history(c, [5, 0, 7])
    assert X.shape == (12, 128) and np.array_equal(X[5:], I.history_user(c, 2, 7))
