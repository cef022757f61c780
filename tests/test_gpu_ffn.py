"""GPU parity of the SiLU-gated block (matrix-core path for d = 128 / 256, bf16) against the CPU oracle."""
import numpy as np
import pytest
import torch

from oracle import vista_oracle as O
from paper_2510_22049_amd import binding as V
from paper_2510_22049_amd import inputs as I
from tests.helpers import assert_blocks_close, dev, host64

pytestmark = pytest.mark.gpu


def bf(x):
    return I.round_to(np.asarray(x, dtype=np.float32), "bf16")


def run(y, Wg, Wu, Wo, eps=None):
    out = torch.full(y.shape, float("nan"), device="cuda", dtype=torch.bfloat16)
    kw = {} if eps is None else {"eps": eps}
    V.vista_sglu_ffn(dev(y, "bf16"), dev(Wg, "bf16"), dev(Wu, "bf16"), dev(Wo, "bf16"), out, **kw)
    torch.cuda.synchronize()
    return host64(out)


def weights(g, d, d_ff):
    return (bf(g.normal(size=(d, d_ff)) / np.sqrt(d)), bf(g.normal(size=(d, d_ff)) / np.sqrt(d)),
            bf(g.normal(size=(d_ff, d)) / np.sqrt(d_ff)))


@pytest.mark.parametrize("rows,d,d_ff", [
    (512, 256, 512),     # the end-to-end configuration's widths, whole workgroups
    (1000, 256, 512),    # ragged last workgroup
    (33, 256, 64),       # two hidden steps, one row into the second wave
    (1, 128, 32),        # a single row, a single hidden step
    (300, 128, 256),
    (129, 128, 160),     # hidden width not a multiple of 64
])
def test_ffn_matches_oracle(rows, d, d_ff):
    g = np.random.default_rng(rows + d_ff)
    y = bf(g.normal(size=(rows, d)) * g.uniform(0.2, 3.0, size=(rows, 1)))    # rows of different norms
    Wg, Wu, Wo = weights(g, d, d_ff)
    got, want = run(y, Wg, Wu, Wo), O.sglu_ffn(y, Wg, Wu, Wo)
    blocks = [slice(i, min(i + 128, rows)) for i in range(0, rows, 128)]
    for b in blocks:
        assert_blocks_close(got[b][None], want[b][None], "bf16", f"rows {b.start}..{b.stop} d={d} d_ff={d_ff}")


def test_ffn_routes_every_index_to_its_place():
    """Indexing, exact: with W_u = 0 except one 1 per hidden unit and W_o a permutation, and a gate
    that is the constant SiLU(8) on every hidden unit, out[m][perm[f]] = SiLU(8 r) * r * y[m][src[f]]
    for small integers y; ratios between outputs of a row are then exact small-integer ratios."""
    rows, d, d_ff = 70, 256, 256
    g = np.random.default_rng(5)
    y = np.zeros((rows, d), np.float32)
    y[:, 1:] = g.integers(1, 4, size=(rows, d - 1))
    y[:, 0] = 16.0                                     # the gate reads only channel 0
    src = g.permutation(np.arange(1, d))[:d_ff - 1]
    src = np.concatenate([src, src[:1]])
    perm = g.permutation(d)[:d_ff]
    Wg = np.zeros((d, d_ff), np.float32); Wg[0, :] = 0.5
    Wu = np.zeros((d, d_ff), np.float32); Wu[src, np.arange(d_ff)] = 1.0
    Wo = np.zeros((d_ff, d), np.float32); Wo[np.arange(d_ff), perm] = 1.0
    got = run(bf(y), bf(Wg), bf(Wu), bf(Wo))
    want = O.sglu_ffn(bf(y), bf(Wg), bf(Wu), bf(Wo))
    assert_blocks_close(got[None], want[None], "bf16", "routing")
    untouched = np.setdiff1d(np.arange(d), perm)
    assert np.all(got[:, untouched] == 0.0)
    # the same source value must give bit-identical outputs wherever it is routed
    for m in (0, 31, 32, 69):
        vals = {}
        for f in range(d_ff):
            vals.setdefault(float(y[m, src[f]]), set()).add(float(got[m, perm[f]]))
        assert all(len(v) == 1 for v in vals.values())


def test_ffn_is_row_independent_and_scale_invariant_without_eps():
    g = np.random.default_rng(6)
    rows, d, d_ff = 200, 256, 128
    y = bf(g.normal(size=(rows, d)))
    Wg, Wu, Wo = weights(g, d, d_ff)
    a = run(y, Wg, Wu, Wo, eps=1e-30)
    b = run(bf(4.0 * y), Wg, Wu, Wo, eps=1e-30)            # a power of two: exact in bf16
    assert np.array_equal(a, b)
    c = run(y[37:38], Wg, Wu, Wo, eps=1e-30)               # one row on its own
    assert np.array_equal(c[0], a[37])
