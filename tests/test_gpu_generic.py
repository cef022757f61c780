"""GPU parity of the plain fp32-ALU path against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import vista_oracle as O
from paper_2510_22049_amd import binding as V
from paper_2510_22049_amd import inputs as I
from tests.helpers import assert_blocks_close, dev, host64, torch_dtype

pytestmark = pytest.mark.gpu


def run_summarize(X, off, Q, Wk, Wv, H, dtype, **kw):
    B = len(off) - 1
    S, d = Q.shape[-2:]
    out = torch.full((B, S, d), float("nan"), device="cuda", dtype=torch_dtype(dtype))
    offd = torch.from_numpy(np.asarray(off, dtype=np.int64)).cuda()
    ws = V.vista_summarize(dev(X, dtype), offd, dev(Q, dtype), dev(Wk, dtype), dev(Wv, dtype), out, H=H, **kw)
    torch.cuda.synchronize()
    assert int(ws[:4].view(torch.int32).item()) == 0
    return host64(out)


def run_attend(T, Y, H, dtype):
    out = torch.full(T.shape, float("nan"), device="cuda", dtype=torch_dtype(dtype))
    V.vista_target_attend(dev(T, dtype), dev(Y, dtype), out, H=H)
    torch.cuda.synchronize()
    return host64(out)


def test_config1_tiny_stage1_and_stage2():
    """1 user, L=1024, d=64, one head, S=16, fp32; then 32 candidates over the 16 summaries."""
    c = I.CONFIGS[1]
    lens = I.lengths(c)
    off = I.offsets_from_lengths(lens)
    X, Q = I.history(c, lens), I.virtual_queries(c)
    Wk, Wv = I.projection(c, "W_k"), I.projection(c, "W_v")
    got = run_summarize(X, off, Q, Wk, Wv, c.H, c.dtype)
    want = O.summarize(X, off, Q, Wk, Wv, c.H)
    assert_blocks_close(got, want, c.dtype, "config 1 stage 1")
    T = I.candidates_user(c, 0)[None]
    got2 = run_attend(T, got.astype(np.float32), c.H, c.dtype)        # stage 2 consumes the GPU summaries
    want2 = O.target_attend(T, got, c.H)
    assert_blocks_close(got2, want2, c.dtype, "config 1 stage 2")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("H,d,S", [(1, 64, 16), (4, 64, 40), (2, 96, 7)])
def test_generic_jagged_shapes(dtype, H, d, S):
    """Ragged lengths (empty, single item, across several segments), shared and per-user queries."""
    g = np.random.default_rng(7)
    lens = [300, 0, 1, 37, 64, 0, 513]
    off = I.offsets_from_lengths(lens)
    X = I.round_to(g.normal(size=(off[-1], d)).astype(np.float32), dtype)
    Wk = I.round_to((g.normal(size=(d, d)) / np.sqrt(d)).astype(np.float32), dtype)
    Wv = I.round_to((g.normal(size=(d, d)) / np.sqrt(d)).astype(np.float32), dtype)
    for per_user in (False, True):
        shape = (len(lens), S, d) if per_user else (S, d)
        Q = I.round_to(g.normal(size=shape).astype(np.float32), dtype)
        got = run_summarize(X, off, Q, Wk, Wv, H, dtype, segment_items=64)
        want = O.summarize(X, off, Q, Wk, Wv, H)
        assert_blocks_close(got, want, dtype, f"generic stage 1 per_user={per_user}")
        assert np.all(got[1] == 0) and np.all(got[5] == 0)
    T = I.round_to(g.normal(size=(3, 11, d)).astype(np.float32), dtype)
    Y = I.round_to(g.normal(size=(3, S, d)).astype(np.float32), dtype)
    assert_blocks_close(run_attend(T, Y, H, dtype), O.target_attend(T, Y, H), dtype, "generic stage 2")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_generic_scale_override(dtype):
    """A non-default score scale on the plain path, both stages."""
    g = np.random.default_rng(17)
    lens, d, S, H = [90, 0, 300], 64, 24, 2
    off = I.offsets_from_lengths(lens)
    rnd = lambda shape, s=1.0: I.round_to((g.normal(size=shape) * s).astype(np.float32), dtype)
    X, Q, Wk, Wv = rnd((off[-1], d)), rnd((S, d)), rnd((d, d), d ** -0.5), rnd((d, d), d ** -0.5)
    got = run_summarize(X, off, Q, Wk, Wv, H, dtype, scale=0.6)
    assert_blocks_close(got, O.summarize(X, off, Q, Wk, Wv, H, scale=0.6), dtype, "plain stage 1, scale 0.6")
    T, Y = rnd((2, 9, d)), rnd((2, S, d))
    out = torch.full(T.shape, float("nan"), device="cuda", dtype=torch_dtype(dtype))
    V.vista_target_attend(dev(T, dtype), dev(Y, dtype), out, H=H, scale=0.6)
    torch.cuda.synchronize()
    assert_blocks_close(host64(out), O.target_attend(T, Y, H, scale=0.6), dtype, "plain stage 2, scale 0.6")


def test_generic_exact_integer_indexing():
    """Q = 0, W_v = I, integer X: out * L_b must be the exact column sums of user b's rows."""
    lens = [7, 0, 33, 1, 64, 200, 95]
    off = I.offsets_from_lengths(lens)
    N, d = int(off[-1]), 64
    X = np.zeros((N, d), dtype=np.float32)
    X[:, 0] = 1
    X[:, 1] = np.arange(N) % 251
    X[:, 2] = np.arange(N)
    eye = np.eye(d, dtype=np.float32)
    got = run_summarize(X, off, np.zeros((4, d), np.float32), eye, eye, 2, "f32", segment_items=32)
    for b, L in enumerate(lens):
        if L == 0:
            assert np.all(got[b] == 0)
            continue
        want = X[off[b]:off[b + 1]].astype(np.float64).sum(axis=0)
        np.testing.assert_allclose(got[b] * L, np.repeat(want[None], 4, axis=0), rtol=3e-7)


def test_generic_ffn():
    g = np.random.default_rng(9)
    for dtype in ("f32", "bf16"):
        y = I.round_to(g.normal(size=(37, 64)).astype(np.float32), dtype)
        Wg = I.round_to((g.normal(size=(64, 96)) / 8).astype(np.float32), dtype)
        Wu = I.round_to((g.normal(size=(64, 96)) / 8).astype(np.float32), dtype)
        Wo = I.round_to((g.normal(size=(96, 64)) / 10).astype(np.float32), dtype)
        out = torch.full((37, 64), float("nan"), device="cuda", dtype=torch_dtype(dtype))
        V.vista_sglu_ffn(dev(y, dtype), dev(Wg, dtype), dev(Wu, dtype), dev(Wo, dtype), out)
        torch.cuda.synchronize()
        assert_blocks_close(host64(out)[None], O.sglu_ffn(y, Wg, Wu, Wo)[None], dtype, "ffn")


def test_device_side_offsets_check_reports_but_never_faults():
    d, S = 64, 16
    X = np.ones((100, d), np.float32)
    bad = torch.tensor([0, 70, 40, 100], dtype=torch.int64, device="cuda")       # decreasing
    out = torch.zeros((3, S, d), device="cuda")
    eye = np.eye(d, dtype=np.float32)
    ws = V.vista_summarize(dev(X, "f32"), bad, dev(np.zeros((S, d), np.float32), "f32"), dev(eye, "f32"),
                           dev(eye, "f32"), out, H=1)
    torch.cuda.synchronize()
    assert int(ws[:4].view(torch.int32).item()) == V.VISTA_ERR_OFFSETS
    with pytest.raises(V.VistaError):
        V.vista_summarize(dev(X, "f32"), bad, dev(np.zeros((S, d), np.float32), "f32"), dev(eye, "f32"),
                          dev(eye, "f32"), out, H=1, offsets_host=bad.cpu())
