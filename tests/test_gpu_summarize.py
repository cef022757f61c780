"""GPU parity of the MFMA stage-1 path (bf16, head width 32) against the CPU oracle."""
import numpy as np
import pytest
import torch

from oracle import vista_oracle as O
from paper_2510_22049_amd import binding as V
from paper_2510_22049_amd import inputs as I
from tests.helpers import assert_blocks_close, block_errors, dev, host64

pytestmark = pytest.mark.gpu


def bf(x):
    return I.round_to(np.asarray(x, dtype=np.float32), "bf16")


def run(X, off, Q, Wk, Wv, H, **kw):
    B = len(off) - 1
    S, d = Q.shape[-2:]
    out = torch.full((B, S, d), float("nan"), device="cuda", dtype=torch.bfloat16)
    offd = torch.from_numpy(np.asarray(off, dtype=np.int64)).cuda()
    ws = V.vista_summarize(dev(X, "bf16"), offd, dev(Q, "bf16"), dev(Wk, "bf16"), dev(Wv, "bf16"), out, H=H, **kw)
    torch.cuda.synchronize()
    assert int(ws[:4].view(torch.int32).item()) == 0
    return host64(out)


def problem(seed, lens, d, S, per_user=False, xscale=1.0):
    g = np.random.default_rng(seed)
    off = I.offsets_from_lengths(lens)
    X = bf(g.normal(size=(off[-1], d)) * xscale)
    Q = bf(g.normal(size=(len(lens), S, d) if per_user else (S, d)))
    Wk, Wv = bf(g.normal(size=(d, d)) / np.sqrt(d)), bf(g.normal(size=(d, d)) / np.sqrt(d))
    return X, off, Q, Wk, Wv


LENS = [700, 0, 1, 31, 32, 33, 2100, 64, 0, 95, 1029]


@pytest.mark.parametrize("d,H,S", [(128, 4, 256), (128, 4, 64), (128, 4, 128), (128, 4, 512), (256, 8, 512), (256, 8, 256),
                                   (256, 8, 128), (256, 8, 64)])
@pytest.mark.parametrize("seg", [0, 64, 992])
def test_mfma_jagged_matches_oracle(d, H, S, seg):
    """Empty, single-item, one-tile, ragged and multi-segment users; shared queries."""
    X, off, Q, Wk, Wv = problem(1, LENS, d, S)
    got = run(X, off, Q, Wk, Wv, H, segment_items=seg)
    want = O.summarize(X, off, Q, Wk, Wv, H)
    assert_blocks_close(got, want, "bf16", f"d={d} S={S} seg={seg}")
    assert np.all(got[1] == 0) and np.all(got[8] == 0)


@pytest.mark.parametrize("d,H,S", [(128, 4, 256), (256, 8, 512)])
def test_mfma_per_user_queries(d, H, S):
    X, off, Q, Wk, Wv = problem(2, LENS, d, S, per_user=True)
    got = run(X, off, Q, Wk, Wv, H, segment_items=512, offsets_host=torch.from_numpy(off))
    assert_blocks_close(got, O.summarize(X, off, Q, Wk, Wv, H), "bf16", "per-user queries")


@pytest.mark.parametrize("d,H,S", [(128, 4, 256), (256, 8, 512)])
@pytest.mark.parametrize("scale", [0.03, 0.5])
def test_mfma_scale_override(d, H, S, scale):
    """A non-default score scale reaches the kernel (it is folded into the key weights)."""
    X, off, Q, Wk, Wv = problem(8, [700, 0, 33, 1300], d, S)
    got = run(X, off, Q, Wk, Wv, H, segment_items=256, scale=scale)
    want = O.summarize(X, off, Q, Wk, Wv, H, scale=scale)
    assert_blocks_close(got, want, "bf16", f"scale={scale}")
    assert block_errors(O.summarize(X, off, Q, Wk, Wv, H)[[0, 3]], want[[0, 3]]).max() > 5e-2   # the override matters


def test_mfma_large_scores_mix_both_softmax_routes():
    """Item norms straddle the bound |q||k| <= 60 (base 2): tiles switch from the constant
    reference to the running maximum inside a piece."""
    X, off, Q, Wk, Wv = problem(3, [300, 77, 1500], 128, 256, xscale=6.0)
    X[40:60] = bf(X[40:60] / 6.0)               # a stretch of small items inside a large-score user
    got = run(X, off, Q, Wk, Wv, 4, segment_items=256)
    assert_blocks_close(got, O.summarize(X, off, Q, Wk, Wv, 4), "bf16", "xscale=6")


def test_mfma_running_maximum_route_everywhere():
    """Huge key norms in channels the queries do not look at: every tile fails the norm bound
    (so the running-maximum route runs throughout) while the scores themselves stay moderate."""
    g = np.random.default_rng(31)
    d, S = 128, 256
    lens = [257, 40, 900]
    off = I.offsets_from_lengths(lens)
    X = g.normal(size=(off[-1], d))
    Q = g.normal(size=(S, d))
    for h in range(4):
        X[:, 32 * h + 16:32 * h + 32] *= 300.0
        Q[:, 32 * h + 16:32 * h + 32] = 0.0
    X[:, ::7] -= 3.0                            # shift the scores so their maximum is far from 0
    X, Q = bf(X), bf(Q)
    eye = np.eye(d, dtype=np.float32)
    Wv = bf(g.normal(size=(d, d)) / np.sqrt(d) / 50)
    got = run(X, off, Q, eye, Wv, 4, segment_items=128)
    assert_blocks_close(got, O.summarize(X, off, Q, eye, Wv, 4), "bf16", "all-general")


def test_mfma_all_scores_very_negative():
    """Every score sits near -260 (base 2) through a constant channel pair: a reference
    maximum stuck at 0 would underflow every weight to 0/0; the shift itself cancels exactly."""
    X, off, Q, Wk, Wv = problem(4, [200, 45, 1000], 128, 64)
    eye = np.eye(128, dtype=np.float32)
    for h in range(4):
        X[:, 32 * h] = 32.0
        Q[:, 32 * h] = -32.0
    got = run(X, off, Q, eye, Wv, 4, segment_items=128)
    assert_blocks_close(got, O.summarize(X, off, Q, eye, Wv, 4), "bf16", "negative scores")


@pytest.mark.parametrize("big,seg", [(11.0, 64), (11.0, 0), (16.0, 96)])
def test_mfma_beacon_rows_are_found_exactly(big, seg):
    """Indexing, bit-exact: query i is made to select one row of the user (first, last, tile
    edges, middle); the output must be that row's integer payload, exactly."""
    d, H, S = 128, 4, 64
    lens = [1, 2, 31, 32, 33, 64, 65, 0, 700, 1503, 97]
    off = I.offsets_from_lengths(lens)
    g = np.random.default_rng(5)
    X = bf(g.normal(size=(off[-1], d)))
    X[:, :32] = 0
    X[:, 16:32] = g.integers(0, 200, size=(off[-1], 16))          # payload of ordinary rows
    Q = np.zeros((S, d), np.float32)
    want = {}
    for b, L in enumerate(lens):
        picks = [p for p in (0, L - 1, 31, 32, 63, L // 2) if 0 <= p < L]
        for i, pos in enumerate((0, L - 1, 31, 32, 63, L // 2)):
            if not 0 <= pos < L:
                continue
            row = off[b] + pos
            X[row, i] = big
            X[row, 16:19] = (b + 1, pos % 256, pos // 256)
            want[(b, i)] = (b + 1, pos % 256, pos // 256)
    for i in range(6):
        Q[i, i] = big
    eye = np.eye(d, dtype=np.float32)
    got = run(X, off, bf(Q), eye, eye, H, segment_items=seg)
    for (b, i), code in want.items():
        L = lens[b]
        rows = off[b] + np.array([p for p in (0, L - 1, 31, 32, 63, L // 2) if 0 <= p < L])
        same = [r for r in rows if X[r, i] == big]
        if len(same) > 1:
            continue                                              # query i has two beacons in a tiny user
        found = got[b, i, 16:19]            # weights of the other rows are < 2^-30: far below half a unit
        assert tuple(np.rint(found)) == code and np.abs(found - code).max() < 1e-4, (b, i, found, code)


def test_mfma_is_bitwise_reproducible_and_isolated():
    """Same inputs -> same bits; poisoning one user's rows leaves the others' bits unchanged."""
    X, off, Q, Wk, Wv = problem(6, [500, 260, 1200, 33], 128, 256)
    a = run(X, off, Q, Wk, Wv, 4, segment_items=256)
    for _ in range(5):
        assert np.array_equal(a, run(X, off, Q, Wk, Wv, 4, segment_items=256))
    X2 = X.copy()
    X2[off[1]:off[2]] = bf(X2[off[1]:off[2]] * 3 + 1)
    c = run(X2, off, Q, Wk, Wv, 4, segment_items=256)
    for u in (0, 2, 3):
        assert np.array_equal(a[u], c[u])
    assert not np.array_equal(a[1], c[1])


def test_mfma_agrees_with_plain_path_on_gpu():
    """Cross-check (not the oracle): the fp32-ALU kernels on the same bf16-representable inputs."""
    X, off, Q, Wk, Wv = problem(7, [400, 90, 0, 800], 128, 256)
    got = run(X, off, Q, Wk, Wv, 4)
    out32 = torch.empty((4, 256, 128), device="cuda")
    V.vista_summarize(dev(X, "f32"), torch.from_numpy(off).cuda(), dev(Q, "f32"), dev(Wk, "f32"), dev(Wv, "f32"),
                      out32, H=4)
    torch.cuda.synchronize()
    assert block_errors(got, host64(out32)).max() < 2e-2


@pytest.mark.parametrize("d,H,S", [(128, 4, 256), (128, 4, 128), (64, 1, 16)])
def test_degenerate_batches(d, H, S):
    """No items at all (every user empty), and a batch whose only content is one item."""
    g = np.random.default_rng(21)
    Q = bf(g.normal(size=(S, d)))
    Wk, Wv = bf(g.normal(size=(d, d)) / np.sqrt(d)), bf(g.normal(size=(d, d)) / np.sqrt(d))
    got = run(np.zeros((0, d), np.float32), [0, 0, 0, 0], Q, Wk, Wv, H)
    assert got.shape == (3, S, d) and np.all(got == 0)
    X = bf(g.normal(size=(1, d)))
    got = run(X, [0, 0, 1, 1], Q, Wk, Wv, H)
    want = O.summarize(X, [0, 0, 1, 1], Q, Wk, Wv, H)
    assert np.all(got[0] == 0) and np.all(got[2] == 0)
    assert_blocks_close(got[1:2], want[1:2], "bf16", "one item")
    assert np.all(got[1] == got[1][0])          # a single item: every query returns its value row


def test_nothing_is_written_outside_out_and_the_stated_workspace():
    """Canary bytes before and after `out` and after the workspace's stated size survive the call
    (jagged users, several segments, both kernel families)."""
    for d, H, S, dtype in ((128, 4, 256, "bf16"), (64, 2, 24, "f32")):
        g = np.random.default_rng(71)
        lens = [700, 0, 33, 1300]
        off = I.offsets_from_lengths(lens)
        r = lambda shape, s=1.0: I.round_to((g.normal(size=shape) * s).astype(np.float32), dtype)
        X, Q, Wk, Wv = r((off[-1], d)), r((S, d)), r((d, d), d ** -0.5), r((d, d), d ** -0.5)
        tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
        esz = 2 if dtype == "bf16" else 4
        pad = 4096
        n_out = len(lens) * S * d * esz
        raw = torch.full((pad + n_out + pad,), 0xA5, dtype=torch.uint8, device="cuda")
        out = raw[pad:pad + n_out].view(tdt).view(len(lens), S, d)
        desc = V.summarize_desc(len(lens), S, d, H, V.VISTA_BF16 if dtype == "bf16" else V.VISTA_F32, int(off[-1]),
                                segment_items=128)
        need = V.vista_summarize_workspace_bytes(desc)
        wraw = torch.full((need + pad,), 0x5A, dtype=torch.uint8, device="cuda")
        V.vista_summarize(dev(X, dtype), torch.from_numpy(off).cuda(), dev(Q, dtype), dev(Wk, dtype), dev(Wv, dtype), out,
                          H=H, segment_items=128, workspace=wraw[:need], offsets_host=torch.from_numpy(off))
        torch.cuda.synchronize()
        assert bool((raw[:pad] == 0xA5).all()) and bool((raw[pad + n_out:] == 0xA5).all()), "write outside out"
        assert bool((wraw[need:] == 0x5A).all()), "write beyond the stated workspace size"
        assert_blocks_close(host64(out), O.summarize(X, off, Q, Wk, Wv, H), dtype, "canary case")
