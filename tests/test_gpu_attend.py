"""GPU parity of stage 2 (candidate attention over cached summaries) against the CPU oracle."""
import numpy as np
import pytest
import torch

from oracle import vista_oracle as O
from paper_2510_22049_amd import binding as V
from paper_2510_22049_amd import inputs as I
from tests.helpers import assert_blocks_close, block_errors, dev, floored_errors, host64

pytestmark = pytest.mark.gpu


def bf(x):
    return I.round_to(np.asarray(x, dtype=np.float32), "bf16")


def run(T, Y, H):
    out = torch.full(T.shape, float("nan"), device="cuda", dtype=torch.bfloat16)
    V.vista_target_attend(dev(T, "bf16"), dev(Y, "bf16"), out, H=H)
    torch.cuda.synchronize()
    return host64(out)


@pytest.mark.parametrize("B,C,S,d,H", [
    (3, 512, 256, 128, 4),      # serving shape, few users
    (5, 77, 256, 128, 4),       # ragged candidate tail
    (2, 1, 32, 128, 4),         # one candidate, one key block
    (4, 33, 96, 128, 4),        # S = 3 key blocks
    (3, 100, 128, 256, 8),      # 8 heads = two head groups
    (2, 64, 512, 256, 8),       # S = 512: sixteen key blocks, the whole of LDS
    (3, 200, 512, 128, 4),      # S = 512, several rounds with a ragged tail
    (2, 130, 320, 128, 4),      # S = 10 key blocks
    (2, 50, 288, 128, 4),       # S = 9 key blocks goes down the plain path
    (2, 100, 64, 64, 2),        # a single pair of heads
    (3, 70, 128, 192, 6),       # three head pairs
    (1, 640, 256, 128, 4),      # one user, ten rounds: several workgroups share the user
])
def test_attend_matches_oracle(B, C, S, d, H):
    g = np.random.default_rng(B * 1000 + C)
    T, Y = bf(g.normal(size=(B, C, d))), bf(g.normal(size=(B, S, d)))
    assert_blocks_close(run(T, Y, H), O.target_attend(T, Y, H), "bf16", f"B={B} C={C} S={S} d={d}")


def test_attend_large_scores_take_the_true_maximum():
    """Norms beyond the bound |q||k| <= 60 (base 2) in channels that the other side zeroes:
    the maximum-first route runs, and a constant shift of -260 must cancel exactly."""
    g = np.random.default_rng(11)
    B, C, S, d, H = 2, 70, 256, 128, 4
    T, Y = g.normal(size=(B, C, d)), g.normal(size=(B, S, d))
    for h in range(H):
        T[:, :, 32 * h] = -32.0
        Y[:, :, 32 * h] = 32.0
    T, Y = bf(T), bf(Y)
    assert_blocks_close(run(T, Y, H), O.target_attend(T, Y, H), "bf16", "shifted scores")


@pytest.mark.parametrize("S,nbits,payload_max", [(256, 8, 200), (32, 5, 3), (512, 9, 200), (512, 9, 3)])
def test_attend_selects_the_matching_summary_exactly(S, nbits, payload_max):
    """Indexing, bit-exact: candidate c points at summary token (7c+3+h) mod S through a +-6 code
    of the token index (one differing bit costs 18 bits of weight); the output must be that
    token's integer payload.  Large payloads push |k| over the norm bound (maximum-first
    route), the small-S case stays on the constant-reference route."""
    B, C, d, H = 2, 150, 128, 4
    g = np.random.default_rng(12)
    Y = np.zeros((B, S, d), np.float32)
    T = np.zeros((B, C, d), np.float32)
    bits = ((np.arange(S)[:, None] >> np.arange(nbits)[None]) & 1) * 2 - 1
    for h in range(H):
        Y[:, :, 32 * h:32 * h + nbits] = 6.0 * bits
        Y[:, :, 32 * h + 16:32 * h + 32] = g.integers(0, payload_max, size=(B, S, 16))
        pick = (7 * np.arange(C) + 3 + h) % S
        T[:, :, 32 * h:32 * h + nbits] = 6.0 * bits[pick]
    got = run(bf(T), bf(Y), H)
    for h in range(H):
        pick = (7 * np.arange(C) + 3 + h) % S
        want = Y[:, pick, 32 * h + 16:32 * h + 32]
        found = got[:, :, 32 * h + 16:32 * h + 32]
        assert np.array_equal(np.rint(found), want) and np.abs(found - want).max() < 2e-2


def test_candidates_do_not_see_each_other_on_gpu():
    """Changing one candidate changes only its own output row, bit for bit."""
    g = np.random.default_rng(13)
    T, Y = bf(g.normal(size=(2, 96, 128))), bf(g.normal(size=(2, 256, 128)))
    a = run(T, Y, 4)
    T2 = T.copy()
    T2[1, 40] = bf(T2[1, 40] * 2 + 1)
    b = run(T2, Y, 4)
    mask = np.ones((2, 96), bool)
    mask[1, 40] = False
    assert np.array_equal(a[mask], b[mask]) and not np.array_equal(a[1, 40], b[1, 40])


def test_config4_all_users():
    """Serving workload at its full launch shape (1024 users x 512 candidates): every user's
    block against the oracle, which is fed with the host copy of the very tensors the kernel read."""
    c = I.CONFIGS[4]
    g = torch.Generator(device="cuda")
    g.manual_seed(4)
    T = torch.randn((c.B, c.C, c.d), device="cuda", generator=g).to(torch.bfloat16)
    Y = torch.randn((c.B, c.S, c.d), device="cuda", generator=g).to(torch.bfloat16)
    for u in (0, 1, 511, 1023):                      # a few users carry the seeded host streams
        T[u] = dev(I.candidates_user(c, u), "bf16")
        Y[u] = dev(I.summaries_user(c, u), "bf16")
    out = torch.full((c.B, c.C, c.d), float("nan"), device="cuda", dtype=torch.bfloat16)
    V.vista_target_attend(T, Y, out, H=c.H)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out.float()).all())
    got, Th, Yh = host64(out), host64(T), host64(Y)
    worst = 0.0
    for b0 in range(0, c.B, 128):
        want = O.target_attend(Th[b0:b0 + 128], Yh[b0:b0 + 128], c.H)
        worst = max(worst, assert_blocks_close(got[b0:b0 + 128], want, "bf16", f"config 4 users {b0}.."))
        if b0 == 0:
            print(f"config 4: floored element-wise error of users 0..127 {floored_errors(got[:128], want).max():.2e}")
    print(f"config 4: worst block error over all {c.B} users {worst:.2e}", flush=True)


@pytest.mark.parametrize("scale", [0.05, 0.4])
def test_attend_scale_override(scale):
    """A non-default score scale (MFMA path: folded into the key operand; plain path: S = 288)."""
    g = np.random.default_rng(41)
    for (B, C, S, d, H) in ((2, 130, 256, 128, 4), (2, 40, 288, 128, 4)):
        T, Y = bf(g.normal(size=(B, C, d))), bf(g.normal(size=(B, S, d)))
        out = torch.full(T.shape, float("nan"), device="cuda", dtype=torch.bfloat16)
        V.vista_target_attend(dev(T, "bf16"), dev(Y, "bf16"), out, H=H, scale=scale)
        torch.cuda.synchronize()
        want = O.target_attend(T, Y, H, scale=scale)
        assert_blocks_close(host64(out), want, "bf16", f"scale={scale} S={S}")
        # the override must matter: the default-scale result is a different one
        assert block_errors(O.target_attend(T, Y, H), want).max() > 5e-2
