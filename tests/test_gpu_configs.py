"""The five workload configurations at their full launch shapes, checked against the CPU oracle.

Where the full oracle would take minutes, it is evaluated on outputs it can compute one by
one: a sample of the query rows (each query's softmax is independent of the others) or a
sample of users; finiteness is checked on everything."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

from oracle import vista_oracle as O
from paper_2510_22049_amd import binding as V
from paper_2510_22049_amd import inputs as I
from tests.helpers import assert_blocks_close, assert_in_value_hull, dev, host64

pytestmark = pytest.mark.gpu


def history_on_device(c, lens):
    """Packed bf16 history [N, d] built user by user from the seeded host streams."""
    off = I.offsets_from_lengths(lens)
    X = torch.empty((int(off[-1]), c.d), device="cuda", dtype=torch.bfloat16)

    def one(b):
        bits = I.to_bf16_bits(I.history_user(c, b, int(lens[b])))
        return b, torch.from_numpy(bits.view(np.int16))

    with ThreadPoolExecutor(max_workers=8) as ex:
        for b, t in ex.map(one, range(len(lens))):
            X[off[b]:off[b + 1]] = t.cuda().view(torch.bfloat16)
    return X, off


def assert_summaries_in_hull(out, X, off, Wv, what):
    """Every user, any size: a summary channel lies inside the range of that channel of the user's
    values X_b W_v (formed here with a library matmul in fp32)."""
    W = Wv.float()
    for b in range(len(off) - 1):
        if off[b + 1] > off[b]:
            assert_in_value_hull(out[b], X[off[b]:off[b + 1]].float() @ W, f"{what} user {b}")


def summarize(X, off, Q, Wk, Wv, H):
    B = len(off) - 1
    S, d = Q.shape[-2:]
    out = torch.full((B, S, d), float("nan"), device="cuda", dtype=torch.bfloat16)
    ws = V.vista_summarize(X, torch.from_numpy(off).cuda(), Q, Wk, Wv, out, H=H, offsets_host=torch.from_numpy(off))
    torch.cuda.synchronize()
    assert int(ws[:4].view(torch.int32).item()) == 0
    assert bool(torch.isfinite(out.float()).all())
    return out


def test_config2_jagged_batch_all_users():
    """64 users, lognormal lengths (median 8k, [1k, 100k]), d=128, 4 heads, S=256, bf16: every output."""
    c = I.CONFIGS[2]
    lens = I.lengths(c)
    X, off = history_on_device(c, lens)
    Q, Wk, Wv = I.virtual_queries(c), I.projection(c, "W_k"), I.projection(c, "W_v")
    out = summarize(X, off, dev(Q, "bf16"), dev(Wk, "bf16"), dev(Wv, "bf16"), c.H)
    assert_summaries_in_hull(out, X, off, dev(Wv, "bf16"), "config 2")
    got = host64(out)
    want = np.zeros_like(got)
    for b in range(c.B):
        Xb = I.history_user(c, b, int(lens[b]))
        want[b] = O.summarize(Xb, [0, len(Xb)], Q, Wk, Wv, c.H)[0]
    err = assert_blocks_close(got, want, "bf16", "config 2")
    print(f"config 2: N={off[-1]} max block error {err:.2e}")


def test_config3_lifelong_sampled_queries():
    """8 users x 1,000,000 items (split over ~1000 segments): 16 sampled query rows per user."""
    c = I.CONFIGS[3]
    lens = I.lengths(c)
    X, off = history_on_device(c, lens)
    Q, Wk, Wv = I.virtual_queries(c), I.projection(c, "W_k"), I.projection(c, "W_v")
    out = summarize(X, off, dev(Q, "bf16"), dev(Wk, "bf16"), dev(Wv, "bf16"), c.H)
    assert_summaries_in_hull(out, X, off, dev(Wv, "bf16"), "config 3")
    rows = np.array([0, 1, 31, 32, 63, 64, 100, 127, 128, 129, 191, 200, 222, 254, 255, 77])
    got = host64(out[:, torch.from_numpy(rows).cuda()])
    for b in (0, 3, 7):
        Xb = I.history_user(c, b, int(lens[b]))
        want = O.summarize(Xb, [0, len(Xb)], Q[rows], Wk, Wv, c.H)
        assert_blocks_close(got[b:b + 1], want, "bf16", f"config 3 user {b}")


def test_config5_end_to_end_sampled_users():
    """256 users, lengths U[10k, 100k], two stacked layers (d=256, 8 heads, S=512) with the gated
    block between, then 256 candidates per user.  Each call is checked against the oracle fed
    with the GPU's (bf16) inputs of that call, for the shortest, the longest and two more users."""
    c = I.CONFIGS[5]
    lens = I.lengths(c)
    X, off = history_on_device(c, lens)
    Q0 = I.virtual_queries(c)
    W = {k: I.projection(c, k[:3], int(k[3])) for k in ("W_k0", "W_v0", "W_k1", "W_v1")}
    Wg, Wu, Wo = I.ffn_weights(c)
    y1 = summarize(X, off, dev(Q0, "bf16"), dev(W["W_k0"], "bf16"), dev(W["W_v0"], "bf16"), c.H)
    q1 = torch.full_like(y1, float("nan"))
    V.vista_sglu_ffn(y1, dev(Wg, "bf16"), dev(Wu, "bf16"), dev(Wo, "bf16"), q1)
    y2 = summarize(X, off, q1, dev(W["W_k1"], "bf16"), dev(W["W_v1"], "bf16"), c.H)
    cand = torch.empty((c.B, c.C, c.d), device="cuda", dtype=torch.bfloat16)
    users = sorted({int(np.argmin(lens)), int(np.argmax(lens)), 17, 255})
    g = torch.Generator(device="cuda")
    g.manual_seed(5)
    cand.copy_(torch.randn((c.B, c.C, c.d), device="cuda", generator=g))
    for u in users:
        cand[u] = dev(I.candidates_user(c, u), "bf16")
    out = torch.full((c.B, c.C, c.d), float("nan"), device="cuda", dtype=torch.bfloat16)
    V.vista_target_attend(cand, y2, out, H=c.H)
    torch.cuda.synchronize()
    for t in (q1, out):
        assert bool(torch.isfinite(t.float()).all())
    assert_summaries_in_hull(y1, X, off, dev(W["W_v0"], "bf16"), "config 5 layer 1")      # all 256 users
    assert_summaries_in_hull(y2, X, off, dev(W["W_v1"], "bf16"), "config 5 layer 2")
    assert_in_value_hull(out, y2, "config 5 stage 2")
    rows = np.arange(0, c.S, 16)                       # 32 sampled query rows of each layer
    for u in users:
        Xu = I.history_user(c, u, int(lens[u]))
        w1 = O.summarize(Xu, [0, len(Xu)], Q0[rows], W["W_k0"], W["W_v0"], c.H)
        assert_blocks_close(host64(y1[u, rows])[None], w1, "bf16", f"config 5 layer 1 user {u}")
        wq = O.sglu_ffn(host64(y1[u]), Wg, Wu, Wo)
        assert_blocks_close(host64(q1[u])[None], wq[None], "bf16", f"config 5 gated block user {u}")
        w2 = O.summarize(Xu, [0, len(Xu)], host64(q1[u, rows]), W["W_k1"], W["W_v1"], c.H)
        assert_blocks_close(host64(y2[u, rows])[None], w2, "bf16", f"config 5 layer 2 user {u}")
        w3 = O.target_attend(host64(cand[u])[None], host64(y2[u])[None], c.H)
        assert_blocks_close(host64(out[u])[None], w3, "bf16", f"config 5 stage 2 user {u}")
