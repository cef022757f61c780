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
from tests.helpers import assert_blocks_close, assert_in_value_hull, dev, floored_errors, host64

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
    print(f"config 2: N={off[-1]} max block error {err:.2e}, floored element-wise {floored_errors(got, want).max():.2e}",
          flush=True)


def spread_rows(S, per_block):
    """Sampled query rows: `per_block` rows of every block of 32 queries, at positions that move from
    block to block, so every wave slot and both half-wave positions of the kernels are hit."""
    rows = []
    for k in range(S // 32):
        picks = {0, 31} if per_block >= 4 else set()
        j = 0
        while len(picks) < per_block:
            picks.add((5 * k + 7 + 11 * j) % 32)
            j += 1
        rows += [32 * k + r for r in sorted(picks)]
    return np.array(rows)


def test_config3_lifelong_all_users_sampled_queries():
    """8 users x 1,000,000 items (split over ~1000 segments): all eight users, 32 query rows each
    (four of every block of 32 queries; each query's softmax is independent of the others)."""
    c = I.CONFIGS[3]
    lens = I.lengths(c)
    X, off = history_on_device(c, lens)
    Q, Wk, Wv = I.virtual_queries(c), I.projection(c, "W_k"), I.projection(c, "W_v")
    out = summarize(X, off, dev(Q, "bf16"), dev(Wk, "bf16"), dev(Wv, "bf16"), c.H)
    assert_summaries_in_hull(out, X, off, dev(Wv, "bf16"), "config 3")
    rows = spread_rows(c.S, 4)
    assert len(rows) == 32
    got = host64(out[:, torch.from_numpy(rows).cuda()])
    for b in range(c.B):
        Xb = I.history_user(c, b, int(lens[b]))
        want = O.summarize(Xb, [0, len(Xb)], Q[rows], Wk, Wv, c.H)
        err = assert_blocks_close(got[b:b + 1], want, "bf16", f"config 3 user {b}")
        print(f"config 3 user {b}: block error {err:.2e}, floored element-wise {floored_errors(got[b:b + 1], want)[0]:.2e}",
              flush=True)


@pytest.mark.parametrize("form", ["silu", "qla"])
def test_config3_lifelong_further_forms(form):
    """The lifelong shape (8 x 1,000,000 items, ~1000 segments per call) through the SiLU score
    form and through quasi-linear attention: the first, a middle and the last user, 32 query rows
    each (every output row of both forms depends on its own query only)."""
    c = I.CONFIGS[3]
    lens = I.lengths(c)
    X, off = history_on_device(c, lens)
    Q, Wk, Wv = I.virtual_queries(c), I.projection(c, "W_k"), I.projection(c, "W_v")
    attn = V.VISTA_ATTN_SILU if form == "silu" else V.VISTA_ATTN_QLA
    out = torch.full((c.B, c.S, c.d), float("nan"), device="cuda", dtype=torch.bfloat16)
    ws = V.vista_summarize(X, torch.from_numpy(off).cuda(), dev(Q, "bf16"), dev(Wk, "bf16"), dev(Wv, "bf16"), out,
                           H=c.H, offsets_host=torch.from_numpy(off), attn=attn)
    torch.cuda.synchronize()
    assert int(ws[:4].view(torch.int32).item()) == 0
    assert bool(torch.isfinite(out.float()).all())
    rows = spread_rows(c.S, 4)
    got = host64(out[:, torch.from_numpy(rows).cuda()])
    oracle = O.summarize_silu if form == "silu" else O.summarize_qla
    for b in (0, 3, c.B - 1):
        Xb = I.history_user(c, b, int(lens[b]))
        want = oracle(Xb, [0, len(Xb)], Q[rows], Wk, Wv, c.H)
        err = assert_blocks_close(got[b:b + 1], want, "bf16", f"config 3 {form} user {b}")
        print(f"config 3 {form} user {b}: block error {err:.2e}", flush=True)


def test_config5_end_to_end_sampled_users():
    """256 users, lengths U[10k, 100k], two stacked layers (d=256, 8 heads, S=512) with the gated
    block between, then 256 candidates per user.  Every call of the chain is checked against the
    oracle fed with the GPU's (bf16) inputs of that call, for the shortest and the longest user and
    eight seeded picks (48 query rows of each layer: three of every block of 32)."""
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
    picks = I.stream(c.index, "parity_users").choice(c.B, size=8, replace=False)
    users = sorted({int(np.argmin(lens)), int(np.argmax(lens)), *map(int, picks)})
    assert len(users) >= 8
    g = torch.Generator(device="cuda")
    g.manual_seed(5)
    cand = torch.randn((c.B, c.C, c.d), device="cuda", generator=g).to(torch.bfloat16)
    out = torch.full((c.B, c.C, c.d), float("nan"), device="cuda", dtype=torch.bfloat16)
    V.vista_target_attend(cand, y2, out, H=c.H)
    torch.cuda.synchronize()
    for t in (q1, out):
        assert bool(torch.isfinite(t.float()).all())
    assert_summaries_in_hull(y1, X, off, dev(W["W_v0"], "bf16"), "config 5 layer 1")      # all 256 users
    assert_summaries_in_hull(y2, X, off, dev(W["W_v1"], "bf16"), "config 5 layer 2")
    assert_in_value_hull(out, y2, "config 5 stage 2")
    # stage 2 and the gated block: every one of the 256 users against the oracle
    want3 = O.target_attend(host64(cand), host64(y2), c.H)
    e3 = assert_blocks_close(host64(out), want3, "bf16", "config 5 stage 2 (all users)")
    wantq = O.sglu_ffn(host64(y1).reshape(-1, c.d), Wg, Wu, Wo).reshape(c.B, c.S, c.d)
    eq = assert_blocks_close(host64(q1), wantq, "bf16", "config 5 gated block (all users)")
    print(f"config 5: stage 2 worst block error {e3:.2e}, gated block {eq:.2e} (all {c.B} users)", flush=True)
    rows = spread_rows(c.S, 3)
    for u in users:
        Xu = I.history_user(c, u, int(lens[u]))
        w1 = O.summarize(Xu, [0, len(Xu)], Q0[rows], W["W_k0"], W["W_v0"], c.H)
        e1 = assert_blocks_close(host64(y1[u, rows])[None], w1, "bf16", f"config 5 layer 1 user {u}")
        w2 = O.summarize(Xu, [0, len(Xu)], host64(q1[u, rows]), W["W_k1"], W["W_v1"], c.H)
        e2 = assert_blocks_close(host64(y2[u, rows])[None], w2, "bf16", f"config 5 layer 2 user {u}")
        print(f"config 5 user {u} (L={int(lens[u])}): layer 1 {e1:.2e}, layer 2 {e2:.2e}", flush=True)
