"""Pins for the CPU oracle: it is checked against things other than itself --
scalar brute force, a library attention routine, closed forms and invariants
that the paper's definitions fix (Sec. 3.2, 3.2.1, 3.3; App. B for the
block-sum re-association)."""
import math

import numpy as np
import pytest
import torch

from oracle import vista_oracle as O


def rng(seed):
    return np.random.default_rng(seed)


# ------------------------------------------------------------ brute force

def brute_summarize(X, off, Q, Wk, Wv, H, scale):
    """Scalar loops straight from RowSoftmax(QK^T)V, one number at a time."""
    B = len(off) - 1
    S, d = Q.shape[-2:]
    dh = d // H
    out = [[[0.0] * d for _ in range(S)] for _ in range(B)]
    for b in range(B):
        rows = range(off[b], off[b + 1])
        if len(rows) == 0:
            continue
        K = {j: [sum(X[j][t] * Wk[t][c] for t in range(d)) for c in range(d)] for j in rows}
        V = {j: [sum(X[j][t] * Wv[t][c] for t in range(d)) for c in range(d)] for j in rows}
        for h in range(H):
            for i in range(S):
                q = Q[b][i] if Q.ndim == 3 else Q[i]
                s = {j: scale * sum(q[h * dh + t] * K[j][h * dh + t] for t in range(dh)) for j in rows}
                den = sum(math.exp(s[j]) for j in rows)
                for c in range(dh):
                    out[b][i][h * dh + c] = sum(math.exp(s[j]) / den * V[j][h * dh + c] for j in rows)
    return np.array(out)


def brute_target(T, Y, H, scale):
    B, C, d = T.shape
    S = Y.shape[1]
    dh = d // H
    out = np.zeros((B, C, d))
    for b in range(B):
        for c in range(C):
            for h in range(H):
                s = [scale * sum(T[b, c, h * dh + t] * Y[b, j, h * dh + t] for t in range(dh)) for j in range(S)]
                den = sum(math.exp(v) for v in s)
                for t in range(dh):
                    out[b, c, h * dh + t] = sum(math.exp(s[j]) / den * Y[b, j, h * dh + t] for j in range(S))
    return out


@pytest.mark.parametrize("H,per_user_q", [(1, False), (2, False), (4, True)])
def test_summarize_brute_force(H, per_user_q):
    g = rng(10 + H)
    lens = [5, 0, 1, 7]
    off = np.concatenate([[0], np.cumsum(lens)])
    d, S = 8, 3
    X = g.normal(size=(off[-1], d))
    Q = g.normal(size=(len(lens), S, d) if per_user_q else (S, d))
    Wk, Wv = g.normal(size=(d, d)), g.normal(size=(d, d))
    scale = 0.37
    got = O.summarize(X, off, Q, Wk, Wv, H, scale)
    want = brute_summarize(X.tolist(), off.tolist(), Q, Wk.tolist(), Wv.tolist(), H, scale)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-14)
    assert np.all(got[1] == 0.0)                       # empty history -> zeros


def test_summarize_default_scale_is_inv_sqrt_dh():
    g = rng(3)
    off = np.array([0, 6])
    X, Q = g.normal(size=(6, 8)), g.normal(size=(2, 8))
    Wk, Wv = g.normal(size=(8, 8)), g.normal(size=(8, 8))
    want = brute_summarize(X.tolist(), off.tolist(), Q, Wk.tolist(), Wv.tolist(), 2, 1 / math.sqrt(4))
    np.testing.assert_allclose(O.summarize(X, off, Q, Wk, Wv, 2), want, rtol=1e-12)


@pytest.mark.parametrize("H", [1, 2])
def test_target_attend_brute_force(H):
    g = rng(20 + H)
    T, Y = g.normal(size=(2, 5, 4)), g.normal(size=(2, 3, 4))
    np.testing.assert_allclose(O.target_attend(T, Y, H, 0.7), brute_target(T, Y, H, 0.7), rtol=1e-12)


# ------------------------------------------------------- library routine

def sdpa(Q, K, V, H, scale, mask=None):
    """torch's attention on [1, H, n, dh] views: an independent multi-head path."""
    def split(A):
        n, d = A.shape
        return torch.from_numpy(A).reshape(n, H, d // H).permute(1, 0, 2)[None]
    o = torch.nn.functional.scaled_dot_product_attention(split(Q), split(K), split(V), attn_mask=mask, scale=scale)
    return o[0].permute(1, 0, 2).reshape(Q.shape[0], -1).numpy()


@pytest.mark.parametrize("H", [1, 4])
def test_summarize_matches_torch_sdpa(H):
    g = rng(30 + H)
    lens = [33, 70, 1]
    off = np.concatenate([[0], np.cumsum(lens)])
    d, S = 16, 9
    X, Q = g.normal(size=(off[-1], d)), g.normal(size=(S, d))
    Wk, Wv = g.normal(size=(d, d)) / 4, g.normal(size=(d, d)) / 4
    got = O.summarize(X, off, Q, Wk, Wv, H)
    for b in range(3):
        Xb = X[off[b]:off[b + 1]]
        want = sdpa(Q, Xb @ Wk, Xb @ Wv, H, 1 / math.sqrt(d // H))
        np.testing.assert_allclose(got[b], want, rtol=1e-10, atol=1e-12)


def test_jagged_equals_padded_and_masked():
    """A jagged batch equals the zero-padded batch with padded keys masked out."""
    g = rng(41)
    lens = [4, 19, 11]
    off = np.concatenate([[0], np.cumsum(lens)])
    d, S, H, Lmax = 8, 5, 2, 19
    X, Q = g.normal(size=(off[-1], d)), g.normal(size=(S, d))
    Wk, Wv = g.normal(size=(d, d)), g.normal(size=(d, d))
    got = O.summarize(X, off, Q, Wk, Wv, H)
    for b, L in enumerate(lens):
        Xp = np.zeros((Lmax, d))
        Xp[:L] = X[off[b]:off[b + 1]]
        mask = torch.zeros(1, 1, S, Lmax, dtype=torch.float64)
        mask[..., L:] = -math.inf
        want = sdpa(Q, Xp @ Wk, Xp @ Wv, H, 1 / math.sqrt(d // H), mask)
        np.testing.assert_allclose(got[b], want, rtol=1e-10, atol=1e-12)


def test_target_attend_matches_torch_sdpa():
    g = rng(42)
    T, Y = g.normal(size=(3, 7, 16)), g.normal(size=(3, 6, 16))
    got = O.target_attend(T, Y, 4)
    for b in range(3):
        np.testing.assert_allclose(got[b], sdpa(T[b], Y[b], Y[b], 4, 0.5), rtol=1e-10, atol=1e-12)


# ------------------------------------------------------------ closed forms

def test_identical_history_rows_give_x_Wv():
    g = rng(50)
    x = g.normal(size=(1, 12))
    X = np.repeat(x, 40, axis=0)
    Q, Wk, Wv = g.normal(size=(5, 12)), g.normal(size=(12, 12)), g.normal(size=(12, 12))
    out = O.summarize(X, [0, 40], Q, Wk, Wv, 3)
    np.testing.assert_allclose(out[0], np.repeat(x @ Wv, 5, axis=0), rtol=1e-12)


@pytest.mark.parametrize("zero", ["Q", "W_k"])
def test_zero_scores_give_column_mean_of_values(zero):
    g = rng(51)
    X = g.normal(size=(23, 8))
    Q, Wk, Wv = g.normal(size=(4, 8)), g.normal(size=(8, 8)), g.normal(size=(8, 8))
    if zero == "Q":
        Q = np.zeros_like(Q)
    else:
        Wk = np.zeros_like(Wk)
    out = O.summarize(X, [0, 23], Q, Wk, Wv, 2)
    np.testing.assert_allclose(out[0], np.repeat((X @ Wv).mean(axis=0)[None], 4, axis=0), rtol=1e-12)


def test_single_item_gives_its_value_row():
    g = rng(52)
    X = g.normal(size=(1, 8))
    Q, Wk, Wv = g.normal(size=(6, 8)), g.normal(size=(8, 8)), g.normal(size=(8, 8))
    out = O.summarize(X, [0, 1], Q, Wk, Wv, 4)
    np.testing.assert_allclose(out[0], np.repeat(X @ Wv, 6, axis=0), rtol=1e-12)


def test_two_keys_closed_form():
    """One head, two items: weights are sigmoid(+-scale*(s1-s2))."""
    q = np.array([[1.0, 2.0]])
    X = np.array([[0.5, -1.0], [2.0, 0.25]])
    I = np.eye(2)
    s1, s2 = 0.3 * (q @ X[0]), 0.3 * (q @ X[1])
    w1 = 1 / (1 + math.exp((s2 - s1).item()))
    out = O.summarize(X, [0, 2], q, I, I, 1, 0.3)
    np.testing.assert_allclose(out[0, 0], w1 * X[0] + (1 - w1) * X[1], rtol=1e-13)


def test_orientation_of_W_is_input_rows_output_columns():
    """K = X @ W_k: with W_k = e_0 e_1^T only K[:,1] = X[:,0] is non-zero."""
    X = np.array([[3.0, 0.0], [1.0, 0.0]])
    Wk = np.array([[0.0, 1.0], [0.0, 0.0]])
    q = np.array([[0.0, 1.0]])
    out = O.summarize(X, [0, 2], q, Wk, np.eye(2), 1, 1.0)
    w = math.exp(3.0) / (math.exp(3.0) + math.exp(1.0))
    np.testing.assert_allclose(out[0, 0], [3 * w + 1 * (1 - w), 0.0], rtol=1e-13)


def test_stage2_closed_forms():
    g = rng(53)
    y = g.normal(size=(1, 1, 8))
    Y = np.repeat(y, 6, axis=1)
    T = g.normal(size=(1, 4, 8))
    np.testing.assert_allclose(O.target_attend(T, Y, 2)[0], np.repeat(y[0], 4, axis=0), rtol=1e-12)
    Y2 = g.normal(size=(1, 6, 8))
    out = O.target_attend(np.zeros((1, 3, 8)), Y2, 2)
    np.testing.assert_allclose(out[0], np.repeat(Y2[0].mean(axis=0)[None], 3, axis=0), rtol=1e-12)


# -------------------------------------------------------------- invariants

def _problem(seed, lens, d=8, S=4):
    g = rng(seed)
    off = np.concatenate([[0], np.cumsum(lens)])
    return (g.normal(size=(off[-1], d)), off, g.normal(size=(S, d)),
            g.normal(size=(d, d)), g.normal(size=(d, d)))


def test_history_permutation_invariance():
    X, off, Q, Wk, Wv = _problem(60, [17, 9])
    base = O.summarize(X, off, Q, Wk, Wv, 2)
    Xp = X.copy()
    Xp[:17] = X[:17][rng(1).permutation(17)]
    np.testing.assert_allclose(O.summarize(Xp, off, Q, Wk, Wv, 2), base, rtol=1e-11, atol=1e-13)


def test_users_are_independent_and_permute():
    X, off, Q, Wk, Wv = _problem(61, [6, 10, 3])
    base = O.summarize(X, off, Q, Wk, Wv, 2)
    X2 = X.copy()
    X2[6:16] += 5.0                                    # disturb user 1 only
    out2 = O.summarize(X2, off, Q, Wk, Wv, 2)
    assert np.array_equal(out2[0], base[0]) and np.array_equal(out2[2], base[2])
    assert not np.allclose(out2[1], base[1])
    Xs = np.concatenate([X[16:19], X[0:6], X[6:16]])   # users in order 2, 0, 1
    outs = O.summarize(Xs, [0, 3, 9, 19], Q, Wk, Wv, 2)
    np.testing.assert_allclose(outs, base[[2, 0, 1]], rtol=1e-13)


def test_candidates_are_independent():
    g = rng(62)
    T, Y = g.normal(size=(1, 5, 8)), g.normal(size=(1, 7, 8))
    base = O.target_attend(T, Y, 2)
    T2 = T.copy()
    T2[0, 3] = 9.0
    out = O.target_attend(T2, Y, 2)
    keep = [0, 1, 2, 4]
    assert np.array_equal(out[0, keep], base[0, keep])


def test_row_shift_invariance():
    """A constant added to every score of a row (a constant key column paired
    with a constant query column) leaves the result unchanged."""
    X, off, Q, Wk, Wv = _problem(63, [12], d=6)
    base = O.summarize(X, off, Q, Wk, Wv, 1)
    Xa = np.concatenate([X, np.ones((12, 1))], axis=1)
    Qa = np.concatenate([Q, np.full((4, 1), 3.0)], axis=1)
    Wka = np.zeros((7, 7)); Wka[:6, :6] = Wk; Wka[6, 6] = 1.0
    Wva = np.zeros((7, 7)); Wva[:6, :6] = Wv
    out = O.summarize(Xa, off, Qa, Wka, Wva, 1, 1 / math.sqrt(6))
    np.testing.assert_allclose(out[0][:, :6], base[0], rtol=1e-11)


def partial(Q, K, V, H, scale):
    """(m, l, O) of one piece of the history: running maximum, sum of
    exponentials and un-normalised output (App. B: block sums may be taken first)."""
    n, d = Q.shape
    dh = d // H
    m, l, Oacc = np.zeros((H, n)), np.zeros((H, n)), np.zeros((n, d))
    for h in range(H):
        c = slice(h * dh, (h + 1) * dh)
        s = scale * Q[:, c] @ K[:, c].T
        m[h] = s.max(axis=1)
        e = np.exp(s - m[h][:, None])
        l[h] = e.sum(axis=1)
        Oacc[:, c] = e @ V[:, c]
    return m, l, Oacc


@pytest.mark.parametrize("cuts", [[13], [1, 2, 30], [7, 14, 21, 28, 35]])
def test_split_and_merge_equals_whole(cuts):
    X, off, Q, Wk, Wv = _problem(64, [40])
    H, scale = 2, 0.5
    whole = O.summarize(X, off, Q, Wk, Wv, H, scale)[0]
    K, V = X @ Wk, X @ Wv
    edges = [0] + cuts + [40]
    parts = [partial(Q, K[a:b], V[a:b], H, scale) for a, b in zip(edges[:-1], edges[1:])]
    m = np.max([p[0] for p in parts], axis=0)
    l = sum(p[1] * np.exp(p[0] - m) for p in parts)
    dh = 4
    out = np.zeros_like(whole)
    for h in range(H):
        c = slice(h * dh, (h + 1) * dh)
        acc = sum(p[2][:, c] * np.exp(p[0][h] - m[h])[:, None] for p in parts)
        out[:, c] = acc / l[h][:, None]
    np.testing.assert_allclose(out, whole, rtol=1e-12)


def test_exact_integer_indexing():
    """Q = 0, W_v = I, integer X: out * L is the exact column sum of the user's rows."""
    lens = [7, 0, 33, 1, 64]
    off = np.concatenate([[0], np.cumsum(lens)])
    N, d = off[-1], 4
    X = np.zeros((N, d))
    X[:, 0] = 1
    X[:, 1] = np.arange(N) % 251
    X[:, 2] = np.arange(N)
    X[:, 3] = (np.arange(N) * 7) % 13
    out = O.summarize(X, off, np.zeros((2, d)), np.eye(d), np.eye(d), 2)
    for b, L in enumerate(lens):
        if L == 0:
            assert np.all(out[b] == 0)
            continue
        want = X[off[b]:off[b + 1]].sum(axis=0)
        np.testing.assert_allclose(out[b] * L, np.repeat(want[None], 2, axis=0), rtol=1e-14)


# ---------------------------------------------------------------- gated block

def test_sglu_brute_force_and_torch():
    g = rng(70)
    y = g.normal(size=(3, 4))
    Wg, Wu, Wo = g.normal(size=(4, 6)), g.normal(size=(4, 6)), g.normal(size=(6, 4))
    got = O.sglu_ffn(y, Wg, Wu, Wo)
    want = np.zeros((3, 4))
    for r in range(3):
        rms = math.sqrt(sum(v * v for v in y[r]) / 4 + 1e-6)
        yh = [v / rms for v in y[r]]
        hid = []
        for f in range(6):
            a = sum(yh[t] * Wg[t, f] for t in range(4))
            u = sum(yh[t] * Wu[t, f] for t in range(4))
            hid.append(a / (1 + math.exp(-a)) * u)
        for c in range(4):
            want[r, c] = sum(hid[f] * Wo[f, c] for f in range(6))
    np.testing.assert_allclose(got, want, rtol=1e-12)
    ty = torch.from_numpy(y)
    th = ty / torch.sqrt((ty * ty).mean(-1, keepdim=True) + 1e-6)
    tw = (torch.nn.functional.silu(th @ torch.from_numpy(Wg)) * (th @ torch.from_numpy(Wu))) @ torch.from_numpy(Wo)
    np.testing.assert_allclose(got, tw.numpy(), rtol=1e-12)


def test_sglu_properties():
    g = rng(71)
    y = g.normal(size=(5, 8))
    Wg, Wu, Wo = g.normal(size=(8, 16)), g.normal(size=(8, 16)), g.normal(size=(16, 8))
    assert np.all(O.sglu_ffn(y, np.zeros_like(Wg), Wu, Wo) == 0)      # SiLU(0) = 0 closes the gate
    np.testing.assert_allclose(O.sglu_ffn(7.0 * y, Wg, Wu, Wo, eps=0.0), O.sglu_ffn(y, Wg, Wu, Wo, eps=0.0), rtol=1e-12)
    np.testing.assert_allclose(O.sglu_ffn(y, Wg, Wu, 2 * Wo), 2 * O.sglu_ffn(y, Wg, Wu, Wo), rtol=1e-13)
    np.testing.assert_allclose(O.silu(np.array([0.0, 1.0, -2.0])),
                               [0.0, 1 / (1 + math.exp(-1)), -2 / (1 + math.exp(2))], rtol=1e-15)
