"""Pins of the oracle's further attention forms (CPU only): the SiLU score form, quasi-linear
attention, the self term, the cache codec and the QLA gradients, each against something other
than itself -- scalar loops, the paper's mask formula written out with an explicit mask matrix,
library routines (torch SDPA with a mask, torch autograd), finite differences, closed forms."""
import numpy as np
import pytest
import torch

from oracle import vista_oracle as O


def rnd(seed, *shape, scale=1.0):
    return np.random.default_rng(seed).normal(size=shape) * scale


def sigmoid(x):
    return 1.0 / (1.0 + np.exp(-x))


def problem(seed, lens, d, S, per_user=False):
    g = np.random.default_rng(seed)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    X = g.normal(size=(off[-1], d))
    Q = g.normal(size=(len(lens), S, d) if per_user else (S, d))
    return X, off, Q, g.normal(size=(d, d)) / np.sqrt(d), g.normal(size=(d, d)) / np.sqrt(d)


# ------------------------------------------------------------------ SiLU score form

def silu_loops(X, off, Q, Wk, Wv, H, scale, self_term):
    """(1/L) sum_j SiLU(scale q.k_j) v_j with scalar loops (App. B, closing formula)."""
    B = len(off) - 1
    S, d = Q.shape[-2:]
    dh = d // H
    out = np.zeros((B, S, d))
    for b in range(B):
        L = off[b + 1] - off[b]
        if L == 0:
            continue
        q_all = Q[b] if Q.ndim == 3 else Q
        for i in range(S):
            for h in range(H):
                for j in range(-1 if self_term else 0, L):
                    src = q_all[i] if j < 0 else X[off[b] + j]
                    k = [sum(src[t] * Wk[t, h * dh + c] for t in range(d)) for c in range(dh)]
                    v = [sum(src[t] * Wv[t, h * dh + c] for t in range(d)) for c in range(dh)]
                    s = scale * sum(q_all[i, h * dh + c] * k[c] for c in range(dh))
                    w = s * sigmoid(s)
                    for c in range(dh):
                        out[b, i, h * dh + c] += w * v[c] / L
    return out


@pytest.mark.parametrize("H,per_user,self_term,scale", [(1, False, False, 1.0), (2, True, False, 0.7),
                                                        (2, False, True, 1.0), (4, True, True, 0.3)])
def test_silu_form_brute_force(H, per_user, self_term, scale):
    X, off, Q, Wk, Wv = problem(1, [5, 0, 1, 7], 8, 3, per_user)
    got = O.summarize_silu(X, off, Q, Wk, Wv, H, scale=scale, self_term=self_term)
    np.testing.assert_allclose(got, silu_loops(X, off, Q, Wk, Wv, H, scale, self_term), rtol=1e-12, atol=1e-13)
    assert np.all(got[1] == 0)


def test_silu_form_default_has_no_score_scale():
    X, off, Q, Wk, Wv = problem(2, [6], 8, 2)
    np.testing.assert_allclose(O.summarize_silu(X, off, Q, Wk, Wv, 2), O.summarize_silu(X, off, Q, Wk, Wv, 2, scale=1.0))
    assert not np.allclose(O.summarize_silu(X, off, Q, Wk, Wv, 2), O.summarize_silu(X, off, Q, Wk, Wv, 2, scale=0.5))


def test_silu_matches_torch_silu():
    x = rnd(3, 50, scale=4.0)
    np.testing.assert_allclose(O.silu(x), torch.nn.functional.silu(torch.from_numpy(x)).numpy(), rtol=1e-13)


def test_silu_form_closed_forms():
    g = np.random.default_rng(4)
    d, S, H = 8, 3, 2
    Q, Wk, Wv = g.normal(size=(S, d)), g.normal(size=(d, d)), g.normal(size=(d, d))
    x = g.normal(size=d)
    # identical rows: the mean of L equal terms is the term: SiLU(q.k) (x W_v), per head
    out = O.summarize_silu(np.tile(x, (9, 1)), [0, 9], Q, Wk, Wv, H)[0]
    k, v = x @ Wk, x @ Wv
    for h in range(H):
        c = slice(4 * h, 4 * h + 4)
        s = Q[:, c] @ k[c]
        np.testing.assert_allclose(out[:, c], (s * sigmoid(s))[:, None] * v[c][None], rtol=1e-12)
    # one item: no averaging at all
    np.testing.assert_allclose(O.summarize_silu(x[None], [0, 1], Q, Wk, Wv, H)[0], out, rtol=1e-12)
    # zero queries: SiLU(0) = 0
    X = g.normal(size=(11, d))
    assert np.all(O.summarize_silu(X, [0, 11], np.zeros((S, d)), Wk, Wv, H) == 0)
    # large positive scores: SiLU(s) -> s, so the form tends to the linear one (Q K^T) V / L
    Xp = np.abs(X)
    lin = (np.abs(Q) * 40) @ (Xp @ np.abs(Wk)).T
    big = O.summarize_silu(Xp, [0, 11], np.abs(Q) * 40, np.abs(Wk), Wv, 1)[0]
    np.testing.assert_allclose(big, (lin @ (Xp @ Wv)) / 11, rtol=1e-9)


def test_silu_form_invariants():
    X, off, Q, Wk, Wv = problem(5, [13], 8, 4)
    full = O.summarize_silu(X, off, Q, Wk, Wv, 2)[0]
    perm = np.random.default_rng(6).permutation(13)
    np.testing.assert_allclose(O.summarize_silu(X[perm], off, Q, Wk, Wv, 2)[0], full, rtol=1e-12, atol=1e-14)
    # block sums (App. B): L out = L1 out1 + L2 out2 for any cut
    for cut in (1, 5, 12):
        a = O.summarize_silu(X[:cut], [0, cut], Q, Wk, Wv, 2)[0]
        b = O.summarize_silu(X[cut:], [0, 13 - cut], Q, Wk, Wv, 2)[0]
        np.testing.assert_allclose(13 * full, cut * a + (13 - cut) * b, rtol=1e-12, atol=1e-13)
    # zero rows contribute nothing (k = 0, SiLU(0) = 0) but count in N
    Xpad = np.vstack([X, np.zeros((7, 8))])
    np.testing.assert_allclose(20 * O.summarize_silu(Xpad, [0, 20], Q, Wk, Wv, 2)[0], 13 * full, rtol=1e-12, atol=1e-13)
    # users are independent
    X2, off2, _, _, _ = problem(7, [13, 4], 8, 4)
    X2[:13] = X
    np.testing.assert_allclose(O.summarize_silu(X2, off2, Q, Wk, Wv, 2)[0], full, rtol=1e-13)


def mask_M(n, m):
    """Target rows of App. B's mask: [ones(m, n) | I_m]."""
    return np.hstack([np.ones((m, n)), np.eye(m)])


def test_silu_self_term_is_the_papers_mask_formula():
    """App. B: O[T] = (silu(Q[T] K^T) . M) V with K, V = [source; target] stacked and M = [1 | I]."""
    X, off, Q, Wk, Wv = problem(8, [9], 8, 4)
    got = O.summarize_silu(X, off, Q, Wk, Wv, 1, self_term=True)[0]
    K, V = np.vstack([X @ Wk, Q @ Wk]), np.vstack([X @ Wv, Q @ Wv])
    s = Q @ K.T
    want = ((s * sigmoid(s)) * mask_M(9, 4)) @ V / 9
    np.testing.assert_allclose(got, want, rtol=1e-12)


# ------------------------------------------------------------------ quasi-linear attention

def qla_loops(X, off, Q, Wk, Wv, H, self_term):
    B = len(off) - 1
    S, d = Q.shape[-2:]
    dh = d // H
    phi = lambda t: t * sigmoid(t)
    out = np.zeros((B, S, d))
    for b in range(B):
        L = off[b + 1] - off[b]
        if L == 0:
            continue
        q_all = Q[b] if Q.ndim == 3 else Q
        for h in range(H):
            Z = np.zeros((dh, dh))
            for j in range(L):
                x = X[off[b] + j]
                for a in range(dh):
                    ka = sum(x[t] * Wk[t, h * dh + a] for t in range(d))
                    for c in range(dh):
                        Z[a, c] += phi(ka) * sum(x[t] * Wv[t, h * dh + c] for t in range(d))
            for i in range(S):
                for c in range(dh):
                    out[b, i, h * dh + c] = sum(phi(q_all[i, h * dh + a]) * phi(Z[a, c]) for a in range(dh))
                if self_term:
                    ks = [sum(q_all[i, t] * Wk[t, h * dh + a] for t in range(d)) for a in range(dh)]
                    dot = sum(phi(q_all[i, h * dh + a]) * phi(ks[a]) for a in range(dh))
                    for c in range(dh):
                        out[b, i, h * dh + c] += dot * sum(q_all[i, t] * Wv[t, h * dh + c] for t in range(d))
    return out


@pytest.mark.parametrize("H,per_user,self_term", [(1, False, False), (2, True, False), (2, False, True), (4, True, True)])
def test_qla_brute_force(H, per_user, self_term):
    X, off, Q, Wk, Wv = problem(11, [5, 0, 1, 7], 8, 3, per_user)
    got = O.summarize_qla(X, off, Q, Wk, Wv, H, self_term=self_term)
    np.testing.assert_allclose(got, qla_loops(X, off, Q, Wk, Wv, H, self_term), rtol=1e-12, atol=1e-13)
    assert np.all(got[1] == 0)


def test_qla_with_identity_activation_is_the_linear_form(monkeypatch):
    """With phi = identity the form is Q (K^T V) = (Q K^T) V (Eq. 1 without the normalisation), and
    with the self term it is App. B's mixed-mask product ((Q K^T) . M) V."""
    monkeypatch.setattr(O, "silu", lambda x: x)
    X, off, Q, Wk, Wv = problem(12, [9], 8, 4)
    K, V = X @ Wk, X @ Wv
    np.testing.assert_allclose(O.summarize_qla(X, off, Q, Wk, Wv, 1)[0], (Q @ K.T) @ V, rtol=1e-11)
    for h in range(2):                                       # heads: column slices, nothing crosses
        c = slice(4 * h, 4 * h + 4)
        np.testing.assert_allclose(O.summarize_qla(X, off, Q, Wk, Wv, 2)[0][:, c], (Q[:, c] @ K[:, c].T) @ V[:, c], rtol=1e-11)
    Kall, Vall = np.vstack([K, Q @ Wk]), np.vstack([V, Q @ Wv])
    want = ((Q @ Kall.T) * mask_M(9, 4)) @ Vall
    np.testing.assert_allclose(O.summarize_qla(X, off, Q, Wk, Wv, 1, self_term=True)[0], want, rtol=1e-11)


def test_qla_state_is_a_sum_over_blocks_and_order_free():
    K, V = rnd(13, 17, 8), rnd(14, 17, 8)
    Z = O.qla_state(K, V, 2)
    assert Z.shape == (2, 4, 4)
    for cut in (1, 8, 16):
        np.testing.assert_allclose(O.qla_state(K[:cut], V[:cut], 2) + O.qla_state(K[cut:], V[cut:], 2), Z, rtol=1e-12, atol=1e-13)
    perm = np.random.default_rng(15).permutation(17)
    np.testing.assert_allclose(O.qla_state(K[perm], V[perm], 2), Z, rtol=1e-12, atol=1e-13)
    # one item: an outer product
    k, v = K[:1], V[:1]
    np.testing.assert_allclose(O.qla_state(k, v, 1)[0], np.outer(k[0] * sigmoid(k[0]), v[0]), rtol=1e-13)


def test_qla_closed_forms():
    X, off, Q, Wk, Wv = problem(16, [6], 8, 3)
    assert np.all(O.summarize_qla(X, off, np.zeros_like(Q), Wk, Wv, 2) == 0)            # phi(0) = 0
    assert np.all(O.summarize_qla(X, off, Q, Wk, np.zeros_like(Wv), 2) == 0)            # Z = 0, phi(0) = 0
    # orientation: the state is phi(K)^T V, not V^T phi(K): a rank-one case tells them apart
    e0, e1 = np.eye(8)[0], np.eye(8)[1]
    x = (e0 * 2.0)[None]
    Wk2 = np.zeros((8, 8)); Wk2[0, 0] = 1.0          # k = 2 e0
    Wv2 = np.zeros((8, 8)); Wv2[0, 1] = 1.0          # v = 2 e1
    out = O.summarize_qla(x, [0, 1], (e0 * 3.0)[None], Wk2, Wv2, 1)[0, 0]
    z01 = O.silu(np.array(2.0)) * 2.0
    want = np.zeros(8); want[1] = O.silu(np.array(3.0)) * O.silu(np.array(z01))
    np.testing.assert_allclose(out, want, rtol=1e-13)


# ------------------------------------------------------------------ self term of the softmax form

def test_softmax_self_term_is_masked_attention_over_sources_and_targets():
    """Eq. 3 / App. B's mask: query i sees all L source keys and, of the targets, only itself.
    Library special case: torch SDPA over the stacked keys with the boolean mask [1 | I]."""
    X, off, Q, Wk, Wv = problem(21, [9], 8, 4)
    got = O.summarize(X, off, Q, Wk, Wv, 1, self_term=True)[0]
    K, V = np.vstack([X @ Wk, Q @ Wk]), np.vstack([X @ Wv, Q @ Wv])
    t = lambda a: torch.from_numpy(a)[None]
    mask = torch.from_numpy(mask_M(9, 4).astype(bool))[None]
    want = torch.nn.functional.scaled_dot_product_attention(t(Q), t(K), t(V), attn_mask=mask)[0].numpy()
    np.testing.assert_allclose(got, want, rtol=1e-10)
    # multi-head, per-user queries, empty user: brute force on one row
    X, off, Q, Wk, Wv = problem(22, [4, 0, 3], 8, 2, per_user=True)
    out = O.summarize(X, off, Q, Wk, Wv, 2, self_term=True)
    assert np.all(out[1] == 0)
    b, i, h = 2, 1, 1
    c = slice(4, 8)
    keys = np.vstack([X[off[b]:off[b + 1]] @ Wk, (Q[b, i] @ Wk)[None]])[:, c]
    vals = np.vstack([X[off[b]:off[b + 1]] @ Wv, (Q[b, i] @ Wv)[None]])[:, c]
    s = keys @ Q[b, i, c] / 2.0
    w = np.exp(s - s.max()); w /= w.sum()
    np.testing.assert_allclose(out[b, i, c], w @ vals, rtol=1e-12)


def test_target_attend_self_term():
    T, Y = rnd(23, 2, 5, 8), rnd(24, 2, 6, 8)
    got = O.target_attend(T, Y, 2, self_term=True)
    for b in range(2):
        for cidx in range(5):
            for h in range(2):
                c = slice(4 * h, 4 * h + 4)
                keys = np.vstack([Y[b][:, c], T[b, cidx, c][None]])
                s = keys @ T[b, cidx, c] / 2.0
                w = np.exp(s - s.max()); w /= w.sum()
                np.testing.assert_allclose(got[b, cidx, c], w @ keys, rtol=1e-12)
    # changing another candidate never changes this one
    T2 = T.copy(); T2[0, 3] += 1.0
    got2 = O.target_attend(T2, Y, 2, self_term=True)
    assert np.array_equal(got[0, :3], got2[0, :3]) and not np.array_equal(got[0, 3], got2[0, 3])


# ------------------------------------------------------------------ cache codec

def test_codec_brute_force_and_rounding():
    g = np.random.default_rng(31)
    H, dh = 2, 8
    Y = g.normal(size=(3, 4, H * dh)).astype(np.float32)
    Y[1, 2, :dh] = 0.0                               # an all-zero (token, head) group
    Y[0, 0, :4] = [127.0, 0.5, 1.5, -2.5]            # amax = 127: scale 1, halves round to even
    Y[0, 0, 4:dh] = 0.25
    codes, scales = O.quantize_summaries(Y, H)
    assert codes.dtype == np.int8 and scales.dtype == np.float32
    assert codes.shape == Y.shape and scales.shape == (3, 4, H)
    assert list(codes[0, 0, :4]) == [127, 0, 2, -2] and scales[0, 0, 0] == 1.0
    assert np.all(codes[1, 2, :dh] == 0) and scales[1, 2, 0] == 0.0 and scales[1, 2, 1] > 0
    for idx in np.ndindex(3, 4, H):
        grp = Y[idx[0], idx[1], idx[2] * dh:(idx[2] + 1) * dh]
        amax = np.float32(np.abs(grp).max())
        if amax == 0:
            continue
        inv = np.float32(127) / amax
        want = [int(np.rint(np.float32(v * inv))) for v in grp]
        assert list(codes[idx[0], idx[1], idx[2] * dh:(idx[2] + 1) * dh]) == want
        assert scales[idx] == np.float32(amax / np.float32(127))
        assert np.abs(want).max() == 127
    deq = O.dequantize_summaries(codes, scales)
    step = np.repeat(scales, dh, axis=-1)
    assert np.all(np.abs(deq - Y) <= step * 0.5000001 + 1e-12)
    again, _ = O.quantize_summaries(deq, H)          # a fixed point of the codec
    assert np.array_equal(again, codes)
    # one head: the whole row shares the scale
    c1, s1 = O.quantize_summaries(Y, 1)
    assert s1.shape == (3, 4, 1) and np.all(np.abs(c1).max(axis=-1) == 127)


# ------------------------------------------------------------------ gradients of QLA

def qla_forward_torch(Q, K, V, H):
    dh = Q.shape[1] // H
    outs = []
    for h in range(H):
        c = slice(h * dh, (h + 1) * dh)
        Z = torch.nn.functional.silu(K[:, c]).T @ V[:, c]
        outs.append(torch.nn.functional.silu(Q[:, c]) @ torch.nn.functional.silu(Z))
    return torch.cat(outs, dim=1)


@pytest.mark.parametrize("H", [1, 2])
def test_qla_backward_matches_autograd_and_finite_differences(H):
    Q, K, V, dO = rnd(41, 3, 8), rnd(42, 6, 8), rnd(43, 6, 8), rnd(44, 3, 8)
    dQ, dK, dV = O.qla_backward(Q, K, V, dO, H)
    tq, tk, tv = (torch.tensor(a, requires_grad=True) for a in (Q, K, V))
    (qla_forward_torch(tq, tk, tv, H) * torch.from_numpy(dO)).sum().backward()
    for got, want in ((dQ, tq.grad), (dK, tk.grad), (dV, tv.grad)):
        np.testing.assert_allclose(got, want.numpy(), rtol=1e-10, atol=1e-12)
    # central differences of the oracle's own forward, one entry of each tensor
    def loss(Qx, Kx, Vx):
        out = np.zeros_like(Qx)
        Z = O.qla_state(Kx, Vx, H)
        dh = 8 // H
        for h in range(H):
            c = slice(h * dh, (h + 1) * dh)
            out[:, c] = O.silu(Qx[:, c]) @ O.silu(Z[h])
        return (out * dO).sum()
    eps = 1e-6
    for name, arr, grad, idx in (("Q", Q, dQ, (1, 5)), ("K", K, dK, (4, 2)), ("V", V, dV, (0, 7))):
        hi, lo = arr.copy(), arr.copy()
        hi[idx] += eps; lo[idx] -= eps
        args_hi = {"Q": (hi, K, V), "K": (Q, hi, V), "V": (Q, K, hi)}[name]
        args_lo = {"Q": (lo, K, V), "K": (Q, lo, V), "V": (Q, K, lo)}[name]
        fd = (loss(*args_hi) - loss(*args_lo)) / (2 * eps)
        assert abs(fd - grad[idx]) <= 1e-6 * max(1.0, abs(fd))


def test_qla_backward_with_identity_activation_is_eqs_7_9_11(monkeypatch):
    """App. B.1 for the source part of the linear core: dQ = dO Z with Z = V^T K,
    dK = V W^T and dV = K W with W = Q^T dO."""
    monkeypatch.setattr(O, "silu", lambda x: x)
    monkeypatch.setattr(O, "silu_prime", lambda x: np.ones_like(x))
    Q, K, V, dO = rnd(45, 3, 8), rnd(46, 6, 8), rnd(47, 6, 8), rnd(48, 3, 8)
    dQ, dK, dV = O.qla_backward(Q, K, V, dO, 1)
    Z, W = V.T @ K, Q.T @ dO
    np.testing.assert_allclose(dQ, dO @ Z, rtol=1e-11)
    np.testing.assert_allclose(dK, V @ W.T, rtol=1e-11)
    np.testing.assert_allclose(dV, K @ W, rtol=1e-11)


@pytest.mark.parametrize("H", [1, 2])
def test_qla_backward_self_matches_autograd_and_finite_differences(H):
    """The diagonal (self) term: autograd of a forward written with torch ops, and central
    differences of the oracle's own forward (summarize_qla with the self term minus without,
    which leaves exactly the diagonal term)."""
    n, d = 4, 8
    Q, Ks, Vs, dO = rnd(51, n, d), rnd(52, n, d), rnd(53, n, d), rnd(54, n, d)
    dQ, dK, dV = O.qla_backward_self(Q, Ks, Vs, dO, H)
    tq, tk, tv = (torch.tensor(a, requires_grad=True) for a in (Q, Ks, Vs))
    dh = d // H
    out = []
    for h in range(H):
        c = slice(h * dh, (h + 1) * dh)
        u = (torch.nn.functional.silu(tq[:, c]) * torch.nn.functional.silu(tk[:, c])).sum(dim=1, keepdim=True)
        out.append(u * tv[:, c])
    (torch.cat(out, dim=1) * torch.from_numpy(dO)).sum().backward()
    for got, want in ((dQ, tq.grad), (dK, tk.grad), (dV, tv.grad)):
        np.testing.assert_allclose(got, want.numpy(), rtol=1e-10, atol=1e-12)

    # the oracle's forward: K' = Q W_k and V' = Q W_v with W_k = W_v = I makes K' = V' = Q, so
    # perturbing one seed entry moves all three; the chain rule sums the three gradients
    X = rnd(55, 5, d)
    I8 = np.eye(d)
    def diag_term(Qx):
        return (O.summarize_qla(X, [0, 5], Qx, I8, I8, H, self_term=True)
                - O.summarize_qla(X, [0, 5], Qx, I8, I8, H))[0]
    gQ, gK, gV = O.qla_backward_self(Q, Q, Q, dO, H)
    total = gQ + gK + gV
    eps = 1e-6
    for idx in ((0, 0), (2, 5), (3, 7)):
        hi, lo = Q.copy(), Q.copy()
        hi[idx] += eps; lo[idx] -= eps
        fd = ((diag_term(hi) - diag_term(lo)) * dO).sum() / (2 * eps)
        assert abs(fd - total[idx]) <= 1e-6 * max(1.0, abs(fd))


def test_qla_backward_self_with_identity_activation_is_eqs_8_10_12(monkeypatch):
    """App. B.1, target part of the linear core: with U = Delta(Q, K') and X = Delta(dO, V') kept as
    diagonals, dQ gains X K', dK' = X Q and dV' = U dO."""
    monkeypatch.setattr(O, "silu", lambda x: x)
    monkeypatch.setattr(O, "silu_prime", lambda x: np.ones_like(x))
    Q, Ks, Vs, dO = rnd(56, 4, 8), rnd(57, 4, 8), rnd(58, 4, 8), rnd(59, 4, 8)
    dQ, dK, dV = O.qla_backward_self(Q, Ks, Vs, dO, 1)
    U = np.diag((Q * Ks).sum(axis=1))
    Xd = np.diag((dO * Vs).sum(axis=1))
    np.testing.assert_allclose(dQ, Xd @ Ks, rtol=1e-12)
    np.testing.assert_allclose(dK, Xd @ Q, rtol=1e-12)
    np.testing.assert_allclose(dV, U @ dO, rtol=1e-12)
    # a planted mistake (the two diagonals swapped) is caught
    assert np.abs(U @ Ks - dQ).max() > 1e-3
