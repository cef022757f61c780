"""CPU oracle for the VISTA hot path -- TEST INFRASTRUCTURE, NOT THE PRODUCT.

A plain, slow, fp64 numpy statement of what the two stages compute, written
from the paper's definitions.  Only tests/, the smoke check and the benchmark's
cpu_baseline leg may import it; the product path never does.  It shares no code
with the HIP path and imports nothing from the package.

What is computed (every function below cites the passage it follows):

* stage 1, ``summarize``: the S virtual seed embeddings, shared across users,
  act as the queries of a multi-head softmax attention over one user's history
  (Sec. 3.2, first paragraph; the attention itself is the "typical" form
  RowSoftmax(Q K^T) V of Sec. 3.2.1, unnumbered equation).  K = X W_k and
  V = X W_v are the projections of the history items.
* stage 2, ``target_attend``: every candidate item attends, on its own, to the
  user's S summary tokens with the same softmax attention (Sec. 3.3; the rule
  that candidates never attend to each other is Sec. 3.2.1, first paragraph and
  the remark after Eq. 2).
* ``sglu_ffn``: the SiLU-gated block between two stacked summarization layers
  (Sec. 3.2.2 names a "Simple Gated Linear Unit" but prints no formula; the
  reading used here is stated in the function).

* ``summarize_silu``: the pointwise SiLU score form, (1/N) sum_j SiLU(q . k_j) v_j
  (App. B: the closing formula for SiLU attention from targets to sources, with
  the 1/N factor of the appendix's opening paragraph).
* ``summarize_qla``: quasi-linear attention, phi(Q) phi(phi(K)^T V) with phi = SiLU
  and no row normalisation (Sec. 3.2.2, the target-side QLU equation with the
  seeds as the targets and the history as the source; block sums of App. B).
* ``self_term=True`` on any of them adds the query's attention to itself
  (Eq. 3; the Delta term of Sec. 3.2.2; the I_m block of App. B's mask M).
* ``quantize_summaries`` / ``dequantize_summaries``: the cached summaries are
  "quantized ... and dequantized" (Sec. 3.1); the paper gives no scheme, this
  build's is stated in the functions.
* ``qla_backward``: gradients of the quasi-linear form with respect to Q, K, V
  (App. B.1, Eqs. 7, 9, 11 for the linear core; the activation factors follow the
  pattern the appendix shows for its shifted-ELU variant); ``qla_backward_self``:
  those of the target-side diagonal term (second term of Eq. 8, Eqs. 10 and 12).

Every result has a plain closed definition, so the code is that definition:
two-pass softmax, no tiling, no running maximum, no fusion.  numpy's matmul
serves as the matrix-product step.

Pins (tests/test_oracle_*.py, all CPU): scalar brute-force loops on tiny inputs;
torch's scaled_dot_product_attention in fp64 on the single-head case; closed
forms (identical keys give the mean of the values, zero queries give the column
mean, one item gives its value row); invariants (jagged == padded-and-masked,
history permutation, user independence, candidate independence, shift
invariance, split-and-merge of the history at any cut); and exact-integer
indexing cases.  The paper prints no worked numeric example, so no value is
pinned to the paper itself.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


def _softmax_rows(s: np.ndarray) -> np.ndarray:
    """RowSoftmax of Sec. 3.2.1: each row is exponentiated and divided by its sum.

    The row maximum is subtracted first; that leaves the value unchanged and
    keeps exp() in range."""
    e = np.exp(s - s.max(axis=1, keepdims=True))
    return e / e.sum(axis=1, keepdims=True)


def attention(Q: np.ndarray, K: np.ndarray, V: np.ndarray, H: int, scale: float) -> np.ndarray:
    """Multi-head RowSoftmax(scale * Q_h K_h^T) V_h (Sec. 3.2.1, unnumbered eq.).

    Heads are the H contiguous column slices of width d/H of Q, K and V; the
    per-head outputs are written back to the same column slices (App. D lists
    4 attention heads but no formula; this is the usual reading).
    Q [n, d], K [L, d], V [L, d] -> [n, d]."""
    n, d = Q.shape
    dh = d // H
    out = np.zeros((n, d), dtype=F64)
    for h in range(H):
        c = slice(h * dh, (h + 1) * dh)
        s = (Q[:, c] @ K[:, c].T) * scale          # [n, L] scores
        p = _softmax_rows(s)                        # each query over all L keys
        out[:, c] = p @ V[:, c]
    return out


def default_scale(d: int, H: int) -> float:
    """1/sqrt(d_h).  The paper prints Q K^T without a factor but calls the form
    "typical"; the usual scaled form is taken."""
    return 1.0 / np.sqrt(d // H)


def _self_softmax(Q, K, V, Ks, Vs, H: int, scale: float) -> np.ndarray:
    """Softmax attention in which query i also sees one key/value of its own: row i of
    Ks, Vs (Eq. 3: a target attends to itself and to no other target; in App. B's mask M
    this is the identity block beside the all-ones source block).  The softmax of query i
    runs over the L source keys and its own key together."""
    n, d = Q.shape
    dh = d // H
    out = np.zeros((n, d), dtype=F64)
    for h in range(H):
        c = slice(h * dh, (h + 1) * dh)
        s = (Q[:, c] @ K[:, c].T) * scale                     # [n, L]
        s_self = (Q[:, c] * Ks[:, c]).sum(axis=1) * scale     # [n]
        m = np.maximum(s.max(axis=1), s_self) if s.shape[1] else s_self
        e = np.exp(s - m[:, None])
        e_self = np.exp(s_self - m)
        den = e.sum(axis=1) + e_self
        out[:, c] = (e @ V[:, c] + e_self[:, None] * Vs[:, c]) / den[:, None]
    return out


def summarize(history, offsets, queries, W_k, W_v, H: int, scale: float | None = None,
              self_term: bool = False) -> np.ndarray:
    """Stage 1 (Sec. 3.2): virtual seeds attend over each user's history.

    history [N, d] packed rows; offsets int64 [B+1] (user b owns rows
    offsets[b] .. offsets[b+1]-1); queries [S, d] shared by all users or
    [B, S, d] per user; W_k, W_v [d, d] with K = X @ W_k, V = X @ W_v.
    Returns [B, S, d] in fp64.  A user with no history gets zeros (the paper is
    silent; zeros are the neutral summary and never NaN).
    Keys and values are history items only: the seeds do not attend to
    themselves, and there is no positional term or mask (Sec. 3.2.2 reports no
    difference between causal and full attention for the history).
    self_term=True: every seed additionally attends to itself, with key seed W_k and
    value seed W_v (Eq. 3; the seeds take the place of the targets).  Users without
    history still get zeros."""
    X = np.asarray(history, dtype=F64)
    Wk = np.asarray(W_k, dtype=F64)
    Wv = np.asarray(W_v, dtype=F64)
    Qall = np.asarray(queries, dtype=F64)
    off = np.asarray(offsets, dtype=np.int64)
    B = off.size - 1
    S, d = Qall.shape[-2:]
    sc = default_scale(d, H) if scale is None else float(scale)
    out = np.zeros((B, S, d), dtype=F64)
    for b in range(B):
        Xb = X[off[b]:off[b + 1]]
        if Xb.shape[0] == 0:
            continue
        Q = Qall[b] if Qall.ndim == 3 else Qall
        if self_term:
            out[b] = _self_softmax(Q, Xb @ Wk, Xb @ Wv, Q @ Wk, Q @ Wv, H, sc)
        else:
            out[b] = attention(Q, Xb @ Wk, Xb @ Wv, H, sc)
    return out


def target_attend(candidates, summaries, H: int, scale: float | None = None,
                  self_term: bool = False) -> np.ndarray:
    """Stage 2 (Sec. 3.3): each candidate attends to its user's summary tokens.

    candidates [B, C, d], summaries [B, S, d] -> [B, C, d] in fp64.  The
    summaries serve as keys and as values (they are already in model space; the
    library call carries no projection weights).  Each candidate is one query
    row, so no candidate sees another (Sec. 3.2.1).
    self_term=True: the candidate also attends to itself (Eq. 3: Diag(T T^T) T); with no
    projections its own embedding is that key and that value."""
    T = np.asarray(candidates, dtype=F64)
    Y = np.asarray(summaries, dtype=F64)
    B, C, d = T.shape
    sc = default_scale(d, H) if scale is None else float(scale)
    out = np.zeros((B, C, d), dtype=F64)
    for b in range(B):
        if self_term:
            out[b] = _self_softmax(T[b], Y[b], Y[b], T[b], T[b], H, sc)
        else:
            out[b] = attention(T[b], Y[b], Y[b], H, sc)
    return out


def silu(x: np.ndarray) -> np.ndarray:
    """SiLU(x) = x * sigmoid(x), the activation the paper uses (Sec. 3.2.2)."""
    with np.errstate(over="ignore"):          # exp(-x) = inf for very negative x gives x / inf = -0: the limit
        return x / (1.0 + np.exp(-x))


def _jagged(history, offsets, queries, W_k, W_v):
    X = np.asarray(history, dtype=F64)
    Qall = np.asarray(queries, dtype=F64)
    off = np.asarray(offsets, dtype=np.int64)
    return X, Qall, off, np.asarray(W_k, dtype=F64), np.asarray(W_v, dtype=F64)


def summarize_silu(history, offsets, queries, W_k, W_v, H: int, scale: float | None = None,
                   self_term: bool = False) -> np.ndarray:
    """Stage 1 with the pointwise SiLU score form (App. B, closing formula):
        out[i] = (1/N) sum_j SiLU(scale * q_i . k_j) v_j          per head,
    N = the user's number of history items (App. B opens by putting a 1/N factor in place
    of the row normalisation; N is read as that user's own length).  The paper prints no
    score scale: scale=None means 1.
    self_term=True adds SiLU(scale * q_i . k_i') v_i' inside the same 1/N, with k' = seed W_k
    and v' = seed W_v (the second term of the same formula).  No history: zeros."""
    X, Qall, off, Wk, Wv = _jagged(history, offsets, queries, W_k, W_v)
    B = off.size - 1
    S, d = Qall.shape[-2:]
    dh = d // H
    sc = 1.0 if scale is None else float(scale)
    out = np.zeros((B, S, d), dtype=F64)
    for b in range(B):
        Xb = X[off[b]:off[b + 1]]
        L = Xb.shape[0]
        if L == 0:
            continue
        Q = Qall[b] if Qall.ndim == 3 else Qall
        K, V = Xb @ Wk, Xb @ Wv
        for h in range(H):
            c = slice(h * dh, (h + 1) * dh)
            acc = silu((Q[:, c] @ K[:, c].T) * sc) @ V[:, c]
            if self_term:
                Ks, Vs = Q @ Wk, Q @ Wv
                acc = acc + silu((Q[:, c] * Ks[:, c]).sum(axis=1) * sc)[:, None] * Vs[:, c]
            out[b][:, c] = acc / L
    return out


def qla_state(K: np.ndarray, V: np.ndarray, H: int) -> np.ndarray:
    """Z_h = phi(K_h)^T V_h for every head, [H, d_h, d_h] (Sec. 3.2.2: the inner product of
    the QLU equations; App. B: the sum over blocks of K_j^T V_j)."""
    L, d = K.shape
    dh = d // H
    Z = np.zeros((H, dh, dh), dtype=F64)
    for h in range(H):
        c = slice(h * dh, (h + 1) * dh)
        Z[h] = silu(K[:, c]).T @ V[:, c]
    return Z


def summarize_qla(history, offsets, queries, W_k, W_v, H: int, self_term: bool = False) -> np.ndarray:
    """Stage 1 with quasi-linear attention (Sec. 3.2.2, target-side QLU equation with the
    seeds as targets and the history as source), per head and with phi = SiLU:
        out = phi(Q_h) phi( phi(K_h)^T V_h )                 (no row normalisation, no 1/N)
    self_term=True adds Delta(phi(Q), phi(K')) V' : row i gets (phi(q_i) . phi(k_i')) v_i'
    with k' = seed W_k, v' = seed W_v.  No history: zeros."""
    X, Qall, off, Wk, Wv = _jagged(history, offsets, queries, W_k, W_v)
    B = off.size - 1
    S, d = Qall.shape[-2:]
    dh = d // H
    out = np.zeros((B, S, d), dtype=F64)
    for b in range(B):
        Xb = X[off[b]:off[b + 1]]
        if Xb.shape[0] == 0:
            continue
        Q = Qall[b] if Qall.ndim == 3 else Qall
        Z = qla_state(Xb @ Wk, Xb @ Wv, H)
        for h in range(H):
            c = slice(h * dh, (h + 1) * dh)
            out[b][:, c] = silu(Q[:, c]) @ silu(Z[h])
            if self_term:
                Ks, Vs = Q @ Wk, Q @ Wv
                out[b][:, c] += (silu(Q[:, c]) * silu(Ks[:, c])).sum(axis=1)[:, None] * Vs[:, c]
    return out


def silu_prime(x: np.ndarray) -> np.ndarray:
    """d/dx SiLU(x) = sigma(x) (1 + x (1 - sigma(x)))."""
    sg = 1.0 / (1.0 + np.exp(-x))
    return sg * (1.0 + x * (1.0 - sg))


def qla_backward(Q, K, V, dO, H: int):
    """Gradients of out = phi(Q_h) phi(phi(K_h)^T V_h) (per head, phi = SiLU) with respect to
    Q [n, d], K [L, d], V [L, d], given dO [n, d].

    App. B.1 derives them for the linear core O = Q K^T V (Eqs. 7, 9, 11 for the source
    part): dQ = dO Z, dK = V W^T, dV = K W with the d x d intermediates Z = V^T K and
    W = Q^T dO.  With the activations in place each product is taken on the activated
    operand and multiplied by the activation's derivative, as the appendix does for its
    shifted-ELU variant; the outer phi on the state contributes phi'(Z) likewise:
        A = phi(Q), P = phi(K), Zs = P^T V, G = phi(Zs)          (forward)
        dA = dO G^T,  dQ = dA * phi'(Q)
        dG = A^T dO (= W),  dZs = dG * phi'(Zs)
        dV = P dZs,   dP = V dZs^T,  dK = dP * phi'(K)
    Returns (dQ, dK, dV) in fp64."""
    Q, K, V, dO = (np.asarray(a, dtype=F64) for a in (Q, K, V, dO))
    d = Q.shape[1]
    dh = d // H
    dQ, dK, dV = np.zeros_like(Q), np.zeros_like(K), np.zeros_like(V)
    for h in range(H):
        c = slice(h * dh, (h + 1) * dh)
        A, P = silu(Q[:, c]), silu(K[:, c])
        Zs = P.T @ V[:, c]
        G = silu(Zs)
        dQ[:, c] = (dO[:, c] @ G.T) * silu_prime(Q[:, c])
        dZs = (A.T @ dO[:, c]) * silu_prime(Zs)
        dV[:, c] = P @ dZs
        dK[:, c] = (V[:, c] @ dZs.T) * silu_prime(K[:, c])
    return dQ, dK, dV


def qla_backward_self(Q, K_self, V_self, dO, H: int):
    """Gradients of the target-side diagonal term of quasi-linear attention (Sec. 3.2.2),
        out_i += Delta(phi(Q), phi(K'))_ii v'_i = (phi(q_i) . phi(k'_i)) v'_i      per head,
    with respect to Q, K' and V' (all [n, d]; K', V' are the targets' own keys and values),
    given dO [n, d].  App. B.1 states them for the linear core (second term of Eq. 8, Eqs. 10
    and 12) with the saved diagonals U = Delta(Q, K') and X = Delta(dO, V'):
        dQ = X K',   dK' = X Q,   dV' = U dO.
    With phi = SiLU in place the products are taken on the activated operands and each
    gradient is multiplied by the derivative of its own activation:
        U_i = phi(q_i) . phi(k'_i),   X_i = dO_i . v'_i
        dQ_i = X_i phi(k'_i) * phi'(q_i),   dK'_i = X_i phi(q_i) * phi'(k'_i),   dV'_i = U_i dO_i.
    Returns (dQ, dK', dV') in fp64; dQ is this term's share, to be added to that of
    qla_backward."""
    Q, Ks, Vs, dO = (np.asarray(a, dtype=F64) for a in (Q, K_self, V_self, dO))
    d = Q.shape[1]
    dh = d // H
    dQ, dK, dV = np.zeros_like(Q), np.zeros_like(Ks), np.zeros_like(Vs)
    for h in range(H):
        c = slice(h * dh, (h + 1) * dh)
        A, P = silu(Q[:, c]), silu(Ks[:, c])
        U = (A * P).sum(axis=1)[:, None]
        X = (dO[:, c] * Vs[:, c]).sum(axis=1)[:, None]
        dQ[:, c] = X * P * silu_prime(Q[:, c])
        dK[:, c] = X * A * silu_prime(Ks[:, c])
        dV[:, c] = U * dO[:, c]
    return dQ, dK, dV


def quantize_summaries(Y, H: int):
    """Cache codec (Sec. 3.1 says the summaries are quantized for the cache and dequantized
    on use, and gives no scheme; this is the build's): symmetric int8 with one scale per
    summary token and head (the head's d/H channels share it),
        amax = max_c |y_c|,  scale = amax / 127,  code_c = round_half_even(y_c * (127 / amax)),
    all in fp32 (the decision that produces an integer is taken in the precision the
    library takes it in).  An all-zero group gets scale 0 and zero codes.
    Y [..., d] -> (codes int8 [..., d], scales float32 [..., H])."""
    y = np.asarray(Y, dtype=np.float32)
    d = y.shape[-1]
    g = y.reshape(y.shape[:-1] + (H, d // H))
    amax = np.abs(g).max(axis=-1)
    safe = np.where(amax > 0, amax, np.float32(1)).astype(np.float32)
    inv = (np.float32(127) / safe).astype(np.float32)
    codes = np.rint((g * inv[..., None]).astype(np.float32))
    codes = np.clip(codes, -127, 127).astype(np.int8)
    codes[amax == 0] = 0
    scales = np.where(amax > 0, (amax / np.float32(127)).astype(np.float32), np.float32(0)).astype(np.float32)
    return codes.reshape(y.shape), scales


def dequantize_summaries(codes, scales) -> np.ndarray:
    """y_c = code_c * scale of its (token, head) (exact in fp64: an 8-bit integer times an fp32 number)."""
    c = np.asarray(codes, dtype=F64)
    sc = np.asarray(scales, dtype=F64)
    H = sc.shape[-1]
    g = c.reshape(c.shape[:-1] + (H, c.shape[-1] // H)) * sc[..., None]
    return g.reshape(c.shape)


def sglu_ffn(y, W_g, W_u, W_o, eps: float = 1e-6) -> np.ndarray:
    """Gated block between stacked summarization layers.

    Sec. 3.2.2 says the SGLU uses the gated function of TransNormerLLM and
    prints no formula.  Reading used by this build: rows are first scaled to
    unit root-mean-square (no learned gain), then
        F(y) = (SiLU(yhat W_g) * (yhat W_u)) W_o,   yhat = y / sqrt(mean(y^2) + eps).
    y [rows, d]; W_g, W_u [d, d_ff]; W_o [d_ff, d] -> [rows, d] fp64."""
    y = np.asarray(y, dtype=F64)
    yhat = y / np.sqrt((y * y).mean(axis=-1, keepdims=True) + eps)
    g = silu(yhat @ np.asarray(W_g, dtype=F64))
    u = yhat @ np.asarray(W_u, dtype=F64)
    return (g * u) @ np.asarray(W_o, dtype=F64)
