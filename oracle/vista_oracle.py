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


def summarize(history, offsets, queries, W_k, W_v, H: int, scale: float | None = None) -> np.ndarray:
    """Stage 1 (Sec. 3.2): virtual seeds attend over each user's history.

    history [N, d] packed rows; offsets int64 [B+1] (user b owns rows
    offsets[b] .. offsets[b+1]-1); queries [S, d] shared by all users or
    [B, S, d] per user; W_k, W_v [d, d] with K = X @ W_k, V = X @ W_v.
    Returns [B, S, d] in fp64.  A user with no history gets zeros (the paper is
    silent; zeros are the neutral summary and never NaN).
    Keys and values are history items only: the seeds do not attend to
    themselves, and there is no positional term or mask (Sec. 3.2.2 reports no
    difference between causal and full attention for the history)."""
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
        out[b] = attention(Q, Xb @ Wk, Xb @ Wv, H, sc)
    return out


def target_attend(candidates, summaries, H: int, scale: float | None = None) -> np.ndarray:
    """Stage 2 (Sec. 3.3): each candidate attends to its user's summary tokens.

    candidates [B, C, d], summaries [B, S, d] -> [B, C, d] in fp64.  The
    summaries serve as keys and as values (they are already in model space; the
    library call carries no projection weights).  Each candidate is one query
    row, so no candidate sees another (Sec. 3.2.1)."""
    T = np.asarray(candidates, dtype=F64)
    Y = np.asarray(summaries, dtype=F64)
    B, C, d = T.shape
    sc = default_scale(d, H) if scale is None else float(scale)
    out = np.zeros((B, C, d), dtype=F64)
    for b in range(B):
        out[b] = attention(T[b], Y[b], Y[b], H, sc)
    return out


def silu(x: np.ndarray) -> np.ndarray:
    """SiLU(x) = x * sigmoid(x), the activation the paper uses (Sec. 3.2.2)."""
    return x / (1.0 + np.exp(-x))


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
