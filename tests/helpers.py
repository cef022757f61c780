"""Test plumbing shared by the GPU parity tests (no arithmetic of the method)."""
import numpy as np
import torch

TOL = {"f32": 1e-4, "bf16": 2e-2}     # max error per output block relative to the block's max |value|


def torch_dtype(name):
    return torch.float32 if name == "f32" else torch.bfloat16


def dev(x: np.ndarray, dtype: str) -> torch.Tensor:
    """Storage-rounded fp32 host values -> device tensor of the storage dtype (exact)."""
    return torch.from_numpy(np.ascontiguousarray(x)).to("cuda").to(torch_dtype(dtype))


def host64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def block_errors(got: np.ndarray, want: np.ndarray) -> np.ndarray:
    """max |got - want| / max |want| over each leading-index block (one user)."""
    g = got.reshape(got.shape[0], -1)
    w = want.reshape(want.shape[0], -1)
    den = np.abs(w).max(axis=1)
    den = np.where(den == 0, 1.0, den)
    return np.abs(g - w).max(axis=1) / den


def floored_errors(got: np.ndarray, want: np.ndarray, floor: float = 1e-3) -> np.ndarray:
    """Element-wise |got - want| / max(|want|, floor x the block's max |want|), worst element per block.
    Reported as information only: near-zero, sign-changing outputs make a bare element-wise ratio
    meaningless, the floor keeps it finite."""
    g = got.reshape(got.shape[0], -1)
    w = want.reshape(want.shape[0], -1)
    top = np.abs(w).max(axis=1, keepdims=True)
    den = np.maximum(np.abs(w), floor * np.where(top == 0, 1.0, top))
    return (np.abs(g - w) / den).max(axis=1)


def assert_blocks_close(got, want, dtype, what=""):
    assert np.all(np.isfinite(got)), f"{what}: non-finite output"
    err = block_errors(got, want)
    worst = int(err.argmax())
    assert err[worst] <= TOL[dtype], f"{what}: block {worst} error {err[worst]:.3e} > {TOL[dtype]:.0e}"
    return float(err.max())


def assert_in_value_hull(out: torch.Tensor, values: torch.Tensor, what="", slack=2.0 ** -7):
    """Property that holds at any size: softmax weights are non-negative and sum to one, so every
    output channel of a block lies between the smallest and the largest value of that channel
    (out [..., rows, d] against values [..., n, d], compared on the device in fp32; `slack` x the
    channel's largest magnitude allows for the bf16 roundings of values, weights and output)."""
    v = values.float()
    lo, hi = v.amin(dim=-2, keepdim=True), v.amax(dim=-2, keepdim=True)
    tol = slack * torch.maximum(lo.abs(), hi.abs())
    o = out.float()
    assert bool(((o >= lo - tol) & (o <= hi + tol)).all()), f"{what}: output outside the hull of its values"
