"""vista_summarize_static (the entry point that allocates nothing) against vista_summarize:
same kernels, same schedule, so the outputs must agree bit for bit -- on two calls in a row,
the second with a smaller input that leaves stale records of the first behind in the scratch."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2510_22049_amd import binding as V
from paper_2510_22049_amd import inputs as I
from tests.helpers import dev, host64

pytestmark = pytest.mark.gpu


def bf(x):
    return I.round_to(np.asarray(x, dtype=np.float32), "bf16")


def both(lens, d, H, S, seed, dtype="bf16", per_user=False, seg=0):
    g = np.random.default_rng(seed)
    off = I.offsets_from_lengths(lens)
    B = len(lens)
    rnd = lambda shape, s=1.0: I.round_to((g.normal(size=shape) * s).astype(np.float32), dtype)
    X, Q = rnd((off[-1], d)), rnd((B, S, d) if per_user else (S, d))
    Wk, Wv = rnd((d, d), d ** -0.5), rnd((d, d), d ** -0.5)
    args = (dev(X, dtype), torch.from_numpy(off).cuda(), dev(Q, dtype), dev(Wk, dtype), dev(Wv, dtype))
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    a = torch.full((B, S, d), float("nan"), device="cuda", dtype=tdt)
    b = torch.full((B, S, d), float("nan"), device="cuda", dtype=tdt)
    print(f"static scratch case: lens={lens} d={d} S={S} dtype={dtype}", flush=True)
    V.vista_summarize_static(*args, a, H=H, segment_items=seg, offsets_host=torch.from_numpy(off))
    V.vista_summarize(*args, b, H=H, segment_items=seg, offsets_host=torch.from_numpy(off))
    torch.cuda.synchronize()
    assert bool(torch.isfinite(a.float()).all())
    assert torch.equal(a, b)
    return host64(a)


def test_static_scratch_two_calls_second_smaller():
    both([5000, 0, 1200, 33, 9000, 700], 128, 4, 256, seed=1)       # MFMA path, several segments per user
    both([300, 40], 128, 4, 256, seed=2)                            # smaller: stale records stay behind
    both([700, 0, 2100, 64], 256, 8, 512, seed=3, per_user=True, seg=512)
    both([90, 0, 300], 64, 2, 24, seed=4, dtype="f32")              # plain path on the same scratch
    both([17], 128, 4, 64, seed=5)


def test_static_scratch_rejects_what_does_not_fit():
    c = I.CONFIGS[3]                                                # 8 x 1M items needs ~150 MB of records
    desc = V.summarize_desc(c.B, c.S, c.d, c.H, V.VISTA_BF16, 8_000_000)
    assert V.vista_summarize_workspace_bytes(desc) > V.VISTA_STATIC_SCRATCH_BYTES
    one = C.c_void_p(256)
    st = V.lib().vista_summarize_static(C.byref(desc), one, one, None, one, one, one, one, None)
    assert st == V.VISTA_ERR_SCRATCH
    assert b"static scratch" in V.lib().vista_status_string(st)
    c2 = I.CONFIGS[2]                                               # the jagged batch fits
    desc2 = V.summarize_desc(c2.B, c2.S, c2.d, c2.H, V.VISTA_BF16, 768597)
    assert V.vista_summarize_workspace_bytes(desc2) <= V.VISTA_STATIC_SCRATCH_BYTES
