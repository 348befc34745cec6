"""Helpers of the GPU parity tests: upload seeded inputs, run the HIP path, compare with the oracle."""
from __future__ import annotations

import numpy as np
import torch

from paper_2512_13368_amd import binding as B
from paper_2512_13368_amd.inputs import Inputs, Workload, bf16_bits

TOL = {"fp32": 1e-4, "bf16": 2e-2}


def params(w: Workload, **kw) -> B.Params:
    return B.Params(w.B, w.H, w.L, w.d, w.block, w.topk, w.window,
                    B.F32 if w.dtype == "fp32" else B.BF16, stis_mode=2 if w.bidir else int(w.stis_block > 0),
                    stis_block=w.stis_block, **kw)


def to_dev(a: np.ndarray, dtype: str):
    """fp32 host array -> device tensor of the storage type (bf16 values are already representable)."""
    if dtype == "bf16":
        return torch.from_numpy(bf16_bits(a).view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


class Dev:
    def __init__(self, x: Inputs):
        w = x.w
        self.Q, self.K, self.V = (to_dev(a, w.dtype) for a in (x.Q, x.K, x.V))
        self.dO = None if x.dO is None else to_dev(x.dO, w.dtype)
        self.vl = torch.from_numpy(x.valid_len).cuda()
        self.gw = torch.from_numpy(x.gate_w).cuda()
        self.gb = torch.from_numpy(x.gate_b).cuda()


def host(t) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def assert_close(got, ref, tol, what=""):
    """|got-ref| <= tol*(|ref| + rms(ref)) elementwise."""
    got = np.asarray(got, dtype=np.float64).reshape(ref.shape)
    assert np.all(np.isfinite(got)), f"{what}: non-finite values"
    rms = float(np.sqrt(np.mean(ref * ref)))
    err = np.abs(got - ref)
    bound = tol * (np.abs(ref) + rms)
    bad = err > bound
    if bad.any():
        idx = np.unravel_index(np.argmax(err - bound), ref.shape)
        raise AssertionError(f"{what}: {int(bad.sum())} of {ref.size} elements off; worst at {idx}: "
                             f"got {got[idx]!r} ref {ref[idx]!r} (rms {rms:.3e}, tol {tol})")


def pick_pairs(w: Workload, n: int, seed: int = 0):
    """A few (row, head) pairs for full-size spot checks; always includes the first and last pair."""
    total = w.B * w.H
    if n >= total:
        return list(range(total))
    rng = np.random.default_rng(seed)
    mid = rng.choice(np.arange(1, total - 1), size=n - 2, replace=False) if n > 2 else []
    return sorted({0, total - 1, *[int(t) for t in mid]})
