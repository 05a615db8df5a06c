"""Helpers for the GPU parity tests: host copies for the oracle, tolerance scales, compare.

Tolerances: sampled IDs bit-exact; means and gradients within
max relative error 1e-5 (fp32 features) / 1e-2 (bf16 features).  "Relative" is taken
against max(|ref|, A): A is the mean magnitude of the rows that were averaged (forward) or
the sum of the magnitudes of the contributions (backward), so that an output that is small
only through cancellation is not held to an impossible bound."""
from __future__ import annotations

import numpy as np
import torch

TOL = {torch.float32: 1e-5, torch.bfloat16: 1e-2}


def host_x(x: torch.Tensor):
    """Feature table as the oracle takes it: float32 array, or uint16 bit patterns + bf16=True."""
    if x.dtype == torch.bfloat16:
        return x.cpu().view(torch.int16).numpy().view(np.uint16), True
    return x.cpu().numpy(), False


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def forward_scales(x: torch.Tensor, ids1: torch.Tensor, ids2):
    """A for out (and out_h1): mean |x| over the rows each output averaged, on the device."""
    xa = x
    if ids2 is None:
        m = (ids1 >= 0)
        rows = xa[ids1.clamp(min=0).long()].abs().float() * m[..., None]
        return (rows.sum(1) / m.sum(1).clamp(min=1)[:, None]).double().cpu().numpy(), None
    B, k1, k2 = ids2.shape
    a_h1 = torch.zeros((B, k1, x.shape[1]), dtype=torch.float32, device=x.device)
    step = max(1, (1 << 26) // max(1, k1 * k2 * x.shape[1]))
    for b0 in range(0, B, step):
        sl = slice(b0, b0 + step)
        m = (ids2[sl] >= 0)
        rows = xa[ids2[sl].clamp(min=0).long()].abs().float() * m[..., None]
        a_h1[sl] = rows.sum(2) / m.sum(2).clamp(min=1)[..., None]
    live = ((ids2 >= 0).sum(2) > 0) & (ids1 >= 0)
    a_out = (a_h1 * live[..., None]).sum(1) / live.sum(1).clamp(min=1)[:, None]
    return a_out.double().cpu().numpy(), a_h1.double().cpu().numpy()


def assert_close(got: np.ndarray, ref: np.ndarray, scale: np.ndarray, tol: float, what: str):
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.isfinite(got).all(), what + ": non-finite values"
    bound = tol * np.maximum(np.abs(ref), scale)
    err = np.abs(got - ref)
    bad = err > bound
    if bad.any():
        i = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError("%s: %d of %d elements out of tolerance %g; worst at %s: got %r ref %r scale %r"
                             % (what, int(bad.sum()), err.size, tol, i, got[i], ref[i], scale[i]))
    return float((err / np.maximum(np.maximum(np.abs(ref), scale), 1e-300)).max())


def assert_ids_equal(got: torch.Tensor, ref: np.ndarray, what: str):
    g = got.cpu().numpy()
    assert g.dtype == np.int32 and g.shape == ref.shape, (what, g.shape, ref.shape)
    if not np.array_equal(g, ref):
        bad = np.argwhere(g != ref)
        raise AssertionError("%s: %d mismatching IDs, first at %s: got %d ref %d"
                             % (what, len(bad), tuple(bad[0]), g[tuple(bad[0])], ref[tuple(bad[0])]))
