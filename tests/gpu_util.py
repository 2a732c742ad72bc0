"""Helpers for the GPU parity tests: move seeded host arrays into separately
allocated device tensors, wrap them as buffer sets, and bring results back."""
from __future__ import annotations

from typing import List, Sequence

import numpy as np


def to_device(arrays: Sequence[np.ndarray], offset_elems: int = 0):
    """One device allocation per tensor.  With offset_elems > 0 each tensor is a
    view starting that many elements into a larger allocation, so its address is
    not 16-byte aligned."""
    import torch
    out = []
    for a in arrays:
        t = torch.from_numpy(np.ascontiguousarray(a))
        if offset_elems:
            big = torch.empty(a.size + offset_elems + 8, dtype=t.dtype, device="cuda")
            view = big[offset_elems:offset_elems + a.size]
            view.copy_(t)
            out.append(view)
        else:
            out.append(t.to("cuda"))
    return out


def empty_like_device(counts: Sequence[int], dtype, offset_elems: int = 0, fill=None):
    import torch
    td = {np.float32: torch.float32, np.float16: torch.float16}[dtype]
    out = []
    for c in counts:
        big = torch.empty(c + offset_elems + 8, dtype=td, device="cuda")
        if fill is not None:
            big.fill_(fill)
        out.append(big[offset_elems:offset_elems + c])
    return out


def to_host(tensors) -> List[np.ndarray]:
    return [t.detach().cpu().numpy() for t in tensors]


def bits(a: np.ndarray) -> np.ndarray:
    return a.view(np.uint32 if a.dtype == np.float32 else np.uint16)


def assert_bits_equal(got: Sequence[np.ndarray], want: Sequence[np.ndarray], what: str = "",
                      nan_as_class: bool = False) -> None:
    assert len(got) == len(want)
    for t, (g, w) in enumerate(zip(got, want)):
        assert g.dtype == w.dtype and g.shape == w.shape, (what, t)
        gb, wb = bits(g), bits(w)
        if nan_as_class:
            gn, wn = np.isnan(g), np.isnan(w)
            assert np.array_equal(gn, wn), (what, t, "NaN positions differ")
            gb, wb = gb[~gn], wb[~wn]
        if not np.array_equal(gb, wb):
            bad = np.flatnonzero(gb != wb)
            raise AssertionError(
                f"{what}: tensor {t} differs at {bad.size} of {gb.size} elements, first index "
                f"{bad[0]}: got {gb[bad[0]]:#x} want {wb[bad[0]]:#x}")


def assert_close_params(got: Sequence[np.ndarray], want: Sequence[np.ndarray], what: str = "") -> None:
    """The stated tolerance for updated parameters: relative error <= 1e-6, or
    absolute error <= 1e-7 near zero."""
    for t, (g, w) in enumerate(zip(got, want)):
        err = np.abs(g.astype(np.float64) - w.astype(np.float64))
        ok = (err <= 1e-6 * np.abs(w.astype(np.float64))) | (err <= 1e-7)
        assert np.all(ok), (what, t, float(err.max()))
