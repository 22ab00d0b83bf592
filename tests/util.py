"""Shared helpers of the GPU parity tests (host <-> device plumbing only)."""
import numpy as np
import torch


def u16(t: torch.Tensor) -> np.ndarray:
    """Bit patterns of a 16-bit tensor as a 1-D numpy uint16 array (host copy)."""
    return t.detach().reshape(-1).view(torch.int16).cpu().numpy().view(np.uint16).copy()


def from_u16(a: np.ndarray, device) -> torch.Tensor:
    return torch.from_numpy(a.view(np.int16).copy()).to(device).view(torch.bfloat16)


def payload_to_host(I, V, counts):
    return (I.cpu().numpy().astype(np.int32), V.cpu().numpy().view(np.uint16), counts.cpu().numpy().view(np.uint32))


def assert_payload_equal(got, want, label=""):
    """Element-by-element, tolerance 0: indices, values, counts, and the untouched fill beyond counts."""
    gI, gV, gc = got
    wI, wV, wc = want
    assert np.array_equal(gc, wc), f"{label}: counts differ at buckets {np.flatnonzero(gc != wc)[:8]}"
    assert gI.shape == wI.shape and gV.shape == wV.shape, f"{label}: payload shape"
    bad = np.flatnonzero((gI != wI).any(axis=1) | (gV != wV).any(axis=1))
    assert bad.size == 0, f"{label}: payload differs in buckets {bad[:8]}"
