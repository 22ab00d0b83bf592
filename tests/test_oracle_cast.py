"""Pins for the oracle's fused cast + diff (Alg. 1: CastAndCopy followed by the diff, Sec. 3.4 Trainer hook)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_07330_amd import synth


def torch_round(x: np.ndarray) -> np.ndarray:
    return torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def test_rounding_matches_a_library_cast_on_every_non_nan_class():
    rng = np.random.default_rng(0)
    parts = [
        (rng.standard_normal(1 << 20) * 0.02).astype(np.float32),
        rng.integers(0, 1 << 32, size=1 << 20, dtype=np.uint64).astype(np.uint32).view(np.float32),   # any pattern
        np.array([0.0, -0.0, np.inf, -np.inf, 3.3895314e38, 3.4028235e38, -3.4028235e38, 1e-45, 1e-40, 1.1754944e-38],
                 np.float32),
    ]
    # exact ties: BF16 keeps 8 significant bits, so x.xxxxxxx1|1000... patterns sit half way
    base = rng.integers(0, 1 << 16, size=4096, dtype=np.uint32) << 16
    parts.append((base | 0x8000).astype(np.uint32).view(np.float32))
    parts.append((base | 0x7FFF).astype(np.uint32).view(np.float32))
    parts.append((base | 0x8001).astype(np.uint32).view(np.float32))
    x = np.concatenate(parts)
    finite_or_inf = ~np.isnan(x)
    got, want = oracle.round_bf16(x), torch_round(x)
    assert np.array_equal(got[finite_or_inf], want[finite_or_inf])
    assert np.all(got[~finite_or_inf] == 0x7FC0)
    # ties to even by hand: 1 + 2^-8 is half way between 0x3F80 and 0x3F81 -> even (0x3F80); 1 + 3*2^-8 -> 0x3F82
    ties = np.array([1 + 2 ** -8, 1 + 3 * 2 ** -8, 1 + 2 ** -8 + 2 ** -20], np.float32)
    assert oracle.round_bf16(ties).tolist() == [0x3F80, 0x3F82, 0x3F81]


@pytest.mark.parametrize("n,be", [(100003, 4096), (65536, 65536), (5, 2)])
def test_fused_equals_cast_then_extract(n, be):
    rng = np.random.default_rng(n)
    w = rng.integers(0, 1 << 16, size=n, dtype=np.uint16)
    master = (rng.standard_normal(n)).astype(np.float32)
    keep = rng.random(n) < 0.9                                       # 90 % of the master weights round to the old value
    master[keep] = (w[keep].astype(np.uint32) << 16).view(np.float32)
    new = torch_round(master)
    nan = np.isnan(master)
    new[nan] = 0x7FC0
    ref_old = w.copy()
    rI, rV, rc, _ = oracle.extract(ref_old, new, be)                 # the two-step definition
    w2 = w.copy()
    I, V, c, ovf = oracle.extract_cast(w2, master, be)
    assert ovf == 0 and np.array_equal(c, rc) and np.array_equal(I, rI) and np.array_equal(V, rV)
    assert np.array_equal(w2, new)                                   # the model parameters now hold the cast
    # brute force of the definition
    want = [i for i in range(n) if new[i] != w[i]]
    assert np.concatenate([I[b, :c[b]] for b in range(len(c))]).tolist() == want


def test_generated_master_weights_round_back_and_list_form():
    wl = synth.workload(2, tiny=True)
    a = synth.WeightSet(wl, "cpu"); b = synth.WeightSet(wl, "cpu")
    synth.fill_base(a, 5)
    nchanged, _ = synth.make_update(b, a, 5)
    master = torch.empty(wl.numel, dtype=torch.float32)
    synth.master_from_(master, b.flat, 5)
    m = master.numpy()
    assert not np.array_equal(m.view(np.uint32) & 0xFFFF, np.zeros(m.size, np.uint32))   # genuinely 32-bit values
    assert np.array_equal(oracle.round_bf16(m), np.concatenate(b.to_numpy_u16()))
    ws = a.to_numpy_u16()
    ms, off = [], 0
    for t in wl.tensors:
        ms.append(m[off:off + t.numel].copy()); off += t.numel
    I, V, c, _ = oracle.extract_cast_multi(ws, ms, a.numels, wl.bucket_elems)
    rI, rV, rc, _ = oracle.extract_multi(a.to_numpy_u16(), b.to_numpy_u16(), a.numels, wl.bucket_elems)
    assert int(c.sum()) == nchanged
    assert np.array_equal(c, rc) and np.array_equal(I, rI) and np.array_equal(V, rV)
    assert all(np.array_equal(x, y) for x, y in zip(ws, b.to_numpy_u16()))
