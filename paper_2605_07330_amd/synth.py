"""Seeded synthetic workloads: Qwen3-shaped BF16 weight sets and their sparse updates.

This module only *makes inputs*.  It holds none of the method's arithmetic (no diff,
no compaction, no scatter) and is the one module that both the CPU oracle's tests and
the GPU library's tests may import.  Everything is plain torch and runs on CPU or GPU.

The weight sets are stand-ins shaped like the models the paper measures on (Sec. 2.2,
Table 2 and Sec. 4.1 use Qwen3-30B-A3B and other open models); the real checkpoints and RL
deltas are not needed: extraction and reconstruction never look at a value except to
compare bit patterns.  The update densities bracket what Table 2 reports for BF16
(about 0.6-1 % of elements change per step).

Recipe for one update (one "step"):
  * base weights  ~ N(0, 0.02) in fp32, rounded to BF16 (norm vectors are 1.0);
    the FP8 stand-ins further down use the same shapes with E4M3 patterns and one-step moves;
  * a change mask, iid Bernoulli(p) per element unless the workload says otherwise;
  * at masked positions  new = bf16(old + N(0, 1e-3*|old| + 1e-6)); if the rounding gives
    back the old pattern the value is moved one BF16 step in the direction of the noise
    (away from zero when the noise is exactly 0), so that every masked position differs
    bitwise and the mask is the exact ground truth for the changed-index set.  Relative
    noise of 1e-3 is below half a BF16 ulp, so most changes are one-ulp moves, as the
    paper's absorption argument (Sec. 3, "BF16 absorption") predicts for real updates.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, Iterable, List, Optional, Sequence, Tuple

import torch

MiB = 1 << 20


@dataclasses.dataclass(frozen=True)
class TensorSpec:
    name: str
    rows: int
    cols: int
    kind: str            # embed | lm_head | attn | router | expert | mlp | norm
    layer: int = -1
    expert: int = -1

    @property
    def numel(self) -> int:
        return self.rows * self.cols


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    tensors: Tuple[TensorSpec, ...]
    bucket_elems: int
    density: float                 # iid density p; for the skewed workload the largest per-tensor density
    skewed: bool = False

    @property
    def numel(self) -> int:
        return sum(t.numel for t in self.tensors)

    @property
    def num_buckets(self) -> int:
        return (self.numel + self.bucket_elems - 1) // self.bucket_elems


# ----------------------------------------------------------------------------------------------
# shapes
# ----------------------------------------------------------------------------------------------

def _dense_model(prefix: str, layers: int, hidden: int, q_out: int, kv_out: int, ffn: int, vocab: int,
                 norms: bool) -> List[TensorSpec]:
    ts = [TensorSpec(f"{prefix}.embed", vocab, hidden, "embed")]
    for l in range(layers):
        ts += [
            TensorSpec(f"{prefix}.{l}.q_proj", q_out, hidden, "attn", l),
            TensorSpec(f"{prefix}.{l}.k_proj", kv_out, hidden, "attn", l),
            TensorSpec(f"{prefix}.{l}.v_proj", kv_out, hidden, "attn", l),
            TensorSpec(f"{prefix}.{l}.o_proj", hidden, q_out, "attn", l),
            TensorSpec(f"{prefix}.{l}.gate_proj", ffn, hidden, "mlp", l),
            TensorSpec(f"{prefix}.{l}.up_proj", ffn, hidden, "mlp", l),
            TensorSpec(f"{prefix}.{l}.down_proj", hidden, ffn, "mlp", l),
        ]
        if norms:
            ts += [TensorSpec(f"{prefix}.{l}.input_norm", 1, hidden, "norm", l),
                   TensorSpec(f"{prefix}.{l}.post_attn_norm", 1, hidden, "norm", l)]
    ts.append(TensorSpec(f"{prefix}.lm_head", vocab, hidden, "lm_head"))
    return ts


def _moe_model(prefix: str, layers: int, hidden: int, q_out: int, kv_out: int, experts: int, eff: int,
               vocab: int) -> List[TensorSpec]:
    ts = [TensorSpec(f"{prefix}.embed", vocab, hidden, "embed")]
    for l in range(layers):
        ts += [
            TensorSpec(f"{prefix}.{l}.q_proj", q_out, hidden, "attn", l),
            TensorSpec(f"{prefix}.{l}.k_proj", kv_out, hidden, "attn", l),
            TensorSpec(f"{prefix}.{l}.v_proj", kv_out, hidden, "attn", l),
            TensorSpec(f"{prefix}.{l}.o_proj", hidden, q_out, "attn", l),
            TensorSpec(f"{prefix}.{l}.router", experts, hidden, "router", l),
        ]
        for e in range(experts):
            ts += [
                TensorSpec(f"{prefix}.{l}.e{e}.gate_proj", eff, hidden, "expert", l, e),
                TensorSpec(f"{prefix}.{l}.e{e}.up_proj", eff, hidden, "expert", l, e),
                TensorSpec(f"{prefix}.{l}.e{e}.down_proj", hidden, eff, "expert", l, e),
            ]
    ts.append(TensorSpec(f"{prefix}.lm_head", vocab, hidden, "lm_head"))
    return ts


def workload(cfg: int, density: Optional[float] = None, tiny: bool = False) -> Workload:
    """The five benchmark workloads.  ``tiny=True`` keeps the structure (tensor order, kinds,
    tensors that straddle buckets, several small tensors per bucket, a short last bucket) at a
    size a CPU finishes in well under a second."""
    if cfg == 0:
        side = 256 if tiny else 2048
        return Workload("single-2048x2048" if not tiny else "single-256x256",
                        (TensorSpec("w", side, side, "mlp"),), side * side // 4, density or 0.01)
    if cfg == 1:
        if tiny:
            ts = _dense_model("q8b", 3, 64, 64, 16, 192, 2374, norms=True)
            return Workload("qwen3-8b-tiny", tuple(ts), 40000, density or 0.01)
        ts = _dense_model("q8b", 36, 4096, 4096, 1024, 12288, 151936, norms=True)
        return Workload("qwen3-8b", tuple(ts), 64 * MiB // 2, density or 0.01)
    if cfg in (2, 3):
        if tiny:
            ts = _moe_model("q30b", 3, 32, 64, 8, 16, 12, 2374)
            return Workload("qwen3-30b-a3b-tiny" + ("-skewed" if cfg == 3 else ""), tuple(ts), 8192,
                            density or (0.05 if cfg == 3 else 0.01), skewed=(cfg == 3))
        ts = _moe_model("q30b", 48, 2048, 4096, 512, 128, 768, 151936)
        return Workload("qwen3-30b-a3b" + ("-skewed" if cfg == 3 else ""), tuple(ts), 64 * MiB // 2,
                        density or (0.05 if cfg == 3 else 0.01), skewed=(cfg == 3))
    if cfg == 4:
        if tiny:
            ts = _dense_model("q32b", 4, 80, 128, 16, 400, 2374, norms=False)
            return Workload("qwen3-32b-tiny", tuple(ts), 100000, density or 0.01)
        ts = _dense_model("q32b", 64, 5120, 8192, 1024, 25600, 151936, norms=False)
        return Workload("qwen3-32b", tuple(ts), 256 * MiB // 2, density or 0.01)
    raise ValueError(f"unknown workload {cfg}")


# ----------------------------------------------------------------------------------------------
# values
# ----------------------------------------------------------------------------------------------

_CHUNK = 1 << 26


def _gen(device, *key: int) -> torch.Generator:
    g = torch.Generator(device=device)
    s = 0x9E3779B97F4A7C15
    for k in key:
        s = ((s ^ (int(k) + 0x632BE59BD9B4E019)) * 0xD1342543DE82EF95) % (1 << 63)
    g.manual_seed(s)
    return g


def fill_base_(flat: torch.Tensor, seed: int, salt: int = 0) -> None:
    """flat (bf16, 1-D) <- bf16(N(0, 0.02)), chunk by chunk."""
    n = flat.numel()
    for c, lo in enumerate(range(0, n, _CHUNK)):
        hi = min(n, lo + _CHUNK)
        g = _gen(flat.device, seed, salt, c, 1)
        x = torch.randn(hi - lo, generator=g, device=flat.device, dtype=torch.float32) * 0.02
        flat[lo:hi] = x.to(torch.bfloat16)


def bump_bits(ob: torch.Tensor, toward_pos_inf: torch.Tensor, zero_noise: torch.Tensor) -> torch.Tensor:
    """Neighbouring BF16 pattern of ``ob`` (int32 holding a 16-bit pattern) in the given direction;
    away from zero where ``zero_noise``.  Never returns ``ob`` itself, never steps into Inf/NaN."""
    sign = ob >> 15
    mag = ob & 0x7FFF
    grow = torch.where(zero_noise, torch.ones_like(zero_noise), toward_pos_inf == (sign == 0))
    grow = torch.where(mag >= 0x7F7F, torch.zeros_like(grow), grow)          # stay finite
    cross = (~grow) & (mag == 0)                                              # +0 going down, -0 going up
    new_mag = torch.where(grow, mag + 1, mag - 1)
    new_mag = torch.where(cross, torch.ones_like(mag), new_mag)
    new_sign = torch.where(cross, 1 - sign, sign)
    return (new_sign << 15) | new_mag


def perturb_(new_flat: torch.Tensor, old_flat: torch.Tensor, mask: torch.Tensor, g: torch.Generator) -> None:
    """new_flat <- old_flat, with masked positions moved as the recipe in the module docstring says."""
    old_f = old_flat.float()
    noise = torch.randn(old_f.shape, generator=g, device=old_f.device, dtype=torch.float32)
    noise = noise * (1e-3 * old_f.abs() + 1e-6)
    cand = (old_f + noise).to(torch.bfloat16)
    ob = old_flat.view(torch.int16).to(torch.int32) & 0xFFFF
    cb = cand.view(torch.int16).to(torch.int32) & 0xFFFF
    bumped = bump_bits(ob, noise > 0, noise == 0)
    nb = torch.where(cb == ob, bumped, cb)
    nb = torch.where(mask, nb, ob)
    # back to a 16-bit pattern held in int16
    nb = torch.where(nb >= 0x8000, nb - 0x10000, nb).to(torch.int16)
    new_flat.view(torch.int16).copy_(nb)


def iid_update_(new_flat: torch.Tensor, old_flat: torch.Tensor, p: float, seed: int, salt: int = 0,
                want_mask: bool = False) -> Tuple[int, Optional[torch.Tensor]]:
    """iid Bernoulli(p) update of a flat BF16 buffer, chunk by chunk.  Returns (#changed, mask|None)."""
    n = old_flat.numel()
    changed = 0
    masks = []
    for c, lo in enumerate(range(0, n, _CHUNK)):
        hi = min(n, lo + _CHUNK)
        g = _gen(old_flat.device, seed, salt, c, 2)
        if p <= 0.0:
            new_flat[lo:hi] = old_flat[lo:hi]
            mask = torch.zeros(hi - lo, dtype=torch.bool, device=old_flat.device) if want_mask else None
        else:
            mask = torch.rand(hi - lo, generator=g, device=old_flat.device) < p
            perturb_(new_flat[lo:hi], old_flat[lo:hi], mask, g)
            changed += int(mask.sum().item())
        if want_mask:
            masks.append(mask)
    return changed, (torch.cat(masks) if want_mask and masks else
                     (torch.zeros(0, dtype=torch.bool, device=old_flat.device) if want_mask else None))


def masked_update_(new_flat: torch.Tensor, old_flat: torch.Tensor, mask: torch.Tensor, seed: int, salt: int) -> int:
    g = _gen(old_flat.device, seed, salt, 0, 3)
    perturb_(new_flat, old_flat, mask, g)
    return int(mask.sum().item())


# ----------------------------------------------------------------------------------------------
# weight sets
# ----------------------------------------------------------------------------------------------

class WeightSet:
    """A list of BF16 tensors, one per TensorSpec.

    ``slab=True`` carves them from one allocation, end to end (every tensor of the benchmark
    workloads is a multiple of 2048 elements, so each stays 4 KiB-aligned); ``slab=False`` gives
    each tensor its own allocation, optionally misaligned by ``misalign`` elements to exercise the
    2-byte-alignment path."""

    def __init__(self, wl: Workload, device, slab: bool = True, misalign: int = 0):
        self.wl = wl
        self.device = torch.device(device)
        self.flat: Optional[torch.Tensor] = None
        self.tensors: List[torch.Tensor] = []
        self._keep: List[torch.Tensor] = []
        if slab:
            self.flat = torch.empty(wl.numel, dtype=torch.bfloat16, device=self.device)
            off = 0
            for t in wl.tensors:
                self.tensors.append(self.flat[off:off + t.numel])
                off += t.numel
        else:
            for k, t in enumerate(wl.tensors):
                pad = (misalign * (k % 3 + 1)) % 8 if misalign else 0
                buf = torch.empty(t.numel + pad, dtype=torch.bfloat16, device=self.device)
                self._keep.append(buf)
                self.tensors.append(buf[pad:pad + t.numel])

    @property
    def numels(self) -> List[int]:
        return [t.numel for t in self.wl.tensors]

    def copy_from(self, other: "WeightSet") -> None:
        if self.flat is not None and other.flat is not None:
            self.flat.copy_(other.flat)
        else:
            for a, b in zip(self.tensors, other.tensors):
                a.copy_(b)

    def equal(self, other: "WeightSet") -> bool:
        """Bitwise equality, tensor by tensor (the paper's Sec. 4.2 check compares tensor by tensor)."""
        for a, b in zip(self.tensors, other.tensors):
            if a.numel() and not torch.equal(a.view(torch.int16), b.view(torch.int16)):
                return False
        return True

    def to_numpy_u16(self):
        import numpy as np
        return [t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16).copy() for t in self.tensors]


def fill_base(ws: WeightSet, seed: int) -> None:
    """Base values: N(0, 0.02) everywhere, 1.0 in norm vectors."""
    if ws.flat is not None:
        fill_base_(ws.flat, seed)
    else:
        for k, t in enumerate(ws.tensors):
            fill_base_(t, seed, salt=1000 + k)
    for spec, t in zip(ws.wl.tensors, ws.tensors):
        if spec.kind == "norm":
            t.fill_(1.0)


def tensor_density(wl: Workload, spec: TensorSpec, active_experts: Dict[int, set]) -> float:
    """Nominal per-tensor density.  Skewed workload: 8 of the experts of each layer at 5 %, the rest
    unchanged; attention and router at 1 %; lm_head at 0.2 %; the embedding is handled row-wise."""
    if not wl.skewed:
        return wl.density
    if spec.kind == "expert":
        return 0.05 if spec.expert in active_experts.get(spec.layer, ()) else 0.0
    if spec.kind in ("attn", "router"):
        return 0.01
    if spec.kind == "lm_head":
        return 0.002
    return 0.01


def _active_experts(wl: Workload, seed: int, step: int) -> Dict[int, set]:
    layers = sorted({t.layer for t in wl.tensors if t.kind == "expert"})
    out: Dict[int, set] = {}
    for l in layers:
        ne = 1 + max(t.expert for t in wl.tensors if t.kind == "expert" and t.layer == l)
        g = _gen("cpu", seed, step, l, 4)
        k = min(8, max(1, ne // 16)) if ne < 128 else 8
        out[l] = set(torch.randperm(ne, generator=g)[:k].tolist())
    return out


def _embedding_row_mask(spec: TensorSpec, device, seed: int, step: int) -> torch.Tensor:
    """Rows touched iid at 0.001; a touched row is fully changed with prob. 0.1, else iid 1 % inside it."""
    g = _gen(device, seed, step, 5)
    touched = torch.rand(spec.rows, generator=g, device=device) < 0.001
    if spec.rows < 100000:                      # tiny stand-ins: make sure the structure shows up at all
        touched = torch.rand(spec.rows, generator=g, device=device) < 0.02
    full = touched & (torch.rand(spec.rows, generator=g, device=device) < 0.1)
    mask = torch.zeros(spec.rows, spec.cols, dtype=torch.bool, device=device)
    rows = torch.nonzero(touched & ~full).flatten()
    if rows.numel():
        mask[rows] = torch.rand(rows.numel(), spec.cols, generator=g, device=device) < 0.01
    mask[torch.nonzero(full).flatten()] = True
    return mask.flatten()


def make_update(new: WeightSet, old: WeightSet, seed: int, step: int = 1, want_masks: bool = False
                ) -> Tuple[int, Optional[List[torch.Tensor]]]:
    """new <- old with one synthetic sparse update.  Returns (#changed elements, per-tensor masks|None)."""
    wl = old.wl
    if not wl.skewed and old.flat is not None and new.flat is not None and not want_masks:
        changed, _ = iid_update_(new.flat, old.flat, wl.density, seed, salt=step)
        return changed, None
    act = _active_experts(wl, seed, step) if wl.skewed else {}
    total = 0
    masks: List[torch.Tensor] = []
    for k, (spec, o, n) in enumerate(zip(wl.tensors, old.tensors, new.tensors)):
        if wl.skewed and spec.kind == "embed":
            m = _embedding_row_mask(spec, o.device, seed, step)
            total += masked_update_(n, o, m, seed, salt=step * 1000003 + k)
        else:
            p = tensor_density(wl, spec, act)
            if p <= 0.0 and not want_masks:
                n.copy_(o)
                continue
            c, m = iid_update_(n, o, p, seed, salt=step * 1000003 + k, want_mask=want_masks)
            total += c
        if want_masks:
            masks.append(m)
    return total, (masks if want_masks else None)


def master_from_(master_flat: torch.Tensor, w_flat: torch.Tensor, seed: int, salt: int = 0) -> None:
    """FP32 master weights that round (nearest even) to the given BF16 weights: master = w * (1 + u * 2^-10)
    with u uniform in (-1, 1).  The relative offset stays below half a BF16 ulp (2^-9 of the value at
    least), so the rounding gives w back; zeros stay zero."""
    n = w_flat.numel()
    for c, lo in enumerate(range(0, n, _CHUNK)):
        hi = min(n, lo + _CHUNK)
        g = _gen(w_flat.device, seed, salt, c, 6)
        u = torch.rand(hi - lo, generator=g, device=w_flat.device, dtype=torch.float32) * 2.0 - 1.0
        master_flat[lo:hi] = w_flat[lo:hi].float() * (1.0 + u * (2.0 ** -10))


# ----------------------------------------------------------------------------------------------
# FP8 stand-ins (Sec. 2.1 measures 0.0655 % changed elements at FP8 synchronisation precision)
# ----------------------------------------------------------------------------------------------

FP8_DENSITY = 0.000655


class ByteSet:
    """The tensors of a workload as one-byte patterns (FP8 E4M3), carved end to end from one uint8 slab."""

    def __init__(self, wl: Workload, device):
        self.wl = wl
        self.device = torch.device(device)
        self.flat = torch.empty(wl.numel, dtype=torch.uint8, device=self.device)
        self.tensors: List[torch.Tensor] = []
        off = 0
        for t in wl.tensors:
            self.tensors.append(self.flat[off:off + t.numel])
            off += t.numel

    @property
    def numels(self) -> List[int]:
        return [t.numel for t in self.wl.tensors]

    def copy_from(self, other: "ByteSet") -> None:
        self.flat.copy_(other.flat)

    def equal(self, other: "ByteSet") -> bool:
        return all(torch.equal(a, b) for a, b in zip(self.tensors, other.tensors) if a.numel())


def fill_base_fp8_(flat: torch.Tensor, seed: int, salt: int = 0) -> None:
    """flat (uint8, 1-D) <- the E4M3 patterns of N(0, 1), chunk by chunk (FP8 weights are stored with a scale
    factor that brings them into the format's range; the stand-in takes them already scaled)."""
    n = flat.numel()
    for c, lo in enumerate(range(0, n, _CHUNK)):
        hi = min(n, lo + _CHUNK)
        g = _gen(flat.device, seed, salt, c, 7)
        x = torch.randn(hi - lo, generator=g, device=flat.device, dtype=torch.float32)
        flat[lo:hi] = x.to(torch.float8_e4m3fn).view(torch.uint8)


def iid_update_fp8_(new_flat: torch.Tensor, old_flat: torch.Tensor, p: float, seed: int, salt: int = 0
                    ) -> Tuple[int, torch.Tensor]:
    """new <- old with iid Bernoulli(p) positions moved to a neighbouring E4M3 value: one step in pattern space,
    up or down at random, away from zero at +-0 and downwards from the largest finite magnitude (0x7E), so that
    no NaN pattern (0x7F / 0xFF) appears and every masked position differs.  Returns (#changed, mask)."""
    n = old_flat.numel()
    changed = 0
    masks = []
    for c, lo in enumerate(range(0, n, _CHUNK)):
        hi = min(n, lo + _CHUNK)
        g = _gen(old_flat.device, seed, salt, c, 8)
        mask = torch.rand(hi - lo, generator=g, device=old_flat.device) < p
        up = torch.rand(hi - lo, generator=g, device=old_flat.device) < 0.5
        ob = old_flat[lo:hi].to(torch.int32)
        sign, mag = ob & 0x80, ob & 0x7F
        step = torch.where(up, torch.ones_like(mag), -torch.ones_like(mag))
        step = torch.where(mag == 0, torch.ones_like(mag), step)
        step = torch.where(mag >= 0x7E, -torch.ones_like(mag), step)
        nb = torch.where(mask, sign | (mag + step), ob)
        new_flat[lo:hi] = nb.to(torch.uint8)
        changed += int(mask.sum().item())
        masks.append(mask)
    return changed, torch.cat(masks) if masks else torch.zeros(0, dtype=torch.bool, device=old_flat.device)


def payload_capacity(wl: Workload, max_bucket_count: Optional[int] = None) -> int:
    """Per-bucket payload slots: from the known worst bucket when given, else 1.25 * p * be + 4096
    (five sigma of an iid 1 % bucket of 33.5 M elements is under 3000)."""
    if max_bucket_count is not None:
        return int(max_bucket_count) + 64
    return int(1.25 * wl.density * wl.bucket_elems) + 4096
