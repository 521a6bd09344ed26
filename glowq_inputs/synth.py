"""Seeded synthetic workloads shaped like the paper's inference setting.

The paper runs W4A16 (INT4 weights, group size 128, 16-bit activations) with
rank-64 corrections on Llama checkpoints (Sec. 4.1) and reports heavy-tailed,
anisotropic input spectra for the grouped modules (Sec. 3.1, Fig. 2).  Neither
the checkpoints nor the prompts are available, so the inputs drawn here stand
in for them: Gaussian weights of the Llama layer shapes and activations whose
channels carry log-normal scales plus a few large outlier channels.

Nothing in this file quantises, packs, factorises or multiplies: it draws
numbers and converts them to 16-bit storage with library casts, nothing more.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Sequence, Tuple

import numpy as np

WEIGHT_STD = 0.02          # W ~ N(0, 0.02^2)
CHANNEL_LOG_SIGMA = 0.5    # per-channel scale exp(0.5 * g), g ~ N(0, 1)
OUTLIER_FRACTION = 0.01    # 1 % of the input channels ...
OUTLIER_GAIN = 20.0        # ... are multiplied by 20


@dataclass(frozen=True)
class UnitShape:
    """One unit of the restore policy (Sec. 3.3): an input-sharing group
    (q/k/v or gate/up) or a solo module (o_proj, down_proj)."""

    name: str
    d_in: int
    d_outs: Tuple[int, ...]

    @property
    def n_modules(self) -> int:
        return len(self.d_outs)

    @property
    def rows(self) -> int:
        return int(sum(self.d_outs))


def _llama_block(hidden: int, inter: int, kv: int) -> List[UnitShape]:
    return [
        UnitShape("qkv", hidden, (hidden, kv, kv)),
        UnitShape("o", hidden, (hidden,)),
        UnitShape("gate_up", hidden, (inter, inter)),
        UnitShape("down", inter, (hidden,)),
    ]


# The five workloads.  "T" lists the token counts each one is run at; "act" is
# the 16-bit activation type ("f16" or "bf16"); "G" the quantisation group size.
CONFIGS: Dict[int, dict] = {
    1: dict(name="tiny", seed=0, r=16, G=64, act="f16", T=(16,), outliers=False,
            layers=1, block=[UnitShape("qkv", 256, (256, 256, 256))]),
    2: dict(name="llama2-7b-qkv-decode", seed=2, r=64, G=128, act="f16",
            T=(1, 2, 4, 8, 16), outliers=True, layers=1,
            block=[UnitShape("qkv", 4096, (4096, 4096, 4096))]),
    3: dict(name="llama2-7b-gateup-prefill", seed=3, r=64, G=128, act="bf16",
            T=(2048,), outliers=True, layers=1,
            block=[UnitShape("gate_up", 4096, (11008, 11008))]),
    4: dict(name="llama3-8b-block", seed=4, r=128, G=128, act="f16", T=(512,),
            outliers=True, layers=1, block=_llama_block(4096, 14336, 1024)),
    5: dict(name="llama2-13b-glowq-s-stack", seed=5, r=64, G=128, act="f16",
            T=(1, 1024), outliers=True, layers=40,
            block=_llama_block(5120, 13824, 5120),
            restore_fraction=0.25, mask_seed=5),
}


def config_units(cfg_id: int) -> List[UnitShape]:
    """All units of a workload, layer after layer, in execution order."""
    cfg = CONFIGS[cfg_id]
    return [u for _ in range(cfg["layers"]) for u in cfg["block"]]


# --------------------------------------------------------------------------
# 16-bit storage casts (library conversions, round-to-nearest-even)
# --------------------------------------------------------------------------
def to_act_bits(values: np.ndarray, act: str) -> np.ndarray:
    """Round float values to fp16 / bf16 and return the uint16 bit patterns."""
    v32 = np.ascontiguousarray(values, dtype=np.float32)
    if act == "f16":
        return v32.astype(np.float16).view(np.uint16)
    if act == "bf16":
        import torch

        t = torch.from_numpy(v32).to(torch.bfloat16)
        return t.view(torch.int16).numpy().view(np.uint16).copy()
    raise ValueError(f"unknown activation type {act!r}")


def from_act_bits(bits: np.ndarray, act: str) -> np.ndarray:
    """Widen fp16 / bf16 bit patterns to float64 (exact)."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    if act == "f16":
        return b.view(np.float16).astype(np.float64)
    if act == "bf16":
        return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    raise ValueError(f"unknown activation type {act!r}")


# --------------------------------------------------------------------------
# recipe inputs: full-precision weights and anisotropic activations
# --------------------------------------------------------------------------
def _rng(*key: int) -> np.random.Generator:
    return np.random.default_rng(np.random.SeedSequence([int(k) for k in key]))


def gen_module_weight(seed: int, unit: int, module: int, d_out: int,
                      d_in: int) -> np.ndarray:
    """fp32 W[d_out][d_in] ~ N(0, 0.02^2); stream keyed by (seed, unit, module)."""
    rng = _rng(seed, unit, module, 101)
    w = rng.standard_normal((d_out, d_in), dtype=np.float32)
    w *= np.float32(WEIGHT_STD)
    return w


def gen_activations(seed: int, unit: int, T: int, d_in: int, act: str,
                    outliers: bool = True) -> np.ndarray:
    """uint16 bit patterns of X[T][d_in] in the activation type.

    X[t][k] = c_k * n_tk with c_k = exp(0.5 g_k), g, n ~ N(0, 1); when
    `outliers` is set, floor(0.01 d_in) seeded channels get c_k *= 20.
    """
    rng = _rng(seed, unit, 202)
    g = rng.standard_normal(d_in)
    c = np.exp(CHANNEL_LOG_SIGMA * g)
    if outliers:
        n_out = int(np.floor(OUTLIER_FRACTION * d_in))
        idx = rng.permutation(d_in)[:n_out]
        c[idx] *= OUTLIER_GAIN
    n = rng.standard_normal((T, d_in), dtype=np.float32)
    x = n * c.astype(np.float32)[None, :]
    return to_act_bits(x, act)


def gen_restore_mask(seed: int, n_units: int, fraction: float) -> np.ndarray:
    """uint8 mask with exactly round(fraction * n_units) ones: the first
    entries of a seeded permutation (stands in for the top-k of Sec. 3.3)."""
    k = int(round(fraction * n_units))
    perm = _rng(seed, 303).permutation(n_units)
    mask = np.zeros(n_units, dtype=np.uint8)
    mask[perm[:k]] = 1
    return mask


# --------------------------------------------------------------------------
# direct inputs: already-quantised bytes with matched value distributions
# --------------------------------------------------------------------------
def gen_direct_unit(seed: int, unit: int, shape: UnitShape, T: int, r: int,
                    G: int, act: str, device: str = "cpu") -> dict:
    """Random stored operands of one unit, drawn directly in storage form.

    For workloads whose full-precision weights would not fit a test's time
    budget (tens of GB of fp32), the stored operands are drawn with the value
    distributions the recipe path produces instead of being derived:
    nibbles uniform in [0, 15]; scales ~ 0.0073 * exp(0.1 n) (the (max-min)/15
    of 128 N(0, 0.02^2) samples); integer zero-points uniform in [5, 10];
    factors N(0, sigma/rows) and N(0, sigma/d_in) with sigma the size of the
    leading singular value of a quantisation-noise matrix of that shape; X as
    in `gen_activations` with outlier channels.  Returns torch tensors on
    `device`: wq int32 [O][d_in/8] per module (canonical words), scales and
    zeros float16 [O][d_in/G], A [O][r], B [r][d_in], X [T][d_in] in `act`.
    """
    import torch

    tdt = {"f16": torch.float16, "bf16": torch.bfloat16}[act]
    gen = torch.Generator(device=device)
    gen.manual_seed((int(seed) * 1000003 + int(unit)) * 7919 + 404)
    d_in = shape.d_in
    e_std = 0.0073 / np.sqrt(12.0)
    sigma = e_std * (np.sqrt(shape.rows) + np.sqrt(d_in))
    out = {"modules": []}
    for d_out in shape.d_outs:
        wq = torch.randint(-2**31, 2**31 - 1, (d_out, d_in // 8), generator=gen,
                           device=device, dtype=torch.int64).to(torch.int32)
        sc = 0.0073 * torch.exp(0.1 * torch.randn(d_out, d_in // G, generator=gen,
                                                  device=device))
        zp = torch.randint(5, 11, (d_out, d_in // G), generator=gen, device=device)
        A = torch.randn(d_out, r, generator=gen, device=device) * float(
            np.sqrt(sigma / shape.rows))
        out["modules"].append(dict(
            wq=wq, scales=sc.to(torch.float16), zeros=zp.to(torch.float16),
            A=A.to(tdt), d_out=d_out))
    B = torch.randn(r, d_in, generator=gen, device=device) * float(np.sqrt(sigma / d_in))
    c = torch.exp(CHANNEL_LOG_SIGMA * torch.randn(d_in, generator=gen, device=device))
    n_out = int(np.floor(OUTLIER_FRACTION * d_in))
    idx = torch.randperm(d_in, generator=gen, device=device)[:n_out]
    c[idx] *= OUTLIER_GAIN
    X = torch.randn(T, d_in, generator=gen, device=device) * c[None, :]
    out["B"] = B.to(tdt)
    out["X"] = X.to(tdt)
    return out


def gen_direct_layerwise_B(seed: int, unit: int, shape: UnitShape, r: int, act: str,
                           device: str = "cpu") -> list:
    """One right factor per module, [r][d_in] each, drawn like the shared B of
    `gen_direct_unit` (same scale, different stream per module): the operands the
    layer-wise comparison mode reads in the place of the shared factor."""
    import torch

    tdt = {"f16": torch.float16, "bf16": torch.bfloat16}[act]
    d_in = shape.d_in
    e_std = 0.0073 / np.sqrt(12.0)
    out = []
    for i, d_out in enumerate(shape.d_outs):
        gen = torch.Generator(device=device)
        gen.manual_seed(((int(seed) * 1000003 + int(unit)) * 7919 + 505) * 31 + i)
        sigma = e_std * (np.sqrt(d_out) + np.sqrt(d_in))
        B = torch.randn(r, d_in, generator=gen, device=device) * float(np.sqrt(sigma / d_in))
        out.append(B.to(tdt))
    return out
