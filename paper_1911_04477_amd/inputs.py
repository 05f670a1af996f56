"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

This module only draws random tensors and describes workload shapes.  It holds
none of the method's arithmetic (no sign, no packing, no convolution): both the
CPU oracle and the HIP path receive the very same host-generated float arrays.

The paper measured on the CIFAR-10 test set with a trained network (section 4.1,
4.2); neither exists here, so CIFAR-/ImageNet-shaped i.i.d. tensors stand in.
Every tensor is drawn once on the host from a seeded CPU generator.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np
import torch

BASE_SEED = 191104477


def _gen(seed: int) -> torch.Generator:
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed))
    return g


def randn(shape, g: torch.Generator) -> np.ndarray:
    """i.i.d. N(0,1) fp32."""
    return torch.randn(*shape, generator=g, dtype=torch.float32).numpy()


def rand_scale(n: int, g: torch.Generator) -> np.ndarray:
    """Per-channel scale ~ U(0.5, 1.5), fp32."""
    return (torch.rand(n, generator=g, dtype=torch.float32) + 0.5).numpy()


def rand_bias(n: int, g: torch.Generator) -> np.ndarray:
    """Per-channel bias ~ N(0, 0.1^2), fp32."""
    return (torch.randn(n, generator=g, dtype=torch.float32) * 0.1).numpy()


_SPECIALS = np.array(
    [0.0, -0.0, 1e-45, -1e-45, 1.1754944e-38, -1.1754944e-38, np.nan, np.inf, -np.inf],
    dtype=np.float32,
)


def inject_specials(a: np.ndarray, seed: int, frac: float = 1e-3, with_nan: bool = True) -> np.ndarray:
    """Overwrite a seeded fraction of entries with values that stress the sign
    predicate: +0.0, -0.0, smallest denormals, smallest normals, NaN, +-inf.
    Returns a new array; at least one entry of each kind is planted when the
    array is large enough."""
    out = np.array(a, dtype=np.float32, copy=True)
    flat = out.reshape(-1)
    rng = np.random.default_rng(seed)
    pool = _SPECIALS if with_nan else _SPECIALS[~np.isnan(_SPECIALS)]
    n = max(int(flat.size * frac), min(flat.size, pool.size))
    if n == 0:
        return out
    pos = rng.choice(flat.size, size=n, replace=False)
    vals = pool[np.arange(n) % pool.size]
    flat[pos] = vals
    return out


# ----------------------------------------------------------------------------
# Workload descriptions (shapes only).
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class GemmShape:
    M: int
    N: int
    K: int


@dataclass(frozen=True)
class ConvShape:
    N: int
    C: int
    H: int
    W: int
    D: int
    kH: int
    kW: int
    sH: int = 1
    sW: int = 1
    pH: int = 0
    pW: int = 0

    @property
    def OH(self) -> int:
        return (self.H + 2 * self.pH - self.kH) // self.sH + 1

    @property
    def OW(self) -> int:
        return (self.W + 2 * self.pW - self.kW) // self.sW + 1

    @property
    def K(self) -> int:
        return self.C * self.kH * self.kW

    @property
    def P(self) -> int:
        return self.N * self.OH * self.OW

    @property
    def bit_macs(self) -> int:
        return self.D * self.P * self.K


CFG1 = GemmShape(M=64, N=64, K=256)
CFG2 = GemmShape(M=256, N=4096, K=4096)
CFG3 = ConvShape(N=128, C=128, H=32, W=32, D=128, kH=3, kW=3, sH=1, sW=1, pH=1, pW=1)
CFG5A = ConvShape(N=64, C=256, H=56, W=56, D=256, kH=3, kW=3, sH=1, sW=1, pH=1, pW=1)
CFG5B = ConvShape(N=64, C=200, H=56, W=56, D=256, kH=1, kW=1, sH=2, sW=2, pH=0, pW=0)


def cfg1(seed: int = BASE_SEED + 1) -> Dict[str, np.ndarray]:
    g = _gen(seed)
    return {"A": randn((CFG1.M, CFG1.K), g), "B": randn((CFG1.N, CFG1.K), g)}


def fc_inputs(shape: GemmShape, seed: int) -> Dict[str, np.ndarray]:
    """Activations [M,K], weights [N,K], per-output-feature scale/bias [N]."""
    g = _gen(seed)
    return {
        "act": randn((shape.M, shape.K), g),
        "wt": randn((shape.N, shape.K), g),
        "scale": rand_scale(shape.N, g),
        "bias": rand_bias(shape.N, g),
    }


def cfg2(seed: int = BASE_SEED + 2) -> Dict[str, np.ndarray]:
    return fc_inputs(CFG2, seed)


def conv_inputs(shape: ConvShape, seed: int, batch: Optional[int] = None) -> Dict[str, np.ndarray]:
    """x NCHW, w [D,C,kH,kW], per-output-channel scale/bias [D]."""
    g = _gen(seed)
    n = shape.N if batch is None else batch
    return {
        "x": randn((n, shape.C, shape.H, shape.W), g),
        "w": randn((shape.D, shape.C, shape.kH, shape.kW), g),
        "scale": rand_scale(shape.D, g),
        "bias": rand_bias(shape.D, g),
    }


def cfg3(seed: int = BASE_SEED + 3) -> Dict[str, np.ndarray]:
    return conv_inputs(CFG3, seed)


def cfg5a(seed: int = BASE_SEED + 5) -> Dict[str, np.ndarray]:
    return conv_inputs(CFG5A, seed)


def cfg5b(seed: int = BASE_SEED + 6) -> Dict[str, np.ndarray]:
    return conv_inputs(CFG5B, seed)


# ----------------------------------------------------------------------------
# Config 4: the VGG-small stack as a data table.
#
# The six widths 128-128-256-256-512-512 are read as the output widths of all
# six convolutions, the first of which (3->128) stays fp32; hence five binarized
# 3x3 convolutions, with a 2x2 max-pool after convolutions 2, 4 and 6
# (32 -> 16 -> 8 -> 4, 512*4*4 = 8192), a binarized FC 8192->1024 and an fp32
# FC 1024->10.  ``reading="B"`` inserts a sixth binarized conv 128->128 so that
# six binarized convs follow the fp32 one (pools after every second binarized
# conv).
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class StackLayer:
    kind: str  # "conv_f32" | "bconv" | "bfc" | "fc_f32"
    cin: int
    cout: int
    hw: int = 0  # input spatial size (square) for conv layers
    pool: bool = False  # 2x2/2 max-pool on this layer's int32 output


def vgg_small_layers(reading: str = "A") -> List[StackLayer]:
    if reading == "A":
        return [
            StackLayer("conv_f32", 3, 128, 32, pool=False),
            StackLayer("bconv", 128, 128, 32, pool=True),
            StackLayer("bconv", 128, 256, 16, pool=False),
            StackLayer("bconv", 256, 256, 16, pool=True),
            StackLayer("bconv", 256, 512, 8, pool=False),
            StackLayer("bconv", 512, 512, 8, pool=True),
            StackLayer("bfc", 8192, 1024),
            StackLayer("fc_f32", 1024, 10),
        ]
    if reading == "B":
        return [
            StackLayer("conv_f32", 3, 128, 32, pool=False),
            StackLayer("bconv", 128, 128, 32, pool=False),
            StackLayer("bconv", 128, 128, 32, pool=True),
            StackLayer("bconv", 128, 256, 16, pool=False),
            StackLayer("bconv", 256, 256, 16, pool=True),
            StackLayer("bconv", 256, 512, 8, pool=False),
            StackLayer("bconv", 512, 512, 8, pool=True),
            StackLayer("bfc", 8192, 1024),
            StackLayer("fc_f32", 1024, 10),
        ]
    raise ValueError("reading must be 'A' or 'B'")


def stack_bit_macs(layers: List[StackLayer], batch: int) -> int:
    total = 0
    for L in layers:
        if L.kind == "bconv":
            total += batch * L.hw * L.hw * L.cout * L.cin * 9
        elif L.kind == "bfc":
            total += batch * L.cin * L.cout
    return total


def cfg4(batch: int = 256, seed: int = BASE_SEED + 4, reading: str = "A") -> Dict[str, object]:
    """Input image batch and per-layer random parameters of the stack."""
    g = _gen(seed)
    layers = vgg_small_layers(reading)
    params = []
    x = randn((batch, 3, 32, 32), g)
    for L in layers:
        if L.kind in ("conv_f32", "bconv"):
            w = randn((L.cout, L.cin, 3, 3), g)
        else:
            w = randn((L.cout, L.cin), g)
        p = {"w": w}
        if L.kind != "fc_f32":
            p["scale"] = rand_scale(L.cout, g)
            p["bias"] = rand_bias(L.cout, g)
        else:
            p["bias"] = rand_bias(L.cout, g)
        params.append(p)
    return {"x": x, "layers": layers, "params": params}
