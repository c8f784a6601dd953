"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

This module holds NO arithmetic of the method: it only draws random tensors of the
shapes, value sets and densities of the workloads (U-Net-shaped feature maps with
+-1 activations, ternary weights with a Bernoulli keep mask, integer thresholds,
N(0,1) images), and lists the channel plan of the network.  Both the CPU oracle and
the HIP library are fed from here, so random-number portability never matters.

The tensors stand in for the paper's segmentation datasets and trained weights
(Sec. 4.1; Sec. 3.1.1 reports the sparsity range of trained masks), which are not
available; everything is generated from (config id, seed, layer index, tensor id).
"""
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

# tensor ids inside one layer's random stream
_ACT, _SIGN, _KEEP, _THETA, _IMG, _STEMW, _CLSW, _CLSB, _KEEPP = range(9)


def _rng(config_id: int, seed: int, layer: int, tensor: int) -> np.random.Generator:
    return np.random.default_rng([config_id, seed, layer, tensor])


def pm1_bits(rng: np.random.Generator, shape) -> np.ndarray:
    """Bernoulli(0.5) values in {-1,+1} as int8."""
    b = rng.integers(0, 2, size=shape, dtype=np.int8)
    b *= 2
    b -= 1
    return b


def ternary_weights(config_id: int, seed: int, layer: int, cout: int, cin: int,
                    keep: float) -> np.ndarray:
    """OHWI [cout,3,3,cin] int8: sign Bernoulli(0.5), kept with probability `keep`."""
    sign = pm1_bits(_rng(config_id, seed, layer, _SIGN), (cout, 3, 3, cin))
    kept = _rng(config_id, seed, layer, _KEEP).random((cout, 3, 3, cin), dtype=np.float32) < keep
    return (sign * kept).astype(np.int8)


def thresholds(config_id: int, seed: int, layer: int, cout: int, bound: int) -> np.ndarray:
    """int32 [cout], uniform on the integers -bound..+bound inclusive."""
    return _rng(config_id, seed, layer, _THETA).integers(-bound, bound + 1, size=cout,
                                                         dtype=np.int32)


def activations(config_id: int, seed: int, layer: int, n: int, h: int, w: int,
                c: int) -> np.ndarray:
    """NHWC int8 in {-1,+1}, Bernoulli(0.5)."""
    return pm1_bits(_rng(config_id, seed, layer, _ACT), (n, h, w, c))


@dataclass
class ConvCase:
    a: np.ndarray       # [N,H,W,Cin] int8 +-1
    w: np.ndarray       # [Cout,3,3,Cin] int8 ternary
    theta: np.ndarray   # [Cout] int32
    keep: float


def conv_case(config_id: int, seed: int, n: int, h: int, w: int, cin: int, cout: int,
              keep: float, theta_bound: Optional[int] = None, layer: int = 0) -> ConvCase:
    """One masked-binary 3x3 layer's inputs.  theta_bound defaults to floor(9*cin/16)."""
    if theta_bound is None:
        theta_bound = (9 * cin) // 16
    return ConvCase(a=activations(config_id, seed, layer, n, h, w, cin),
                    w=ternary_weights(config_id, seed, layer, cout, cin, keep),
                    theta=thresholds(config_id, seed, layer, cout, theta_bound),
                    keep=keep)


def ternary_tconv_weights(config_id: int, seed: int, layer: int, cout: int, cin: int,
                          keep: float) -> np.ndarray:
    """[cout,2,2,cin] int8 for the 2x2 stride-2 transposed layer."""
    sign = pm1_bits(_rng(config_id, seed, layer, _SIGN), (cout, 2, 2, cin))
    kept = _rng(config_id, seed, layer, _KEEP).random((cout, 2, 2, cin), dtype=np.float32) < keep
    return (sign * kept).astype(np.int8)


def unet_channel_plan(base: int = 64, levels: int = 4,
                      transposed: bool = False) -> List[Tuple[str, int, int, int]]:
    """(name, cin, cout, level) of every masked-binary 3x3 layer in execution order.

    `level` is the resolution level (1 = full resolution, levels+1 = bottleneck).
    Encoder level l: two convs ending at base*2^(l-1) channels.  Bottleneck: doubles
    once more.  Decoder level l: the up-sampled feature keeps its channel count
    (nearest-neighbour up-sampling), so the first conv sees skip + up channels.  With
    transposed=True the decoder up-samples with a transposed layer that maps 2c -> c
    channels (not listed here), so the first conv sees c + c channels.
    """
    plan = []
    c_prev = base
    for l in range(1, levels + 1):
        c = base << (l - 1)
        plan.append((f"enc{l}a", c_prev, c, l))
        plan.append((f"enc{l}b", c, c, l))
        c_prev = c
    c_mid = base << levels
    plan.append(("mida", c_prev, c_mid, levels + 1))
    plan.append(("midb", c_mid, c_mid, levels + 1))
    c_up = c_mid
    for l in range(levels, 0, -1):
        c = base << (l - 1)
        if transposed:
            c_up = c          # the transposed layer halves the channel count (Sec. 2.1)
        plan.append((f"dec{l}a", c + c_up, c, l))
        plan.append((f"dec{l}b", c, c, l))
        c_up = c
    return plan


@dataclass
class UNetCase:
    image: np.ndarray                  # [N,3,H,W] float32
    stem_w: np.ndarray                 # [base,3,3,3] float32 (O,ky,kx,ci)
    convs: List[Tuple[np.ndarray, np.ndarray]]   # (w OHWI int8, theta int32) per layer
    cls_w: np.ndarray                  # [n_classes, base] float32
    cls_b: np.ndarray                  # [n_classes] float32
    plan: List[Tuple[str, int, int, int]]
    keeps: List[float]
    levels: int
    base: int
    n_classes: int
    up_convs: Optional[List[Tuple[np.ndarray, np.ndarray]]] = None   # transposed decoder


def cost_aware_zero_fractions(plan, h: int, w: int, mean_zero: float) -> List[float]:
    """Per-layer zero fraction for the sparsity-stress workload: layers with a higher
    cost score (Sec. 3.1.2: equal-weight sum of min-max normalised operation count
    and parameter count) get more zeros; spread 0.2 around `mean_zero`, clamped."""
    ops = np.array([2.0 * (h >> (lv - 1)) * (w >> (lv - 1)) * 9 * ci * co
                    for _, ci, co, lv in plan])
    par = np.array([9.0 * ci * co for _, ci, co, _ in plan])

    def norm(v):
        return (v - v.min()) / (v.max() - v.min())

    s = 0.5 * norm(ops) + 0.5 * norm(par)
    z = np.clip(mean_zero + 0.2 * (s - s.mean()), 0.02, 0.98)
    return [float(v) for v in z]


def unet_case(config_id: int, seed: int, n: int, h: int, w: int, base: int = 64,
              levels: int = 4, n_classes: int = 19,
              keep: Optional[float] = None,
              keeps: Optional[Sequence[float]] = None,
              transposed: bool = False) -> UNetCase:
    """Whole-network inputs.  keep=None and keeps=None draws each layer's keep
    probability uniformly in [0.4, 0.8]; thresholds are uniform in +-floor(9*cin/16)."""
    plan = unet_channel_plan(base, levels, transposed)
    image = _rng(config_id, seed, 0, _IMG).standard_normal((n, 3, h, w), dtype=np.float32)
    stem_w = _rng(config_id, seed, 0, _STEMW).standard_normal((base, 3, 3, 3), dtype=np.float32)
    convs, used = [], []
    for i, (_, ci, co, _) in enumerate(plan):
        if keeps is not None:
            k = float(keeps[i])
        elif keep is not None:
            k = float(keep)
        else:
            k = float(_rng(config_id, seed, i + 1, _KEEPP).uniform(0.4, 0.8))
        used.append(k)
        convs.append((ternary_weights(config_id, seed, i + 1, co, ci, k),
                      thresholds(config_id, seed, i + 1, co, (9 * ci) // 16)))
    cls_w = (_rng(config_id, seed, 0, _CLSW).standard_normal((n_classes, base), dtype=np.float32)
             / np.float32(8.0))
    cls_b = _rng(config_id, seed, 0, _CLSB).standard_normal((n_classes,), dtype=np.float32)
    up_convs = None
    if transposed:
        up_convs = []
        for j, l in enumerate(range(levels, 0, -1)):
            c = base << (l - 1)
            k = float(keep) if keep is not None else 0.6
            up_convs.append((ternary_tconv_weights(config_id, seed, 100 + j, c, 2 * c, k),
                             thresholds(config_id, seed, 100 + j, c, (2 * c) // 8)))
    return UNetCase(up_convs=up_convs, image=image, stem_w=stem_w, convs=convs, cls_w=cls_w, cls_b=cls_b,
                    plan=plan, keeps=used, levels=levels, base=base, n_classes=n_classes)


def conv_macs(n: int, h: int, w: int, cin: int, cout: int) -> int:
    """Dense-equivalent multiply-accumulates of one 3x3 layer (masked and padded taps
    counted; Sec. 3.1.2 counts a multiply and an add as two operations)."""
    return n * h * w * 9 * cin * cout


def unet_conv_macs(plan, n: int, h: int, w: int) -> int:
    return sum(conv_macs(n, h >> (lv - 1), w >> (lv - 1), ci, co) for _, ci, co, lv in plan)
