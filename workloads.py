"""Seeded synthetic inputs and workload shapes.

Shared by the tests, the benchmark and the smoke check as the single source of
inputs for BOTH the HIP path and the CPU oracle.  It holds shapes and random
draws only -- none of the method's arithmetic.

Recipe (stands in for the public image datasets the paper trains on: CIFAR-shaped
3x32x32 inputs with 10/100 classes, ImageNet-shaped 3x224x224 with 1000 classes):
  * block input x0 ~ N(0,1), ``numpy.random.default_rng(seed_x)`` drawn in
    float64 and rounded to float32;
  * conv weights He-normal, std = sqrt(2 / (C_in*kh*kw)), seed_w;
  * BN gamma = 1, beta = 0 (``affine="ones"``) or gamma = 1 + 0.25 N(0,1),
    beta = 0.25 N(0,1) (``affine="random"``, used by tests so that no gradient
    path is degenerate);
  * gradient of the block output / loss weights dy ~ N(0,1), seed_t.
Tensors are drawn layer by layer in a fixed order so a shape always gets the
same numbers.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Tuple

import numpy as np

PARAM_NAMES = ("g1", "b1", "W1", "g2", "b2", "W3")


@dataclass(frozen=True)
class BlockCfg:
    n: int
    c0: int
    h: int
    w: int
    layers: int
    growth: int
    bottleneck: int  # B (normally 4*growth); 0 = no bottleneck
    eps: float = 1e-5

    @property
    def c_out(self) -> int:
        return self.c0 + self.layers * self.growth

    def c_in(self, layer: int) -> int:  # layer is 1-based
        return self.c0 + (layer - 1) * self.growth

    @property
    def pixels(self) -> int:
        return self.n * self.h * self.w


def param_shapes(cfg: BlockCfg, layer: int) -> Dict[str, Tuple[int, ...]]:
    c, k, B = cfg.c_in(layer), cfg.growth, cfg.bottleneck
    if B > 0:
        return {"g1": (c,), "b1": (c,), "W1": (B, c), "g2": (B,), "b2": (B,), "W3": (k, B, 3, 3)}
    return {"g1": (c,), "b1": (c,), "W3": (k, c, 3, 3)}


def make_block_inputs(cfg: BlockCfg, seed_x: int = 0, seed_w: int = 1, seed_t: int = 2,
                      affine: str = "ones"):
    """Returns (x0, layer_params, dy): float32 numpy arrays, NCHW.

    ``layer_params[l-1]`` is a dict name -> array for layer l (names as in
    PARAM_NAMES; W1/g2/b2 absent without a bottleneck).
    """
    rx = np.random.default_rng(seed_x)
    rw = np.random.default_rng(seed_w)
    rt = np.random.default_rng(seed_t)
    x0 = rx.standard_normal((cfg.n, cfg.c0, cfg.h, cfg.w)).astype(np.float32)
    layers: List[Dict[str, np.ndarray]] = []
    for l in range(1, cfg.layers + 1):
        p: Dict[str, np.ndarray] = {}
        for name, shp in param_shapes(cfg, l).items():
            if name.startswith("W"):
                fan_in = int(np.prod(shp[1:]))
                p[name] = (rw.standard_normal(shp) * np.sqrt(2.0 / fan_in)).astype(np.float32)
            elif name.startswith("g"):
                if affine == "random":
                    p[name] = (1.0 + 0.25 * rw.standard_normal(shp)).astype(np.float32)
                else:
                    p[name] = np.ones(shp, dtype=np.float32)
            else:
                if affine == "random":
                    p[name] = (0.25 * rw.standard_normal(shp)).astype(np.float32)
                else:
                    p[name] = np.zeros(shp, dtype=np.float32)
        layers.append(p)
    dy = rt.standard_normal((cfg.n, cfg.c_out, cfg.h, cfg.w)).astype(np.float32)
    return x0, layers, dy


# --------------------------------------------------------------- workloads

def config1() -> BlockCfg:
    """Single small dense block (fp32): batch 2, 16 channels in, 8x8, 4 layers, k=12, B=48."""
    return BlockCfg(n=2, c0=16, h=8, w=8, layers=4, growth=12, bottleneck=48)


def densenet_bc_blocks(depth: int, growth: int, batch: int, image: int = 32) -> List[BlockCfg]:
    """Dense blocks of a CIFAR-shaped DenseNet-BC: stem to 2k channels, three
    blocks of (depth-4)/6 bottleneck layers, compression 0.5, 2x2 pooling between."""
    per = (depth - 4) // 6
    c, s, out = 2 * growth, image, []
    for _ in range(3):
        out.append(BlockCfg(batch, c, s, s, per, growth, 4 * growth))
        c = (c + per * growth) // 2
        s //= 2
    return out


def imagenet_blocks(layers: Tuple[int, ...], growth: int, stem: int, batch: int) -> List[BlockCfg]:
    """Dense blocks of an ImageNet-shaped DenseNet: stride-2 stem + stride-2 pool
    take 224 to 56; compression 0.5 and 2x2 pooling between blocks."""
    c, s, out = stem, 56, []
    for m in layers:
        out.append(BlockCfg(batch, c, s, s, m, growth, 4 * growth))
        c = (c + m * growth) // 2
        s //= 2
    return out


def config2(batch: int = 64) -> List[BlockCfg]:
    """DenseNet-BC L=100 k=12 (fp32), batch 64, 32x32 inputs."""
    return densenet_bc_blocks(100, 12, batch)


def config3(batch: int = 64) -> List[BlockCfg]:
    """DenseNet-BC L=250 k=24 (fp32), batch 64."""
    return densenet_bc_blocks(250, 24, batch)


def config4(batch: int = 32) -> List[BlockCfg]:
    """DenseNet-161-shaped (k=48, blocks 6-12-36-24, stem 96), batch 32."""
    return imagenet_blocks((6, 12, 36, 24), 48, 96, batch)


def config5(batch: int = 32) -> List[BlockCfg]:
    """DenseNet-264-shaped (k=32, blocks 6-12-64-48, stem 64), batch 32."""
    return imagenet_blocks((6, 12, 64, 48), 32, 64, batch)


# --------------------------------------------------------------- whole CIFAR-shaped networks

@dataclass(frozen=True)
class NetCfg:
    """DenseNet-BC on square 3-channel images: stem to 2k channels, three dense blocks of
    (depth-4)/6 bottleneck layers (B = 4k), transitions with compression 0.5, linear head."""
    n: int
    image: int
    depth: int
    growth: int
    classes: int
    eps: float = 1e-5

    def blocks(self) -> List[BlockCfg]:
        return [BlockCfg(b.n, b.c0, b.h, b.w, b.layers, b.growth, b.bottleneck, self.eps)
                for b in densenet_bc_blocks(self.depth, self.growth, self.n, self.image)]


def make_net_inputs(cfg: NetCfg, seed_x: int = 0, seed_w: int = 1, seed_t: int = 2, affine: str = "ones"):
    """Returns (x, labels, params): x (n,3,image,image) float32 ~ N(0,1); labels int32 uniform in
    [0, classes); params a dict: 'stem' (2k,3,3,3); 'block0..2' lists of per-layer dicts as in
    make_block_inputs; 'trans0', 'trans1' dicts g, b, W (C/2, C); 'tail' dict g, b, Wl
    (classes, C), bl (zeros).  Conv and linear weights He-normal, BN affine as in
    make_block_inputs."""
    rx = np.random.default_rng(seed_x)
    rw = np.random.default_rng(seed_w)
    rt = np.random.default_rng(seed_t)
    x = rx.standard_normal((cfg.n, 3, cfg.image, cfg.image)).astype(np.float32)
    labels = rt.integers(0, cfg.classes, size=cfg.n).astype(np.int32)

    def he(shape):
        return (rw.standard_normal(shape) * np.sqrt(2.0 / int(np.prod(shape[1:])))).astype(np.float32)

    def gam(c):
        return (1.0 + 0.25 * rw.standard_normal(c)).astype(np.float32) if affine == "random" else np.ones(c, np.float32)

    def bet(c):
        return (0.25 * rw.standard_normal(c)).astype(np.float32) if affine == "random" else np.zeros(c, np.float32)

    params = {"stem": he((2 * cfg.growth, 3, 3, 3))}
    for b, bc in enumerate(cfg.blocks()):
        _, layers, _ = make_block_inputs(bc, seed_x + 100 + b, seed_w + 100 + b, seed_t + 100 + b, affine)
        params[f"block{b}"] = layers
        c = bc.c_out
        if b < 2:
            params[f"trans{b}"] = {"g": gam(c), "b": bet(c), "W": he((c // 2, c))}
        else:
            params["tail"] = {"g": gam(c), "b": bet(c), "Wl": he((cfg.classes, c)),
                              "bl": np.zeros(cfg.classes, np.float32)}
    return x, labels, params


def net_config2(batch: int = 64) -> NetCfg:
    """DenseNet-BC L=100 k=12, 32x32 inputs, 10 classes."""
    return NetCfg(batch, 32, 100, 12, 10)


def net_config3(batch: int = 64) -> NetCfg:
    """DenseNet-BC L=250 k=24, 32x32 inputs, 100 classes."""
    return NetCfg(batch, 32, 250, 24, 100)


# --------------------------------------------------------------- whole ImageNet-shaped networks

@dataclass(frozen=True)
class InetCfg:
    """ImageNet-shaped DenseNet-BC on square 3-channel images: 7x7 stride-2 stem to 2k channels,
    BN-ReLU, 3x3 stride-2 max pool, four dense blocks of layers[b] bottleneck layers (B = 4k),
    transitions with compression 0.5 and 2x2 average pooling, linear head."""
    n: int
    image: int
    growth: int
    layers: Tuple[int, int, int, int]
    classes: int
    eps: float = 1e-5

    def blocks(self) -> List[BlockCfg]:
        c, s, out = 2 * self.growth, self.image // 4, []
        for m in self.layers:
            out.append(BlockCfg(self.n, c, s, s, m, self.growth, 4 * self.growth, self.eps))
            c = (c + m * self.growth) // 2
            s //= 2
        return out


def make_inet_inputs(cfg: InetCfg, seed_x: int = 0, seed_w: int = 1, seed_t: int = 2, affine: str = "ones"):
    """Returns (x, labels, params): x (n,3,image,image) float32 ~ N(0,1); labels int32 uniform in
    [0, classes); params a dict: 'stem' dict W (2k,3,7,7), g, b; 'block0..3' lists of per-layer dicts
    as in make_block_inputs; 'trans0..2' dicts g, b, W (C/2, C); 'tail' dict g, b, Wl (classes, C),
    bl (zeros).  Conv and linear weights He-normal, BN affine as in make_block_inputs."""
    rx = np.random.default_rng(seed_x)
    rw = np.random.default_rng(seed_w)
    rt = np.random.default_rng(seed_t)
    x = rx.standard_normal((cfg.n, 3, cfg.image, cfg.image)).astype(np.float32)
    labels = rt.integers(0, cfg.classes, size=cfg.n).astype(np.int32)

    def he(shape):
        return (rw.standard_normal(shape) * np.sqrt(2.0 / int(np.prod(shape[1:])))).astype(np.float32)

    def gam(c):
        return (1.0 + 0.25 * rw.standard_normal(c)).astype(np.float32) if affine == "random" else np.ones(c, np.float32)

    def bet(c):
        return (0.25 * rw.standard_normal(c)).astype(np.float32) if affine == "random" else np.zeros(c, np.float32)

    cs = 2 * cfg.growth
    params = {"stem": {"W": he((cs, 3, 7, 7)), "g": gam(cs), "b": bet(cs)}}
    for b, bc in enumerate(cfg.blocks()):
        tiny = BlockCfg(1, bc.c0, 1, 1, bc.layers, bc.growth, bc.bottleneck, bc.eps)   # the parameters do not depend on n, h, w
        _, layers, _ = make_block_inputs(tiny, seed_x + 100 + b, seed_w + 100 + b, seed_t + 100 + b, affine)
        params[f"block{b}"] = layers
        c = bc.c_out
        if b < 3:
            params[f"trans{b}"] = {"g": gam(c), "b": bet(c), "W": he((c // 2, c))}
        else:
            params["tail"] = {"g": gam(c), "b": bet(c), "Wl": he((cfg.classes, c)),
                              "bl": np.zeros(cfg.classes, np.float32)}
    return x, labels, params


def inet_config4(batch: int = 32) -> InetCfg:
    """DenseNet-161-shaped: k = 48, blocks 6-12-36-24, 224x224 inputs, 1000 classes."""
    return InetCfg(batch, 224, 48, (6, 12, 36, 24), 1000)


def inet_config5(batch: int = 32) -> InetCfg:
    """DenseNet-264-shaped: k = 32, blocks 6-12-64-48, 224x224 inputs, 1000 classes."""
    return InetCfg(batch, 224, 32, (6, 12, 64, 48), 1000)
