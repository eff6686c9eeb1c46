"""Workload shapes and seeded synthetic inputs.

This module holds none of the method's arithmetic: it only names the shapes of
the benchmark configurations (parameter counts and per-layer tensor layouts of
the ResNets the paper trains, Section 4.2) and draws seeded numpy inputs with
the value distributions of the noisy quadratic.  Both the GPU tests and the CPU
oracle are fed from here, so the two sides always see identical inputs.
"""
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np

DEFAULT_SEED = 0x161104581


# --------------------------------------------------------------------------
# Per-layer tensor layouts (segment tables)

def _resnet_tensors(block: str, layers: Tuple[int, ...], num_classes: int = 1000):
    """(name, numel, kind) for every parameter tensor of an ImageNet ResNet, in
    module order.  kind is one of conv, bn_gamma, bn_beta, fc_weight, fc_bias."""
    out = []

    def conv(name, cin, cout, ksz):
        out.append((name + ".weight", cout * cin * ksz * ksz, "conv"))

    def bn(name, c):
        out.append((name + ".weight", c, "bn_gamma"))
        out.append((name + ".bias", c, "bn_beta"))

    conv("conv1", 3, 64, 7)
    bn("bn1", 64)
    expansion = 4 if block == "bottleneck" else 1
    inplanes = 64
    for li, (planes, nblocks) in enumerate(zip((64, 128, 256, 512), layers)):
        for b in range(nblocks):
            stride = 2 if (b == 0 and li > 0) else 1
            p = "layer%d.%d" % (li + 1, b)
            if block == "bottleneck":
                conv(p + ".conv1", inplanes, planes, 1)
                bn(p + ".bn1", planes)
                conv(p + ".conv2", planes, planes, 3)
                bn(p + ".bn2", planes)
                conv(p + ".conv3", planes, planes * 4, 1)
                bn(p + ".bn3", planes * 4)
            else:
                conv(p + ".conv1", inplanes, planes, 3)
                bn(p + ".bn1", planes)
                conv(p + ".conv2", planes, planes, 3)
                bn(p + ".bn2", planes)
            if b == 0 and (stride != 1 or inplanes != planes * expansion):
                conv(p + ".downsample.0", inplanes, planes * expansion, 1)
                bn(p + ".downsample.1", planes * expansion)
            inplanes = planes * expansion
    out.append(("fc.weight", inplanes * num_classes, "fc_weight"))
    out.append(("fc.bias", num_classes, "fc_bias"))
    return out


_LR_SCALE = {"conv": 1.0, "bn_gamma": 1.0, "bn_beta": 2.0, "fc_weight": 1.0, "fc_bias": 2.0}


def resnet_layout(name: str):
    """Segment table of a ResNet laid out as back-to-back per-layer tensors:
    (seg_offsets int64[S+1], seg_lr_scale float32[S], names)."""
    if name == "resnet18":
        t = _resnet_tensors("basic", (2, 2, 2, 2))
    elif name == "resnet50":
        t = _resnet_tensors("bottleneck", (3, 4, 6, 3))
    else:
        raise ValueError(name)
    sizes = np.array([n for _, n, _ in t], dtype=np.int64)
    offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    scales = np.array([_LR_SCALE[kind] for _, _, kind in t], dtype=np.float32)
    return offsets, scales, [nm for nm, _, _ in t]


RESNET18_D = 11_689_512
RESNET50_D = 25_557_032


# --------------------------------------------------------------------------
# Benchmark / parity configurations

@dataclass
class Config:
    name: str
    rule: str                 # "gossip" | "gossip_stale" | "gossip_pull" | "gossip_push" | "async_tick" | "allreduce" | "easgd" | "local"
    k: int
    d: int
    steps: int
    sigma: float = 0.1
    lr: float = 0.05
    momentum: float = 0.9
    beta: float = 0.5         # gossip mixing weight
    alpha_e: Optional[float] = None   # EASGD moving rate
    layout: Optional[str] = None      # segmented layout name, None = flat
    seed: int = DEFAULT_SEED
    weight_decay: float = 0.0         # extras of the paper's training runs (Section 4.2)
    nesterov: bool = False
    tau: int = 1                      # communication period: exchange on every tau-th step, local steps between
    # matrix layout the benchmark runs the configuration in: 0 = row-major, else the blocked layout's columns per
    # block (16 Ki columns is where every rule's kernel streamed fastest or within a point of it on MI355X)
    block_columns: int = 0


CONFIGS = {
    "tiny": Config("tiny", "gossip", 4, 65_536, 100, sigma=0.01),
    "allreduce_r18": Config("allreduce_r18", "allreduce", 8, RESNET18_D, 200, block_columns=16384),
    "gossip_r18": Config("gossip_r18", "gossip", 32, RESNET18_D, 200, block_columns=16384),
    "gossip_r50": Config("gossip_r50", "gossip", 32, RESNET50_D, 200, block_columns=16384),
    "easgd_r50": Config("easgd_r50", "easgd", 16, RESNET50_D, 200, alpha_e=0.9 / 16, block_columns=16384),
    "seg_gossip_r50_k128": Config("seg_gossip_r50_k128", "gossip", 128, RESNET50_D, 100, layout="resnet50",
                                  block_columns=16384),
    # beyond the five benchmark configurations: the other gossip forms the paper describes, at the metric shape
    "pull_gossip_r50": Config("pull_gossip_r50", "gossip_pull", 32, RESNET50_D, 100, block_columns=16384),       # iid targets, Algorithm 3
    "push_gossip_r50": Config("push_gossip_r50", "gossip_push", 32, RESNET50_D, 100, block_columns=16384),       # Algorithm 4
    "stale_gossip_r50": Config("stale_gossip_r50", "gossip_stale", 32, RESNET50_D, 100, block_columns=16384),    # Section 6.2.1
    "async_r50": Config("async_r50", "async_tick", 32, RESNET50_D, 100),   # Section 6.1.2, one step = k ticks; one row per tick: row-major
    "local_r50": Config("local_r50", "local", 32, RESNET50_D, 100, block_columns=16384),                         # no exchange: tau -> infinity
    "paper_setup_r18": Config("paper_setup_r18", "gossip_push", 16, RESNET18_D, 100, lr=0.1,  # Section 4.2's recipe
                              weight_decay=1e-4, nesterov=True, tau=10, block_columns=16384),
}


def round_up(n: int, m: int) -> int:
    return (n + m - 1) // m * m


# --------------------------------------------------------------------------
# Seeded inputs (numpy's own generator: nothing here is the method's Philox)

@dataclass
class Inputs:
    x: np.ndarray        # (k, ld) parameters
    v: np.ndarray        # (k, ld) momentum buffers
    g: np.ndarray        # (k, ld) gradients
    xstar: np.ndarray    # (ld,) optimum of the quadratic
    h: np.ndarray        # (ld,) curvatures
    center: np.ndarray   # (ld,) EASGD centre
    x0: np.ndarray       # (ld,) common starting point
    d: int = 0
    ld: int = 0
    k: int = 0


def make_inputs(k: int, d: int, ld: Optional[int] = None, seed: int = 0, identical_rows: bool = False) -> Inputs:
    """x ~ N(0,1) per replica (or one shared row), v ~ 0.1 N(0,1), g ~ N(0,1),
    x* ~ N(0,1), h ~ U(0.1,1), centre ~ N(0,1).  Padding columns (d..ld) are
    filled with a sentinel so that a kernel touching them is caught."""
    ld = d if ld is None else ld
    assert ld >= d
    rng = np.random.default_rng(seed)

    def rows(scale):
        a = np.full((k, ld), 777.0, np.float32)
        a[:, :d] = (rng.standard_normal((k, d)) * scale).astype(np.float32)
        return a

    def vec(draw):
        a = np.full(ld, 777.0, np.float32)
        a[:d] = draw(d).astype(np.float32)
        return a

    x = rows(1.0)
    if identical_rows:
        x[:, :d] = x[0, :d]
    v = rows(0.1)
    g = rows(1.0)
    xstar = vec(rng.standard_normal)
    h = vec(lambda n: rng.uniform(0.1, 1.0, n))
    center = vec(rng.standard_normal)
    x0 = vec(rng.standard_normal)
    return Inputs(x, v, g, xstar, h, center, x0, d, ld, k)


def to_blocked(a, block_columns: int):
    """The (k, ld) row-major matrix `a` (numpy array or torch tensor) in the
    library's blocked layout: blocks of `block_columns` columns, each block
    holding its k row pieces back to back.  Returned with the same (k, ld)
    shape; only the order of the k * ld elements in memory differs."""
    k, ld = a.shape
    assert block_columns > 0 and ld % block_columns == 0
    pieces = a.reshape(k, ld // block_columns, block_columns)
    if hasattr(pieces, "permute"):
        return pieces.permute(1, 0, 2).contiguous().reshape(k, ld)
    return np.ascontiguousarray(pieces.transpose(1, 0, 2)).reshape(k, ld)


def from_blocked(b, block_columns: int):
    """Inverse of `to_blocked`."""
    k, ld = b.shape
    assert block_columns > 0 and ld % block_columns == 0
    pieces = b.reshape(ld // block_columns, k, block_columns)
    if hasattr(pieces, "permute"):
        return pieces.permute(1, 0, 2).contiguous().reshape(k, ld)
    return np.ascontiguousarray(pieces.transpose(1, 0, 2)).reshape(k, ld)


def random_segments(d: int, n_seg: int, seed: int, align: int = 1):
    """A seeded segment table with n_seg segments covering 0..d whose interior
    boundaries are multiples of `align`, and per-segment scales in U(0.5, 2)."""
    rng = np.random.default_rng(seed)
    assert 1 <= n_seg
    slots = d // align
    if n_seg - 1 > max(slots - 1, 0):
        raise ValueError("too many segments for this d / align")
    cuts = np.sort(rng.choice(np.arange(1, slots), size=n_seg - 1, replace=False)) * align if n_seg > 1 else np.array([], np.int64)
    offsets = np.concatenate([[0], cuts, [d]]).astype(np.int64)
    scales = rng.uniform(0.5, 2.0, n_seg).astype(np.float32)
    return offsets, scales


def make_special_inputs(k: int, d: int, ld: Optional[int] = None, seed: int = 0) -> Inputs:
    """Inputs that sit where fp32 arithmetic is fragile, for bit-exact parity:
    subnormals, +0 / -0, the smallest normals (whose products with lr, mu or
    beta land in the subnormal range), ordinary values, and magnitudes around
    1e36..1e37 (large, but such that no sum or difference the rules form can
    overflow, so every result is a finite number with one defined bit
    pattern).  Each element draws its class independently, so one column mixes
    classes across replicas.  h stays in [0.1, 1]."""
    ld = d if ld is None else ld
    assert ld >= d
    rng = np.random.default_rng(seed)

    def draw(shape):
        cls = rng.integers(0, 6, size=shape)
        sign = rng.integers(0, 2, size=shape).astype(np.uint32) << np.uint32(31)
        mant = rng.integers(0, 1 << 23, size=shape).astype(np.uint32)
        bits = np.zeros(shape, np.uint32)
        bits = np.where(cls == 0, mant, bits)                                          # subnormal (exponent field 0)
        bits = np.where(cls == 1, np.uint32(0), bits)                                  # zero
        bits = np.where(cls == 2, (np.uint32(1) << np.uint32(23)) | mant, bits)        # smallest normals, 1.2e-38..2.4e-38
        bits = np.where(cls == 3, (rng.integers(120, 131, size=shape).astype(np.uint32) << np.uint32(23)) | mant, bits)   # ~1
        bits = np.where(cls == 4, (rng.integers(246, 250, size=shape).astype(np.uint32) << np.uint32(23)) | mant, bits)   # 1e36..1e37
        bits = np.where(cls == 5, (rng.integers(1, 30, size=shape).astype(np.uint32) << np.uint32(23)) | mant, bits)      # tiny normals
        return (bits | sign).astype(np.uint32).view(np.float32)

    def rows():
        a = np.full((k, ld), 777.0, np.float32)
        a[:, :d] = draw((k, d))
        return a

    def vec(vals):
        a = np.full(ld, 777.0, np.float32)
        a[:d] = vals
        return a

    x, v, g = rows(), rows(), rows()
    xstar = vec(draw(d))
    h = vec(rng.uniform(0.1, 1.0, d).astype(np.float32))
    center = vec(draw(d))
    x0 = vec(draw(d))
    return Inputs(x, v, g, xstar, h, center, x0, d, ld, k)
