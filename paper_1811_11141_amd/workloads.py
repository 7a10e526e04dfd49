"""Seeded synthetic inputs for the merged-gradient reduction path.

This module only *describes inputs*: layer sizes p_l, per-layer backward times
t_b(l), the all-reduce cost constants (a, b), and seeded gradient / weight
values.  It holds none of the method's arithmetic (no planning, no packing, no
reduction, no update) so that both the CPU oracle's tests and the HIP path can
draw the same bits from it without sharing any code of the method itself.

The gradient sets stand in for the paper's ImageNet CNN workloads (Section V:
GoogLeNet at batch 64 and ResNet-50 at batch 32, fp32 parameters, layer sizes
mostly between 1e2 and 5e6).  Only the parameter *shapes* of the standard
architectures are used; values are Gaussian and backward times are proportional
to each tensor's backward FLOPs, because the paper leaves T_b unspecified
(Eq. 18) and its measured layer traces are not available.

Tensor order is forward definition order (index 0 = the paper's layer 1),
weight before bias and BN scale before BN shift.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

import numpy as np

# A 10 Gb/s link moves one byte in 8e-7 ms (Section V-A uses 10GbE).
BETA_10GBE_MS_PER_BYTE = 8.0e-7
# Effective backward rate used to turn FLOPs into milliseconds (a free constant:
# the paper's T_b(p, G, theta) of Eq. 18 is never specified).
G_EFF_FLOPS = 2.0e12
BASE_SEED = 1811_11141


# Per-byte all-reduce cost b (ms per byte) handed to the planner for N workers on that link: the
# values of Table II's ring row with gamma = 0, as numbers (the formula belongs to the method, not
# to an input generator; the oracle's tests check these against it).
RING_B_MS_PER_BYTE = {1: 0.0, 2: 8.0e-7, 3: 1.0666666666666665e-6, 4: 1.2e-6, 6: 1.3333333333333334e-6, 8: 1.4e-6,
                      12: 1.4666666666666665e-6, 16: 1.5e-6, 32: 1.55e-6, 64: 1.575e-6}


def ring_b_ms_per_byte(n_workers: int) -> float:
    if n_workers not in RING_B_MS_PER_BYTE:
        raise ValueError(f"no cost constant stored for {n_workers} workers")
    return RING_B_MS_PER_BYTE[n_workers]


@dataclass
class Workload:
    """One synthetic gradient set: sizes, backward times and cost constants."""

    name: str
    p: np.ndarray            # uint64 [L] elements per tensor, index 0 = layer 1
    tb_ms: np.ndarray        # float64 [L] backward time of each tensor
    n_workers: int           # N replicas
    a_ms: float              # all-reduce startup
    b_ms_per_byte: float     # all-reduce per-byte cost
    sigma: float             # std of gradient values
    tf_ms: float = 0.0
    names: List[str] = field(default_factory=list)

    @property
    def L(self) -> int:
        return int(self.p.shape[0])

    @property
    def P(self) -> int:
        return int(self.p.sum())


# --------------------------------------------------------------------------
# Architecture shape tables.  Each entry: (name, n_params, backward_flops/sample)
# --------------------------------------------------------------------------

class _Net:
    def __init__(self) -> None:
        self.rows: List[Tuple[str, int, float]] = []

    def conv(self, name: str, cin: int, cout: int, k: int, hout: int, wout: int,
             bias: bool, groups: int = 1) -> None:
        n_w = cout * (cin // groups) * k * k
        macs = n_w * hout * wout
        # data gradient + weight gradient, 2 flops per multiply-accumulate
        self.rows.append((name + ".weight", n_w, 4.0 * macs))
        if bias:
            self.rows.append((name + ".bias", cout, float(cout * hout * wout)))

    def bn(self, name: str, c: int, h: int, w: int) -> None:
        self.rows.append((name + ".gamma", c, float(c * h * w)))
        self.rows.append((name + ".beta", c, float(c * h * w)))

    def fc(self, name: str, cin: int, cout: int, bias: bool = True) -> None:
        self.rows.append((name + ".weight", cin * cout, 4.0 * cin * cout))
        if bias:
            self.rows.append((name + ".bias", cout, float(cout)))


def _resnet50() -> _Net:
    net = _Net()
    net.conv("conv1", 3, 64, 7, 112, 112, bias=False)
    net.bn("bn1", 64, 112, 112)
    inplanes, size = 64, 56
    for stage, (planes, blocks) in enumerate(zip((64, 128, 256, 512), (3, 4, 6, 3))):
        for blk in range(blocks):
            stride = 2 if (blk == 0 and stage > 0) else 1
            out = size // stride
            pre = f"layer{stage + 1}.{blk}"
            # stride sits on the first 1x1 convolution (the original Caffe model)
            net.conv(pre + ".conv1", inplanes, planes, 1, out, out, bias=False)
            net.bn(pre + ".bn1", planes, out, out)
            net.conv(pre + ".conv2", planes, planes, 3, out, out, bias=False)
            net.bn(pre + ".bn2", planes, out, out)
            net.conv(pre + ".conv3", planes, planes * 4, 1, out, out, bias=False)
            net.bn(pre + ".bn3", planes * 4, out, out)
            if blk == 0:
                net.conv(pre + ".downsample", inplanes, planes * 4, 1, out, out, bias=False)
                net.bn(pre + ".downsample_bn", planes * 4, out, out)
            inplanes, size = planes * 4, out
    net.fc("fc", 2048, 1000)
    return net


def _inception(net: _Net, name: str, cin: int, c1: int, c3r: int, c3: int,
               c5r: int, c5: int, cp: int, s: int) -> int:
    net.conv(name + ".1x1", cin, c1, 1, s, s, bias=True)
    net.conv(name + ".3x3_reduce", cin, c3r, 1, s, s, bias=True)
    net.conv(name + ".3x3", c3r, c3, 3, s, s, bias=True)
    net.conv(name + ".5x5_reduce", cin, c5r, 1, s, s, bias=True)
    net.conv(name + ".5x5", c5r, c5, 5, s, s, bias=True)
    net.conv(name + ".pool_proj", cin, cp, 1, s, s, bias=True)
    return c1 + c3 + c5 + cp


def _aux_head(net: _Net, name: str, cin: int) -> None:
    net.conv(name + ".conv", cin, 128, 1, 4, 4, bias=True)
    net.fc(name + ".fc1", 2048, 1024)
    net.fc(name + ".fc2", 1024, 1000)


def _googlenet() -> _Net:
    net = _Net()
    net.conv("conv1", 3, 64, 7, 112, 112, bias=True)
    net.conv("conv2_reduce", 64, 64, 1, 56, 56, bias=True)
    net.conv("conv2", 64, 192, 3, 56, 56, bias=True)
    c = _inception(net, "3a", 192, 64, 96, 128, 16, 32, 32, 28)
    c = _inception(net, "3b", c, 128, 128, 192, 32, 96, 64, 28)
    c = _inception(net, "4a", c, 192, 96, 208, 16, 48, 64, 14)
    _aux_head(net, "aux1", c)
    c = _inception(net, "4b", c, 160, 112, 224, 24, 64, 64, 14)
    c = _inception(net, "4c", c, 128, 128, 256, 24, 64, 64, 14)
    c = _inception(net, "4d", c, 112, 144, 288, 32, 64, 64, 14)
    _aux_head(net, "aux2", c)
    c = _inception(net, "4e", c, 256, 160, 320, 32, 128, 128, 14)
    c = _inception(net, "5a", c, 256, 160, 320, 32, 128, 128, 7)
    c = _inception(net, "5b", c, 384, 192, 384, 48, 128, 128, 7)
    net.fc("fc", c, 1000)
    return net


def _alexnet() -> _Net:
    # one-column variant (64/192/384/256/256 filters, no grouped convolutions)
    net = _Net()
    net.conv("conv1", 3, 64, 11, 55, 55, bias=True)
    net.conv("conv2", 64, 192, 5, 27, 27, bias=True)
    net.conv("conv3", 192, 384, 3, 13, 13, bias=True)
    net.conv("conv4", 384, 256, 3, 13, 13, bias=True)
    net.conv("conv5", 256, 256, 3, 13, 13, bias=True)
    net.fc("fc6", 9216, 4096)
    net.fc("fc7", 4096, 4096)
    net.fc("fc8", 4096, 1000)
    return net


def _vgg16() -> _Net:
    net = _Net()
    cfg = [(64, 224), (64, 224), (128, 112), (128, 112), (256, 56), (256, 56), (256, 56),
           (512, 28), (512, 28), (512, 28), (512, 14), (512, 14), (512, 14)]
    cin = 3
    for i, (cout, s) in enumerate(cfg):
        net.conv(f"conv{i + 1}", cin, cout, 3, s, s, bias=True)
        cin = cout
    net.fc("fc6", 25088, 4096)
    net.fc("fc7", 4096, 4096)
    net.fc("fc8", 4096, 1000)
    return net


_ARCH = {
    # name: (builder, batch, N, sigma)
    "resnet50": (_resnet50, 32, 8, 1e-3),
    "googlenet": (_googlenet, 64, 8, 1e-3),
    "alexnet": (_alexnet, 128, 8, 1e-3),
    "vgg16": (_vgg16, 32, 16, 1e-3),
}

CNN_WORKLOADS = tuple(_ARCH)


def cnn_workload(name: str, a_ms: float = 0.5, g_eff: float = G_EFF_FLOPS,
                 n_workers: int | None = None) -> Workload:
    """ResNet-50 / GoogLeNet / AlexNet / VGG-16 shaped gradient set."""
    builder, batch, n_default, sigma = _ARCH[name]
    n = n_default if n_workers is None else int(n_workers)
    rows = builder().rows
    p = np.array([r[1] for r in rows], dtype=np.uint64)
    tb = np.array([r[2] * batch / g_eff * 1e3 for r in rows], dtype=np.float64)
    return Workload(name=name, p=p, tb_ms=tb, n_workers=n, a_ms=float(a_ms),
                    b_ms_per_byte=ring_b_ms_per_byte(n), sigma=sigma,
                    names=[r[0] for r in rows])


def tiny_workload(seed: int, L: int = 8, n_workers: int = 4) -> Workload:
    """Tiny net: sizes log-uniform in [64, 65536], t_b ~ U[0.1, 2] ms, a = 0.5, b = 1e-6."""
    rng = np.random.default_rng(seed)
    p = np.clip(np.rint(2.0 ** rng.uniform(6.0, 16.0, size=L)), 64, 65536).astype(np.uint64)
    tb = rng.uniform(0.1, 2.0, size=L)
    return Workload(name=f"tiny{L}-seed{seed}", p=p, tb_ms=tb, n_workers=n_workers,
                    a_ms=0.5, b_ms_per_byte=1e-6, sigma=1e-2,
                    names=[f"t{i + 1}" for i in range(L)])


def custom_workload(p: Sequence[int], n_workers: int, tb_ms: Sequence[float] | None = None,
                    a_ms: float = 0.5, b_ms_per_byte: float = 1e-6, sigma: float = 1e-2,
                    name: str = "custom") -> Workload:
    p_arr = np.asarray(p, dtype=np.uint64)
    tb = np.ones(len(p_arr)) if tb_ms is None else np.asarray(tb_ms, dtype=np.float64)
    return Workload(name=name, p=p_arr, tb_ms=tb, n_workers=n_workers, a_ms=a_ms,
                    b_ms_per_byte=b_ms_per_byte, sigma=sigma,
                    names=[f"t{i + 1}" for i in range(len(p_arr))])


def replica_seed(seed: int, g: int) -> int:
    return seed * 64 + g


def make_tensors(wl: Workload, seed: int, device: str = "cpu", sigma: float | None = None,
                 stream_id: int = 0):
    """One fp32 tensor per layer, values ~ N(0, sigma), from a seeded torch generator.

    `stream_id` separates independent draws made with the same seed (replica g of
    the gradients uses stream g; weights use a stream past the replicas).
    """
    import torch

    gen = torch.Generator(device=device)
    gen.manual_seed(replica_seed(seed, stream_id))
    s = wl.sigma if sigma is None else sigma
    out = []
    for n in wl.p.tolist():
        t = torch.empty(int(n), dtype=torch.float32, device=device)
        t.normal_(0.0, s, generator=gen)
        out.append(t)
    return out


def make_gradients(wl: Workload, seed: int, device: str = "cpu"):
    """grads[g][l]: replica g's gradient of layer l+1 (N lists of L tensors)."""
    return [make_tensors(wl, seed, device, stream_id=g) for g in range(wl.n_workers)]


def make_weights(wl: Workload, seed: int, device: str = "cpu"):
    """Weights ~ N(0, 0.1) and zero momentum buffers."""
    import torch

    w = make_tensors(wl, seed, device, sigma=0.1, stream_id=63)
    v = [torch.zeros_like(t) for t in w]
    return w, v


def random_bit_patterns(wl: Workload, seed: int, n_replicas: int | None = None):
    """Arbitrary 32-bit patterns (NaN payloads, -0.0, denormals included) viewed as fp32.

    Only meaningful for the pure bit-copy steps (pack / unpack).
    """
    rng = np.random.default_rng(seed)
    n = wl.n_workers if n_replicas is None else n_replicas
    special = np.array([0x00000000, 0x80000000, 0x7FC00001, 0xFFC12345, 0x7F800000,
                        0xFF800000, 0x00000001, 0x807FFFFF, 0x7F7FFFFF], dtype=np.uint32)
    out = []
    for _ in range(n):
        rep = []
        for cnt in wl.p.tolist():
            bits = rng.integers(0, 2 ** 32, size=int(cnt), dtype=np.uint64).astype(np.uint32)
            k = min(len(special), int(cnt))
            pos = rng.choice(int(cnt), size=k, replace=False)
            bits[pos] = special[:k]
            rep.append(bits)
        out.append(rep)
    return out
