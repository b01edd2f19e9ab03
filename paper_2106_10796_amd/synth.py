"""Seeded synthetic inputs: layer lists and gradient / weight values.

This module holds no arithmetic of the method itself.  It only says what the
buffers look like (shapes of the models the paper trains: ResNet-20, ResNet-50,
VGG-16; Sec. 4) and fills them with seeded random values.  Both the HIP path
and the CPU oracle are fed from here: values are generated once (on whatever
device is asked for) and the same bits are handed to both sides.
"""
import math
from dataclasses import dataclass, field
from typing import List, Tuple

import torch

BASE_SEED = 210610796


# ---------------------------------------------------------------------------
# layer lists (architecture facts, definition order)
# ---------------------------------------------------------------------------
def _conv(cout, cin, k):
    return cout * cin * k * k


def resnet20_layers() -> List[Tuple[str, int]]:
    """CIFAR ResNet-20: 3x3 stem, 3 stages x 3 basic blocks (16/32/64), fc 64x10."""
    L = [("conv1.weight", _conv(16, 3, 3)), ("bn1.gamma", 16), ("bn1.beta", 16)]
    cin = 16
    for s, c in enumerate((16, 32, 64)):
        for b in range(3):
            p = "stage%d.block%d." % (s + 1, b)
            L += [(p + "conv1.weight", _conv(c, cin, 3)), (p + "bn1.gamma", c), (p + "bn1.beta", c),
                  (p + "conv2.weight", _conv(c, c, 3)), (p + "bn2.gamma", c), (p + "bn2.beta", c)]
            if b == 0 and cin != c:
                L += [(p + "proj.weight", _conv(c, cin, 1)), (p + "proj_bn.gamma", c), (p + "proj_bn.beta", c)]
            cin = c
    L += [("fc.weight", 64 * 10), ("fc.bias", 10)]
    assert len(L) == 65 and sum(n for _, n in L) == 272474
    return L


def resnet50_layers() -> List[Tuple[str, int]]:
    """ImageNet ResNet-50: 7x7 stem, (3,4,6,3) bottlenecks of width (64,128,256,512), fc 2048x1000."""
    L = [("conv1.weight", _conv(64, 3, 7)), ("bn1.gamma", 64), ("bn1.beta", 64)]
    cin = 64
    for s, (blocks, w) in enumerate(zip((3, 4, 6, 3), (64, 128, 256, 512))):
        for b in range(blocks):
            p = "stage%d.block%d." % (s + 1, b)
            L += [(p + "conv1.weight", _conv(w, cin, 1)), (p + "bn1.gamma", w), (p + "bn1.beta", w),
                  (p + "conv2.weight", _conv(w, w, 3)), (p + "bn2.gamma", w), (p + "bn2.beta", w),
                  (p + "conv3.weight", _conv(4 * w, w, 1)), (p + "bn3.gamma", 4 * w), (p + "bn3.beta", 4 * w)]
            if b == 0:
                L += [(p + "down.weight", _conv(4 * w, cin, 1)), (p + "down_bn.gamma", 4 * w),
                      (p + "down_bn.beta", 4 * w)]
            cin = 4 * w
    L += [("fc.weight", 2048 * 1000), ("fc.bias", 1000)]
    assert len(L) == 161 and sum(n for _, n in L) == 25557032
    return L


def vgg16_layers() -> List[Tuple[str, int]]:
    """VGG-16: 13 3x3 convs with bias, fc 25088x4096, 4096x4096, 4096x1000 with bias."""
    L = []
    cin = 3
    for i, c in enumerate((64, 64, 128, 128, 256, 256, 256, 512, 512, 512, 512, 512, 512)):
        L += [("conv%d.weight" % (i + 1), _conv(c, cin, 3)), ("conv%d.bias" % (i + 1), c)]
        cin = c
    for i, (a, b) in enumerate(((25088, 4096), (4096, 4096), (4096, 1000))):
        L += [("fc%d.weight" % (i + 1), a * b), ("fc%d.bias" % (i + 1), b)]
    assert len(L) == 32 and sum(n for _, n in L) == 138357544
    return L


# ---------------------------------------------------------------------------
# the five workloads
# ---------------------------------------------------------------------------
@dataclass
class Config:
    name: str
    cid: int
    sizes: List[int]
    num_workers: int
    k: int
    iterations: int
    threshold: float
    lr: float
    grad_dist: str            # "normal" | "normal_per_tensor" | "normal_outliers" | "laplace"
    grad_param: float = 0.0   # std (normal / normal_outliers) or scale b (laplace)
    weight_std: float = math.sqrt(0.05)
    description: str = ""
    tensor_std: List[float] = field(default_factory=list)

    @property
    def num_tensors(self):
        return len(self.sizes)

    @property
    def elements(self):
        return sum(self.sizes)

    @property
    def bytes_per_element(self):
        """Algorithmic HBM bytes per element of one compressed fused step: read g, r, W
        and N-1 peers' codes, write r, W, Wloc and the own codes = 24 + N/4."""
        return 24.0 + self.num_workers / 4.0


def _seed(*parts) -> int:
    """A 63-bit seed from integers (splitmix-style mixing of the parts)."""
    x = BASE_SEED
    for p in parts:
        x = (x ^ (int(p) + 0x9E3779B97F4A7C15 + ((x << 6) & 0xFFFFFFFFFFFFFFFF) + (x >> 2))) & 0xFFFFFFFFFFFFFFFF
        x = (x * 0xBF58476D1CE4E5B9) & 0xFFFFFFFFFFFFFFFF
        x ^= x >> 31
    return x & 0x7FFFFFFFFFFFFFFF


def _per_tensor_std(cid: int, num_tensors: int) -> List[float]:
    """sigma_i = 10^(-4 + 3 u_i): log-uniform in [1e-4, 1e-1], u_i from the tensor's seed."""
    out = []
    for i in range(num_tensors):
        g = torch.Generator(device="cpu")
        g.manual_seed(_seed(cid, 77, i))
        u = float(torch.rand(1, generator=g).item())
        out.append(10.0 ** (-4.0 + 3.0 * u))
    return out


def config(name: str) -> Config:
    """The five workloads (single tensor, ResNet-20, ResNet-50, VGG-16, 4 GiB flat bucket)."""
    if name == "c1_single":
        # N(0, 0.01) read as mean / variance: std 0.1 (with std 0.01 no code could ever fire at t = 0.5)
        return Config(name, 1, [65536], 4, 4, 8, 0.5, 0.1, "normal", 0.1,
                      description="single fp32 tensor, 65,536 elements")
    if name == "c2_resnet20":
        sizes = [n for _, n in resnet20_layers()]
        return Config(name, 2, sizes, 8, 4, 20, 0.5, 0.1, "normal_per_tensor",
                      tensor_std=_per_tensor_std(2, len(sizes)), description="ResNet-20-shaped layer list")
    if name == "c3_resnet50":
        sizes = [n for _, n in resnet50_layers()]
        return Config(name, 3, sizes, 16, 8, 50, 0.5, 0.1, "normal_per_tensor",
                      tensor_std=_per_tensor_std(3, len(sizes)), description="ResNet-50-shaped layer list")
    if name == "c4_vgg16":
        sizes = [n for _, n in vgg16_layers()]
        return Config(name, 4, sizes, 16, 8, 20, 0.5, 0.1, "normal_outliers", 0.005,
                      description="VGG-16-shaped layer list")
    if name == "c5_flat4g":
        return Config(name, 5, [1 << 30], 16, 16, 10, 0.05, 0.1, "laplace", 0.02,
                      description="flat 2^30-element fp32 bucket (4 GiB)")
    raise KeyError(name)


CONFIG_NAMES = ["c1_single", "c2_resnet20", "c3_resnet50", "c4_vgg16", "c5_flat4g"]


def scaled(cfg: Config, sizes: List[int], name_suffix: str) -> Config:
    """Same recipe on other tensor sizes (used by tests that need small or ragged tensors)."""
    c = Config(cfg.name + name_suffix, cfg.cid, list(sizes), cfg.num_workers, cfg.k, cfg.iterations,
               cfg.threshold, cfg.lr, cfg.grad_dist, cfg.grad_param, cfg.weight_std, cfg.description)
    if cfg.grad_dist == "normal_per_tensor":
        c.tensor_std = _per_tensor_std(cfg.cid, len(sizes))
    return c


# ---------------------------------------------------------------------------
# values
# ---------------------------------------------------------------------------
def _generator(device, seed):
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def fill_grad(out: torch.Tensor, cfg: Config, worker: int, step: int, tensor: int, dense: bool = False):
    """Fill `out` (fp32, any device) with worker `worker`'s gradient of tensor `tensor` at step `step`.

    dense=True is the parity variant: every tensor gets std equal to the threshold,
    so about a third of the codes are non-zero from the first compressed step (under
    the literal recipes most codes stay zero for the whole run, which exercises
    little of the quantiser).
    """
    gen = _generator(out.device, _seed(cfg.cid, 1, worker, step, tensor))
    n = out.numel()
    if dense:
        out.normal_(0.0, 1.0, generator=gen).mul_(cfg.threshold)
        return out
    if cfg.grad_dist == "normal":
        out.normal_(0.0, 1.0, generator=gen).mul_(cfg.grad_param)
    elif cfg.grad_dist == "normal_per_tensor":
        out.normal_(0.0, 1.0, generator=gen).mul_(cfg.tensor_std[tensor])
    elif cfg.grad_dist == "normal_outliers":
        out.normal_(0.0, 1.0, generator=gen).mul_(cfg.grad_param)
        # each element independently, with probability 1 %, is ten times larger
        block = 1 << 26
        for s in range(0, n, block):
            e = min(n, s + block)
            m = torch.rand(e - s, generator=gen, device=out.device) < 0.01
            out[s:e].mul_(torch.where(m, 10.0, 1.0))
    elif cfg.grad_dist == "laplace":
        # inverse CDF: x = -b sign(u) log(1 - 2|u|), u uniform in (-1/2, 1/2)
        block = 1 << 26
        for s in range(0, n, block):
            e = min(n, s + block)
            u = torch.rand(e - s, generator=gen, device=out.device).sub_(0.5)
            mag = torch.log1p(u.abs().mul(-2.0).clamp_(min=-1.0 + 1e-7)).mul_(-cfg.grad_param)
            out[s:e].copy_(torch.where(u < 0, -mag, mag))
    else:
        raise ValueError(cfg.grad_dist)
    return out


def fill_weight(out: torch.Tensor, cfg: Config, tensor: int):
    gen = _generator(out.device, _seed(cfg.cid, 2, tensor))
    out.normal_(0.0, 1.0, generator=gen).mul_(cfg.weight_std)
    return out
