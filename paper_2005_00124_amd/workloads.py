"""Seeded synthetic inputs for the WAGMA-SGD hot path.

This module holds input generators only: model shapes, initial weights,
gradients and the per-workload constants.  It contains none of the method's
arithmetic (no update rule, no grouping, no averaging, no lateness hash) and is
the one module that both the GPU path's callers and the CPU oracle's callers
use, so that both sides see bit-identical floats.

The five workloads stand in for the training state of the paper's experiments
(Section 6: ResNet-50 on ImageNet, Transformer on WMT17), which need datasets
that are not available here: only the parameter counts, the per-tensor shapes
and the value distributions are reproduced.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Callable, List, Tuple

import torch

BASE_SEED = 200500124

# (name, shape, kind, fan_in, fan_out); kind in
# {"he_normal", "xavier_uniform", "embedding", "ones", "zeros", "normal"}.
Tensor = Tuple[str, Tuple[int, ...], str, int, int]


def flat_tensors(n: int, std: float) -> List[Tensor]:
    return [("flat", (n,), "normal:%r" % std, 0, 0)]


def resnet50_tensors(num_classes: int = 1000) -> List[Tensor]:
    """ResNet-50 v1 parameter list (Section 6.2 names the network; layout per He et al. 2016).

    Stem 7x7x3x64, four stages of bottleneck blocks [3, 4, 6, 3] with widths
    64/128/256/512 (1x1, 3x3, 1x1 convolutions, each followed by batch norm
    scale and shift, a 1x1 projection in the first block of a stage) and a
    2048 x num_classes classifier.  1000 classes give 25,557,032 parameters;
    the paper's 25,559,081 is the 1001-class variant.
    """
    out: List[Tensor] = []

    def conv(name, kh, kw, cin, cout):
        out.append((name, (kh, kw, cin, cout), "he_normal", kh * kw * cin, cout))

    def bn(name, c):
        out.append((name + ".gamma", (c,), "ones", 0, 0))
        out.append((name + ".beta", (c,), "zeros", 0, 0))

    conv("stem.conv", 7, 7, 3, 64)
    bn("stem.bn", 64)
    cin = 64
    for si, (width, blocks) in enumerate(zip((64, 128, 256, 512), (3, 4, 6, 3))):
        for bi in range(blocks):
            p = "stage%d.block%d" % (si + 1, bi)
            conv(p + ".conv1", 1, 1, cin, width)
            bn(p + ".bn1", width)
            conv(p + ".conv2", 3, 3, width, width)
            bn(p + ".bn2", width)
            conv(p + ".conv3", 1, 1, width, 4 * width)
            bn(p + ".bn3", 4 * width)
            if bi == 0:
                conv(p + ".proj", 1, 1, cin, 4 * width)
                bn(p + ".proj_bn", 4 * width)
            cin = 4 * width
    out.append(("fc.weight", (2048, num_classes), "he_normal", 2048, num_classes))
    out.append(("fc.bias", (num_classes,), "zeros", 0, 0))
    return out


def transformer_tensors(d_model: int, d_ff: int, vocab: int = 33708,
                        layers: int = 6) -> List[Tensor]:
    """Encoder-decoder Transformer parameter list (Section 6.3; Vaswani et al. 2017).

    ``layers`` encoder and decoder layers, bias-free attention projections,
    feed-forward with biases, layer norms, one embedding tied between source,
    target and output.  vocab = 33,708 with d_model = 512 reproduces the
    paper's 61,362,176 parameters exactly.
    """
    out: List[Tensor] = []
    d = d_model

    def mat(name, a, b):
        out.append((name, (a, b), "xavier_uniform", a, b))

    def ln(name):
        out.append((name + ".scale", (d,), "ones", 0, 0))
        out.append((name + ".bias", (d,), "zeros", 0, 0))

    def attn(name):
        for x in ("q", "k", "v", "o"):
            mat(name + "." + x, d, d)

    def ffn(name):
        mat(name + ".w1", d, d_ff)
        out.append((name + ".b1", (d_ff,), "zeros", 0, 0))
        mat(name + ".w2", d_ff, d)
        out.append((name + ".b2", (d,), "zeros", 0, 0))

    out.append(("embedding", (vocab, d), "embedding", d, 0))
    for i in range(layers):
        p = "enc%d" % i
        attn(p + ".self")
        ln(p + ".ln1")
        ffn(p + ".ffn")
        ln(p + ".ln2")
    ln("enc.final_ln")
    for i in range(layers):
        p = "dec%d" % i
        attn(p + ".self")
        ln(p + ".ln1")
        attn(p + ".cross")
        ln(p + ".ln2")
        ffn(p + ".ffn")
        ln(p + ".ln3")
    ln("dec.final_ln")
    return out


def count_params(tensors: List[Tensor]) -> int:
    return sum(math.prod(t[1]) for t in tensors)


@dataclass(frozen=True)
class Workload:
    """One seeded workload: the constants of a run and its input recipe."""
    index: int                 # 1-based, as the workloads are listed
    name: str
    P: int                     # simulated processes (replicas)
    S: int                     # group size
    tau: int                   # global synchronisation period
    iters: int
    tensors: Callable[[], List[Tensor]]
    grad_std: float
    q: float                   # probability that a process is late in an iteration
    lr: float = 0.1
    mu: float = 0.9

    @property
    def n(self) -> int:
        return count_params(self.tensors())

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index

    @property
    def stale_threshold(self) -> int:
        """Integer threshold floor(q * 2^32) used by the lateness hash."""
        return min(int(math.floor(self.q * 4294967296.0)), 4294967295)

    def grad_seed(self, t: int) -> int:
        return self.seed * 1000003 + t


WORKLOADS = (
    Workload(1, "flat-1M P=4 S=2", 4, 2, 5, 10,
             lambda: flat_tensors(1048576, 0.02), 1e-3, 0.0),
    Workload(2, "resnet50-shaped 25.6M P=16 S=4", 16, 4, 10, 50,
             resnet50_tensors, 1e-3, 0.2),
    Workload(3, "transformer-base-shaped 61.4M P=16 S=4", 16, 4, 10, 50,
             lambda: transformer_tensors(512, 2048), 1e-4, 0.1),
    Workload(4, "resnet50-shaped 25.6M P=64 S=8", 64, 8, 16, 50,
             resnet50_tensors, 1e-3, 0.25),
    Workload(5, "transformer-big-shaped 210.8M P=32 S=8", 32, 8, 8, 20,
             lambda: transformer_tensors(1024, 4096), 1e-4, 0.2),
)


def workload(index: int) -> Workload:
    return WORKLOADS[index - 1]


def make_generator(seed: int, device) -> torch.Generator:
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    return gen


def init_model_row(tensors: List[Tensor], row: torch.Tensor, gen: torch.Generator) -> None:
    """Fill the 1-D fp32 tensor ``row`` (length >= n) with one freshly initialised model."""
    at = 0
    for _name, shape, kind, fan_in, fan_out in tensors:
        k = math.prod(shape)
        seg = row[at:at + k]
        if kind == "he_normal":
            seg.normal_(0.0, math.sqrt(2.0 / fan_in), generator=gen)
        elif kind == "xavier_uniform":
            a = math.sqrt(6.0 / (fan_in + fan_out))
            seg.uniform_(-a, a, generator=gen)
        elif kind == "embedding":
            seg.normal_(0.0, fan_in ** -0.5, generator=gen)
        elif kind == "ones":
            seg.fill_(1.0)
        elif kind == "zeros":
            seg.zero_()
        elif kind.startswith("normal:"):
            seg.normal_(0.0, float(kind.split(":", 1)[1]), generator=gen)
        else:
            raise ValueError("unknown init kind %r" % kind)
        at += k


def fill_initial_state(wl: Workload, w: torch.Tensor, m: torch.Tensor, pub: torch.Tensor) -> None:
    """w, m, pub: (P, ld) fp32.  All replicas start from one model; m = 0; pub = w."""
    n = wl.n
    gen = make_generator(wl.seed, w.device)
    w.zero_()
    init_model_row(wl.tensors(), w[0, :n], gen)
    for p in range(1, wl.P):
        w[p, :n].copy_(w[0, :n])
    m.zero_()
    pub.copy_(w)


def fill_gradients(wl: Workload, t: int, g: torch.Tensor) -> None:
    """g: (P, ld) fp32; every replica draws its own gradient for iteration t."""
    n = wl.n
    gen = make_generator(wl.grad_seed(t), g.device)
    for p in range(wl.P):
        g[p, :n].normal_(0.0, wl.grad_std, generator=gen)


def sample_columns(n: int, count: int, seed: int, tile: int = 4096, tensor_sizes=None,
                   ends: int = 256) -> torch.Tensor:
    """A sorted int64 column set for sampled parity: ``ends`` columns at both ends of the row
    (with the ragged tail), columns on each side of multiples of ``tile``, the first and last
    four columns of every tensor of the flattened model (``tensor_sizes``: their lengths in
    row order), and a seeded random rest up to ``count`` columns."""
    cols = set(range(min(n, ends)))
    cols.update(range(max(0, n - ends), n))
    gen = torch.Generator()
    gen.manual_seed(seed)
    if n > tile:
        edges = torch.randint(1, max(2, n // tile), (32,), generator=gen) * tile
        for e in edges.tolist():
            cols.update(c for c in range(e - 4, e + 4) if 0 <= c < n)
    if tensor_sizes is not None:
        at = 0
        for size in tensor_sizes:
            cols.update(c for c in range(at, min(at + 4, at + size)))
            cols.update(c for c in range(max(at, at + size - 4), at + size))
            at += size
        if at != n:
            raise ValueError("tensor sizes do not add up to n")
    need = max(0, count - len(cols))
    if need:
        cols.update(torch.randint(0, n, (need,), generator=gen).tolist())
    return torch.tensor(sorted(cols), dtype=torch.int64)
