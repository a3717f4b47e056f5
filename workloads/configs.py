"""Variable lists (shapes only) of the five benchmark configurations.

The paper evaluates ResNet-50, Transformer and NCF (Section 6, Table 1); the
cost of the weight update depends on tensor sizes and dtypes only, so these
lists reproduce the architectures' parameter shapes and nothing else: no
dataset, no trained weights.  Each list is written from the architecture's
public description (layer counts, widths).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from math import prod
from typing import Dict, List, Tuple

Shape = Tuple[int, ...]


@dataclass(frozen=True)
class Workload:
    name: str
    index: int                      # position in the configuration list; seeds derive from it
    shapes: Tuple[Shape, ...]
    optimizer: str                  # "adam" | "momentum" | "lamb"
    hyper: Dict[str, float] = field(default_factory=dict)
    replicas: Tuple[int, ...] = (1,)
    weight_std: float = 0.02
    grad_std: float = 1e-3
    mixed_bf16: bool = False        # fp32 master + bf16 copy of the weights

    @property
    def numel(self) -> List[int]:
        return [prod(s) for s in self.shapes]

    @property
    def total(self) -> int:
        return sum(self.numel)

    @property
    def seed(self) -> int:
        return 1234 + self.index


def _tiny() -> List[Shape]:
    return [(1000, 128), (512, 512), (512,), (2048, 512), (512, 2048), (128,)]


def _resnet50() -> List[Shape]:
    """53 convolutions [k,k,Cin,Cout], a (gamma, beta) pair after each, one FC layer."""
    shapes: List[Shape] = []

    def conv_bn(k: int, cin: int, cout: int) -> None:
        shapes.append((k, k, cin, cout))
        shapes.append((cout,))
        shapes.append((cout,))

    conv_bn(7, 3, 64)
    cin = 64
    for width, blocks in ((64, 3), (128, 4), (256, 6), (512, 3)):
        for b in range(blocks):
            conv_bn(1, cin, width)
            conv_bn(3, width, width)
            conv_bn(1, width, 4 * width)
            if b == 0:                       # projection shortcut of the stage's first block
                conv_bn(1, cin, 4 * width)
            cin = 4 * width
    shapes.append((2048, 1000))
    shapes.append((1000,))
    return shapes


def _dense(shapes: List[Shape], din: int, dout: int) -> None:
    shapes.append((din, dout))
    shapes.append((dout,))


def _layernorm(shapes: List[Shape], d: int) -> None:
    shapes.append((d,))
    shapes.append((d,))


def _attention(shapes: List[Shape], d: int) -> None:
    for _ in range(4):                       # query, key, value, output projections
        _dense(shapes, d, d)


def _transformer_big() -> List[Shape]:
    d, ff, vocab = 1024, 4096, 32768
    shapes: List[Shape] = [(vocab, d)]       # embedding shared by encoder, decoder and softmax
    for _ in range(6):                       # encoder layers
        _attention(shapes, d)
        _layernorm(shapes, d)
        _dense(shapes, d, ff)
        _dense(shapes, ff, d)
        _layernorm(shapes, d)
    _layernorm(shapes, d)
    for _ in range(6):                       # decoder layers
        _attention(shapes, d)
        _layernorm(shapes, d)
        _attention(shapes, d)                # encoder-decoder attention
        _layernorm(shapes, d)
        _dense(shapes, d, ff)
        _dense(shapes, ff, d)
        _layernorm(shapes, d)
    _layernorm(shapes, d)
    return shapes


def _bert_large() -> List[Shape]:
    d, ff, vocab = 1024, 4096, 30522
    shapes: List[Shape] = [(vocab, d), (512, d), (2, d)]
    _layernorm(shapes, d)
    for _ in range(24):
        _attention(shapes, d)
        _layernorm(shapes, d)
        _dense(shapes, d, ff)
        _dense(shapes, ff, d)
        _layernorm(shapes, d)
    _dense(shapes, d, d)                     # pooler
    _dense(shapes, d, d)                     # masked-LM transform
    _layernorm(shapes, d)
    shapes.append((vocab,))                  # masked-LM output bias
    _dense(shapes, d, 2)                     # next-sentence head
    return shapes


def _lm_1p5b() -> List[Shape]:
    d, ff, vocab = 1600, 6400, 50304
    shapes: List[Shape] = [(vocab, d)]
    for _ in range(48):
        _layernorm(shapes, d)
        _attention(shapes, d)
        _layernorm(shapes, d)
        _dense(shapes, d, ff)
        _dense(shapes, ff, d)
    _layernorm(shapes, d)
    return shapes


_ADAM = {"lr": 1e-3, "beta1": 0.9, "beta2": 0.999, "eps": 1e-8, "weight_decay": 0.0}

CONFIGS: Tuple[Workload, ...] = (
    Workload("tiny", 0, tuple(_tiny()), "adam", dict(_ADAM), replicas=(4,),
             weight_std=0.02, grad_std=1e-2),
    Workload("resnet50", 1, tuple(_resnet50()), "momentum",
             {"lr": 0.1, "mu": 0.9, "weight_decay": 5e-5}, replicas=(1, 32),
             weight_std=0.02, grad_std=1e-3),
    Workload("transformer_big", 2, tuple(_transformer_big()), "adam", dict(_ADAM), replicas=(16,),
             weight_std=0.02, grad_std=1e-3),
    Workload("bert_large", 3, tuple(_bert_large()), "lamb",
             {"lr": 1e-3, "beta1": 0.9, "beta2": 0.999, "eps": 1e-6, "weight_decay": 0.01},
             replicas=(8, 64), weight_std=0.02, grad_std=1e-3),
    Workload("lm_1p5b", 4, tuple(_lm_1p5b()), "adam", dict(_ADAM), replicas=(1, 128),
             weight_std=0.02, grad_std=1e-4, mixed_bf16=True),
)


def get_workload(name: str) -> Workload:
    for w in CONFIGS:
        if w.name == name:
            return w
    raise KeyError(name)
