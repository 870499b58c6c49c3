"""Tensor-shape lists of the workload models, in forward (registration) order.

The paper evaluates on AlexNet, VGG, AWD-LM and BERT and, in its appendix on
network interference, a ResNet (Section 5.1 "Workloads"; Appendix D).  Only the
layer shapes matter to model aggregation, so these lists carry architecture
shapes only: no dataset, no trained weight.  Gradient and parameter values are
synthetic (see values.py).

Each builder returns a list of (name, shape) in the order a framework would
register the tensors (first layer first).  Back-propagation produces gradients
in the reverse of this order.
"""
from __future__ import annotations

from dataclasses import dataclass
from math import prod
from typing import Callable, Dict, List, Sequence, Tuple

Tensor = Tuple[str, Tuple[int, ...]]


def _numel(shape: Sequence[int]) -> int:
    return int(prod(shape))


def mlp() -> List[Tensor]:
    """784-512-10 perceptron: two weight matrices and their biases."""
    return [
        ("fc1.weight", (512, 784)),
        ("fc1.bias", (512,)),
        ("fc2.weight", (10, 512)),
        ("fc2.bias", (10,)),
    ]


def alexnet() -> List[Tensor]:
    convs = [(64, 3, 11), (192, 64, 5), (384, 192, 3), (256, 384, 3), (256, 256, 3)]
    fcs = [(4096, 9216), (4096, 4096), (1000, 4096)]
    out: List[Tensor] = []
    for i, (co, ci, k) in enumerate(convs, 1):
        out.append((f"conv{i}.weight", (co, ci, k, k)))
        out.append((f"conv{i}.bias", (co,)))
    for i, (o, n) in enumerate(fcs, 6):
        out.append((f"fc{i}.weight", (o, n)))
        out.append((f"fc{i}.bias", (o,)))
    return out


def vgg16() -> List[Tensor]:
    widths = [64, 64, 128, 128, 256, 256, 256, 512, 512, 512, 512, 512, 512]
    out: List[Tensor] = []
    ci = 3
    for i, co in enumerate(widths, 1):
        out.append((f"conv{i}.weight", (co, ci, 3, 3)))
        out.append((f"conv{i}.bias", (co,)))
        ci = co
    for i, (o, n) in enumerate([(4096, 25088), (4096, 4096), (1000, 4096)], 14):
        out.append((f"fc{i}.weight", (o, n)))
        out.append((f"fc{i}.bias", (o,)))
    return out


def resnet50() -> List[Tensor]:
    out: List[Tensor] = []

    def conv_bn(name: str, co: int, ci: int, k: int) -> None:
        out.append((f"{name}.conv.weight", (co, ci, k, k)))
        out.append((f"{name}.bn.gamma", (co,)))
        out.append((f"{name}.bn.beta", (co,)))

    conv_bn("stem", 64, 3, 7)
    cin = 64
    for s, (depth, width) in enumerate(zip([3, 4, 6, 3], [64, 128, 256, 512]), 1):
        for b in range(depth):
            pre = f"stage{s}.block{b}"
            conv_bn(pre + ".a", width, cin, 1)
            conv_bn(pre + ".b", width, width, 3)
            conv_bn(pre + ".c", width * 4, width, 1)
            if b == 0:
                conv_bn(pre + ".down", width * 4, cin, 1)
            cin = width * 4
    out.append(("fc.weight", (1000, 2048)))
    out.append(("fc.bias", (1000,)))
    return out


def bert_base() -> List[Tensor]:
    h, ffn, layers = 768, 3072, 12
    out: List[Tensor] = [
        ("emb.word", (30522, h)),
        ("emb.position", (512, h)),
        ("emb.type", (2, h)),
        ("emb.ln.gamma", (h,)),
        ("emb.ln.beta", (h,)),
    ]
    for l in range(layers):
        pre = f"layer{l}"
        for nm in ("q", "k", "v", "o"):
            out.append((f"{pre}.attn.{nm}.weight", (h, h)))
            out.append((f"{pre}.attn.{nm}.bias", (h,)))
        out.append((f"{pre}.attn.ln.gamma", (h,)))
        out.append((f"{pre}.attn.ln.beta", (h,)))
        out.append((f"{pre}.ffn.in.weight", (ffn, h)))
        out.append((f"{pre}.ffn.in.bias", (ffn,)))
        out.append((f"{pre}.ffn.out.weight", (h, ffn)))
        out.append((f"{pre}.ffn.out.bias", (h,)))
        out.append((f"{pre}.ffn.ln.gamma", (h,)))
        out.append((f"{pre}.ffn.ln.beta", (h,)))
    out.append(("pooler.weight", (h, h)))
    out.append(("pooler.bias", (h,)))
    return out


def awd_lm() -> List[Tensor]:
    vocab, emb, hid = 33278, 400, 1150
    out: List[Tensor] = [("encoder.weight", (vocab, emb))]
    dims = [(emb, hid), (hid, hid), (hid, emb)]
    for l, (nin, nh) in enumerate(dims):
        out.append((f"rnn{l}.w_ih", (4 * nh, nin)))
        out.append((f"rnn{l}.w_hh", (4 * nh, nh)))
        out.append((f"rnn{l}.b_ih", (4 * nh,)))
        out.append((f"rnn{l}.b_hh", (4 * nh,)))
    # decoder weight is tied to the encoder: only its bias is a tensor of its own
    out.append(("decoder.bias", (vocab,)))
    return out


MODEL_BUILDERS: Dict[str, Callable[[], List[Tensor]]] = {
    "mlp": mlp,
    "alexnet": alexnet,
    "resnet50": resnet50,
    "vgg16": vgg16,
    "bert_base": bert_base,
    "awd_lm": awd_lm,
}


@dataclass(frozen=True)
class JobSpec:
    """One training job as the service sees it: layer sizes, worker count W and
    the optimizer's scalars, plus the spread of its synthetic values."""

    model: str
    layer_numel: Tuple[int, ...]
    W: int
    lr: float
    momentum: float
    wd: float
    grad_std: float
    param_std: float

    @property
    def n_params(self) -> int:
        return sum(self.layer_numel)


# (W, lr, momentum, wd, grad_std) of the single-job configurations
_SINGLE = {
    "mlp": (2, 0.1, 0.9, 1e-4, 0.01),
    "alexnet": (8, 0.01, 0.9, 5e-4, 1e-3),
    "resnet50": (16, 0.1, 0.9, 1e-4, 1e-3),
    "vgg16": (8, 0.01, 0.9, 5e-4, 1e-3),
    "bert_base": (8, 0.01, 0.9, 1e-4, 1e-3),
    "awd_lm": (8, 0.01, 0.9, 1e-4, 1e-3),
}


def job_config(model: str, W: int | None = None) -> JobSpec:
    w0, lr, mu, wd, gstd = _SINGLE[model]
    numel = tuple(_numel(s) for _, s in MODEL_BUILDERS[model]())
    return JobSpec(model, numel, w0 if W is None else int(W), lr, mu, wd, gstd, 0.05)


def packed_wave_jobs(seed: int = 42) -> List[JobSpec]:
    """Twelve concurrent jobs sharing one aggregation wave: 3 ResNet-50, 3 VGG-16,
    2 AlexNet, 2 BERT-base, 2 AWD-LM, each with W drawn from {2, 4, 8, 16} by the
    counter-based generator of values.py (stream "W-draw", one draw per job in
    list order)."""
    from .values import draw_from

    models = ["resnet50"] * 3 + ["vgg16"] * 3 + ["alexnet"] * 2 + ["bert_base"] * 2 + ["awd_lm"] * 2
    ws = draw_from(seed, "W-draw", len(models), (2, 4, 8, 16))
    return [job_config(m, w) for m, w in zip(models, ws)]
