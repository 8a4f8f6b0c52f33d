"""Synthetic gradient-set shapes for the five benchmark configurations.

Only tensor *sizes* matter to the aggregation path, so each model is described
by the list of its trainable tensors in forward order.  The lists follow the
published architectures (the paper's experiments, section 6 "DNN models", use
the same families of networks); no weights or datasets are involved.

This module holds no arithmetic of the aggregation method: it is shared by the
CPU oracle's tests and by the GPU path's tests and benchmark.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple

KB = 1 << 10
MB = 1 << 20

Tensor = Tuple[str, Tuple[int, ...]]


def _numel(shape: Tuple[int, ...]) -> int:
    n = 1
    for d in shape:
        n *= d
    return n


# --------------------------------------------------------------------------
# model tensor lists (forward order)
# --------------------------------------------------------------------------
def mlp() -> List[Tensor]:
    dims = [784, 256, 256, 10]
    out: List[Tensor] = []
    for i in range(3):
        out.append((f"fc{i + 1}.w", (dims[i], dims[i + 1])))
        out.append((f"fc{i + 1}.b", (dims[i + 1],)))
    return out


def _conv_bn(out: List[Tensor], name: str, kh: int, kw: int, cin: int, cout: int) -> None:
    out.append((f"{name}.kernel", (kh, kw, cin, cout)))
    out.append((f"{name}.bn.gamma", (cout,)))
    out.append((f"{name}.bn.beta", (cout,)))


def resnet50() -> List[Tensor]:
    out: List[Tensor] = []
    _conv_bn(out, "stem", 7, 7, 3, 64)
    cin = 64
    for stage, (blocks, p) in enumerate(zip([3, 4, 6, 3], [64, 128, 256, 512]), start=1):
        for b in range(blocks):
            pre = f"s{stage}.b{b}"
            _conv_bn(out, f"{pre}.c1", 1, 1, cin, p)
            _conv_bn(out, f"{pre}.c2", 3, 3, p, p)
            _conv_bn(out, f"{pre}.c3", 1, 1, p, 4 * p)
            if b == 0:
                _conv_bn(out, f"{pre}.proj", 1, 1, cin, 4 * p)
            cin = 4 * p
    out.append(("fc.w", (2048, 1000)))
    out.append(("fc.b", (1000,)))
    return out


def vgg16() -> List[Tensor]:
    out: List[Tensor] = []
    chans = [(3, 64), (64, 64), (64, 128), (128, 128), (128, 256), (256, 256), (256, 256),
             (256, 512), (512, 512), (512, 512), (512, 512), (512, 512), (512, 512)]
    for i, (cin, cout) in enumerate(chans, start=1):
        out.append((f"conv{i}.w", (3, 3, cin, cout)))
        out.append((f"conv{i}.b", (cout,)))
    for i, (fin, fout) in enumerate([(25088, 4096), (4096, 4096), (4096, 1000)], start=1):
        out.append((f"fc{i}.w", (fin, fout)))
        out.append((f"fc{i}.b", (fout,)))
    return out


def inception_v3() -> List[Tensor]:
    out: List[Tensor] = []
    n = [0]

    def conv(kh: int, kw: int, cin: int, cout: int) -> None:
        _conv_bn(out, f"conv{n[0]}", kh, kw, cin, cout)
        n[0] += 1

    # stem
    conv(3, 3, 3, 32); conv(3, 3, 32, 32); conv(3, 3, 32, 64); conv(1, 1, 64, 80); conv(3, 3, 80, 192)
    # three "A" blocks
    for cin, pool in [(192, 32), (256, 64), (288, 64)]:
        conv(1, 1, cin, 64)
        conv(1, 1, cin, 48); conv(5, 5, 48, 64)
        conv(1, 1, cin, 64); conv(3, 3, 64, 96); conv(3, 3, 96, 96)
        conv(1, 1, cin, pool)
    # grid reduction 288 -> 768
    conv(3, 3, 288, 384)
    conv(1, 1, 288, 64); conv(3, 3, 64, 96); conv(3, 3, 96, 96)
    # four "C" blocks
    for c in [128, 160, 160, 192]:
        conv(1, 1, 768, 192)
        conv(1, 1, 768, c); conv(1, 7, c, c); conv(7, 1, c, 192)
        conv(1, 1, 768, c); conv(7, 1, c, c); conv(1, 7, c, c); conv(7, 1, c, c); conv(1, 7, c, 192)
        conv(1, 1, 768, 192)
    # grid reduction 768 -> 1280
    conv(1, 1, 768, 192); conv(3, 3, 192, 320)
    conv(1, 1, 768, 192); conv(1, 7, 192, 192); conv(7, 1, 192, 192); conv(3, 3, 192, 192)
    # two "E" blocks
    for cin in [1280, 2048]:
        conv(1, 1, cin, 320)
        conv(1, 1, cin, 384); conv(1, 3, 384, 384); conv(3, 1, 384, 384)
        conv(1, 1, cin, 448); conv(3, 3, 448, 384); conv(1, 3, 384, 384); conv(3, 1, 384, 384)
        conv(1, 1, cin, 192)
    out.append(("fc.w", (2048, 1000)))
    out.append(("fc.b", (1000,)))
    return out


def transformer_encoder() -> List[Tensor]:
    h, ffn, layers, vocab = 1024, 4096, 24, 30522
    out: List[Tensor] = [
        ("emb.word", (vocab, h)), ("emb.pos", (512, h)), ("emb.type", (2, h)),
        ("emb.ln.gamma", (h,)), ("emb.ln.beta", (h,)),
    ]
    for l in range(layers):
        p = f"l{l}"
        for nm in ["q", "k", "v", "o"]:
            out.append((f"{p}.attn.{nm}.w", (h, h)))
            out.append((f"{p}.attn.{nm}.b", (h,)))
        out.append((f"{p}.ln1.gamma", (h,))); out.append((f"{p}.ln1.beta", (h,)))
        out.append((f"{p}.ffn.in.w", (h, ffn))); out.append((f"{p}.ffn.in.b", (ffn,)))
        out.append((f"{p}.ffn.out.w", (ffn, h))); out.append((f"{p}.ffn.out.b", (h,)))
        out.append((f"{p}.ln2.gamma", (h,))); out.append((f"{p}.ln2.beta", (h,)))
    out.append(("pooler.w", (h, h)))
    out.append(("pooler.b", (h,)))
    return out


def alexnet_v2() -> List[Tensor]:
    """The paper's model table lists 16 parameters, 191.9 MiB (section 6, "DNN models")."""
    out: List[Tensor] = []
    layers = [(11, 11, 3, 64), (5, 5, 64, 192), (3, 3, 192, 384), (3, 3, 384, 384), (3, 3, 384, 256),
              (5, 5, 256, 4096), (1, 1, 4096, 4096), (1, 1, 4096, 1000)]      # fc6-fc8 are convolutions
    for i, (kh, kw, cin, cout) in enumerate(layers, start=1):
        out.append((f"l{i}.w", (kh, kw, cin, cout)))
        out.append((f"l{i}.b", (cout,)))
    return out


def resnet_v2_152() -> List[Tensor]:
    """Pre-activation ResNet-152 with beta-only batch norms: the paper's table lists 363
    parameters, 229.5 MiB."""
    out: List[Tensor] = [("conv1.w", (7, 7, 3, 64)), ("conv1.b", (64,))]
    cin = 64
    for stage, (units, p) in enumerate(zip([3, 8, 36, 3], [64, 128, 256, 512]), start=1):
        for u in range(units):
            pre = f"b{stage}.u{u}"
            out.append((f"{pre}.preact.beta", (cin,)))
            if u == 0:
                out.append((f"{pre}.shortcut.w", (1, 1, cin, 4 * p)))
                out.append((f"{pre}.shortcut.b", (4 * p,)))
            out.append((f"{pre}.conv1.w", (1, 1, cin, p))); out.append((f"{pre}.conv1.bn.beta", (p,)))
            out.append((f"{pre}.conv2.w", (3, 3, p, p))); out.append((f"{pre}.conv2.bn.beta", (p,)))
            out.append((f"{pre}.conv3.w", (1, 1, p, 4 * p))); out.append((f"{pre}.conv3.b", (4 * p,)))
            cin = 4 * p
    out.append(("postnorm.beta", (2048,)))
    out.append(("logits.w", (1, 1, 2048, 1000)))
    out.append(("logits.b", (1000,)))
    return out


# --------------------------------------------------------------------------
# configurations
# --------------------------------------------------------------------------
SPLIT_NONE, SPLIT_FIXED, SPLIT_ADAPTIVE = 0, 1, 2
F32, BF16 = 0, 1


@dataclass(frozen=True)
class Workload:
    """One benchmark configuration: a tensor list plus the plan parameters."""
    name: str
    tensors: Tuple[Tensor, ...]          # forward order
    world: int                           # W, number of worker replicas
    dtype: int                           # F32 or BF16
    batch_threshold_bytes: int           # T
    split_mode: int
    split_bytes: int                     # S
    max_depth: int = 8
    align_bytes: int = 16
    num_streams: int = 2
    extra: dict = field(default_factory=dict, compare=False)

    @property
    def elem_size(self) -> int:
        return 4 if self.dtype == F32 else 2

    def update_order(self) -> List[Tensor]:
        """Order in which gradients become ready: the last layer's first.

        Backpropagation produces gradients from the output layer towards the
        input; the batcher (section 4.2) walks parameters by ascending update
        time, so the plan is fed the forward list reversed (within a layer the
        bias therefore precedes the weight)."""
        return list(reversed(self.tensors))

    def elems(self) -> List[int]:
        return [_numel(s) for _, s in self.update_order()]

    @property
    def total_elems(self) -> int:
        return sum(self.elems())

    def algorithmic_bytes(self) -> int:
        """Every replica element read once and written once."""
        return 2 * self.world * self.total_elems * self.elem_size


def workload(name: str) -> Workload:
    if name == "mlp":
        return Workload("mlp", tuple(mlp()), 4, F32, 64 * KB, SPLIT_NONE, 0)
    if name == "resnet50":
        return Workload("resnet50", tuple(resnet50()), 8, F32, 1 * MB, SPLIT_NONE, 0)
    if name == "vgg16":
        return Workload("vgg16", tuple(vgg16()), 8, F32, 1 * MB, SPLIT_FIXED, 4 * MB)
    if name == "inception_v3":
        return Workload("inception_v3", tuple(inception_v3()), 16, F32, 2 * MB, SPLIT_ADAPTIVE, 8 * MB)
    if name == "transformer":
        return Workload("transformer", tuple(transformer_encoder()), 8, BF16, 4 * MB, SPLIT_FIXED, 16 * MB)
    # the two remaining models of the paper's table, with the VGG-16 plan parameters
    if name == "alexnet_v2":
        return Workload("alexnet_v2", tuple(alexnet_v2()), 8, F32, 1 * MB, SPLIT_FIXED, 4 * MB)
    if name == "resnet_v2_152":
        return Workload("resnet_v2_152", tuple(resnet_v2_152()), 8, F32, 1 * MB, SPLIT_FIXED, 4 * MB)
    raise KeyError(name)


ALL = ("mlp", "resnet50", "vgg16", "inception_v3", "transformer")
EXTRA = ("alexnet_v2", "resnet_v2_152")
