"""Gradient layouts of the five benchmark configurations.

Pure bookkeeping: lists of parameter-tensor sizes in model-definition order and the
bucket tables built from them.  No arithmetic of the method lives here; the module is
shared by the CPU oracle's tests and the GPU path's tests/bench as an input recipe.

The models are the ones the paper evaluates (Table 1: ResNet-50 with 25,559,081
parameters; an LSTM video classifier) plus two transformer-shaped layouts for scale.
Layer-wise buckets follow the paper's description of gradient exchange as one
reduction per layer/tensor, possibly fused into larger messages (Sections 1 and 3).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Sequence, Tuple

Tensor = Tuple[str, int]


def flat_tensors(numel: int) -> List[Tensor]:
    return [("flat", int(numel))]


def resnet50_tensors(num_classes: int = 1001) -> List[Tensor]:
    """Bottleneck ResNet-50; the 1001-class head reproduces Table 1's 25,559,081."""
    t: List[Tensor] = []

    def conv_bn(name: str, cin: int, cout: int, k: int) -> None:
        t.append((f"{name}.conv", k * k * cin * cout))
        t.append((f"{name}.bn.gamma", cout))
        t.append((f"{name}.bn.beta", cout))

    conv_bn("stem", 3, 64, 7)
    cin = 64
    for s, (blocks, width) in enumerate(zip((3, 4, 6, 3), (64, 128, 256, 512))):
        for b in range(blocks):
            base = f"stage{s}.block{b}"
            conv_bn(base + ".a", cin, width, 1)
            conv_bn(base + ".b", width, width, 3)
            conv_bn(base + ".c", width, 4 * width, 1)
            if b == 0:
                conv_bn(base + ".down", cin, 4 * width, 1)
            cin = 4 * width
    t.append(("fc.weight", 2048 * num_classes))
    t.append(("fc.bias", num_classes))
    return t


def lstm_tensors(layers: int = 2, inp: int = 2048, hidden: int = 2048,
                 classes: int = 101) -> List[Tensor]:
    """Stacked LSTM (4*H*(I+H+1) weights per layer) followed by a dense classifier."""
    t: List[Tensor] = []
    i = inp
    for l in range(layers):
        t.append((f"lstm{l}.w_ih", 4 * hidden * i))
        t.append((f"lstm{l}.w_hh", 4 * hidden * hidden))
        t.append((f"lstm{l}.bias", 4 * hidden))
        i = hidden
    t.append(("fc.weight", hidden * classes))
    t.append(("fc.bias", classes))
    return t


def transformer_tensors(layers: int, d: int, ffn: int, vocab: int = 50257,
                        positions: int = 1024) -> List[Tensor]:
    """Decoder-only transformer in the GPT-2 arrangement."""
    t: List[Tensor] = [("wte", vocab * d), ("wpe", positions * d)]
    for l in range(layers):
        b = f"h{l}"
        t += [(b + ".ln1.gamma", d), (b + ".ln1.beta", d),
              (b + ".qkv.weight", d * 3 * d), (b + ".qkv.bias", 3 * d),
              (b + ".proj.weight", d * d), (b + ".proj.bias", d),
              (b + ".ln2.gamma", d), (b + ".ln2.beta", d),
              (b + ".fc1.weight", d * ffn), (b + ".fc1.bias", ffn),
              (b + ".fc2.weight", ffn * d), (b + ".fc2.bias", d)]
    t += [("lnf.gamma", d), ("lnf.beta", d)]
    return t


@dataclass(frozen=True)
class BucketTable:
    """Buckets inside one flat per-process arena.

    offset[b] (elements) is where bucket b starts, numel[b] its length.  Starts are
    aligned to `align` elements (16 bytes of the gradient dtype, so that the fp32 state
    arrays are at least as aligned); the gap after a bucket is padding that carries no
    data.  arena_numel is the allocation size per process, in elements.
    """
    offset: Tuple[int, ...]
    numel: Tuple[int, ...]
    arena_numel: int
    align: int

    @property
    def n_buckets(self) -> int:
        return len(self.numel)

    @property
    def total(self) -> int:
        return sum(self.numel)


def _round_up(x: int, a: int) -> int:
    return (x + a - 1) // a * a


def buckets_per_tensor(tensors: Sequence[Tensor], align: int) -> BucketTable:
    off, num, cur = [], [], 0
    for _, n in tensors:
        off.append(cur)
        num.append(n)
        cur = _round_up(cur + n, align)
    return BucketTable(tuple(off), tuple(num), cur, align)


def buckets_greedy(tensors: Sequence[Tensor], cap_bytes: int, grad_bytes: int,
                   align: int) -> BucketTable:
    """Fill buckets in definition order up to cap_bytes of gradient data, cutting only
    at tensor boundaries; a tensor larger than the cap is a bucket of its own."""
    groups: List[int] = []
    cur = 0
    for _, n in tensors:
        if cur and (cur + n) * grad_bytes > cap_bytes:
            groups.append(cur)
            cur = 0
        cur += n
    if cur:
        groups.append(cur)
    return buckets_per_tensor([("g", n) for n in groups], align)


@dataclass(frozen=True)
class Config:
    name: str
    P: int
    mode: str            # "solo" | "majority"
    grad_dtype: str      # "f32" | "bf16"
    steps: int
    times: str           # compute-time recipe, see workloads.times
    tensors: Tuple[Tensor, ...]
    buckets: BucketTable
    lr: float = 0.1
    mu: float = 0.9
    grad_sigma: float = 1e-3
    param_sigma: float = 0.02
    seed: int = 190804207

    @property
    def numel(self) -> int:
        return self.buckets.total


_CAP = 25 * 2 ** 20


def config(k: int) -> Config:
    """Configuration k = 1..5 (the benchmark list is 1-based)."""
    if k == 1:
        ts = flat_tensors(2 ** 20)
        return Config("cfg1_flat1M_P4_solo", 4, "solo", "f32", 10, "uniform_1_2",
                      tuple(ts), buckets_per_tensor(ts, 4), seed=190804207 + 1)
    if k == 2:
        ts = resnet50_tensors()
        return Config("cfg2_resnet50_P8_majority", 8, "majority", "f32", 100,
                      "lognormal_0.3_straggler2x", tuple(ts), buckets_per_tensor(ts, 4),
                      seed=190804207 + 2)
    if k == 3:
        ts = lstm_tensors()
        return Config("cfg3_lstm_P16_solo", 16, "solo", "f32", 100, "pareto_1.5",
                      tuple(ts), buckets_per_tensor(ts, 4), seed=190804207 + 3)
    if k == 4:
        ts = transformer_tensors(24, 1024, 4096)
        return Config("cfg4_transformer350M_P32_majority", 32, "majority", "f32", 50,
                      "lognormal_0.5", tuple(ts), buckets_greedy(ts, _CAP, 4, 4),
                      seed=190804207 + 4)
    if k == 5:
        ts = transformer_tensors(48, 1600, 6400)
        return Config("cfg5_gpt2xl_P16_solo_bf16", 16, "solo", "bf16", 20, "pareto_1.2",
                      tuple(ts), buckets_greedy(ts, _CAP, 2, 8), seed=190804207 + 5)
    raise ValueError(f"no configuration {k}")


def scaled(cfg: Config, max_tensor: int) -> Config:
    """Same layout with every tensor clipped to max_tensor elements: keeps the bucket
    count, the mix of tiny and large buckets and the ragged sizes, at a size a CPU
    reference finishes quickly."""
    ts = [(n, min(s, max_tensor)) for n, s in cfg.tensors]
    align = cfg.buckets.align
    if cfg.name.startswith(("cfg4", "cfg5")):
        gb = 2 if cfg.grad_dtype == "bf16" else 4
        # cap scaled so that several tensors still share a bucket
        bt = buckets_greedy(ts, max(4 * max_tensor * gb, 64), gb, align)
    else:
        bt = buckets_per_tensor(ts, align)
    return Config(cfg.name + f"_clip{max_tensor}", cfg.P, cfg.mode, cfg.grad_dtype,
                  cfg.steps, cfg.times, tuple(ts), bt, cfg.lr, cfg.mu, cfg.grad_sigma,
                  cfg.param_sigma, cfg.seed)
