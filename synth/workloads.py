"""Tensor lists and hyper-parameters of the five synthetic workloads.

Shapes are the public architecture dimensions of the models the workloads are
named after; values come from ``synth.rng``.  The optimizer-scaling experiment
of the paper (section 6.4) runs optimizer steps over randomized gradients on
real model shapes, which is what these workloads stand in for.  Nothing here
assigns tensors to buckets: that is part of the method.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional

from .rng import BASE_SEED, GAMMA, STREAM_LAYOUT, splitmix64_scalar, stream_base

MIB = 1 << 20


@dataclass(frozen=True)
class TensorSpec:
    name: str
    numel: int
    weight_decay: bool


@dataclass
class Workload:
    name: str
    tensors: List[TensorSpec]
    num_workers: int
    grad_dtype: str            # "f32" | "bf16"
    grad_dist: str             # "normal" | "t3"
    grad_sigma: float
    steps: int
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    weight_decay: float = 0.01
    max_grad_norm: float = 0.0             # <= 0: no clipping
    bucket_cap_bytes: int = 25 * MIB       # in gradient bytes
    explicit_buckets: Optional[List[int]] = None   # bucket id per tensor (model order), or None
    random_arrival: bool = False
    param_sigma: float = 0.02
    seed: int = BASE_SEED
    notes: str = ""

    @property
    def num_params(self) -> int:
        return sum(t.numel for t in self.tensors)

    @property
    def grad_bytes(self) -> int:
        return 4 if self.grad_dtype == "f32" else 2


def _tiny() -> Workload:
    ts = [TensorSpec(f"t{i}", 262144, True) for i in range(4)]
    return Workload("tiny", ts, num_workers=4, grad_dtype="f32", grad_dist="normal", grad_sigma=1e-3,
                    steps=10, explicit_buckets=[0, 1, 2, 3])


def _gpt_like(d: int, layers: int, ffn: int, vocab: int, ctx: int, mask_1d: bool) -> List[TensorSpec]:
    wd1 = not mask_1d
    ts = [TensorSpec("tok_emb", vocab * d, True), TensorSpec("pos_emb", ctx * d, True)]
    for l in range(layers):
        p = f"h{l}."
        ts += [
            TensorSpec(p + "ln1.w", d, wd1), TensorSpec(p + "ln1.b", d, wd1),
            TensorSpec(p + "attn_in.w", d * 3 * d, True), TensorSpec(p + "attn_in.b", 3 * d, wd1),
            TensorSpec(p + "attn_out.w", d * d, True), TensorSpec(p + "attn_out.b", d, wd1),
            TensorSpec(p + "ln2.w", d, wd1), TensorSpec(p + "ln2.b", d, wd1),
            TensorSpec(p + "fc.w", d * ffn, True), TensorSpec(p + "fc.b", ffn, wd1),
            TensorSpec(p + "proj.w", ffn * d, True), TensorSpec(p + "proj.b", d, wd1),
        ]
    ts += [TensorSpec("ln_f.w", d, wd1), TensorSpec("ln_f.b", d, wd1)]
    return ts


def _gpt2_small() -> Workload:
    ts = _gpt_like(768, 12, 3072, 50257, 1024, mask_1d=False)
    return Workload("gpt2s", ts, num_workers=8, grad_dtype="bf16", grad_dist="normal", grad_sigma=1e-3,
                    steps=20, bucket_cap_bytes=25 * MIB)


def _gpt_1p3b() -> Workload:
    ts = _gpt_like(2048, 24, 8192, 50257, 2048, mask_1d=True)
    return Workload("gpt1p3b", ts, num_workers=16, grad_dtype="bf16", grad_dist="t3", grad_sigma=1e-3,
                    steps=10, max_grad_norm=1.0, bucket_cap_bytes=25 * MIB)


def _llama7b_tensors() -> List[TensorSpec]:
    d, ffn, vocab, layers = 4096, 11008, 32000, 32
    ts = [TensorSpec("tok_emb", vocab * d, True)]
    for l in range(layers):
        p = f"l{l}."
        ts += [TensorSpec(p + "attn_norm", d, False)]
        ts += [TensorSpec(p + n, d * d, True) for n in ("wq", "wk", "wv", "wo")]
        ts += [TensorSpec(p + "ffn_norm", d, False)]
        ts += [TensorSpec(p + "w1", d * ffn, True), TensorSpec(p + "w3", d * ffn, True),
               TensorSpec(p + "w2", ffn * d, True)]
    ts += [TensorSpec("norm_f", d, False), TensorSpec("lm_head", vocab * d, True)]
    return ts


def _llama7b() -> Workload:
    return Workload("llama7b", _llama7b_tensors(), num_workers=8, grad_dtype="bf16", grad_dist="normal",
                    grad_sigma=1e-3, steps=5, max_grad_norm=1.0, bucket_cap_bytes=50 * MIB)


def _llama7b_w1() -> Workload:
    """The paper's own situation: the shadow receives ONE already-reduced gradient per bucket (W = 1)."""
    return Workload("llama7b_w1", _llama7b_tensors(), num_workers=1, grad_dtype="bf16", grad_dist="normal",
                    grad_sigma=3.5e-4, steps=3, max_grad_norm=1.0, bucket_cap_bytes=50 * MIB)


def _ragged7b() -> Workload:
    """7B tensor list plus 1,709 small ragged tensors at seeded positions.

    Extra sizes are log-uniform in [64, 2**20], bumped off multiples of 128;
    every tensor's weight-decay flag is a seeded coin flip.
    """
    seed = BASE_SEED
    base = stream_base(seed, STREAM_LAYOUT)
    core = _llama7b_tensors()
    n_extra = 2000 - len(core)

    def u(n: int) -> int:
        return splitmix64_scalar(base + (n + 1) * GAMMA)

    extras = []
    for k in range(n_extra):
        frac = (u(3 * k) >> 11) / float(1 << 53)
        n = int(math.floor(64.0 * math.exp(frac * math.log((1 << 20) / 64.0))))
        n = max(64, min(n, 1 << 20))
        if n % 128 == 0:
            n += 1 + u(3 * k + 1) % 127
        pos = u(3 * k + 2) % (len(core) + 1)
        extras.append((pos, k, n))
    # stable insertion: extras with the same position keep their draw order
    out: List[TensorSpec] = []
    by_pos = {}
    for pos, k, n in extras:
        by_pos.setdefault(pos, []).append((k, n))
    for i in range(len(core) + 1):
        for k, n in by_pos.get(i, []):
            out.append(TensorSpec(f"x{k}", n, True))
        if i < len(core):
            out.append(core[i])
    flagged = []
    for i, t in enumerate(out):
        flag = bool(u(1_000_000 + i) & 1)
        flagged.append(TensorSpec(t.name, t.numel, flag))
    return Workload("ragged7b", flagged, num_workers=32, grad_dtype="bf16", grad_dist="normal",
                    grad_sigma=1e-3, steps=3, max_grad_norm=0.5, bucket_cap_bytes=50 * MIB,
                    random_arrival=True)


WORKLOADS = {
    "tiny": _tiny,
    "gpt2s": _gpt2_small,
    "gpt1p3b": _gpt_1p3b,
    "llama7b": _llama7b,
    "llama7b_w1": _llama7b_w1,
    "ragged7b": _ragged7b,
}


def get_workload(name: str) -> Workload:
    return WORKLOADS[name]()
