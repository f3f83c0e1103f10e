"""Shared plumbing of the GPU parity tests: the oracle-side helpers and the comparison.

Inputs come from ``synth`` only (``synth.Inputs``); the GPU-side plumbing (arenas, views, the
library's context) is ``paper_2507_13522_amd.replica.GpuShadow``; both are re-exported here for
the tests.  The CPU oracle is imported only inside the helpers that run it.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List

import numpy as np

import paper_2507_13522_amd as sh
import synth
from paper_2507_13522_amd.replica import BENCH_BATCH_BYTES, BENCH_STREAMS, OPTIMIZERS, GpuShadow  # noqa: F401
from synth.inputs import TILE_PERIOD, Inputs  # noqa: F401


def oracle_layout(wl: synth.Workload):
    import oracle
    return oracle.build_layout([(t.numel, t.weight_decay) for t in wl.tensors], wl.grad_bytes, wl.bucket_cap_bytes,
                               wl.explicit_buckets)


def oracle_hparams(wl: synth.Workload, mean: bool = True, optimizer: str = "adamw"):
    import oracle
    return oracle.HParams(lr=wl.lr, beta1=wl.beta1, beta2=wl.beta2, eps=wl.eps, weight_decay=wl.weight_decay,
                          max_grad_norm=wl.max_grad_norm, mean=mean, optimizer=optimizer)


def lib_layout(wl: synth.Workload) -> sh.Layout:
    return sh.Layout([(t.numel, t.weight_decay) for t in wl.tensors], wl.grad_bytes, wl.bucket_cap_bytes,
                     wl.explicit_buckets)


def lib_hparams(wl: synth.Workload, num_streams: int = 2, mean: bool = True, batch_bytes: int = 0,
                optimizer: str = "adamw") -> sh.HParams:
    return sh.HParams(lr=wl.lr, beta1=wl.beta1, beta2=wl.beta2, eps=wl.eps, weight_decay=wl.weight_decay,
                      max_grad_norm=wl.max_grad_norm, num_workers=wl.num_workers,
                      grad_dtype=sh.GRAD_BF16 if wl.grad_dtype == "bf16" else sh.GRAD_F32,
                      reduce_op=sh.REDUCE_MEAN if mean else sh.REDUCE_SUM, num_streams=num_streams,
                      optimizer=OPTIMIZERS[optimizer], batch_bytes=batch_bytes)


def assert_layouts_agree(ol, ll: sh.Layout) -> None:
    assert ll.num_buckets == len(ol.buckets) and ll.num_params == ol.num_params
    prev_end = 0
    for b, ob in enumerate(ol.buckets):
        off, n, nt = ll.bucket(b)
        assert n == ob.numel and nt == len(ob.segments) and off % 64 == 0 and off >= prev_end and off - prev_end < 64
        prev_end = off + n
        for s in ob.segments:
            tb, tob, toa = ll.tensor(s.tensor)
            assert (tb, tob, toa) == (b, s.offset, off + s.offset)
    assert ll.arena_numel == (prev_end + 63) // 64 * 64


def run_oracle_full(wl: synth.Workload, inputs: Inputs, steps: int, orders=None, mean: bool = True, precision: str = "f32",
                    on_step=None, optimizer: str = "adamw"):
    """Whole-model oracle run (small and medium workloads)."""
    import oracle
    lay = oracle_layout(wl)
    starts = lay.logical_starts()
    params = [inputs.param_np(s, b.numel) for s, b in zip(starts, lay.buckets)]
    orc = oracle.OracleShadow(lay, oracle_hparams(wl, mean, optimizer), params, precision=precision)
    for t in range(1, steps + 1):
        grads = {b: [inputs.grad_np(t, w, starts[b], lay.buckets[b].numel) for w in range(wl.num_workers)]
                 for b in range(len(lay.buckets))}
        orc.step(grads)
        if on_step:
            on_step(t, orc)
    return orc


@dataclass
class Diff:
    max_rel: float
    n_bits_differ: int
    max_ulp: int

    def __str__(self) -> str:
        return f"max_rel={self.max_rel:.3e} bits_differ={self.n_bits_differ} max_ulp={self.max_ulp}"


def diff(got: np.ndarray, ref: np.ndarray) -> Diff:
    """max |got-ref| / max(|ref|, 1e-30), number of elements whose bits differ, largest distance in ulps."""
    got = np.ascontiguousarray(got, dtype=np.float32)
    ref = np.ascontiguousarray(ref, dtype=np.float32)
    assert got.shape == ref.shape
    if got.size == 0:
        return Diff(0.0, 0, 0)
    gb, rb = got.view(np.int32).astype(np.int64), ref.view(np.int32).astype(np.int64)
    nd = int(np.count_nonzero(gb != rb))
    if nd == 0:
        return Diff(0.0, 0, 0)
    g64, r64 = got.astype(np.float64), ref.astype(np.float64)
    rel = float(np.max(np.abs(g64 - r64) / np.maximum(np.abs(r64), 1e-30)))
    mono = lambda x: np.where(x < 0, -(x & 0x7FFFFFFF), x)
    ulp = int(np.max(np.abs(mono(gb) - mono(rb))))
    return Diff(rel, nd, ulp)


REL_TOL = 1e-6      # max relative error on param, m and v


def assert_state_matches(got, ref, what: str, exact: bool = True) -> List[Diff]:
    out = []
    for name, g, r in zip("pmv", got, ref):
        d = diff(g, r)
        out.append(d)
        assert d.max_rel <= REL_TOL, f"{what} {name}: {d}"
        if exact:
            assert d.n_bits_differ == 0, f"{what} {name}: expected identical bits, {d}"
    return out
