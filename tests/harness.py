"""Shared plumbing of the GPU parity tests: inputs, arenas, comparison.

Inputs come from ``synth`` only.  Small cases use a distinct value per element;
cases at model size use tiled inputs (element e takes the tile's value at
e mod L, L prime) so that the oracle can obtain the global gradient norm from
one tile with multiplicities and then check sampled elements and whole sampled
buckets exactly.  Tiles are always generated on the CPU and uploaded, so both
sides see the same bits whatever the device's float arithmetic does.
"""
from __future__ import annotations

import os
from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

import paper_2507_13522_amd as sh
import synth

# The CPU oracle is imported only inside the helpers that run it (oracle_layout, oracle_hparams,
# run_oracle_full): the GPU-side plumbing below, which bench.py also uses, never touches it.

TILE_PERIOD = 1_000_003          # prime
# launch configuration that bench.py times (and the full-size parity test repeats)
BENCH_STREAMS = 1
BENCH_BATCH_BYTES = 4 << 30


class Inputs:
    """Gradient views and initial parameters of a workload, on CPU (numpy) and on the GPU (torch)."""

    def __init__(self, wl: synth.Workload, period: Optional[int] = None, device: Optional[str] = None):
        self.wl, self.period, self.device = wl, period, device
        self._tiles: Dict = {}
        self._tiles_dev: Dict = {}

    # -- CPU ---------------------------------------------------------------
    def _tile(self, key):
        if key not in self._tiles:
            idx = torch.arange(self.period, dtype=torch.int64)
            if key == "param":
                t = synth.param_values(self.wl.seed, idx, self.wl.param_sigma)
            else:
                step, w = key
                t = synth.grad_values(self.wl.seed, step, w, idx, self.wl.grad_dist, self.wl.grad_sigma, self.wl.grad_dtype)
            self._tiles[key] = t
            if len(self._tiles) > 80:
                self._tiles.pop(next(iter(self._tiles)))
        return self._tiles[key]

    def grad_at(self, step: int, w: int, idx: torch.Tensor) -> torch.Tensor:
        """CPU tensor (float32, or int16 bfloat16 patterns) at logical element indices idx."""
        if self.period:
            return synth.tiled(self._tile((step, w)), idx)
        return synth.grad_values(self.wl.seed, step, w, idx, self.wl.grad_dist, self.wl.grad_sigma, self.wl.grad_dtype)

    def param_at(self, idx: torch.Tensor) -> torch.Tensor:
        if self.period:
            return synth.tiled(self._tile("param"), idx)
        return synth.param_values(self.wl.seed, idx, self.wl.param_sigma)

    def _range_np(self, key, start: int, n: int) -> np.ndarray:
        """Values at the contiguous logical range [start, start+n) of a tiled input (wrap-around copies)."""
        tile = self._tile(key).numpy()
        L = tile.size
        out = np.empty(n, tile.dtype)
        pos, src = 0, start % L
        while pos < n:
            k = min(L - src, n - pos)
            out[pos:pos + k] = tile[src:src + k]
            pos += k
            src = 0
        return out

    def grad_np(self, step: int, w: int, start: int, n: int) -> np.ndarray:
        if self.period:
            a = self._range_np((step, w), start, n)
        else:
            a = self.grad_at(step, w, torch.arange(start, start + n, dtype=torch.int64)).numpy()
        return a.view(np.uint16).copy() if self.wl.grad_dtype == "bf16" else a.copy()

    def param_np(self, start: int, n: int) -> np.ndarray:
        if self.period:
            return self._range_np("param", start, n)
        return self.param_at(torch.arange(start, start + n, dtype=torch.int64)).numpy().copy()

    # -- GPU ---------------------------------------------------------------
    def _tile_dev(self, key):
        if key not in self._tiles_dev:
            self._tiles_dev[key] = self._tile(key).to(self.device)
            if len(self._tiles_dev) > 80:
                self._tiles_dev.pop(next(iter(self._tiles_dev)))
        return self._tiles_dev[key]

    def fill_grad_dev(self, out: torch.Tensor, step: int, w: int, start: int) -> None:
        n = out.numel()
        if self.period:
            idx = torch.arange(start, start + n, dtype=torch.int64, device=self.device)
            torch.index_select(self._tile_dev((step, w)), 0, idx % self.period, out=out)
        else:
            out.copy_(self.grad_at(step, w, torch.arange(start, start + n, dtype=torch.int64)))

    def fill_param_dev(self, out: torch.Tensor, start: int) -> None:
        n = out.numel()
        if self.period:
            idx = torch.arange(start, start + n, dtype=torch.int64, device=self.device)
            torch.index_select(self._tile_dev("param"), 0, idx % self.period, out=out)
        else:
            out.copy_(self.param_at(torch.arange(start, start + n, dtype=torch.int64)))


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


OPTIMIZERS = {"adamw": sh.OPT_ADAMW, "adam": sh.OPT_ADAM, "sgd": sh.OPT_SGD}


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


# Replicas whose arenas reach this size are placed by the library's device plan (one 256 GiB allocation made first
# thing, arenas and staging buffer at the advised offsets); smaller ones, the parity cases, by its stride advice.
DEVICE_PLAN_MIN_ARENA_BYTES = 256 << 20


class GpuShadow:
    """The library on cuda:0 over torch-allocated arenas, with every bucket's W views resident."""

    def __init__(self, wl: synth.Workload, inputs: Inputs, num_streams: int = 2, mean: bool = True,
                 torch_streams: bool = False, resident_grads: bool = True, init_from=None, start_step: int = 0,
                 advised_placement: bool = True, batch_bytes: int = 0, refold: bool = False, optimizer: str = "adamw",
                 ring_bytes: int = 0):
        assert torch.cuda.is_available()
        self.wl, self.inputs = wl, inputs
        self.dev = torch.device("cuda:0")
        inputs.device = self.dev
        self.layout = lib_layout(wl)
        L = self.layout
        self.buckets = [L.bucket(b) for b in range(L.num_buckets)]
        self.logical_start, acc = [], 0
        for off, n, _ in self.buckets:
            self.logical_start.append(acc)
            acc += n
        A = L.arena_numel
        clip = wl.max_grad_norm > 0
        narr = 4 if (clip and not refold) else 3          # re-fold mode: clipping without a scratch arena
        W = wl.num_workers
        stage_bytes = max(L.staging_bytes(W), 256) if resident_grads else 0
        # ring_bytes > 0 (timing only): the views do not all fit, so bucket after bucket takes the next piece of a
        # ring of that size and later buckets reuse the memory of earlier ones; contents are then meaningless
        self._ring_off = None
        if resident_grads and ring_bytes:
            self._ring_off, cur = [], 0
            for b in range(L.num_buckets):
                need = (L.staging_view(W, b, W - 1) - L.staging_view(W, b, 0)) + self.buckets[b][1] * wl.grad_bytes
                need = (need + (2 << 20) - 1) // (2 << 20) * (2 << 20)
                assert need <= ring_bytes, "ring smaller than one bucket's views"
                if cur + need > ring_bytes:
                    cur = 0
                self._ring_off.append(cur)
                cur += need
            stage_bytes = ring_bytes
        plan = None
        if advised_placement and A * 4 >= DEVICE_PLAN_MIN_ARENA_BYTES:
            plan = L.device_plan(narr == 4, stage_bytes)
        self._stage = None
        if plan is not None:
            # model-size workloads: ONE 256 GiB allocation, arenas and staging at the planned offsets
            self._state = torch.empty(plan.block_bytes, dtype=torch.uint8, device=self.dev)
            offs = [plan.param_offset, plan.m_offset, plan.v_offset] + ([plan.scratch_offset] if narr == 4 else [])
            arenas = [self._state[o:o + A * 4].view(torch.float32) for o in offs]
            if resident_grads:
                self._stage = self._state[plan.staging_offset:plan.staging_offset + stage_bytes]
        else:
            # placement follows the library's advice: the arenas are carved from one allocation, a power-of-two
            # stride apart; the gradient views sit in a bucket-major staging buffer
            stride = L.arena_stride() if advised_placement else (A * 4 + 255) // 256 * 256
            self._state = torch.empty((narr - 1) * stride + A * 4, dtype=torch.uint8, device=self.dev)
            arenas = [self._state[k * stride:k * stride + A * 4].view(torch.float32) for k in range(narr)]
            if resident_grads:
                self._stage = torch.empty(stage_bytes, dtype=torch.uint8, device=self.dev)
        self.p, self.m, self.v = arenas[:3]
        self.r = arenas[3] if narr == 4 else None
        self.m.zero_()
        self.v.zero_()
        if init_from is None:
            for (off, n, _), ls in zip(self.buckets, self.logical_start):
                inputs.fill_param_dev(self.p[off:off + n], ls)
        else:
            self.p.copy_(init_from[0]); self.m.copy_(init_from[1]); self.v.copy_(init_from[2])
        gdt = torch.int16 if wl.grad_dtype == "bf16" else torch.float32
        self.gdt = gdt
        self.hp = lib_hparams(wl, num_streams, mean, batch_bytes, optimizer)
        self.optimizer = optimizer
        self._tstreams = [torch.cuda.Stream(device=self.dev) for _ in range(num_streams)] if torch_streams else None
        torch.cuda.synchronize()
        self.ctx = sh.Shadow(L, self.hp, self.p.data_ptr(), self.m.data_ptr(), None if optimizer == "sgd" else self.v.data_ptr(),
                             self.r.data_ptr() if self.r is not None else None, start_step,
                             [s.cuda_stream for s in self._tstreams] if self._tstreams else None)
        self._views = None
        if resident_grads:
            self._views = [self.ctx.views_array([self.view(b, w).data_ptr() for w in range(W)])
                           for b in range(len(self.buckets))]

    def view(self, b: int, w: int) -> torch.Tensor:
        """Worker w's gradient view of bucket b inside the staging buffer."""
        n = self.buckets[b][1]
        W = self.wl.num_workers
        off = self.layout.staging_view(W, b, w)
        if self._ring_off is not None:
            off = self._ring_off[b] + off - self.layout.staging_view(W, b, 0)
        return self._stage[off:off + n * self.wl.grad_bytes].view(self.gdt)

    def fill_grads(self, step: int, buckets: Optional[Sequence[int]] = None) -> None:
        for b in (range(len(self.buckets)) if buckets is None else buckets):
            for w in range(self.wl.num_workers):
                self.inputs.fill_grad_dev(self.view(b, w), step, w, self.logical_start[b])
        torch.cuda.synchronize()

    def apply_step(self, step: int, order: Optional[Sequence[int]] = None) -> None:
        for b in (range(len(self.buckets)) if order is None else order):
            self.ctx.apply_bucket(b, self._views[b], step)

    def run_step(self, step: int, order: Optional[Sequence[int]] = None) -> None:
        self.fill_grads(step)
        self.apply_step(step, order)
        self.ctx.sync()

    def bucket_state(self, b: int):
        off, n, _ = self.buckets[b]
        self.ctx.sync()
        return tuple(x[off:off + n].cpu().numpy() for x in (self.p, self.m, self.v))

    def close(self) -> None:
        self.ctx.destroy()


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
