"""Inputs of a workload as arrays: gradient views and initial parameters, on the CPU (numpy) and on a GPU (torch).

Data plumbing only (no arithmetic of the method).  Small cases give every element its own
value; cases at model size use tiled inputs (element e takes the tile's value at e mod L, L
prime), so that a checker can obtain global statistics from one tile with multiplicities.
Tiles are always generated on the CPU and uploaded, so both sides of a comparison read the
same bits whatever the device's float arithmetic does.
"""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np
import torch

from .rng import grad_values, param_values, tiled
from .workloads import Workload

TILE_PERIOD = 1_000_003          # prime
FILL_PIECE = 1 << 27             # elements filled per step on the device


class Inputs:
    def __init__(self, wl: Workload, period: Optional[int] = None, device: Optional[str] = None):
        self.wl, self.period, self.device = wl, period, device
        self._tiles: Dict = {}
        self._tiles_dev: Dict = {}

    # -- CPU ---------------------------------------------------------------
    def _tile(self, key):
        if key not in self._tiles:
            idx = torch.arange(self.period, dtype=torch.int64)
            if key == "param":
                t = param_values(self.wl.seed, idx, self.wl.param_sigma)
            else:
                step, w = key
                t = grad_values(self.wl.seed, step, w, idx, self.wl.grad_dist, self.wl.grad_sigma, self.wl.grad_dtype)
            self._tiles[key] = t
            if len(self._tiles) > 80:
                self._tiles.pop(next(iter(self._tiles)))
        return self._tiles[key]

    def grad_at(self, step: int, w: int, idx: torch.Tensor) -> torch.Tensor:
        """CPU tensor (float32, or int16 bfloat16 patterns) at logical element indices idx."""
        if self.period:
            return tiled(self._tile((step, w)), idx)
        return grad_values(self.wl.seed, step, w, idx, self.wl.grad_dist, self.wl.grad_sigma, self.wl.grad_dtype)

    def param_at(self, idx: torch.Tensor) -> torch.Tensor:
        if self.period:
            return tiled(self._tile("param"), idx)
        return param_values(self.wl.seed, idx, self.wl.param_sigma)

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

    def _fill_tiled_dev(self, key, out: torch.Tensor, start: int) -> None:
        """out[i] = tile[(start + i) mod period], in pieces so that the index arrays stay small beside a large out."""
        tile, n = self._tile_dev(key), out.numel()
        for s in range(0, n, FILL_PIECE):
            k = min(FILL_PIECE, n - s)
            idx = torch.arange(start + s, start + s + k, dtype=torch.int64, device=self.device)
            torch.index_select(tile, 0, idx % self.period, out=out[s:s + k])

    def fill_grad_dev(self, out: torch.Tensor, step: int, w: int, start: int) -> None:
        if self.period:
            self._fill_tiled_dev((step, w), out, start)
        else:
            out.copy_(self.grad_at(step, w, torch.arange(start, start + out.numel(), dtype=torch.int64)))

    def fill_param_dev(self, out: torch.Tensor, start: int) -> None:
        if self.period:
            self._fill_tiled_dev("param", out, start)
        else:
            out.copy_(self.param_at(torch.arange(start, start + out.numel(), dtype=torch.int64)))
