"""Seeded synthetic inputs for the five benchmark configurations.

This module only draws random numbers and lays them out; it holds none of the
method's arithmetic and is the one piece that the tests hand to both the GPU
library and the CPU oracle (each side receives the same bytes).

The inputs stand in for the paper's training runs (Sec. V-A3: WideResNets on
CIFAR/ImageNet, BERT on SQuAD), which need datasets and trained models that
are not available here.  What they keep from those workloads: every worker
starts from the same model (Listing 1, model_generator), gradients are a
shared signal plus per-worker noise (Assumption 2, bounded variance), the
flat-vector sizes are those of ResNet-18 / ResNet-50 / VGG-16, and the ragged
case is a layer list with sizes spread over four orders of magnitude
(Sec. V-A1, layer-by-layer synchronisation).

Recipe (one ``torch.Generator`` per run, seeded with the configuration's seed,
draw order fixed):
  1. ``x0 ~ N(0, 0.02^2)`` of length P, copied to all W rows;
  2. configuration 3 only: per-worker scale ``c_i ~ U(0.5, 2)``, once;
  3. every iteration: ``mu ~ N(0,1)^P``, then ``z ~ N(0,1)^(W x P)``,
     ``G = c_i * (mu + 0.5 z)`` in fp32 (``c_i = 1`` unless configuration 3),
     rounded to bf16 (nearest even) for configuration 5.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import List, Optional, Tuple

import numpy as np
import torch


@dataclass(frozen=True)
class Config:
    name: str
    W: int
    group: int            # size of every group
    P: int                # columns per replica (ragged: filled in by segments())
    T: int
    seed: int
    lr: float
    worker_scale: bool = False
    bf16_grads: bool = False
    ragged: bool = False

    @property
    def sizes(self) -> List[int]:
        return [self.group] * (self.W // self.group)


CONFIGS = {
    1: Config("cfg1 W=8 g=4 P=1,048,576 fp32", 8, 4, 1_048_576, 20, 0, 0.01),
    2: Config("cfg2 W=16 g=4 P=11,689,512 fp32 (ResNet-18-sized)", 16, 4, 11_689_512, 10, 1, 0.01),
    3: Config("cfg3 W=32 g=8 P=25,557,032 fp32 (ResNet-50-sized)", 32, 8, 25_557_032, 5, 2, 0.01,
              worker_scale=True),
    4: Config("cfg4 W=64 g=8 P=138,357,544 fp32 (VGG-16-sized)", 64, 8, 138_357_544, 3, 3, 0.005),
    5: Config("cfg5 W=32 g=4 ragged 199 segments ~110M, bf16 grads", 32, 4, 0, 5, 4, 0.01,
              bf16_grads=True, ragged=True),
}


def padded_ld(P: int, pad: int = 256) -> int:
    """Leading dimension used by the benchmark layout: the row length rounded
    up to an odd multiple of ``pad`` elements.  With ``pad`` = 256 every row of
    an fp32 stack starts on a 1-KiB boundary, so each 1-KiB wavefront access
    of the kernels covers one aligned KiB of its row (measured 2-4 % faster
    than rows that start on other 256-byte boundaries), and the odd multiple
    keeps the row pitch away from large powers of two, where rows of equal
    column would map to the same memory channels."""
    n = (int(P) + pad - 1) // pad
    if n % 2 == 0:
        n += 1
    return n * pad


def ragged_segments(seed: int = 4, n_segments: int = 199, lo: int = 256, hi: int = 4_194_304,
                    total_range: Tuple[int, int] = (99_000_000, 121_000_000),
                    pad: int = 256) -> Tuple[List[Tuple[int, int]], int, int]:
    """Layer list of configuration 5: ``n_segments`` lengths log-uniform in
    ``[lo, hi]``; the first draw (attempt 0, 1, ...) whose total lies in
    ``total_range`` is taken.  Offsets are padded up to multiples of ``pad``
    elements (1 KiB of fp32) and the leading dimension to an odd multiple of
    it, as in :func:`padded_ld`.  Returns ``(segments as (offset, length), ld,
    attempt)``.
    """
    attempt = 0
    while True:
        rng = np.random.Generator(np.random.Philox(key=[seed, attempt]))
        lengths = np.rint(np.exp(rng.uniform(math.log(lo), math.log(hi), n_segments))).astype(np.int64)
        if total_range[0] <= int(lengths.sum()) <= total_range[1]:
            break
        attempt += 1
    segs, off = [], 0
    for n in lengths.tolist():
        segs.append((off, int(n)))
        off += (int(n) + pad - 1) // pad * pad
    return segs, padded_ld(off, pad), attempt


class Run:
    """Random stream of one configuration on one device."""

    def __init__(self, cfg: Config, device, P: Optional[int] = None, ld: Optional[int] = None):
        self.cfg = cfg
        self.device = torch.device(device)
        self.P = cfg.P if P is None else P
        self.ld = self.P if ld is None else ld
        self.gen = torch.Generator(device=self.device)
        self.gen.manual_seed(cfg.seed)
        self.scale = None

    def init_params(self, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        """``X[W, ld]`` fp32, all rows equal to one ``N(0, 0.02^2)`` vector (written into ``out`` if given)."""
        x0 = torch.empty(self.ld, dtype=torch.float32, device=self.device)
        x0.normal_(0.0, 0.02, generator=self.gen)
        if out is not None:
            X = out
            X.copy_(x0.unsqueeze(0).expand(self.cfg.W, self.ld))
        else:
            X = x0.unsqueeze(0).repeat(self.cfg.W, 1).contiguous()
        if self.cfg.worker_scale:
            self.scale = torch.empty(self.cfg.W, 1, dtype=torch.float32, device=self.device)
            self.scale.uniform_(0.5, 2.0, generator=self.gen)
        return X

    def gradients(self, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        """Gradient stack of the next iteration, ``[W, ld]`` fp32 or bf16."""
        W = self.cfg.W
        mu = torch.empty(self.ld, dtype=torch.float32, device=self.device)
        mu.normal_(generator=self.gen)
        if out is not None and out.dtype == torch.float32:
            G = out
        else:
            G = torch.empty(W, self.ld, dtype=torch.float32, device=self.device)
        G.normal_(generator=self.gen)
        G.mul_(0.5).add_(mu)
        if self.scale is not None:
            G.mul_(self.scale)
        if self.cfg.bf16_grads:
            if out is not None and out.dtype == torch.bfloat16:
                out.copy_(G)
                return out
            return G.to(torch.bfloat16)
        return G


TILE = 256      # columns per tile of the tiled layout


def to_tiled(stack: torch.Tensor, P: int, tile_stride: Optional[int] = None) -> torch.Tensor:
    """Copy of the first P columns of a row-major ``[W, ld]`` stack in the tiled layout: element
    (i, p) at ``(p // 256) * tile_stride + i * 256 + p % 256`` of a flat tensor (``tile_stride``
    defaults to ``W * 256``).  Slots that stand for no column (beyond P in the last block, between
    blocks) are filled with a recognisable constant.  Layout only: no arithmetic of the method."""
    W = stack.shape[0]
    n_tiles = (P + TILE - 1) // TILE
    ts = W * TILE if tile_stride is None else tile_stride
    padded = torch.full((W, n_tiles * TILE), 7.0, dtype=stack.dtype, device=stack.device)
    padded[:, :P] = stack[:, :P]
    out = torch.full((max(n_tiles, 1) * ts,), 7.0, dtype=stack.dtype, device=stack.device)
    out[:n_tiles * ts].view(n_tiles, ts)[:, :W * TILE] = padded.view(W, n_tiles, TILE).permute(1, 0, 2).reshape(n_tiles, W * TILE)
    return out


def from_tiled(tiled: torch.Tensor, P: int, W: int, tile_stride: Optional[int] = None) -> torch.Tensor:
    """Row-major ``[W, n_tiles * 256]`` copy of a tiled stack (columns beyond P are its unused slots)."""
    n_tiles = (P + TILE - 1) // TILE
    ts = W * TILE if tile_stride is None else tile_stride
    blocks = tiled[:n_tiles * ts].view(n_tiles, ts)[:, :W * TILE].reshape(n_tiles, W, TILE)
    return blocks.permute(1, 0, 2).reshape(W, n_tiles * TILE).contiguous()


def tensor_to_numpy(t: torch.Tensor) -> np.ndarray:
    """Host copy of a tensor; bf16 comes back as its raw uint16 bit patterns."""
    t = t.detach()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()
