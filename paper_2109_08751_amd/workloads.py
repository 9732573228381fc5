"""Seeded synthetic Allgather workloads (numpy only).

This module holds input generation and nothing of the method: no schedule, no
slot arithmetic.  Both the CPU oracle's tests and the HIP path's tests and
benchmark take their payloads from here, so the two sides see identical bytes.

The five fixed configurations stand in for the paper's OSU `osu_allgather`
sweep (Section IV-A: block sizes on the 1 B .. 1 MiB times-two ladder, process
counts covering power-of-two, even and odd values up to a few hundred).
Allgather is oblivious to the values it moves; the distributions only make a
misplaced block detectable.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

DEFAULT_SEED = 210908751

_GAMMA = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def splitmix64(x: np.ndarray) -> np.ndarray:
    """First output of a SplitMix64 generator whose state starts at `x`
    (uint64 array): add the golden-ratio increment, two xor-shift-multiply
    rounds, final xor-shift (Steele, Lea, Flood 2014)."""
    with np.errstate(over="ignore"):
        z = x.astype(np.uint64) + _GAMMA
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        return z ^ (z >> np.uint64(31))


def _draws(seed: int, rank: int, n: int, start: int = 0) -> np.ndarray:
    """splitmix64(seed ^ (rank << 32 | j)) for j in [start, start + n)."""
    j = np.arange(start, start + n, dtype=np.uint64)
    key = (np.uint64(rank) << np.uint64(32)) | j
    return splitmix64(np.uint64(seed) ^ key)


def _unit(draws: np.ndarray) -> np.ndarray:
    """Top 24 bits as a float64 in [0, 1)."""
    return (draws >> np.uint64(40)).astype(np.float64) / float(1 << 24)


@dataclass(frozen=True)
class Workload:
    name: str
    p: int            # virtual ranks
    block_bytes: int  # bytes each rank contributes
    kind: str         # "u8" | "i32" | "f32_uniform" | "f32_normal"
    note: str

    @property
    def recv_bytes(self) -> int:
        return self.p * self.p * self.block_bytes

    @property
    def send_bytes(self) -> int:
        return self.p * self.block_bytes


WORKLOADS = {
    "cfg1": Workload("cfg1", 6, 1 << 10, "u8", "p=6 (non-power-of-two), 1 KiB uint8 blocks"),
    "cfg2": Workload("cfg2", 64, 64 << 10, "i32", "p=64, 64 KiB int32 blocks"),
    "cfg3": Workload("cfg3", 96, 4 << 10, "f32_uniform", "p=96, 4 KiB fp32 blocks in [-1,1)"),
    "cfg4": Workload("cfg4", 128, 1 << 20, "f32_normal", "p=128, 1 MiB fp32 N(0,1) blocks"),
    "cfg5": Workload("cfg5", 257, 256 << 10, "u8", "p=257, 256 KiB uint8 blocks"),
}


def make_block(kind: str, rank: int, block_bytes: int, seed: int = DEFAULT_SEED) -> np.ndarray:
    """One rank's block as raw bytes (uint8 array of block_bytes)."""
    if kind == "u8":
        return (_draws(seed, rank, block_bytes) & np.uint64(0xFF)).astype(np.uint8)
    if block_bytes % 4:
        raise ValueError("4-byte element kinds need block_bytes % 4 == 0")
    n = block_bytes // 4
    if kind == "i32":
        v = (_draws(seed, rank, n) & np.uint64(0xFFFFFFFF)).astype(np.uint32)
    elif kind == "f32_uniform":
        v = (2.0 * _unit(_draws(seed, rank, n)) - 1.0).astype(np.float32)
    elif kind == "f32_normal":
        # Box-Muller on two uniforms per value; u1 is shifted off zero.
        u1 = _unit(_draws(seed, rank, n)) + 1.0 / float(1 << 25)
        u2 = _unit(_draws(seed, rank, n, start=n))
        v = (np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)).astype(np.float32)
    else:
        raise ValueError(f"unknown payload kind {kind!r}")
    return v.view(np.uint8)


def make_send(w: Workload, seed: int = DEFAULT_SEED) -> np.ndarray:
    """All ranks' send blocks: uint8 array [p, block_bytes], rank r in row r."""
    out = np.empty((w.p, w.block_bytes), dtype=np.uint8)
    for r in range(w.p):
        out[r] = make_block(w.kind, r, w.block_bytes, seed)
    return out


def make_send_raw(p: int, block_bytes: int, seed: int = DEFAULT_SEED) -> np.ndarray:
    """uint8 payload for an arbitrary (p, block_bytes), e.g. odd block sizes."""
    return make_send(Workload("adhoc", p, block_bytes, "u8", ""), seed)


POISON = 0xA5
