"""Seeded synthetic rank buffers.  Serves the tests, the benchmark and the oracle's callers alike.

This module holds none of the method's arithmetic: it only makes input bits.
Every value is a pure function of (seed, rank, element index), so any slice
of any rank's buffer can be regenerated on its own and slab-wise generation
gives the same bits as generating the whole buffer at once (for the integer
derived distributions exactly; `normal` goes through libm's log/cos, so a
caller that needs both sides of a comparison to see identical bits generates
once and hands the same array to both).

Distributions
  u32       uniform 32-bit integers (as int32)
  uniform   fp32 in [-1, 1): (u24 / 2^23) - 1, exact in binary32
  smallint  integers in [-8, 8] (every partial sum of up to 2^10 of them is exact in fp16 and fp32)
  normal    N(0, 1) by Box-Muller in double, rounded once to the target dtype
  wide      `uniform` scaled by an exact power of two, 2^-12 .. 2^12 (2^-14 .. 2^10 for fp16, whose sums are taken in
            binary32 and round only when operands are 14 or more binades apart): neighbouring elements differ by many
            binades, so many sums round and a sum taken in another order has other bits
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from typing import Optional

import numpy as np

_GOLD = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)

POISON_U32 = 0x7FC0DEAD      # a quiet NaN as fp32, a large positive int32
POISON_U16 = 0x7E5A          # a quiet NaN as fp16


def _mix(x: np.ndarray) -> np.ndarray:
    """64-bit finalising mix (the splitmix64 output function)."""
    with np.errstate(over="ignore"):
        x = (x ^ (x >> np.uint64(30))) * _M1
        x = (x ^ (x >> np.uint64(27))) * _M2
        return x ^ (x >> np.uint64(31))


def raw64(seed: int, rank: int, start: int, count: int, stream: int = 0) -> np.ndarray:
    """count 64-bit words for elements start .. start+count-1 of `rank`'s buffer."""
    with np.errstate(over="ignore"):
        key = _mix(np.array([(seed * 0x1000003 + rank * 0x10001 + stream * 0x101 + 1) & 0xFFFFFFFFFFFFFFFF],
                            dtype=np.uint64))[0]
        idx = np.arange(start, start + count, dtype=np.uint64)
        return _mix(idx * _GOLD + key)


def generate(dist: str, dtype: str, seed: int, rank: int, start: int, count: int) -> np.ndarray:
    """Elements start .. start+count-1 of rank's buffer, as a numpy array of the target dtype."""
    npdt = {"i32": np.int32, "f32": np.float32, "f16": np.float16}[dtype]
    r = raw64(seed, rank, start, count)
    if dist == "u32":
        v = (r >> np.uint64(32)).astype(np.uint32).view(np.int32)
        if dtype != "i32":
            raise ValueError("u32 is an integer distribution")
        return v
    if dist == "uniform":
        u24 = (r >> np.uint64(40)).astype(np.float32)
        v = u24 * np.float32(2.0 ** -23) - np.float32(1.0)
        return v.astype(npdt)
    if dist == "smallint":
        v = ((r >> np.uint64(40)) % np.uint64(17)).astype(np.int64) - 8
        return v.astype(npdt)
    if dist == "wide":
        if dtype == "i32":
            raise ValueError("wide is a floating distribution")
        u24 = (r >> np.uint64(40)).astype(np.float32)
        if dtype == "f32":
            e = ((r >> np.uint64(8)) % np.uint64(25)).astype(np.int32) - 12
        else:
            e = ((r >> np.uint64(8)) % np.uint64(25)).astype(np.int32) - 14
        return np.ldexp(u24 * np.float32(2.0 ** -23) - np.float32(1.0), e).astype(npdt)
    if dist == "normal":
        r2 = raw64(seed, rank, start, count, stream=1)
        u1 = ((r >> np.uint64(11)).astype(np.float64) + 1.0) * (2.0 ** -53)      # (0, 1]
        u2 = (r2 >> np.uint64(11)).astype(np.float64) * (2.0 ** -53)             # [0, 1)
        z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
        if dtype == "i32":
            raise ValueError("normal is a floating distribution")
        return z.astype(npdt)
    raise ValueError(f"unknown distribution {dist}")


def rank_buffer(dist: str, dtype: str, seed: int, rank: int, num_elems: int,
                threads: int = 8, slab: int = 1 << 22) -> np.ndarray:
    """A whole rank buffer, generated slab by slab on a few threads (numpy releases the GIL)."""
    npdt = {"i32": np.int32, "f32": np.float32, "f16": np.float16}[dtype]
    out = np.empty(num_elems, dtype=npdt)
    starts = list(range(0, num_elems, slab))

    def fill(s):
        n = min(slab, num_elems - s)
        out[s:s + n] = generate(dist, dtype, seed, rank, s, n)

    if len(starts) <= 1 or threads <= 1:
        for s in starts:
            fill(s)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, starts))
    return out


def poison(buf: np.ndarray, lo: int, hi: int) -> None:
    """Overwrite elements lo..hi-1 with a recognisable pattern (regions the collective must never read)."""
    if buf.dtype.itemsize == 4:
        buf.view(np.uint32)[lo:hi] = POISON_U32
    else:
        buf.view(np.uint16)[lo:hi] = POISON_U16


def is_poison(buf: np.ndarray) -> np.ndarray:
    if buf.dtype.itemsize == 4:
        return buf.view(np.uint32) == POISON_U32
    return buf.view(np.uint16) == POISON_U16


# ---- the same integer-derived bits made on the device with torch (bench and full-size tests) ----

def torch_generate(dist: str, dtype: str, seed: int, rank: int, start: int, count: int, device):
    """Bit-identical to generate() for u32 / uniform / smallint, computed with torch integer ops on `device`."""
    import torch

    def lsr(x, k):      # logical shift right on int64
        return (x >> k) & ((1 << (64 - k)) - 1)

    def s64(v):         # python int -> two's complement int64 value
        v &= 0xFFFFFFFFFFFFFFFF
        return v - (1 << 64) if v >= (1 << 63) else v

    def mix(x):
        x = (x ^ lsr(x, 30)) * s64(int(_M1))
        x = (x ^ lsr(x, 27)) * s64(int(_M2))
        return x ^ lsr(x, 31)

    key = int(_mix(np.array([(seed * 0x1000003 + rank * 0x10001 + 1) & 0xFFFFFFFFFFFFFFFF], dtype=np.uint64))[0])
    idx = torch.arange(start, start + count, dtype=torch.int64, device=device)
    r = mix(idx * s64(int(_GOLD)) + s64(key))
    tdt = {"i32": torch.int32, "f32": torch.float32, "f16": torch.float16}[dtype]
    if dist == "u32":
        v = lsr(r, 32)                          # 0 .. 2^32-1 in int64
        v = torch.where(v >= (1 << 31), v - (1 << 32), v)
        return v.to(torch.int32)
    if dist == "uniform":
        u24 = lsr(r, 40).to(torch.float32)
        return (u24 * (2.0 ** -23) - 1.0).to(tdt)
    if dist == "smallint":
        return (lsr(r, 40) % 17 - 8).to(tdt)
    if dist == "normal":
        # same recipe as generate(); log/cos come from the device's libm, so the last bit of the
        # double may differ from numpy's: a caller that compares against host code reads these back
        key2 = int(_mix(np.array([(seed * 0x1000003 + rank * 0x10001 + 0x101 + 1) & 0xFFFFFFFFFFFFFFFF],
                                 dtype=np.uint64))[0])
        r2 = mix(idx * s64(int(_GOLD)) + s64(key2))
        u1 = (lsr(r, 11).to(torch.float64) + 1.0) * (2.0 ** -53)
        u2 = lsr(r2, 11).to(torch.float64) * (2.0 ** -53)
        z = torch.sqrt(-2.0 * torch.log(u1)) * torch.cos(2.0 * np.pi * u2)
        return z.to(tdt)
    raise ValueError(f"{dist} has no device generator")


def torch_rank_buffer(dist: str, dtype: str, seed: int, rank: int, num_elems: int, device, slab: int = 1 << 25):
    """A whole rank buffer on `device`, generated slab by slab to bound the temporaries."""
    import torch
    tdt = {"i32": torch.int32, "f32": torch.float32, "f16": torch.float16}[dtype]
    out = torch.empty(num_elems, dtype=tdt, device=device)
    for s in range(0, num_elems, slab):
        n = min(slab, num_elems - s)
        out[s:s + n] = torch_generate(dist, dtype, seed, rank, s, n, device)
    return out
