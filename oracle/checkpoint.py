"""Oracle for the per-stage checkpoint file (Section 4, "Checkpointing": a stage dumps its own parameters, no
coordination with other stages).  Test infrastructure only (see package docstring).

The paper fixes no format; the one used here: 8 bytes ``PDCKPT1\\0``; u32 precision (0 fp32, 1 bf16 with fp32
master); u32 zero; u64 parameter count; i64 version id; u64 checksum; then the fp32 weights and the fp32 momentum in
the flat parameter layout, all little-endian.  The checksum folds each array 8 bytes at a time,
``h = ((h ^ word) * 0x100000001b3) mod 2**64`` starting from ``0xcbf29ce484222325`` (weights first, then momentum;
an odd last float of an array is zero-extended to 8 bytes).  Written out here in plain Python integers.
"""
from __future__ import annotations

import struct

import numpy as np

MAGIC = b"PDCKPT1\x00"
_MASK = (1 << 64) - 1


def checksum(weights: np.ndarray, momentum: np.ndarray) -> int:
    h = 0xCBF29CE484222325
    for arr in (weights, momentum):
        raw = np.ascontiguousarray(arr, dtype="<f4").tobytes()
        if len(raw) % 8:
            raw += b"\x00\x00\x00\x00"
        for (word,) in struct.iter_unpack("<Q", raw):
            h = ((h ^ word) * 0x100000001B3) & _MASK
    return h


def write(path: str, weights: np.ndarray, momentum: np.ndarray, version: int, precision: int) -> None:
    w = np.ascontiguousarray(weights, dtype="<f4")
    m = np.ascontiguousarray(momentum, dtype="<f4")
    assert w.shape == m.shape and w.ndim == 1
    with open(path, "wb") as f:
        f.write(MAGIC + struct.pack("<IIQqQ", precision, 0, w.size, version, checksum(w, m)))
        f.write(w.tobytes())
        f.write(m.tobytes())


def read(path: str):
    """(weights, momentum, version, precision); raises ValueError if the file does not verify."""
    raw = open(path, "rb").read()
    if len(raw) < 40 or raw[:8] != MAGIC:
        raise ValueError("no checkpoint header")
    precision, zero, n, version, chk = struct.unpack("<IIQqQ", raw[8:40])
    if zero != 0 or precision > 1 or version < 0 or len(raw) != 40 + 8 * n:
        raise ValueError("bad checkpoint header or size")
    w = np.frombuffer(raw, dtype="<f4", count=n, offset=40)
    m = np.frombuffer(raw, dtype="<f4", count=n, offset=40 + 4 * n)
    if checksum(w, m) != chk:
        raise ValueError("checksum mismatch")
    return w.copy(), m.copy(), version, precision
