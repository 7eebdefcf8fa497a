"""Reference encoders of the GPU library's own operand layouts (test infrastructure).

Not part of the paper's method and therefore not part of the oracle: these are the containers in which the library
keeps the INT4 codes of Sec. 5.2 in HBM -- the fp6 operand form read by the 6-bit floating-point matrix cores, and the
weight-streaming layout read by decode-sized calls -- written out as plain Python walks from the layouts'
definitions in include/basq.h, so that the repacking kernels can be checked bit by bit.  Pinned by
tests/test_layout_ref.py (format facts, hand-placed single codes, round trips).  Shares no code with the library.
"""
from __future__ import annotations

import functools

import numpy as np


# ------------------------------------------------------------------------------------------------
# The fp6 operand form of a code matrix.
#   e2m3 (OCP Microscaling FP6): 1 sign bit, 2 exponent bits (bias 1), 3 mantissa bits, no Inf/NaN;
#   value = (-1)^s * 2^(e-1) * (1 + m/8) for e > 0, (-1)^s * (m/8) for e = 0.
#   Code q is stored as the number q/8.
# ------------------------------------------------------------------------------------------------
def e2m3_value(code: int) -> float:
    """Value of a 6-bit e2m3 pattern, from the format definition."""
    s, e, m = (code >> 5) & 1, (code >> 3) & 3, code & 7
    mag = m / 8.0 if e == 0 else 2.0 ** (e - 1) * (1.0 + m / 8.0)
    return -mag if s else mag


@functools.lru_cache(maxsize=None)
def e2m3_code_table() -> tuple:
    """The e2m3 pattern whose value is q/8, for q = 0..15 (found by searching the 64 patterns; +0 for 0)."""
    table = []
    for q in range(16):
        hits = [c for c in range(64) if e2m3_value(c) == q / 8.0 and not (c >> 5)]
        assert len(hits) == 1, (q, hits)
        table.append(hits[0])
    return tuple(table)


def pack_fp6(q: np.ndarray) -> np.ndarray:
    """[R, K] 4-bit codes (one per byte), K % 128 == 0 -> the fp6 operand form, a flat uint8 array of
    ceil(R/32)*32 * 3K/4 bytes.  Blocks of 3072 bytes per (chunk c of 128 codes, block rb of 32 rows),
    block (c, rb) at (c*ceil(R/32) + rb)*3072.  Inside a block, row r and group f (codes 128c+32f ..+31)
    are a 24-byte little-endian string of 6-bit fields: its first 16 bytes at 64r + 16*(f ^ ((r>>2)&3)),
    its last 8 bytes at 2048 + 256f + 8r.  Bytes of rows past R are left zero."""
    assert q.dtype == np.uint8 and q.ndim == 2 and q.shape[1] % 128 == 0
    R, K = q.shape
    RB = (R + 31) // 32
    table = np.array(e2m3_code_table(), dtype=np.uint64)
    out = np.zeros(K // 128 * RB * 3072, dtype=np.uint8)
    fields = table[q].reshape(R, K // 32, 32)                      # 6-bit patterns, grouped by 32
    shifts = (np.arange(32, dtype=np.uint64) * np.uint64(6))
    for row in range(R):
        rb, r = divmod(row, 32)
        for g in range(K // 32):
            # the 192-bit string as a Python integer, then 24 little-endian bytes
            val = 0
            for e in range(32):
                val |= int(fields[row, g, e]) << int(shifts[e])
            b = np.frombuffer(val.to_bytes(24, "little"), dtype=np.uint8)
            c, f = divmod(g, 4)
            base = (c * RB + rb) * 3072
            m = base + 64 * r + 16 * (f ^ ((r >> 2) & 3))
            t = base + 2048 + 256 * f + 8 * r
            out[m:m + 16] = b[:16]
            out[t:t + 8] = b[16:]
    return out


def unpack_fp6(buf: np.ndarray, R: int, K: int) -> np.ndarray:
    """Values (float64, [R, K]) stored in an fp6 operand form buffer: the inverse walk of pack_fp6 followed
    by e2m3_value."""
    RB = (R + 31) // 32
    vals = np.array([e2m3_value(c) for c in range(64)])
    out = np.empty((R, K), dtype=np.float64)
    for row in range(R):
        rb, r = divmod(row, 32)
        for g in range(K // 32):
            c, f = divmod(g, 4)
            base = (c * RB + rb) * 3072
            m = base + 64 * r + 16 * (f ^ ((r >> 2) & 3))
            t = base + 2048 + 256 * f + 8 * r
            val = int.from_bytes(bytes(buf[m:m + 16]) + bytes(buf[t:t + 8]), "little")
            for e in range(32):
                out[row, 32 * g + e] = vals[(val >> (6 * e)) & 63]
    return out


def pack_decode16(p: np.ndarray) -> np.ndarray:
    """[N, K/2] canonical packed weight bytes, K % 128 == 0 -> the weight-streaming layout of the decode
    path, a flat uint8 array of ceil(N/16)*16 * K/2 bytes.  It is a pure permutation of 16-byte pieces:
    block nb (rows 16nb..16nb+15) at nb*16*K/2; chunk c (bytes 64c..64c+63 of every row) is the KB at
    c*1024 inside the block; piece (s, r) at (16s + r)*16 holds bytes 64c+16s .. +15 of row 16nb + r.
    Rows past N are zeros."""
    assert p.dtype == np.uint8 and p.ndim == 2 and p.shape[1] % 64 == 0
    N, KB = p.shape
    NB = (N + 15) // 16
    out = np.zeros(NB * 16 * KB, dtype=np.uint8)
    for n in range(N):
        nb, r = divmod(n, 16)
        for c in range(KB // 64):
            for s_ in range(4):
                dst = nb * 16 * KB + c * 1024 + (16 * s_ + r) * 16
                out[dst:dst + 16] = p[n, 64 * c + 16 * s_: 64 * c + 16 * s_ + 16]
    return out
