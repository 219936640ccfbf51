"""Counter-based random numbers for the synthetic inputs, written out twice with identical results: in NumPy (this
file, for tensors made on the host) and in HIP (csrc/synth_gen.hip, for tensors made on the GPU).

Philox-4x32-10 (the published counter-based generator) gives four 32-bit integers per counter block; a Box-Muller
transform turns them into four standard normals.  Its logarithm, sine and cosine are short polynomials evaluated in
double precision with additions, multiplications, one division and one square root only -- operations IEEE 754
rounds identically on every machine -- so that a tensor is a pure function of (seed, stream, shape), the same
bytes on a CPU and on a GPU.  No step of the pruning method lives here.

Element i of stream s with seed k comes from counter block i // 4 (counter words: block low, block high, s, 0;
key words: k low, k high), output i % 4.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

_M0, _M1 = np.uint64(0xD2511F53), np.uint64(0xCD9E8D57)
_W0, _W1 = 0x9E3779B9, 0xBB67AE85
_MASK32 = np.uint64(0xFFFFFFFF)
_U32 = np.uint64(32)


def philox4x32_10_words(c0, c1, c2, c3, k0: int, k1: int):
    """Philox-4x32 with ten rounds on counter words c0 .. c3 (arrays of 32-bit values held in uint64) and key
    words k0, k1: four arrays of 32-bit outputs."""
    c0, c1, c2, c3 = (np.asarray(c, dtype=np.uint64) for c in (c0, c1, c2, c3))
    for _ in range(10):
        p0, p1 = _M0 * c0, _M1 * c2                     # 32 x 32 -> 64 bit products, exact in uint64
        n0 = (p1 >> _U32) ^ c1 ^ np.uint64(k0)
        n1 = p1 & _MASK32
        n2 = (p0 >> _U32) ^ c3 ^ np.uint64(k1)
        n3 = p0 & _MASK32
        c0, c1, c2, c3 = n0, n1, n2, n3
        k0, k1 = (k0 + _W0) & 0xFFFFFFFF, (k1 + _W1) & 0xFFFFFFFF
    return c0, c1, c2, c3


def philox4x32_10(block: np.ndarray, stream: int, seed: int):
    """Four uint32-valued arrays: the outputs of the counter blocks `block` (uint64 array) of one stream."""
    block = np.asarray(block, dtype=np.uint64)
    return philox4x32_10_words(block & _MASK32, block >> _U32, np.full(block.shape, stream & 0xFFFFFFFF, dtype=np.uint64),
                               np.zeros(block.shape, dtype=np.uint64), seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)


def _ln_unit(x: np.ndarray) -> np.ndarray:
    """ln((x + 0.5) / 2^32) for 32-bit integers x (held in uint64), by the polynomial the device code uses."""
    u = (x.astype(np.float64) + 0.5) * (1.0 / 4294967296.0)
    bits = u.view(np.uint64)
    e = ((bits >> np.uint64(52)) & np.uint64(0x7FF)).astype(np.int64) - 1022
    m = ((bits & np.uint64(0x000FFFFFFFFFFFFF)) | np.uint64(0x3FE0000000000000)).view(np.float64)
    small = m < 0.70710678118654752440
    m = np.where(small, m * 2.0, m)
    e = np.where(small, e - 1, e)
    z = (m - 1.0) / (m + 1.0)
    z2 = z * z
    p = np.full(z.shape, 1.0 / 21.0)
    for d in (19.0, 17.0, 15.0, 13.0, 11.0, 9.0, 7.0, 5.0, 3.0):
        p = p * z2 + 1.0 / d
    p = p * z2 + 1.0
    return e.astype(np.float64) * 0.69314718055994530942 + 2.0 * z * p


_SIN = (-1.0 / 25852016738884976640000.0, 1.0 / 51090942171709440000.0, -1.0 / 121645100408832000.0,
        1.0 / 355687428096000.0, -1.0 / 1307674368000.0, 1.0 / 6227020800.0, -1.0 / 39916800.0, 1.0 / 362880.0,
        -1.0 / 5040.0, 1.0 / 120.0, -1.0 / 6.0)
_COS = (1.0 / 1124000727777607680000.0, -1.0 / 2432902008176640000.0, 1.0 / 6402373705728000.0,
        -1.0 / 20922789888000.0, 1.0 / 87178291200.0, -1.0 / 479001600.0, 1.0 / 3628800.0, -1.0 / 40320.0,
        1.0 / 720.0, -1.0 / 24.0)


def _cos_sin_turn(x: np.ndarray):
    """cos and sin of 2 pi x / 2^32 for 32-bit integers x: quadrant from the top two bits, Taylor polynomials."""
    a = (x & np.uint64(0x3FFFFFFF)).astype(np.float64) * (1.57079632679489661923 / 1073741824.0)
    a2 = a * a
    ps = np.full(a.shape, _SIN[0])
    for c in _SIN[1:]:
        ps = ps * a2 + c
    ps = ps * a2 + 1.0
    sn = a * ps
    pc = np.full(a.shape, _COS[0])
    for c in _COS[1:]:
        pc = pc * a2 + c
    pc = pc * a2 + 1.0 / 2.0
    cs = 1.0 - a2 * pc
    q = (x >> np.uint64(30)).astype(np.int64)
    c = np.select([q == 0, q == 1, q == 2], [cs, -sn, -cs], default=sn)
    s = np.select([q == 0, q == 1, q == 2], [sn, cs, -sn], default=-cs)
    return c, s


def _normals_of_blocks(blocks: np.ndarray, stream: int, seed: int) -> np.ndarray:
    """[len(blocks), 4] standard normals (float64) of the given counter blocks."""
    x, y, z, w = philox4x32_10(blocks, stream, seed)
    r1 = np.sqrt(-2.0 * _ln_unit(x))
    c1, s1 = _cos_sin_turn(y)
    r2 = np.sqrt(-2.0 * _ln_unit(z))
    c2, s2 = _cos_sin_turn(w)
    return np.stack([r1 * c1, r1 * s1, r2 * c2, r2 * s2], axis=1)


def normals(n: int, stream: int, seed: int, first: int = 0) -> np.ndarray:
    """Standard normals (float64) number first .. first + n - 1 of a stream."""
    b0, b1 = first // 4, (first + n + 3) // 4
    out = _normals_of_blocks(np.arange(b0, b1, dtype=np.uint64), stream, seed).reshape(-1)
    return out[first - 4 * b0: first - 4 * b0 + n]


def normals_at(index: np.ndarray, stream: int, seed: int) -> np.ndarray:
    """The standard normals of a stream at the given element numbers (any shape)."""
    index = np.asarray(index, dtype=np.uint64)
    four = _normals_of_blocks((index >> np.uint64(2)).reshape(-1), stream, seed)
    lane = (index & np.uint64(3)).reshape(-1).astype(np.int64)
    return np.take_along_axis(four, lane[:, None], axis=1).reshape(index.shape)


def bits32(n: int, stream: int, seed: int) -> np.ndarray:
    """The first n 32-bit outputs (uint32) of a stream."""
    blocks = np.arange((n + 3) // 4, dtype=np.uint64)
    out = np.stack(philox4x32_10(blocks, stream, seed), axis=1).reshape(-1)
    return out[:n].astype(np.uint32)


def to_bf16_bits(f32: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns, round to nearest, ties to even (finite values)."""
    b = np.ascontiguousarray(f32, dtype=np.float32).view(np.uint32)
    return ((b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)).astype(np.uint16)


def fill_normal_host(rows: int, cols: int, seed: int, stream: int, scale: float = 1.0,
                     col_scale: Optional[np.ndarray] = None, kind: Optional[np.ndarray] = None,
                     first_row: int = 0) -> np.ndarray:
    """float32 rows first_row .. first_row + rows - 1 of a matrix with `cols` columns: element (r, c) =
    value(r * cols + c) * scale * col_scale[c], where value(i) is normal number i of `stream`, or, in the columns
    with kind[c] != 0, a Student-t draw with three degrees of freedom z0 / sqrt((z1^2 + z2^2 + z3^2) / 3) whose
    four normals are number i of streams stream .. stream + 3."""
    z = normals(rows * cols, stream, seed, first=first_row * cols).reshape(rows, cols)
    if kind is not None and np.any(kind):
        cols_t = np.nonzero(kind)[0].astype(np.uint64)
        at = (np.arange(first_row, first_row + rows, dtype=np.uint64) * np.uint64(cols))[:, None] + cols_t[None, :]
        z1, z2, z3 = (normals_at(at, stream + j, seed) for j in (1, 2, 3))
        z[:, cols_t.astype(np.int64)] = z[:, cols_t.astype(np.int64)] / np.sqrt((z1 * z1 + z2 * z2 + z3 * z3) / 3.0)
    v = z * scale
    if col_scale is not None:
        v = v * np.asarray(col_scale, dtype=np.float32).astype(np.float64)[None, :]
    return v.astype(np.float32)


# ---------------------------------------------------------------------------------------------------------------
# the device twin (csrc/synth_gen.hip, built into libmosaic_synth.so next to the pruning library)

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "csrc", "libmosaic_synth.so")
_lib = None


def device_lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(f"{_LIB_PATH} is missing: run `python -m paper_2504_06323_amd.build` first")
        lib = ctypes.CDLL(_LIB_PATH)
        vp, i64, u64, u32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_uint64, ctypes.c_uint32
        lib.synth_fill_normal.restype = ctypes.c_int
        lib.synth_fill_normal.argtypes = [vp, ctypes.c_int, i64, i64, i64, u64, u32, vp, vp, ctypes.c_double, vp]
        lib.synth_fill_bits.restype = ctypes.c_int
        lib.synth_fill_bits.argtypes = [vp, i64, u64, u32, vp]
        _lib = lib
    return _lib
