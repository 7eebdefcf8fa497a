"""CPU oracle for the W4A4 rotated linear layer of BASE-Q.

TEST INFRASTRUCTURE ONLY.  A plain, slow implementation of what the GPU library computes,
written from the paper; the GPU sources and this package share no code and neither imports the
other.  Only the tests, the smoke check and the benchmark's CPU-baseline leg may call it.

What is computed (row-vector convention: the paper's y = Q_w(WR) Q_a(R^-1 x - b^c) + (W R b^c + b),
Sec. 4 Eq. 14, with orthogonal R becomes Y = Q_a(X R - b^c) . Q_w(W')^T + c, W' = W R):

  rotate            r = (X H_n) / sqrt(n)                 dense definition, fp64 -> fp32   (Sec. 3.1)
  quantize_tokens   Eq. 4 with per-token range, clip      fixed fp32 op order (C file)     (Eq. 4, Sec. 5)
  quantize_weights  per-output-channel asymmetric INT4    fp32 ops                         (Sec. 5, see note)
  int_gemm          ACC = Qa . Qw^T                       int32 triple loop (C file)       (Sec. 5.2)
  dequant           scales, zero-point term, bias         fp64 -> bf16                     (Eq. 14, Fig. 6)

Pinned by tests/test_oracle_*.py against facts the paper and the mathematics fix.  Readings of
points the paper leaves open that no such fact can pin ("parity unpinned"): how the clip ratio
enters (lo = clip_lo*min, hi = clip_hi*max); that the fused bias c is built from the dequantised
weights; that the asymmetric scale s^a is one value per channel.

Note on weights: the paper deploys per-channel symmetric weights; the workload definition this
build follows asks for per-channel asymmetric INT4 (bf16 scale and zero-point).  Symmetric is
the special case zero-point = 8.
"""
from __future__ import annotations

import ctypes
import functools
import os
import subprocess
from typing import NamedTuple, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libbasq_oracle.so")
_SRC_PATH = os.path.join(_HERE, "basq_oracle_kernels.c")


# ------------------------------------------------------------------------------------------------
# build / load of the C part
# ------------------------------------------------------------------------------------------------

def build(force: bool = False) -> str:
    """Compile the C file of the oracle with gcc (no FMA contraction, OpenMP over rows)."""
    if (not force and os.path.exists(_LIB_PATH)
            and os.path.getmtime(_LIB_PATH) >= os.path.getmtime(_SRC_PATH)):
        return _LIB_PATH
    cmd = ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-std=c11",
           "-o", _LIB_PATH, _SRC_PATH, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB_PATH


@functools.lru_cache(maxsize=1)
def _lib() -> ctypes.CDLL:
    build()
    lib = ctypes.CDLL(_LIB_PATH)
    c = ctypes
    lib.orc_quantize_tokens.restype = c.c_int
    lib.orc_quantize_tokens.argtypes = [c.c_void_p, c.c_int64, c.c_int64, c.c_int64, c.c_void_p, c.c_void_p,
                                        c.c_float, c.c_float, c.c_int, c.c_void_p, c.c_void_p, c.c_void_p,
                                        c.c_void_p]
    lib.orc_int_gemm.restype = c.c_int
    lib.orc_int_gemm.argtypes = [c.c_void_p, c.c_void_p, c.c_int64, c.c_int64, c.c_int64, c.c_void_p]
    lib.orc_num_threads.restype = c.c_int
    return lib


def num_threads() -> int:
    """Threads the C loops run on."""
    return int(_lib().orc_num_threads())


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


# ------------------------------------------------------------------------------------------------
# storage formats
# ------------------------------------------------------------------------------------------------

def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> the fp32 values they denote (exact)."""
    assert bits.dtype == np.uint16
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def f64_to_bf16(y: np.ndarray) -> np.ndarray:
    """Round fp64 (or fp32) values to bf16 with round-half-to-even in ONE rounding; returns uint16 bits.

    Going through fp32 would round twice.  The fp32 value nearest to y is taken first; when that
    lands exactly on a bf16 tie although y itself was not on it, the fp32 value is moved one ulp
    back toward y so the second rounding sees which side y is on.
    """
    y = np.asarray(y, dtype=np.float64)
    f = y.astype(np.float32)
    bits = f.view(np.uint32).copy()
    finite = np.isfinite(f)
    on_tie = (bits & np.uint32(0xFFFF)) == np.uint32(0x8000)
    err = np.where(finite, y - f.astype(np.float64), 0.0)       # exact: both are fp64-representable
    away = (np.abs(y) > np.abs(f.astype(np.float64)))            # y lies farther from zero than f
    fix = finite & on_tie & (err != 0.0)
    bits = np.where(fix & away, bits + np.uint32(1), bits)
    bits = np.where(fix & ~away, bits - np.uint32(1), bits)
    # round-half-to-even on the low 16 bits
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = (bits + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    nan = np.isnan(f)
    out = np.where(nan, np.uint32(0x7FC0), rounded).astype(np.uint16)
    return out


def pack_codes(q: np.ndarray) -> np.ndarray:
    """[R, K] 4-bit codes (one per byte) -> [R, K/2] bytes; low nibble = even k, high nibble = odd k."""
    assert q.dtype == np.uint8 and q.shape[-1] % 2 == 0
    return (q[..., 0::2] | (q[..., 1::2] << np.uint8(4))).astype(np.uint8)


def unpack_codes(p: np.ndarray) -> np.ndarray:
    """Inverse of pack_codes."""
    assert p.dtype == np.uint8
    out = np.empty(p.shape[:-1] + (p.shape[-1] * 2,), dtype=np.uint8)
    out[..., 0::2] = p & np.uint8(0x0F)
    out[..., 1::2] = p >> np.uint8(4)
    return out


# ------------------------------------------------------------------------------------------------
# Hadamard matrices (Sec. 3.1: orthogonal Hadamard rotation, entries +-n^(-1/2))
# ------------------------------------------------------------------------------------------------

def hadamard_sylvester(n: int) -> np.ndarray:
    """Sylvester matrix by its recursion H_1 = [1], H_2n = [[H, H], [H, -H]]; int8 entries +-1."""
    assert n >= 1 and (n & (n - 1)) == 0, "n must be a power of two"
    H = np.ones((1, 1), dtype=np.int8)
    while H.shape[0] < n:
        H = np.block([[H, H], [H, -H]])
    return H


# GF(27) = GF(3)[t] / (t^3 + 2t + 1); element a0 + a1 t + a2 t^2 has index a0 + 3 a1 + 9 a2.
def _gf27_digits(e: int):
    return (e % 3, (e // 3) % 3, e // 9)


def _gf27_index(a0: int, a1: int, a2: int) -> int:
    return (a0 % 3) + 3 * (a1 % 3) + 9 * (a2 % 3)


def _gf27_sub(x: int, y: int) -> int:
    a, b = _gf27_digits(x), _gf27_digits(y)
    return _gf27_index(a[0] - b[0], a[1] - b[1], a[2] - b[2])


def _gf27_mul(x: int, y: int) -> int:
    a, b = _gf27_digits(x), _gf27_digits(y)
    p = [0] * 5                                   # plain polynomial product, degree <= 4
    for i in range(3):
        for j in range(3):
            p[i + j] += a[i] * b[j]
    # reduce with t^3 = -2t - 1 = t + 2 (mod 3), highest degree first
    for d in (4, 3):
        c = p[d]
        p[d] = 0
        p[d - 2] += c          # c * t^(d-3) * t
        p[d - 3] += 2 * c      # c * t^(d-3) * 2
    return _gf27_index(p[0], p[1], p[2])


def gf27_squares() -> frozenset:
    """The non-zero squares of GF(27) (there are (27-1)/2 = 13)."""
    return frozenset(_gf27_mul(e, e) for e in range(1, 27))


def hadamard_paley28() -> np.ndarray:
    """Paley type-I Hadamard matrix of order 28 = 27 + 1 (27 = 3 mod 4).

    With chi the quadratic character of GF(27) and Q[a][b] = chi(a - b) (skew-symmetric),
    H = I + S,  S = [[0, 1^T], [-1, Q]].  Not symmetric, so the side it multiplies on matters.
    """
    sq = gf27_squares()

    def chi(e: int) -> int:
        return 0 if e == 0 else (1 if e in sq else -1)

    H = np.zeros((28, 28), dtype=np.int8)
    H[0, :] = 1
    H[1:, 0] = -1
    H[0, 0] = 1
    for i in range(1, 28):
        for j in range(1, 28):
            H[i, j] = chi(_gf27_sub(i - 1, j - 1)) + (1 if i == j else 0)
    return H


@functools.lru_cache(maxsize=4)
def hadamard_matrix(n: int) -> np.ndarray:
    """Unnormalised +-1 rotation matrix of size n: Sylvester for n = 2^t, H_28 (x) H_(n/28) for
    n = 28 * 2^t with channel index k = i * (n/28) + j, i the H_28 index (Kronecker product)."""
    if n & (n - 1) == 0:
        return hadamard_sylvester(n)
    assert n % 28 == 0 and ((n // 28) & (n // 28 - 1)) == 0, "n must be 2^t or 28 * 2^t"
    return np.kron(hadamard_paley28(), hadamard_sylvester(n // 28)).astype(np.int8)


def rotate_f64(x: np.ndarray, rot_size: int) -> np.ndarray:
    """x . (H_n / sqrt(n)) on each block of n = rot_size consecutive channels, kept in fp64.

    x: [M, K] real values (the bf16 activations widened exactly).  The product with the dense +-1
    matrix is taken in fp64 (for bf16 inputs of ordinary dynamic range every partial sum is exact)
    and scaled by 1/sqrt(n) in fp64.
    """
    x = np.asarray(x, dtype=np.float64)
    M, K = x.shape
    n = int(rot_size)
    assert K % n == 0
    H = hadamard_matrix(n).astype(np.float64)
    u = x.reshape(M * (K // n), n) @ H
    return (u * (1.0 / np.sqrt(np.float64(n)))).reshape(M, K)


def rotate(x: np.ndarray, rot_size: int) -> np.ndarray:
    """r = fp32(x . (H_n / sqrt(n))): rotate_f64 rounded once to fp32 -- the activations the
    quantiser sees."""
    return rotate_f64(x, rot_size).astype(np.float32)


def channel_bias(x_calib: np.ndarray, rot_size: int) -> np.ndarray:
    """b^c: the per-channel mean of the rotated calibration activations (Sec. 3.2: the variance of
    channel means is what the bias removes).  By linearity the mean is taken first, in fp64, and
    rotated once; fp32 result."""
    mean = np.asarray(x_calib, dtype=np.float64).mean(axis=0, keepdims=True)
    return rotate(mean, rot_size)[0]


# ------------------------------------------------------------------------------------------------
# activation quantiser (Eq. 4; per-token asymmetric dynamic, Sec. 5 "Deployment Details")
# ------------------------------------------------------------------------------------------------

class TokenQuant(NamedTuple):
    codes: np.ndarray    # uint8 [M, K], values 0 .. 2^bits-1
    scale: np.ndarray    # fp32 [M, K/G]  step s
    lo: np.ndarray       # fp32 [M, K/G]  lower bound z
    rowsum: np.ndarray   # int32 [M, K/G] sum of codes


def quantize_tokens(r: np.ndarray, bias: Optional[np.ndarray], act_scale: Optional[np.ndarray],
                    clip_lo: float, clip_hi: float, bits: int = 4, group_size: int = 0) -> TokenQuant:
    """Steps of the C routine orc_quantize_tokens (see its header for the exact fp32 sequence)."""
    r = np.ascontiguousarray(r, dtype=np.float32)
    M, K = r.shape
    G = K if group_size in (0, None) else int(group_size)
    b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float32)
    s = None if act_scale is None else np.ascontiguousarray(act_scale, dtype=np.float32)
    assert b is None or b.shape == (K,)
    assert s is None or s.shape == (K,)
    codes = np.empty((M, K), dtype=np.uint8)
    scale = np.empty((M, K // G), dtype=np.float32)
    lo = np.empty((M, K // G), dtype=np.float32)
    rowsum = np.empty((M, K // G), dtype=np.int32)
    rc = _lib().orc_quantize_tokens(_ptr(r), M, K, G, _ptr(b), _ptr(s), clip_lo, clip_hi, bits,
                                    _ptr(codes), _ptr(scale), _ptr(lo), _ptr(rowsum))
    if rc != 0:
        raise ValueError("orc_quantize_tokens: bad argument")
    return TokenQuant(codes, scale, lo, rowsum)


def dequantize_tokens(tq: TokenQuant) -> np.ndarray:
    """x_hat = q * s + z (Eq. 4), fp64; [M, K]."""
    M, K = tq.codes.shape
    G = K // tq.scale.shape[1]
    s = np.repeat(tq.scale.astype(np.float64), G, axis=1)
    z = np.repeat(tq.lo.astype(np.float64), G, axis=1)
    return tq.codes.astype(np.float64) * s + z


# ------------------------------------------------------------------------------------------------
# weight quantiser (offline; per output channel, asymmetric INT4, clip 1.0)
# ------------------------------------------------------------------------------------------------

class WeightQuant(NamedTuple):
    codes: np.ndarray     # uint8 [N, K]
    scale_bits: np.ndarray  # uint16 [N]  bf16 step sw
    zero_bits: np.ndarray   # uint16 [N]  bf16 zero-point zp (integer valued, code units)
    colsum: np.ndarray    # int32 [N]   sum_k codes
    wsum: np.ndarray      # fp32 [N]    sw * (colsum - K * zp) = sum_k W_hat[n, k]

    @property
    def scale(self) -> np.ndarray:
        return bf16_to_f32(self.scale_bits)

    @property
    def zero(self) -> np.ndarray:
        return bf16_to_f32(self.zero_bits)


def quantize_weights(w_rot: np.ndarray, bits: int = 4) -> WeightQuant:
    """Round-to-nearest quantisation of rotated-basis weights W'[N, K], one (sw, zp) per row:

        lo, hi = min_k W', max_k W';  sw = bf16((hi - lo) / L)  (1 if not positive finite)
        zp = clamp(rne(-lo / sw), 0, L);  q = clamp(rne(W' / sw) + zp, 0, L);  W_hat = sw * (q - zp)

    every operation a single fp32 operation; sw is rounded to bf16 before it is used.
    """
    w = np.ascontiguousarray(w_rot, dtype=np.float32)
    N, K = w.shape
    L = np.float32((1 << bits) - 1)
    lo = w.min(axis=1)
    hi = w.max(axis=1)
    with np.errstate(all="ignore"):
        sw32 = (hi - lo) / L
        sw32 = np.where((sw32 > 0) & np.isfinite(sw32), sw32, np.float32(1.0)).astype(np.float32)
        sw_bits = f64_to_bf16(sw32)
        sw = bf16_to_f32(sw_bits)
        zp = np.clip(np.rint(-lo / sw), np.float32(0), L).astype(np.float32)
        q = np.clip(np.rint(w / sw[:, None]) + zp[:, None], np.float32(0), L)
    codes = q.astype(np.uint8)
    colsum = codes.astype(np.int64).sum(axis=1).astype(np.int32)
    wsum = (sw.astype(np.float64) * (colsum.astype(np.float64) - K * zp.astype(np.float64))).astype(np.float32)
    return WeightQuant(codes, sw_bits, f64_to_bf16(zp), colsum, wsum)


def dequantize_weights(wq: WeightQuant) -> np.ndarray:
    """W_hat = sw * (q - zp), fp64 [N, K]."""
    return wq.scale.astype(np.float64)[:, None] * (wq.codes.astype(np.float64) - wq.zero.astype(np.float64)[:, None])


def fused_bias(wq: WeightQuant, bias: Optional[np.ndarray], layer_bias: Optional[np.ndarray]) -> np.ndarray:
    """c = W_hat . b^c + b  (the "fused bias" of Eq. 14, built from the dequantised weights); fp32 [N]."""
    N = wq.codes.shape[0]
    c = np.zeros(N, dtype=np.float64)
    if bias is not None:
        c += dequantize_weights(wq) @ np.asarray(bias, dtype=np.float64)
    if layer_bias is not None:
        c += np.asarray(layer_bias, dtype=np.float64)
    return c.astype(np.float32)


# ------------------------------------------------------------------------------------------------
# integer GEMM and de-quantisation
# ------------------------------------------------------------------------------------------------

def int_gemm(qa: np.ndarray, qw: np.ndarray) -> np.ndarray:
    """ACC[m, n] = sum_k qa[m, k] * qw[n, k] -- int32 triple loop (C file)."""
    qa = np.ascontiguousarray(qa, dtype=np.uint8)
    qw = np.ascontiguousarray(qw, dtype=np.uint8)
    M, K = qa.shape
    N, K2 = qw.shape
    assert K == K2
    acc = np.empty((M, N), dtype=np.int32)
    if _lib().orc_int_gemm(_ptr(qa), _ptr(qw), M, N, K, _ptr(acc)) != 0:
        raise ValueError("orc_int_gemm: bad argument")
    return acc


def int_gemm_blas(qa: np.ndarray, qw: np.ndarray) -> np.ndarray:
    """The same product through the fp64 library matmul: operands are integers <= 255 and every
    partial sum stays below 2^53, so no rounding can occur whatever the summation order.  Used
    where the triple loop would take minutes; the tests pin it to int_gemm."""
    acc = qa.astype(np.float64) @ qw.astype(np.float64).T
    return acc.astype(np.int64).astype(np.int32)


def dequant(acc: np.ndarray, tq: TokenQuant, wq: WeightQuant, c: Optional[np.ndarray]) -> np.ndarray:
    """Y[m, n] = s_m sw_n (ACC - zp_n rowsum_m) + lo_m wsum_n + c_n   in fp64 (per-token quantisation).

    This is sum_k x_hat[m, k] W_hat[n, k] + c_n with x_hat = s q_a + lo and W_hat = sw (q_w - zp):
    the zero-point term uses the row sums of the activation codes, the lower-bound term the row
    sums of the dequantised weights (Fig. 6: de-quantisation with the bias folded in).
    """
    assert tq.scale.shape[1] == 1, "per-token quantisation only"
    s = tq.scale[:, 0].astype(np.float64)[:, None]
    lo = tq.lo[:, 0].astype(np.float64)[:, None]
    rs = tq.rowsum[:, 0].astype(np.float64)[:, None]
    sw = wq.scale.astype(np.float64)[None, :]
    zp = wq.zero.astype(np.float64)[None, :]
    y = s * sw * (acc.astype(np.float64) - zp * rs) + lo * wq.wsum.astype(np.float64)[None, :]
    if c is not None:
        y = y + np.asarray(c, dtype=np.float64)[None, :]
    return y


class LinearResult(NamedTuple):
    r: np.ndarray          # fp32 [M, K] rotated activations
    tq: TokenQuant
    acc: np.ndarray        # int32 [M, N]
    y: np.ndarray          # fp64 [M, N]
    y_bf16: np.ndarray     # uint16 [M, N]


def linear(x: np.ndarray, rot_size: int, bias: Optional[np.ndarray], act_scale: Optional[np.ndarray],
           clip_lo: float, clip_hi: float, wq: WeightQuant, c: Optional[np.ndarray],
           *, r: Optional[np.ndarray] = None, use_blas_gemm: bool = False) -> LinearResult:
    """The whole layer.  ``r`` given: skip the rotation and start from these rotated activations
    (used to check codes and accumulators bit for bit on the GPU's own rotation output)."""
    if r is None:
        r = rotate(x, rot_size)
    tq = quantize_tokens(r, bias, act_scale, clip_lo, clip_hi)
    acc = (int_gemm_blas if use_blas_gemm else int_gemm)(tq.codes, wq.codes)
    y = dequant(acc, tq, wq, c)
    return LinearResult(r, tq, acc, y, f64_to_bf16(y))


def group_colsums(wq: WeightQuant, group_size: int) -> np.ndarray:
    """colsum[g, n] = sum of the weight codes of output channel n over the K-channels of group g; int32 [K/G, N]."""
    N, K = wq.codes.shape
    G = int(group_size)
    assert K % G == 0
    return wq.codes.astype(np.int64).reshape(N, K // G, G).sum(axis=2).T.astype(np.int32).copy()


def dequant_grouped(acc_g: np.ndarray, tq: TokenQuant, wq: WeightQuant, c: Optional[np.ndarray]) -> np.ndarray:
    """Group-wise activation ranges (every run of G channels of a token has its own s, z; Eq. 4 per group):

        Y[m, n] = sw_n * ( sum_g ( s_mg ACC_g[m, n] + z_mg colsum_g[n] ) - zp_n * sum_g ( s_mg rowsum_mg + G z_mg ) ) + c_n

    acc_g: int [K/G, M, N], the integer products of one group each.  It is the per-token formula of dequant()
    applied to each group with its own activation constants and the group's share of the weight sums."""
    ng, M, N = acc_g.shape
    K = wq.codes.shape[1]
    G = K // ng
    assert tq.scale.shape == (M, ng)
    s = tq.scale.astype(np.float64)
    z = tq.lo.astype(np.float64)
    rs = tq.rowsum.astype(np.float64)
    cs = group_colsums(wq, G).astype(np.float64)                     # [ng, N]
    f = np.zeros((M, N), dtype=np.float64)
    for g in range(ng):
        f += s[:, g:g + 1] * acc_g[g].astype(np.float64) + z[:, g:g + 1] * cs[g][None, :]
    rterm = (s * rs + G * z).sum(axis=1)[:, None]
    sw = wq.scale.astype(np.float64)[None, :]
    zp = wq.zero.astype(np.float64)[None, :]
    y = sw * (f - zp * rterm)
    if c is not None:
        y = y + np.asarray(c, dtype=np.float64)[None, :]
    return y


def linear_grouped(x: np.ndarray, rot_size: int, bias: Optional[np.ndarray], act_scale: Optional[np.ndarray],
                   clip_lo: float, clip_hi: float, group_size: int, wq: WeightQuant, c: Optional[np.ndarray],
                   *, r: Optional[np.ndarray] = None) -> LinearResult:
    """The layer with group-wise activation ranges, by its definition: the de-quantised activations
    x_hat = s_mg q + z_mg (Eq. 4 per group) times the de-quantised weights W_hat = sw (q_w - zp), plus c, in fp64.
    ``acc`` of the result is the plain integer product of the codes (all groups together)."""
    if r is None:
        r = rotate(x, rot_size)
    tq = quantize_tokens(r, bias, act_scale, clip_lo, clip_hi, group_size=group_size)
    y = dequantize_tokens(tq) @ dequantize_weights(wq).T
    if c is not None:
        y = y + np.asarray(c, dtype=np.float64)[None, :]
    acc = int_gemm_blas(tq.codes, wq.codes)
    return LinearResult(r, tq, acc, y, f64_to_bf16(y))


def linear_full_precision(x: np.ndarray, rot_size: int, w_rot: np.ndarray,
                          layer_bias: Optional[np.ndarray] = None) -> np.ndarray:
    """Unquantised layer (X R) W'^T + b in fp64 -- not a parity target; used for the Eq. 14
    identity and to report the quantisation signal-to-noise ratio of a synthetic layer."""
    y = rotate_f64(x, rot_size) @ np.asarray(w_rot, dtype=np.float64).T
    if layer_bias is not None:
        y = y + np.asarray(layer_bias, dtype=np.float64)[None, :]
    return y
