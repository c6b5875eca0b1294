"""CPU oracle of the W8A8 FP8 variant of the fused MoE layer (paper Sec. 4.3: "W8A8 FP8, 128x128 block
scales"; Sec. 2.2 phase 2: the activation is re-quantised to FP8 between the projections).

TEST INFRASTRUCTURE ONLY.  Nothing in the product may import this module; only tests/, the smoke check and the
benchmark's cpu_baseline leg use it.  It shares no code with the HIP path.  Plain numpy in float64, written out
from the definitions:

* FP8 = OCP E4M3 ("e4m3fn"): 1 sign, 4 exponent (bias 7), 3 mantissa bits, subnormals in steps of 2^-9,
  largest finite value 448, no infinities, S.1111.111 = NaN.  Encoding rounds to nearest, ties to the even
  code, and saturates at +-448.
* A block scale is a power of two stored as an E8M0 byte b (scale = 2^(b-127)): the smallest power of two s
  with amax/s <= 448, amax being the largest magnitude in the block (b = 127 for an all-zero block).  The paper
  only says "block scales"; powers of two are the reading taken here (the scale format the chip's scaled
  matrix instructions consume), stated in the design notes.
* Weights W [K, N] carry one scale per 128 x 128 block; activations one scale per token and 128 consecutive
  k-values (the usual companion of 128 x 128 weight blocks, paper silent).
* Layer: x -> per-group quantisation -> gate/up projections on the dequantised values -> SiLU(g)*u -> rounded to
  bf16 (what leaves the first kernel) -> per-group quantisation -> down projection -> router-weighted sum.
"""
from __future__ import annotations

import math

import numpy as np

E4M3_MAX = 448.0
GROUP = 128

# every non-negative finite E4M3 value, indexed by its code 0..126
_POS = np.array([(m * 2.0 ** -9) if e == 0 else (1.0 + m / 8.0) * 2.0 ** (e - 7)
                 for e in range(16) for m in range(8)][:127], dtype=np.float64)


def e4m3_decode(codes) -> np.ndarray:
    """uint8 codes -> float64 values (NaN for 0x7F / 0xFF)."""
    c = np.asarray(codes, dtype=np.uint8)
    mag = c & 0x7F
    val = np.where(mag == 0x7F, np.nan, _POS[np.minimum(mag, 126)])
    return np.where(c & 0x80, -val, val)


def e4m3_encode(x) -> np.ndarray:
    """float64 values -> uint8 codes: nearest representable value, ties to the even code, saturating at 448.
    By definition: look the magnitude up among the 127 finite values."""
    x = np.asarray(x, dtype=np.float64)
    a = np.minimum(np.abs(x), E4M3_MAX)
    hi = np.searchsorted(_POS, a, side="left")            # first value >= a
    hi = np.minimum(hi, 126)
    lo = np.maximum(hi - 1, 0)
    d_hi, d_lo = _POS[hi] - a, a - _POS[lo]
    pick_hi = (d_hi < d_lo) | ((d_hi == d_lo) & (hi % 2 == 0))
    code = np.where(pick_hi, hi, lo).astype(np.uint8)
    return np.where(np.signbit(x), code | 0x80, code).astype(np.uint8)


def e8m0_byte(amax: float) -> int:
    """Byte b of the smallest power of two 2^(b-127) with amax / 2^(b-127) <= 448 (127 when amax == 0)."""
    amax = float(amax)
    if amax == 0.0:
        return 127
    e = int(math.floor(math.log2(amax / E4M3_MAX)))       # a guess, corrected by the definition below
    while math.ldexp(E4M3_MAX, e) < amax:
        e += 1
    while math.ldexp(E4M3_MAX, e - 1) >= amax:
        e -= 1
    return int(min(max(e + 127, 0), 254))


def e8m0_bytes(amax) -> np.ndarray:
    """e8m0_byte for an array, in closed form: with amax = f * 2^ex, f in [0.5, 1), and 448 = 0.875 * 2^9 the
    smallest admissible exponent is ex - 9 when f <= 0.875 and ex - 8 otherwise (tested against e8m0_byte)."""
    amax = np.asarray(amax, dtype=np.float64)
    f, ex = np.frexp(amax)
    e = np.where(f <= 0.875, ex - 9, ex - 8)
    return np.where(amax == 0.0, 127, np.clip(e + 127, 0, 254)).astype(np.uint8)


def e8m0_scale(b) -> np.ndarray:
    return np.ldexp(1.0, np.asarray(b, dtype=np.int64) - 127)


def quantize_rows(X):
    """X [T, K] (K multiple of 128) -> (codes uint8 [T, K], scale bytes uint8 [T, K/128]): one scale per row and
    128 consecutive k-values."""
    X = np.asarray(X, dtype=np.float64)
    T, K = X.shape
    assert K % GROUP == 0
    G = X.reshape(T, K // GROUP, GROUP)
    sb = e8m0_bytes(np.abs(G).max(axis=2))
    codes = e4m3_encode(G / e8m0_scale(sb)[:, :, None]).reshape(T, K)
    return codes, sb


def quantize_blocks(W):
    """W [K, N] (both multiples of 128) -> (codes uint8 [K, N], scale bytes uint8 [K/128, N/128])."""
    W = np.asarray(W, dtype=np.float64)
    K, N = W.shape
    assert K % GROUP == 0 and N % GROUP == 0
    B = W.reshape(K // GROUP, GROUP, N // GROUP, GROUP)
    sb = e8m0_bytes(np.abs(B).max(axis=(1, 3)))
    codes = e4m3_encode(B / e8m0_scale(sb)[:, None, :, None]).reshape(K, N)
    return codes, sb


def dequantize_rows(codes, sb) -> np.ndarray:
    return e4m3_decode(codes) * np.repeat(e8m0_scale(sb), GROUP, axis=1)


def dequantize_blocks(codes, sb) -> np.ndarray:
    return e4m3_decode(codes) * np.repeat(np.repeat(e8m0_scale(sb), GROUP, axis=0), GROUP, axis=1)


def round_bf16(a) -> np.ndarray:
    """float64 -> nearest bfloat16 value (8 significant bits, ties to even), returned as float64.  Straight from
    the float64 value, so there is no double rounding through float32."""
    v = np.asarray(a, dtype=np.float64)
    m, e = np.frexp(np.abs(v))                    # |v| = m * 2^e, m in [0.5, 1)
    q = m * 256.0                                 # 8 significant bits: integer part in [128, 256)
    r = np.floor(q)
    frac = q - r
    r = r + ((frac > 0.5) | ((frac == 0.5) & (r % 2 == 1)))
    return np.where(v == 0.0, v, np.copysign(np.ldexp(r / 256.0, e), v))


def silu(x):
    return x / (1.0 + np.exp(-x))


def moe_fp8(X, ids, w, Wg, Wu, Wd, E: int, rows=None) -> np.ndarray:
    """W8A8 fused MoE layer by definition, float64.

    X: float64 [T, H] (the exact values of the bf16 activations); ids int [T, k]; w float [T, k];
    Wg, Wu: dict expert -> (codes uint8 [H, I], scale bytes [H/128, I/128]); Wd: dict -> ([I, H], [I/128, H/128]).
    rows: token rows to evaluate (default all).  Pairs whose expert id is outside [0, E) contribute nothing."""
    X = np.asarray(X, dtype=np.float64)
    T, H = X.shape
    rows = list(range(T)) if rows is None else [int(r) for r in rows]
    out = np.zeros((len(rows), H), np.float64)
    deq = {}

    def weights(e):
        if e not in deq:
            deq[e] = (dequantize_blocks(*Wg[e]), dequantize_blocks(*Wu[e]), dequantize_blocks(*Wd[e]))
        return deq[e]

    for n, t in enumerate(rows):
        xq = dequantize_rows(*quantize_rows(X[t:t + 1]))            # [1, H]: what the first projection multiplies
        for j in range(ids.shape[1]):
            e = int(ids[t, j])
            if e < 0 or e >= E:
                continue
            g_w, u_w, d_w = weights(e)
            g = xq @ g_w
            u = xq @ u_w
            a = round_bf16(silu(g) * u)                              # the activation leaves the first kernel as bf16
            aq = dequantize_rows(*quantize_rows(a))
            out[n] += float(w[t, j]) * (aq @ d_w)[0]
    return out
