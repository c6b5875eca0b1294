"""Pins of the FP8 (W8A8, 128x128 block scales; Sec. 4.3) oracle against things other than itself: torch's
float8_e4m3fn conversions, hand values of the format, the definition of the block scale, quantisation error
bounds, and an independent scalar re-computation of a tiny layer."""
import math

import numpy as np
import pytest
import torch

from oracle import fp8, oracle


def test_decode_matches_torch_for_every_code():
    codes = np.arange(256, dtype=np.uint8)
    want = torch.from_numpy(codes).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    got = fp8.e4m3_decode(codes)
    assert np.array_equal(np.isnan(got), np.isnan(want))
    assert np.array_equal(got[~np.isnan(got)], want[~np.isnan(want)])
    # hand values of the format: 1.0, the largest finite value, the smallest subnormal, the smallest normal
    assert fp8.e4m3_decode(np.uint8(0x38)) == 1.0 and fp8.e4m3_decode(np.uint8(0x7E)) == 448.0
    assert fp8.e4m3_decode(np.uint8(0x01)) == 2.0 ** -9 and fp8.e4m3_decode(np.uint8(0x08)) == 2.0 ** -6
    assert fp8.e4m3_decode(np.uint8(0xB8)) == -1.0


def test_encode_matches_torch_in_range_including_every_tie():
    vals = fp8.e4m3_decode(np.arange(127, dtype=np.uint8))
    mids = (vals[:-1] + vals[1:]) / 2                       # every tie between neighbours
    rng = np.random.default_rng(0)
    x = np.concatenate([vals, mids, np.nextafter(mids, 0), np.nextafter(mids, 1e9),
                        rng.uniform(-448, 448, 20000), rng.normal(0, 1, 20000), rng.normal(0, 0.01, 20000)])
    x = np.concatenate([x, -x]).astype(np.float32).astype(np.float64)   # torch converts from float32
    want = torch.from_numpy(x.astype(np.float32)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = fp8.e4m3_encode(x)
    nz = x != 0                                             # the sign of zero is kept by both; compare it apart
    assert np.array_equal(got[nz], want[nz])
    assert fp8.e4m3_encode(np.array([0.0]))[0] == 0 and fp8.e4m3_encode(np.array([-0.0]))[0] == 0x80


def test_encode_hand_cases_round_trip_and_saturation():
    assert list(fp8.e4m3_encode(np.array([1.0, 448.0, 2.0 ** -9, 2.0 ** -10, 3 * 2.0 ** -10, 1.0625, 1.1875]))) == \
        [0x38, 0x7E, 0x01, 0x00, 0x02, 0x38, 0x3A]          # ties go to the even code: 1.0625 -> 1.0, 1.1875 -> 1.25
    codes = np.arange(127, dtype=np.uint8)
    assert np.array_equal(fp8.e4m3_encode(fp8.e4m3_decode(codes)), codes)          # every finite value is a fixed point
    assert list(fp8.e4m3_encode(np.array([449.0, 1e9, -1e9, 464.0]))) == [0x7E, 0x7E, 0xFE, 0x7E]   # saturates, never NaN


def test_block_scale_is_the_smallest_admissible_power_of_two():
    assert fp8.e8m0_byte(448.0) == 127 and fp8.e8m0_byte(448.0001) == 128 and fp8.e8m0_byte(224.0) == 126
    assert fp8.e8m0_byte(1.0) == 127 - 8 and fp8.e8m0_byte(1.75) == 127 - 8 and fp8.e8m0_byte(1.7500001) == 127 - 7
    assert fp8.e8m0_byte(0.0) == 127
    rng = np.random.default_rng(1)
    amax = np.concatenate([np.exp(rng.uniform(-20, 20, 2000)), 448.0 * 2.0 ** np.arange(-20, 20), 1.75 * 2.0 ** np.arange(-20, 20)])
    vec = fp8.e8m0_bytes(amax)
    for a, b in zip(amax, vec):
        assert b == fp8.e8m0_byte(a)
        s = 2.0 ** (int(b) - 127)
        assert a / s <= 448.0 < a / (s / 2)                   # the definition: admissible, and the next smaller power is not


def test_quantisation_layouts_and_error_bounds():
    rng = np.random.default_rng(2)
    X = rng.normal(0, 1, (5, 384)) * np.exp(rng.uniform(-3, 3, (5, 1)))
    codes, sb = fp8.quantize_rows(X)
    assert codes.shape == (5, 384) and sb.shape == (5, 3)
    Xd = fp8.dequantize_rows(codes, sb)
    for t in range(5):
        for g in range(3):
            blk = X[t, 128 * g:128 * g + 128]
            s = 2.0 ** (int(sb[t, g]) - 127)
            assert sb[t, g] == fp8.e8m0_byte(np.abs(blk).max())                       # group structure: 128 k-values of one row
            err = np.abs(Xd[t, 128 * g:128 * g + 128] - blk)
            # half an ulp: relative 2^-4 for normal codes, absolute 2^-10 * scale in the subnormal range
            assert (err <= np.maximum(np.abs(blk) * 2.0 ** -4, s * 2.0 ** -10) + 1e-300).all()
    W = rng.normal(0, 0.05, (256, 384))
    W[128:, 128:256] *= 40.0                                                          # one block with a different range
    wc, wsb = fp8.quantize_blocks(W)
    assert wsb.shape == (2, 3) and wsb[1, 1] > wsb[0, 0]
    for i in range(2):
        for j in range(3):
            assert wsb[i, j] == fp8.e8m0_byte(np.abs(W[128 * i:128 * i + 128, 128 * j:128 * j + 128]).max())
    Wd = fp8.dequantize_blocks(wc, wsb)
    assert np.abs(Wd - W).max() <= np.abs(W).max() * 2.0 ** -4
    # values that are representable with scale 1 survive exactly
    exact = fp8.e4m3_decode(rng.integers(0, 127, (2, 128)).astype(np.uint8))
    exact[0, 0] = 448.0; exact[1, 0] = 320.0; exact[1, 1] = 448.0
    c2, s2 = fp8.quantize_rows(exact)
    assert (s2 == 127).all() and np.array_equal(fp8.dequantize_rows(c2, s2), exact)


def test_round_bf16_matches_torch():
    rng = np.random.default_rng(3)
    v = np.concatenate([rng.normal(0, 1, 5000), rng.normal(0, 1e-3, 5000), np.array([1.00390625, 1.01171875, 0.0, -0.0, 3.0])])
    v32 = v.astype(np.float32)                                                       # torch rounds from float32
    want = torch.from_numpy(v32).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(fp8.round_bf16(v32.astype(np.float64)), want)


def _bits(a):
    return torch.from_numpy(np.asarray(a, np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def test_layer_against_a_scalar_recomputation():
    """Tiny layer (H = I = 128, two experts, top-2) re-computed with Python scalars and math.fsum: quantise x, two dot
    products per feature, SiLU * up, bf16 rounding, quantise, down projection, weighted sum."""
    rng = np.random.default_rng(4)
    H = I = 128
    X = fp8.round_bf16(rng.normal(0, 1.0, (3, H)))
    Wg = {e: fp8.quantize_blocks(rng.normal(0, H ** -0.5, (H, I))) for e in range(2)}
    Wu = {e: fp8.quantize_blocks(rng.normal(0, H ** -0.5, (H, I))) for e in range(2)}
    Wd = {e: fp8.quantize_blocks(rng.normal(0, I ** -0.5, (I, H))) for e in range(2)}
    ids = np.array([[0, 1], [1, 0], [1, 5]], np.int32)       # the last pair names an expert that does not exist
    w = rng.uniform(0.1, 0.9, (3, 2)).astype(np.float32)
    got = fp8.moe_fp8(X, ids, w, Wg, Wu, Wd, E=2)

    def q_row(v):                                            # one group of 128: (dequantised values)
        b = fp8.e8m0_byte(max(abs(float(t)) for t in v))
        s = 2.0 ** (b - 127)
        return [float(fp8.e4m3_decode(fp8.e4m3_encode(np.array([float(t) / s])))[0]) * s for t in v]

    for t in range(3):
        xq = q_row(X[t])
        ref = [0.0] * H
        for j in range(2):
            e = int(ids[t, j])
            if not 0 <= e < 2:
                continue
            g_w, u_w, d_w = (fp8.dequantize_blocks(*W[e]) for W in (Wg, Wu, Wd))
            a = []
            for i in range(I):
                g = math.fsum(xq[k] * g_w[k, i] for k in range(H))
                u = math.fsum(xq[k] * u_w[k, i] for k in range(H))
                a.append(float(fp8.round_bf16(np.array([g / (1.0 + math.exp(-g)) * u]))[0]))
            aq = q_row(a)
            for h in range(H):
                ref[h] += float(w[t, j]) * math.fsum(aq[i] * d_w[i, h] for i in range(I))
        assert np.allclose(got[t], ref, rtol=1e-10, atol=1e-12)


def test_layer_reduces_to_the_unquantised_definition_when_nothing_is_lost():
    """Weights and activations that E4M3 holds exactly with scale 1, and a down projection that makes the
    intermediate irrelevant to rounding (identity-like on exact small integers is not available, so W_down = 0 and
    W_up = 0 cases, plus linearity in the router weights)."""
    rng = np.random.default_rng(5)
    H, I, E = 128, 256, 3
    X = fp8.round_bf16(rng.normal(0, 1, (4, H)))
    mk = lambda k, n, sd: fp8.quantize_blocks(rng.normal(0, sd, (k, n)))
    Wg = {e: mk(H, I, 0.1) for e in range(E)}
    Wu = {e: mk(H, I, 0.1) for e in range(E)}
    Wd = {e: mk(I, H, 0.1) for e in range(E)}
    ids = rng.integers(0, E, (4, 2)).astype(np.int32)
    w = rng.uniform(0.1, 1, (4, 2)).astype(np.float32)
    base = fp8.moe_fp8(X, ids, w, Wg, Wu, Wd, E)
    assert np.abs(base).max() > 0
    zero = {e: (np.zeros((I, H), np.uint8), np.full((I // 128, H // 128), 127, np.uint8)) for e in range(E)}
    assert (fp8.moe_fp8(X, ids, w, Wg, Wu, zero, E) == 0).all()                     # W_down = 0
    zero_u = {e: (np.zeros((H, I), np.uint8), np.full((H // 128, I // 128), 127, np.uint8)) for e in range(E)}
    assert (fp8.moe_fp8(X, ids, w, Wg, zero_u, Wd, E) == 0).all()                   # W_up = 0
    assert np.allclose(fp8.moe_fp8(X, ids, 2 * w, Wg, Wu, Wd, E), 2 * base, rtol=1e-12)   # linear in the router weights
    perm = np.array([2, 0, 3, 1])
    assert np.allclose(fp8.moe_fp8(X[perm], ids[perm], w[perm], Wg, Wu, Wd, E), base[perm], rtol=1e-12)
    assert np.allclose(fp8.moe_fp8(X, ids, w, Wg, Wu, Wd, E, rows=[3, 1]), base[[3, 1]], rtol=1e-12)


def test_layer_is_close_to_the_bf16_layer_it_approximates():
    """Against the bf16 oracle on the unquantised weights: the W8A8 result differs by quantisation noise only
    (3 mantissa bits: a few percent), far from what a wrong scale, a transposed block grid or a dropped term gives."""
    rng = np.random.default_rng(6)
    H, I, E, T, k = 256, 384, 4, 6, 2
    Xf = fp8.round_bf16(rng.normal(0, 1, (T, H)))
    Wg = fp8.round_bf16(rng.normal(0, H ** -0.5, (E, H, I)))
    Wu = fp8.round_bf16(rng.normal(0, H ** -0.5, (E, H, I)))
    Wd = fp8.round_bf16(rng.normal(0, I ** -0.5, (E, I, H)))
    Wg[1, :128, 128:256] *= 16.0                                                      # block scales must differ to pass
    ids = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    w = rng.uniform(0.2, 0.8, (T, k)).astype(np.float32)
    ref = oracle.moe(_bits(Xf), ids, w, _bits(Wg), _bits(Wu), _bits(Wd), E=E)
    q = lambda W: {e: fp8.quantize_blocks(W[e]) for e in range(E)}
    got = fp8.moe_fp8(Xf, ids, w, q(Wg), q(Wu), q(Wd), E)
    rel = np.linalg.norm(got - ref) / np.linalg.norm(ref)
    assert 1e-3 < rel < 8e-2, rel
