"""Pins for the oracle's fused-MoE definition (Sec. 2.2): a hand-computed scalar
case, numpy/torch fp64 library GEMMs for the dense special cases, a tile-ordered
re-implementation that goes through the align output, and algebraic invariants
chosen so that a dropped term, a wrong index or a transposed operand fails."""
import math

import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2604_26039_amd import synth

TINY = synth.SHAPES["tiny"]


def make(shape, T, seed, beta=1.0, x_std=None):
    X, Wg, Wu, Wd = synth.layer_tensors(shape, T, seed, x_std=x_std)
    ids, w = synth.routing(T, shape, beta, seed)
    return synth.bits(X), synth.bits(Wg), synth.bits(Wu), synth.bits(Wd), ids, w


def numpy_moe(Xb, Wgb, Wub, Wdb, ids, w, E, round_mid=False):
    """Same definition, different route: go through the align output tile by tile
    with numpy matmuls, then scatter-add rows back to their tokens."""
    X, Wg, Wu, Wd = (synth.bits_to_f64(a) for a in (Xb, Wgb, Wub, Wdb))
    T, H = X.shape
    k = ids.shape[1]
    bm = 4
    s, te, counts, meta = oracle.align(ids.reshape(-1), T, k, E, bm)
    out = np.zeros((T, H))
    P = T * k
    for m in range(int(meta[1])):
        e = int(te[m])
        pairs = s[m * bm:(m + 1) * bm]
        pairs = pairs[pairs != P]
        rows = pairs // k
        g = X[rows] @ Wg[e]
        u = X[rows] @ Wu[e]
        a = g / (1.0 + np.exp(-g)) * u
        if round_mid:
            a = np.array([[oracle.bf16_bits_to_f64(oracle.f64_to_bf16_bits(v)) for v in r] for r in a])
        y = a @ Wd[e]
        np.add.at(out, rows, w.reshape(-1)[pairs][:, None].astype(np.float64) * y)
    return out


def test_scalar_case_by_hand():
    # H = I = 1, one expert: out = w * SiLU(x*wg) * (x*wu) * wd
    x, wg, wu, wd, gate = 2.0, 1.0, 0.5, 4.0, 0.75
    b = lambda v: np.array(oracle.f64_to_bf16_bits(v), np.uint16)
    out = oracle.moe(b(x).reshape(1, 1), np.zeros((1, 1), np.int32), np.full((1, 1), gate, np.float32),
                     b(wg).reshape(1, 1, 1), b(wu).reshape(1, 1, 1), b(wd).reshape(1, 1, 1), E=1)
    expect = gate * (2.0 / (1.0 + math.exp(-2.0))) * 1.0 * 4.0
    assert out[0, 0] == pytest.approx(expect, rel=1e-15)


@pytest.mark.parametrize("beta,x_std", [(1.0, None), (0.2, None), (1.0, 4.0)])
def test_matches_tile_ordered_numpy(beta, x_std):
    Xb, Wgb, Wub, Wdb, ids, w = make(TINY, 16, seed=7, beta=beta, x_std=x_std)
    ref = oracle.moe(Xb, ids, w, Wgb, Wub, Wdb, E=TINY.E)
    alt = numpy_moe(Xb, Wgb, Wub, Wdb, ids, w, TINY.E)
    assert np.abs(ref - alt).max() <= 1e-12 * np.abs(ref).max()
    assert np.abs(ref).max() > 0


def test_round_mid_matches_tile_ordered_numpy():
    shape = synth.Shape("s", 64, 96, 4, 2)
    Xb, Wgb, Wub, Wdb, ids, w = make(shape, 6, seed=2, x_std=3.0)
    ref = oracle.moe(Xb, ids, w, Wgb, Wub, Wdb, E=4, round_mid=True)
    alt = numpy_moe(Xb, Wgb, Wub, Wdb, ids, w, 4, round_mid=True)
    assert np.abs(ref - alt).max() <= 1e-12 * np.abs(ref).max()
    exact = oracle.moe(Xb, ids, w, Wgb, Wub, Wdb, E=4)
    rel = np.linalg.norm(ref - exact) / np.linalg.norm(exact)
    assert 0 < rel < 2 ** -8  # one bf16 rounding of the activation


def test_single_expert_is_dense_swiglu_mlp_via_library_gemms():
    shape = synth.Shape("dense", 128, 192, 1, 1)
    X, Wg, Wu, Wd = synth.layer_tensors(shape, 9, seed=11, x_std=2.0)
    ids = np.zeros((9, 1), np.int32)
    w = np.ones((9, 1), np.float32)
    ref = oracle.moe(synth.bits(X), ids, w, synth.bits(Wg), synth.bits(Wu), synth.bits(Wd), E=1)
    Xd, Wgd, Wud, Wdd = (t.double() for t in (X, Wg[0], Wu[0], Wd[0]))
    dense = (torch.nn.functional.silu(Xd @ Wgd) * (Xd @ Wud)) @ Wdd
    assert np.abs(ref - dense.numpy()).max() <= 1e-12 * np.abs(ref).max()


def test_identical_experts_reduce_to_dense_mlp_for_any_routing():
    shape = synth.Shape("same", 64, 128, 8, 3)
    X, Wg, Wu, Wd = synth.layer_tensors(shape, 12, seed=4, x_std=2.0)
    Wg[:] = Wg[0]; Wu[:] = Wu[0]; Wd[:] = Wd[0]
    ids, w = synth.routing(12, shape, 0.5, seed=4)  # softmax gates sum to 1
    ref = oracle.moe(synth.bits(X), ids, w, synth.bits(Wg), synth.bits(Wu), synth.bits(Wd), E=8)
    Xd = X.double()
    dense = (torch.nn.functional.silu(Xd @ Wg[0].double()) * (Xd @ Wu[0].double())) @ Wd[0].double()
    scale = w.astype(np.float64).sum(axis=1, keepdims=True)
    assert np.abs(ref - scale * dense.numpy()).max() <= 1e-12 * np.abs(ref).max()


def test_linearity_and_zero_in_gate_weights():
    Xb, Wgb, Wub, Wdb, ids, w = make(TINY, 8, seed=3)
    a = oracle.moe(Xb, ids, w, Wgb, Wub, Wdb, E=TINY.E)
    z = oracle.moe(Xb, ids, np.zeros_like(w), Wgb, Wub, Wdb, E=TINY.E)
    assert (z == 0).all()
    w2 = np.zeros_like(w); w2[:, 0] = w[:, 0]
    w3 = w - w2
    b = oracle.moe(Xb, ids, w2, Wgb, Wub, Wdb, E=TINY.E) + oracle.moe(Xb, ids, w3, Wgb, Wub, Wdb, E=TINY.E)
    assert np.abs(a - b).max() <= 1e-13 * np.abs(a).max()
    c = oracle.moe(Xb, ids, 2 * w, Wgb, Wub, Wdb, E=TINY.E)
    assert np.abs(c - 2 * a).max() <= 1e-13 * np.abs(a).max()


def test_token_permutation_permutes_rows_and_row_subset_matches():
    Xb, Wgb, Wub, Wdb, ids, w = make(TINY, 10, seed=5)
    a = oracle.moe(Xb, ids, w, Wgb, Wub, Wdb, E=TINY.E)
    perm = np.random.default_rng(0).permutation(10)
    b = oracle.moe(Xb[perm], ids[perm], w[perm], Wgb, Wub, Wdb, E=TINY.E)
    assert (b == a[perm]).all()
    rows = np.array([7, 2, 2, 9], np.int32)
    c = oracle.moe(Xb, ids, w, Wgb, Wub, Wdb, E=TINY.E, rows=rows)
    assert (c == a[rows]).all()


def test_zero_up_or_zero_gate_gives_zero():
    Xb, Wgb, Wub, Wdb, ids, w = make(TINY, 4, seed=6)
    assert (oracle.moe(Xb, ids, w, Wgb, np.zeros_like(Wub), Wdb, E=TINY.E) == 0).all()
    assert (oracle.moe(Xb, ids, w, np.zeros_like(Wgb), Wub, Wdb, E=TINY.E) == 0).all()  # SiLU(0) = 0


def test_gate_and_up_are_not_interchangeable_and_weights_not_transposed():
    # swapping gate and up changes the result (SiLU is applied to the gate branch only);
    # a non-square H != I layer would read out of shape if an operand were transposed
    shape = synth.Shape("s", 32, 48, 2, 1)
    Xb, Wgb, Wub, Wdb, ids, w = make(shape, 3, seed=8, x_std=3.0)
    a = oracle.moe(Xb, ids, w, Wgb, Wub, Wdb, E=2)
    b = oracle.moe(Xb, ids, w, Wub, Wgb, Wdb, E=2)
    assert np.abs(a - b).max() > 1e-3 * np.abs(a).max()


def test_sparse_expert_dict_and_missing_expert():
    Xb, Wgb, Wub, Wdb, ids, w = make(TINY, 6, seed=9)
    full = oracle.moe(Xb, ids, w, Wgb, Wub, Wdb, E=TINY.E, rows=[1, 4])
    used = set(ids[[1, 4]].reshape(-1).tolist())
    d = lambda W: {e: W[e] for e in used}
    part = oracle.moe(Xb, ids, w, d(Wgb), d(Wub), d(Wdb), E=TINY.E, rows=[1, 4])
    assert (part == full).all()
    other = [t for t in range(6) if not set(ids[t].tolist()) <= used]
    if other:
        with pytest.raises(ValueError):
            oracle.moe(Xb, ids, w, d(Wgb), d(Wub), d(Wdb), E=TINY.E, rows=other[:1])


def test_dropped_ids_contribute_nothing():
    Xb, Wgb, Wub, Wdb, ids, w = make(TINY, 4, seed=10)
    ids2 = ids.copy(); ids2[:, 1] = TINY.E + 3
    w0 = w.copy(); w0[:, 1] = 0
    a = oracle.moe(Xb, ids2, w, Wgb, Wub, Wdb, E=TINY.E)
    b = oracle.moe(Xb, ids, w0, Wgb, Wub, Wdb, E=TINY.E)
    assert (a == b).all()


def test_bf16_rounding_ties_to_even_and_matches_torch():
    f = oracle.f64_to_bf16_bits
    assert f(1.0) == 0x3F80
    assert f(1.0 + 2.0 ** -8) == 0x3F80           # tie -> even (down)
    assert f(1.0 + 3 * 2.0 ** -8) == 0x3F82       # tie -> even (up)
    assert f(1.0 + 2.0 ** -8 + 2.0 ** -40) == 0x3F81  # just above the tie: a float detour would lose this
    assert f(-0.0) == 0x8000 and f(0.0) == 0
    assert f(float("inf")) == 0x7F80 and f(3.4e38) == 0x7F80  # overflow past the largest bf16
    assert f(2.0 ** -133) == 0x0001 and f(2.0 ** -134) == 0x0000  # smallest subnormal, tie to even
    v = torch.randn(2000, generator=torch.Generator().manual_seed(0), dtype=torch.float32) * 3
    ours = np.array([f(float(x)) for x in v], np.uint16)
    assert (ours == synth.bits(v.to(torch.bfloat16))).all()
    assert all(oracle.bf16_bits_to_f64(int(b)) == float(t) for b, t in zip(ours[:50], v.to(torch.bfloat16)[:50].float()))
