"""Host-side checks of libramp.so that need no GPU: the library loads, exports every symbol the
header declares, enumerates a sane configuration family, and its cost-model fit/select agree
with the oracle (predictions and argmin; the raw b/c split is not identifiable)."""
import os
import re

import numpy as np
import pytest

from oracle import oracle
from paper_2604_26039_amd import ramp, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "ramp.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = sorted(set(re.findall(r"\b(ramp_[a-z_0-9]+)\s*\(", hdr)))
    assert declared, "no declarations found"
    L = ramp.lib()
    for name in declared:
        assert hasattr(L, name), f"libramp.so does not export {name}"
    assert sorted(ramp.EXPORTS) == declared


def shape_of(name, T):
    s = synth.SHAPES[name]
    return ramp.Shape(T, s.k, s.E, s.H, s.I)


@pytest.mark.parametrize("name", ["tiny", "olmoe", "qwen3", "mixtral", "dsv3"])
def test_config_family(name):
    sh = shape_of(name, 64)
    cfgs = ramp.configs(sh)
    assert len(cfgs) >= 12
    assert len({c.key() for c in cfgs}) == len(cfgs)
    bms = {c.bm for c in cfgs}
    assert {16, 64, 256} <= bms
    if name == "tiny":
        assert {4, 16} <= bms
    for c in cfgs:
        assert (2 * sh.I) % c.bn == 0 and sh.H % c.bn == 0 and sh.H % c.bk == 0 and sh.I % c.bk == 0
        assert ramp.config_ntiles(sh, c) == 2 * sh.I // c.bn + sh.H // c.bn
        W = ramp.config_wave_capacity(c)
        assert W >= 256 and W % 256 == 0
        assert ramp.fused_moe_workspace_bytes(sh, c) > 0


@pytest.mark.parametrize("name", ["tiny", "olmoe", "qwen3", "mixtral", "dsv3"])
def test_fp8_config_family(name):
    """The W8A8 FP8 family (Sec. 4.3) is enumerated apart from the bf16 one and sized by the same queries."""
    sh = shape_of(name, 64)
    cfgs = ramp.fp8_configs(sh)
    assert len(cfgs) >= 4 and len({c.key() for c in cfgs}) == len(cfgs)
    assert not any(c.mode & ramp.FP8_MODE for c in ramp.configs(sh))
    for c in cfgs:
        assert c.mode & ramp.FP8_MODE and c.bk == 128
        assert (2 * sh.I) % c.bn == 0 and sh.H % c.bn == 0
        assert ramp.config_ntiles(sh, c) == 2 * sh.I // c.bn + sh.H // c.bn
        W = ramp.fp8_config_wave_capacity(c)
        assert W >= 256 and W % 256 == 0
        assert ramp.fused_moe_fp8_workspace_bytes(sh, c) > ramp.fused_moe_workspace_bytes(sh, ramp.configs(sh)[0]) // 8
    assert ramp.fp8_pack_bytes(sh) > 3 * sh.E * sh.H * sh.I
    off, strides = ramp.fp8_pack_layout(sh)
    assert off[0] == 2 * sh.I * sh.H and off[1] == sh.I * sh.H and strides[0] % 4 == 0 and strides[0] >= sh.H // 128
    with pytest.raises(ramp.RampError):
        ramp.fp8_config_wave_capacity(ramp.configs(sh)[0])


def test_unknown_config_is_rejected():
    bad = ramp.Config(24, 64, 128, 2, 2, 0)  # bm=24 is not in the family
    with pytest.raises(ramp.RampError) as ei:
        ramp.config_wave_capacity(bad)
    assert ei.value.status == ramp.EUNSUPPORTED
    assert "not instantiated" in ramp.last_error()


@pytest.mark.parametrize("T,k,E,bm", [(16, 2, 16, 4), (1, 8, 64, 16), (4096, 8, 64, 256), (0, 8, 4, 16), (3, 8, 256, 7)])
def test_align_capacity_matches_oracle(T, k, E, bm):
    assert ramp.align_capacity(T, k, E, bm) == oracle.align_capacity(T, k, E, bm)


@pytest.mark.parametrize("name,T,beta", [("olmoe", 256, 0.2), ("dsv3", 8192, 1.0), ("qwen3", 1, 1.0), ("mixtral", 1024, "zipf1.2")])
def test_grid_matches_oracle(name, T, beta):
    """ramp_grid = Eq. 1 per configuration, plus the distinct-tile and pair sums, against the oracle's Eq. 1 and a
    plain count."""
    s = synth.SHAPES[name]
    sh = shape_of(name, T)
    cfgs = ramp.configs(sh)
    nt = [ramp.config_ntiles(sh, c) for c in cfgs]
    ids, _ = synth.routing(T, s, beta, seed=3)
    counts = np.zeros(s.E, np.int32)
    for e in ids.reshape(-1):
        counts[e] += 1
    g, d, pairs = ramp.grid(s.E, cfgs, nt, counts)
    assert pairs == T * s.k
    active = int((counts > 0).sum())
    for i, c in enumerate(cfgs):
        assert g[i] == oracle.grid(counts, c.bm, nt[i])
        assert d[i] == active * nt[i]
    with pytest.raises(ramp.RampError):
        ramp.grid(s.E, cfgs, [0] * len(cfgs), counts)


def test_shape_limits_of_the_pair_index_division():
    """The kernels divide pair indices by k with a 64-bit multiplication by ceil(2^40/k): exact for k <= 1024 and
    pairs < 2^30 as long as the product fits 64 bits, so shapes beyond that are not enumerated."""
    for k in (1, 2, 3, 7, 8, 64, 1000, 1024):
        magic = -(-(1 << 40) // k)
        for p in (0, 1, k - 1, k, k + 1, 12345 * k + k - 1, (1 << 24) * k - 1, min((1 << 30) - 1, (1 << 24) * k)):
            if p * magic < (1 << 64):
                assert (p * magic) >> 40 == p // k, (k, p)
    assert ramp.num_configs(ramp.Shape(1 << 18, 8, 64, 2048, 1024)) > 0        # 2^21 pairs
    assert ramp.num_configs(ramp.Shape((1 << 24) + 16, 1, 64, 128, 128)) == 0   # k = 1: product would overflow
    assert ramp.num_configs(ramp.Shape(4, 1025, 64, 2048, 1024)) == 0           # k > 1024


def synthetic_profile(rng, n_cfg, n_pts):
    W = rng.choice([256, 512, 1024, 2048], n_cfg).astype(np.int32)
    g = np.empty((n_cfg, n_pts), np.int64)
    t = np.empty((n_cfg, n_pts), np.float64)
    for c in range(n_cfg):
        scale = rng.choice([8, 60, 900])
        g[c] = rng.integers(1, 40, n_pts) * scale
        t[c] = 8 + rng.uniform(0.001, 0.05) * g[c] + rng.uniform(0, 4) * np.log(g[c] + 1) + rng.normal(0, 0.3, n_pts)
    return W, g, t


def test_fit_predictions_match_oracle():
    rng = np.random.default_rng(0)
    W, g, t = synthetic_profile(rng, 30, 25)
    theta = ramp.cost_model_fit(W, g, t)
    saw_log = saw_nolog = False
    for c in range(30):
        th_o, use_log = oracle.fit_cost_model(g[c], t[c], int(W[c]))
        saw_log |= use_log
        saw_nolog |= not use_log
        assert (theta[c, 3] != 0) == use_log
        Xd = oracle.design_matrix(g[c], int(W[c]))
        q = np.array([1, 7, 100, 5000, 200000], float)
        Xq = oracle.design_matrix(q, int(W[c]))
        for X in (Xd, Xq):
            po, pl = X @ th_o, X @ theta[c].astype(np.float64)
            assert np.abs(po - pl).max() <= 2e-5 * np.abs(po).max()  # theta is stored as fp32
        # identifiable quantities
        assert theta[c, 0] == pytest.approx(th_o[0], rel=1e-5, abs=1e-4)
        assert theta[c, 1] / W[c] + theta[c, 2] == pytest.approx(th_o[1] / W[c] + th_o[2], rel=1e-5)
    assert saw_log and saw_nolog


@pytest.mark.parametrize("flags", [0, 15])
def test_five_term_fit_and_select_match_oracle(flags):
    """ramp_cost_model_fit5 / select5 (Sec. 5.3 ablation) against the oracle's five-term fit: predictions on the
    profiling grids and beyond, and the argmin of a brute-force evaluation."""
    rng = np.random.default_rng(11)
    n_cfg, n_pts = 12, 25
    W, g, t = synthetic_profile(rng, n_cfg, n_pts)
    t = t + 0.5 * (g / W[:, None]) ** 2
    distinct = np.maximum(1, g // 3) if flags & ramp.CM_DISTINCT_TILES else None
    pairs = rng.integers(8, 60000, n_pts).astype(np.int64) if flags & ramp.CM_PAIRS else None
    theta5 = ramp.cost_model_fit(W, g, t, distinct=distinct, pairs=pairs, flags=flags, terms=5)
    assert theta5.shape == (n_cfg, 5)
    for c in range(n_cfg):
        th_o, _ = oracle.fit_cost_model(g[c], t[c], int(W[c]), n_terms=5, distinct=None if distinct is None else distinct[c],
                                        relative=bool(flags & ramp.CM_RELATIVE), wave_floor=bool(flags & ramp.CM_WAVE_FLOOR),
                                        pairs=pairs)
        for i in range(n_pts):
            kw = dict(distinct=None if distinct is None else distinct[c, i], wave_floor=bool(flags & ramp.CM_WAVE_FLOOR),
                      pairs=None if pairs is None else pairs[i])
            po = oracle.predict5(th_o, g[c, i], int(W[c]), **kw)
            pl = oracle.predict5(theta5[c].astype(np.float64), g[c, i], int(W[c]), **kw)
            assert abs(po - pl) <= 5e-5 * max(abs(po), 1.0)
    # select5 on a histogram: brute force over the oracle's five-term prediction with the library's coefficients
    E = 16
    counts = rng.integers(0, 300, E).astype(np.int32)
    cfgs = [ramp.Config(int(bm), 128, 64, 4, 2, 0) for bm in rng.choice([4, 16, 64, 256], n_cfg)]
    nt = rng.integers(2, 40, n_cfg).astype(np.int32)
    best, pred = ramp.cost_model_select(E, cfgs, nt, W, theta5, counts, want_pred=True, flags=flags, terms=5)
    active, P = int((counts > 0).sum()), int(counts.sum())
    want = []
    for c in range(n_cfg):
        gc = oracle.grid(counts, cfgs[c].bm, int(nt[c]))
        want.append(oracle.predict5(theta5[c].astype(np.float64), gc, int(W[c]),
                                    distinct=active * int(nt[c]) if flags & ramp.CM_DISTINCT_TILES else None,
                                    wave_floor=bool(flags & ramp.CM_WAVE_FLOOR), pairs=P if flags & ramp.CM_PAIRS else None))
    assert np.allclose(pred, want, rtol=1e-12, atol=1e-9)
    assert best == int(np.argmin(want))


def test_fit_handles_constant_grid():
    # every profiling point has the same grid (T=1: one tile per routed expert whatever the skew)
    W = np.array([256], np.int32)
    g = np.full((1, 25), 40, np.int64)
    t = np.full((1, 25), 17.0) + np.linspace(-0.1, 0.1, 25)[None]
    theta = ramp.cost_model_fit(W, g, t)
    th_o, _ = oracle.fit_cost_model(g[0], t[0], 256)
    x = oracle.design_matrix([40], 256)[0]
    assert x @ theta[0].astype(float) == pytest.approx(17.0, rel=1e-5)
    assert x @ th_o == pytest.approx(17.0, rel=1e-9)


def test_select_matches_oracle_bit_for_bit():
    rng = np.random.default_rng(1)
    sh = shape_of("olmoe", 256)
    cfgs = ramp.configs(sh)
    n = len(cfgs)
    nt = [ramp.config_ntiles(sh, c) for c in cfgs]
    wc = [ramp.config_wave_capacity(c) for c in cfgs]
    bm = [c.bm for c in cfgs]
    for trial in range(25):
        theta = (np.abs(rng.normal(0, 1, (n, 4))) * [20, 3, 0.02, 2]).astype(np.float32)
        beta = rng.choice([1.0, 0.5, 0.2, 0.1])
        counts = synth.histogram_subset(int(rng.choice([1, 16, 64, 256, 1024])), sh.k, sh.E, beta, seed=trial)
        best, pred = ramp.cost_model_select(sh.E, cfgs, nt, wc, theta, counts, want_pred=True)
        b_o, p_o = oracle.select(bm, nt, wc, theta, counts)
        assert best == b_o
        assert (pred == p_o).all()


def test_select_rejects_bad_arguments():
    sh = shape_of("tiny", 16)
    cfgs = ramp.configs(sh)[:2]
    with pytest.raises(ramp.RampError):
        ramp.cost_model_select(sh.E, cfgs, [1, 1], [0, 256], np.zeros((2, 4), np.float32), np.zeros(sh.E, np.int32))


def test_adapted_model_fit_and_select_match_oracle():
    """RAMP_CM_RELATIVE | RAMP_CM_DISTINCT_TILES: predictions agree with the oracle's fit, and the
    selection is bit-identical to the oracle's for the same theta."""
    rng = np.random.default_rng(4)
    sh = shape_of("qwen3", 512)
    cfgs = ramp.configs(sh)
    n = len(cfgs)
    nt = np.array([ramp.config_ntiles(sh, c) for c in cfgs])
    wc = np.array([ramp.config_wave_capacity(c) for c in cfgs])
    bm = [c.bm for c in cfgs]
    hists = [synth.histogram_subset(int(T), sh.k, sh.E, b, seed=i) for i, (T, b) in
             enumerate((T, b) for T in (1, 6, 40, 250, 1500) for b in (1.0, 0.7, 0.4, 0.25, 0.12))]
    g = np.array([[oracle.grid(h, bm[c], int(nt[c])) for h in hists] for c in range(n)], np.int64)
    act = np.array([int((h > 0).sum()) for h in hists])
    u = nt[:, None] * act[None, :]
    t = 9 + 0.02 * g + 0.3 * u + rng.normal(0, 0.2, g.shape) + 0.002 * g * rng.random(g.shape)
    flags = ramp.CM_RELATIVE | ramp.CM_DISTINCT_TILES
    theta = ramp.cost_model_fit(wc, g, t, distinct=u, flags=flags)
    for c in range(0, n, 3):
        th_o, use_log = oracle.fit_cost_model(g[c], t[c], int(wc[c]), distinct=u[c], relative=True)
        X = oracle.design_matrix(g[c], int(wc[c]), u[c])
        po, pl = X @ th_o, X @ theta[c].astype(np.float64)
        assert np.abs(po - pl).max() <= 5e-5 * np.abs(po).max()
        assert (theta[c, 3] != 0) == use_log
    for i, h in enumerate(hists[::4]):
        best, pred = ramp.cost_model_select(sh.E, cfgs, nt, wc, theta, h, want_pred=True, flags=flags)
        b_o, p_o = oracle.select(bm, nt, wc, theta, h, distinct_tiles=True)
        assert best == b_o and (pred == p_o).all()
    with pytest.raises(ramp.RampError):
        ramp.cost_model_fit(wc, g, t, distinct=None, flags=flags)   # distinct tiles required
    with pytest.raises(ramp.RampError):
        ramp.cost_model_fit(wc, g, -t, distinct=u, flags=flags)     # relative fit needs positive times


def test_mi355x_model_fit_and_select_match_oracle():
    """All four variant flags together (relative fit, distinct tiles, wave floor, pair-count term)."""
    rng = np.random.default_rng(6)
    sh = shape_of("olmoe", 256)
    cfgs = ramp.configs(sh)
    n = len(cfgs)
    nt = np.array([ramp.config_ntiles(sh, c) for c in cfgs])
    wc = np.array([ramp.config_wave_capacity(c) for c in cfgs])
    bm = [c.bm for c in cfgs]
    hists = [synth.histogram_subset(int(T), sh.k, sh.E, b, seed=i) for i, (T, b) in
             enumerate((T, b) for T in (1, 8, 45, 300, 2000) for b in (1.0, 0.7, 0.4, 0.25, 0.12))]
    g = np.array([[oracle.grid(h, bm[c], int(nt[c])) for h in hists] for c in range(n)], np.int64)
    act = np.array([int((h > 0).sum()) for h in hists])
    P = np.array([int(h.sum()) for h in hists], np.int64)
    u = nt[:, None] * act[None, :]
    t = 9 + 6 * np.maximum(g / wc[:, None], 1) + 0.3 * u + 2e-3 * P[None, :] + rng.normal(0, 0.2, g.shape)
    flags = ramp.CM_RELATIVE | ramp.CM_DISTINCT_TILES | ramp.CM_WAVE_FLOOR | ramp.CM_PAIRS
    theta = ramp.cost_model_fit(wc, g, t, distinct=u, pairs=P, flags=flags)
    for c in range(0, n, 3):
        th_o, used = oracle.fit_cost_model(g[c], t[c], int(wc[c]), distinct=u[c], relative=True, wave_floor=True, pairs=P)
        X = oracle.design_matrix(g[c], int(wc[c]), u[c], wave_floor=True, pairs=P)
        po, pl = X @ th_o, X @ theta[c].astype(np.float64)
        assert used and np.abs(po - pl).max() <= 5e-5 * np.abs(po).max()
    for h in hists[::3]:
        best, pred = ramp.cost_model_select(sh.E, cfgs, nt, wc, theta, h, want_pred=True, flags=flags)
        b_o, p_o = oracle.select(bm, nt, wc, theta, h, distinct_tiles=True, wave_floor=True, pairs_term=True)
        assert best == b_o and (pred == p_o).all()
    with pytest.raises(ramp.RampError):
        ramp.cost_model_fit(wc, g, t, distinct=u, pairs=None, flags=flags)   # pair counts required
    with pytest.raises(ramp.RampError):
        ramp.cost_model_fit(wc, g, t, distinct=u, pairs=P, flags=flags | 64)  # unknown flag


def test_config_rounds_and_the_rounds_model_against_the_oracle():
    """ramp_config_rounds by hand (a persistent launch hands out 8 * group_m M-tiles per round, group_m = 32 / N-tiles
    clamped to 1..8 or the GROUP_M mode; every other kernel one M-tile), ramp_grid's g_r and the fit / select entry
    points with RAMP_CM_ROUNDS against the oracle."""
    sh = shape_of("dsv3", 8192)
    by_key = {c.key(): c for c in ramp.configs(sh)}
    assert list(ramp.config_rounds(sh, by_key[(256, 256, 32, 8, 4, 1025)])) == [16, 16, 8, 28]     # 32/16 = 2, 32/28 -> 1
    assert list(ramp.config_rounds(sh, by_key[(272, 256, 32, 8, 4, 1025)])) == [16, 16, 8, 28]
    assert list(ramp.config_rounds(sh, by_key[(256, 128, 32, 8, 4, 1027)])) == [8, 32, 8, 56]
    assert list(ramp.config_rounds(sh, ramp.Config(256, 256, 32, 8, 4, 9217))) == [32, 16, 32, 28]   # GROUP_M 4
    assert list(ramp.config_rounds(sh, ramp.Config(256, 256, 32, 8, 4, 13313))) == [64, 16, 64, 28]  # GROUP_M 8
    assert list(ramp.config_rounds(sh, by_key[(256, 256, 32, 8, 4, 1)])) == [1, 16, 1, 28]           # not persistent
    q = shape_of("qwen3", 8192)
    assert list(ramp.config_rounds(q, ramp.Config(256, 256, 32, 8, 4, 1025))) == [40, 6, 32, 8]      # 32/6 = 5, 32/8 = 4
    o = shape_of("olmoe", 4096)
    assert list(ramp.config_rounds(o, ramp.Config(128, 256, 32, 8, 4, 1025))) == [32, 8, 32, 8]
    with pytest.raises(ramp.RampError):
        ramp.config_rounds(sh, ramp.Config(256, 0, 32, 8, 4, 1025))
    for name, T, beta in (("qwen3", 2048, 0.3), ("dsv3", 8192, 1.0), ("olmoe", 64, 0.2)):
        s = synth.SHAPES[name]
        rs = shape_of(name, T)
        cfgs = ramp.configs(rs)
        n = len(cfgs)
        nt = np.array([ramp.config_ntiles(rs, c) for c in cfgs], np.int32)
        wc = np.array([ramp.config_wave_capacity(c) for c in cfgs], np.int32)
        rounds = np.stack([ramp.config_rounds(rs, c) for c in cfgs])
        assert np.array_equal(rounds[:, 1] + rounds[:, 3], nt)
        rng = np.random.default_rng(T)
        hists = [np.bincount(synth.routing(T, s, beta, seed=i)[0].reshape(-1), minlength=s.E).astype(np.int32) for i in range(12)]
        g = np.stack([ramp.grid(s.E, cfgs, nt, h)[0] for h in hists], 1)
        gr = np.stack([ramp.grid(s.E, cfgs, nt, h, rounds=rounds)[3] for h in hists], 1)
        u = np.stack([ramp.grid(s.E, cfgs, nt, h)[1] for h in hists], 1)
        P = np.array([int(h.sum()) for h in hists], np.int64)
        for i, c in enumerate(cfgs):
            for j, h in enumerate(hists):
                assert gr[i, j] == oracle.grid_rounds(h, c.bm, rounds[i])
            if not c.mode & 0x400:
                assert np.array_equal(gr[i], g[i])
        t = 20.0 + 3.0 * gr / wc[:, None] + 0.01 * u + 1e-3 * P[None, :] * rng.uniform(0.9, 1.1, (n, len(hists)))
        flags = ramp.CM_RELATIVE | ramp.CM_DISTINCT_TILES | ramp.CM_WAVE_FLOOR | ramp.CM_PAIRS | ramp.CM_ROUNDS
        theta = ramp.cost_model_fit(wc, g, t, distinct=u, pairs=P, flags=flags, grid_rounds=gr)
        for i in range(n):
            th_o, _ = oracle.fit_cost_model(g[i], t[i], int(wc[i]), distinct=u[i], relative=True, wave_floor=True, pairs=P,
                                            wave_grid=gr[i])
            X = oracle.design_matrix(g[i], int(wc[i]), u[i], True, P, gr[i])
            assert np.allclose(X @ theta[i].astype(np.float64), X @ th_o, rtol=2e-5)
        for h in hists[:4]:
            best, pred = ramp.cost_model_select(s.E, cfgs, nt, wc, theta, h, want_pred=True, flags=flags, rounds=rounds)
            b_o, p_o = oracle.select_rounds([c.bm for c in cfgs], nt, wc, theta, h, rounds, distinct_tiles=True,
                                            wave_floor=True, pairs_term=True)
            assert best == b_o and np.array_equal(pred, p_o)
        with pytest.raises(ramp.RampError):
            ramp.cost_model_fit(wc, g, t, distinct=u, pairs=P, flags=flags)                  # g_r required with the flag
        with pytest.raises(ramp.RampError):
            ramp.cost_model_select(s.E, cfgs, nt, wc, theta, hists[0], flags=flags)         # and the rounds in the selection


def test_select_table_layout_and_host_polling():
    """Host pieces of the device-resident dispatch: the table image follows the documented layout and the
    poll / wait calls read a result block without touching the GPU."""
    sh = shape_of("olmoe", 256)
    cfgs = ramp.configs(sh)
    n = len(cfgs)
    nt = np.array([ramp.config_ntiles(sh, c) for c in cfgs], np.int32)
    wc = np.array([ramp.config_wave_capacity(c) for c in cfgs], np.int32)
    theta = np.arange(4 * n, dtype=np.float32).reshape(n, 4)
    rounds = np.stack([ramp.config_rounds(sh, c) for c in cfgs])
    table = ramp.select_table_build(cfgs, nt, wc, theta, flags=26, rounds=rounds)
    assert table.nbytes == 128 + 48 * n == ramp.lib().ramp_select_table_bytes(n)
    hdr = table[:128].view(np.int32)
    assert hdr[1] == n and hdr[3] == 26
    bms = list(hdr[4:4 + hdr[2]])
    assert sorted(bms) == sorted({c.bm for c in cfgs}) and len(set(bms)) == len(bms)
    rows = table[128:].reshape(n, 48)
    ints = rows[:, :16].copy().view(np.int32).reshape(n, 4)
    assert [bms[i] for i in ints[:, 0]] == [c.bm for c in cfgs]
    assert np.array_equal(ints[:, 1], nt) and np.array_equal(ints[:, 2], wc)
    assert np.array_equal(rows[:, 16:32].copy().view(np.float32).reshape(n, 4), theta)
    assert np.array_equal(rows[:, 32:].copy().view(np.int32).reshape(n, 4), rounds)
    # without rounds the rows say "one M-tile per round" (the plain grid)
    plain = ramp.select_table_build(cfgs, nt, wc, theta, flags=10)[128:].reshape(n, 48)[:, 32:].copy().view(np.int32).reshape(n, 4)
    assert (plain[:, 0] == 1).all() and (plain[:, 2] == 1).all() and np.array_equal(plain[:, 1], nt)
    with pytest.raises(ramp.RampError):
        ramp.select_table_build(cfgs, nt, np.zeros(n, np.int32), theta)   # wave capacity must be positive
    with pytest.raises(ramp.RampError):
        ramp.select_table_build(cfgs, nt, wc, theta, flags=16)            # the rounds flag needs the rounds
    # result block: word (best << 32 | ticket) | n_cfg | 0 | pred | counts
    nbytes = ramp.select_result_bytes(sh.E, n)
    assert nbytes >= 16 + 8 * n + 4 * sh.E and nbytes % 64 == 0
    import ctypes
    block = np.zeros(nbytes, np.uint8)
    best = ctypes.c_int(-1)
    L = ramp.lib()
    assert L.ramp_select_poll(block.ctypes.data, 5, ctypes.byref(best)) == 1      # not there yet
    assert L.ramp_select_wait(block.ctypes.data, 5, 0.05, ctypes.byref(best)) == ramp.EHIP   # bounded wait
    block[:8] = np.array([(23 << 32) | 5], np.uint64).view(np.uint8)
    assert L.ramp_select_poll(block.ctypes.data, 5, ctypes.byref(best)) == 0 and best.value == 23
    assert L.ramp_select_wait(block.ctypes.data, 5, 0.05, ctypes.byref(best)) == 0 and best.value == 23


def test_region_classify_matches_oracle_and_tab3():
    """Eq. 2-5 / Tab. 2 calculators of the library against the oracle's (which are pinned to Tab. 3), with the
    paper's H200 thresholds; Tab. 3's region letters and GROUP_M predictions (Sec. 4.1) come out."""
    import os
    golden = os.path.join(os.path.dirname(__file__), "golden", "tab3_regions.txt")
    rows = [l.split() for l in open(golden) if l.strip() and not l.startswith("#")]
    h200 = ramp.RegionThresholds(186.0, 45.0 * 2 ** 20, 1, 132, 48.0, 0.2)
    letters = dict(olmoe="A", qwen3="A", dsv3_ep8="A", mixtral="B", dsv3_tp8="A", phi_moe="B", jamba="B", dbrx="B")
    for model, N, K, rho, lam, kap in rows:
        N, K = int(N), int(K)
        sh = ramp.Shape(64, 2, 8, K, N // 2)
        cfg = ramp.Config(64, 256, 128, 4, 3, 0)
        for grid in (20, 131, 133, 1200):
            r = ramp.region_classify(sh, cfg, grid, h200)
            assert r.rho == oracle.rho(N, K, 256, 128) == float(rho)
            assert r.lam == oracle.lam(N, 256) == int(lam)
            assert r.kappa == oracle.kappa(K, 128) == float(kap)
            assert r.omega == oracle.omega(grid, 132)
            assert r.group_m_threshold == oracle.group_m_threshold(45.0 * 2 ** 20, 256, 128, 1) == 1440.0
            assert r.name[0] == letters[model]
            assert r.name[1] == ("1" if grid < 132 else "2" if grid <= 8 * 132 else "3")
            assert bool(r.group_m) == (letters[model] == "B")          # Sec. 4.1: holds for all 8 models
            assert bool(r.split_k) == (float(kap) >= 48 and grid / 132 < 0.2)
            assert bool(r.wide_tile) == (grid > 132)
    # this chip's defaults: 256 units, bf16 elements, 3 MB of one XCD's L2
    sh = shape_of("mixtral", 64)
    cfg = ramp.configs(sh)[0]
    r = ramp.region_classify(sh, cfg, 512)
    assert r.omega == 2.0 and r.group_m_threshold == 3.0 * 2 ** 20 / (cfg.bn * cfg.bk * 2)
    assert r.rho == 2 * sh.I * sh.H / (cfg.bn * cfg.bk)
    with pytest.raises(ramp.RampError):
        ramp.region_classify(sh, cfg, -1)
    with pytest.raises(ramp.RampError):
        ramp.region_classify(sh, cfg, 10, ramp.RegionThresholds(0.0, 1.0, 1, 1, 48.0, 0.2))


def test_bench_refuses_more_than_one_gpu():
    """bench.py is a single-GPU benchmark: --gpus N > 1 (or a multi-rank launch) exits with a message, before
    anything touches a GPU."""
    import os, subprocess, sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    for extra_env, argv in (({}, ["--gpus", "2"]), ({"WORLD_SIZE": "4"}, [])):
        env = dict(os.environ, **extra_env)
        r = subprocess.run([sys.executable, os.path.join(root, "bench.py")] + argv, capture_output=True, text=True, env=env, timeout=60)
        assert r.returncode == 2 and "single-GPU" in r.stderr and r.stdout.strip() == ""


def test_fitted_table_round_trip(tmp_path):
    """tuner.save_model / load_model: the table comes back bit for bit and is refused for another shape or family."""
    from paper_2604_26039_amd import tuner
    fam = tuner.Family.of(synth.SHAPES["olmoe"], 64)
    rng = np.random.default_rng(3)
    theta = rng.uniform(0.01, 50, (len(fam.cfgs), 4)).astype(np.float32)
    path = str(tmp_path / "olmoe.json")
    tuner.save_model(path, fam, theta, tuner.MI355X_MODEL, extra=dict(note="test"))
    got, flags = tuner.load_model(path, fam)
    assert got.dtype == np.float32 and np.array_equal(got, theta) and flags == tuner.MI355X_MODEL
    assert os.path.getsize(path) < 64 * 1024
    with pytest.raises(ValueError):
        tuner.load_model(path, tuner.Family.of(synth.SHAPES["qwen3"], 64))
    other = tuner.Family.of(synth.SHAPES["olmoe"], 64)
    other.cfgs = other.cfgs[1:] + other.cfgs[:1]
    with pytest.raises(ValueError):
        tuner.load_model(path, other)
