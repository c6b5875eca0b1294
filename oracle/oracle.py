"""CPU oracle for the routing-aware fused MoE layer (RaMP, arxiv 2604.26039).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's
cpu_baseline leg are the only callers.  Nothing here touches the GPU library
and the GPU library never imports this module.

The slow loops live in ramp_oracle.c (plain C, fp64); this file binds them
with ctypes and adds the parts that are a few lines of numpy:

  fit_cost_model      least-squares fit of Eq. 6 per configuration
                      (Sec. 4.2 "Fitting", adaptive log term)
  regret, static_choice, geomean_speedup
                      the evaluation quantities of Sec. 5.1-5.3
  padding_waste, balancedness, rho/lambda/kappa/omega
                      Fig. 1, Sec. 2.1 and Eq. 2-5 helpers

Readings of the paper that the text leaves open (all listed in the design
notes): Eq. 6's columns g/SM and g are proportional, so the fit is the
minimum-norm least-squares solution and only predictions are compared; log is
the natural log; the median of an even number of grids is the lower one;
regret is (t_selected - t_best)/t_best.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ramp_oracle.c")
_LIB = os.path.join(_HERE, "libramp_oracle.so")


def build(force: bool = False) -> str:
    """Compile ramp_oracle.c with gcc (-O2, OpenMP) into libramp_oracle.so."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp",
               "-ffp-contract=off", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i32p = ctypes.POINTER(ctypes.c_int32)
        u16p = ctypes.POINTER(ctypes.c_uint16)
        u16pp = ctypes.POINTER(u16p)
        f32p = ctypes.POINTER(ctypes.c_float)
        f64p = ctypes.POINTER(ctypes.c_double)
        lib.oracle_align_capacity.restype = ctypes.c_int64
        lib.oracle_align_capacity.argtypes = [ctypes.c_int] * 4
        lib.oracle_align.restype = ctypes.c_int
        lib.oracle_align.argtypes = [i32p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                     i32p, i32p, i32p, i32p]
        lib.oracle_grid.restype = ctypes.c_int64
        lib.oracle_grid.argtypes = [i32p, ctypes.c_int, ctypes.c_int, ctypes.c_int]
        lib.oracle_moe.restype = ctypes.c_int
        lib.oracle_moe.argtypes = [u16p, i32p, f32p, u16pp, u16pp, u16pp,
                                   ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                   i32p, ctypes.c_int, ctypes.c_int, f64p]
        lib.oracle_predict.restype = ctypes.c_double
        lib.oracle_predict.argtypes = [f32p, ctypes.c_int64, ctypes.c_int]
        lib.oracle_select.restype = ctypes.c_int
        lib.oracle_select.argtypes = [ctypes.c_int, i32p, i32p, i32p, f32p, i32p, ctypes.c_int, ctypes.c_int, f64p]
        lib.oracle_f64_to_bf16.restype = ctypes.c_uint16
        lib.oracle_f64_to_bf16.argtypes = [ctypes.c_double]
        lib.oracle_bf16_to_f64.restype = ctypes.c_double
        lib.oracle_bf16_to_f64.argtypes = [ctypes.c_uint16]
        _lib = lib
    return _lib


def _ptr(a: np.ndarray, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


# --------------------------------------------------------------------------- bf16

def f64_to_bf16_bits(x: float) -> int:
    return int(_load().oracle_f64_to_bf16(float(x)))


def bf16_bits_to_f64(b: int) -> float:
    return float(_load().oracle_bf16_to_f64(int(b)))


# --------------------------------------------------------------------------- align

def align_capacity(T: int, k: int, E: int, bm: int) -> int:
    return int(_load().oracle_align_capacity(T, k, E, bm))


def align(ids, T: int, k: int, E: int, bm: int):
    """Eq. 1 first factor / Fig. 1: returns (sorted, tile_expert, counts, meta)."""
    ids = _i32(ids).reshape(-1)
    assert ids.size == T * k
    cap = align_capacity(T, k, E, bm)
    sorted_ids = np.empty(cap, np.int32)
    tile_expert = np.empty(cap // bm, np.int32)
    counts = np.empty(E, np.int32)
    meta = np.empty(4, np.int32)
    rc = _load().oracle_align(_ptr(ids, ctypes.c_int32), T, k, E, bm,
                              _ptr(sorted_ids, ctypes.c_int32), _ptr(tile_expert, ctypes.c_int32),
                              _ptr(counts, ctypes.c_int32), _ptr(meta, ctypes.c_int32))
    if rc != 0:
        raise ValueError(f"oracle_align failed: {rc}")
    return sorted_ids, tile_expert, counts, meta


def grid(counts, bm: int, ntiles: int) -> int:
    """Eq. 1: (sum_e ceil(n_e/bm)) * ntiles."""
    c = _i32(counts)
    return int(_load().oracle_grid(_ptr(c, ctypes.c_int32), c.size, bm, ntiles))


def padding_waste(counts, bm: int):
    """Fig. 1: padded slots that hold no pair.  Returns (absolute, fraction of padded slots)."""
    c = np.asarray(counts, dtype=np.int64)
    padded = (-(-c // bm)) * bm
    waste = int((padded - c).sum())
    total = int(padded.sum())
    return waste, (waste / total if total else 0.0)


def balancedness(counts) -> float:
    """Sec. 2.1: entropy of the expert histogram divided by ln E."""
    c = np.asarray(counts, dtype=np.float64)
    E = c.size
    tot = c.sum()
    if tot <= 0 or E <= 1:
        return 1.0
    p = c[c > 0] / tot
    return float(-(p * np.log(p)).sum() / math.log(E))


# --------------------------------------------------------------------------- MoE layer

def _expert_ptrs(W, E: int, shape):
    """W: array [E, a, b] of uint16, or dict {e: array [a, b]}.  Returns (ctypes array, keepalive)."""
    u16p = ctypes.POINTER(ctypes.c_uint16)
    arr = (u16p * E)()
    keep = []
    for e in range(E):
        if isinstance(W, dict):
            w = W.get(e)
        else:
            w = W[e]
        if w is None:
            arr[e] = ctypes.cast(None, u16p)
            continue
        w = np.ascontiguousarray(w, dtype=np.uint16)
        assert w.shape == shape, (w.shape, shape)
        keep.append(w)
        arr[e] = _ptr(w, ctypes.c_uint16)
    return arr, keep


def moe(X, ids, w, Wg, Wu, Wd, E: int, rows=None, round_mid: bool = False) -> np.ndarray:
    """Sec. 2.2 by definition, fp64.

    X [T,H] uint16 (bf16 bits); ids [T,k] int32; w [T,k] float32;
    Wg, Wu [E,H,I] and Wd [E,I,H] uint16, each either a full array or a dict
    {expert: matrix} holding only the experts the evaluated rows use.
    Returns fp64 [len(rows) or T, H].
    """
    X = np.ascontiguousarray(X, dtype=np.uint16)
    T, H = X.shape
    ids = _i32(ids).reshape(T, -1)
    k = ids.shape[1]
    w = np.ascontiguousarray(w, dtype=np.float32).reshape(T, k)
    if isinstance(Wg, dict):
        I = next(iter(Wg.values())).shape[1]
    else:
        I = Wg.shape[2]
    pg, kg = _expert_ptrs(Wg, E, (H, I))
    pu, ku = _expert_ptrs(Wu, E, (H, I))
    pd, kd = _expert_ptrs(Wd, E, (I, H))
    if rows is None:
        n_rows, rows_p = T, ctypes.cast(None, ctypes.POINTER(ctypes.c_int32))
        rows_a = None
    else:
        rows_a = _i32(rows)
        n_rows, rows_p = rows_a.size, _ptr(rows_a, ctypes.c_int32)
    out = np.empty((n_rows, H), np.float64)
    rc = _load().oracle_moe(_ptr(X, ctypes.c_uint16), _ptr(ids, ctypes.c_int32), _ptr(w, ctypes.c_float),
                            pg, pu, pd, T, k, E, H, I, rows_p, n_rows, int(round_mid),
                            _ptr(out, ctypes.c_double))
    if rc != 0:
        raise ValueError(f"oracle_moe failed: {rc}")
    del kg, ku, kd, rows_a
    return out


# --------------------------------------------------------------------------- Eq. 6

def predict(theta4, g: int, wave_cap: int) -> float:
    th = np.ascontiguousarray(theta4, dtype=np.float32)
    return float(_load().oracle_predict(_ptr(th, ctypes.c_float), int(g), int(wave_cap)))


def select(bm, ntiles, wave_cap, theta, counts, distinct_tiles: bool = False, wave_floor: bool = False,
           pairs_term: bool = False):
    """Evaluate the cost model for all configs on one histogram.  Returns (argmin, predictions).
    Default: Eq. 6 as printed.  distinct_tiles: the traffic term uses (#active experts * ntiles)
    instead of g; wave_floor: the wave term is max(g/W, 1); pairs_term: the fourth term is the number
    of routed pairs instead of ln(g+1)."""
    bm, ntiles, wave_cap, counts = _i32(bm), _i32(ntiles), _i32(wave_cap), _i32(counts)
    theta = np.ascontiguousarray(theta, dtype=np.float32).reshape(-1, 4)
    n = bm.size
    assert ntiles.size == n and wave_cap.size == n and theta.shape[0] == n
    pred = np.empty(n, np.float64)
    options = (1 if distinct_tiles else 0) | (2 if wave_floor else 0) | (4 if pairs_term else 0)
    best = _load().oracle_select(n, _ptr(bm, ctypes.c_int32), _ptr(ntiles, ctypes.c_int32),
                                 _ptr(wave_cap, ctypes.c_int32), _ptr(theta, ctypes.c_float),
                                 _ptr(counts, ctypes.c_int32), counts.size, options,
                                 _ptr(pred, ctypes.c_double))
    return int(best), pred


def grid_rounds(counts, bm: int, rounds4) -> int:
    """The g_r of the "rounds" departure from Eq. 6: for each of the two launches (R, ntiles) of a configuration,
    its M-tiles (first factor of Eq. 1) rounded up to a whole number of hand-out rounds of R M-tiles, times the
    N-tiles of that launch.  R = 1 in both launches gives back Eq. 1."""
    m_tiles = sum((int(n) + bm - 1) // bm for n in counts if int(n) > 0)
    r_up, nt_up, r_down, nt_down = (int(v) for v in rounds4)
    return (-(-m_tiles // r_up)) * r_up * nt_up + (-(-m_tiles // r_down)) * r_down * nt_down


def design_matrix(g, wave_cap: int, distinct=None, wave_floor: bool = False, pairs=None, wave_grid=None) -> np.ndarray:
    """Rows [1, w, m, l].  As printed (Eq. 6): w = g/W, m = g, l = ln(g+1).  distinct: m = the
    distinct-weight-tile count; wave_floor: w = max(g/W, 1); pairs: l = routed pairs of each point;
    wave_grid: the wave term alone counts these grids (grid_rounds) instead of g."""
    g = np.asarray(g, dtype=np.float64)
    m = g if distinct is None else np.asarray(distinct, dtype=np.float64)
    w = (g if wave_grid is None else np.asarray(wave_grid, dtype=np.float64)) / float(wave_cap)
    if wave_floor:
        w = np.maximum(w, 1.0)
    last = np.log(g + 1.0) if pairs is None else np.asarray(pairs, dtype=np.float64)
    return np.stack([np.ones_like(g), w, m, last], axis=1)


def lower_median(v) -> float:
    s = np.sort(np.asarray(v, dtype=np.float64))
    return float(s[(s.size - 1) // 2])


def fit_cost_model(g, t_us, wave_cap: int, n_terms: int = 4, distinct=None, relative: bool = False,
                   wave_floor: bool = False, pairs=None, wave_grid=None):
    """Sec. 4.2 "Fitting" for ONE configuration.

    distinct / relative / wave_floor / pairs are the documented departures from the printed recipe
    that the GPU library also offers: the traffic column holds the number of distinct weight tiles
    instead of g, the residuals are relative (every row divided by its measured time), the wave
    column is max(g/W, 1), the fourth column is the routed-pair count (then always fitted)
    instead of the logarithm, and (wave_grid) the wave column counts whole hand-out rounds (grid_rounds).

    g: profiling grids, t_us: measured times.  The log column is used only if
    the (lower) median profiling grid is below wave_cap.  Solves the literal
    four-column system in the minimum-norm least-squares sense.
    n_terms = 2 / 3 reproduce the ablation rows (a + k*g; a + b*g/W + c*g); n_terms = 5 adds the fifth
    term of Sec. 5.3 (g^2, here (g/W)^2: the same column up to the configuration's constant W^2) and
    returns theta[5].
    Returns (theta as float64, use_log).
    """
    g = np.asarray(g, dtype=np.float64)
    t = np.asarray(t_us, dtype=np.float64)
    X = design_matrix(g, wave_cap, distinct, wave_floor, pairs, wave_grid)
    use_log = (n_terms >= 4) and (pairs is not None or lower_median(g) < wave_cap)
    cols = [0, 1, 2] + ([3] if use_log else [])
    if n_terms == 2:
        cols = [0, 2]
    if n_terms == 5:
        X = np.concatenate([X, ((g / float(wave_cap)) ** 2)[:, None]], axis=1)
        cols = cols + [4]
    A, rhs = X[:, cols], t
    if relative:
        A, rhs = A / t[:, None], np.ones_like(t)
    sol = np.linalg.lstsq(A, rhs, rcond=None)[0]
    theta = np.zeros(5 if n_terms == 5 else 4, np.float64)
    theta[cols] = sol
    return theta, use_log


def select_rounds(bm, ntiles, wave_cap, theta, counts, rounds, distinct_tiles: bool = False, wave_floor: bool = False,
                  pairs_term: bool = False):
    """select() with the wave term on grid_rounds (rounds: [n_cfg, 4]); plain fp64, one configuration at a time.
    Returns (lowest index with the smallest prediction, predictions)."""
    counts = [int(n) for n in counts]
    active, pairs = sum(1 for n in counts if n > 0), sum(n for n in counts if n > 0)
    theta = np.asarray(theta, dtype=np.float32).reshape(-1, 4).astype(np.float64)
    pred = np.empty(len(bm), np.float64)
    for c in range(len(bm)):
        g = grid(counts, int(bm[c]), int(ntiles[c]))
        x = design_matrix([g], int(wave_cap[c]), [active * int(ntiles[c])] if distinct_tiles else None, wave_floor,
                          [pairs] if pairs_term else None, [grid_rounds(counts, int(bm[c]), rounds[c])])[0]
        t = float(theta[c][0]) * float(x[0])
        for j in (1, 2, 3):     # term by term, in the order the model is written
            t = t + float(theta[c][j]) * float(x[j])
        pred[c] = t
    return int(np.argmin(pred)), pred


def predict5(theta5, g: int, wave_cap: int, distinct=None, wave_floor: bool = False, pairs=None) -> float:
    """Five-term model of Sec. 5.3 on one grid: the row of design_matrix plus (g/W)^2, times theta5."""
    x = design_matrix([g], wave_cap, None if distinct is None else [distinct], wave_floor, None if pairs is None else [pairs])[0]
    th = np.asarray(theta5, np.float64)
    return float(x @ th[:4] + th[4] * (float(g) / float(wave_cap)) ** 2)


def regret(t_meas_row, chosen: int) -> float:
    """(t_selected - t_best) / t_best over one operating point's measured times."""
    t = np.asarray(t_meas_row, dtype=np.float64)
    return float(t[chosen] / t.min() - 1.0)


def static_choice(t_meas_uniform_row) -> int:
    """Static dispatch: the configuration that is fastest under uniform routing at this batch size."""
    return int(np.argmin(np.asarray(t_meas_uniform_row, dtype=np.float64)))


def geomean_speedup(t_static, t_ra) -> float:
    r = np.asarray(t_static, dtype=np.float64) / np.asarray(t_ra, dtype=np.float64)
    return float(np.exp(np.log(r).mean()))


# --------------------------------------------------------------------------- Eq. 2-5

def rho(N: int, K: int, ttn: int, tile_k: int) -> float:
    """Eq. 2: MMA tile operations per block."""
    return N * K / (ttn * tile_k)


def lam(N: int, ttn: int) -> int:
    """Eq. 3: number of N-tiles."""
    return -(-N // ttn)


def kappa(K: int, tile_k: int) -> float:
    """Eq. 3: K-loop depth."""
    return K / tile_k


def omega(grid_size: int, n_units: int) -> float:
    """Eq. 5: grid over the number of compute units."""
    return grid_size / n_units


def group_m_threshold(l2_eff_bytes: float, ttn: int, tile_k: int, elem_bytes: int) -> float:
    """Eq. 4 right-hand side."""
    return l2_eff_bytes / (ttn * tile_k * elem_bytes)
