"""One-time profiling, cost-model fitting and dispatch on top of the C ABI (paper Sec. 4.2
"Fitting", Sec. 4.4, Sec. 5.1 protocol).

Nothing here computes the layer: it allocates device buffers with torch, calls the library,
times it with HIP events and feeds grids/times to ramp_cost_model_fit / ramp_cost_model_select.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Sequence

import numpy as np
import torch

from . import ramp, synth


def fit_batch_sizes(sweep_T: Sequence[int], n: int = 5) -> List[int]:
    """Profiling batch sizes: n log-spaced values from 1 up to half of the largest benchmark
    batch, so the largest benchmark batch is an extrapolation (Sec. 5.2)."""
    hi = max(4, max(sweep_T) // 2)
    vals = np.unique(np.round(np.geomspace(1, hi, n)).astype(int))
    return [int(v) for v in vals]


FIT_BETAS = [1.0, 0.7, 0.4, 0.25, 0.12]  # none of them is a benchmark skew level


class LayerSet:
    """`n_layers` copies of one synthetic MoE layer (distinct weights at distinct addresses), so a
    timing loop that walks over them reads weights from HBM as a model's layers would, instead
    of re-reading one layer out of the 256 MB last-level cache."""

    def __init__(self, shape: synth.Shape, T_max: int, n_layers: int, seed: int, device="cuda:0", x_std=None,
                 fp8: bool = False, bf16: bool = True):
        """fp8: also keep the W8A8 packed copy of every layer (packed_fp8); bf16=False drops the bf16 packed copies."""
        self.shape, self.T_max, self.device = shape, T_max, device
        self.packed = []
        self.packed_fp8 = []
        self.X = None
        for l in range(n_layers):
            X, Wg, Wu, Wd = synth.layer_tensors(shape, T_max if l == 0 else 1, seed + 7919 * l, device=device, x_std=x_std)
            if l == 0:
                self.X = X
            rs = ramp.Shape(T_max, shape.k, shape.E, shape.H, shape.I)
            if bf16:
                buf = torch.empty(ramp.pack_bytes(rs), dtype=torch.uint8, device=device)
                ramp.pack_weights(rs, Wg, Wu, Wd, buf)
                torch.cuda.synchronize()
                self.packed.append(buf)
            if fp8:
                buf8 = torch.empty(ramp.fp8_pack_bytes(rs), dtype=torch.uint8, device=device)
                ramp.fp8_pack_weights(rs, Wg, Wu, Wd, buf8)
                torch.cuda.synchronize()
                self.packed_fp8.append(buf8)
            if l == 0:
                self.raw0 = (Wg, Wu, Wd)  # kept for oracle checks
            else:
                del Wg, Wu, Wd
        self.n_layers = n_layers
        self._ws = None
        self.out = torch.empty((T_max, shape.H), dtype=torch.bfloat16, device=device)

    def rs(self, T: int) -> ramp.Shape:
        s = self.shape
        return ramp.Shape(T, s.k, s.E, s.H, s.I)

    def workspace(self, nbytes: int) -> torch.Tensor:
        if self._ws is None or self._ws.numel() < nbytes:
            self._ws = None
            self._ws = torch.empty(int(nbytes * 1.25) + 4096, dtype=torch.uint8, device=self.device)
        return self._ws


@dataclass
class Point:
    T: int
    beta: object
    seed: int
    ids: np.ndarray = field(repr=False, default=None)
    w: np.ndarray = field(repr=False, default=None)
    counts: np.ndarray = field(repr=False, default=None)

    def materialise(self, shape: synth.Shape):
        if self.ids is None:
            self.ids, self.w = synth.routing(self.T, shape, self.beta, self.seed)
            self.counts = np.bincount(self.ids.reshape(-1), minlength=shape.E).astype(np.int32)
        return self


def time_config(layers: LayerSet, cfg: ramp.Config, pt: Point, warmup: int = 10, iters: int = 50,
                budget_ms: float = 400.0, hot: bool = False) -> float:
    """Median time in microseconds of ramp_fused_moe(cfg) at one operating point, HIP events
    around each call, walking over the layer copies (Sec. 5.1: 10 warm-up + 50 timed, median).
    The iteration count is cut so one measurement stays within budget_ms.  hot=True re-uses one
    weight copy, so whatever part of the active experts fits the 256 MB last-level cache stays there."""
    pt.materialise(layers.shape)
    T = pt.T
    rs = layers.rs(T)
    dev = layers.device
    d_ids = torch.from_numpy(pt.ids).to(dev)
    d_w = torch.from_numpy(pt.w).to(dev)
    is_fp8 = bool(cfg.mode & ramp.FP8_MODE)
    ws = layers.workspace(ramp.fused_moe_fp8_workspace_bytes(rs, cfg) if is_fp8 else ramp.fused_moe_workspace_bytes(rs, cfg))
    X = layers.X[:T]
    out = layers.out[:T]
    L = 1 if hot else layers.n_layers

    def call(i):
        if is_fp8:
            ramp.fused_moe_fp8(rs, cfg, X, d_ids, d_w, layers.packed_fp8[i % L], out, ws)
        else:
            ramp.fused_moe(rs, cfg, X, d_ids, d_w, layers.packed[i % L], out, ws)

    # one probing call decides how many iterations the budget allows
    call(0)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    call(1)
    e1.record()
    torch.cuda.synchronize()
    one = max(e0.elapsed_time(e1), 1e-3)
    if one * 3 > budget_ms:
        # a call that takes a large share of the budget (a small-tile configuration far outside its regime): the two
        # calls above were the warm-up, three timed calls give the median
        iters, warmup = 3, 0
    else:
        iters = int(max(5, min(iters, budget_ms / one)))
        warmup = int(max(1, min(warmup, iters // 3)))
    for i in range(warmup):
        call(i)
    starts = [torch.cuda.Event(enable_timing=True) for _ in range(iters)]
    stops = [torch.cuda.Event(enable_timing=True) for _ in range(iters)]
    for i in range(iters):
        starts[i].record()
        call(i)
        stops[i].record()
    torch.cuda.synchronize()
    t = np.array([s.elapsed_time(e) for s, e in zip(starts, stops)]) * 1e3
    return float(np.median(t))


@dataclass
class Family:
    shape: ramp.Shape
    cfgs: List[ramp.Config]
    ntiles: np.ndarray
    wave_cap: np.ndarray
    rounds: np.ndarray = None   # int32 [n_cfg, 4]: M-tiles per hand-out round and N-tiles of the two launches

    def __post_init__(self):
        if self.rounds is None:
            self.rounds = np.stack([ramp.config_rounds(self.shape, c) for c in self.cfgs]).astype(np.int32)

    @staticmethod
    def of(s: synth.Shape, T: int = 1, fp8: bool = False) -> "Family":
        """The bf16 tile family of the shape, or (fp8=True) the W8A8 FP8 one."""
        rs = ramp.Shape(T, s.k, s.E, s.H, s.I)
        cfgs = ramp.fp8_configs(rs) if fp8 else ramp.configs(rs)
        cap = ramp.fp8_config_wave_capacity if fp8 else ramp.config_wave_capacity
        return Family(rs, cfgs, np.array([ramp.config_ntiles(rs, c) for c in cfgs], np.int32),
                      np.array([cap(c) for c in cfgs], np.int32))

    def grid(self, counts: np.ndarray) -> np.ndarray:
        """Eq. 1 for every configuration (computed by the library)."""
        return ramp.grid(self.shape.E, self.cfgs, self.ntiles, counts)[0]


def profile(layers: LayerSet, fam: Family, points: Sequence[Point], log=None, **timing) -> tuple:
    """Times every configuration at every point.  Returns (grid [n_cfg,n_pts], time_us [n_cfg,n_pts])."""
    n_cfg, n_pts = len(fam.cfgs), len(points)
    grid = np.zeros((n_cfg, n_pts), np.int64)
    t_us = np.zeros((n_cfg, n_pts), np.float64)
    for j, pt in enumerate(points):
        pt.materialise(layers.shape)
        grid[:, j] = fam.grid(pt.counts)
        for i, cfg in enumerate(fam.cfgs):
            t_us[i, j] = time_config(layers, cfg, pt, **timing)
        if log:
            b = int(np.argmin(t_us[:, j]))
            log(f"  T={pt.T:<5} beta={pt.beta!s:<8} best {t_us[b, j]:9.1f} us  {fam.cfgs[b]}")
    return grid, t_us


# The dispatch model used on this chip: Eq. 6 fitted on relative residuals, with the traffic term on distinct weight
# tiles, a wave term that has a floor of one wave and counts whole hand-out rounds of the persistent kernels, and the
# routed pairs as fourth term.  EQ6 (= 0) is the model exactly as printed.
MI355X_MODEL = ramp.CM_RELATIVE | ramp.CM_DISTINCT_TILES | ramp.CM_WAVE_FLOOR | ramp.CM_PAIRS | ramp.CM_ROUNDS


def grid_rounds(fam: Family, counts_list: Sequence[np.ndarray]) -> np.ndarray:
    """[n_cfg, n_pts]: the g_r of CM_ROUNDS at every point (from the library)."""
    return np.stack([ramp.grid(fam.shape.E, fam.cfgs, fam.ntiles, c, rounds=fam.rounds)[3] for c in counts_list], axis=1)


def distinct_tiles(fam: Family, counts_list: Sequence[np.ndarray]) -> np.ndarray:
    """[n_cfg, n_pts]: active experts x ntiles(c), the distinct weight tiles a point touches (from the library)."""
    return np.stack([ramp.grid(fam.shape.E, fam.cfgs, fam.ntiles, c)[1] for c in counts_list], axis=1)


def fit(fam: Family, grid: np.ndarray, t_us: np.ndarray, counts_list=None, flags: int = ramp.CM_EQ6) -> np.ndarray:
    distinct = distinct_tiles(fam, counts_list) if (flags & ramp.CM_DISTINCT_TILES) else None
    pairs = None
    if flags & ramp.CM_PAIRS:
        pairs = np.array([ramp.grid(fam.shape.E, fam.cfgs, fam.ntiles, c)[2] for c in counts_list], np.int64)
    gr = grid_rounds(fam, counts_list) if (flags & ramp.CM_ROUNDS) else None
    return ramp.cost_model_fit(fam.wave_cap, grid, t_us, distinct=distinct, pairs=pairs, flags=flags, grid_rounds=gr)


def fit5(fam: Family, grid: np.ndarray, t_us: np.ndarray, counts_list=None, flags: int = ramp.CM_EQ6) -> np.ndarray:
    """The five-term ablation of Sec. 5.3 (a fifth column g^2): theta5 [n_cfg, 5]."""
    distinct = distinct_tiles(fam, counts_list) if (flags & ramp.CM_DISTINCT_TILES) else None
    pairs = None
    if flags & ramp.CM_PAIRS:
        pairs = np.array([ramp.grid(fam.shape.E, fam.cfgs, fam.ntiles, c)[2] for c in counts_list], np.int64)
    gr = grid_rounds(fam, counts_list) if (flags & ramp.CM_ROUNDS) else None
    return ramp.cost_model_fit(fam.wave_cap, grid, t_us, distinct=distinct, pairs=pairs, flags=flags, terms=5, grid_rounds=gr)


def select5(fam: Family, theta5: np.ndarray, counts: np.ndarray, flags: int = ramp.CM_EQ6) -> int:
    return ramp.cost_model_select(fam.shape.E, fam.cfgs, fam.ntiles, fam.wave_cap, theta5, counts, flags=flags, terms=5,
                                  rounds=fam.rounds if (flags & ramp.CM_ROUNDS) else None)


def select(fam: Family, theta: np.ndarray, counts: np.ndarray, flags: int = ramp.CM_EQ6) -> int:
    return ramp.cost_model_select(fam.shape.E, fam.cfgs, fam.ntiles, fam.wave_cap, theta, counts, flags=flags,
                                  rounds=fam.rounds if (flags & ramp.CM_ROUNDS) else None)


def save_model(path: str, fam: Family, theta: np.ndarray, flags: int, extra: dict = None) -> None:
    """Writes the fitted table of one shape (Sec. 4.2: four numbers per configuration, a few KB) as JSON, keyed by
    the configuration tuples so that a table is never applied to a different family."""
    import json
    s = fam.shape
    doc = dict(shape=dict(k=s.k, E=s.E, H=s.H, I=s.I), flags=int(flags),
               configs=[list(c.key()) for c in fam.cfgs], ntiles=[int(v) for v in fam.ntiles],
               wave_cap=[int(v) for v in fam.wave_cap],
               theta=[[float(v) for v in row] for row in np.asarray(theta, np.float32).reshape(len(fam.cfgs), 4)])
    if extra:
        doc["info"] = extra
    with open(path, "w") as f:
        json.dump(doc, f)


def load_model(path: str, fam: Family):
    """(theta float32 [n_cfg,4], flags) from save_model's file; raises if it was fitted for another shape,
    family or tile accounting (then the shape has to be profiled again)."""
    import json
    with open(path) as f:
        doc = json.load(f)
    s = fam.shape
    if doc["shape"] != dict(k=s.k, E=s.E, H=s.H, I=s.I):
        raise ValueError(f"{path}: fitted for shape {doc['shape']}, not {dict(k=s.k, E=s.E, H=s.H, I=s.I)}")
    if [tuple(c) for c in doc["configs"]] != [c.key() for c in fam.cfgs]:
        raise ValueError(f"{path}: fitted for a different configuration family")
    if list(doc["ntiles"]) != [int(v) for v in fam.ntiles] or list(doc["wave_cap"]) != [int(v) for v in fam.wave_cap]:
        raise ValueError(f"{path}: tile counts or wave capacities differ from this build's")
    theta = np.asarray(doc["theta"], np.float32).reshape(len(fam.cfgs), 4)
    if not np.isfinite(theta).all():
        raise ValueError(f"{path}: non-finite coefficients")
    return theta, int(doc["flags"])


class Dispatcher:
    """Runtime dispatch (Sec. 4.4).  Three ways to get from the routing of a call to a configuration index:

    select()        device-resident: one enqueue (histogram + model + argmin on the device), the result lands in
                    pinned host memory and the host polls its ticket word.  No copy, no stream synchronisation.
    select_async()  never waits: enqueues the selection for this call's routing and returns the choice of the
                    latest selection that has already finished (the previous call's, in a steady stream of calls
                    of one batch size; the first call waits once).
    select_host()   histogram kernel -> E counts copied to pinned host memory -> stream synchronisation ->
                    ramp_cost_model_select on the host.
    All marshalling is done once here."""

    def __init__(self, fam: Family, theta: np.ndarray, flags: int, T: int, device="cuda:0"):
        import ctypes
        self.fam, self.flags, self.T = fam, flags, T
        s = fam.shape
        self.E, self.k = s.E, s.k
        self.n_cfg = len(fam.cfgs)
        self._cfgs = (ramp.Config * len(fam.cfgs))(*fam.cfgs)
        self._nt = np.ascontiguousarray(fam.ntiles, np.int32)
        self._wc = np.ascontiguousarray(fam.wave_cap, np.int32)
        self._rounds = np.ascontiguousarray(fam.rounds, np.int32)
        self._theta = np.ascontiguousarray(theta, np.float32)
        self.d_counts = torch.zeros(self.E, dtype=torch.int32, device=device)
        self.h_counts = torch.zeros(self.E, dtype=torch.int32).pin_memory()
        self._h_ptr = self.h_counts.data_ptr()
        self.ws = torch.empty(max(256, ramp.align_workspace_bytes(T, s.k, s.E)), dtype=torch.uint8, device=device)
        self._best = ctypes.c_int(-1)
        self._best_ref = ctypes.byref(self._best)
        self._lib = ramp.lib()
        # device-resident path: table on the device, two result blocks in pinned host memory used in turn
        self.table = torch.from_numpy(ramp.select_table_build(fam.cfgs, fam.ntiles, fam.wave_cap, theta, flags, rounds=fam.rounds)).to(device)
        nbytes = ramp.select_result_bytes(self.E, self.n_cfg)
        self.results = [torch.zeros(nbytes, dtype=torch.uint8).pin_memory() for _ in range(2)]
        self._res_ptr = [r.data_ptr() for r in self.results]
        self._table_ptr, self._ws_ptr, self._ws_bytes = self.table.data_ptr(), self.ws.data_ptr(), self.ws.numel()
        self.ticket = 0
        self.cached = None

    def _enqueue(self, d_ids: torch.Tensor) -> int:
        self.ticket = self.ticket % 0xFFFFFFFF + 1  # 1 .. 2^32-1; 0 is what an unused result block holds
        rc = self._lib.ramp_select_device(d_ids.data_ptr(), self.T, self.k, self.E, self.n_cfg, self._table_ptr,
                                          self._res_ptr[self.ticket & 1], self.ticket, None, self._ws_ptr,
                                          self._ws_bytes, torch.cuda.current_stream().cuda_stream)
        if rc != ramp.OK:
            raise ramp.RampError(rc, ramp.last_error())
        return self.ticket

    def select(self, d_ids: torch.Tensor) -> int:
        t = self._enqueue(d_ids)
        rc = self._lib.ramp_select_wait(self._res_ptr[t & 1], t, 10.0, self._best_ref)
        if rc != ramp.OK:
            raise ramp.RampError(rc, ramp.last_error())
        self.cached = self._best.value
        return self.cached

    def select_async(self, d_ids: torch.Tensor) -> int:
        prev = self.ticket
        if prev and self._lib.ramp_select_poll(self._res_ptr[prev & 1], prev, self._best_ref) == 0:
            self.cached = self._best.value
        t = self._enqueue(d_ids)
        if self.cached is None:  # nothing has finished yet (first call): wait once
            rc = self._lib.ramp_select_wait(self._res_ptr[t & 1], t, 10.0, self._best_ref)
            if rc != ramp.OK:
                raise ramp.RampError(rc, ramp.last_error())
            self.cached = self._best.value
        return self.cached

    def begin_step(self):
        """Per-step cache (Sec. 4.4): the first select_step() of a step dispatches on its own routing, the later
        layers of the step reuse that choice (this dispatcher serves one batch size, the cache key of the paper)."""
        self._step_choice = None

    def select_step(self, d_ids: torch.Tensor) -> int:
        if getattr(self, "_step_choice", None) is None:
            self._step_choice = self.select(d_ids)
        return self._step_choice

    def last_counts(self) -> np.ndarray:
        """Expert histogram of the latest finished selection (from its result block)."""
        t = self.ticket
        return ramp.select_result_unpack(self.results[t & 1], self.E, self.n_cfg)[3]

    def select_host(self, d_ids: torch.Tensor) -> int:
        stream = torch.cuda.current_stream()
        ramp.moe_histogram(d_ids, self.T, self.k, self.E, self.d_counts, self.ws, stream)
        self.h_counts.copy_(self.d_counts, non_blocking=True)
        stream.synchronize()  # this path's one host sync
        rc = self._lib.ramp_cost_model_select_rounds(self.E, len(self.fam.cfgs), self._cfgs, self._nt.ctypes.data,
                                                     self._rounds.ctypes.data, self._wc.ctypes.data, self._theta.ctypes.data,
                                                     self._h_ptr, self.flags, 4, self._best_ref, None)
        if rc != ramp.OK:
            raise ramp.RampError(rc, ramp.last_error())
        return self._best.value


def entropy_beta(counts) -> float:
    """The paper's balancedness (Sec. 2.1), reported next to the subset fraction."""
    c = np.asarray(counts, np.float64)
    tot = c.sum()
    if tot <= 0 or c.size <= 1:
        return 1.0
    p = c[c > 0] / tot
    return float(-(p * np.log(p)).sum() / math.log(c.size))


def roofline_lower_bound_us(s: synth.Shape, T: int, counts: np.ndarray, hbm_tbs: float = 8.0,
                            mfma_pflops: float = 2.5, weight_bytes: int = 2):
    """Algorithmic minimum time: weights of the active experts once + activations in/out + routing,
    against HBM peak; 6*P*H*I flops against the dense MFMA peak of the operand type (bf16 2.5, FP8 5.0 PFLOP/s;
    weight_bytes 2 or 1).  Returns (t_hbm, t_mfma, bytes, flops)."""
    e_act = int((np.asarray(counts) > 0).sum())
    P = int(np.asarray(counts).sum())
    nbytes = e_act * 3 * s.H * s.I * weight_bytes + 2 * T * s.H * 2 + P * 8
    flops = 6.0 * P * s.H * s.I
    return nbytes / (hbm_tbs * 1e12) * 1e6, flops / (mfma_pflops * 1e15) * 1e6, nbytes, flops
