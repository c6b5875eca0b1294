"""Thin ctypes binding of libramp.so: argument marshalling only.

Every function has the name of the C entry point it wraps (include/ramp.h) minus the
`ramp_` prefix.  Device buffers are torch tensors (torch is used for device memory and
streams only); all arithmetic of the path runs in the library's HIP kernels.  There is no
CPU fallback: if the library is missing the first call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np
import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libramp.so")

OK, EINVAL, ENOSPC, EUNSUPPORTED, EHIP = 0, -1, -2, -3, -4
CM_EQ6, CM_RELATIVE, CM_DISTINCT_TILES, CM_WAVE_FLOOR, CM_PAIRS, CM_ROUNDS = 0, 1, 2, 4, 8, 16


class Shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("T", "k", "E", "H", "I")]

    def __repr__(self):
        return f"Shape(T={self.T}, k={self.k}, E={self.E}, H={self.H}, I={self.I})"


class Config(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("bm", "bn", "bk", "waves", "stages", "mode")]

    def key(self):
        return (self.bm, self.bn, self.bk, self.waves, self.stages, self.mode)

    def __repr__(self):
        return f"Config(bm={self.bm}, bn={self.bn}, bk={self.bk}, waves={self.waves}, stages={self.stages}, mode={self.mode})"


class RegionThresholds(ctypes.Structure):
    _fields_ = [("rho_c", ctypes.c_double), ("l2_eff_bytes", ctypes.c_double), ("elem_bytes", ctypes.c_int32),
                ("units", ctypes.c_int32), ("split_k_kappa", ctypes.c_double), ("split_k_omega", ctypes.c_double)]


class Region(ctypes.Structure):
    _fields_ = [("rho", ctypes.c_double), ("lam", ctypes.c_double), ("kappa", ctypes.c_double),
                ("omega", ctypes.c_double), ("group_m_threshold", ctypes.c_double), ("region", ctypes.c_int32),
                ("group_m", ctypes.c_int32), ("split_k", ctypes.c_int32), ("wide_tile", ctypes.c_int32)]

    NAMES = ("A1", "A2", "A3", "B1", "B2", "B3")

    @property
    def name(self):
        return self.NAMES[self.region]


class RampError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"ramp status {status}: {msg}")
        self.status = status


_lib = None


def lib() -> ctypes.CDLL:
    """Load libramp.so (built by `python -m paper_2604_26039_amd.build`); raise if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2604_26039_amd.build` first")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32p, f32p = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p
        sp, cp = ctypes.POINTER(Shape), ctypes.POINTER(Config)
        sz, ci = ctypes.c_size_t, ctypes.c_int
        L.ramp_last_error.restype = ctypes.c_char_p
        L.ramp_last_error.argtypes = []
        L.ramp_num_configs.restype = ci
        L.ramp_num_configs.argtypes = [sp]
        L.ramp_get_config.restype = ci
        L.ramp_get_config.argtypes = [sp, ci, cp]
        L.ramp_config_ntiles.restype = ci
        L.ramp_config_ntiles.argtypes = [sp, cp]
        L.ramp_config_wave_capacity.restype = ci
        L.ramp_config_wave_capacity.argtypes = [cp]
        L.ramp_config_runtime_occupancy.restype = ci
        L.ramp_config_runtime_occupancy.argtypes = [cp, ctypes.POINTER(ci)]
        L.ramp_align_capacity.restype = sz
        L.ramp_align_capacity.argtypes = [ci, ci, ci, ci]
        L.ramp_align_workspace_bytes.restype = sz
        L.ramp_align_workspace_bytes.argtypes = [ci, ci, ci]
        L.ramp_moe_histogram.restype = ci
        L.ramp_moe_histogram.argtypes = [i32p, ci, ci, ci, i32p, vp, sz, vp]
        L.ramp_moe_align.restype = ci
        L.ramp_moe_align.argtypes = [i32p, ci, ci, ci, ci, i32p, i32p, i32p, i32p, vp, sz, vp]
        L.ramp_pack_bytes.restype = sz
        L.ramp_pack_bytes.argtypes = [sp]
        L.ramp_pack_weights.restype = ci
        L.ramp_pack_weights.argtypes = [sp, vp, vp, vp, vp, vp]
        L.ramp_fused_moe_workspace_bytes.restype = sz
        L.ramp_fused_moe_workspace_bytes.argtypes = [sp, cp]
        L.ramp_fused_moe_workspace_layout.restype = ci
        L.ramp_fused_moe_workspace_layout.argtypes = [sp, cp, ctypes.POINTER(sz)]
        L.ramp_fused_moe.restype = ci
        L.ramp_fused_moe.argtypes = [sp, cp, vp, i32p, f32p, vp, vp, vp, sz, vp]
        L.ramp_fused_moe_static.restype = ci
        L.ramp_fused_moe_static.argtypes = [sp, cp, vp, i32p, f32p, vp, vp, vp]
        L.ramp_fused_moe_selected_workspace_bytes.restype = sz
        L.ramp_fused_moe_selected_workspace_bytes.argtypes = [sp, ci, cp]
        L.ramp_fused_moe_selected.restype = ci
        L.ramp_fused_moe_selected.argtypes = [sp, ci, cp, i32p, vp, i32p, f32p, vp, vp, vp, sz, vp]
        L.ramp_fp8_num_configs.restype = ci
        L.ramp_fp8_num_configs.argtypes = [sp]
        L.ramp_fp8_get_config.restype = ci
        L.ramp_fp8_get_config.argtypes = [sp, ci, cp]
        L.ramp_fp8_config_wave_capacity.restype = ci
        L.ramp_fp8_config_wave_capacity.argtypes = [cp]
        L.ramp_fp8_pack_bytes.restype = sz
        L.ramp_fp8_pack_bytes.argtypes = [sp]
        L.ramp_fp8_pack_weights.restype = ci
        L.ramp_fp8_pack_weights.argtypes = [sp, vp, vp, vp, vp, vp]
        L.ramp_fp8_pack_layout.restype = ci
        L.ramp_fp8_pack_layout.argtypes = [sp, ctypes.POINTER(sz), ctypes.POINTER(ctypes.c_int32)]
        L.ramp_fp8_quantize_rows.restype = ci
        L.ramp_fp8_quantize_rows.argtypes = [vp, ci, ci, vp, vp, vp]
        L.ramp_fused_moe_fp8_workspace_bytes.restype = sz
        L.ramp_fused_moe_fp8_workspace_bytes.argtypes = [sp, cp]
        L.ramp_fused_moe_fp8.restype = ci
        L.ramp_fused_moe_fp8.argtypes = [sp, cp, vp, i32p, f32p, vp, vp, vp, sz, vp]
        L.ramp_cost_model_fit.restype = ci
        L.ramp_cost_model_fit.argtypes = [ci, vp, ci, vp, vp, vp, vp, ci, vp]
        L.ramp_cost_model_select.restype = ci
        L.ramp_cost_model_select.argtypes = [ci, ci, cp, vp, vp, vp, vp, ci, ctypes.POINTER(ci), vp]
        L.ramp_cost_model_fit5.restype = ci
        L.ramp_cost_model_fit5.argtypes = [ci, vp, ci, vp, vp, vp, vp, ci, vp]
        L.ramp_cost_model_select5.restype = ci
        L.ramp_cost_model_select5.argtypes = [ci, ci, cp, vp, vp, vp, vp, ci, ctypes.POINTER(ci), vp]
        L.ramp_cost_model_fit_rounds.restype = ci
        L.ramp_cost_model_fit_rounds.argtypes = [ci, vp, ci, vp, vp, vp, vp, vp, ci, ci, vp]
        L.ramp_cost_model_select_rounds.restype = ci
        L.ramp_cost_model_select_rounds.argtypes = [ci, ci, cp, vp, vp, vp, vp, vp, ci, ci, ctypes.POINTER(ci), vp]
        L.ramp_config_rounds.restype = ci
        L.ramp_config_rounds.argtypes = [sp, cp, ctypes.POINTER(ctypes.c_int32)]
        L.ramp_grid.restype = ci
        L.ramp_grid.argtypes = [ci, ci, cp, vp, vp, vp, vp, vp, vp, vp]
        L.ramp_region_classify.restype = ci
        L.ramp_region_classify.argtypes = [sp, cp, ctypes.c_longlong, ctypes.POINTER(RegionThresholds), ctypes.POINTER(Region)]
        L.ramp_select_table_bytes.restype = sz
        L.ramp_select_table_bytes.argtypes = [ci]
        L.ramp_select_table_build.restype = ci
        L.ramp_select_table_build.argtypes = [ci, cp, vp, vp, vp, ci, vp, vp, sz]
        L.ramp_select_result_bytes.restype = sz
        L.ramp_select_result_bytes.argtypes = [ci, ci]
        L.ramp_select_device.restype = ci
        L.ramp_select_device.argtypes = [i32p, ci, ci, ci, ci, vp, vp, ctypes.c_uint32, vp, vp, sz, vp]
        L.ramp_select_poll.restype = ci
        L.ramp_select_poll.argtypes = [vp, ctypes.c_uint32, ctypes.POINTER(ci)]
        L.ramp_select_wait.restype = ci
        L.ramp_select_wait.argtypes = [vp, ctypes.c_uint32, ctypes.c_double, ctypes.POINTER(ci)]
        L.ramp_probe_enable.restype = ci
        L.ramp_probe_enable.argtypes = [ci]
        L.ramp_probe_read.restype = ci
        L.ramp_probe_read.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ci)]
        L.ramp_mfma_rate_probe.restype = ci
        L.ramp_mfma_rate_probe.argtypes = [vp, ci, vp, vp, ctypes.POINTER(ctypes.c_double)]
        L.ramp_copy_bytes.restype = ci
        L.ramp_copy_bytes.argtypes = [vp, vp, sz, vp]
        _lib = L
    return _lib


EXPORTS = [
    "ramp_last_error", "ramp_num_configs", "ramp_get_config", "ramp_config_ntiles", "ramp_config_wave_capacity", "ramp_config_runtime_occupancy",
    "ramp_align_capacity", "ramp_align_workspace_bytes", "ramp_moe_histogram", "ramp_moe_align", "ramp_pack_bytes",
    "ramp_pack_weights", "ramp_fused_moe_workspace_bytes", "ramp_fused_moe_workspace_layout", "ramp_fused_moe", "ramp_fused_moe_static",
    "ramp_fused_moe_selected_workspace_bytes", "ramp_fused_moe_selected",
    "ramp_fp8_num_configs", "ramp_fp8_get_config", "ramp_fp8_config_wave_capacity", "ramp_fp8_pack_bytes", "ramp_fp8_pack_weights",
    "ramp_fp8_pack_layout", "ramp_fp8_quantize_rows", "ramp_fused_moe_fp8_workspace_bytes", "ramp_fused_moe_fp8",
    "ramp_cost_model_fit", "ramp_cost_model_select", "ramp_cost_model_fit5", "ramp_cost_model_select5",
    "ramp_cost_model_fit_rounds", "ramp_cost_model_select_rounds", "ramp_config_rounds", "ramp_grid", "ramp_region_classify", "ramp_select_table_bytes", "ramp_select_table_build",
    "ramp_select_result_bytes", "ramp_select_device", "ramp_select_poll", "ramp_select_wait", "ramp_copy_bytes", "ramp_mfma_rate_probe", "ramp_probe_enable", "ramp_probe_read",
]


def _check(rc: int):
    if rc != OK:
        raise RampError(rc, lib().ramp_last_error().decode())


def last_error() -> str:
    return lib().ramp_last_error().decode()


def _dev(t: Optional[torch.Tensor]) -> int:
    if t is None:
        return 0
    assert t.is_cuda and t.is_contiguous(), "device buffers must be contiguous GPU tensors"
    return t.data_ptr()


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _np(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


# ----------------------------------------------------------------------------- configuration family

def num_configs(shape: Shape) -> int:
    n = lib().ramp_num_configs(ctypes.byref(shape))
    if n < 0:
        _check(n)
    return n


def get_config(shape: Shape, idx: int) -> Config:
    c = Config()
    _check(lib().ramp_get_config(ctypes.byref(shape), idx, ctypes.byref(c)))
    return c


def configs(shape: Shape):
    return [get_config(shape, i) for i in range(num_configs(shape))]


def config_ntiles(shape: Shape, cfg: Config) -> int:
    n = lib().ramp_config_ntiles(ctypes.byref(shape), ctypes.byref(cfg))
    if n < 0:
        _check(n)
    return n


def config_wave_capacity(cfg: Config) -> int:
    n = lib().ramp_config_wave_capacity(ctypes.byref(cfg))
    if n < 0:
        _check(n)
    return n


def config_runtime_occupancy(cfg: Config):
    """(up-projection, down-projection) workgroups per compute unit according to the HIP runtime (needs a GPU)."""
    out = (ctypes.c_int * 2)()
    _check(lib().ramp_config_runtime_occupancy(ctypes.byref(cfg), out))
    return int(out[0]), int(out[1])


# ----------------------------------------------------------------------------- align

def align_capacity(T: int, k: int, E: int, bm: int) -> int:
    return int(lib().ramp_align_capacity(T, k, E, bm))


def align_workspace_bytes(T: int, k: int, E: int) -> int:
    return int(lib().ramp_align_workspace_bytes(T, k, E))


def moe_histogram(topk_ids: torch.Tensor, T: int, k: int, E: int, expert_counts: torch.Tensor,
                  ws: Optional[torch.Tensor], stream=None):
    _check(lib().ramp_moe_histogram(_dev(topk_ids), T, k, E, _dev(expert_counts), _dev(ws),
                                    ws.numel() * ws.element_size() if ws is not None else 0, _stream(stream)))


def moe_align(topk_ids, T, k, E, bm, sorted_pair_ids, tile_expert, expert_counts, meta, ws, stream=None):
    _check(lib().ramp_moe_align(_dev(topk_ids), T, k, E, bm, _dev(sorted_pair_ids), _dev(tile_expert),
                                _dev(expert_counts), _dev(meta), _dev(ws),
                                ws.numel() * ws.element_size() if ws is not None else 0, _stream(stream)))


# ----------------------------------------------------------------------------- weights and the fused layer

def pack_bytes(shape: Shape) -> int:
    return int(lib().ramp_pack_bytes(ctypes.byref(shape)))


def pack_weights(shape: Shape, W_gate, W_up, W_down, packed, stream=None):
    _check(lib().ramp_pack_weights(ctypes.byref(shape), _dev(W_gate), _dev(W_up), _dev(W_down), _dev(packed),
                                   _stream(stream)))


def fused_moe_workspace_bytes(shape: Shape, cfg: Config) -> int:
    return int(lib().ramp_fused_moe_workspace_bytes(ctypes.byref(shape), ctypes.byref(cfg)))


def fused_moe_workspace_layout(shape: Shape, cfg: Config):
    off = (ctypes.c_size_t * 4)()
    _check(lib().ramp_fused_moe_workspace_layout(ctypes.byref(shape), ctypes.byref(cfg), off))
    return [int(v) for v in off]


def fused_moe(shape: Shape, cfg: Config, X, topk_ids, topk_w, packed_weights, out, ws, stream=None):
    _check(lib().ramp_fused_moe(ctypes.byref(shape), ctypes.byref(cfg), _dev(X), _dev(topk_ids), _dev(topk_w),
                                _dev(packed_weights), _dev(out), _dev(ws), ws.numel() * ws.element_size(),
                                _stream(stream)))


STATIC_WS_BYTES = 64 << 20


def fused_moe_static(shape: Shape, cfg: Config, X, topk_ids, topk_w, packed_weights, out, stream=None):
    """ramp_fused_moe on the library's built-in workspace (no allocation anywhere)."""
    _check(lib().ramp_fused_moe_static(ctypes.byref(shape), ctypes.byref(cfg), _dev(X), _dev(topk_ids), _dev(topk_w),
                                       _dev(packed_weights), _dev(out), _stream(stream)))


def fused_moe_selected_workspace_bytes(shape: Shape, cfgs: Sequence[Config]) -> int:
    arr = (Config * len(cfgs))(*cfgs)
    return lib().ramp_fused_moe_selected_workspace_bytes(ctypes.byref(shape), len(cfgs), arr)


def fused_moe_selected(shape: Shape, cfgs: Sequence[Config], selected_idx: torch.Tensor, X, topk_ids, topk_w,
                       packed_weights, out, ws, stream=None):
    """Every candidate is enqueued; on the device only cfgs[selected_idx[0]] runs (selected_idx: device int32)."""
    arr = (Config * len(cfgs))(*cfgs)
    _check(lib().ramp_fused_moe_selected(ctypes.byref(shape), len(cfgs), arr, _dev(selected_idx), _dev(X), _dev(topk_ids),
                                         _dev(topk_w), _dev(packed_weights), _dev(out), _dev(ws),
                                         ws.numel() * ws.element_size(), _stream(stream)))


# ----------------------------------------------------------------------------- W8A8 FP8 variant

FP8_MODE = 0x10000


def fp8_configs(shape: Shape):
    n = lib().ramp_fp8_num_configs(ctypes.byref(shape))
    if n < 0:
        _check(n)
    out = []
    for i in range(n):
        c = Config()
        _check(lib().ramp_fp8_get_config(ctypes.byref(shape), i, ctypes.byref(c)))
        out.append(c)
    return out


def fp8_config_wave_capacity(cfg: Config) -> int:
    n = lib().ramp_fp8_config_wave_capacity(ctypes.byref(cfg))
    if n < 0:
        _check(n)
    return n


def fp8_pack_bytes(shape: Shape) -> int:
    return int(lib().ramp_fp8_pack_bytes(ctypes.byref(shape)))


def fp8_pack_weights(shape: Shape, W_gate, W_up, W_down, packed, stream=None):
    _check(lib().ramp_fp8_pack_weights(ctypes.byref(shape), _dev(W_gate), _dev(W_up), _dev(W_down), _dev(packed),
                                       _stream(stream)))


def fp8_pack_layout(shape: Shape):
    """(offsets[6], strides[2]) of the packed FP8 buffer, see ramp_fp8_pack_layout."""
    off = (ctypes.c_size_t * 6)()
    st = (ctypes.c_int32 * 2)()
    _check(lib().ramp_fp8_pack_layout(ctypes.byref(shape), off, st))
    return [int(v) for v in off], [int(v) for v in st]


def fp8_quantize_rows(src: torch.Tensor, codes: torch.Tensor, scales: torch.Tensor, stream=None):
    rows, K = src.shape
    _check(lib().ramp_fp8_quantize_rows(_dev(src), rows, K, _dev(codes), _dev(scales), _stream(stream)))


def fused_moe_fp8_workspace_bytes(shape: Shape, cfg: Config) -> int:
    return int(lib().ramp_fused_moe_fp8_workspace_bytes(ctypes.byref(shape), ctypes.byref(cfg)))


def fused_moe_fp8(shape: Shape, cfg: Config, X, topk_ids, topk_w, packed_fp8, out, ws, stream=None):
    _check(lib().ramp_fused_moe_fp8(ctypes.byref(shape), ctypes.byref(cfg), _dev(X), _dev(topk_ids), _dev(topk_w),
                                    _dev(packed_fp8), _dev(out), _dev(ws), ws.numel() * ws.element_size(),
                                    _stream(stream)))


def probe_enable(stage: int):
    _check(lib().ramp_probe_enable(stage))


def probe_read():
    """Returns (total_ms, launches) of the probed stage since the last read."""
    ms, n = ctypes.c_double(0.0), ctypes.c_int(0)
    _check(lib().ramp_probe_read(ctypes.byref(ms), ctypes.byref(n)))
    return ms.value, n.value


def copy_bytes(dst: torch.Tensor, src: torch.Tensor, nbytes: int, stream=None):
    _check(lib().ramp_copy_bytes(_dev(dst), _dev(src), nbytes, _stream(stream)))


def mfma_rate_probe(operands: torch.Tensor, rounds: int, sink: torch.Tensor, stream=None) -> float:
    """Enqueues the register-resident MFMA loop; returns the flops of the launch (the caller times it)."""
    fl = ctypes.c_double(0.0)
    _check(lib().ramp_mfma_rate_probe(_dev(operands), rounds, _dev(sink), _stream(stream), ctypes.byref(fl)))
    return fl.value


# ----------------------------------------------------------------------------- cost model (host)

def cost_model_fit(wave_cap: Sequence[int], grid, time_us, distinct=None, pairs=None, flags: int = CM_EQ6,
                   terms: int = 4, grid_rounds=None) -> np.ndarray:
    """grid, time_us (and distinct with CM_DISTINCT_TILES, grid_rounds with CM_ROUNDS): [n_cfg, n_pts]; pairs (with
    CM_PAIRS): [n_pts].  Returns theta float32 [n_cfg, terms]; terms = 5 is the Sec. 5.3 ablation."""
    assert terms in (4, 5)
    grid = _np(grid, np.int64)
    time_us = _np(time_us, np.float64)
    n_cfg, n_pts = grid.shape
    assert time_us.shape == (n_cfg, n_pts)
    if distinct is not None:
        distinct = _np(distinct, np.int64)
        assert distinct.shape == (n_cfg, n_pts)
    if pairs is not None:
        pairs = _np(pairs, np.int64)
        assert pairs.shape == (n_pts,)
    wc = _np(wave_cap, np.int32)
    assert wc.size == n_cfg
    theta = np.zeros((n_cfg, terms), np.float32)
    if grid_rounds is not None or (flags & CM_ROUNDS):
        if grid_rounds is not None:
            grid_rounds = _np(grid_rounds, np.int64)
            assert grid_rounds.shape == (n_cfg, n_pts)
        _check(lib().ramp_cost_model_fit_rounds(n_cfg, wc.ctypes.data, n_pts, grid.ctypes.data,
                                                grid_rounds.ctypes.data if grid_rounds is not None else None,
                                                distinct.ctypes.data if distinct is not None else None,
                                                pairs.ctypes.data if pairs is not None else None, time_us.ctypes.data,
                                                flags, terms, theta.ctypes.data))
        return theta
    fn = lib().ramp_cost_model_fit if terms == 4 else lib().ramp_cost_model_fit5
    _check(fn(n_cfg, wc.ctypes.data, n_pts, grid.ctypes.data,
              distinct.ctypes.data if distinct is not None else None,
              pairs.ctypes.data if pairs is not None else None, time_us.ctypes.data, flags, theta.ctypes.data))
    return theta


def cost_model_select(E: int, cfgs: Sequence[Config], ntiles, wave_cap, theta, expert_counts, want_pred=False,
                      flags: int = CM_EQ6, terms: int = 4, rounds=None):
    """rounds: int32 [n_cfg, 4] (config_rounds of every configuration), required with CM_ROUNDS."""
    assert terms in (4, 5)
    n = len(cfgs)
    arr = (Config * n)(*cfgs)
    nt, wc = _np(ntiles, np.int32), _np(wave_cap, np.int32)
    th = _np(theta, np.float32).reshape(n, terms)
    counts = _np(expert_counts, np.int32)
    assert counts.size == E and nt.size == n and wc.size == n
    best = ctypes.c_int(-1)
    pred = np.zeros(n, np.float64) if want_pred else None
    if rounds is not None or (flags & CM_ROUNDS):
        rd = None if rounds is None else _np(rounds, np.int32)
        assert rd is None or rd.shape == (n, 4)
        _check(lib().ramp_cost_model_select_rounds(E, n, arr, nt.ctypes.data, rd.ctypes.data if rd is not None else None,
                                                   wc.ctypes.data, th.ctypes.data,
                                                   counts.ctypes.data, flags, terms, ctypes.byref(best),
                                                   pred.ctypes.data if want_pred else None))
        return (best.value, pred) if want_pred else best.value
    fn = lib().ramp_cost_model_select if terms == 4 else lib().ramp_cost_model_select5
    _check(fn(E, n, arr, nt.ctypes.data, wc.ctypes.data, th.ctypes.data, counts.ctypes.data,
              flags, ctypes.byref(best), pred.ctypes.data if want_pred else None))
    return (best.value, pred) if want_pred else best.value


def config_rounds(shape: Shape, cfg: Config) -> np.ndarray:
    """{R_up, ntiles_up, R_down, ntiles_down}: M-tiles per hand-out round and N-tiles of the two launches."""
    out = (ctypes.c_int32 * 4)()
    _check(lib().ramp_config_rounds(ctypes.byref(shape), ctypes.byref(cfg), out))
    return np.array(list(out), np.int32)


def grid(E: int, cfgs: Sequence[Config], ntiles, expert_counts, rounds=None):
    """Eq. 1 per configuration on one histogram: (grid int64 [n_cfg], distinct int64 [n_cfg], pairs int), and with
    rounds (int32 [n_cfg, 4]) a fourth value: grid_rounds int64 [n_cfg], the g_r of CM_ROUNDS."""
    n = len(cfgs)
    arr = (Config * n)(*cfgs)
    nt = _np(ntiles, np.int32)
    counts = _np(expert_counts, np.int32)
    assert counts.size == E and nt.size == n
    g, d = np.zeros(n, np.int64), np.zeros(n, np.int64)
    pairs = ctypes.c_int64(0)
    if rounds is not None:
        rd = _np(rounds, np.int32)
        assert rd.shape == (n, 4)
        gr = np.zeros(n, np.int64)
        _check(lib().ramp_grid(E, n, arr, nt.ctypes.data, counts.ctypes.data, g.ctypes.data, d.ctypes.data,
                               ctypes.addressof(pairs), rd.ctypes.data, gr.ctypes.data))
        return g, d, int(pairs.value), gr
    _check(lib().ramp_grid(E, n, arr, nt.ctypes.data, counts.ctypes.data, g.ctypes.data, d.ctypes.data,
                           ctypes.addressof(pairs), None, None))
    return g, d, int(pairs.value)


# ----------------------------------------------------------------------------- device-resident dispatch

def select_table_build(cfgs: Sequence[Config], ntiles, wave_cap, theta, flags: int = CM_EQ6, rounds=None) -> np.ndarray:
    """Host image (uint8) of the table ramp_select_device reads; copy it to the device once.  rounds: int32 [n_cfg, 4],
    required with CM_ROUNDS."""
    n = len(cfgs)
    arr = (Config * n)(*cfgs)
    nt, wc = _np(ntiles, np.int32), _np(wave_cap, np.int32)
    th = _np(theta, np.float32).reshape(n, 4)
    table = np.zeros(lib().ramp_select_table_bytes(n), np.uint8)
    rd = None if rounds is None else _np(rounds, np.int32)
    assert rd is None or rd.shape == (n, 4)
    _check(lib().ramp_select_table_build(n, arr, nt.ctypes.data, wc.ctypes.data, th.ctypes.data, flags,
                                         rd.ctypes.data if rd is not None else None, table.ctypes.data, table.nbytes))
    return table


def select_result_bytes(E: int, n_cfg: int) -> int:
    return lib().ramp_select_result_bytes(E, n_cfg)


def select_device(topk_ids, T: int, k: int, E: int, n_cfg: int, table: torch.Tensor, result: torch.Tensor, ticket: int,
                  ws: Optional[torch.Tensor], best_idx_dev: Optional[torch.Tensor] = None, stream=None):
    """result: pinned host tensor (polled with select_poll / select_wait) or a device tensor."""
    assert result.is_contiguous() and (result.is_cuda or result.is_pinned())
    _check(lib().ramp_select_device(_dev(topk_ids), T, k, E, n_cfg, _dev(table), result.data_ptr(), ticket,
                                    _dev(best_idx_dev), _dev(ws), ws.numel() * ws.element_size() if ws is not None else 0,
                                    _stream(stream)))


def select_poll(result: torch.Tensor, ticket: int) -> Optional[int]:
    """Index chosen by the enqueue that carried `ticket`, or None while it has not finished."""
    best = ctypes.c_int(-1)
    rc = lib().ramp_select_poll(result.data_ptr(), ticket, ctypes.byref(best))
    if rc < 0:
        _check(rc)
    return best.value if rc == 0 else None


def select_wait(result: torch.Tensor, ticket: int, timeout_s: float = 10.0) -> int:
    best = ctypes.c_int(-1)
    _check(lib().ramp_select_wait(result.data_ptr(), ticket, timeout_s, ctypes.byref(best)))
    return best.value


def select_result_unpack(result: torch.Tensor, E: int, n_cfg: int):
    """(ticket, best, pred_us [n_cfg] fp64, expert_counts [E]) from a host copy of a result block."""
    raw = result.cpu().numpy().view(np.uint8)
    word = int(raw[:8].view(np.uint64)[0])
    ticket, best = word & 0xFFFFFFFF, int(np.int32(word >> 32))
    pred = raw[16:16 + 8 * n_cfg].view(np.float64).copy()
    counts = raw[16 + 8 * n_cfg:16 + 8 * n_cfg + 4 * E].view(np.int32).copy()
    return ticket, best, pred, counts


# ----------------------------------------------------------------------------- performance regions (host)

def region_classify(shape: Shape, cfg: Config, grid: int, thresholds: Optional[RegionThresholds] = None) -> Region:
    out = Region()
    _check(lib().ramp_region_classify(ctypes.byref(shape), ctypes.byref(cfg), int(grid),
                                      ctypes.byref(thresholds) if thresholds is not None else None, ctypes.byref(out)))
    return out
