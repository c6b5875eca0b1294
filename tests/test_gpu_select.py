"""GPU parity: ramp_select_device (histogram + cost model + argmin in one enqueue, result polled in pinned
host memory) against the oracle's select on the oracle's histogram, through the C ABI.  Covers the
single-launch and the chunked histogram paths, every benchmark shape, empty input, out-of-range ids, both
the printed model and the four-flag variant, and the asynchronous use of two result blocks."""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2604_26039_amd import ramp, synth, tuner

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

ALL_FLAGS = ramp.CM_RELATIVE | ramp.CM_DISTINCT_TILES | ramp.CM_WAVE_FLOOR | ramp.CM_PAIRS | ramp.CM_ROUNDS
NO_ROUNDS = ALL_FLAGS & ~ramp.CM_ROUNDS


def family(name, T):
    s = synth.SHAPES[name]
    fam = tuner.Family.of(s, T)
    return s, fam


def synthetic_theta(fam, seed):
    """Positive coefficients of the size a fit on this chip produces, different for every configuration."""
    rng = np.random.default_rng(seed)
    n = len(fam.cfgs)
    th = np.empty((n, 4), np.float32)
    th[:, 0] = rng.uniform(15, 60, n)
    th[:, 1] = rng.uniform(5, 80, n)
    th[:, 2] = rng.uniform(0.01, 0.5, n)
    th[:, 3] = rng.uniform(1e-4, 5e-3, n)
    return th


def device_select(ids_np, T, s, fam, theta, flags, result=None, ticket=1, guard=True):
    n = len(fam.cfgs)
    table = torch.from_numpy(ramp.select_table_build(fam.cfgs, fam.ntiles, fam.wave_cap, theta, flags, rounds=fam.rounds)).to(DEV)
    nbytes = ramp.select_result_bytes(s.E, n)
    if result is None:
        result = torch.zeros(nbytes + (64 if guard else 0), dtype=torch.uint8).pin_memory()
        result[nbytes:] = 0xAB
    ids = torch.from_numpy(np.ascontiguousarray(ids_np.reshape(-1), dtype=np.int32)).to(DEV)
    ws = torch.empty(max(256, ramp.align_workspace_bytes(T, s.k, s.E)), dtype=torch.uint8, device=DEV)
    best_dev = torch.full((2,), -7, dtype=torch.int32, device=DEV)
    ramp.select_device(ids, T, s.k, s.E, n, table, result, ticket, ws, best_idx_dev=best_dev)
    best = ramp.select_wait(result, ticket, timeout_s=20.0)
    torch.cuda.synchronize()
    tk, b2, pred, counts = ramp.select_result_unpack(result, s.E, n)
    assert tk == ticket and b2 == best
    assert best_dev.cpu().tolist() == [best, -7]
    if guard:
        assert (result[nbytes:] == 0xAB).all(), "write past the end of the result block"
    return best, pred, counts


def oracle_histogram(ids, k, E):
    """n_e from the oracle's align (its third output); pairs outside [0,E) are dropped."""
    ids = np.ascontiguousarray(np.asarray(ids).reshape(-1), dtype=np.int32)
    return oracle.align(ids, ids.size // k, k, E, 16)[2]


def oracle_select(fam, theta, counts, flags):
    bm = [c.bm for c in fam.cfgs]
    if flags & ramp.CM_ROUNDS:
        return oracle.select_rounds(bm, fam.ntiles, fam.wave_cap, theta, counts, fam.rounds,
                                    distinct_tiles=bool(flags & ramp.CM_DISTINCT_TILES),
                                    wave_floor=bool(flags & ramp.CM_WAVE_FLOOR), pairs_term=bool(flags & ramp.CM_PAIRS))
    return oracle.select(bm, fam.ntiles, fam.wave_cap, theta, counts,
                         distinct_tiles=bool(flags & ramp.CM_DISTINCT_TILES),
                         wave_floor=bool(flags & ramp.CM_WAVE_FLOOR), pairs_term=bool(flags & ramp.CM_PAIRS))


CASES = [
    ("tiny", 16, 0.2), ("olmoe", 1, 1.0), ("olmoe", 16, 0.5), ("olmoe", 256, 1.0), ("olmoe", 257, 0.2),
    ("olmoe", 1024, 0.1),    # 8192 pairs: last size whose histogram the select kernel makes itself
    ("olmoe", 1025, 1.0),    # first size that takes the chunked histogram launch
    ("olmoe", 4096, 1.0), ("olmoe", 4096, 0.1), ("qwen3", 8192, 0.08), ("qwen3", 32, 0.3),
    ("mixtral", 8192, "zipf1.2"), ("mixtral", 1, 1.0), ("dsv3", 8192, 0.1), ("dsv3", 64, 1.0), ("dsv3", 2048, 0.2),
]


@pytest.mark.parametrize("name,T,beta", CASES)
@pytest.mark.parametrize("flags", [ALL_FLAGS, NO_ROUNDS, ramp.CM_EQ6])
def test_select_device_matches_oracle(name, T, beta, flags):
    s, fam = family(name, T)
    ids, _ = synth.routing(T, s, beta, seed=3 * T + 1)
    theta = synthetic_theta(fam, seed=T)
    best, pred, counts = device_select(ids, T, s, fam, theta, flags)
    ref_counts = oracle_histogram(ids, s.k, s.E)
    assert np.array_equal(counts, ref_counts)
    b_o, p_o = oracle_select(fam, theta, ref_counts, flags)
    if flags & ramp.CM_PAIRS:
        # no transcendental in this variant: same fp64 operations in the same order
        assert np.array_equal(pred, p_o) and best == b_o
    else:
        # the printed model's logarithm may differ in the last bit between math libraries
        assert np.abs(pred - p_o).max() <= 1e-12 * np.abs(p_o).max()
        assert best == b_o or abs(p_o[best] - p_o[b_o]) <= 1e-12 * abs(p_o[b_o])
    # and the host entry point agrees with both
    b_h, p_h = ramp.cost_model_select(s.E, fam.cfgs, fam.ntiles, fam.wave_cap, theta, ref_counts, want_pred=True, flags=flags,
                                      rounds=fam.rounds if flags & ramp.CM_ROUNDS else None)
    assert b_h == b_o and np.array_equal(p_h, p_o)


def test_select_device_empty_and_dropped_ids():
    s, fam = family("olmoe", 64)
    theta = synthetic_theta(fam, seed=5)
    best, pred, counts = device_select(np.zeros(0, np.int32), 0, s, fam, theta, ALL_FLAGS)
    assert (counts == 0).all()
    b_o, p_o = oracle_select(fam, theta, counts, ALL_FLAGS)
    assert best == b_o and np.array_equal(pred, p_o)
    ids, _ = synth.routing(64, s, 0.5, seed=2)
    ids = ids.copy().reshape(-1)
    ids[::7] = -1
    ids[3::11] = s.E
    best, pred, counts = device_select(ids, 64, s, fam, theta, ALL_FLAGS)
    ref = oracle_histogram(ids, s.k, s.E)
    assert np.array_equal(counts, ref)
    b_o, p_o = oracle_select(fam, theta, ref, ALL_FLAGS)
    assert best == b_o and np.array_equal(pred, p_o)


def test_select_device_ties_take_the_lowest_index():
    s, fam = family("olmoe", 256)
    theta = np.tile(np.array([[20.0, 0.0, 0.0, 0.0]], np.float32), (len(fam.cfgs), 1))  # every prediction equal
    ids, _ = synth.routing(256, s, 1.0, seed=9)
    best, pred, _ = device_select(ids, 256, s, fam, theta, ALL_FLAGS)
    assert best == 0 and (pred == 20.0).all()
    theta[17, 0] = 19.0
    theta[40, 0] = 19.0
    best, _, _ = device_select(ids, 256, s, fam, theta, ALL_FLAGS)
    assert best == 17


def test_dispatcher_resident_async_and_host_agree():
    """The three dispatch modes of the tuner on a stream of calls whose routing changes: the device-resident and
    the host select see this call's histogram; the asynchronous one returns the choice of the previous call."""
    s, fam = family("olmoe", 512)
    theta = synthetic_theta(fam, seed=11)
    disp = tuner.Dispatcher(fam, theta, ALL_FLAGS, 512, device=DEV)
    betas = [1.0, 1.0, 0.1, 0.1, 0.5, 1.0, 0.2]
    batches = [torch.from_numpy(synth.routing(512, s, b, seed=i)[0].reshape(-1).astype(np.int32)).to(DEV)
               for i, b in enumerate(betas)]
    expect = [oracle_select(fam, theta, oracle_histogram(b.cpu().numpy(), s.k, s.E), ALL_FLAGS)[0] for b in batches]
    for b, e in zip(batches, expect):
        assert disp.select(b) == e
        assert np.array_equal(disp.last_counts(), oracle_histogram(b.cpu().numpy(), s.k, s.E))
        assert disp.select_host(b) == e
    # per-step cache: the first layer of a step decides for the whole step
    disp.begin_step()
    assert [disp.select_step(b) for b in batches[2:5]] == [expect[2]] * 3
    disp.begin_step()
    assert disp.select_step(batches[0]) == expect[0]
    disp2 = tuner.Dispatcher(fam, theta, ALL_FLAGS, 512, device=DEV)
    got = []
    for b in batches:
        got.append(disp2.select_async(b))
        torch.cuda.synchronize()  # the enqueued selection has finished before the next call polls it
    assert got[0] == expect[0]          # the first call waits for its own selection
    assert got[1:] == expect[:-1]       # afterwards: the previous call's


def test_select_device_rejects_bad_arguments():
    s, fam = family("olmoe", 16)
    n = len(fam.cfgs)
    theta = synthetic_theta(fam, seed=1)
    table = torch.from_numpy(ramp.select_table_build(fam.cfgs, fam.ntiles, fam.wave_cap, theta, 0)).to(DEV)
    result = torch.zeros(ramp.select_result_bytes(s.E, n), dtype=torch.uint8).pin_memory()
    ids = torch.zeros(16 * s.k, dtype=torch.int32, device=DEV)
    ws = torch.empty(256, dtype=torch.uint8, device=DEV)
    with pytest.raises(ramp.RampError):
        ramp.select_device(ids, 16, s.k, s.E, n, table, result, 0, ws)          # ticket 0 is reserved
    with pytest.raises(ramp.RampError):
        ramp.select_device(ids, 16, s.k, 2000, n, table, result, 1, ws)         # E above the limit
    with pytest.raises(ramp.RampError):
        ramp.select_device(ids, 4096, s.k, s.E, n, table, result, 1, ws)        # workspace too small for the chunked path
    assert ramp.select_poll(result, 1) is None                                   # nothing was enqueued
    # a table for another configuration count is rejected by the kernel itself; nothing is evaluated
    ramp.select_device(ids, 16, s.k, s.E, n - 1, table, result, 7, ws)
    with pytest.raises(ramp.RampError):
        ramp.select_wait(result, 7, timeout_s=20.0)
    torch.cuda.synchronize()


def _candidates(fam):
    """One configuration of each kernel family, small and large token blocks."""
    pick = []
    for want in (lambda c: c.mode & 0x100 and c.bm <= 16, lambda c: c.mode & 0x400 and c.bm == 256,
                 lambda c: not (c.mode & 0x700) and c.bm == 64, lambda c: c.mode & 0x200):
        pick += [c for c in fam.cfgs if want(c)][:1]
    return pick


@pytest.mark.parametrize("T,beta", [(1, 1.0), (96, 0.2), (700, 1.0)])
def test_fused_moe_selected_equals_the_selected_configuration(T, beta):
    """Every candidate is enqueued behind the device-side index; the output is bit-identical to ramp_fused_moe
    with the candidate the index names, whichever it is; the others leave no trace in the output."""
    s = synth.SHAPES["olmoe"]
    fam = tuner.Family.of(s, T)
    cands = _candidates(fam)
    assert len(cands) == 4
    X, Wg, Wu, Wd = synth.layer_tensors(s, T, seed=T, device=DEV, x_std=1.0)
    rs = ramp.Shape(T, s.k, s.E, s.H, s.I)
    packed = torch.empty(ramp.pack_bytes(rs), dtype=torch.uint8, device=DEV)
    ramp.pack_weights(rs, Wg, Wu, Wd, packed)
    ids, w = synth.routing(T, s, beta, seed=5)
    d_ids = torch.from_numpy(np.ascontiguousarray(ids, np.int32)).to(DEV)
    d_w = torch.from_numpy(np.ascontiguousarray(w, np.float32)).to(DEV)
    nbytes = ramp.fused_moe_selected_workspace_bytes(rs, cands)
    assert nbytes >= max(ramp.fused_moe_workspace_bytes(rs, c) for c in cands)
    for pos, cfg in enumerate(cands):
        ref = torch.zeros((T, s.H), dtype=torch.bfloat16, device=DEV)
        ws1 = torch.empty(ramp.fused_moe_workspace_bytes(rs, cfg), dtype=torch.uint8, device=DEV)
        ramp.fused_moe(rs, cfg, X, d_ids, d_w, packed, ref, ws1)
        sel = torch.tensor([pos, -7], dtype=torch.int32, device=DEV)
        ws = torch.full((nbytes + 1024,), 0xFF, dtype=torch.uint8, device=DEV)
        out = torch.full((T + 1, s.H), 777.0, dtype=torch.bfloat16, device=DEV)
        ramp.fused_moe_selected(rs, cands, sel, X, d_ids, d_w, packed, out, ws[:nbytes])
        torch.cuda.synchronize()
        assert (ws[nbytes:] == 0xFF).all() and (out[T] == 777.0).all()
        assert torch.equal(out[:T].view(torch.int16), ref.view(torch.int16)), f"candidate {pos} {cfg}"


def test_select_and_layer_in_one_hip_graph():
    """Histogram, cost model, argmin and the layer with the chosen configuration captured once as a HIP graph: no
    host decision between the selection and the launch.  Replays with different routing pick different candidates
    and match the eager result of the candidate the oracle's select names."""
    s = synth.SHAPES["olmoe"]
    T = 96
    fam_all = tuner.Family.of(s, T)
    cands = _candidates(fam_all)
    fam = tuner.Family(fam_all.shape, cands, np.array([ramp.config_ntiles(fam_all.shape, c) for c in cands], np.int32),
                       np.array([ramp.config_wave_capacity(c) for c in cands], np.int32))
    # coefficients under which balanced routing prefers the first candidate and skewed routing another one
    theta = np.array([[10, 0.0, 0.00, 1e-3], [10, 0.0, 0.00, 1e-3], [10, 0.0, 0.00, 1e-3], [10, 0.0, 0.0, 1e-3]], np.float32)
    theta[0, 2], theta[1, 2], theta[2, 2], theta[3, 2] = 0.001, 0.2, 0.05, 0.05
    theta[0, 0], theta[1, 0] = 30.0, 10.0
    X, Wg, Wu, Wd = synth.layer_tensors(s, T, seed=3, device=DEV, x_std=1.0)
    rs = ramp.Shape(T, s.k, s.E, s.H, s.I)
    packed = torch.empty(ramp.pack_bytes(rs), dtype=torch.uint8, device=DEV)
    ramp.pack_weights(rs, Wg, Wu, Wd, packed)
    n = len(cands)
    table = torch.from_numpy(ramp.select_table_build(cands, fam.ntiles, fam.wave_cap, theta, ALL_FLAGS, rounds=fam.rounds)).to(DEV)
    result = torch.zeros(ramp.select_result_bytes(s.E, n), dtype=torch.uint8, device=DEV)  # device block: nothing is polled
    sel = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    d_ids = torch.zeros((T, s.k), dtype=torch.int32, device=DEV)
    d_w = torch.zeros((T, s.k), dtype=torch.float32, device=DEV)
    out = torch.zeros((T, s.H), dtype=torch.bfloat16, device=DEV)
    ws_sel = torch.empty(max(256, ramp.align_workspace_bytes(T, s.k, s.E)), dtype=torch.uint8, device=DEV)
    ws = torch.empty(ramp.fused_moe_selected_workspace_bytes(rs, cands), dtype=torch.uint8, device=DEV)

    def enqueue(stream):
        ramp.select_device(d_ids, T, s.k, s.E, n, table, result, 1, ws_sel, best_idx_dev=sel, stream=stream)
        ramp.fused_moe_selected(rs, cands, sel, X, d_ids, d_w, packed, out, ws, stream=stream)

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        enqueue(side)
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            enqueue(side)
    torch.cuda.current_stream().wait_stream(side)
    chosen = []
    for rep, beta in enumerate((1.0, 0.1, 1.0, 0.2)):
        ids, w = synth.routing(T, s, beta, seed=60 + rep)
        d_ids.copy_(torch.from_numpy(np.ascontiguousarray(ids, np.int32)))
        d_w.copy_(torch.from_numpy(np.ascontiguousarray(w, np.float32)))
        out.fill_(777.0)
        ws.fill_(0xFF)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        want = oracle_select(fam, theta, oracle_histogram(ids, s.k, s.E), ALL_FLAGS)[0]
        assert int(sel.cpu()[0]) == want
        chosen.append(want)
        ref = torch.zeros_like(out)
        ws1 = torch.empty(ramp.fused_moe_workspace_bytes(rs, cands[want]), dtype=torch.uint8, device=DEV)
        ramp.fused_moe(rs, cands[want], X, d_ids, d_w, packed, ref, ws1)     # eager work between replays
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), ref.view(torch.int16)), f"replay {rep} candidate {want}"
    assert len(set(chosen)) >= 2, f"the replays should exercise more than one candidate, got {chosen}"


def test_fused_moe_selected_with_no_candidate_selected_touches_nothing_else():
    """An index outside the candidate list (what a rejected table leaves behind) deselects every launch, the combine
    included: the call succeeds, `out` and the workspace keep their previous contents, and argument errors are
    rejected on the host."""
    s = synth.SHAPES["olmoe"]
    T = 40
    fam = tuner.Family.of(s, T)
    cands = _candidates(fam)[:2]
    X, Wg, Wu, Wd = synth.layer_tensors(s, T, seed=2, device=DEV, x_std=1.0)
    rs = ramp.Shape(T, s.k, s.E, s.H, s.I)
    packed = torch.empty(ramp.pack_bytes(rs), dtype=torch.uint8, device=DEV)
    ramp.pack_weights(rs, Wg, Wu, Wd, packed)
    ids, w = synth.routing(T, s, 0.5, seed=1)
    d_ids = torch.from_numpy(np.ascontiguousarray(ids, np.int32)).to(DEV)
    d_w = torch.from_numpy(np.ascontiguousarray(w, np.float32)).to(DEV)
    nbytes = ramp.fused_moe_selected_workspace_bytes(rs, cands)
    ws = torch.full((nbytes + 512,), 0xAB, dtype=torch.uint8, device=DEV)   # stale bytes, NaN patterns as floats
    out = torch.full((T + 1, s.H), 777.0, dtype=torch.bfloat16, device=DEV)
    for bad in (-1, len(cands), 1 << 20):
        sel = torch.tensor([bad], dtype=torch.int32, device=DEV)
        ramp.fused_moe_selected(rs, cands, sel, X, d_ids, d_w, packed, out, ws[:nbytes])
        torch.cuda.synchronize()
        assert (ws == 0xAB).all(), "a deselected launch wrote into the workspace"
        assert (out == 777.0).all(), "a call with no candidate selected must leave `out` untouched"
    sel = torch.tensor([-1], dtype=torch.int32, device=DEV)
    with pytest.raises(ramp.RampError):
        ramp.fused_moe_selected(rs, cands, sel, X, d_ids, d_w, packed, out, ws[:nbytes - 256])   # workspace too small
    with pytest.raises(ramp.RampError):
        ramp.fused_moe_selected(rs, cands * 9, sel, X, d_ids, d_w, packed, out, ws[:nbytes])     # more than 16 candidates
