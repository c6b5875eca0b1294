"""Pins for the oracle's align step (Eq. 1 first factor, Fig. 1): brute force in
Python, invariants, closed forms and the Fig. 1 caption fixture."""
import os

import numpy as np
import pytest

from oracle import oracle
from paper_2604_26039_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def brute_align(ids, E, bm):
    """Rebuild the layout from scratch by sorting pairs on (expert, p)."""
    P = len(ids)
    pairs = sorted((int(e), p) for p, e in enumerate(ids) if 0 <= e < E)
    blocks, tile_e = [], []
    for e in range(E):
        mine = [p for (ee, p) in pairs if ee == e]
        if not mine:
            continue
        while len(mine) % bm:
            mine.append(P)
        blocks += mine
        tile_e += [e] * (len(mine) // bm)
    return blocks, tile_e


CASES = [
    (16, 2, 16, 4, 1.0), (16, 2, 16, 16, 0.2), (16, 2, 16, 4, 0.2), (7, 3, 5, 3, 1.0),
    (1, 8, 64, 16, 1.0), (33, 8, 64, 7, 0.1), (64, 8, 128, 32, 0.08), (5, 1, 1, 2, 1.0),
]


@pytest.mark.parametrize("T,k,E,bm,beta", CASES)
def test_align_matches_brute_force(T, k, E, bm, beta):
    ids, _ = synth.routing_subset(T, k, E, beta, seed=T * 31 + bm)
    flat = ids.reshape(-1)
    s, te, counts, meta = oracle.align(flat, T, k, E, bm)
    blocks, tile_e = brute_align(flat.tolist(), E, bm)
    P = T * k
    assert meta[0] == len(blocks) and meta[1] == len(tile_e) and meta[2] == 0 and meta[3] == 0
    assert s[: len(blocks)].tolist() == blocks
    assert (s[len(blocks):] == P).all()
    assert te[: len(tile_e)].tolist() == tile_e
    assert (te[len(tile_e):] == -1).all()
    assert counts.tolist() == np.bincount(flat, minlength=E).tolist()


@pytest.mark.parametrize("T,k,E,bm,beta", CASES)
def test_align_invariants(T, k, E, bm, beta):
    ids, _ = synth.routing_subset(T, k, E, beta, seed=99 + T)
    flat = ids.reshape(-1)
    s, te, counts, meta = oracle.align(flat, T, k, E, bm)
    P = T * k
    P_pad, M_tiles = int(meta[0]), int(meta[1])
    # every (token, expert) pair is placed exactly once
    placed = s[s != P]
    assert sorted(placed.tolist()) == list(range(P))
    # padding waste = sum_e (ceil(n_e/bm)*bm - n_e)
    waste = sum(-(-int(n) // bm) * bm - int(n) for n in counts)
    assert int((s[:P_pad] == P).sum()) == waste
    assert oracle.padding_waste(counts, bm)[0] == waste
    # M_tiles is the first factor of Eq. 1
    assert M_tiles == sum(-(-int(n) // bm) for n in counts) == oracle.grid(counts, bm, 1)
    assert P_pad == M_tiles * bm
    assert len(s) == oracle.align_capacity(T, k, E, bm) >= P_pad
    # tile membership, monotone experts, increasing p inside an expert
    assert (np.diff(te[:M_tiles]) >= 0).all()
    for m in range(M_tiles):
        row = s[m * bm:(m + 1) * bm]
        real = row[row != P]
        assert len(real) >= 1
        assert (flat[real] == te[m]).all()
        assert (np.diff(real) > 0).all()
        # padding only at the end of a tile
        assert (row[: len(real)] != P).all()
    for e in range(E):
        mine = np.concatenate([s[m * bm:(m + 1) * bm] for m in range(M_tiles) if te[m] == e] or [np.zeros(0, np.int32)])
        mine = mine[mine != P]
        assert (np.diff(mine) > 0).all()


def test_bm1_is_stable_counting_sort():
    ids, _ = synth.routing_subset(50, 4, 32, 0.3, seed=5)
    flat = ids.reshape(-1)
    s, te, counts, meta = oracle.align(flat, 50, 4, 32, 1)
    order = np.argsort(flat, kind="stable")
    assert meta[0] == 200 and meta[1] == 200
    assert s[:200].tolist() == order.tolist()
    assert te[:200].tolist() == flat[order].tolist()
    assert oracle.padding_waste(counts, 1) == (0, 0.0)


def test_bm_at_least_max_count_gives_one_tile_per_active_expert():
    ids, _ = synth.routing_subset(40, 2, 16, 0.5, seed=3)
    flat = ids.reshape(-1)
    counts = np.bincount(flat, minlength=16)
    bm = int(counts.max())
    _, te, _, meta = oracle.align(flat, 40, 2, 16, bm)
    assert meta[1] == int((counts > 0).sum())
    assert te[: meta[1]].tolist() == np.nonzero(counts)[0].tolist()


def test_all_counts_at_most_one_same_grid_for_every_bm():
    # Sec. 5.2: when every expert receives <= 1 token the grid is identical for every bm
    ids = np.arange(8, dtype=np.int32) * 3  # one token, 8 distinct experts out of 32
    tiles = {bm: int(oracle.align(ids, 1, 8, 32, bm)[3][1]) for bm in (1, 2, 4, 16, 64, 104)}
    assert set(tiles.values()) == {8}


def test_out_of_range_ids_are_dropped_and_counted():
    ids = np.array([0, 5, -1, 2, 7, 2, 9, 0], np.int32)  # E=7: -1, 7, 9 dropped
    s, te, counts, meta = oracle.align(ids, 4, 2, 7, 2)
    assert meta[2] == 3
    assert counts.tolist() == [2, 0, 2, 0, 0, 1, 0]
    assert s[: meta[0]].tolist() == [0, 7, 3, 5, 1, 8]
    assert te[: meta[1]].tolist() == [0, 2, 5]


def test_duplicate_expert_within_a_token_is_placed_twice():
    ids = np.array([3, 3], np.int32)
    s, te, counts, meta = oracle.align(ids, 1, 2, 4, 4)
    assert counts[3] == 2 and s[:4].tolist() == [0, 1, 2, 2] and meta[1] == 1


def test_empty_input():
    s, te, counts, meta = oracle.align(np.zeros(0, np.int32), 0, 8, 4, 16)
    assert len(s) == 0 and len(te) == 0 and counts.tolist() == [0] * 4 and meta.tolist() == [0, 0, 0, 0]


def test_fig1_caption_fixture():
    """Fig. 1 caption: 60 % waste at bm=16 vs 20 % at bm=4 under skewed routing."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "fig1_caption.txt")) if l.strip() and not l.startswith("#")]
    hdr = rows[0]
    E, T, k = int(hdr[1]), int(hdr[3]), int(hdr[5])
    counts = [int(v) for v in rows[1][1:]]
    assert len(counts) == E and sum(counts) == T * k and max(counts) <= T
    # realise the histogram as a routing with k distinct experts per token
    ids = realise_histogram(counts, T, k)
    for r in rows[2:]:
        bm, frac = int(r[1]), float(r[3])
        s, te, c, meta = oracle.align(ids.reshape(-1), T, k, E, bm)
        assert c.tolist() == counts
        waste = int((s[: meta[0]] == T * k).sum())
        assert waste / meta[0] == pytest.approx(frac, abs=1e-12)
        assert oracle.padding_waste(counts, bm)[1] == pytest.approx(frac, abs=1e-12)


def realise_histogram(counts, T, k):
    """Deal experts to tokens round-robin, most-loaded first, so each token gets k distinct experts."""
    slots = []
    for e in np.argsort(-np.asarray(counts), kind="stable"):
        slots += [int(e)] * counts[e]
    ids = np.array(slots, np.int32).reshape(k, T).T.copy()  # token t gets slots t, T+t, ...
    for t in range(T):
        assert len(set(ids[t].tolist())) == k
    return ids


def test_tiny_config_skew_direction():
    # the benchmark's own tiny draw: bm=4 wastes less than bm=16 under beta=0.2
    ids, _ = synth.routing_subset(16, 2, 16, 0.2, seed=0)
    counts = np.bincount(ids.reshape(-1), minlength=16)
    assert oracle.padding_waste(counts, 4)[0] < oracle.padding_waste(counts, 16)[0]


def test_balancedness_closed_forms():
    assert oracle.balancedness([5] * 64) == pytest.approx(1.0)
    assert oracle.balancedness([7] + [0] * 63) == pytest.approx(0.0)
    # uniform over m of E experts -> ln m / ln E
    assert oracle.balancedness([3] * 8 + [0] * 56) == pytest.approx(np.log(8) / np.log(64))
