"""Pins for the oracle's routing (top-1 choice, arrival-order slots, capacity drop).

None of these call the GPU library.  Each pin is independent of the oracle's own code:
the paper's worked example, an O(T^2) brute force, a one-hot/cumsum formulation in numpy,
and structural invariants.
"""
import os

import numpy as np
import pytest

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _read_golden(name):
    d = {}
    with open(os.path.join(GOLD, name)) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, *v = line.split()
            d[k] = v
    return d


def test_paper_worked_example(orc):
    g = _read_golden("routing_worked_example.txt")
    T, E = int(g["T"][0]), int(g["E"][0])
    Cap = orc.capacity(T, E, float(g["capacity_factor"][0]))
    assert Cap == int(g["C"][0])
    expert = np.array(g["expert"], np.int32)
    # logits that realise the example's assignment through the oracle's own top-1 choice
    logits = np.full((T, E), -1.0, np.float32)
    logits[np.arange(T), expert] = 1.0
    e2, p, P = orc.top1_softmax(logits)
    assert e2.tolist() == expert.tolist()
    slot, counts, kept, tok = orc.route(e2, E, Cap)
    assert slot.tolist() == [int(v) for v in g["slot"]]
    assert counts.tolist() == [int(v) for v in g["counts"]]
    assert kept.tolist() == [int(v) for v in g["kept"]]
    assert tok.reshape(-1).tolist() == [int(v) for v in g["token_of_slot"]]


def brute_force_route(expert, E, Cap):
    T = len(expert)
    slot = np.empty(T, np.int32)
    for t in range(T):
        rank = sum(1 for u in range(t) if expert[u] == expert[t])
        slot[t] = rank if rank < Cap else -1
    counts = np.array([sum(1 for u in range(T) if expert[u] == e) for e in range(E)], np.int32)
    return slot, counts


def onehot_cumsum_route(expert, E, Cap):
    T = len(expert)
    M = np.zeros((T, E), np.int64)
    M[np.arange(T), expert] = 1
    pos = np.cumsum(M, axis=0) - 1
    mypos = pos[np.arange(T), expert]
    slot = np.where(mypos < Cap, mypos, -1).astype(np.int32)
    counts = M.sum(0).astype(np.int32)
    return slot, counts


@pytest.mark.parametrize("T,E,cf", [(1, 1, 1.0), (7, 3, 1.0), (64, 4, 1.0), (257, 5, 0.5), (512, 16, 1.25),
                                     (300, 64, 1.0), (129, 2, 0.1)])
def test_route_matches_brute_force_and_cumsum(orc, T, E, cf):
    rng = np.random.default_rng(T * 131 + E)
    # skewed choice so that some experts overflow
    w = 1.0 / (np.arange(E) + 1.0)
    expert = rng.choice(E, size=T, p=w / w.sum()).astype(np.int32)
    Cap = orc.capacity(T, E, cf)
    slot, counts, kept, tok = orc.route(expert, E, Cap)
    s_bf, c_bf = brute_force_route(expert, E, Cap)
    s_oh, c_oh = onehot_cumsum_route(expert, E, Cap)
    assert np.array_equal(slot, s_bf) and np.array_equal(slot, s_oh)
    assert np.array_equal(counts, c_bf) and np.array_equal(counts, c_oh)
    assert np.array_equal(kept, np.minimum(counts, Cap))


def check_invariants(expert, slot, counts, kept, tok, E, Cap):
    T = len(expert)
    assert counts.sum() == T
    assert (kept <= Cap).all() and (kept >= 0).all()
    assert kept.sum() == (slot >= 0).sum()
    assert ((slot >= -1) & (slot < Cap)).all()
    for e in range(E):
        idx = np.nonzero(expert == e)[0]
        ks = slot[idx]
        good = ks[ks >= 0]
        # kept slots are exactly 0..kept-1, increasing with the token index (arrival order)
        assert np.array_equal(good, np.arange(kept[e]))
        # every dropped token comes after every kept one
        if (ks < 0).any() and (ks >= 0).any():
            assert idx[ks < 0].min() > idx[ks >= 0].max()
        # dropped iff exclusive rank >= C
        assert np.array_equal(ks < 0, np.arange(len(idx)) >= Cap)
        # inverse map
        assert np.array_equal(tok[e, :kept[e]], idx[:kept[e]])
        assert (tok[e, kept[e]:] == -1).all()


@pytest.mark.parametrize("seed", range(6))
def test_route_invariants_random(orc, seed):
    rng = np.random.default_rng(seed)
    T = int(rng.integers(1, 3000))
    E = int(rng.integers(1, 70))
    cf = float(rng.choice([0.25, 0.5, 1.0, 1.25, 2.0]))
    Cap = orc.capacity(T, E, cf)
    logits = rng.standard_normal((T, E)).astype(np.float32)
    logits += (-2.0 * np.log(np.arange(E) + 1.0)).astype(np.float32)[None, :]
    expert, p, P = orc.top1_softmax(logits)
    slot, counts, kept, tok = orc.route(expert, E, Cap)
    check_invariants(expert, slot, counts, kept, tok, E, Cap)


def test_top1_ties_and_signed_zero(orc):
    # all equal -> expert 0; two-way ties -> lower index; -0.0 and +0.0 compare equal
    L = np.zeros((5, 4), np.float32)
    L[1] = [1, 3, 3, 2]
    L[2] = [-0.0, 0.0, -1, -1]
    L[3] = [0.0, -0.0, -1, -1]
    L[4] = [-5, -5, -5, -4]
    e, p, P = orc.top1_softmax(L)
    assert e.tolist() == [0, 1, 0, 0, 3]
    assert np.allclose(p[0], 0.25)


def test_route_degenerate_cases(orc):
    # everything to expert 0 with C < T: first C kept, rest dropped
    T, E = 100, 4
    Cap = orc.capacity(T, E, 1.0)
    e = np.zeros(T, np.int32)
    slot, counts, kept, tok = orc.route(e, E, Cap)
    assert slot[:Cap].tolist() == list(range(Cap)) and (slot[Cap:] == -1).all()
    assert counts.tolist() == [T, 0, 0, 0] and kept.tolist() == [Cap, 0, 0, 0]
    # everything to the last expert
    e = np.full(T, E - 1, np.int32)
    slot, counts, kept, tok = orc.route(e, E, Cap)
    assert kept.tolist() == [0, 0, 0, Cap]
    # E = 1, capacity factor >= 1: nothing dropped, slot == token index
    slot, counts, kept, tok = orc.route(np.zeros(T, np.int32), 1, orc.capacity(T, 1, 1.0))
    assert slot.tolist() == list(range(T))
    # C = 1
    e = np.array([2, 2, 1, 2, 1, 0], np.int32)
    slot, counts, kept, tok = orc.route(e, 3, 1)
    assert slot.tolist() == [0, -1, 0, -1, -1, 0]
    assert counts.tolist() == [1, 2, 3] and kept.tolist() == [1, 1, 1]


def test_capacity_formula(orc):
    assert orc.capacity(256, 4, 1.0) == 64
    assert orc.capacity(8192, 16, 1.25) == 640
    assert orc.capacity(16384, 16, 1.25) == 1280
    assert orc.capacity(16384, 64, 1.0) == 256
    assert orc.capacity(10, 3, 1.0) == 4          # ceil(3.33)
    assert orc.capacity(7, 2, 1.25) == 5          # ceil(4.375)
