"""Pins for the oracle's duplicate token dropping (paper Section 5.1): the drop of rank r keeps rows
r, r+G, ... of every expert chunk, the gather after the all-gather restores the chunk.  No GPU."""
import os

import numpy as np
import pytest

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def chunks(E, Cap, w, seed=0):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((E, Cap, w)).astype(np.float32)


@pytest.mark.parametrize("G", [1, 2, 3, 4, 8])
@pytest.mark.parametrize("Cap", [1, 7, 16, 37])
def test_drop_is_a_strided_slice_and_gather_inverts_it(orc, G, Cap):
    E, w = 3, 5
    D = chunks(E, Cap, w, seed=G * 100 + Cap)
    Cg = -(-Cap // G)
    shares = []
    for r in range(G):
        s = orc.dtd_drop(D, G, r)
        assert s.shape == (E, Cg, w)
        want = np.zeros((E, Cg, w), np.float32)
        part = D[:, r::G, :]                      # the array library's own strided slice
        want[:, :part.shape[1]] = part
        assert np.array_equal(s, want)
        shares.append(s)
    back = orc.dtd_gather(np.stack(shares), Cap)
    assert np.array_equal(back, D)


def test_every_row_leaves_the_group_exactly_once_and_messages_shrink_by_G(orc):
    E, Cap, G = 4, 22, 4
    ids = np.arange(E * Cap, dtype=np.float32).reshape(E, Cap, 1) + 1.0      # row id, never 0
    seen = np.zeros(E * Cap + 1, np.int64)
    rows_sent = 0
    for r in range(G):
        s = orc.dtd_drop(ids, G, r)
        rows_sent += s.shape[0] * s.shape[1]
        for v in s.ravel():
            if v != 0:
                seen[int(v)] += 1
    assert (seen[1:] == 1).all()
    assert rows_sent == G * E * -(-Cap // G)                  # each rank sends ceil(C/G) rows per expert instead of C
    assert rows_sent < E * Cap * G / (G - 1)                  # and in total about one copy of the chunk, not G


def test_order_inside_a_share_is_the_order_of_the_chunk(orc):
    D = np.arange(2 * 9 * 1, dtype=np.float32).reshape(2, 9, 1)
    s = orc.dtd_drop(D, 3, 1)
    assert s[0, :, 0].tolist() == [1.0, 4.0, 7.0] and s[1, :, 0].tolist() == [10.0, 13.0, 16.0]
    # a transposed (rank, row) convention would put row 3 r + j here
    assert orc.dtd_drop(D, 3, 0)[0, :, 0].tolist() == [0.0, 3.0, 6.0]


def test_papers_two_gpu_example(orc):
    """Section 5.1 / Figure 5: in a group of two, the first GPU keeps a1 and the second a2 (and a3 / a4 in the
    other group); the all-gather gives both back to both."""
    rows = [l.split() for l in open(os.path.join(GOLD, "dtd_worked_example.txt")) if l.strip() and not l.startswith("#")]
    assert len(rows) == 4
    for G, r, held, kept in rows:
        G, r = int(G), int(r)
        held = [float(v) for v in held.split(",")]
        chunk = np.array(held, np.float32).reshape(1, len(held), 1)      # one expert chunk, activations by id
        share = orc.dtd_drop(chunk, G, r)
        assert share.ravel().tolist() == [float(kept)]
    both = np.stack([orc.dtd_drop(np.array([[[1.0], [2.0]]], np.float32), 2, r) for r in range(2)])
    assert orc.dtd_gather(both, 2).ravel().tolist() == [1.0, 2.0]


def test_backward_swaps_the_two_steps(orc):
    """The backward pass replaces the all-gather by a drop and the drop by an all-gather (Section 5.1): the drop is
    linear and its transpose is the gather restricted to one rank's rows, so <drop(u), v> == <u, gather_r(v)>."""
    E, Cap, w, G = 2, 10, 3, 4
    rng = np.random.default_rng(5)
    u = rng.standard_normal((E, Cap, w)).astype(np.float32)
    for r in range(G):
        v = rng.standard_normal((E, -(-Cap // G), w)).astype(np.float32)
        # rows of v beyond the chunk's end carry nothing
        for j in range(v.shape[1]):
            if j * G + r >= Cap:
                v[:, j] = 0
        only_r = np.zeros((G,) + v.shape, np.float32)
        only_r[r] = v
        lhs = float((orc.dtd_drop(u, G, r).astype(np.float64) * v).sum())
        rhs = float((u.astype(np.float64) * orc.dtd_gather(only_r, Cap)).sum())
        assert abs(lhs - rhs) < 1e-9
