"""Pins for the oracle's model of the paper's engine schedule (Sec. 4.3.2, 5.2.2, 6.3.2):
hand-worked cases, closed forms, invariants.  (The paper's own example is in a figure that
did not survive; its measured efficiencies need its trained models: parity unpinned.)"""
import numpy as np

import oracle


def model(blocks, P, Q, K, L, exact_2d=True):
    nr = np.array([[b[0] for b in row] for row in blocks])
    nc = np.array([[b[1] for b in row] for row in blocks])
    return oracle.sharing_model(nr, nc, P, Q, K, L, exact_2d=exact_2d)


def test_single_block_ragged_edges():
    # 5 x 3 kernel on a 2 x 2 PEGroup: ceil(5/2) * ceil(3/2) = 6 cycles for 15 multiply-adds
    r = model([[(5, 3)]], 2, 2, 1, 1)
    assert r["cycles_none"] == 6 and r["work"] == 15 and abs(r["eff_none"] - 15 / 24) < 1e-15
    # alone on a 1 x 1 torus a PEGroup is its own neighbour: sharing changes nothing
    assert r["cycles_horizontal"] == 6 and r["cycles_vertical"] == 6 and r["cycles_2d"] == 6


def test_horizontal_sharing_by_hand():
    # two PEGroups side by side, 2 x 2 PEs: a 4 x 8 kernel next to an empty block.
    # alone: 2 * 4 = 8 cycles, the neighbour idles: efficiency 32 / (4 * 2 * 8) = 1/2;
    # handing 4 of the 8 columns over: 4 cycles each: efficiency 1
    r = model([[(4, 8), (0, 0)]], 2, 2, 1, 2)
    assert r["cycles_none"] == 8 and r["eff_none"] == 0.5
    assert r["cycles_horizontal"] == 4 and r["eff_horizontal"] == 1.0
    assert r["cycles_vertical"] == 8                      # nobody below to take rows (K = 1)
    assert r["cycles_2d"] == 4
    # shares come in multiples of Q: a 4 x 6 kernel can hand over 2 or 4 columns:
    # (4 x 4 | 4 x 2) -> max(4, 2) = 4; there is no 3 + 3 split
    r = model([[(4, 6), (0, 0)]], 2, 2, 1, 2)
    assert r["cycles_none"] == 6 and r["cycles_horizontal"] == 4


def test_vertical_sharing_by_hand():
    # two PEGroups on top of each other: an 8 x 4 kernel above an empty block; at most half
    # of the rows may go down: 4 x 4 stays (4 cycles), 4 x 4 goes (4 cycles)
    r = model([[(8, 4)], [(0, 0)]], 2, 2, 2, 1)
    assert r["cycles_none"] == 8 and r["cycles_vertical"] == 4 and r["cycles_horizontal"] == 8 and r["cycles_2d"] == 4
    # the half-of-the-rows limit: a 6 x 4 kernel may hand down 0 or 2 rows (not 4): (4 x 4 | 2 x 4) -> 4
    r = model([[(6, 4)], [(0, 0)]], 2, 2, 2, 1)
    assert r["cycles_none"] == 6 and r["cycles_vertical"] == 4
    # heavy block in the lower row hands to the upper one through the torus
    r = model([[(0, 0)], [(8, 4)]], 2, 2, 2, 1)
    assert r["cycles_vertical"] == 4


def test_two_dimensional_beats_both_by_hand():
    # 2 x 2 PEGroups of 2 x 2 PEs, one 8 x 8 kernel (16 cycles alone), three empty blocks.
    # One direction: half of it goes away, 8 cycles.  Both directions, full-height horizontal
    # part (shape 0) with dnh = 2, dmv = 4: right gets 8 x 2 (4 cycles), below gets 4 x 6 (6),
    # 4 x 6 stays (6): largest load 6.  Nothing does better: the three parts hold 64
    # multiply-adds, i.e. 16 cycles of a 2 x 2 PEGroup, so one of them takes at least 6
    # (shares are even: part sizes are products of even numbers, 5 cycles + 5 + 5 < 16).
    r = model([[(8, 8), (0, 0)], [(0, 0), (0, 0)]], 2, 2, 2, 2)
    assert r["cycles_none"] == 16 and r["cycles_horizontal"] == 8 and r["cycles_vertical"] == 8
    assert r["cycles_2d"] == 6


def test_uniform_blocks_need_no_sharing():
    r = model([[(8, 4)] * 4] * 2, 4, 4, 2, 2, exact_2d=False)
    assert r["iterations"] == 2 and r["eff_none"] == 1.0 and r["eff_horizontal"] == 1.0 and r["eff_vertical"] == 1.0


def test_invariants_on_random_blocks():
    rng = np.random.default_rng(0)
    for trial in range(6):
        nr = rng.integers(0, 7, (3, 4))
        nc = rng.integers(0, 7, (3, 4))
        r = oracle.sharing_model(nr, nc, 2, 2, 2, 2, exact_2d=True)
        assert r["iterations"] == 4 and r["work"] == int((nr * nc).sum())
        assert r["cycles_2d"] <= min(r["cycles_horizontal"], r["cycles_vertical"])
        assert max(r["cycles_horizontal"], r["cycles_vertical"]) <= r["cycles_none"]
        assert r["cycles_2d"] * 2 * 2 * 2 * 2 >= r["work"]            # efficiency at most 1
        for k in ("none", "horizontal", "vertical", "2d"):
            assert 0.0 <= r["eff_" + k] <= 1.0
