"""Rank groups of MoE Parallel Folding (Section 3.2) against group lists worked by hand
(tests/golden/folding_groups.txt), against numpy's reshape/transpose, and by their invariants."""
import os

import numpy as np
import pytest

from paper_2504_14960_amd.folding import generate_mappings, groups_of_rank

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "folding_groups.txt")
CASES = {"A": dict(args=(64, 2, 2, 2, 2, 2)), "B": dict(args=(16, 2, 2, 4, 1, 2)),
         "C": dict(args=(16, 2, 1, 4, 1, 2), pp_outermost=True)}


def _golden():
    want = {}
    for ln in open(GOLDEN):
        if not ln.strip() or ln.startswith("#"):
            continue
        head, body = ln.split(":")
        case, grid, axis = head.split()
        want[(case, grid, axis)] = [[int(v) for v in g.split()] for g in body.split("|")]
    return want


def test_hand_worked_group_lists():
    want = _golden()
    assert len(want) == 24
    for case, spec in CASES.items():
        attn, moe = generate_mappings(*spec["args"], pp_outermost=spec.get("pp_outermost", False))
        for (c, grid, axis), groups in want.items():
            if c == case:
                assert (attn if grid == "attn" else moe)[axis] == groups, (case, grid, axis)


@pytest.mark.parametrize("world,tp,cp,ep,etp,pp", [(64, 2, 2, 2, 2, 2), (32, 4, 1, 2, 2, 2), (48, 2, 3, 6, 1, 2),
                                                    (16, 2, 2, 4, 1, 2), (8, 1, 1, 8, 1, 1), (24, 2, 1, 1, 2, 3)])
def test_against_numpy_reshape(world, tp, cp, ep, etp, pp):
    """A group along one axis is a row of the rank grid with that axis moved last (library reshape/moveaxis)."""
    attn, moe = generate_mappings(world, tp, cp, ep, etp, pp)
    ga = np.arange(world).reshape(world // (tp * cp * pp), pp, cp, tp)
    gm = np.arange(world).reshape(world // (etp * ep * pp), pp, ep, etp)
    for nm, ax in (("DP", 0), ("PP", 1), ("CP", 2), ("TP", 3)):
        assert attn[nm] == np.moveaxis(ga, ax, -1).reshape(-1, ga.shape[ax]).tolist()
    for nm, ax in (("DP", 0), ("PP", 1), ("EP", 2), ("TP", 3)):
        assert moe[nm] == np.moveaxis(gm, ax, -1).reshape(-1, gm.shape[ax]).tolist()


@pytest.mark.parametrize("outer", [False, True])
def test_invariants(outer):
    world, tp, cp, ep, etp, pp = 64, 4, 2, 8, 1, 2
    attn, moe = generate_mappings(world, tp, cp, ep, etp, pp, pp_outermost=outer)
    sizes = {"attn": dict(TP=tp, CP=cp, PP=pp, DP=world // (tp * cp * pp)),
             "moe": dict(TP=etp, EP=ep, PP=pp, DP=world // (etp * ep * pp))}
    for grid, groups in (("attn", attn), ("moe", moe)):
        for axis, gl in groups.items():
            flat = [r for g in gl for r in g]
            assert sorted(flat) == list(range(world))                 # the groups of an axis partition the ranks
            assert all(len(g) == sizes[grid][axis] for g in gl)
            assert all(g == sorted(g) for g in gl)
        for r in (0, 17, 63):
            mine = groups_of_rank(groups, r)
            common = set(range(world))
            for g in mine.values():
                common &= set(g)
            assert common == {r}                                      # four coordinates name one rank
    # the folding: an EP group of 8 covers whole attention TP x CP blocks, and the pipeline groups agree
    assert sorted(map(tuple, attn["PP"])) == sorted(map(tuple, moe["PP"]))
    for g in moe["EP"]:
        blocks = {tuple(groups_of_rank(attn, r)["TP"]) for r in g}
        assert sum(len(b) for b in blocks) == len(g)


def test_restriction_and_argument_errors():
    with pytest.raises(ValueError, match="pipeline groups"):
        generate_mappings(16, 2, 1, 4, 1, 2)              # tp*cp = 2, etp*ep = 4, pp > 1
    generate_mappings(16, 2, 1, 4, 1, 1)                  # no pipeline: nothing to agree on
    generate_mappings(16, 2, 1, 4, 1, 2, pp_outermost=True)
    with pytest.raises(ValueError, match="multiple"):
        generate_mappings(60, 2, 2, 2, 2, 2)
    with pytest.raises(ValueError, match="positive"):
        generate_mappings(64, 0, 2, 2, 2, 2)
    # tp != etp: the MoE grid is shaped with etp (ETP groups of one rank, not of tp ranks)
    _, moe = generate_mappings(16, 2, 2, 4, 1, 2)
    assert all(len(g) == 1 for g in moe["TP"]) and len(moe["TP"]) == 16
