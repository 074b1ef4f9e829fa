"""Rank groups of MoE Parallel Folding (Section 3.2; the appendix "Parallel Groups Initialization").

Host-only utility, no GPU and no collective involved: it answers "which ranks
form my TP / CP / PP / DP group in the attention layers, and my ETP / EP / PP /
EDP group in the MoE layers" for a folded configuration.

Section 3.2 lays the ``world`` ranks out on two four-dimensional grids, one per
layer kind, both filled in rank order with the last axis varying fastest:

    attention:  DP  x PP x CP x TP        DP  = world / (TP * CP * PP)
    MoE:        EDP x PP x EP x ETP       EDP = world / (ETP * EP * PP)

A group along one axis is the set of ranks that agree in the three other
coordinates, listed by ascending coordinate on that axis; the groups of an axis
are listed in row-major order of the three other coordinates.  The MoE grid is
shaped with ETP (the appendix listing shapes it with the attention TP, which only
works when the two are equal).  The one restriction the section states is
checked: every rank must find the same pipeline group on both grids.
With ``pp_outermost=True`` the pipeline axis is the slowest one on both grids
(PP x DP x CP x TP and PP x EDP x EP x ETP); the pipeline groups then agree for
every choice of the other degrees.
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple

Groups = Dict[str, List[List[int]]]


def _axis_groups(sizes: Sequence[int], axis: int) -> List[List[int]]:
    """Groups along `axis` of a row-major grid with the given axis sizes."""
    strides = [1] * len(sizes)
    for i in range(len(sizes) - 2, -1, -1):
        strides[i] = strides[i + 1] * sizes[i + 1]
    others = [i for i in range(len(sizes)) if i != axis]
    groups: List[List[int]] = []
    coord = [0] * len(others)
    while True:
        base = sum(c * strides[i] for c, i in zip(coord, others))
        groups.append([base + j * strides[axis] for j in range(sizes[axis])])
        k = len(others) - 1            # next combination of the other coordinates, last one fastest
        while k >= 0:
            coord[k] += 1
            if coord[k] < sizes[others[k]]:
                break
            coord[k] = 0
            k -= 1
        if k < 0:
            return groups


def _grid(names: Sequence[str], sizes: Sequence[int]) -> Groups:
    return {nm: _axis_groups(sizes, i) for i, nm in enumerate(names)}


def generate_mappings(world_size: int, tp: int, cp: int, ep: int, etp: int, pp: int,
                      pp_outermost: bool = False) -> Tuple[Groups, Groups]:
    """Returns (attention groups, MoE groups): dictionaries with the keys "TP", "CP", "PP", "DP" and
    "TP", "EP", "PP", "DP" (the MoE layer's TP and DP being ETP and EDP), each a list of rank lists."""
    for nm, v in (("world_size", world_size), ("tp", tp), ("cp", cp), ("ep", ep), ("etp", etp), ("pp", pp)):
        if not isinstance(v, int) or v < 1:
            raise ValueError(f"{nm} must be a positive integer, got {v!r}")
    if world_size % (tp * cp * pp):
        raise ValueError(f"world_size {world_size} is not a multiple of tp*cp*pp = {tp * cp * pp}")
    if world_size % (etp * ep * pp):
        raise ValueError(f"world_size {world_size} is not a multiple of etp*ep*pp = {etp * ep * pp}")
    dp = world_size // (tp * cp * pp)
    edp = world_size // (etp * ep * pp)
    if pp_outermost:
        attn = _grid(("PP", "DP", "CP", "TP"), (pp, dp, cp, tp))
        moe = _grid(("PP", "DP", "EP", "TP"), (pp, edp, ep, etp))
    else:
        attn = _grid(("DP", "PP", "CP", "TP"), (dp, pp, cp, tp))
        moe = _grid(("DP", "PP", "EP", "TP"), (edp, pp, ep, etp))
    if sorted(map(tuple, attn["PP"])) != sorted(map(tuple, moe["PP"])):
        raise ValueError(
            "the pipeline groups of the attention and the MoE grid differ "
            f"(tp*cp = {tp * cp}, etp*ep = {etp * ep}): Section 3.2 requires them to be the same; "
            "choose degrees with tp*cp == etp*ep or pp_outermost=True")
    return attn, moe


def groups_of_rank(groups: Groups, rank: int) -> Dict[str, List[int]]:
    """The one group per axis that holds `rank`."""
    out = {}
    for nm, gl in groups.items():
        hit = [g for g in gl if rank in g]
        if len(hit) != 1:
            raise ValueError(f"rank {rank} lies in {len(hit)} {nm} groups")
        out[nm] = hit[0]
    return out
