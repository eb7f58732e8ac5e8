"""Plain-Python statement of the communication performance model (paper Section 5).

TEST INFRASTRUCTURE ONLY, like the rest of this package: the library's own implementation is
compiled C++ and shares nothing with this file.

Section 5.1: ring all-gather / reduce-scatter / all-reduce times; the five per-layer terms for
I in R^{m x k}, W in R^{k x n} on (Gx, Gy, Gz, Gdata); layers of the other kind swap Gx with Gy and
beta_x with beta_y; a network is the sum over its layers.  Section 5.2: the group hierarchy
X, Y, Z, data and the bandwidth each level sees (Case 1 / Case 2).

The equations as printed belong to Algorithm 1 as printed (K split over Y, N over X); here
`as_printed=True` selects them and `as_printed=False` the swapped kind.

Pins (tests/test_comm_model.py): values worked by hand from the printed equations, the 8-GPU group
example of Section 5.2, the two figures' bandwidth cases, limits and monotonicity.
"""
from __future__ import annotations

from fractions import Fraction
from typing import Iterable, List, Sequence, Tuple


def t_all_gather(G, m, beta):
    return Fraction(1) / beta * (G - 1) * m


def t_reduce_scatter(G, m, beta):
    return Fraction(1) / beta * Fraction(G - 1, G) * m


def t_all_reduce(G, m, beta):
    return Fraction(2) / beta * Fraction(G - 1, G) * m


def bandwidths(G: Sequence[int], beta_intra, beta_inter, G_node: int, placement_aware: bool = True):
    """(beta_x, beta_y, beta_z, beta_data) for G = (Gx, Gy, Gz, Gdata)."""
    out = []
    for i in range(4):
        if not placement_aware:
            out.append(Fraction(beta_inter))
            continue
        upto = 1
        for j in range(i + 1):
            upto *= G[j]
        if upto <= G_node:                      # Case 1: the whole group inside a node
            out.append(Fraction(beta_intra))
        else:                                   # Case 2: inter-node rings share the node's links
            before = 1
            for j in range(i):
                before *= G[j]
            out.append(Fraction(beta_inter) / min(G_node, before))
    return out


def layer_terms(G: Sequence[int], beta: Sequence, m, k, n, as_printed: bool = True):
    """The five terms (t_AG,z, t_RS,z, t_AR,y, t_AR,x, t_AR,data) in elements / (elements per second)."""
    Gx, Gy, Gz, Gd = G
    bx, by, bz, bd = beta
    if not as_printed:                          # the other kind of layer: swap the X and Y roles
        Gx, Gy, bx, by = Gy, Gx, by, bx
    ag_z = t_all_gather(Gz, Fraction(k * n, Gx * Gy * Gz), bz)
    rs_z = t_reduce_scatter(Gz, Fraction(k * n, Gx * Gy), bz)
    ar_y = t_all_reduce(Gy, Fraction(m * n, Gz * Gx), by)
    ar_x = t_all_reduce(Gx, Fraction(m * k, Gz * Gy), bx)
    ar_d = t_all_reduce(Gd, Fraction(k * n, Gx * Gy * Gz), bd)
    return ag_z, rs_z, ar_y, ar_x, ar_d


def model_time(G, beta_intra, beta_inter, G_node, layers: Iterable[Tuple[int, int, bool]], batch_rows: int,
               placement_aware: bool = True):
    """Total over layers (k, n, as_printed); m = batch_rows / Gdata."""
    beta = bandwidths(G, beta_intra, beta_inter, G_node, placement_aware)
    m = Fraction(batch_rows, G[3])
    return sum((sum(layer_terms(G, beta, m, k, n, p)) for (k, n, p) in layers), Fraction(0))


def factorizations(n_gpus: int) -> List[Tuple[int, int, int, int]]:
    out = []
    for gx in range(1, n_gpus + 1):
        if n_gpus % gx:
            continue
        for gy in range(1, n_gpus // gx + 1):
            if (n_gpus // gx) % gy:
                continue
            rest = n_gpus // gx // gy
            for gz in range(1, rest + 1):
                if rest % gz == 0:
                    out.append((gx, gy, gz, rest // gz))
    return out


def rank_of(G, coord):
    ix, iy, iz, d = coord
    return ix + G[0] * (iy + G[1] * (iz + G[2] * d))


def groups(G, level: int) -> List[Tuple[int, ...]]:
    """All process groups of one level (0 = X ... 3 = data) as tuples of ranks."""
    world = G[0] * G[1] * G[2] * G[3]
    seen, out = set(), []
    for r in range(world):
        c = [r % G[0], r // G[0] % G[1], r // (G[0] * G[1]) % G[2], r // (G[0] * G[1] * G[2])]
        key = tuple(c[:level] + c[level + 1:])
        if key in seen:
            continue
        seen.add(key)
        members = []
        for v in range(G[level]):
            cc = list(c)
            cc[level] = v
            members.append(rank_of(G, cc))
        out.append(tuple(members))
    return out
