"""The communication performance model (paper Section 5), host only.

1. The plain-Python oracle (oracle/comm_model.py, exact rational arithmetic) is pinned to what the
   paper fixes: the ring equations worked by hand, the five per-layer terms worked by hand from the
   printed equations, the 8-GPU group example of Section 5.2, the two figures' bandwidth cases,
   limits (a group of one costs nothing) and monotonicity.
2. The library's C++ implementation is compared with that oracle on seeded random cases."""
import itertools
import random
from fractions import Fraction as F

import pytest

import paper_2305_13525_amd as axo
from oracle import comm_model as cm
from paper_2305_13525_amd import comm

OK, BAD_GRID, BAD_COORD, INDIVISIBLE, NULL_PTR, BAD_SIZE, BAD_ARG = 0, -1, -2, -3, -4, -10, -11


# ---- pins of the oracle -------------------------------------------------------------------------

def test_ring_equations_by_hand():
    # Section 5.1: G = 4 GPUs, 12 units per GPU, bandwidth 3 units/s
    assert cm.t_all_gather(4, 12, 3) == 12          # (4-1) * 12 / 3
    assert cm.t_reduce_scatter(4, 12, 3) == 3       # (3/4) * 12 / 3
    assert cm.t_all_reduce(4, 12, 3) == 6           # 2 * (3/4) * 12 / 3
    # an all-reduce is a reduce-scatter followed by an all-gather of the scattered piece
    for G, m, b in [(2, 10, 1), (8, 64, 5), (7, 21, 2)]:
        assert cm.t_all_reduce(G, m, b) == cm.t_reduce_scatter(G, m, b) + cm.t_all_gather(G, F(m, G), b)
    # a group of one GPU communicates nothing
    assert cm.t_all_gather(1, 5, 1) == cm.t_reduce_scatter(1, 5, 1) == cm.t_all_reduce(1, 5, 1) == 0


def test_layer_terms_by_hand_from_the_printed_equations():
    # m = 48, k = 24, n = 36 on (Gx, Gy, Gz, Gdata) = (2, 3, 4, 5), every bandwidth 1
    G, beta = (2, 3, 4, 5), (1, 1, 1, 1)
    ag, rs, ary, arx, ard = cm.layer_terms(G, beta, 48, 24, 36, as_printed=True)
    assert ag == 3 * F(24 * 36, 2 * 3 * 4)                 # (Gz-1) kn/(GxGyGz)             = 108
    assert rs == F(3, 4) * F(24 * 36, 2 * 3)               # ((Gz-1)/Gz) kn/(GxGy)          = 108
    assert ary == 2 * F(2, 3) * F(48 * 36, 4 * 2)          # 2 ((Gy-1)/Gy) mn/(GzGx)        = 288
    assert arx == 2 * F(1, 2) * F(48 * 24, 4 * 3)          # 2 ((Gx-1)/Gx) mk/(GzGy)        = 96
    assert ard == 2 * F(4, 5) * F(24 * 36, 2 * 3 * 4)      # 2 ((Gd-1)/Gd) kn/(GxGyGz)      = 57.6
    assert (ag, rs, ary, arx) == (108, 108, 288, 96) and ard == F(288, 5)
    # distinct bandwidths go to the right terms
    ag, rs, ary, arx, ard = cm.layer_terms(G, (2, 3, 4, 5), 48, 24, 36, True)
    assert (ag, rs, ary, arx, ard) == (F(108, 4), F(108, 4), F(288, 3), F(96, 2), F(288, 25))
    # the other kind of layer swaps Gx with Gy and beta_x with beta_y
    sw = cm.layer_terms((3, 2, 4, 5), (3, 2, 4, 5), 48, 24, 36, as_printed=False)
    assert sw == (ag, rs, ary, arx, ard)


def test_group_example_of_section_5_2():
    G = (2, 2, 2, 2)
    assert cm.groups(G, 0) == [(0, 1), (2, 3), (4, 5), (6, 7), (8, 9), (10, 11), (12, 13), (14, 15)]
    assert cm.groups(G, 1)[:4] == [(0, 2), (1, 3), (4, 6), (5, 7)]
    assert cm.groups(G, 2)[:4] == [(0, 4), (1, 5), (2, 6), (3, 7)]
    assert cm.groups(G, 3)[0] == (0, 8)


def test_bandwidth_cases_of_the_two_figures():
    # Figure "spanning eight GPUs on two nodes": one group of 8 over nodes of 4, nothing below it
    assert cm.bandwidths((8, 1, 1, 1), 100, 10, 4)[0] == 10
    # Figure "two simultaneous ... each spanning four GPUs": X pairs inside the node, Y groups of 4 across
    b = cm.bandwidths((2, 4, 1, 1), 100, 10, 4)
    assert b[0] == 100 and b[1] == 5
    # the reduction is bounded by the GPUs per node
    assert cm.bandwidths((4, 4, 4, 1), 100, 10, 4) == [100, F(10, 4), F(10, 4), F(10, 4)]
    # Case 1 all the way: everything fits one node
    assert cm.bandwidths((2, 2, 2, 1), 100, 10, 8) == [100, 100, 100, 100]
    # placement-agnostic: one constant
    assert cm.bandwidths((2, 4, 2, 2), 100, 10, 4, placement_aware=False) == [10, 10, 10, 10]


def test_model_properties():
    layers = [(64, 192, True), (64, 64, False), (64, 256, True), (256, 64, False)]
    base = cm.model_time((2, 2, 2, 2), 100, 10, 4, layers, 1024)
    # faster links never make the modelled time longer, and the time scales as 1/bandwidth
    assert cm.model_time((2, 2, 2, 2), 200, 10, 4, layers, 1024) <= base
    assert cm.model_time((2, 2, 2, 2), 200, 20, 4, layers, 1024) == base / 2
    # more rows cost more
    assert cm.model_time((2, 2, 2, 2), 100, 10, 4, layers, 2048) > base
    # a network is the sum of its layers
    beta = cm.bandwidths((2, 2, 2, 2), 100, 10, 4)
    assert base == sum(sum(cm.layer_terms((2, 2, 2, 2), beta, F(1024, 2), k, n, p)) for k, n, p in layers)
    # a pair of layers, one of each kind, costs the same with the X and Y group sizes exchanged when
    # every bandwidth is equal (the model is symmetric in X and Y up to the transposition)
    pair = [(96, 48, True), (48, 96, False)]
    a = cm.model_time((2, 4, 1, 1), 7, 7, 64, pair, 64, placement_aware=False)
    b = cm.model_time((4, 2, 1, 1), 7, 7, 64, [(k, n, not p) for k, n, p in pair], 64, placement_aware=False)
    assert a == b
    # enumeration: all ordered factorizations
    assert len(cm.factorizations(8)) == 20 and len(cm.factorizations(1)) == 1
    assert all(a * b * c * d == 32 for a, b, c, d in cm.factorizations(32))


# ---- the library against the oracle ---------------------------------------------------------------

def net(bi, be, gn, aware=1):
    return comm.CommNet(float(bi), float(be), gn, aware)


def close(a, b):
    return abs(a - float(b)) <= 1e-12 * max(1.0, abs(float(b)))


def test_library_ring_times():
    for G, m, b in [(1, 5.0, 2.0), (2, 1e6, 3e9), (8, 123456.0, 153.6e9), (1024, 7.0, 1.0)]:
        assert close(comm.axo_comm_ring_all_gather(G, m, b), cm.t_all_gather(G, F(m), F(b)))
        assert close(comm.axo_comm_ring_reduce_scatter(G, m, b), cm.t_reduce_scatter(G, F(m), F(b)))
        assert close(comm.axo_comm_ring_all_reduce(G, m, b), cm.t_all_reduce(G, F(m), F(b)))
    assert comm.axo_comm_ring_all_reduce(0, 1.0, 1.0) < 0 and comm.axo_comm_ring_all_gather(2, -1.0, 1.0) < 0
    assert comm.axo_comm_ring_reduce_scatter(2, 1.0, 0.0) < 0


def test_library_bandwidths_and_layer_terms_random():
    rng = random.Random(5)
    for _ in range(300):
        G = tuple(rng.choice([1, 2, 3, 4, 8]) for _ in range(4))
        gn = rng.choice([1, 2, 4, 8])
        bi, be = rng.choice([100, 153.6, 300]), rng.choice([12.5, 25, 50])
        aware = rng.random() < 0.8
        cfg, nt = comm.CommConfig(*G), net(bi, be, gn, int(aware))
        _, beta = comm.axo_comm_bandwidths(cfg, nt)
        ref = cm.bandwidths(G, F(bi), F(be), gn, aware)
        assert all(close(a, b) for a, b in zip(beta, ref))
        m, k, n = rng.randrange(1, 5000), rng.randrange(1, 5000), rng.randrange(1, 5000)
        tr = rng.randrange(2)
        _, t = comm.axo_comm_layer_time(cfg, nt, comm.CommLayer(k, n, tr, 0), m, 2.0)
        ag, rs, ary, arx, ard = [2 * x for x in cm.layer_terms(G, ref, m, k, n, as_printed=bool(tr))]
        assert close(t.ag_z, ag) and close(t.rs_z, rs) and close(t.ar_fwd, ary) and close(t.ar_bwd, arx)
        assert close(t.ar_data, ard) and close(t.total, ag + rs + ary + arx + ard)


def gpt_layers(h):
    return [(h, 3 * h, 0), (h, h, 1), (h, 4 * h, 0), (4 * h, h, 1)]


def test_library_model_time_and_ranking():
    h, batch = 7168, 32768                   # the running example of Section 4
    layers = [comm.CommLayer(k, n, t, 0) for k, n, t in gpt_layers(h)]
    ref_layers = [(k, n, bool(t)) for k, n, t in gpt_layers(h)]
    nt = net(100e9, 25e9, 4)
    rc, total, terms = comm.axo_comm_model_time(comm.CommConfig(2, 2, 4, 1), nt, layers, batch, 2.0)
    assert close(total, 2 * cm.model_time((2, 2, 4, 1), F(100e9), F(25e9), 4, ref_layers, batch))
    assert close(terms.total, total) and terms.ar_data == 0.0

    rc, cfgs, times, n_found = comm.axo_comm_rank_configs(32, nt, layers, batch, 2.0)
    feasible = [G for G in cm.factorizations(32)
                if batch % G[3] == 0 and (batch // G[3]) % G[2] == 0
                and all(k % (G[1] if t else G[0]) == 0 and n % (G[0] if t else G[1]) == 0 for k, n, t in gpt_layers(h))]
    assert n_found == len(feasible) == len(cfgs)
    ref = sorted(feasible, key=lambda G: (cm.model_time(G, F(100e9), F(25e9), 4, ref_layers, batch), G))
    assert cfgs == ref
    assert all(b >= a * (1 - 1e-12) for a, b in zip(times, times[1:]))
    for G, t in zip(cfgs, times):
        assert close(t, 2 * cm.model_time(G, F(100e9), F(25e9), 4, ref_layers, batch))
    # truncated output still reports the number of feasible configurations
    rc, c3, t3, n3 = comm.axo_comm_rank_configs(32, nt, layers, batch, 2.0, max_out=3)
    assert n3 == n_found and c3 == cfgs[:3]
    # placement changes the ranking (the point of Section 5.2)
    rc, flat, _, _ = comm.axo_comm_rank_configs(32, net(100e9, 25e9, 4, 0), layers, batch, 2.0)
    assert flat != cfgs


def test_library_mi355x_preset_and_rank_mapping():
    nt = comm.axo_comm_net_mi355x()
    assert (nt.G_node, nt.placement_aware) == (8, 1) and nt.beta_intra > nt.beta_inter > 0
    cfg = comm.CommConfig(2, 2, 2, 2)
    assert [comm.axo_comm_rank_to_coord(cfg, r)[1] for r in (0, 1, 2, 3, 4, 8, 15)] == \
        [(0, 0, 0, 0), (1, 0, 0, 0), (0, 1, 0, 0), (1, 1, 0, 0), (0, 0, 1, 0), (0, 0, 0, 1), (1, 1, 1, 1)]
    G = (2, 3, 4, 5)
    cfg = comm.CommConfig(*G)
    for c in itertools.product(range(2), range(3), range(4), range(5)):
        rc, r = comm.axo_comm_coord_to_rank(cfg, c)
        assert r == cm.rank_of(G, c) and comm.axo_comm_rank_to_coord(cfg, r)[1] == c
    assert comm.axo_comm_rank_to_coord(cfg, 120, check=False)[0] == BAD_COORD
    assert comm.axo_comm_coord_to_rank(cfg, (2, 0, 0, 0), check=False)[0] == BAD_COORD


def test_library_argument_errors():
    cfg, nt, layer = comm.CommConfig(2, 2, 2, 2), net(1, 1, 4), comm.CommLayer(8, 8, 0, 0)
    assert comm.axo_comm_bandwidths(comm.CommConfig(0, 1, 1, 1), nt, check=False)[0] == BAD_GRID
    assert comm.axo_comm_bandwidths(cfg, net(0, 1, 4), check=False)[0] == BAD_ARG
    assert comm.axo_comm_bandwidths(cfg, net(1, 1, 0), check=False)[0] == BAD_ARG
    assert comm.axo_comm_layer_time(cfg, nt, comm.CommLayer(8, 8, 2, 0), 4, 2.0, check=False)[0] == BAD_ARG
    assert comm.axo_comm_layer_time(cfg, nt, comm.CommLayer(8, 8, 0, 1), 4, 2.0, check=False)[0] == BAD_ARG
    assert comm.axo_comm_layer_time(cfg, nt, layer, -1, 2.0, check=False)[0] == BAD_SIZE
    assert comm.axo_comm_layer_time(cfg, nt, layer, 4, 0.0, check=False)[0] == BAD_SIZE
    assert comm.axo_comm_model_time(cfg, nt, [layer], 7, 2.0, check=False)[0] == INDIVISIBLE
    assert comm.axo_comm_rank_configs(0, nt, [layer], 8, 2.0, check=False)[0] == BAD_SIZE
    L = axo.library()
    assert L.axo_comm_bandwidths(None, None, None) == NULL_PTR
    assert L.axo_comm_net_mi355x(None) == NULL_PTR
