"""Pins for oracle/placement.py: the values the paper prints, the closed forms'
special cases, and brute force for the shard geometry."""
from fractions import Fraction

import pytest

from oracle import placement as pl

GB = 10 ** 9


def test_table1_and_bytes_per_param(golden):
    P = int(golden["P_70b"])
    sz = pl.state_bytes(P)
    assert sz["theta"] == int(golden["theta_GB"]) * GB
    assert sz["grad"] == int(golden["grad_GB"]) * GB
    # Omega groups master weights with Adam's m and v (Table 1 caption).
    assert sz["omega"] == (int(golden["master_GB"]) + int(golden["adam_mv_GB"])) * GB
    assert sum(sz.values()) == int(golden["model_state_GB"]) * GB
    assert sum(sz.values()) == int(golden["bytes_per_param"]) * P


def test_memory_example(golden):
    P, N = int(golden["P_70b"]), int(golden["N_example"])
    dp = pl.memory(pl.STRATEGIES["dp"], P, N)
    z3 = pl.memory(pl.STRATEGIES["zero3"], P, N)
    assert dp == int(golden["dp_per_device_GB"]) * GB
    assert z3 == int(golden["zero3_per_device_GB"]) * GB == 2 * P
    assert dp / z3 == int(golden["memory_reduction"])


def test_communication_example(golden):
    P, N = int(golden["P_70b"]), int(golden["N_example"])
    dp = pl.communication(pl.STRATEGIES["dp"], P, N)
    z3 = pl.communication(pl.STRATEGIES["zero3"], P, N)
    assert dp == Fraction(golden["dp_comm_P_times"]) * P
    assert z3 == Fraction(golden["zero3_comm_P_times"]) * P
    assert round(dp / GB) == int(golden["dp_comm_GB_approx"])
    assert round(z3 / GB) == int(golden["zero3_comm_GB_approx"])
    assert z3 / dp == Fraction(golden["zero3_over_dp_comm"])


@pytest.mark.parametrize("N", [2, 3, 6, 8, 64, 1024])
def test_ratio_is_exactly_three_halves_for_every_N(N):
    # |Theta| = |G| so the (N-1)/N factor cancels (Section 7.1, communication validation).
    P = 12345678 * N
    assert (pl.communication(pl.STRATEGIES["zero3"], P, N) * 2 ==
            pl.communication(pl.STRATEGIES["dp"], P, N) * 3)


def test_figure1_memory_labels():
    s, N = 4096, 8
    assert pl.mu("R", s, N) == s
    assert pl.mu("S", s, N) == Fraction(s, N)
    assert pl.mu("S*", s, N) == Fraction(s, N)          # persistent part
    assert pl.mu("M", s, N) == 0
    assert pl.mu("O", s, N) == 0
    assert pl.mu("S*", s, N, s_unit=100) == Fraction(s, N) + 100   # Eq. 9
    assert pl.mu("M", s, N, s_unit=100) == 100                      # Eq. 10


def test_corollary1_deltas():
    P, N = 7 * 10 ** 9, 8
    sz = pl.state_bytes(P)
    dp, z1, z2, z3 = (pl.STRATEGIES[k] for k in ("dp", "zero1", "zero2", "zero3"))
    # 1: sharding Omega saves memory, communication unchanged.
    assert pl.communication(z1, P, N) == pl.communication(dp, P, N)
    assert pl.memory(dp, P, N) - pl.memory(z1, P, N) == Fraction(sz["omega"] * (N - 1), N)
    # 2: sharding G halves the synchronisation volume.
    assert pl.communication(z2, P, N) * 2 == pl.communication(z1, P, N)
    # 3: S* for Theta adds exactly two all-gathers.
    assert (pl.communication(z3, P, N) - pl.communication(z2, P, N) ==
            Fraction(2 * (N - 1) * sz["theta"], N))


def test_collective_costs():
    assert pl.all_reduce(8, 800) == 1400
    assert pl.reduce_scatter(8, 800) == 700
    assert pl.all_gather(8, 800) == 700
    assert pl.all_reduce(4, 100) == pl.reduce_scatter(4, 100) + pl.all_gather(4, 100)


@pytest.mark.parametrize("psi,N,align", [(24, 4, 1), (25, 4, 1), (23, 6, 1), (100, 6, 4),
                                         (1, 3, 1), (1535, 6, 256), (1537, 6, 256), (0, 2, 1)])
def test_shard_geometry_brute_force(psi, N, align):
    owners = {}
    prev_end = 0
    lengths = set()
    for i in range(N):
        psi_pad, off, n, valid = pl.shard_geometry(psi, N, i, align)
        assert psi_pad % (N * max(1, align)) == 0 and psi_pad >= psi
        assert psi_pad - psi < N * max(1, align)
        assert off == prev_end            # contiguous, ordered
        prev_end = off + n
        lengths.add(n)
        assert 0 <= valid <= n
        for e in range(off, off + valid):
            assert e not in owners
            owners[e] = i
    assert len(lengths) == 1 and prev_end == psi_pad
    assert sorted(owners) == list(range(psi))   # every element has exactly one owner


def test_shard_geometry_matches_eq2_when_divisible():
    psi, N = 1_048_576, 4
    for i in range(N):
        _, off, n, valid = pl.shard_geometry(psi, N, i)
        assert off == i * psi // N and off + n == (i + 1) * psi // N and valid == n


def test_figure2_groups(golden):
    T, D = int(golden["fig2_tp_degree"]), int(golden["fig2_dp_degree"])
    tp, dp = pl.tp_dp_groups(T, D)
    assert tp[0] == [int(x) for x in golden["fig2_tp_group0"].split()]
    assert tp[1] == [int(x) for x in golden["fig2_tp_group1"].split()]
    pairs = [tuple(int(x) for x in p.split("-")) for p in golden["fig2_dp_pairs"].split()]
    assert [tuple(g) for g in dp] == pairs


@pytest.mark.parametrize("A,B", [(4, 2), (1, 8), (8, 1), (3, 5)])
def test_group_calculus_partitions_the_devices(A, B):
    for groups in (*pl.tp_dp_groups(A, B), *pl.pp_dp_groups(A, B)):
        flat = sorted(d for g in groups for d in g)
        assert flat == list(range(A * B))                      # every device in exactly one group
    tp, dp = pl.tp_dp_groups(A, B)
    for g in tp:
        for h in dp:
            assert len(set(g) & set(h)) == 1                   # inner and outer groups cross once
    stages, pipes = pl.pp_dp_groups(A, B)
    assert all(len(s_) == B for s_ in stages) and all(len(p_) == A for p_ in pipes)
    assert all(p_[k + 1] - p_[k] == B for p_ in pipes for k in range(A - 1))


def test_algorithm1_thresholds(golden):
    GBy = 10 ** 9
    th = float(golden["alg1_dp_threshold"])
    assert th == 0.7 and float(golden["alg1_layer_threshold"]) == 0.3
    # 70B on 80 GB devices: 1120 GB model state, 140 GB per device at N=8 -> neither fits
    spec, tp = pl.select_strategy(70 * GBy, 80 * GBy, 8, layer_bytes=30 * GBy, fast_interconnect=True)
    assert spec == pl.STRATEGIES["zero3"] and tp
    assert pl.select_strategy(70 * GBy, 80 * GBy, 8, 30 * GBy, False) == (pl.STRATEGIES["zero3"], False)
    assert pl.select_strategy(70 * GBy, 80 * GBy, 8, 20 * GBy, True) == (pl.STRATEGIES["zero3"], False)
    # 1B: 16 GB < 56 GB -> data parallel; 7B: 112 GB, /8 = 14 GB -> ZeRO-3
    assert pl.select_strategy(1 * GBy, 80 * GBy, 8)[0] == pl.STRATEGIES["dp"]
    assert pl.select_strategy(7 * GBy, 80 * GBy, 8) == (pl.STRATEGIES["zero3"], False)
    # strict inequalities at the boundary: 16P == 0.7 M_d is not "<"
    assert pl.select_strategy(7, 160, 8)[0] == pl.STRATEGIES["zero3"]     # 112 == 0.7 * 160
    assert pl.select_strategy(7, 161, 8)[0] == pl.STRATEGIES["dp"]
    # on a 288 GB device the 7B model fits plain data parallelism (112 GB < 201.6 GB)
    assert pl.select_strategy(7 * GBy, 288 * GBy, 8)[0] == pl.STRATEGIES["dp"]
    assert pl.select_strategy(70 * GBy, 288 * GBy, 8)[0] == pl.STRATEGIES["zero3"]


def test_composed_cost_worked_by_hand(golden):
    """Figure 2's TP(4) x DP(2) on the 70B model, figures worked by hand from Theorems 1-2:
    a device holds a quarter of 1120 GB; its data-parallel All-Reduce moves 2(D-1)/D of a
    quarter of |G| = 140 GB."""
    GBy = 10 ** 9
    P = int(golden["P_70b"])
    T, D = int(golden["fig2_tp_degree"]), int(golden["fig2_dp_degree"])
    assert pl.composed_cost(pl.STRATEGIES["dp"], P, T, D) == (280 * GBy, 35 * GBy)
    # ZeRO-3 across the two groups: 1/8 of the state again, 3 x (1/2) x 35 GB inside the group
    assert pl.composed_cost(pl.STRATEGIES["zero3"], P, T, D) == (140 * GBy, Fraction(105 * GBy, 2))
    # degenerate compositions: no inner strategy is the outer strategy; a single outer
    # device has nobody to synchronise with
    for modes in pl.STRATEGIES.values():
        assert pl.composed_cost(modes, P, 1, 8) == (pl.memory(modes, P, 8), pl.communication(modes, P, 8))
        assert pl.composed_cost(modes, P, 8, 1)[1] == 0
    # sharding fully over the outer group leaves what sharding over all T*D devices leaves
    assert pl.composed_cost(pl.STRATEGIES["zero3"], P, T, D)[0] == pl.memory(pl.STRATEGIES["zero3"], P, T * D)
