"""Pins for the oracle of the communication model (Sec. IV-B, Eq. 1-7): hand-worked values, the
two bandwidth examples the paper walks through, closed forms and counting arguments."""
import math

import pytest

from oracle import comm_model as cm


def test_hand_worked_layer_times():
    # worked by hand from Eq. 1-5 with beta = 1 byte/s and 1 byte per element
    t = cm.layer_comm_time(8, 8, 8, (2, 2, 2, 2), (1, 1, 1, 1), bytes_per_element=1)
    assert (t["ag_z"], t["rs_z"], t["ar_y"], t["ar_x"], t["ar_data"], t["total"]) == (8, 8, 16, 16, 8, 56)
    # asymmetric sizes and group sizes: m=4, k=6, n=10, G=(2,3,1,5)
    t = cm.layer_comm_time(4, 6, 10, (2, 3, 1, 5), (1, 1, 1, 1), bytes_per_element=1)
    assert t["ag_z"] == 0 and t["rs_z"] == 0
    assert t["ar_y"] == pytest.approx(2 * (2 / 3) * 20) and t["ar_x"] == pytest.approx(8) and t["ar_data"] == pytest.approx(16)
    assert t["total"] == pytest.approx(152 / 3)
    # the same layer with a 'transposed' weight: X and Y trade places
    t = cm.layer_comm_time(4, 6, 10, (2, 3, 1, 5), (1, 1, 1, 1), bytes_per_element=1, transposed=True)
    assert t["ar_y"] == pytest.approx(40 / 3) and t["ar_x"] == pytest.approx(16) and t["total"] == pytest.approx(136 / 3)
    # distinct bandwidths land on the right terms
    t = cm.layer_comm_time(8, 8, 8, (2, 2, 2, 2), (2, 4, 8, 16), bytes_per_element=1)
    assert (t["ar_x"], t["ar_y"], t["ag_z"], t["rs_z"], t["ar_data"]) == (8, 4, 1, 1, 0.5)
    # bytes per element and bandwidth scale the way a time must
    a = cm.layer_comm_time(5, 7, 11, (2, 2, 2, 2), (3, 3, 3, 3), 2)["total"]
    assert cm.layer_comm_time(5, 7, 11, (2, 2, 2, 2), (6, 6, 6, 6), 2)["total"] == pytest.approx(a / 2)
    assert cm.layer_comm_time(5, 7, 11, (2, 2, 2, 2), (3, 3, 3, 3), 4)["total"] == pytest.approx(a * 2)
    assert cm.layer_comm_time(5, 7, 11, (1, 1, 1, 1), (3, 3, 3, 3), 2)["total"] == 0


def test_bandwidth_examples_of_the_paper():
    inter = 100.0
    # one group of eight GPUs over two nodes of four: the ring crosses the node boundary once each
    # way and gets the whole inter-node bandwidth
    assert cm.group_bandwidths((8, 1, 1, 1), 4, inter, {})[0] == inter
    # two simultaneous rings of four GPUs across two nodes share it
    assert cm.group_bandwidths((2, 4, 1, 1), 4, inter, {(1, 2): 55.0})[:2] == (55.0, inter / 2)
    # never divided by more than the GPUs of a node
    assert cm.group_bandwidths((4, 4, 4, 1), 4, inter, {(1, 4): 70.0})[:3] == (70.0, inter / 4, inter / 4)
    # groups inside a node read the profiled table at (product of the inner sizes, own size)
    db = {(1, 2): 10.0, (2, 2): 20.0, (4, 2): 30.0, (1, 4): 40.0, (2, 4): 50.0, (1, 8): 60.0}
    assert cm.group_bandwidths((2, 2, 2, 2), 8, inter, db) == (10.0, 20.0, 30.0, inter / 8)
    assert cm.group_bandwidths((1, 4, 2, 1), 8, inter, db) == (math.inf, 40.0, 30.0, math.inf)
    assert cm.group_bandwidths((1, 1, 8, 4), 8, inter, db) == (math.inf, math.inf, 60.0, inter / 8)


def test_enumeration_counts_and_products():
    # ordered factorisations into 4 factors: prod over primes of C(e + 3, 3)
    for g, count in [(1, 1), (2, 4), (8, 20), (12, 40), (64, 84), (36, 100)]:
        grids = cm.enumerate_grids(g)
        assert len(grids) == count == len(set(grids))
        assert all(a * b * c * d == g for a, b, c, d in grids)
        assert grids == sorted(grids)


def test_ranking_closed_form_with_two_gpus():
    # G = 2, one layer, equal bandwidths b: the four grids cost m k (X), m n (Y), k n (Z: all-gather
    # plus reduce-scatter) and k n (data), times bytes / b
    m, k, n, b = 3, 5, 7, 2.0
    db = {(1, 2): b}
    rows = cm.rank_grids(2, [(m, k, n, False)], 8, 1.0, db, bytes_per_element=1)
    assert [g for _, g in rows] == [(2, 1, 1, 1), (1, 2, 1, 1), (1, 1, 1, 2), (1, 1, 2, 1)]
    assert [t for t, _ in rows] == pytest.approx([m * k / b, m * n / b, k * n / b, k * n / b])
    # a transposed layer swaps the first two
    rows = cm.rank_grids(2, [(m, k, n, True)], 8, 1.0, db, bytes_per_element=1)
    assert [g for _, g in rows][:2] == [(1, 2, 1, 1), (2, 1, 1, 1)]
    # the network time is the sum over layers: the plain layer pays the X all-reduce on m x k, the
    # transposed layer (weight n x k) uses the X group as its Y group: all-reduce on m x k again
    both = cm.network_comm_time([(m, k, n, False), (m, n, k, True)], (2, 1, 1, 1), 8, 1.0, db, 1)
    assert both == pytest.approx(2 * m * k / b)
