"""The library's communication model (host-only entry points of the C ABI) against the oracle."""
import math
import random
import time

import pytest

from oracle import comm_model as cm
from paper_2502_08145_amd import binding as B


def full_db(g_node, rng):
    return {(inner, size): rng.uniform(50e9, 400e9)
            for inner in range(1, g_node + 1) for size in range(2, g_node + 1) if inner * size <= g_node}


def gpt_layers(hidden, tokens):
    # QKV, attention output, FC1, FC2 of one transformer block; alternate layers are 'transposed'
    return [(tokens, hidden, 3 * hidden, False), (tokens, hidden, hidden, True),
            (tokens, hidden, 4 * hidden, False), (tokens, 4 * hidden, hidden, True)]


def test_layer_terms_and_bandwidths_match_the_oracle():
    rng = random.Random(20250208)
    for _ in range(300):
        g_node = rng.choice([1, 2, 4, 8])
        grid = tuple(rng.choice([1, 2, 3, 4, 6, 8, 16]) for _ in range(4))
        db = full_db(g_node, rng)
        inter = rng.uniform(10e9, 100e9)
        want_b = cm.group_bandwidths(grid, g_node, inter, db)
        got_b = B.axonn_comm_group_bandwidths(grid, g_node, inter, db)
        assert got_b == pytest.approx(want_b, rel=1e-15)
        m, k, n = (rng.randrange(1, 1 << 16) for _ in range(3))
        tr = rng.random() < 0.5
        bpe = rng.choice([1.0, 2.0, 4.0])
        want = cm.layer_comm_time(m, k, n, grid, want_b, bpe, tr)
        got = B.axonn_comm_layer_time(m, k, n, grid, got_b, bpe, tr)
        for key in want:
            assert got[key] == pytest.approx(want[key], rel=1e-13, abs=0.0), (key, grid, tr)


@pytest.mark.parametrize("g_total,g_node", [(1, 8), (8, 8), (12, 4), (64, 4), (96, 8), (1024, 8)])
def test_ranking_matches_the_oracle(g_total, g_node):
    rng = random.Random(g_total * 31 + g_node)
    db = full_db(g_node, rng)
    layers = gpt_layers(8192, 4096) * 3
    want = cm.rank_grids(g_total, layers, g_node, 25e9, db)
    got = B.axonn_comm_rank_grids(g_total, layers, g_node, 25e9, db)
    assert [g for _, g in got] == [g for _, g in want]
    assert [t for t, _ in got] == pytest.approx([t for t, _ in want], rel=1e-12)
    assert B.axonn_comm_rank_grids(g_total, layers, g_node, 25e9, db, top=3) == got[:3]


def test_errors_and_missing_table_entries():
    db = {(1, 2): 1e11}
    with pytest.raises(B.AxonnError):                      # (2, 2) is needed for G_y inside an 8-GPU node
        B.axonn_comm_group_bandwidths((2, 2, 1, 1), 8, 1e10, db)
    with pytest.raises(B.AxonnError):
        B.axonn_comm_group_bandwidths((0, 1, 1, 1), 8, 1e10, db)
    with pytest.raises(B.AxonnError):
        B.axonn_comm_rank_grids(0, [], 8, 1e10, db)
    with pytest.raises(B.AxonnError):
        B.axonn_comm_rank_grids(4, [(8, 8, 8, False)], 8, 1e10, db)   # some grid needs a missing entry
    assert B.axonn_comm_rank_grids(1, [(8, 8, 8, False)], 8, 1e10, {}) == [(0.0, (1, 1, 1, 1))]
    with pytest.raises(B.AxonnError):
        B.axonn_comm_layer_time(8, 8, 8, (2, 1, 1, 1), (0.0, 1, 1, 1))   # a communicating group needs a bandwidth


def test_paper_scale_job_is_ranked_quickly_and_sensibly():
    # 32,768 GPUs in nodes of 8 (the paper's largest runs are of this order): 816 grids
    rng = random.Random(7)
    db = full_db(8, rng)
    layers = gpt_layers(16384, 16384)
    t0 = time.perf_counter()
    rows = B.axonn_comm_rank_grids(32768, layers, 8, 25e9, db)
    t_lib = time.perf_counter() - t0
    assert len(rows) == math.comb(15 + 3, 3) == len(cm.enumerate_grids(32768))
    assert all(rows[i][0] <= rows[i + 1][0] for i in range(len(rows) - 1))
    t0 = time.perf_counter()
    want = cm.rank_grids(32768, layers, 8, 25e9, db)
    t_oracle = time.perf_counter() - t0
    assert [g for _, g in rows[:20]] == [g for _, g in want[:20]]
    print(f"ranking 816 grids x 4 layers: library {t_lib * 1e3:.1f} ms, oracle {t_oracle * 1e3:.1f} ms")
    # pure data parallelism and pure single-axis tensor parallelism are never the best at this scale
    assert rows[0][1] not in [(1, 1, 1, 32768), (32768, 1, 1, 1), (1, 32768, 1, 1), (1, 1, 32768, 1)]
