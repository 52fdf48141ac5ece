"""Pins for the request-count model of Section 4.5 (no GPU)."""
import os

import numpy as np

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))


def _golden():
    g = {}
    for line in open(os.path.join(HERE, "golden", "fig4_fig5_requests.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        g[k] = [int(x) for x in v]
    return g


def test_paper_example_seven_requests_become_five():
    g = _golden()
    rows = g["nodes"]
    D, E, W, L = g["features"][0], g["elem_bytes"][0], g["warp_threads"][0], g["line_bytes"][0]
    i = g["highlighted_output_row"][0]
    assert oracle.count_requests(rows, None, D, E, W, L, i, i + 1) == g["requests_unmodified"][0]
    s = [oracle.circular_shift(k, r, D, L // E) for k, r in enumerate(rows)]
    assert s[i] == g["shift_of_highlighted_row"][0]
    assert oracle.count_requests(rows, s, D, E, W, L, i, i + 1) == g["requests_shifted"][0]


def test_aligned_rows_need_no_shift_and_cost_the_line_count():
    # D*E a multiple of the line: every row is aligned, shift 0, requests = D*E/L per row
    rows = [5, 0, 9, 9]
    D, E, W, L = 8, 4, 4, 16
    assert [oracle.circular_shift(i, r, D, L // E) for i, r in enumerate(rows)] == [0, 0, 0, 0]
    assert oracle.count_requests(rows, None, D, E, W, L) == len(rows) * (D * E // L)


def test_shift_aligns_lanes_with_lines_and_never_costs_more():
    rng = np.random.default_rng(3)
    D, E, W, L = 11, 4, 4, 16
    rows = rng.integers(0, 50, size=12).tolist()
    s = [oracle.circular_shift(i, r, D, L // E) for i, r in enumerate(rows)]
    naive = oracle.count_requests(rows, None, D, E, W, L)
    fixed = oracle.count_requests(rows, s, D, E, W, L)
    assert fixed <= naive
    # each lane's address is congruent to its lane number modulo the line
    for i, r in enumerate(rows):
        for j in range(D):
            if j + s[i] < D:            # lanes that do not wrap around the row end
                assert (r * D + j + s[i]) % (L // E) == (i * D + j) % (L // E)


def test_empty_range_counts_zero():
    assert oracle.count_requests([1, 2], None, 4, 4, 4, 16, 1, 1) == 0
