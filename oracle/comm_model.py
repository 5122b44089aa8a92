"""Plain Python statement of the paper's communication performance model (TEST INFRASTRUCTURE ONLY).

Sec. IV-B of the paper ("performance model" subsection): ring collectives, start-up costs ignored,
so a collective's time is (bytes each process sends) / (bandwidth of its process group).

* layer_comm_time   Eq. 1-5 (the five collectives of one FC layer with an m x k input batch and a
                    k x n weight) and their sum, Eq. 6; a layer with a 'transposed' weight swaps the
                    roles of the X and Y groups.
* group_bandwidths  the bandwidth each of the four process groups sees: groups that fit in a node
                    read it from a profiled table keyed by (product of the inner group sizes, own
                    size); groups that span nodes get Eq. 7, beta_inter / min(G_node, product of the
                    inner group sizes).  Hierarchy, innermost first: X, Y, Z, data.
* enumerate_grids / rank_grids   every ordered factorisation G_x * G_y * G_z * G_data = G, ranked by
                    the summed time over a list of layers.

Everything is written the way the equations read; nothing here is shared with the library.
"""
from __future__ import annotations

import math


def layer_comm_time(m, k, n, grid, beta, bytes_per_element=2.0, transposed=False):
    """Eq. 1-6.  grid = (G_x, G_y, G_z, G_data), beta = (beta_x, beta_y, beta_z, beta_data) in bytes/s.
    Returns a dict with the five terms and 'total' (seconds)."""
    gx, gy, gz, gd = grid
    bx, by, bz, bd = beta
    if transposed:                      # the X and Y groups trade places for this layer
        gx, gy = gy, gx
        bx, by = by, bx
    e = float(bytes_per_element)

    def over(beta_i, g_i, amount):      # a group of one process communicates nothing
        return 0.0 if g_i == 1 else amount / beta_i
    t = {
        "ag_z": over(bz, gz, (gz - 1) * (k * n * e) / (gx * gy * gz)),                 # Eq. 1
        "rs_z": over(bz, gz, ((gz - 1) / gz) * (k * n * e) / (gx * gy)),                # Eq. 2
        "ar_y": over(by, gy, 2.0 * ((gy - 1) / gy) * (m * n * e) / (gz * gx)),          # Eq. 3
        "ar_x": over(bx, gx, 2.0 * ((gx - 1) / gx) * (m * k * e) / (gz * gy)),          # Eq. 4
        "ar_data": over(bd, gd, 2.0 * ((gd - 1) / gd) * (k * n * e) / (gx * gy * gz)),  # Eq. 5
    }
    t["total"] = t["ag_z"] + t["rs_z"] + t["ar_y"] + t["ar_x"] + t["ar_data"]            # Eq. 6
    return t


def group_bandwidths(grid, g_node, beta_inter, intra_db):
    """Bandwidth of the X, Y, Z and data groups.  intra_db maps (inner product, group size) to the
    profiled bandwidth of such a group inside a node."""
    betas = []
    inner = 1
    for g in grid:
        if g == 1:
            betas.append(math.inf)                       # never used: the group does not communicate
        elif inner * g <= g_node:
            betas.append(float(intra_db[(inner, g)]))    # case 1: inside a node, profiled
        else:
            betas.append(beta_inter / min(g_node, inner))  # case 2: Eq. 7
        inner *= g
    return tuple(betas)


def network_comm_time(layers, grid, g_node, beta_inter, intra_db, bytes_per_element=2.0):
    """Sum of Eq. 6 over layers; a layer is (m, k, n, transposed)."""
    beta = group_bandwidths(grid, g_node, beta_inter, intra_db)
    return sum(layer_comm_time(m, k, n, grid, beta, bytes_per_element, tr)["total"] for m, k, n, tr in layers)


def enumerate_grids(g_total):
    """All (G_x, G_y, G_z, G_data) of positive integers with product g_total, in lexicographic order."""
    out = []
    for gx in range(1, g_total + 1):
        if g_total % gx:
            continue
        r1 = g_total // gx
        for gy in range(1, r1 + 1):
            if r1 % gy:
                continue
            r2 = r1 // gy
            for gz in range(1, r2 + 1):
                if r2 % gz:
                    continue
                out.append((gx, gy, gz, r2 // gz))
    return out


def rank_grids(g_total, layers, g_node, beta_inter, intra_db, bytes_per_element=2.0):
    """[(time, grid)] sorted by time, ties by grid."""
    rows = [(network_comm_time(layers, g, g_node, beta_inter, intra_db, bytes_per_element), g)
            for g in enumerate_grids(g_total)]
    rows.sort()
    return rows
