// Communication performance model of the 4D-parallel method (paper Sec. IV-B, Eq. 1-7): host-only
// arithmetic that ranks the grids G_x x G_y x G_z x G_data a job of G GPUs could use by the time
// their collectives take.  It tells a multi-GPU deployment which shard shapes the GEMM kernels of
// this library will be asked for.  No GPU is touched.
#pragma once
#include <stdint.h>

#include <algorithm>
#include <cmath>
#include <vector>

#include "../../include/axonn_linear.h"

namespace axonn {

// Eq. 1-5 and their sum (Eq. 6) for one layer: out = {ag_z, rs_z, ar_y, ar_x, ar_data, total}.
inline void comm_layer_terms(const axonn_comm_layer_t& L, const int grid[4], const double beta[4],
                             double bytes_per_element, double out[6]) {
    double gx = grid[0], gy = grid[1];
    const double gz = grid[2], gd = grid[3];
    double bx = beta[0], by = beta[1];
    const double bz = beta[2], bd = beta[3];
    if (L.transposed) {   // a layer with a 'transposed' weight uses the X groups as Y groups and vice versa
        std::swap(gx, gy);
        std::swap(bx, by);
    }
    const double m = (double)L.m, k = (double)L.k, n = (double)L.n, e = bytes_per_element;
    out[0] = gz > 1 ? (gz - 1) * (k * n * e) / (gx * gy * gz) / bz : 0.0;
    out[1] = gz > 1 ? ((gz - 1) / gz) * (k * n * e) / (gx * gy) / bz : 0.0;
    out[2] = gy > 1 ? 2.0 * ((gy - 1) / gy) * (m * n * e) / (gz * gx) / by : 0.0;
    out[3] = gx > 1 ? 2.0 * ((gx - 1) / gx) * (m * k * e) / (gz * gy) / bx : 0.0;
    out[4] = gd > 1 ? 2.0 * ((gd - 1) / gd) * (k * n * e) / (gx * gy * gz) / bd : 0.0;
    out[5] = out[0] + out[1] + out[2] + out[3] + out[4];
}

// Bandwidth of each process group (hierarchy X, Y, Z, data, innermost first): profiled table inside
// a node, Eq. 7 across nodes.  false if the table lacks an entry that is needed.
inline bool comm_group_bandwidths(const int grid[4], int g_node, double beta_inter, const double* intra_bw,
                                  double beta[4]) {
    int64_t inner = 1;
    for (int i = 0; i < 4; ++i) {
        const int64_t g = grid[i];
        if (g == 1) {
            beta[i] = HUGE_VAL;   // the group does not communicate
        } else if (inner * g <= g_node) {
            const double b = intra_bw ? intra_bw[inner * (g_node + 1) + g] : 0.0;
            if (!(b > 0.0)) return false;
            beta[i] = b;
        } else {
            beta[i] = beta_inter / (double)std::min<int64_t>(g_node, inner);
        }
        inner *= g;
    }
    return true;
}

}  // namespace axonn
