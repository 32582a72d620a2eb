// Host mirrors of the device index arithmetic (Fig. 4b of the paper), the wave model
// (Section II-A, Table I) and the schedule model used by the planner.
#include "host_model.h"

#include <algorithm>
#include <queue>
#include <vector>

#include "../../include/depsync.h"

namespace depsync {

double simulate_chain(int slots, uint32_t gx1, uint32_t gy1, double d1, uint32_t gx2, uint32_t gy2, double d2,
                      int halo, bool stream_sync) {
    if (slots <= 0) return 0.0;
    std::priority_queue<double, std::vector<double>, std::greater<double>> free_at;
    for (int i = 0; i < slots; ++i) free_at.push(0.0);
    std::vector<double> row_done(gy1, 0.0);
    double end1 = 0.0;
    for (uint32_t y = 0; y < gy1; ++y)
        for (uint32_t x = 0; x < gx1; ++x) {
            double t = free_at.top(); free_at.pop();
            t += d1;
            free_at.push(t);
            row_done[y] = std::max(row_done[y], t);
            end1 = std::max(end1, t);
        }
    const uint32_t ratio = gy2 ? (gy1 + gy2 - 1) / gy2 : 1;
    double end = end1;
    for (uint32_t y = 0; y < gy2; ++y) {
        const int lo = std::max<int>(0, (int)(y * ratio) - halo);
        const int hi = std::min<int>((int)gy1 - 1, (int)((y + 1) * ratio) - 1 + halo);
        double ready = 0.0;
        for (int r = lo; r <= hi; ++r) ready = std::max(ready, row_done[r]);
        for (uint32_t x = 0; x < gx2; ++x) {
            double t = free_at.top(); free_at.pop();
            if (stream_sync) t = std::max(t, end1);
            t = std::max(t, ready) + d2;
            free_at.push(t);
            end = std::max(end, t);
        }
    }
    return end;
}

}  // namespace depsync

using depsync::simulate_chain;

extern "C" {

int depsync_row_major(int tile_x, int tile_y, int grid_x, int grid_y) {
    (void)grid_y;
    return tile_y * grid_x + tile_x;
}

int depsync_policy_sem(depsync_policy_kind kind, int tile_x, int tile_y, int grid_x, int grid_y, int stride) {
    (void)grid_x;
    switch (kind) {
        case DEPSYNC_TILESYNC: return tile_x * grid_y + tile_y;
        case DEPSYNC_ROWSYNC: return tile_y;
        case DEPSYNC_STRIDEDSYNC: return stride > 0 ? tile_y * stride + tile_x % stride : DEPSYNC_EINVAL;
        default: return DEPSYNC_EINVAL;
    }
}

int depsync_policy_value(depsync_policy_kind kind, int grid_x, int grid_y, int stride) {
    (void)grid_y;
    switch (kind) {
        case DEPSYNC_TILESYNC: return 1;
        case DEPSYNC_ROWSYNC: return grid_x;
        case DEPSYNC_STRIDEDSYNC: return stride > 0 ? grid_x / stride : DEPSYNC_EINVAL;
        default: return DEPSYNC_EINVAL;
    }
}

int depsync_wave_model(int n_tiles, int occupancy, int n_cu, int* waves, double* utilization) {
    if (n_tiles < 0 || occupancy <= 0 || n_cu <= 0 || !waves || !utilization) return DEPSYNC_EINVAL;
    const int per_wave = occupancy * n_cu;
    *waves = (n_tiles + per_wave - 1) / per_wave;
    *utilization = *waves ? (double)n_tiles / ((double)*waves * per_wave) : 0.0;
    return DEPSYNC_OK;
}

int depsync_sync_count(depsync_policy_kind kind, int prod_grid_x, int prod_grid_y, int cons_grid_x, int cons_grid_y,
                       int prod_rows_per_cons_row) {
    (void)prod_grid_y;
    if (prod_rows_per_cons_row <= 0) return DEPSYNC_EINVAL;
    const int n_cons = cons_grid_x * cons_grid_y;
    switch (kind) {
        case DEPSYNC_TILESYNC: return n_cons * prod_rows_per_cons_row * prod_grid_x;
        case DEPSYNC_ROWSYNC: return n_cons * prod_rows_per_cons_row;
        default: return DEPSYNC_EINVAL;
    }
}

// Exposed for tests of the planner's schedule model.
double depsync_simulate_chain(int slots, int gx1, int gy1, double d1, int gx2, int gy2, double d2, int halo,
                              int stream_sync) {
    return simulate_chain(slots, gx1, gy1, d1, gx2, gy2, d2, halo, stream_sync != 0);
}

}  // extern "C"
