// Host-side arithmetic of the synchronisation subsystem: mirrors of the device index
// functions, the wave model of Section II-A and a small list-scheduling model of a chain that
// the planner uses to choose a macro-tile shape.
#pragma once
#include <stdint.h>

namespace depsync {

// Makespan of a two-stage chain on `slots` workgroup slots.  Stage 1 has gx1*gy1 tiles of
// duration d1, stage 2 gx2*gy2 tiles of duration d2, both issued in row-major order (all
// stage-1 tiles first).  A stage-2 tile of row y reads the stage-1 rows
// [y*rows_ratio - halo, (y+1)*rows_ratio - 1 + halo] (clipped), where rows_ratio = gy1/gy2
// rounded up.  With stream_sync no stage-2 tile is issued before stage 1 has drained; without
// it a tile occupies its slot from issue and starts once the rows it reads are complete.
double simulate_chain(int slots, uint32_t gx1, uint32_t gy1, double d1, uint32_t gx2, uint32_t gy2, double d2,
                      int halo, bool stream_sync);

}  // namespace depsync
