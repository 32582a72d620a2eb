// Index arithmetic of the dependencies between the tiles of two consecutive stages: which
// semaphore a producer tile posts to under each policy (Fig. 4b of the paper), at which K steps
// of a consumer tile a new group of producer tiles has to be waited for, and which producer
// tiles those are.  Plain integer functions, compiled for the device (the tiles call them) and
// for the host (the planner checks with them that every slice a consumer tile loads is covered
// by a wait issued no later than that slice's K step).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "chain_args.h"

namespace depsync {

__host__ __device__ __forceinline__ uint32_t dm_min(uint32_t a, uint32_t b) { return a < b ? a : b; }
__host__ __device__ __forceinline__ int dm_imin(int a, int b) { return a < b ? a : b; }
__host__ __device__ __forceinline__ int dm_imax(int a, int b) { return a > b ? a : b; }

// Semaphore a producer tile (x,y) posts to / a consumer looks at, per policy (Fig. 4b):
//   row:     sem = y                      value = grid_x
//   tile:    sem = x*grid_y + y           value = 1
//   strided: sem = y*stride + x % stride  value = grid_x / stride
__host__ __device__ __forceinline__ uint32_t policy_sem(uint32_t kind, uint32_t x, uint32_t y, uint32_t grid_y, uint32_t stride) {
    switch (kind) {
        case DEP_TILE:
        case DEP_CONV_TILE:
            return x * grid_y + y;
        case DEP_STRIDED:
        case DEP_ATTN_QKV:
            return y * stride + (x % stride);
        default:
            return y;
    }
}

// Range of producer row tiles and the producer column tile a K step depends on.
struct DepRange {
    uint32_t y0, y1;   // inclusive producer row-tile range
    uint32_t x;        // producer column tile (TILE / STRIDED kinds)
};

// Dependency segments of a consumer tile start at multiples of this many K steps of 64 elements
// (0: only at the first step of the tile's K range).
__host__ __device__ __forceinline__ uint32_t dep_seg_steps(const StageDesc& s) {
    switch (s.dep_kind) {
        case DEP_TILE: case DEP_STRIDED: return s.prod_tn / 64;
        case DEP_CONV_TAPROW: return 3 * s.Cin / 64;
        case DEP_CONV_TILE: {   // starts of filter rows and of producer channel tiles inside them
            uint32_t a = 3 * s.Cin / 64, b = s.prod_tn / 64;
            while (b != 0) { const uint32_t r = a % b; a = b; b = r; }
            return a;
        }
        default: return 0;
    }
}

// Does the A slice of K step kt start a new dependency segment, and on what?
// kb: first K step of this workgroup's K range (0 unless the stage is split along K).
__host__ __device__ __forceinline__ bool dep_segment(const StageDesc& s, uint32_t m0, uint32_t tm, uint32_t kt, uint32_t kb, DepRange& r) {
    const uint32_t m_last = dm_min(m0 + tm, s.M) - 1;
    switch (s.dep_kind) {
        case DEP_ROW:
            if (kt != kb) return false;
            r.y0 = m0 / s.prod_tm; r.y1 = m_last / s.prod_tm; r.x = 0;
            return true;
        case DEP_TILE:
        case DEP_STRIDED: {
            const uint32_t k0 = kt * 64;
            if (k0 % s.prod_tn != 0) return false;
            r.x = k0 / s.prod_tn;
            // same semaphore as x - stride, which this workgroup has already waited for if that
            // segment lies inside its K range
            if (s.dep_kind == DEP_STRIDED && r.x >= s.stride && (r.x - s.stride) * (s.prod_tn / 64) >= kb) return false;
            r.y0 = m0 / s.prod_tm; r.y1 = m_last / s.prod_tm;
            return true;
        }
        case DEP_CONV_ROW: {
            if (kt != kb) return false;
            const int lo = (int)m0 - (int)s.W - 1, hi = (int)m_last + (int)s.W + 1;
            r.y0 = (uint32_t)dm_imax(lo, 0) / s.prod_tm;
            r.y1 = (uint32_t)dm_imin(hi, (int)s.M - 1) / s.prod_tm; r.x = 0;
            return true;
        }
        case DEP_CONV_TAPROW:
        case DEP_CONV_TILE: {
            // K runs filter-row major: k = ((fr*3 + fs) * Cin + c).  A new segment starts with
            // every filter row (TAPROW) or every producer channel tile of a filter row's first tap (TILE).
            const uint32_t k0 = kt * 64;
            const uint32_t tap = k0 / s.Cin, c0 = k0 % s.Cin;
            const uint32_t fr = tap / 3, fs = tap % 3;
            if (fs != 0) return false;
            if (s.dep_kind == DEP_CONV_TAPROW) { if (c0 != 0) return false; r.x = 0; }
            else { if (c0 % s.prod_tn != 0) return false; r.x = c0 / s.prod_tn; }
            const int sh = ((int)fr - 1) * (int)s.W;
            const int lo = (int)m0 + sh - 1, hi = (int)m_last + sh + 1;
            if (hi < 0 || lo > (int)s.M - 1) return false;      // whole filter row is padding
            r.y0 = (uint32_t)dm_imax(lo, 0) / s.prod_tm;
            r.y1 = (uint32_t)dm_imin(hi, (int)s.M - 1) / s.prod_tm;
            return true;
        }
        default:
            return false;
    }
}

}  // namespace depsync
