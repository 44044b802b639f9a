// Workgroup id -> work item mappings of the kernels (which tile a workgroup computes).  Plain integer
// functions, usable on the host as well: a host test walks every grid size the launches can have
// and checks that each mapping visits every item exactly once.
#pragma once

#include <hip/hip_runtime.h>

namespace cce {

// Workgroup id -> linear work index such that workgroups resident on one XCD (ids that are
// equal modulo 8 are dispatched to the same XCD) receive consecutive work indices.
__host__ __device__ __forceinline__ int xcd_linear_id(int bid, int nb) {
    const int q = nb >> 3, r = nb & 7;
    const int x = bid & 7, slot = bid >> 3;
    return x * q + (x < r ? x : r) + slot;
}

// The same for grids larger than the number of workgroups resident at once (one per compute
// unit): the mapping is applied inside consecutive rounds of `round` workgroup ids (a
// multiple of 8), so that every XCD receives an equal share of each round instead of one
// contiguous eighth of the whole grid (which would hand all the early -- longest -- work
// items to the first XCDs).
__host__ __device__ __forceinline__ int xcd_round_id(int bid, int nb, int round) {
    const int base = bid - bid % round;
    const int n = (nb - base < round) ? (nb - base) : round;
    return base + xcd_linear_id(bid - base, n);
}

// Two jobs in one grid: the first n1 work items are long (the job with the longer reduction), the
// other n2 short.  Workgroup ids reach the XCDs round robin and
// every XCD starts its own ids in order as its compute units become free, so what an XCD runs is
// the QUEUE of ids congruent to it modulo 8.  Each queue gets an equal share of the long items,
// first, then an equal share of the short ones -- consecutive items of a job stay on one XCD (they
// share an operand band in its L2) -- so that every XCD has short items to back-fill with while its
// long items run.  (Mapping rounds of 256 ids instead hands the first XCDs nothing but long items:
// their queued short items then wait for a whole long reduction while the other XCDs idle --
// measured at N = 16384, D = 2048: 314 us per launch instead of 235.  A grid that fits the machine
// in one round gains too, less: when the short items end, every XCD keeps the same number of long
// ones running instead of four XCDs going idle beside four full ones -- 2.7 % per launch at
// N = 8192, D = 896.)  Needs n1, n2 >= 8.
__host__ __device__ __forceinline__ void xcd_two_job_map(int bid, int n1, int n2, bool& in_first, int& item) {
    const int x = bid & 7, slot = bid >> 3;
    const int q1 = n1 >> 3, r1 = n1 & 7;
    const int c1 = q1 + (x < r1 ? 1 : 0);                 // long items of this XCD
    if (slot < c1) {
        in_first = true;
        item = x * q1 + (x < r1 ? x : r1) + slot;
        return;
    }
    const int n = n1 + n2, q = n >> 3, r = n & 7;
    int before = 0;                                        // short items of the XCDs before this one
    for (int xx = 0; xx < x; ++xx) before += (q + (xx < r ? 1 : 0)) - (q1 + (xx < r1 ? 1 : 0));
    in_first = false;
    item = before + (slot - c1);
}

// Linear index -> (i, j) over an n_i x n_j grid, walking i fastest inside groups of `group`
// consecutive i, then j, then the next group (the last group may be narrower).
__host__ __device__ __forceinline__ void group_map(int lin, int n_i, int n_j, int group, int& i, int& j) {
    const int width = group * n_j;
    const int g = lin / width;
    const int first = g * group;
    const int size = (n_i - first < group) ? (n_i - first) : group;
    const int r = lin - g * width;
    i = first + r % size;
    j = r / size;
}

}  // namespace cce
