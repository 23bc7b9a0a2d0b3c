// Which head tile and which place inside its set of workgroups a workgroup id of a streaming GQA launch stands
// for (see StreamSeat in common.hpp).  Plain arithmetic, shared by the kernels and the host-side checks.
#pragma once
#include <cstdint>

#if defined(__HIPCC__)
#define HELIX_HOST_DEVICE __host__ __device__
#else
#define HELIX_HOST_DEVICE
#endif

namespace helix {

struct SeatOf {
    int ht, wg;
};

// A launch of head_tiles sets of n_base workgroups.  With n_base a multiple of 8 the ids are dealt in groups of
// 8 * head_tiles: 8 consecutive ids to head tile 0, the next 8 to head tile 1, ... -- the workgroups with the same
// place in their sets are then 8 ids apart, i.e. on the same XCD (consecutive ids go round robin over the 8 XCDs).
// Otherwise (launches with little work) set after set.
HELIX_HOST_DEVICE inline SeatOf seat_of(int id, int head_tiles, int n_base)
{
    SeatOf s;
    if ((n_base & 7) == 0) {
        const int grp = id / (8 * head_tiles), in = id - grp * 8 * head_tiles;
        s.ht = in >> 3;
        s.wg = grp * 8 + (in & 7);
    } else {
        s.ht = id / n_base;
        s.wg = id - s.ht * n_base;
    }
    return s;
}

}  // namespace helix
