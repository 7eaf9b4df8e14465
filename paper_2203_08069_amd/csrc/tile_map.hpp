// Block id -> output tile of a contraction launch.  Shared by the kernels and by the host-only
// planning code (and its sanitizer-built test), hence free of HIP types.
#pragma once
#include <stdint.h>

#ifdef __HIPCC__
#define DISTAL_HOST_DEVICE_INLINE __host__ __device__ __forceinline__
#else
#define DISTAL_HOST_DEVICE_INLINE inline
#endif

namespace distal {

// Block id -> output tile.  Hardware hands consecutive workgroup ids to the 8
// XCDs in turn; give each XCD one contiguous range of logical ids, and walk
// that range in bands of GROUP_M tile rows so that tiles resident together
// share A row-panels and B column-panels in that XCD's L2.  GROUP_M is chosen
// per tile shape so that the tiles resident on one XCD (32 CUs) cover a roughly
// square patch of C, which minimises the operand bytes per flop that miss L2.
template <int GROUP_M>
DISTAL_HOST_DEVICE_INLINE void tile_of_block(int bid, int nblocks, int tiles_m, int tiles_n,
                                              int &tm, int &tn) {
    constexpr int NXCD = 8;
    const int per = nblocks / NXCD, rem = nblocks % NXCD;
    const int x = bid % NXCD, q = bid / NXCD;
    const int p = x * per + (x < rem ? x : rem) + q;
    const int width = GROUP_M * tiles_n;
    const int g = p / width, r = p % width;
    const int first = g * GROUP_M;
    const int gs = (tiles_m - first) < GROUP_M ? (tiles_m - first) : GROUP_M;
    tm = first + r % gs;
    tn = r / gs;
}

}  // namespace distal
