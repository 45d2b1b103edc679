// Which bytes the streaming buffer loads of the row kernels may address.
//
// A row is read as nq 16-byte vectors from the 16-byte aligned address at or below its first element
// (elements of the first and last vector that lie outside the row are masked after the load).  The
// compress and residual kernels read groups of consecutive vectors with raw buffer loads through ONE
// descriptor per row (base = that aligned address, stride 0, size = nq * 16 bytes): the group's first
// vector goes into the instruction's scalar offset, a lane's vector within the group into the per-lane
// offset.  On gfx950 such a load (stride 0, no swizzle) is in range iff
//     scalar offset + per-lane offset + 16 <= size
// (both offsets take part in the comparison: measured with loads whose addresses all lie inside one
// allocation, and tested on the device at hand by picospec_check_device()); a lane out of range reads
// zero and touches no memory.  So nothing behind the row's last vector is ever addressed, whatever group a
// look-ahead load asks for.  The functions below state which group a load names; the kernels and the
// host-side check picospec_max_load_byte() both use them, so the check covers what the kernels do.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace picospec {

#ifndef PICOSPEC_COMPRESS_THREADS
#define PICOSPEC_COMPRESS_THREADS 512
#endif
#ifndef PICOSPEC_COMPRESS_RING
#define PICOSPEC_COMPRESS_RING 4
#endif
#ifndef PICOSPEC_SMALL_BF16_RING
#define PICOSPEC_SMALL_BF16_RING 5
#endif

constexpr int kCompressThreads = PICOSPEC_COMPRESS_THREADS;   // one workgroup per row
constexpr int kCompressSample = 8192;                         // elements of the sample that places the threshold
constexpr int kResidualThreads = 1024;                        // one workgroup per sequence
constexpr int kResidualTile = 16384;                          // elements per tile (both dtypes)

// the raw buffer load as the hardware executes it: the end, in bytes from the descriptor's base, of what a lane
// reads (0: out of range, no access)
__host__ __device__ inline int64_t buffer_lane_read_end(int64_t size, int64_t scalar_off, int64_t lane_off) {
    return scalar_off + lane_off + 16 <= size ? scalar_off + lane_off + 16 : 0;
}

// SMALL: the variant for short records (three workgroups per CU: fewer registers, a sub-tile of 8 elements per thread)
template <bool BF16, bool SMALL>
struct CompressGeom {
    static constexpr int N = BF16 ? 8 : 4;                                                   // elements per vector
    static constexpr int SV = (BF16 && SMALL) ? 1 : 2;                                       // vectors per thread and sub-tile
    static constexpr int SUB_VECS = kCompressThreads * SV;                                   // vectors per sub-tile
    static constexpr int RING = (BF16 && SMALL) ? PICOSPEC_SMALL_BF16_RING : PICOSPEC_COMPRESS_RING * (2 / SV);            // sub-tile buffers (look-ahead depth)
    static_assert(kCompressSample % (SUB_VECS * N) == 0, "the sample is a whole number of sub-tiles");
    // first vector of group j (one vector per thread: thread tid takes vector tid of the group) of sub-tile `sub`
    __host__ __device__ static int group_first(int sub, int j) { return sub * SUB_VECS + j * kCompressThreads; }
};

template <bool BF16>
struct ResidualGeom {
    static constexpr int N = BF16 ? 8 : 4;
    static constexpr int NV = kResidualTile / (kResidualThreads * N);     // vectors per thread and tile
    static constexpr int TILE_VECS = kResidualThreads * NV;
    static constexpr int SEG_VECS = NV * 64;                              // a wave's consecutive vectors within a tile
    static constexpr int AHEAD = 3;                                       // tiles in registers (one in use, two in flight)
    // first vector of load jv (64 vectors, one per lane) of wave `wave` in tile `it`
    __host__ __device__ static int group_first(int it, int wave, int jv) { return it * TILE_VECS + wave * SEG_VECS + jv * 64; }
};

}  // namespace picospec
