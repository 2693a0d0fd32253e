// Packed (MFMA-fragment order) operand layout shared by the recurrent kernel files (internal).
//
// For every 64-wide K chunk of a tile an operand is stored in the order the 32x32x16 MFMA consumes
// it: [k-step of 16][32-row block][lane][8 elements], lane = 32 * (k half) + row, zero-padded to whole
// tiles; a wavefront load instruction reads one contiguous kilobyte straight into the registers (or
// the LDS bytes) the MFMA takes it from.
#pragma once
#include "common.h"

namespace lstm {

constexpr int TM = 64;                 // rows of one packed A tile
constexpr int NBLK = 4;                // 32-row blocks of one packed B tile
constexpr int TN = NBLK * 32;          // rows of one packed B tile
constexpr int SK = 64;                 // K elements per packed chunk
constexpr int A_CHUNK = TM * SK;       // elements of one packed A chunk (8 KB)
constexpr int B_CHUNK = TN * SK;       // elements of one packed B chunk (16 KB)

// offset of element (row, kk) inside a packed chunk whose rows form `nblk` blocks of 32
__host__ __device__ inline int frag_offset(int row, int kk, int nblk) {
    const int blk = row >> 5, r = row & 31, ks = kk >> 4, half = (kk >> 3) & 1, j = kk & 7;
    return (((ks * nblk + blk) * 64) + half * 32 + r) * 8 + j;
}

// linear tile index with workgroups of one XCD (id % 8) on neighbouring tiles,
// so that tiles sharing B rows share that XCD's L2
__device__ __forceinline__ int xcd_swizzle(int wg, int total) {
    return (total % 8 == 0) ? (wg % 8) * (total / 8) + wg / 8 : wg;
}

}  // namespace lstm
