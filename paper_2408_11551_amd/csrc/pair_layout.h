// Device-side layout of one block pair (two consecutive stored blocks of a block row, the
// second one absent at an odd tail), shared by the host code that builds the per-pair
// metadata and by the kernels.
//
// A pair is multiplied as ONE 16 x 32 by 32 x NW contraction (MFMA 16x16x32).  Which of the
// 32 k slots a column of the pair occupies is free, as long as the left operand (block
// values) and the right operand (rows of B) agree.  The layout below puts the OCCUPIED
// columns (those holding a stored entry) first and deals them round-robin to the four
// 16-lane groups of the wavefront: the j-th occupied column (ascending) goes to lane group
// j mod 4, position j div 4, i.e. k = 8 * (j mod 4) + j div 4.  A pair with n occupied
// columns then needs only ceil(n / 4) B-row loads per lane instead of 8, and only
// ceil(n / 8) of the four operand dwords carry data.  Unoccupied columns are all zero in
// the block values and are never fetched from B.
//
// Block values: 512 halves per pair; lane l = 16 g + i of the wavefront owns halves
// [8 l, 8 l + 8): row i of the pair, k slots 8 g .. 8 g + 7.
//
// Metadata: 12 int32 per pair
//   [0] block column of the first block      [1] block column of the second block
//   [2] 32-bit occupancy mask (bit c: column c of the first block, bit 16 + c: of the second)
//   [3] number of occupied columns
//   [4 + 2 g], [5 + 2 g]  for lane group g: eight bytes, byte kk = pair column (0..31) held in
//                         slot (g, kk), or 0xFF if the slot is empty
#pragma once

#include <cstdint>

namespace smat {

constexpr int kPairMetaInts = 12;
constexpr int kPairHalves = 512;

#if defined(__HIPCC__)
#define SMAT_HD __host__ __device__
#else
#define SMAT_HD
#endif

// half index, inside the pair, of row i in slot (g, kk)
SMAT_HD inline int pair_half_index(int i, int g, int kk) { return (16 * g + i) * 8 + kk; }

// slot of the occupied column with rank j (number of occupied columns below it)
SMAT_HD inline int slot_group(int j) { return j & 3; }
SMAT_HD inline int slot_pos(int j) { return j >> 2; }

}  // namespace smat
