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
// Block values: 64 L halves per pair, L = 2, 4 or 8 by the class of the block row (the most
// occupied pair of the row has at most 4 L occupied columns, so positions L .. 7 of every
// lane group are empty in the whole row and are not stored).  Lane l = 16 g + i of the
// wavefront owns halves [L l, L l + L): row i of the pair, k slots 8 g .. 8 g + L - 1.  A row
// of class 8 stores the full 16 x 32 values of each pair (1 KiB), a row of class 2 a quarter.
//
// Slot table: for every pair, 4 lane groups x L entries of 32 bits; entry [g][kk] is the row of B that slot (g, kk) multiplies, or K (one past the
// last row) for an empty slot.  A lane reads its group's L entries with one or two loads.
// Two more arrays serve the bind-time value scatter only: the block column of every block
// and the pair's 32-bit occupancy mask (bit c: column c of the first block, bit 16 + c: of
// the second).
#pragma once

#include <cstdint>

#if defined(__HIPCC__)
#define SMAT_HD __host__ __device__
#else
#define SMAT_HD
#endif

namespace smat {

// halves of block values stored per pair in a row of class L
SMAT_HD inline int pair_halves(int L) { return 64 * L; }

// half index, inside the pair, of row i in slot (g, kk), kk < L
SMAT_HD inline int pair_half_index(int L, int i, int g, int kk) { return (16 * g + i) * L + kk; }

// slot of the occupied column with rank j (number of occupied columns below it)
SMAT_HD inline int slot_group(int j) { return j & 3; }
SMAT_HD inline int slot_pos(int j) { return j >> 2; }

}  // namespace smat
