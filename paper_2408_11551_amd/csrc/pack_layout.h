// Device-side layout of one "pack", shared by the host code that builds the per-pack metadata
// and by the kernels.
//
// The matrix units multiply 16 x 32 by 32 x NW per instruction (MFMA 16x16x32).  Which of the
// 32 k slots a column of A occupies is free, as long as the left operand (block values) and
// the right operand (rows of B) agree, and columns of a block that hold no stored entry need
// no slot at all.  A pack is a run of consecutive stored blocks of one block row whose
// OCCUPIED columns (those holding a stored entry) number at most 32 together; a block row is
// cut into packs greedily from the left.  Two full blocks make a pack (one instruction per two
// blocks); blocks of a very sparse matrix, with one or two occupied columns each, share an
// instruction by the dozen.  Either way every stored block is multiplied, block by block, by
// the matrix units -- the instruction merely carries as many blocks as fit.
//
// The occupied columns of a pack (ascending: by block, then by column) are dealt round-robin
// to the four 16-lane groups of the wavefront: the j-th goes to lane group j mod 4, position
// j div 4, i.e. k = 8 * (j mod 4) + j div 4.  A pack with n occupied columns then needs only
// ceil(n / 4) B-row loads per lane instead of 8, and only ceil(n / 8) of the four operand
// dwords carry data.
//
// Block values: 64 L elements per pack (2 bytes each for fp16 / bf16, 1 byte for the 8-bit
// types), L = 2, 4 or 8 by the class of the block row (its fullest pack has at most 4 L occupied
// columns, so positions L .. 7 of every lane group are empty in the whole row and are not
// stored).  Lane l = 16 g + i of the wavefront owns elements [L l, L l + L): row i of the block
// row, k slots 8 g .. 8 g + L - 1.  A 16-bit row of class 8 stores 1 KiB per pack, a row of
// class 2 a quarter of that.
//
// Slot table: for every pack, 4 lane groups x L entries of 32 bits; entry [g][kk] is the row
// of B that slot (g, kk) multiplies, or K (one past the last row) for an empty slot.  A lane
// reads its group's L entries with one or two loads.
//
// Per stored block, for the bind-time value scatter only: its block column, its pack (counted
// inside the block row) and a word holding its 16-bit column occupancy mask (low half) and the
// number of occupied columns of the pack that come before it (high half).
#pragma once

#include <cstdint>

#if defined(__HIPCC__)
#define SMAT_HD __host__ __device__
#else
#define SMAT_HD
#endif

namespace smat {

constexpr int kPackColumns = 32;     // k extent of the instruction

// block values stored per pack in a row of class L
SMAT_HD inline int pack_elems(int L) { return 64 * L; }

// index, inside the pack, of the value of row i in slot (g, kk), kk < L
SMAT_HD inline int pack_elem_index(int L, int i, int g, int kk) { return (16 * g + i) * L + kk; }

// slot of the occupied column with rank j (number of occupied columns of the pack before it)
SMAT_HD inline int slot_group(int j) { return j & 3; }
SMAT_HD inline int slot_pos(int j) { return j >> 2; }

}  // namespace smat
