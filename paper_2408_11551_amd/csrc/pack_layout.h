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
// reads its group's L entries with one load (L = 2, 4); with L = 8 a lane fetches one entry of the pack's 32 and the
// lane groups get their eight through the LDS crossbar.
//
// Entry rows.  A block row whose occupied columns hold hardly more than one stored entry each
// (nnz <= 9/8 of the occupied columns, or 3/2 for matrices too large to stay cached; graphs,
// uniformly random matrices) would store sixteen values per column, fifteen of them zero.  Such
// a row is kept by ENTRY instead (row class 3): its stored entries, by ascending column and, inside
// a column, by row of the block row, are cut into packs of 32; entry number j of a pack takes slot (j mod 4, j div 4) like an occupied
// column would.  The pack's slot table names the B row of every entry (a column with two
// entries is named twice) and carries, in the otherwise unused top byte of entries 0..3 of
// every lane group, the eight 4-bit row numbers of the group's entries (entry kk in bits
// 4 kk .. 4 kk + 3 of the 32 bits formed by those four bytes, lowest entry's byte first).  Its
// values are the 32 entry values alone, group by group (8 g + kk), in one 64-byte unit (the
// 8-bit types use half of it) instead of 1 KiB.  The kernel expands
// them into the left operand in registers: lane (g, i) keeps value kk where the row number of
// entry (g, kk) is i and puts zero elsewhere.
//
// Per stored block, for the bind-time value scatter only (not for entry rows): its block column, its pack (counted
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
constexpr int kEntryClass = 3;       // row class of an entry row (classes 0..2: L = 2, 4, 8)

// slot-table units (32 bytes; 128 values) one pack of a row of class cls takes
SMAT_HD inline int pack_units(int cls) { return cls == kEntryClass ? 4 : 1 << cls; }
// row loads per lane and pack
SMAT_HD inline int class_loads(int cls) { return cls == kEntryClass ? 8 : 2 << cls; }
// 64-byte units of block values one pack of a row of class cls takes (elements of es bytes)
SMAT_HD inline int pack_value_units(int cls, int es) { return cls == kEntryClass ? 1 : (2 << cls) * es; }
// index, inside the pack's value area, of the value of entry (g, kk) of an entry row
SMAT_HD inline int entry_elem_index(int g, int kk) { return 8 * g + kk; }

// block values stored per pack in a row of class L
SMAT_HD inline int pack_elems(int L) { return 64 * L; }

// index, inside the pack, of the value of row i in slot (g, kk), kk < L
SMAT_HD inline int pack_elem_index(int L, int i, int g, int kk) { return (16 * g + i) * L + kk; }

// slot of the occupied column with rank j (number of occupied columns of the pack before it)
SMAT_HD inline int slot_group(int j) { return j & 3; }
SMAT_HD inline int slot_pos(int j) { return j >> 2; }

}  // namespace smat
