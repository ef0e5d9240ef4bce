// Device-side data layout and kernel launchers (gfx950).  Host code includes this
// header without needing hipcc; streams travel as void*.
#pragma once

#include <cstddef>
#include <cstdint>

namespace smat {

// Pointers into the caller's device workspace.  Block rows are padded to an even number of
// blocks; pair P of the whole matrix covers blocks 2P and 2P+1.  See pair_layout.h for the
// layout of a pair's values and metadata.
struct DeviceBcsr {
    const int32_t* perm = nullptr;       // [nbr*16] new row -> old row, -1 beyond M
    const int32_t* row_ptr = nullptr;    // [nbr+1] block offsets (even)
    const int32_t* order = nullptr;      // [nbr] block rows, longest first; bits 28..29: row class
    const uint32_t* slots_off = nullptr; // [nbr] start of the row's slot table, in 32-byte units
    const uint32_t* slots = nullptr;     // slot tables: per pair 4 groups x L entries (L by row class)
    const uint16_t* vals = nullptr;      // [256*n_e]
    const int32_t* blk_col = nullptr;    // [n_e] block column per (padded) block; bind-time scatter only
    const uint32_t* occ = nullptr;       // [n_e/2] occupancy mask per pair; bind-time scatter only
    int64_t M = 0, K = 0, nbr = 0, n_e = 0;
    int64_t max_row_blocks = 0;          // longest block row
    double mean_row_blocks = 0;
    int max_class = 0;                   // highest row class present (0: <=8, 1: <=16, 2: <=32 occupied columns per pair)
};

// Sets n16 16-byte words at dst to zero.
int launch_fill_zero(void* dst, size_t n16, void* stream);

// Scatters the CSR values into the device block layout.  csr_* are device copies of the
// caller's CSR; vals must have been zeroed.
int launch_bcsr_fill(const DeviceBcsr& d, const int64_t* csr_row_ptr, const int32_t* csr_col_idx,
                     const uint16_t* csr_vals, uint16_t* vals_out, void* stream);

// C = A * B.  Returns a hipError_t as int; *variant receives a static string naming the kernel.
int launch_spmm(const DeviceBcsr& d, bool bf16, const void* B, int64_t ldb, float* C, int64_t ldc,
                int64_t N, void* stream, const char** variant);

}  // namespace smat
