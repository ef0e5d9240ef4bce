// Device-side data layout and kernel launchers (gfx950).  Host code includes this
// header without needing hipcc; streams travel as void*.
#pragma once

#include <cstddef>
#include <cstdint>

namespace smat {

// Pointers into the caller's device workspace.  See pack_layout.h for packs, their values and
// their slot tables.
struct DeviceBcsr {
    const int32_t* perm = nullptr;       // [nbr*16] new row -> old row, -1 beyond M
    // Launch table, one record of four words per workgroup of the per-row kernel, in launch
    // order: block row | row class << 28, number of packs, start of the row's slot table in
    // 32-byte units, start of its values in 64-byte units.
    const int32_t* work = nullptr;       // [4 * n_order]
    int64_t n_order = 0;                 // rows the per-row kernel is launched for
    const uint32_t* slots = nullptr;     // slot tables: per pack 4 groups x L entries (L by row class)
    const void* vals = nullptr;          // block values: per pack 64 L elements of 2 bytes (fp16, bf16) or 1 byte;
                                         // entry rows: the pack's 32 entry values in one 64-byte unit
    // bind-time value scatter only
    const int32_t* pack_ptr = nullptr;   // [nbr+1] pack offsets per block row
    const uint32_t* vals_off = nullptr;  // [nbr+1] start of the row's values, 64-byte units
    const int8_t* row_class = nullptr;   // [nbr] 0..2: packs of occupied columns with L = 2, 4, 8; 3: entry row
    const int32_t* blk_ptr = nullptr;    // [nbr+1] stored-block offsets per block row
    const int32_t* blk_col = nullptr;    // [n_blocks] block column, ascending inside a block row
    const int32_t* blk_pack = nullptr;   // [n_blocks] pack of the block, counted inside its block row
    const uint32_t* blk_meta = nullptr;  // [n_blocks] occupancy mask | occupied columns of the pack before the block << 16
    int64_t M = 0, K = 0, nbr = 0;
    int64_t n_packs = 0;                 // packs of the rows in the launch table
    int64_t stream_bytes = 0;            // values + slot tables of those rows
    int64_t b_rows = 0;                  // slots of those rows that name a row of B (each fetched once per column slab)
    int64_t max_row_packs = 0;           // longest block row
    double mean_row_packs = 0;
    int max_class = 0;                   // highest row class present (0: <=8, 1: <=16, 2: <=32 occupied columns per pack, 3: entry rows)
};

// Block-dense parts of the matrix: "super rows" of sixteen consecutive block rows whose block
// columns overlap enough to be walked together (kernels_dense.hip).  The union of a super
// row's block columns, ascending, is cut into steps of cols_per_step block columns (two for the
// 16-bit types = the 32 k slots of one MFMA; four for the 8-bit types = two MFMAs); step q stores
// 1 KiB for every block row that has one of its columns (bit j of step_rows), back to back from
// slot step_base[q].
struct DenseTiles {
    const int32_t* super_rows = nullptr;   // [n] super row index s: block rows 16 s .. 16 s + 15
    const int32_t* step_ptr = nullptr;     // [n+1] offsets into the step arrays
    const int32_t* step_cols = nullptr;    // [cols_per_step * steps] block columns of a step (INT_MAX: none)
    const uint32_t* step_rows = nullptr;   // [steps] 16-bit mask of block rows present in the step
    const uint32_t* step_base = nullptr;   // [steps] first slot of the step
    const void* vals = nullptr;            // [1024 bytes * slots]
    void* scratch = nullptr;               // partial tiles (fp32, or int32 for the integer type) of launches that split the steps of a tile
    size_t scratch_bytes = 0;
    int32_t n = 0;
    double mean_steps = 0;                 // steps per super row, on average
    int cols_per_step = 2;
    bool all_full = false;                 // every step has all sixteen block rows and the block columns 2q, 2q+1 (8-bit types:
                                           // 4q .. 4q+3; q counted inside the super row) and every super row has full_steps
                                           // steps: step q of super row i is step i full_steps + q and its values start at slot
                                           // 16 (i full_steps + q), so the kernel needs none of the step tables
    int32_t full_steps = 0;
};

// Sets n16 16-byte words at dst to zero.
int launch_fill_zero(void* dst, size_t n16, void* stream);

// Scatters the CSR values into the device block layout.  csr_* are device copies of the
// caller's CSR (values as 16-bit words, 8-bit types in the low byte); vals_out holds elements
// of elem_bytes (1 or 2) and must have been zeroed.
int launch_bcsr_fill(const DeviceBcsr& d, const int64_t* csr_row_ptr, const int32_t* csr_col_idx,
                     const uint16_t* csr_vals, void* vals_out, int elem_bytes, void* stream);

// C = A * B.  dtype is a smat_dtype_t; C holds fp32, or int32 for the integer type.  Returns
// a hipError_t as int; *variant receives a static string naming the kernel.
int launch_spmm(const DeviceBcsr& d, int dtype, const void* B, int64_t ldb, void* C, int64_t ldc,
                int64_t N, void* stream, const char** variant);
// The variant for matrices with entry rows at N <= 16, fp16 and bf16 (kernels_narrow.hip).
// Returns kNotNarrow where it does not apply (other types, wider or odd N above 8, no entry rows).
constexpr int kNotNarrow = -1;
int launch_spmm_narrow(const DeviceBcsr& d, int dtype, const void* B, int64_t ldb, void* C, int64_t ldc,
                       int64_t N, void* stream, const char** variant);
// the 8-bit types (kernels_8bit.hip, compiled once per type)
int launch_spmm_e4m3(const DeviceBcsr& d, const void* B, int64_t ldb, void* C, int64_t ldc,
                     int64_t N, void* stream, const char** variant);
int launch_spmm_e5m2(const DeviceBcsr& d, const void* B, int64_t ldb, void* C, int64_t ldc,
                     int64_t N, void* stream, const char** variant);
int launch_spmm_i8(const DeviceBcsr& d, const void* B, int64_t ldb, void* C, int64_t ldc,
                   int64_t N, void* stream, const char** variant);

// Scatters the CSR values of the dense super rows into the tile layout (vals zeroed before).
int launch_dense_fill(const DeviceBcsr& d, const DenseTiles& t, const int64_t* csr_row_ptr,
                      const int32_t* csr_col_idx, const uint16_t* csr_vals, void* vals_out, int elem_bytes, void* stream);

// Workgroups per 128-column tile the dense launch would use for this N (1: no split).
int dense_split(const DenseTiles& t, int64_t N);

// The library's own area for partial tiles on the CURRENT device (a static device array, the same
// for every handle and stream): its device address and size.  The first call on a device looks
// the address up.  Returns a hipError_t as int.
int static_tile_scratch(void** area, size_t* bytes);

// C rows of the dense super rows.  dtype is a smat_dtype_t.  Needs N and ldb multiples of the
// elements in 16 bytes (8, or 16 for the 8-bit types) and B aligned to 16 bytes.
int launch_spmm_dense(const DeviceBcsr& d, const DenseTiles& t, int dtype, const void* B, int64_t ldb,
                      void* C, int64_t ldc, int64_t N, void* stream, const char** variant);

// The canonical BCSR of the paper on the device (Data Structures section), for the ablation
// kernels only (ablation.hip).
struct CanonicalBcsr {
    const int32_t* row_ptr = nullptr;    // [nbr+1]
    const int32_t* col_idx = nullptr;    // [n_blocks]
    const uint16_t* vals = nullptr;      // [n_blocks * 256] row-major 16x16 blocks
    const int32_t* block_map = nullptr;  // [nbr * nbc] index of the stored block or -1 (level 0 only)
    const int32_t* perm = nullptr;       // [nbr*16] new row -> old row, -1 beyond M
    int64_t M = 0, K = 0, nbr = 0, nbc = 0;
};

// level 0: every block of the grid is visited and looked up in block_map, scalar multiply-adds;
// level 1: rowPtr / col iteration, scalar multiply-adds; level 2: rowPtr / col iteration and
// one MFMA 16x16x16 per stored block.  fp16 / bf16, C fp32.
int launch_ablation(const CanonicalBcsr& m, int level, bool bf16, const void* B, int64_t ldb, float* C,
                    int64_t ldc, int64_t N, void* stream);

}  // namespace smat
