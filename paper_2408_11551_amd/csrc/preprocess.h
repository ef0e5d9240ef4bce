// Host-side preprocessing: CSR validation, block-column patterns, Jaccard row
// clustering, identity guard and the BCSR structure (paper sections "Blocked
// format", "Data Structures" and "Preprocessing").  Integer work only; no HIP.
#pragma once

#include <cstdint>
#include <string>
#include <vector>

namespace smat {

constexpr int kBlock = 16;   // h = w = 16

struct Csr {
    int64_t M = 0, K = 0;
    std::vector<int64_t> row_ptr;   // [M+1]
    std::vector<int32_t> col_idx;   // [nnz]
    std::vector<uint16_t> vals;     // [nnz] bit patterns (an 8-bit type sits in the low byte)
};

struct Bcsr {
    int64_t nbr = 0, nbc = 0;
    std::vector<int32_t> perm;       // [M] new -> old
    std::vector<int32_t> row_ptr;    // [nbr+1]
    std::vector<int32_t> col_idx;    // [n_e]
    std::vector<uint16_t> col_mask;  // [n_e] bit c set iff column c of the block holds a stored entry
    int64_t n_blocks = 0, n_blocks_identity = 0;
    bool used_identity = true;
    // row + column reordering only (reorder_columns): new column -> old column, identity if unused
    std::vector<int32_t> col_perm;
    int64_t n_blocks_rows_only = 0;
    int64_t n_clusters = 0;
};

// Returns an empty string when the CSR is well formed, else what is wrong.
std::string validate_csr(int64_t M, int64_t K, const int64_t* row_ptr, const int32_t* col_idx);

// Row patterns: ascending block columns floor(c/16) per row, as a CSR-like pair.
void block_patterns(const Csr& a, std::vector<int64_t>& pat_ptr, std::vector<int32_t>& pat_idx);

// Greedy Jaccard clustering; returns the cluster order (new -> old) and the number of clusters.
int64_t jaccard_cluster(int64_t M, int64_t nbc, const std::vector<int64_t>& pat_ptr,
                        const std::vector<int32_t>& pat_idx, int tau_permille,
                        std::vector<int32_t>& order);

// Number of nonzero blocks when rows are read in the order perm on the 16-row grid.
int64_t count_blocks(int64_t M, int64_t nbc, const std::vector<int64_t>& pat_ptr,
                     const std::vector<int32_t>& pat_idx, const int32_t* perm);

// Full pipeline: patterns -> (optional) clustering -> guard -> BCSR structure and column masks.
void build_bcsr(const Csr& a, bool reorder, int tau_permille, Bcsr& out);

// Row + column variant (the one the paper tried next to the row-only reordering, Preprocessing
// section): after build_bcsr, clusters the columns of A' = P A with the same greedy procedure, a
// column's pattern being the block rows it touches, and keeps the column order Q only if P A Q
// has strictly fewer blocks.  If it does, `a` becomes A Q (columns renumbered, ascending inside
// every row), b.col_perm holds Q (new -> old) and the structure of b is rebuilt; returns whether
// it did.
bool reorder_columns(Csr& a, int tau_permille, Bcsr& b);

// Launch order of the block rows, given their cost as a row_ptr-like prefix array
// (cost of row br = cost_ptr[br+1] - cost_ptr[br]).
void work_order(const std::vector<int32_t>& cost_ptr, std::vector<int32_t>& order);

// Canonical block values (row-major 16x16 per block, zero filled) for export.
void fill_canonical_vals(const Csr& a, const Bcsr& b, uint16_t* vals);

}  // namespace smat
