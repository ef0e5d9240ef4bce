// C ABI of the library (see include/smat.h): handle management, argument checks,
// host <-> device copies.  All arithmetic of the method lives in preprocess.cpp
// (host, integers) and kernels.hip (device).
#include "../../include/smat.h"

#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "kernels.h"
#include "pair_layout.h"
#include "preprocess.h"

struct smat_handle {
    smat::Csr csr;
    smat::Bcsr bcsr;
    smat_dtype_t dtype = SMAT_F16;
    bool bound = false;
    // Device-side block arrays pad every block row to an even number of blocks (the kernel
    // multiplies blocks two at a time); the pad block has no occupied column and zero values.
    std::vector<int32_t> dev_row_ptr;    // [nbr+1] offsets into the padded block arrays
    int64_t n_dev_blocks = 0;
    // Row class: how many B-row loads per lane a pair of the block row needs at most (occupied
    // columns are dealt to four lane groups): 2, 4 or 8 -> class 0, 1, 2.  The slot table of a
    // row takes 16 * L bytes per pair; slots_off counts 32-byte units.
    std::vector<int8_t> row_class;       // [nbr]
    std::vector<uint32_t> slots_off;     // [nbr+1]; also locates the row's block values (256 bytes per unit)
    uint64_t slots_units = 0;
    int max_class = 0;
    // Dense path (kernels.h, DenseTiles): complete super rows of sixteen block rows whose block
    // columns overlap enough.  row_dense marks the block rows it covers.
    std::vector<int32_t> dense_super, step_ptr, step_cols;
    std::vector<uint32_t> step_rows, step_base;
    std::vector<uint8_t> row_dense;      // [nbr]
    uint64_t dense_slots = 0;
    smat::DeviceBcsr dev;                // launch over every block row
    smat::DeviceBcsr dev_rest;           // launch over the block rows the dense path does not cover
    smat::DenseTiles tiles;
    // device copies of the CSR (kept: they live in the caller's workspace anyway)
    const int64_t* d_csr_row_ptr = nullptr;
    const int32_t* d_csr_col_idx = nullptr;
    const uint16_t* d_csr_vals = nullptr;
};

namespace {

thread_local std::string g_error;
thread_local const char* g_kernel = "";

smat_status_t fail(smat_status_t st, const std::string& msg)
{
    g_error = msg;
    return st;
}

smat_status_t hip_fail(const char* what, int err)
{
    return fail(SMAT_ERR_HIP, std::string(what) + ": " + hipGetErrorString(static_cast<hipError_t>(err)));
}

constexpr size_t kAlign = 256;
size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// Workspace layout, every section aligned to 256 bytes.
struct Layout {
    size_t perm, row_ptr, order, order_rest, slots_off, slots, vals, blk_col, occ, csr_row_ptr, csr_col_idx, csr_vals;
    size_t t_super, t_ptr, t_cols, t_rows, t_base, t_vals, total;
};

Layout make_layout(const smat_handle& h)
{
    Layout l{};
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t at = off; off = align_up(off + bytes); return at; };
    const size_t nbr = static_cast<size_t>(h.bcsr.nbr), n_e = static_cast<size_t>(h.n_dev_blocks);
    const size_t nnz = h.csr.col_idx.size();
    l.perm = take(nbr * 16 * sizeof(int32_t));
    l.row_ptr = take((nbr + 1) * sizeof(int32_t));
    l.order = take(nbr * sizeof(int32_t));
    l.order_rest = take(nbr * sizeof(int32_t));
    l.slots_off = take((nbr + 1) * sizeof(uint32_t));
    l.slots = take(static_cast<size_t>(h.slots_units) * 32);
    l.vals = take(static_cast<size_t>(h.slots_units) * 256);
    l.blk_col = take(n_e * sizeof(int32_t));
    l.occ = take(n_e / 2 * sizeof(uint32_t));
    l.csr_row_ptr = take((static_cast<size_t>(h.csr.M) + 1) * sizeof(int64_t));
    l.csr_col_idx = take(nnz * sizeof(int32_t));
    l.csr_vals = take(nnz * sizeof(uint16_t));
    l.t_super = take(h.dense_super.size() * sizeof(int32_t));
    l.t_ptr = take(h.step_ptr.size() * sizeof(int32_t));
    l.t_cols = take(h.step_cols.size() * sizeof(int32_t));
    l.t_rows = take(h.step_rows.size() * sizeof(uint32_t));
    l.t_base = take(h.step_base.size() * sizeof(uint32_t));
    l.t_vals = take(static_cast<size_t>(h.dense_slots) * 1024);
    l.total = off ? off : kAlign;
    return l;
}

// occupancy mask of the pair that starts at block s of a block row ending at block s1
uint32_t pair_occupancy(const smat::Bcsr& b, int32_t s, int32_t s1)
{
    return b.col_mask[s] | (s + 1 < s1 ? static_cast<uint32_t>(b.col_mask[s + 1]) << 16 : 0u);
}

// Decides which complete super rows (sixteen block rows) go to the dense path and lays out
// their steps.  A super row qualifies when walking the union of its block columns wastes
// little: at least 8 union columns, at least half of the (block row, union column) grid
// stored (a band of 37 % fill measured slower here than on the per-row kernel), and blocks whose columns are mostly occupied (>= 8 of 16 on average; blocks with a
// few occupied columns are cheaper on the per-row path, which fetches only those rows of B).
void plan_dense_tiles(smat_handle& h)
{
    const smat::Bcsr& b = h.bcsr;
    const int64_t nbr = b.nbr;
    h.row_dense.assign(static_cast<size_t>(nbr), 0);
    h.step_ptr.assign(1, 0);
    std::vector<int32_t> uni;
    for (int64_t s = 0; (s + 1) * 16 <= nbr; ++s) {
        const int32_t lo = b.row_ptr[s * 16], hi = b.row_ptr[s * 16 + 16];
        if (hi - lo < 64) continue;
        uni.assign(b.col_idx.begin() + lo, b.col_idx.begin() + hi);
        std::sort(uni.begin(), uni.end());
        uni.erase(std::unique(uni.begin(), uni.end()), uni.end());
        int64_t occupied = 0;
        for (int32_t k = lo; k < hi; ++k) occupied += __builtin_popcount(b.col_mask[k]);
        const int64_t n_uni = static_cast<int64_t>(uni.size()), n_blk = hi - lo;
        if (n_uni < 8 || n_blk * 2 < 16 * n_uni || occupied < 8 * n_blk) continue;
        const int64_t steps = (n_uni + 1) / 2;
        if (steps * 16 >= (int64_t{1} << 21) || h.dense_slots + static_cast<uint64_t>(steps) * 16 >= (uint64_t{1} << 31)) continue;
        h.dense_super.push_back(static_cast<int32_t>(s));
        for (int j = 0; j < 16; ++j) h.row_dense[static_cast<size_t>(s * 16 + j)] = 1;
        for (int64_t q = 0; q < steps; ++q) {
            const int32_t c0 = uni[2 * q], c1 = 2 * q + 1 < n_uni ? uni[2 * q + 1] : 0x7FFFFFFF;
            uint32_t rows = 0;
            for (int j = 0; j < 16; ++j) {
                const int32_t* first = b.col_idx.data() + b.row_ptr[s * 16 + j];
                const int32_t* last = b.col_idx.data() + b.row_ptr[s * 16 + j + 1];
                if (std::binary_search(first, last, c0) || std::binary_search(first, last, c1)) rows |= 1u << j;
            }
            h.step_cols.push_back(c0);
            h.step_cols.push_back(c1);
            h.step_rows.push_back(rows);
            h.step_base.push_back(static_cast<uint32_t>(h.dense_slots));
            h.dense_slots += static_cast<uint64_t>(__builtin_popcount(rows));
        }
        h.step_ptr.push_back(static_cast<int32_t>(h.step_rows.size()));
    }
}

// Launch statistics over a subset of block rows.
void row_stats(const smat_handle& h, bool skip_dense, smat::DeviceBcsr& d)
{
    const smat::Bcsr& b = h.bcsr;
    int64_t longest = 0, blocks = 0, rows = 0, padded = 0;
    int cls = 0;
    for (int64_t br = 0; br < b.nbr; ++br) {
        if (skip_dense && h.row_dense[static_cast<size_t>(br)]) continue;
        const int64_t len = b.row_ptr[br + 1] - b.row_ptr[br];
        longest = std::max(longest, len);
        blocks += len;
        padded += (len + 1) / 2 * 2;
        cls = std::max<int>(cls, h.row_class[static_cast<size_t>(br)]);
        ++rows;
    }
    d.n_order = rows;
    d.n_e = padded;
    d.max_row_blocks = longest;
    d.mean_row_blocks = rows ? static_cast<double>(blocks) / static_cast<double>(rows) : 0.0;
    d.max_class = cls;
}

}  // namespace

extern "C" {

void smat_default_options(smat_options_t* opt)
{
    if (!opt) return;
    opt->block_h = 16;
    opt->block_w = 16;
    opt->reorder = 1;
    opt->tau_permille = 700;
}

smat_status_t smat_preprocess(int64_t M, int64_t K, const int64_t* row_ptr, const int32_t* col_idx,
                              const void* vals, smat_dtype_t dtype, const smat_options_t* opt,
                              smat_handle_t** out)
{
    try {
        smat_options_t o;
        smat_default_options(&o);
        if (opt) o = *opt;
        if (!out) return fail(SMAT_ERR_INVALID_ARG, "out is NULL");
        if (M < 0 || K < 0) return fail(SMAT_ERR_INVALID_ARG, "negative matrix size");
        if (!row_ptr) return fail(SMAT_ERR_INVALID_ARG, "row_ptr is NULL");
        if (dtype != SMAT_F16 && dtype != SMAT_BF16) return fail(SMAT_ERR_INVALID_ARG, "unknown dtype");
        if (o.block_h != 16 || o.block_w != 16) return fail(SMAT_ERR_UNSUPPORTED, "only 16x16 blocks are supported");
        if (o.reorder != 0 && o.reorder != 1) return fail(SMAT_ERR_INVALID_ARG, "reorder must be 0 or 1");
        if (o.tau_permille < 0 || o.tau_permille > 1000) return fail(SMAT_ERR_INVALID_ARG, "tau_permille must be in 0..1000");
        if (M >= (int64_t{1} << 31) - 16 || K >= (int64_t{1} << 31) - 16)
            return fail(SMAT_ERR_UNSUPPORTED, "M and K must be below 2^31 - 16");
        if ((M + 15) / 16 >= (int64_t{1} << 28)) return fail(SMAT_ERR_UNSUPPORTED, "more than 2^28 block rows");
        if (K >= (int64_t{1} << 24)) return fail(SMAT_ERR_UNSUPPORTED, "K must be below 2^24");
        if (row_ptr[0] != 0) return fail(SMAT_ERR_BAD_CSR, "row_ptr[0] must be 0");
        for (int64_t r = 0; r < M; ++r)
            if (row_ptr[r + 1] < row_ptr[r]) return fail(SMAT_ERR_BAD_CSR, "row_ptr decreases at row " + std::to_string(r));
        const int64_t nnz = row_ptr[M];
        if (nnz > 0 && (!col_idx || !vals)) return fail(SMAT_ERR_INVALID_ARG, "col_idx or vals is NULL");
        const std::string bad = smat::validate_csr(M, K, row_ptr, col_idx);
        if (!bad.empty()) return fail(SMAT_ERR_BAD_CSR, bad);

        smat_handle* h = new smat_handle();
        h->dtype = dtype;
        h->csr.M = M;
        h->csr.K = K;
        h->csr.row_ptr.assign(row_ptr, row_ptr + M + 1);
        h->csr.col_idx.assign(col_idx, col_idx + nnz);
        h->csr.vals.assign(static_cast<const uint16_t*>(vals), static_cast<const uint16_t*>(vals) + nnz);
        smat::build_bcsr(h->csr, o.reorder != 0, o.tau_permille, h->bcsr);
        h->dev_row_ptr.assign(static_cast<size_t>(h->bcsr.nbr) + 1, 0);
        int64_t padded = 0;
        for (int64_t br = 0; br < h->bcsr.nbr; ++br) {
            const int64_t cnt = h->bcsr.row_ptr[br + 1] - h->bcsr.row_ptr[br];
            padded += (cnt + 1) / 2 * 2;
            if (padded >= (int64_t{1} << 31) - 2) {
                delete h;
                return fail(SMAT_ERR_UNSUPPORTED, "more than 2^31 blocks");
            }
            h->dev_row_ptr[br + 1] = static_cast<int32_t>(padded);
        }
        h->n_dev_blocks = padded;
        const size_t nbr = static_cast<size_t>(h->bcsr.nbr);
        h->row_class.assign(nbr, 0);
        h->slots_off.assign(nbr + 1, 0);
        uint64_t units = 0;
        for (size_t br = 0; br < nbr; ++br) {
            const int32_t s0 = h->bcsr.row_ptr[br], s1 = h->bcsr.row_ptr[br + 1];
            int worst = 0;
            for (int32_t s = s0; s < s1; s += 2)
                worst = std::max(worst, __builtin_popcount(pair_occupancy(h->bcsr, s, s1)));
            const int cls = worst <= 8 ? 0 : (worst <= 16 ? 1 : 2);
            h->row_class[br] = static_cast<int8_t>(cls);
            h->max_class = std::max(h->max_class, cls);
            h->slots_off[br] = static_cast<uint32_t>(units);
            units += static_cast<uint64_t>((s1 - s0 + 1) / 2) << cls;       // 1, 2 or 4 units per pair
            if (units >= (uint64_t{1} << 32)) {
                delete h;
                return fail(SMAT_ERR_UNSUPPORTED, "slot table too large");
            }
        }
        h->slots_off[nbr] = static_cast<uint32_t>(units);
        h->slots_units = units;
        plan_dense_tiles(*h);
        *out = h;
        return SMAT_OK;
    } catch (const std::bad_alloc&) {
        return fail(SMAT_ERR_ALLOC, "out of host memory in smat_preprocess");
    } catch (const std::exception& e) {
        return fail(SMAT_ERR_INVALID_ARG, e.what());
    }
}

smat_status_t smat_get_info(const smat_handle_t* h, int64_t* n_block_rows, int64_t* n_blocks,
                            int64_t* n_blocks_identity, int* used_identity)
{
    if (!h) return fail(SMAT_ERR_INVALID_ARG, "handle is NULL");
    if (n_block_rows) *n_block_rows = h->bcsr.nbr;
    if (n_blocks) *n_blocks = h->bcsr.n_blocks;
    if (n_blocks_identity) *n_blocks_identity = h->bcsr.n_blocks_identity;
    if (used_identity) *used_identity = h->bcsr.used_identity ? 1 : 0;
    return SMAT_OK;
}

smat_status_t smat_export_perm(const smat_handle_t* h, int32_t* perm)
{
    if (!h || (!perm && h->csr.M > 0)) return fail(SMAT_ERR_INVALID_ARG, "NULL argument");
    if (h->csr.M > 0) std::memcpy(perm, h->bcsr.perm.data(), sizeof(int32_t) * static_cast<size_t>(h->csr.M));
    return SMAT_OK;
}

smat_status_t smat_export_bcsr(const smat_handle_t* h, int32_t* row_ptr, int32_t* col_idx, void* vals)
{
    if (!h || !row_ptr) return fail(SMAT_ERR_INVALID_ARG, "NULL argument");
    if (h->bcsr.n_blocks > 0 && !col_idx) return fail(SMAT_ERR_INVALID_ARG, "col_idx is NULL");
    try {
        std::memcpy(row_ptr, h->bcsr.row_ptr.data(), sizeof(int32_t) * h->bcsr.row_ptr.size());
        if (h->bcsr.n_blocks > 0)
            std::memcpy(col_idx, h->bcsr.col_idx.data(), sizeof(int32_t) * h->bcsr.col_idx.size());
        if (vals) smat::fill_canonical_vals(h->csr, h->bcsr, static_cast<uint16_t*>(vals));
        return SMAT_OK;
    } catch (const std::bad_alloc&) {
        return fail(SMAT_ERR_ALLOC, "out of host memory in smat_export_bcsr");
    }
}

smat_status_t smat_device_bytes(const smat_handle_t* h, size_t* bytes)
{
    if (!h || !bytes) return fail(SMAT_ERR_INVALID_ARG, "NULL argument");
    *bytes = make_layout(*h).total;
    return SMAT_OK;
}

smat_status_t smat_bind_device(smat_handle_t* h, void* dev_workspace, size_t bytes, void* stream)
{
    if (!h || !dev_workspace) return fail(SMAT_ERR_INVALID_ARG, "NULL argument");
    if (reinterpret_cast<uintptr_t>(dev_workspace) % kAlign != 0)
        return fail(SMAT_ERR_INVALID_ARG, "dev_workspace must be 256-byte aligned");
    const Layout l = make_layout(*h);
    if (bytes < l.total) return fail(SMAT_ERR_INVALID_ARG, "dev_workspace too small: need " + std::to_string(l.total) + " bytes");
    try {
        hipStream_t s = static_cast<hipStream_t>(stream);
        char* base = static_cast<char*>(dev_workspace);
        const smat::Bcsr& b = h->bcsr;
        const size_t nbr = static_cast<size_t>(b.nbr), n_e = static_cast<size_t>(h->n_dev_blocks);
        const size_t M = static_cast<size_t>(h->csr.M), nnz = h->csr.col_idx.size();

        std::vector<int32_t> perm_padded(nbr * 16, -1);
        std::memcpy(perm_padded.data(), b.perm.data(), sizeof(int32_t) * M);
        // slot tables (pair_layout.h), block columns and occupancy masks; an odd tail is completed
        // by a pad block: column beyond every real one (keeps the row's columns ascending),
        // nothing occupied
        std::vector<uint32_t> slots(static_cast<size_t>(h->slots_units) * 8);
        std::vector<int32_t> blk_col(n_e);
        std::vector<uint32_t> occ_mask(n_e / 2);
        const uint32_t no_row = static_cast<uint32_t>(h->csr.K);        // one past the last row of B
        for (size_t br = 0; br < nbr; ++br) {
            const int32_t s0 = b.row_ptr[br], s1 = b.row_ptr[br + 1];
            const int L = 2 << h->row_class[br];
            size_t blk = static_cast<size_t>(h->dev_row_ptr[br]);
            uint32_t* table = slots.data() + static_cast<size_t>(h->slots_off[br]) * 8;
            for (int32_t s = s0; s < s1; s += 2, blk += 2, table += 4 * L) {
                const bool has2 = s + 1 < s1;
                const uint32_t occ = pair_occupancy(b, s, s1);
                blk_col[blk] = b.col_idx[s];
                blk_col[blk + 1] = has2 ? b.col_idx[s + 1] : 0x7FFFFFFF;
                occ_mask[blk / 2] = occ;
                for (int x = 0; x < 4 * L; ++x) table[x] = no_row;
                int rank = 0;
                for (int c = 0; c < 32; ++c) {
                    if (!(occ >> c & 1u)) continue;
                    const uint32_t row = static_cast<uint32_t>(b.col_idx[s + (c >> 4)]) * 16u + static_cast<uint32_t>(c & 15);
                    table[smat::slot_group(rank) * L + smat::slot_pos(rank)] = row;
                    ++rank;
                }
            }
        }
        std::vector<int32_t> order_cls(nbr), order_rest;
        order_rest.reserve(nbr);
        for (size_t x = 0; x < nbr; ++x) {
            order_cls[x] = b.order[x] | (static_cast<int32_t>(h->row_class[b.order[x]]) << 28);
            if (!h->row_dense[static_cast<size_t>(b.order[x])]) order_rest.push_back(order_cls[x]);
        }

        auto up = [&](size_t off, const void* src, size_t n) -> int {
            if (n == 0) return 0;
            return static_cast<int>(hipMemcpyAsync(base + off, src, n, hipMemcpyHostToDevice, s));
        };
        int e;
        if ((e = up(l.perm, perm_padded.data(), perm_padded.size() * 4))) return hip_fail("copy perm", e);
        if ((e = up(l.row_ptr, h->dev_row_ptr.data(), h->dev_row_ptr.size() * 4))) return hip_fail("copy row_ptr", e);
        if ((e = up(l.order, order_cls.data(), order_cls.size() * 4))) return hip_fail("copy order", e);
        if ((e = up(l.order_rest, order_rest.data(), order_rest.size() * 4))) return hip_fail("copy order", e);
        if ((e = up(l.t_super, h->dense_super.data(), h->dense_super.size() * 4))) return hip_fail("copy tiles", e);
        if ((e = up(l.t_ptr, h->step_ptr.data(), h->step_ptr.size() * 4))) return hip_fail("copy tiles", e);
        if ((e = up(l.t_cols, h->step_cols.data(), h->step_cols.size() * 4))) return hip_fail("copy tiles", e);
        if ((e = up(l.t_rows, h->step_rows.data(), h->step_rows.size() * 4))) return hip_fail("copy tiles", e);
        if ((e = up(l.t_base, h->step_base.data(), h->step_base.size() * 4))) return hip_fail("copy tiles", e);
        if ((e = up(l.slots_off, h->slots_off.data(), h->slots_off.size() * 4))) return hip_fail("copy slot offsets", e);
        if ((e = up(l.slots, slots.data(), slots.size() * 4))) return hip_fail("copy slot tables", e);
        if ((e = up(l.blk_col, blk_col.data(), blk_col.size() * 4))) return hip_fail("copy block columns", e);
        if ((e = up(l.occ, occ_mask.data(), occ_mask.size() * 4))) return hip_fail("copy occupancy", e);
        if ((e = up(l.csr_row_ptr, h->csr.row_ptr.data(), (M + 1) * 8))) return hip_fail("copy csr row_ptr", e);
        if ((e = up(l.csr_col_idx, h->csr.col_idx.data(), nnz * 4))) return hip_fail("copy csr col_idx", e);
        if ((e = up(l.csr_vals, h->csr.vals.data(), nnz * 2))) return hip_fail("copy csr vals", e);

        smat::DeviceBcsr d;
        d.perm = reinterpret_cast<const int32_t*>(base + l.perm);
        d.row_ptr = reinterpret_cast<const int32_t*>(base + l.row_ptr);
        d.order = reinterpret_cast<const int32_t*>(base + l.order);
        d.slots_off = reinterpret_cast<const uint32_t*>(base + l.slots_off);
        d.slots = reinterpret_cast<const uint32_t*>(base + l.slots);
        d.vals = reinterpret_cast<const uint16_t*>(base + l.vals);
        d.blk_col = reinterpret_cast<const int32_t*>(base + l.blk_col);
        d.occ = reinterpret_cast<const uint32_t*>(base + l.occ);
        d.M = h->csr.M;
        d.K = h->csr.K;
        d.nbr = b.nbr;
        smat::DeviceBcsr d_rest = d;
        row_stats(*h, false, d);
        row_stats(*h, true, d_rest);
        d_rest.order = reinterpret_cast<const int32_t*>(base + l.order_rest);
        smat::DenseTiles tiles;
        tiles.super_rows = reinterpret_cast<const int32_t*>(base + l.t_super);
        tiles.step_ptr = reinterpret_cast<const int32_t*>(base + l.t_ptr);
        tiles.step_cols = reinterpret_cast<const int32_t*>(base + l.t_cols);
        tiles.step_rows = reinterpret_cast<const uint32_t*>(base + l.t_rows);
        tiles.step_base = reinterpret_cast<const uint32_t*>(base + l.t_base);
        tiles.vals = reinterpret_cast<const uint16_t*>(base + l.t_vals);
        tiles.n = static_cast<int32_t>(h->dense_super.size());
        tiles.mean_steps = tiles.n ? static_cast<double>(h->step_rows.size()) / tiles.n : 0.0;
        h->d_csr_row_ptr = reinterpret_cast<const int64_t*>(base + l.csr_row_ptr);
        h->d_csr_col_idx = reinterpret_cast<const int32_t*>(base + l.csr_col_idx);
        h->d_csr_vals = reinterpret_cast<const uint16_t*>(base + l.csr_vals);

        if ((e = smat::launch_fill_zero(base + l.vals, static_cast<size_t>(h->slots_units) * 16, s))) return hip_fail("zero block values", e);
        if ((e = smat::launch_bcsr_fill(d, h->d_csr_row_ptr, h->d_csr_col_idx, h->d_csr_vals,
                                        reinterpret_cast<uint16_t*>(base + l.vals), s)))
            return hip_fail("fill block values", e);
        if ((e = smat::launch_fill_zero(base + l.t_vals, static_cast<size_t>(h->dense_slots) * 64, s))) return hip_fail("zero tile values", e);
        if ((e = smat::launch_dense_fill(d, tiles, h->d_csr_row_ptr, h->d_csr_col_idx, h->d_csr_vals,
                                         reinterpret_cast<uint16_t*>(base + l.t_vals), s)))
            return hip_fail("fill tile values", e);
        if ((e = static_cast<int>(hipStreamSynchronize(s)))) return hip_fail("bind synchronize", e);
        h->dev = d;
        h->dev_rest = d_rest;
        h->tiles = tiles;
        h->bound = true;
        return SMAT_OK;
    } catch (const std::bad_alloc&) {
        return fail(SMAT_ERR_ALLOC, "out of host memory in smat_bind_device");
    }
}

smat_status_t smat_export_device_vals(const smat_handle_t* h, void* vals, void* stream)
{
    if (!h) return fail(SMAT_ERR_INVALID_ARG, "handle is NULL");
    if (!h->bound) return fail(SMAT_ERR_NOT_BOUND, "handle is not bound to a device workspace");
    const size_t n_e = static_cast<size_t>(h->bcsr.n_blocks);
    if (n_e == 0) return SMAT_OK;
    if (!vals) return fail(SMAT_ERR_INVALID_ARG, "vals is NULL");
    try {
        std::vector<uint16_t> raw(static_cast<size_t>(h->slots_units) * 128);
        hipStream_t s = static_cast<hipStream_t>(stream);
        int e = static_cast<int>(hipMemcpyAsync(raw.data(), h->dev.vals, raw.size() * 2, hipMemcpyDeviceToHost, s));
        if (e) return hip_fail("read block values", e);
        if ((e = static_cast<int>(hipStreamSynchronize(s)))) return hip_fail("read block values", e);
        uint16_t* out = static_cast<uint16_t*>(vals);
        std::memset(out, 0, n_e * 512);
        for (int64_t br = 0; br < h->bcsr.nbr; ++br) {
            const int32_t s0 = h->bcsr.row_ptr[br], s1 = h->bcsr.row_ptr[br + 1];
            const int L = 2 << h->row_class[static_cast<size_t>(br)];
            const int halves = smat::pair_halves(L);
            const uint16_t* src = raw.data() + static_cast<size_t>(h->slots_off[static_cast<size_t>(br)]) * 128;
            for (int32_t s = s0; s < s1; s += 2, src += halves) {
                const uint32_t occ = pair_occupancy(h->bcsr, s, s1);
                uint8_t used[512];
                std::memset(used, 0, sizeof(used));
                int rank = 0;
                for (int c = 0; c < 32; ++c) {
                    if (!(occ >> c & 1u)) continue;
                    const int g = smat::slot_group(rank), kk = smat::slot_pos(rank);
                    ++rank;
                    uint16_t* blk = out + static_cast<size_t>(s + (c >> 4)) * 256;
                    for (int r = 0; r < 16; ++r) {
                        const int at = smat::pair_half_index(L, r, g, kk);
                        blk[r * 16 + (c & 15)] = src[at];
                        used[at] = 1;
                    }
                }
                // every slot that holds no occupied column must have stayed zero
                for (int q = 0; q < halves; ++q)
                    if (!used[q] && src[q] != 0) return fail(SMAT_ERR_HIP, "device block values: unoccupied slot is not zero");
            }
        }
        return SMAT_OK;
    } catch (const std::bad_alloc&) {
        return fail(SMAT_ERR_ALLOC, "out of host memory in smat_export_device_vals");
    }
}

smat_status_t smat_spmm(const smat_handle_t* h, const void* dB, int64_t ldb, void* dC, int64_t ldc,
                        int64_t N, void* stream)
{
    if (!h) return fail(SMAT_ERR_INVALID_ARG, "handle is NULL");
    if (!h->bound) return fail(SMAT_ERR_NOT_BOUND, "smat_spmm called before smat_bind_device");
    if (N < 0) return fail(SMAT_ERR_INVALID_ARG, "N is negative");
    if (N == 0 || h->csr.M == 0) return SMAT_OK;
    if (!dC || (!dB && h->csr.K > 0)) return fail(SMAT_ERR_INVALID_ARG, "NULL matrix pointer");
    if (ldb < N || ldc < N) return fail(SMAT_ERR_INVALID_ARG, "leading dimension smaller than N");
    if (N > 16 * 65535) return fail(SMAT_ERR_UNSUPPORTED, "N above 1048560");
    const int64_t K = h->csr.K;
    if (K > 0 && ((K - 1) * ldb + N) * 2 >= (int64_t{1} << 31))
        return fail(SMAT_ERR_UNSUPPORTED, "B larger than 2 GiB is not supported");
    if (ldb >= (int64_t{1} << 23)) return fail(SMAT_ERR_UNSUPPORTED, "ldb must be below 2^23");
    // The dense path needs 16-byte rows of B at 8-column granularity; otherwise every block row
    // goes through the per-row kernel.
    const bool bf16 = h->dtype == SMAT_BF16;
    const bool use_tiles = h->tiles.n > 0 && N % 8 == 0 && ldb % 8 == 0 && reinterpret_cast<uintptr_t>(dB) % 16 == 0;
    const char* variant = "";
    thread_local std::string name;
    int e = 0;
    if (use_tiles) {
        if (h->dev_rest.n_order > 0)
            e = smat::launch_spmm(h->dev_rest, bf16, dB, ldb, static_cast<float*>(dC), ldc, N, stream, &variant);
        const char* dense_variant = "";
        if (!e) e = smat::launch_spmm_dense(h->dev, h->tiles, bf16, dB, ldb, static_cast<float*>(dC), ldc, N, stream, &dense_variant);
        name = std::string(dense_variant) + (h->dev_rest.n_order > 0 ? std::string("+") + variant : std::string());
        g_kernel = name.c_str();
    } else {
        e = smat::launch_spmm(h->dev, bf16, dB, ldb, static_cast<float*>(dC), ldc, N, stream, &variant);
        g_kernel = variant;
    }
    if (e) return hip_fail("launch spmm", e);
    return SMAT_OK;
}

void smat_destroy(smat_handle_t* h) { delete h; }

const char* smat_last_error(void) { return g_error.c_str(); }

const char* smat_last_kernel(void) { return g_kernel; }

}  // extern "C"
