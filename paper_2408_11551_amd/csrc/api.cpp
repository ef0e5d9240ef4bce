// C ABI of the library (see include/smat.h): handle management, argument checks,
// host <-> device copies.  All arithmetic of the method lives in preprocess.cpp
// (host, integers) and kernels.hip (device).
#include "../../include/smat.h"
#include "../../include/smat_bench.h"

#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cstdlib>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <memory>
#include <mutex>
#include <new>
#include <stdexcept>
#include <string>
#include <vector>

#include "kernels.h"
#include "pack_layout.h"
#include "preprocess.h"

struct smat_handle {
    smat::Csr csr;
    smat::Bcsr bcsr;
    smat_dtype_t dtype = SMAT_F16;
    int elem_bytes = 2;                  // bytes per stored value of A and B: 2, or 1 for the 8-bit types
    int dense_mode = 0;                  // option dense_tiles
    bool bound = false;
    bool cols_permuted = false;          // row + column reordering took a column order: csr and bcsr are those of P A Q
    // Packs (pack_layout.h): every block row is cut, from the left, into runs of consecutive
    // blocks that hold at most 32 occupied columns together; a pack is what one matrix
    // instruction multiplies.
    std::vector<int32_t> pack_ptr;       // [nbr+1] pack offsets per block row
    std::vector<int32_t> pack_first;     // [n_packs+1] first stored block of every pack
    std::vector<int32_t> blk_pack;       // [n_blocks] pack of the block, counted inside its block row
    std::vector<uint32_t> blk_meta;      // [n_blocks] column mask | occupied columns of the pack before the block << 16
    std::vector<int32_t> order;          // [nbr] block rows in launch order
    // Row class: how many B-row loads per lane a pack of the block row needs at most (occupied
    // columns are dealt to four lane groups): 2, 4 or 8 -> class 0, 1, 2; class 3 is an entry row
    // (pack_layout.h).  The slot table of a row takes 16 * L bytes per pack (128 for an entry row);
    // slots_off counts 32-byte units of it.  Its values take 64 * L elements per pack (one 64-byte
    // unit for an entry row); vals_off counts 64-byte units.
    std::vector<int8_t> row_class;       // [nbr]
    std::vector<uint32_t> slots_off;     // [nbr+1]
    std::vector<uint32_t> vals_off;      // [nbr+1]
    uint64_t slots_units = 0, vals_units = 0;
    int max_class = 0;
    int64_t value_bytes = 0;             // bytes of block values a launch over every block row reads
    int64_t b_rows = 0;                  // slots that name a row of B, over all packs
    std::vector<int32_t> row_b_rows;     // [nbr] the same per block row
    // Dense path (kernels.h, DenseTiles): complete super rows of sixteen block rows whose block
    // columns overlap enough.  row_dense marks the block rows it covers.
    std::vector<int32_t> dense_super, step_ptr, step_cols;
    std::vector<uint32_t> step_rows, step_base;
    std::vector<uint8_t> row_dense;      // [nbr]
    uint64_t dense_slots = 0;
    bool dense_all_full = false;         // every step of every dense super row: all sixteen block rows, block columns 2q and 2q+1,
                                         // and every dense super row has the same number of steps
    int64_t dense_columns = 0;           // occupied columns over the blocks of the dense super rows
    smat::DeviceBcsr dev;                // launch over every block row
    smat::DeviceBcsr dev_rest;           // launch over the block rows the dense path does not cover
    smat::DenseTiles tiles;
    // device copies of the CSR (kept: they live in the caller's workspace anyway)
    const int64_t* d_csr_row_ptr = nullptr;
    const int32_t* d_csr_col_idx = nullptr;
    const uint16_t* d_csr_vals = nullptr;
    // canonical BCSR on the device, for the ablation kernels (smat_ablation_bind)
    smat::CanonicalBcsr ablation;
    bool ablation_bound = false;
    // Areas of partial tiles (split dense launches), one per stream: entry i names the stream
    // that owns area i of the workspace.  A stream keeps its area for the life of the handle;
    // calls on one stream are ordered, so an area is never used by two launches at once.
    int n_scratch_areas = 2;             // option concurrent_streams
    char* scratch_base = nullptr;        // first area (device), set by smat_bind_device
    mutable std::mutex scratch_mutex;
    mutable std::vector<const void*> scratch_owner;
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
// Partial tiles of dense launches that split a tile's steps over several workgroups: a launch
// splits only while tiles x workgroups per tile stays within the 256 compute units, so at most
// 256 partial tiles of 256 x 128 words are in use per launch.  One such area per stream.
constexpr size_t kTileScratchBytes = size_t{256} * 256 * 128 * 4;
size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// Workspace layout, every section aligned to 256 bytes.
struct Layout {
    size_t perm, work, work_rest, slots, vals, pack_ptr, vals_off, row_class, blk_ptr, blk_col, blk_pack, blk_meta;
    size_t csr_row_ptr, csr_col_idx, csr_vals;
    size_t t_super, t_ptr, t_cols, t_rows, t_base, t_vals, t_scratch, total;
};

Layout make_layout(const smat_handle& h)
{
    Layout l{};
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t at = off; off = align_up(off + bytes); return at; };
    const size_t nbr = static_cast<size_t>(h.bcsr.nbr), n_e = static_cast<size_t>(h.bcsr.n_blocks);
    const size_t nnz = h.csr.col_idx.size();
    l.perm = take(nbr * 16 * sizeof(int32_t));
    l.work = take(nbr * 16);
    l.work_rest = take(nbr * 16);
    l.slots = take(static_cast<size_t>(h.slots_units) * 32);
    l.vals = take(static_cast<size_t>(h.vals_units) * 64);
    l.pack_ptr = take((nbr + 1) * sizeof(int32_t));
    l.vals_off = take((nbr + 1) * sizeof(uint32_t));
    l.row_class = take(nbr);
    l.blk_ptr = take((nbr + 1) * sizeof(int32_t));
    l.blk_col = take(n_e * sizeof(int32_t));
    l.blk_pack = take(n_e * sizeof(int32_t));
    l.blk_meta = take(n_e * sizeof(uint32_t));
    l.csr_row_ptr = take((static_cast<size_t>(h.csr.M) + 1) * sizeof(int64_t));
    l.csr_col_idx = take(nnz * sizeof(int32_t));
    l.csr_vals = take(nnz * sizeof(uint16_t));
    l.t_super = take(h.dense_super.size() * sizeof(int32_t));
    l.t_ptr = take(h.step_ptr.size() * sizeof(int32_t));
    l.t_cols = take(h.step_cols.size() * sizeof(int32_t));
    l.t_rows = take(h.step_rows.size() * sizeof(uint32_t));
    l.t_base = take(h.step_base.size() * sizeof(uint32_t));
    l.t_vals = take(static_cast<size_t>(h.dense_slots) * 1024);
    l.t_scratch = take(h.dense_super.empty() ? 0 : kTileScratchBytes * static_cast<size_t>(h.n_scratch_areas));
    l.total = off ? off : kAlign;
    return l;
}

// Decides which complete super rows (sixteen block rows) may go to the dense path and lays out
// their steps.  A super row qualifies when walking the union of its block columns wastes
// little: at least 8 union columns, at least 35 % of the (block row, union column) grid
// stored, and blocks whose columns are mostly occupied (>= 8 of 16 on average; blocks with a
// few occupied columns are cheaper on the per-row path, which fetches only those rows of B).
// With the option dense_tiles = -1 nothing qualifies.
void plan_dense_tiles(smat_handle& h)
{
    const smat::Bcsr& b = h.bcsr;
    const int64_t nbr = b.nbr;
    h.row_dense.assign(static_cast<size_t>(nbr), 0);
    h.step_ptr.assign(1, 0);
    h.dense_all_full = false;
    if (h.dense_mode < 0) return;
    h.dense_all_full = true;             // until a step says otherwise
    std::vector<int32_t> uni;
    // block columns per step: the 32 k slots of a 16-bit MFMA are two block columns; the 8-bit types
    // take four per step (two MFMA 16x16x32 per output tile between barriers), so that a step moves
    // the same bytes and a tile has half as many of them
    const int64_t cps = h.elem_bytes == 1 ? 4 : 2;
    for (int64_t s = 0; (s + 1) * 16 <= nbr; ++s) {
        const int32_t lo = b.row_ptr[s * 16], hi = b.row_ptr[s * 16 + 16];
        if (hi - lo < 64) continue;
        uni.assign(b.col_idx.begin() + lo, b.col_idx.begin() + hi);
        std::sort(uni.begin(), uni.end());
        uni.erase(std::unique(uni.begin(), uni.end()), uni.end());
        int64_t occupied = 0;
        for (int32_t k = lo; k < hi; ++k) occupied += __builtin_popcount(b.col_mask[k]);
        const int64_t n_uni = static_cast<int64_t>(uni.size()), n_blk = hi - lo;
        if (n_uni < 8 || n_blk * 20 < 7 * 16 * n_uni || occupied < 8 * n_blk) continue;
        const int64_t steps = (n_uni + cps - 1) / cps;
        if (steps * 16 >= (int64_t{1} << 21) || h.dense_slots + static_cast<uint64_t>(steps) * 16 >= (uint64_t{1} << 31)) continue;
        h.dense_super.push_back(static_cast<int32_t>(s));
        h.dense_columns += occupied;
        for (int j = 0; j < 16; ++j) h.row_dense[static_cast<size_t>(s * 16 + j)] = 1;
        for (int64_t q = 0; q < steps; ++q) {
            int32_t cols[4];
            for (int64_t e = 0; e < cps; ++e) cols[e] = cps * q + e < n_uni ? uni[cps * q + e] : 0x7FFFFFFF;
            uint32_t rows = 0;
            for (int j = 0; j < 16; ++j) {
                const int32_t* first = b.col_idx.data() + b.row_ptr[s * 16 + j];
                const int32_t* last = b.col_idx.data() + b.row_ptr[s * 16 + j + 1];
                for (int64_t e = 0; e < cps; ++e)
                    if (std::binary_search(first, last, cols[e])) rows |= 1u << j;
            }
            for (int64_t e = 0; e < cps; ++e) h.step_cols.push_back(cols[e]);
            for (int64_t e = 0; e < cps; ++e)
                if (cols[e] != cps * q + e) h.dense_all_full = false;
            if (rows != 0xFFFFu) h.dense_all_full = false;
            h.step_rows.push_back(rows);
            h.step_base.push_back(static_cast<uint32_t>(h.dense_slots));
            h.dense_slots += static_cast<uint64_t>(__builtin_popcount(rows));
        }
        h.step_ptr.push_back(static_cast<int32_t>(h.step_rows.size()));
        if (steps != h.step_ptr[1]) h.dense_all_full = false;      // the first dense super row's count
    }
}

// Stored entries of block row br of A' (rows perm[16 br] ...).
int64_t block_row_nnz(const smat_handle& h, size_t br)
{
    int64_t nnz = 0;
    for (int64_t i = static_cast<int64_t>(br) * 16; i < static_cast<int64_t>(br) * 16 + 16 && i < h.csr.M; ++i) {
        const size_t r = static_cast<size_t>(h.bcsr.perm[static_cast<size_t>(i)]);
        nnz += h.csr.row_ptr[r + 1] - h.csr.row_ptr[r];
    }
    return nnz;
}

// Stored entries of block row br in the order of an entry row's slots (pack_layout.h): by
// column, then by row of the block row.  An item is column << 4 | row.
void entry_order(const smat_handle& h, size_t br, std::vector<uint64_t>& items)
{
    items.clear();
    for (size_t rr = 0; rr < 16 && br * 16 + rr < static_cast<size_t>(h.csr.M); ++rr) {
        const size_t r = static_cast<size_t>(h.bcsr.perm[br * 16 + rr]);
        for (int64_t p = h.csr.row_ptr[r]; p < h.csr.row_ptr[r + 1]; ++p)
            items.push_back(static_cast<uint64_t>(h.csr.col_idx[static_cast<size_t>(p)]) << 4 | static_cast<uint64_t>(rr));
    }
    std::sort(items.begin(), items.end());
}

// Cuts every block row into packs and derives the row classes (pack_layout.h).
void plan_packs(smat_handle& h)
{
    const smat::Bcsr& b = h.bcsr;
    const size_t nbr = static_cast<size_t>(b.nbr), n_e = b.col_idx.size();
    h.pack_ptr.assign(nbr + 1, 0);
    h.pack_first.clear();
    h.blk_pack.assign(n_e, 0);
    h.blk_meta.assign(n_e, 0);
    h.row_class.assign(nbr, 0);
    h.slots_off.assign(nbr + 1, 0);
    h.vals_off.assign(nbr + 1, 0);
    h.max_class = 0;
    h.value_bytes = 0;
    h.b_rows = 0;
    h.row_b_rows.assign(nbr, 0);
    // Cuts block row br into packs of occupied columns; with `record` the per-block records of
    // the bind-time scatter are written.  Returns the number of packs.
    struct Cut { int64_t packs, occupied; int worst; };
    auto cut_row = [&](size_t br, bool record) {
        int in_pack = 0, worst = 0;
        int64_t pack = -1, occupied = 0;
        for (int32_t s = b.row_ptr[br]; s < b.row_ptr[br + 1]; ++s) {
            const int cols = __builtin_popcount(b.col_mask[s]);
            if (pack < 0 || in_pack + cols > smat::kPackColumns) {
                ++pack;
                in_pack = 0;
                if (record) h.pack_first.push_back(s);
            }
            if (record) {
                h.blk_pack[static_cast<size_t>(s)] = static_cast<int32_t>(pack);
                h.blk_meta[static_cast<size_t>(s)] = static_cast<uint32_t>(b.col_mask[s]) | static_cast<uint32_t>(in_pack) << 16;
            }
            in_pack += cols;
            occupied += cols;
            worst = std::max(worst, in_pack);
        }
        return Cut{pack + 1, occupied, worst};
    };
    // How many stored entries per occupied column a block row of the densest class may have
    // and still be kept by entry (pack_layout.h).  A row kept by entry gathers one row of B per
    // entry instead of one per column but streams 2 bytes per entry instead of 32 per column.
    // Measured on uniformly random matrices at N = 8 ... 256: while the values kept by column
    // stay in the 256 MB Infinity Cache from launch to launch the two forms break even at about
    // 1.15 entries per column (1.08: by entry up to 6 % faster, 1.33: 10-20 % slower); once they
    // do not (290 MB), by entry is 11-22 % faster even at 1.33.
    int64_t by_column_bytes = 0;
    for (size_t br = 0; br < nbr; ++br) {
        const Cut c = cut_row(br, false);
        const int cls = c.worst <= 8 ? 0 : (c.worst <= 16 ? 1 : 2);
        by_column_bytes += (c.packs * 64 * h.elem_bytes) << (cls + 1);
    }
    const int64_t entry_limit_16ths = by_column_bytes > 192000000 ? 24 : 18;      // 3/2 or 9/8
    uint64_t units = 0, vunits = 0;
    for (size_t br = 0; br < nbr; ++br) {
        const int32_t s1 = b.row_ptr[br + 1];
        const Cut c = cut_row(br, true);
        const int64_t occupied = c.occupied;
        int cls = c.worst <= 8 ? 0 : (c.worst <= 16 ? 1 : 2);
        int64_t n_packs = c.packs;
        const int64_t nnz = block_row_nnz(h, br);
        if (cls == 2 && nnz * 16 <= occupied * entry_limit_16ths) {
            // entry row: packs of 32 stored entries; the per-block records above are not used for it
            cls = smat::kEntryClass;
            const int64_t by_entry = (nnz + 31) / 32;
            for (int64_t x = n_packs; x < by_entry; ++x) h.pack_first.push_back(s1);
            for (int64_t x = by_entry; x < n_packs; ++x) h.pack_first.pop_back();
            n_packs = by_entry;
            h.value_bytes += n_packs * 32 * h.elem_bytes;
            h.b_rows += nnz;
            h.row_b_rows[br] = static_cast<int32_t>(nnz);
        } else {
            h.value_bytes += (n_packs * 64 * h.elem_bytes) << (cls + 1);
            h.b_rows += occupied;
            h.row_b_rows[br] = static_cast<int32_t>(occupied);
        }
        h.row_class[br] = static_cast<int8_t>(cls);
        h.max_class = std::max(h.max_class, cls);
        h.slots_off[br] = static_cast<uint32_t>(units);
        h.vals_off[br] = static_cast<uint32_t>(vunits);
        units += static_cast<uint64_t>(n_packs) * static_cast<uint64_t>(smat::pack_units(cls));
        vunits += static_cast<uint64_t>(n_packs) * static_cast<uint64_t>(smat::pack_value_units(cls, h.elem_bytes));
        if (units >= (uint64_t{1} << 32) || vunits >= (uint64_t{1} << 32)) throw std::length_error("slot table too large");
        h.pack_ptr[br + 1] = static_cast<int32_t>(h.pack_first.size());
    }
    h.pack_first.push_back(static_cast<int32_t>(n_e));
    h.slots_off[nbr] = static_cast<uint32_t>(units);
    h.vals_off[nbr] = static_cast<uint32_t>(vunits);
    h.slots_units = units;
    h.vals_units = vunits;
    smat::work_order(h.pack_ptr, h.order);
}

// Launch statistics over a subset of block rows.
void row_stats(const smat_handle& h, bool skip_dense, smat::DeviceBcsr& d)
{
    int64_t longest = 0, packs = 0, rows = 0, bytes = 0, b_rows = 0;
    int cls = 0;
    for (int64_t br = 0; br < h.bcsr.nbr; ++br) {
        if (skip_dense && h.row_dense[static_cast<size_t>(br)]) continue;
        const int64_t len = h.pack_ptr[static_cast<size_t>(br) + 1] - h.pack_ptr[static_cast<size_t>(br)];
        longest = std::max(longest, len);
        packs += len;
        const int rc = h.row_class[static_cast<size_t>(br)];
        bytes += len * (rc == smat::kEntryClass ? 32 * h.elem_bytes + 128 : smat::pack_units(rc) * (128 * h.elem_bytes + 32));
        cls = std::max<int>(cls, rc);
        b_rows += h.row_b_rows[static_cast<size_t>(br)];
        ++rows;
    }
    d.n_order = rows;
    d.n_packs = packs;
    d.stream_bytes = bytes;
    d.b_rows = b_rows;
    d.max_row_packs = longest;
    d.mean_row_packs = rows ? static_cast<double>(packs) / static_cast<double>(rows) : 0.0;
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
    opt->dense_tiles = 0;
    opt->concurrent_streams = 2;
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
        if (dtype < SMAT_F16 || dtype > SMAT_I8) return fail(SMAT_ERR_INVALID_ARG, "unknown dtype");
        const bool narrow = dtype >= SMAT_E4M3;
        if (o.block_h != 16 || o.block_w != 16) return fail(SMAT_ERR_UNSUPPORTED, "only 16x16 blocks are supported");
        if (o.reorder < 0 || o.reorder > 2) return fail(SMAT_ERR_INVALID_ARG, "reorder must be 0, 1 or 2");
        if (o.reorder == 2 && o.dense_tiles == 1)
            return fail(SMAT_ERR_UNSUPPORTED, "the dense-tile kernel reads B in whole block columns: not with a column permutation");
        if (o.tau_permille < 0 || o.tau_permille > 1000) return fail(SMAT_ERR_INVALID_ARG, "tau_permille must be in 0..1000");
        if (o.dense_tiles < -1 || o.dense_tiles > 1) return fail(SMAT_ERR_INVALID_ARG, "dense_tiles must be -1, 0 or 1");
        if (o.concurrent_streams == 0) o.concurrent_streams = 2;      // a zeroed options struct: the default
        if (o.concurrent_streams < 1 || o.concurrent_streams > 16) return fail(SMAT_ERR_INVALID_ARG, "concurrent_streams must be in 1..16");
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

        std::unique_ptr<smat_handle> h(new smat_handle());      // freed if anything below throws
        h->dtype = dtype;
        h->elem_bytes = narrow ? 1 : 2;
        h->dense_mode = o.dense_tiles;
        h->n_scratch_areas = o.concurrent_streams;
        h->csr.M = M;
        h->csr.K = K;
        h->csr.row_ptr.assign(row_ptr, row_ptr + M + 1);
        h->csr.col_idx.assign(col_idx, col_idx + nnz);
        if (narrow)      // kept as 16-bit words, value in the low byte
            h->csr.vals.assign(static_cast<const uint8_t*>(vals), static_cast<const uint8_t*>(vals) + nnz);
        else
            h->csr.vals.assign(static_cast<const uint16_t*>(vals), static_cast<const uint16_t*>(vals) + nnz);
        smat::build_bcsr(h->csr, o.reorder != 0, o.tau_permille, h->bcsr);
        if (o.reorder == 2) {
            h->cols_permuted = smat::reorder_columns(h->csr, o.tau_permille, h->bcsr);
            if (h->cols_permuted) h->dense_mode = -1;
        }
        try {
            plan_packs(*h);
        } catch (const std::length_error& e) {
            return fail(SMAT_ERR_UNSUPPORTED, e.what());
        }
        plan_dense_tiles(*h);
        *out = h.release();
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

smat_status_t smat_get_dims(const smat_handle_t* h, int64_t* M, int64_t* K, int* dtype)
{
    if (!h) return fail(SMAT_ERR_INVALID_ARG, "handle is NULL");
    if (M) *M = h->csr.M;
    if (K) *K = h->csr.K;
    if (dtype) *dtype = static_cast<int>(h->dtype);
    return SMAT_OK;
}

smat_status_t smat_get_layout_info(const smat_handle_t* h, int64_t* n_packs, int64_t* value_bytes,
                                   int64_t* table_bytes, int64_t* n_columns)
{
    if (!h) return fail(SMAT_ERR_INVALID_ARG, "handle is NULL");
    if (n_packs) *n_packs = static_cast<int64_t>(h->pack_first.size()) - 1;
    if (value_bytes) *value_bytes = h->value_bytes;
    if (table_bytes) *table_bytes = static_cast<int64_t>(h->slots_units) * 32 + h->bcsr.nbr * (16 + 16 * 4);
    if (n_columns) *n_columns = h->b_rows;
    return SMAT_OK;
}

smat_status_t smat_export_perm(const smat_handle_t* h, int32_t* perm)
{
    if (!h || (!perm && h->csr.M > 0)) return fail(SMAT_ERR_INVALID_ARG, "NULL argument");
    if (h->csr.M > 0) std::memcpy(perm, h->bcsr.perm.data(), sizeof(int32_t) * static_cast<size_t>(h->csr.M));
    return SMAT_OK;
}

smat_status_t smat_export_col_perm(const smat_handle_t* h, int32_t* col_perm, int64_t* n_blocks_rows_only)
{
    if (!h || (!col_perm && h->csr.K > 0)) return fail(SMAT_ERR_INVALID_ARG, "NULL argument");
    for (int64_t c = 0; c < h->csr.K; ++c)
        col_perm[c] = h->cols_permuted ? h->bcsr.col_perm[static_cast<size_t>(c)] : static_cast<int32_t>(c);
    if (n_blocks_rows_only) *n_blocks_rows_only = h->cols_permuted ? h->bcsr.n_blocks_rows_only : h->bcsr.n_blocks;
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
        if (vals && h->elem_bytes == 2) smat::fill_canonical_vals(h->csr, h->bcsr, static_cast<uint16_t*>(vals));
        if (vals && h->elem_bytes == 1) {
            std::vector<uint16_t> wide(static_cast<size_t>(h->bcsr.n_blocks) * 256);
            smat::fill_canonical_vals(h->csr, h->bcsr, wide.data());
            std::copy(wide.begin(), wide.end(), static_cast<uint8_t*>(vals));       // low bytes
        }
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
        const size_t nbr = static_cast<size_t>(b.nbr), n_e = b.col_idx.size();
        const size_t M = static_cast<size_t>(h->csr.M), nnz = h->csr.col_idx.size();

        std::vector<int32_t> perm_padded(nbr * 16, -1);
        std::memcpy(perm_padded.data(), b.perm.data(), sizeof(int32_t) * M);
        // slot tables (pack_layout.h): the B row of every occupied column of every pack
        std::vector<uint32_t> slots(static_cast<size_t>(h->slots_units) * 8, static_cast<uint32_t>(h->csr.K));
        std::vector<uint64_t> items;
        for (size_t br = 0; br < nbr; ++br) {
            uint32_t* table = slots.data() + static_cast<size_t>(h->slots_off[br]) * 8;
            if (h->row_class[br] == smat::kEntryClass) {
                // entry row: one slot per stored entry; the entries' row numbers go into the top
                // bytes of the group's first four slots
                entry_order(*h, br, items);
                for (size_t e = 0; e < items.size(); ++e) {
                    const size_t col = static_cast<size_t>(items[e] >> 4);
                    const uint32_t rr = static_cast<uint32_t>(items[e] & 15u);
                    const int rank = static_cast<int>(e & 31), g = smat::slot_group(rank), kk = smat::slot_pos(rank);
                    uint32_t* group = table + (e >> 5) * 32 + g * 8;
                    group[kk] = (group[kk] & 0xFF000000u) |
                                (h->cols_permuted ? static_cast<uint32_t>(b.col_perm[col]) : static_cast<uint32_t>(col));
                    group[kk >> 1] |= rr << (24 + 4 * (kk & 1));
                }
                continue;
            }
            const int L = 2 << h->row_class[br];
            for (int32_t pk = h->pack_ptr[br]; pk < h->pack_ptr[br + 1]; ++pk, table += 4 * L) {
                int rank = 0;
                for (int32_t s = h->pack_first[static_cast<size_t>(pk)]; s < h->pack_first[static_cast<size_t>(pk) + 1]; ++s)
                    for (int c = 0; c < 16; ++c) {
                        if (!(b.col_mask[s] >> c & 1u)) continue;
                        // the row of B is the ORIGINAL column: through Q when the columns were permuted
                        const size_t col = static_cast<size_t>(b.col_idx[s]) * 16u + static_cast<size_t>(c);
                        table[smat::slot_group(rank) * L + smat::slot_pos(rank)] =
                            h->cols_permuted ? static_cast<uint32_t>(b.col_perm[col]) : static_cast<uint32_t>(col);
                        ++rank;
                    }
            }
        }
        // launch tables: all block rows, and those the dense path does not cover
        std::vector<int32_t> work(nbr * 4), work_rest;
        work_rest.reserve(nbr * 4);
        for (size_t x = 0; x < nbr; ++x) {
            const size_t br = static_cast<size_t>(h->order[x]);
            int32_t* rec = work.data() + 4 * x;
            rec[0] = static_cast<int32_t>(br) | (static_cast<int32_t>(h->row_class[br]) << 28);
            rec[1] = h->pack_ptr[br + 1] - h->pack_ptr[br];
            rec[2] = static_cast<int32_t>(h->slots_off[br]);
            rec[3] = static_cast<int32_t>(h->vals_off[br]);
            if (!h->row_dense[br]) work_rest.insert(work_rest.end(), rec, rec + 4);
        }

        auto up = [&](size_t off, const void* src, size_t n) -> int {
            if (n == 0) return 0;
            return static_cast<int>(hipMemcpyAsync(base + off, src, n, hipMemcpyHostToDevice, s));
        };
        int e;
        if ((e = up(l.perm, perm_padded.data(), perm_padded.size() * 4))) return hip_fail("copy perm", e);
        if ((e = up(l.work, work.data(), work.size() * 4))) return hip_fail("copy launch table", e);
        if ((e = up(l.work_rest, work_rest.data(), work_rest.size() * 4))) return hip_fail("copy launch table", e);
        if ((e = up(l.t_super, h->dense_super.data(), h->dense_super.size() * 4))) return hip_fail("copy tiles", e);
        if ((e = up(l.t_ptr, h->step_ptr.data(), h->step_ptr.size() * 4))) return hip_fail("copy tiles", e);
        if ((e = up(l.t_cols, h->step_cols.data(), h->step_cols.size() * 4))) return hip_fail("copy tiles", e);
        if ((e = up(l.t_rows, h->step_rows.data(), h->step_rows.size() * 4))) return hip_fail("copy tiles", e);
        if ((e = up(l.t_base, h->step_base.data(), h->step_base.size() * 4))) return hip_fail("copy tiles", e);
        if ((e = up(l.slots, slots.data(), slots.size() * 4))) return hip_fail("copy slot tables", e);
        if ((e = up(l.pack_ptr, h->pack_ptr.data(), h->pack_ptr.size() * 4))) return hip_fail("copy pack offsets", e);
        if ((e = up(l.vals_off, h->vals_off.data(), h->vals_off.size() * 4))) return hip_fail("copy value offsets", e);
        if ((e = up(l.row_class, h->row_class.data(), h->row_class.size()))) return hip_fail("copy row classes", e);
        if ((e = up(l.blk_ptr, b.row_ptr.data(), b.row_ptr.size() * 4))) return hip_fail("copy block offsets", e);
        if ((e = up(l.blk_col, b.col_idx.data(), n_e * 4))) return hip_fail("copy block columns", e);
        if ((e = up(l.blk_pack, h->blk_pack.data(), n_e * 4))) return hip_fail("copy block packs", e);
        if ((e = up(l.blk_meta, h->blk_meta.data(), n_e * 4))) return hip_fail("copy block masks", e);
        if ((e = up(l.csr_row_ptr, h->csr.row_ptr.data(), (M + 1) * 8))) return hip_fail("copy csr row_ptr", e);
        if ((e = up(l.csr_col_idx, h->csr.col_idx.data(), nnz * 4))) return hip_fail("copy csr col_idx", e);
        if ((e = up(l.csr_vals, h->csr.vals.data(), nnz * 2))) return hip_fail("copy csr vals", e);
        // the host vectors above must outlive the asynchronous copies: synchronised below, before they go

        smat::DeviceBcsr d;
        d.perm = reinterpret_cast<const int32_t*>(base + l.perm);
        d.work = reinterpret_cast<const int32_t*>(base + l.work);
        d.slots = reinterpret_cast<const uint32_t*>(base + l.slots);
        d.vals = base + l.vals;
        d.pack_ptr = reinterpret_cast<const int32_t*>(base + l.pack_ptr);
        d.vals_off = reinterpret_cast<const uint32_t*>(base + l.vals_off);
        d.row_class = reinterpret_cast<const int8_t*>(base + l.row_class);
        d.blk_ptr = reinterpret_cast<const int32_t*>(base + l.blk_ptr);
        d.blk_col = reinterpret_cast<const int32_t*>(base + l.blk_col);
        d.blk_pack = reinterpret_cast<const int32_t*>(base + l.blk_pack);
        d.blk_meta = reinterpret_cast<const uint32_t*>(base + l.blk_meta);
        d.M = h->csr.M;
        d.K = h->csr.K;
        d.nbr = b.nbr;
        smat::DeviceBcsr d_rest = d;
        row_stats(*h, false, d);
        row_stats(*h, true, d_rest);
        d_rest.work = reinterpret_cast<const int32_t*>(base + l.work_rest);
        smat::DenseTiles tiles;
        tiles.super_rows = reinterpret_cast<const int32_t*>(base + l.t_super);
        tiles.step_ptr = reinterpret_cast<const int32_t*>(base + l.t_ptr);
        tiles.step_cols = reinterpret_cast<const int32_t*>(base + l.t_cols);
        tiles.step_rows = reinterpret_cast<const uint32_t*>(base + l.t_rows);
        tiles.step_base = reinterpret_cast<const uint32_t*>(base + l.t_base);
        tiles.vals = base + l.t_vals;
        tiles.scratch = nullptr;           // a call takes the area of its stream
        tiles.scratch_bytes = 0;
        tiles.n = static_cast<int32_t>(h->dense_super.size());
        tiles.mean_steps = tiles.n ? static_cast<double>(h->step_rows.size()) / tiles.n : 0.0;
        tiles.cols_per_step = h->elem_bytes == 1 ? 4 : 2;
        tiles.all_full = h->dense_all_full && tiles.n > 0;
        tiles.full_steps = tiles.all_full ? h->step_ptr[1] : 0;
        h->d_csr_row_ptr = reinterpret_cast<const int64_t*>(base + l.csr_row_ptr);
        h->d_csr_col_idx = reinterpret_cast<const int32_t*>(base + l.csr_col_idx);
        h->d_csr_vals = reinterpret_cast<const uint16_t*>(base + l.csr_vals);

        if ((e = smat::launch_fill_zero(base + l.vals, static_cast<size_t>(h->vals_units) * 4, s)))
            return hip_fail("zero block values", e);
        if ((e = smat::launch_bcsr_fill(d, h->d_csr_row_ptr, h->d_csr_col_idx, h->d_csr_vals, base + l.vals, h->elem_bytes, s)))
            return hip_fail("fill block values", e);
        if ((e = smat::launch_fill_zero(base + l.t_vals, static_cast<size_t>(h->dense_slots) * 64, s)))
            return hip_fail("zero tile values", e);
        if ((e = smat::launch_dense_fill(d, tiles, h->d_csr_row_ptr, h->d_csr_col_idx, h->d_csr_vals, base + l.t_vals, h->elem_bytes, s)))
            return hip_fail("fill tile values", e);
        if ((e = static_cast<int>(hipStreamSynchronize(s)))) return hip_fail("bind synchronize", e);
        {
            // set-up is the place to find this device's copy of the static area (smat_spmm_static)
            void* area = nullptr;
            size_t area_bytes = 0;
            if ((e = smat::static_tile_scratch(&area, &area_bytes))) return hip_fail("address of the static area for partial tiles", e);
        }
        h->dev = d;
        h->dev_rest = d_rest;
        h->tiles = tiles;
        {
            std::lock_guard<std::mutex> lock(h->scratch_mutex);
            h->scratch_base = h->dense_super.empty() ? nullptr : base + l.t_scratch;
            h->scratch_owner.clear();
        }
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
        const size_t es = static_cast<size_t>(h->elem_bytes);
        std::vector<uint8_t> raw(static_cast<size_t>(h->vals_units) * 64);
        hipStream_t s = static_cast<hipStream_t>(stream);
        int e = static_cast<int>(hipMemcpyAsync(raw.data(), h->dev.vals, raw.size(), hipMemcpyDeviceToHost, s));
        if (e) return hip_fail("read block values", e);
        if ((e = static_cast<int>(hipStreamSynchronize(s)))) return hip_fail("read block values", e);
        // value number `at` of the device copy / of the canonical output, whatever the element size
        auto get = [&](size_t at) -> uint16_t {
            return es == 2 ? reinterpret_cast<const uint16_t*>(raw.data())[at] : raw[at];
        };
        auto put = [&](size_t at, uint16_t v) {
            if (es == 2) static_cast<uint16_t*>(vals)[at] = v;
            else static_cast<uint8_t*>(vals)[at] = static_cast<uint8_t>(v);
        };
        std::memset(vals, 0, n_e * 256 * es);
        std::vector<uint64_t> items;
        for (size_t br = 0; br < static_cast<size_t>(h->bcsr.nbr); ++br) {
            if (h->row_class[br] == smat::kEntryClass) {
                // entry row: the values of the stored entries in the order of the slot tables
                const size_t src0 = static_cast<size_t>(h->vals_off[br]) * (64 / es), stride = 64 / es;   // in elements
                const int32_t* bc0 = h->bcsr.col_idx.data() + h->bcsr.row_ptr[br];
                const int32_t* bc1 = h->bcsr.col_idx.data() + h->bcsr.row_ptr[br + 1];
                entry_order(*h, br, items);
                const int64_t e = static_cast<int64_t>(items.size());
                for (int64_t x = 0; x < e; ++x) {
                    const int32_t col = static_cast<int32_t>(items[static_cast<size_t>(x)] >> 4);
                    const size_t rr = static_cast<size_t>(items[static_cast<size_t>(x)] & 15u);
                    const size_t sb = static_cast<size_t>(std::lower_bound(bc0, bc1, col >> 4) - h->bcsr.col_idx.data());
                    const int rank = static_cast<int>(x & 31);
                    const size_t at = src0 + static_cast<size_t>(x >> 5) * stride +
                                      static_cast<size_t>(smat::entry_elem_index(smat::slot_group(rank), smat::slot_pos(rank)));
                    put(sb * 256 + rr * 16 + static_cast<size_t>(col & 15), get(at));
                }
                // the rest of the last pack's 32 values must have stayed zero
                for (int64_t x = e; x < (e + 31) / 32 * 32; ++x) {
                    const int rank = static_cast<int>(x & 31);
                    if (get(src0 + static_cast<size_t>(x >> 5) * stride +
                            static_cast<size_t>(smat::entry_elem_index(smat::slot_group(rank), smat::slot_pos(rank)))) != 0)
                        return fail(SMAT_ERR_HIP, "device block values: unoccupied slot is not zero");
                }
                continue;
            }
            const int L = 2 << h->row_class[br];
            const int elems = smat::pack_elems(L);
            size_t src = static_cast<size_t>(h->vals_off[br]) * (64 / es);
            for (int32_t pk = h->pack_ptr[br]; pk < h->pack_ptr[br + 1]; ++pk, src += static_cast<size_t>(elems)) {
                uint8_t used[512];
                std::memset(used, 0, sizeof(used));
                int rank = 0;
                for (int32_t sb = h->pack_first[static_cast<size_t>(pk)]; sb < h->pack_first[static_cast<size_t>(pk) + 1]; ++sb) {
                    for (int c = 0; c < 16; ++c) {
                        if (!(h->bcsr.col_mask[sb] >> c & 1u)) continue;
                        const int g = smat::slot_group(rank), kk = smat::slot_pos(rank);
                        ++rank;
                        for (int r = 0; r < 16; ++r) {
                            const int at = smat::pack_elem_index(L, r, g, kk);
                            put(static_cast<size_t>(sb) * 256 + static_cast<size_t>(r * 16 + c), get(src + static_cast<size_t>(at)));
                            used[at] = 1;
                        }
                    }
                }
                // every slot that holds no occupied column must have stayed zero
                for (int q = 0; q < elems; ++q)
                    if (!used[q] && get(src + static_cast<size_t>(q)) != 0)
                        return fail(SMAT_ERR_HIP, "device block values: unoccupied slot is not zero");
            }
        }
        return SMAT_OK;
    } catch (const std::bad_alloc&) {
        return fail(SMAT_ERR_ALLOC, "out of host memory in smat_export_device_vals");
    }
}

}  // extern "C"

namespace {

// The area of partial tiles that belongs to `stream`: the one it already owns, else the first
// free one, else none.
char* scratch_area_of(const smat_handle* h, const void* stream)
{
    if (!h->scratch_base) return nullptr;
    std::lock_guard<std::mutex> lock(h->scratch_mutex);
    for (size_t i = 0; i < h->scratch_owner.size(); ++i)
        if (h->scratch_owner[i] == stream) return h->scratch_base + i * kTileScratchBytes;
    if (static_cast<int>(h->scratch_owner.size()) >= h->n_scratch_areas) return nullptr;
    h->scratch_owner.push_back(stream);
    return h->scratch_base + (h->scratch_owner.size() - 1) * kTileScratchBytes;
}

// smat_spmm with the area for partial tiles given by the caller of this function.
// hard_limit = 0: the launch is planned so that its partial tiles fit scratch_bytes.  Otherwise it
// is planned as if the area were unlimited and refused when its partial tiles exceed hard_limit.
smat_status_t spmm_with_scratch(const smat_handle_t* h, const void* dB, int64_t ldb, void* dC, int64_t ldc,
                                int64_t N, void* stream, void* scratch, size_t scratch_bytes, size_t hard_limit = 0)
{
    // The dense path fetches B in 16-byte pieces (8 columns, or 16 for the 8-bit types) that must lie
    // wholly inside or outside the N columns; otherwise every block row goes through the per-row kernel.  It also has to pay: a tile walks its steps at about
    // 0.7 us each with little to overlap them, so few tiles leave most of the chip idle, while
    // the per-row kernel fetches every occupied column's row of B again for every block row but
    // spreads that over all compute units (about 10 TB/s of L1 fills).  Both estimates are
    // measured rates; the faster path is taken.
    const int piece = 16 / h->elem_bytes;           // columns of B in 16 bytes
    bool use_tiles = h->tiles.n > 0 && N % piece == 0 && ldb % piece == 0 && reinterpret_cast<uintptr_t>(dB) % 16 == 0;
    if (h->dense_mode < 0) use_tiles = false;
    smat::DenseTiles tiles = h->tiles;
    tiles.scratch = scratch;
    tiles.scratch_bytes = scratch ? (hard_limit ? ~size_t{0} >> 1 : scratch_bytes) : 0;
    if (use_tiles && h->dense_mode == 0) {
        const double n_tiles = static_cast<double>(tiles.n) * static_cast<double>((N + 127) / 128);
        const int ks = smat::dense_split(tiles, N);
        const double step_us = h->elem_bytes == 1 ? 1.0 : 0.7;     // an 8-bit step covers twice the block columns
        double t_tiles = std::ceil(n_tiles * ks / 256.0) * (tiles.mean_steps / ks * step_us + 4.0);
        if (ks > 1) t_tiles += 3.0 + n_tiles * (ks + 1) * 256.0 * 128.0 * 4.0 * 2.0 / 4.0e6;     // partial tiles out and in again
        // (two bytes per value also for the 8-bit types: on block-dense rows the per-row kernel did not
        // get faster with them -- 35.6 us against 35 on the band workload -- while the tile kernel did)
        const double t_rows = static_cast<double>(h->dense_columns) * static_cast<double>((N + 15) / 16 * 16) * 2.0 / 10.0e6 + 4.0;
        use_tiles = t_tiles <= t_rows;
    }
    if (use_tiles && hard_limit) {
        const size_t need = static_cast<size_t>(tiles.n) * static_cast<size_t>((N + 127) / 128) * 256 * 128 * 4 *
                            static_cast<size_t>(smat::dense_split(tiles, N));
        if (smat::dense_split(tiles, N) > 1 && need > hard_limit)
            return fail(SMAT_ERR_UNSUPPORTED, "this launch keeps " + std::to_string(need) + " bytes of partial tiles, the static area holds " +
                                                  std::to_string(hard_limit) + ": use smat_spmm, whose area is part of the workspace");
    }
    const char* variant = "";
    thread_local std::string name;
    int e = 0;
    if (use_tiles) {
        if (h->dev_rest.n_order > 0)
            e = smat::launch_spmm(h->dev_rest, h->dtype, dB, ldb, dC, ldc, N, stream, &variant);
        const char* dense_variant = "";
        if (!e) e = smat::launch_spmm_dense(h->dev, tiles, h->dtype, dB, ldb, dC, ldc, N, stream, &dense_variant);
        name = std::string(dense_variant) + (h->dev_rest.n_order > 0 ? std::string("+") + variant : std::string());
        g_kernel = name.c_str();
    } else {
        e = smat::launch_spmm(h->dev, h->dtype, dB, ldb, dC, ldc, N, stream, &variant);
        g_kernel = variant;
    }
    if (e) return hip_fail("launch spmm", e);
    return SMAT_OK;
}

// Argument checks of smat_spmm; SMAT_OK with *nothing_to_do set for an empty product.
smat_status_t check_spmm_args(const smat_handle_t* h, const void* dB, int64_t ldb, const void* dC, int64_t ldc,
                              int64_t N, bool* nothing_to_do)
{
    *nothing_to_do = false;
    if (!h) return fail(SMAT_ERR_INVALID_ARG, "handle is NULL");
    if (!h->bound) return fail(SMAT_ERR_NOT_BOUND, "smat_spmm called before smat_bind_device");
    if (N < 0) return fail(SMAT_ERR_INVALID_ARG, "N is negative");
    if (N == 0 || h->csr.M == 0) { *nothing_to_do = true; return SMAT_OK; }
    if (!dC || (!dB && h->csr.K > 0)) return fail(SMAT_ERR_INVALID_ARG, "NULL matrix pointer");
    if (ldb < N || ldc < N) return fail(SMAT_ERR_INVALID_ARG, "leading dimension smaller than N");
    if (N > 16 * 65535) return fail(SMAT_ERR_UNSUPPORTED, "N above 1048560");
    const int64_t K = h->csr.K;
    if (K > 0 && ((K - 1) * ldb + N) * h->elem_bytes >= (int64_t{1} << 31))
        return fail(SMAT_ERR_UNSUPPORTED, "B larger than 2 GiB is not supported");
    if (ldb >= (int64_t{1} << 23)) return fail(SMAT_ERR_UNSUPPORTED, "ldb must be below 2^23");
    return SMAT_OK;
}

}  // namespace

extern "C" {

smat_status_t smat_spmm(const smat_handle_t* h, const void* dB, int64_t ldb, void* dC, int64_t ldc,
                        int64_t N, void* stream)
{
    bool nothing = false;
    const smat_status_t st = check_spmm_args(h, dB, ldb, dC, ldc, N, &nothing);
    if (st != SMAT_OK || nothing) return st;
    return spmm_with_scratch(h, dB, ldb, dC, ldc, N, stream, scratch_area_of(h, stream), kTileScratchBytes);
}

smat_status_t smat_spmm_static(const smat_handle_t* h, const void* dB, int64_t ldb, void* dC, int64_t ldc,
                               int64_t N, void* stream)
{
    bool nothing = false;
    const smat_status_t st = check_spmm_args(h, dB, ldb, dC, ldc, N, &nothing);
    if (st != SMAT_OK || nothing) return st;
    void* area = nullptr;
    size_t bytes = 0;
    const int e = smat::static_tile_scratch(&area, &bytes);      // looked up at bind time; here from the cache
    if (e) return hip_fail("address of the static area for partial tiles", e);
    return spmm_with_scratch(h, dB, ldb, dC, ldc, N, stream, area, bytes, bytes);
}

// Largest block grid for which the ablation keeps a dense block map (level 0).
static constexpr int64_t kAblationMapEntries = int64_t{1} << 26;

static size_t ablation_vals_bytes(const smat_handle* h) { return align_up(static_cast<size_t>(h->bcsr.n_blocks) * 512); }
static bool ablation_has_map(const smat_handle* h) { return h->bcsr.nbr * h->bcsr.nbc <= kAblationMapEntries; }

smat_status_t smat_ablation_bytes(const smat_handle_t* h, size_t* bytes)
{
    if (!h || !bytes) return fail(SMAT_ERR_INVALID_ARG, "NULL argument");
    if (h->elem_bytes != 2) return fail(SMAT_ERR_UNSUPPORTED, "the ablation kernels handle fp16 and bf16 only");
    if (h->cols_permuted) return fail(SMAT_ERR_UNSUPPORTED, "the ablation kernels read B in whole block columns: not with a column permutation");
    size_t n = ablation_vals_bytes(h);
    if (ablation_has_map(h)) n += align_up(static_cast<size_t>(h->bcsr.nbr * h->bcsr.nbc) * sizeof(int32_t));
    *bytes = n ? n : kAlign;
    return SMAT_OK;
}

smat_status_t smat_ablation_bind(smat_handle_t* h, void* dev_area, size_t bytes, void* stream)
{
    if (!h || !dev_area) return fail(SMAT_ERR_INVALID_ARG, "NULL argument");
    if (!h->bound) return fail(SMAT_ERR_NOT_BOUND, "smat_ablation_bind needs a handle bound with smat_bind_device");
    if (reinterpret_cast<uintptr_t>(dev_area) % kAlign != 0) return fail(SMAT_ERR_INVALID_ARG, "dev_area must be 256-byte aligned");
    size_t need = 0;
    const smat_status_t st = smat_ablation_bytes(h, &need);
    if (st != SMAT_OK) return st;
    if (bytes < need) return fail(SMAT_ERR_INVALID_ARG, "dev_area too small: need " + std::to_string(need) + " bytes");
    try {
        hipStream_t s = static_cast<hipStream_t>(stream);
        char* base = static_cast<char*>(dev_area);
        const smat::Bcsr& b = h->bcsr;
        std::vector<uint16_t> vals(static_cast<size_t>(b.n_blocks) * 256);
        smat::fill_canonical_vals(h->csr, b, vals.data());
        std::vector<int32_t> map;
        if (ablation_has_map(h)) {
            map.assign(static_cast<size_t>(b.nbr * b.nbc), -1);
            for (int64_t br = 0; br < b.nbr; ++br)
                for (int32_t k = b.row_ptr[br]; k < b.row_ptr[br + 1]; ++k)
                    map[static_cast<size_t>(br * b.nbc + b.col_idx[k])] = k;
        }
        int e;
        if (!vals.empty() && (e = static_cast<int>(hipMemcpyAsync(base, vals.data(), vals.size() * 2, hipMemcpyHostToDevice, s))))
            return hip_fail("copy canonical block values", e);
        if (!map.empty() && (e = static_cast<int>(hipMemcpyAsync(base + ablation_vals_bytes(h), map.data(), map.size() * 4, hipMemcpyHostToDevice, s))))
            return hip_fail("copy block map", e);
        if ((e = static_cast<int>(hipStreamSynchronize(s)))) return hip_fail("ablation bind synchronize", e);
        smat::CanonicalBcsr& m = h->ablation;
        m.row_ptr = h->dev.blk_ptr;
        m.col_idx = h->dev.blk_col;
        m.perm = h->dev.perm;
        m.vals = reinterpret_cast<const uint16_t*>(base);
        m.block_map = map.empty() ? nullptr : reinterpret_cast<const int32_t*>(base + ablation_vals_bytes(h));
        m.M = h->csr.M;
        m.K = h->csr.K;
        m.nbr = b.nbr;
        m.nbc = b.nbc;
        h->ablation_bound = true;
        return SMAT_OK;
    } catch (const std::bad_alloc&) {
        return fail(SMAT_ERR_ALLOC, "out of host memory in smat_ablation_bind");
    }
}

smat_status_t smat_ablation_spmm(const smat_handle_t* h, int level, const void* dB, int64_t ldb, void* dC,
                                 int64_t ldc, int64_t N, void* stream)
{
    if (!h) return fail(SMAT_ERR_INVALID_ARG, "handle is NULL");
    if (!h->ablation_bound) return fail(SMAT_ERR_NOT_BOUND, "smat_ablation_spmm called before smat_ablation_bind");
    if (level < 0 || level > 2) return fail(SMAT_ERR_INVALID_ARG, "level must be 0, 1 or 2");
    if (level == 0 && !h->ablation.block_map) return fail(SMAT_ERR_UNSUPPORTED, "level 0 keeps a dense block map: block grid above 2^26 entries");
    if (N < 0) return fail(SMAT_ERR_INVALID_ARG, "N is negative");
    if (N == 0 || h->csr.M == 0) return SMAT_OK;
    if (!dC || (!dB && h->csr.K > 0)) return fail(SMAT_ERR_INVALID_ARG, "NULL matrix pointer");
    if (ldb < N || ldc < N) return fail(SMAT_ERR_INVALID_ARG, "leading dimension smaller than N");
    if (N > 16 * 65535) return fail(SMAT_ERR_UNSUPPORTED, "N above 1048560");
    const int e = smat::launch_ablation(h->ablation, level, h->dtype == SMAT_BF16, dB, ldb, static_cast<float*>(dC), ldc, N, stream);
    if (e) return hip_fail("launch ablation kernel", e);
    return SMAT_OK;
}

void smat_destroy(smat_handle_t* h) { delete h; }

const char* smat_last_error(void) { return g_error.c_str(); }

const char* smat_last_kernel(void) { return g_kernel; }

}  // extern "C"
