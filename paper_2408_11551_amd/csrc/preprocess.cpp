// Host-side preprocessing for the blocked SpMM: see preprocess.h.
//
// The clustering follows the greedy procedure of the paper's Preprocessing
// section (open a cluster with an unclustered row; every other unclustered row
// whose Jaccard distance to the cluster's column union is below the threshold
// is merged).  A row can only pass the test if it shares a block column with
// the union as it stands when the row is reached, so instead of looking at
// every row the scan walks an ascending candidate set fed from an inverted
// index (block column -> rows): when a column enters the union, every later
// unclustered row holding it becomes a candidate and its intersection counter
// goes up by one.  The counter a row carries when the scan reaches it is then
// exactly |row n union|, and rows that never became candidates have an empty
// intersection and could not have merged.  The result is the same permutation
// the row-by-row scan gives.
#include "preprocess.h"

#include <algorithm>
#include <numeric>

namespace smat {

std::string validate_csr(int64_t M, int64_t K, const int64_t* row_ptr, const int32_t* col_idx)
{
    if (row_ptr[0] != 0) return "row_ptr[0] must be 0";
    for (int64_t r = 0; r < M; ++r) {
        if (row_ptr[r + 1] < row_ptr[r]) return "row_ptr decreases at row " + std::to_string(r);
        int64_t prev = -1;
        for (int64_t p = row_ptr[r]; p < row_ptr[r + 1]; ++p) {
            const int64_t c = col_idx[p];
            if (c < 0 || c >= K) return "column out of range in row " + std::to_string(r);
            if (c <= prev) return "columns not strictly ascending in row " + std::to_string(r);
            prev = c;
        }
    }
    return std::string();
}

void block_patterns(const Csr& a, std::vector<int64_t>& pat_ptr, std::vector<int32_t>& pat_idx)
{
    pat_ptr.assign(a.M + 1, 0);
    pat_idx.clear();
    pat_idx.reserve(a.col_idx.size() / 2 + 16);
    for (int64_t r = 0; r < a.M; ++r) {
        int32_t last = -1;
        for (int64_t p = a.row_ptr[r]; p < a.row_ptr[r + 1]; ++p) {
            const int32_t bc = a.col_idx[p] / kBlock;     // columns ascend, so block columns do too
            if (bc != last) { pat_idx.push_back(bc); last = bc; }
        }
        pat_ptr[r + 1] = static_cast<int64_t>(pat_idx.size());
    }
}

namespace {

// Set of row indices that supports "insert" and "smallest member >= from", three
// levels of 64-way summary bits.
class AscendingSet {
public:
    explicit AscendingSet(int64_t n) : n_(n)
    {
        n0_ = (n + 63) / 64; n1_ = (n0_ + 63) / 64; n2_ = (n1_ + 63) / 64;
        l0_.assign(n0_ + 1, 0); l1_.assign(n1_ + 1, 0); l2_.assign(n2_ + 1, 0);
    }
    void insert(int64_t i)
    {
        l0_[i >> 6] |= 1ull << (i & 63);
        l1_[i >> 12] |= 1ull << ((i >> 6) & 63);
        l2_[i >> 18] |= 1ull << ((i >> 12) & 63);
    }
    void erase(int64_t i)
    {
        if ((l0_[i >> 6] &= ~(1ull << (i & 63))) == 0)
            if ((l1_[i >> 12] &= ~(1ull << ((i >> 6) & 63))) == 0)
                l2_[i >> 18] &= ~(1ull << ((i >> 12) & 63));
    }
    // smallest member >= from, or -1
    int64_t next(int64_t from) const
    {
        if (from >= n_) return -1;
        int64_t w0 = from >> 6;
        uint64_t bits = l0_[w0] & (~0ull << (from & 63));
        if (bits) return (w0 << 6) + __builtin_ctzll(bits);
        const int64_t i1 = w0 + 1;                       // first level-0 word still to look at
        if (i1 >= n0_) return -1;
        int64_t w1 = i1 >> 6;
        bits = l1_[w1] & (~0ull << (i1 & 63));
        if (!bits) {
            const int64_t i2 = w1 + 1;                   // first level-1 word still to look at
            if (i2 >= n1_) return -1;
            int64_t w2 = i2 >> 6;
            uint64_t b2 = l2_[w2] & (~0ull << (i2 & 63));
            while (!b2) {
                if (++w2 >= n2_) return -1;
                b2 = l2_[w2];
            }
            w1 = (w2 << 6) + __builtin_ctzll(b2);
            bits = l1_[w1];
        }
        w0 = (w1 << 6) + __builtin_ctzll(bits);
        return (w0 << 6) + __builtin_ctzll(l0_[w0]);
    }
private:
    int64_t n_, n0_, n1_, n2_;
    std::vector<uint64_t> l0_, l1_, l2_;
};

}  // namespace

// kLazy chooses how rows become candidates of the open cluster (the result is the same):
// false: every row ahead of the scan that shares a column with the union is visited; right
// where a row shares many columns with the union (the visits are few next to the counting);
// true: a row is visited only once its count could pass the merge test; right where most
// rows share a single column (one visit per count otherwise).
template <bool kLazy>
static int64_t cluster_rows(int64_t M, int64_t nbc, const std::vector<int64_t>& pat_ptr,
                            const std::vector<int32_t>& pat_idx, int tau_permille,
                            std::vector<int32_t>& order)
{
    order.clear();
    order.reserve(M);
    // inverted index: rows of every block column, ascending
    std::vector<int64_t> inv_ptr(nbc + 1, 0);
    for (int32_t c : pat_idx) ++inv_ptr[c + 1];
    for (int64_t c = 0; c < nbc; ++c) inv_ptr[c + 1] += inv_ptr[c];
    std::vector<int32_t> inv_rows(pat_idx.size());
    {
        std::vector<int64_t> fill(inv_ptr.begin(), inv_ptr.end() - 1);
        for (int64_t r = 0; r < M; ++r)
            for (int64_t q = pat_ptr[r]; q < pat_ptr[r + 1]; ++q)
                inv_rows[fill[pat_idx[q]]++] = static_cast<int32_t>(r);
    }
    std::vector<int64_t> inv_len(nbc);
    for (int64_t c = 0; c < nbc; ++c) inv_len[c] = inv_ptr[c + 1] - inv_ptr[c];

    std::vector<uint8_t> clustered(M, 0);
    // per row ahead of the scan: |row n union of the open cluster|; kLazy: twice that, + 1 if the
    // row is in the candidate set
    std::vector<int32_t> shared(M, 0);
    std::vector<int32_t> touched;             // rows with shared != 0, to be cleared when the cluster closes
    std::vector<int64_t> in_union(nbc, -1);   // id of the cluster whose union holds the column
    std::vector<int32_t> row_len(M);
    for (int64_t r = 0; r < M; ++r) row_len[r] = static_cast<int32_t>(pat_ptr[r + 1] - pat_ptr[r]);
    int64_t shortest = 0;                     // shortest non-empty pattern
    for (int64_t r = 0; r < M; ++r)
        if (row_len[r] > 0 && (shortest == 0 || row_len[r] < shortest)) shortest = row_len[r];
    AscendingSet candidates(M);
    int64_t n_clusters = 0;
    const int64_t keep = 1000 - tau_permille;

    // A column enters the union while the scan stands at row `pos`: every row ahead of the scan
    // that has the column shares one more column with the union.  kLazy: a row is only worth a visit
    // once it could pass the merge test at all.  The test at the visit, with the union U' >= U of
    // that later moment and the row's count n' of then, is 1000 n' > keep (|w| + U' - n'), which
    // implies (1000 + keep) n' > keep (|w| + U); n' is reached at the row's last increment, where
    // the same inequality with the U of that moment (smaller still) therefore holds.  So a row
    // enters the candidate set at the first increment that satisfies it, and no row that would be
    // merged is left out; the exact test is still taken at the visit.  The same bound with the
    // shortest pattern of the matrix in place of |w| comes first, so that most increments read
    // nothing but the counter.
    auto add_column = [&](int32_t c, int64_t pos, int64_t cluster, int64_t& union_size) {
        if (in_union[c] == cluster) return;
        in_union[c] = cluster;
        ++union_size;
        const int64_t least = keep * (shortest + union_size) / (1000 + keep);   // a count must exceed this to matter for any row
        int32_t* rows = inv_rows.data() + inv_ptr[c];
        int64_t kept = 0;
        for (int64_t k = 0; k < inv_len[c]; ++k) {
            const int32_t r = rows[k];
            if (clustered[r]) continue;                  // drop rows that are gone for good
            rows[kept++] = r;
            if (r > pos) {
                if constexpr (kLazy) {
                    const int32_t word = (shared[r] += 2);
                    if (word == 2) touched.push_back(r);
                    const int64_t n = word >> 1;
                    if (!(word & 1) && n > least && (1000 + keep) * n > keep * (row_len[r] + union_size)) {
                        candidates.insert(r);
                        shared[r] = word | 1;
                    }
                } else {
                    if (shared[r]++ == 0) candidates.insert(r);
                }
            }
        }
        inv_len[c] = kept;
    };

    for (int64_t v = 0; v < M; ++v) {
        if (clustered[v]) continue;
        const int64_t cluster = n_clusters++;
        clustered[v] = 1;
        order.push_back(static_cast<int32_t>(v));
        if (pat_ptr[v] == pat_ptr[v + 1]) {
            // empty seed: distance 0 to other empty rows, 1 to everything else
            if (tau_permille > 0)
                for (int64_t w = v + 1; w < M; ++w)
                    if (!clustered[w] && pat_ptr[w] == pat_ptr[w + 1]) {
                        clustered[w] = 1;
                        order.push_back(static_cast<int32_t>(w));
                    }
            continue;
        }
        int64_t union_size = 0;
        for (int64_t q = pat_ptr[v]; q < pat_ptr[v + 1]; ++q) add_column(pat_idx[q], v, cluster, union_size);
        int64_t pos = v;
        for (;;) {
            const int64_t w = candidates.next(pos + 1);
            if (w < 0) break;
            candidates.erase(w);
            pos = w;
            const int64_t inter = kLazy ? shared[w] >> 1 : shared[w];
            if constexpr (!kLazy) shared[w] = 0;        // every row with a count is visited, so this clears them all
            const int64_t uni = row_len[w] + union_size - inter;
            if (1000 * inter > keep * uni) {             // 1 - inter/uni < tau/1000
                clustered[w] = 1;
                order.push_back(static_cast<int32_t>(w));
                for (int64_t q = pat_ptr[w]; q < pat_ptr[w + 1]; ++q) add_column(pat_idx[q], w, cluster, union_size);
            }
        }
        for (int32_t r : touched) shared[r] = 0;
        touched.clear();
    }
    return n_clusters;
}

int64_t jaccard_cluster(int64_t M, int64_t nbc, const std::vector<int64_t>& pat_ptr,
                        const std::vector<int32_t>& pat_idx, int tau_permille,
                        std::vector<int32_t>& order)
{
    // A row of mean length l meets a union of about l columns in l * l / nbc of them on average:
    // below a few, most rows ahead of the scan share one column and would be visited for it.
    const double mean_len = M > 0 ? static_cast<double>(pat_idx.size()) / static_cast<double>(M) : 0.0;
    const bool lazy = nbc > 0 && mean_len * mean_len < 4.0 * static_cast<double>(nbc);
    return lazy ? cluster_rows<true>(M, nbc, pat_ptr, pat_idx, tau_permille, order)
                : cluster_rows<false>(M, nbc, pat_ptr, pat_idx, tau_permille, order);
}

int64_t count_blocks(int64_t M, int64_t nbc, const std::vector<int64_t>& pat_ptr,
                     const std::vector<int32_t>& pat_idx, const int32_t* perm)
{
    std::vector<int64_t> seen_in(nbc, -1);
    int64_t n = 0;
    for (int64_t i = 0; i < M; ++i) {
        const int64_t br = i / kBlock, r = perm[i];
        for (int64_t q = pat_ptr[r]; q < pat_ptr[r + 1]; ++q)
            if (seen_in[pat_idx[q]] != br) { seen_in[pat_idx[q]] = br; ++n; }
    }
    return n;
}

void build_bcsr(const Csr& a, bool reorder, int tau_permille, Bcsr& out)
{
    const int64_t M = a.M;
    out.nbr = (M + kBlock - 1) / kBlock;
    out.nbc = (a.K + kBlock - 1) / kBlock;
    std::vector<int64_t> pat_ptr;
    std::vector<int32_t> pat_idx;
    block_patterns(a, pat_ptr, pat_idx);

    std::vector<int32_t> ident(M);
    std::iota(ident.begin(), ident.end(), 0);
    out.n_blocks_identity = count_blocks(M, out.nbc, pat_ptr, pat_idx, ident.data());
    out.perm = ident;
    out.n_blocks = out.n_blocks_identity;
    out.used_identity = true;
    out.n_clusters = 0;
    if (reorder) {
        std::vector<int32_t> cand;
        out.n_clusters = jaccard_cluster(M, out.nbc, pat_ptr, pat_idx, tau_permille, cand);
        const int64_t n_cand = count_blocks(M, out.nbc, pat_ptr, pat_idx, cand.data());
        if (n_cand < out.n_blocks_identity) {            // strictly fewer, else keep P = I
            out.perm.swap(cand);
            out.n_blocks = n_cand;
            out.used_identity = false;
        }
    }

    // structure: per block row the ascending union of its rows' patterns
    out.row_ptr.assign(out.nbr + 1, 0);
    out.col_idx.clear();
    out.col_idx.reserve(out.n_blocks);
    std::vector<int32_t> tmp;
    for (int64_t br = 0; br < out.nbr; ++br) {
        tmp.clear();
        const int64_t i_end = std::min<int64_t>(M, (br + 1) * kBlock);
        for (int64_t i = br * kBlock; i < i_end; ++i) {
            const int64_t r = out.perm[i];
            tmp.insert(tmp.end(), pat_idx.begin() + pat_ptr[r], pat_idx.begin() + pat_ptr[r + 1]);
        }
        std::sort(tmp.begin(), tmp.end());
        tmp.erase(std::unique(tmp.begin(), tmp.end()), tmp.end());
        out.col_idx.insert(out.col_idx.end(), tmp.begin(), tmp.end());
        out.row_ptr[br + 1] = static_cast<int32_t>(out.col_idx.size());
    }

    // per block: which of its 16 columns hold a stored entry
    out.col_mask.assign(out.col_idx.size(), 0);
    std::vector<int32_t> slot_of(out.nbc, -1);
    for (int64_t br = 0; br < out.nbr; ++br) {
        for (int32_t s = out.row_ptr[br]; s < out.row_ptr[br + 1]; ++s) slot_of[out.col_idx[s]] = s;
        const int64_t i_end = std::min<int64_t>(M, (br + 1) * kBlock);
        for (int64_t i = br * kBlock; i < i_end; ++i) {
            const int64_t r = out.perm[i];
            for (int64_t p = a.row_ptr[r]; p < a.row_ptr[r + 1]; ++p) {
                const int32_t c = a.col_idx[p];
                out.col_mask[slot_of[c / kBlock]] |= static_cast<uint16_t>(1u << (c % kBlock));
            }
        }
    }

}

void work_order(const std::vector<int32_t>& cost_ptr, std::vector<int32_t>& order)
{
    // Workgroups are handed to the eight XCDs of the chip round-robin (workgroup w runs on XCD
    // w mod 8), and every XCD has its own L2.
    //  * Block rows of similar cost (longest <= 1.25 x mean): position w gets a row from the
    //    (w mod 8)-th of eight contiguous ranges of block rows, so that each XCD walks a contiguous
    //    part of the matrix and neighbouring block rows, which tend to touch the same rows of B
    //    (band and mesh matrices), share that XCD's L2.
    //  * Otherwise: longest block rows first, so that the tail of a launch is made of short
    //    ones; the round-robin then gives every XCD the same mix of lengths.
    const int64_t nbr = static_cast<int64_t>(cost_ptr.size()) - 1;
    order.resize(static_cast<size_t>(nbr > 0 ? nbr : 0));
    if (nbr <= 0) return;
    int64_t longest = 0;
    for (int64_t br = 0; br < nbr; ++br)
        longest = std::max<int64_t>(longest, cost_ptr[br + 1] - cost_ptr[br]);
    const bool even_rows = 4 * longest * nbr <= 5 * static_cast<int64_t>(cost_ptr[nbr]);
    if (even_rows) {
        constexpr int kXcds = 8;
        int64_t begin[kXcds + 1];
        for (int x = 0; x <= kXcds; ++x) begin[x] = nbr * x / kXcds;
        int64_t next[kXcds];
        for (int x = 0; x < kXcds; ++x) next[x] = begin[x];
        for (int64_t w = 0; w < nbr; ++w) {
            int x = static_cast<int>(w % kXcds);
            while (next[x] >= begin[x + 1]) x = (x + 1) % kXcds;     // that range is used up: take the next one
            order[w] = static_cast<int32_t>(next[x]++);
        }
    } else {
        std::iota(order.begin(), order.end(), 0);
        std::stable_sort(order.begin(), order.end(), [&](int32_t x, int32_t y) {
            return (cost_ptr[x + 1] - cost_ptr[x]) > (cost_ptr[y + 1] - cost_ptr[y]);
        });
    }
}

void fill_canonical_vals(const Csr& a, const Bcsr& b, uint16_t* vals)
{
    std::fill(vals, vals + static_cast<size_t>(b.n_blocks) * kBlock * kBlock, uint16_t{0});
    std::vector<int32_t> slot_of(b.nbc, -1);
    for (int64_t br = 0; br < b.nbr; ++br) {
        for (int32_t s = b.row_ptr[br]; s < b.row_ptr[br + 1]; ++s) slot_of[b.col_idx[s]] = s;
        const int64_t i_end = std::min<int64_t>(a.M, (br + 1) * kBlock);
        for (int64_t i = br * kBlock; i < i_end; ++i) {
            const int64_t r = b.perm[i];
            for (int64_t p = a.row_ptr[r]; p < a.row_ptr[r + 1]; ++p) {
                const int32_t c = a.col_idx[p];
                const size_t blk = static_cast<size_t>(slot_of[c / kBlock]);
                vals[blk * 256 + static_cast<size_t>(i % kBlock) * 16 + static_cast<size_t>(c % kBlock)] = a.vals[p];
            }
        }
    }
}

}  // namespace smat
