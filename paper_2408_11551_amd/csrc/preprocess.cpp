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
// the row-by-row scan gives.  (The index and the counters are kept per distinct
// row pattern, not per row: rows with the same pattern have the same counter.)
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

// Rows with the same pattern (the sixteen rows of a dense block row, the degrees of freedom of
// one mesh node) have the same intersection with any union, so the counting is done once per
// distinct pattern ("class"), not once per row: the inverted index lists classes, and a class
// whose count makes it a candidate puts all its unclustered rows ahead of the scan into the
// candidate set.
struct PatternClasses {
    std::vector<int32_t> class_of;     // [M]
    std::vector<int32_t> first_row;    // [n] a row that carries the class's pattern
    std::vector<int64_t> member_ptr;   // [n+1]
    std::vector<int32_t> members;      // rows of every class, ascending
};

PatternClasses group_equal_patterns(int64_t M, const std::vector<int64_t>& pat_ptr, const std::vector<int32_t>& pat_idx)
{
    std::vector<uint64_t> hash(M);
    for (int64_t r = 0; r < M; ++r) {
        uint64_t x = 0x9E3779B97F4A7C15ull ^ static_cast<uint64_t>(pat_ptr[r + 1] - pat_ptr[r]);
        for (int64_t q = pat_ptr[r]; q < pat_ptr[r + 1]; ++q) {
            x ^= static_cast<uint64_t>(static_cast<uint32_t>(pat_idx[q])) + 0x9E3779B97F4A7C15ull + (x << 6) + (x >> 2);
            x *= 0xFF51AFD7ED558CCDull;
        }
        hash[r] = x;
    }
    auto same = [&](int32_t a, int32_t b) {
        const int64_t la = pat_ptr[a + 1] - pat_ptr[a];
        return la == pat_ptr[b + 1] - pat_ptr[b] &&
               std::equal(pat_idx.begin() + pat_ptr[a], pat_idx.begin() + pat_ptr[a + 1], pat_idx.begin() + pat_ptr[b]);
    };
    auto less = [&](int32_t a, int32_t b) {            // a total order in which equal patterns are neighbours
        if (hash[a] != hash[b]) return hash[a] < hash[b];
        const auto a0 = pat_idx.begin() + pat_ptr[a], a1 = pat_idx.begin() + pat_ptr[a + 1];
        const auto b0 = pat_idx.begin() + pat_ptr[b], b1 = pat_idx.begin() + pat_ptr[b + 1];
        if (std::lexicographical_compare(a0, a1, b0, b1)) return true;
        if (std::lexicographical_compare(b0, b1, a0, a1)) return false;
        return a < b;                                   // same pattern: by row, so that members ascend
    };
    std::vector<int32_t> by_pattern(M);
    std::iota(by_pattern.begin(), by_pattern.end(), 0);
    std::sort(by_pattern.begin(), by_pattern.end(), less);
    PatternClasses pc;
    pc.class_of.assign(M, 0);
    pc.member_ptr.push_back(0);
    for (int64_t k = 0; k < M; ++k) {
        const int32_t r = by_pattern[k];
        if (k == 0 || !same(by_pattern[k - 1], r)) {
            if (k > 0) pc.member_ptr.push_back(static_cast<int64_t>(pc.members.size()));
            pc.first_row.push_back(r);
        }
        pc.class_of[r] = static_cast<int32_t>(pc.first_row.size()) - 1;
        pc.members.push_back(r);                        // ascending inside a class: ties are ordered by row
    }
    pc.member_ptr.push_back(static_cast<int64_t>(pc.members.size()));
    if (M == 0) pc.member_ptr.assign(1, 0);
    return pc;
}

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
    const PatternClasses pc = group_equal_patterns(M, pat_ptr, pat_idx);
    const int64_t n_classes = static_cast<int64_t>(pc.first_row.size());
    auto class_begin = [&](int64_t k) { return pat_ptr[pc.first_row[k]]; };
    auto class_end = [&](int64_t k) { return pat_ptr[pc.first_row[k] + 1]; };
    // inverted index: classes of every block column
    std::vector<int64_t> inv_ptr(nbc + 1, 0);
    for (int64_t k = 0; k < n_classes; ++k)
        for (int64_t q = class_begin(k); q < class_end(k); ++q) ++inv_ptr[pat_idx[q] + 1];
    for (int64_t c = 0; c < nbc; ++c) inv_ptr[c + 1] += inv_ptr[c];
    std::vector<int32_t> inv_classes(static_cast<size_t>(inv_ptr[nbc]));
    {
        std::vector<int64_t> fill(inv_ptr.begin(), inv_ptr.end() - 1);
        for (int64_t k = 0; k < n_classes; ++k)
            for (int64_t q = class_begin(k); q < class_end(k); ++q)
                inv_classes[fill[pat_idx[q]]++] = static_cast<int32_t>(k);
    }
    std::vector<int64_t> inv_len(nbc);
    for (int64_t c = 0; c < nbc; ++c) inv_len[c] = inv_ptr[c + 1] - inv_ptr[c];

    std::vector<uint8_t> clustered(M, 0);
    std::vector<int32_t> alive(n_classes);    // unclustered rows of the class
    for (int64_t k = 0; k < n_classes; ++k) alive[k] = static_cast<int32_t>(pc.member_ptr[k + 1] - pc.member_ptr[k]);
    // per class: 2 * |pattern n union of the open cluster| + (1 if its rows are in the candidate set)
    std::vector<int32_t> shared(n_classes, 0);
    std::vector<int32_t> touched;             // classes with shared != 0, cleared when the cluster closes
    std::vector<int64_t> in_union(nbc, -1);   // id of the cluster whose union holds the column
    std::vector<int32_t> class_len(n_classes);
    int64_t shortest = 0;                     // shortest non-empty pattern
    for (int64_t k = 0; k < n_classes; ++k) {
        class_len[k] = static_cast<int32_t>(class_end(k) - class_begin(k));
        if (class_len[k] > 0 && (shortest == 0 || class_len[k] < shortest)) shortest = class_len[k];
    }
    AscendingSet candidates(M);
    int64_t n_clusters = 0;
    const int64_t keep = 1000 - tau_permille;

    // A column enters the union while the scan stands at row `pos`: every class that has the
    // column shares one more column with the union, and so does each of its rows.  Only rows
    // ahead of the scan can still be visited; their count when the scan reaches them is the
    // class's.  kLazy: a row is only worth a visit once it could pass the merge test at all.  The
    // test at the visit, with the union U' >= U of that later moment and the count n' of then, is
    // 1000 n' > keep (|w| + U' - n'), which implies (1000 + keep) n' > keep (|w| + U); n' is
    // reached at the last increment, where the same inequality with the U of that moment (smaller
    // still) therefore holds.  So the rows of a class enter the candidate set at the first
    // increment that satisfies it, and no row that would be merged is left out; the exact test is
    // still taken at the visit.  The same bound with the shortest pattern of the matrix in place
    // of |w| comes first, so that most increments read nothing but the counter.
    auto add_column = [&](int32_t c, int64_t pos, int64_t cluster, int64_t& union_size) {
        if (in_union[c] == cluster) return;
        in_union[c] = cluster;
        ++union_size;
        const int64_t least = keep * (shortest + union_size) / (1000 + keep);   // a count must exceed this to matter for any row
        int32_t* classes = inv_classes.data() + inv_ptr[c];
        int64_t kept = 0;
        for (int64_t x = 0; x < inv_len[c]; ++x) {
            const int32_t k = classes[x];
            if (alive[k] == 0) continue;                 // drop classes that are gone for good
            classes[kept++] = k;
            const int32_t word = (shared[k] += 2);
            if (word == 2) touched.push_back(k);
            if (word & 1) continue;                      // its rows are candidates already
            const int64_t n = word >> 1;
            if (kLazy && !(n > least && (1000 + keep) * n > keep * (class_len[k] + union_size))) continue;
            shared[k] = word | 1;
            for (int64_t y = pc.member_ptr[k]; y < pc.member_ptr[k + 1]; ++y) {
                const int32_t r = pc.members[y];
                if (r > pos && !clustered[r]) candidates.insert(r);
            }
        }
        inv_len[c] = kept;
    };

    for (int64_t v = 0; v < M; ++v) {
        if (clustered[v]) continue;
        const int64_t cluster = n_clusters++;
        clustered[v] = 1;
        --alive[pc.class_of[v]];
        order.push_back(static_cast<int32_t>(v));
        if (pat_ptr[v] == pat_ptr[v + 1]) {
            // empty seed: distance 0 to other empty rows, 1 to everything else
            if (tau_permille > 0)
                for (int64_t w = v + 1; w < M; ++w)
                    if (!clustered[w] && pat_ptr[w] == pat_ptr[w + 1]) {
                        clustered[w] = 1;
                        --alive[pc.class_of[w]];
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
            const int32_t k = pc.class_of[w];
            const int64_t inter = shared[k] >> 1;
            const int64_t uni = class_len[k] + union_size - inter;
            if (1000 * inter > keep * uni) {             // 1 - inter/uni < tau/1000
                clustered[w] = 1;
                --alive[k];
                order.push_back(static_cast<int32_t>(w));
                if (inter < class_len[k])                // otherwise every column of the row is in the union already
                    for (int64_t q = pat_ptr[w]; q < pat_ptr[w + 1]; ++q) add_column(pat_idx[q], w, cluster, union_size);
            }
        }
        for (int32_t k : touched) shared[k] = 0;
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

static void build_structure(const Csr& a, const std::vector<int64_t>& pat_ptr, const std::vector<int32_t>& pat_idx, Bcsr& out);

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

    build_structure(a, pat_ptr, pat_idx, out);
}

// Row pointer, block columns and column masks of the BCSR of A' = P A for the permutation
// already in out.perm.
static void build_structure(const Csr& a, const std::vector<int64_t>& pat_ptr, const std::vector<int32_t>& pat_idx, Bcsr& out)
{
    const int64_t M = a.M;
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

bool reorder_columns(Csr& a, int tau_permille, Bcsr& b)
{
    const int64_t M = a.M, K = a.K;
    b.col_perm.resize(static_cast<size_t>(K));
    std::iota(b.col_perm.begin(), b.col_perm.end(), 0);
    b.n_blocks_rows_only = b.n_blocks;
    if (K == 0 || M == 0) return false;
    // column patterns: ascending block rows of A' = P A per column (rows are walked in their new order)
    std::vector<int64_t> cpat_ptr(K + 1, 0);
    std::vector<int32_t> last(K, -1);
    for (int64_t i = 0; i < M; ++i) {
        const int64_t r = b.perm[i];
        const int32_t br = static_cast<int32_t>(i / kBlock);
        for (int64_t p = a.row_ptr[r]; p < a.row_ptr[r + 1]; ++p)
            if (last[a.col_idx[p]] != br) { last[a.col_idx[p]] = br; ++cpat_ptr[a.col_idx[p] + 1]; }
    }
    for (int64_t c = 0; c < K; ++c) cpat_ptr[c + 1] += cpat_ptr[c];
    std::vector<int32_t> cpat_idx(static_cast<size_t>(cpat_ptr[K]));
    {
        std::vector<int64_t> fill(cpat_ptr.begin(), cpat_ptr.end() - 1);
        std::fill(last.begin(), last.end(), -1);
        for (int64_t i = 0; i < M; ++i) {
            const int64_t r = b.perm[i];
            const int32_t br = static_cast<int32_t>(i / kBlock);
            for (int64_t p = a.row_ptr[r]; p < a.row_ptr[r + 1]; ++p)
                if (last[a.col_idx[p]] != br) { last[a.col_idx[p]] = br; cpat_idx[fill[a.col_idx[p]]++] = br; }
        }
    }
    std::vector<int32_t> cand;
    jaccard_cluster(K, b.nbr, cpat_ptr, cpat_idx, tau_permille, cand);
    const int64_t n_cand = count_blocks(K, b.nbr, cpat_ptr, cpat_idx, cand.data());     // blocks of the transpose = blocks of P A Q
    if (n_cand >= b.n_blocks) return false;              // strictly fewer, else keep Q = I
    b.col_perm.swap(cand);
    // A <- A Q: entry (r, c) moves to the new index of column c; columns ascend again inside every row
    std::vector<int32_t> new_of_old(static_cast<size_t>(K));
    for (int64_t c = 0; c < K; ++c) new_of_old[b.col_perm[c]] = static_cast<int32_t>(c);
    std::vector<std::pair<int32_t, uint16_t>> row;
    for (int64_t r = 0; r < M; ++r) {
        row.clear();
        for (int64_t p = a.row_ptr[r]; p < a.row_ptr[r + 1]; ++p) row.emplace_back(new_of_old[a.col_idx[p]], a.vals[p]);
        std::sort(row.begin(), row.end());
        for (size_t x = 0; x < row.size(); ++x) {
            a.col_idx[a.row_ptr[r] + static_cast<int64_t>(x)] = row[x].first;
            a.vals[a.row_ptr[r] + static_cast<int64_t>(x)] = row[x].second;
        }
    }
    std::vector<int64_t> pat_ptr;
    std::vector<int32_t> pat_idx;
    block_patterns(a, pat_ptr, pat_idx);
    b.n_blocks = n_cand;
    build_structure(a, pat_ptr, pat_idx, b);
    return true;
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
