// HIP kernels for gfx950: the SpMM path for block-dense parts of the matrix.
//
// Where sixteen consecutive block rows (a "super row", 256 rows of A') share most of their
// block columns, multiplying every block row on its own makes each wave fetch the same rows
// of B again.  Here one workgroup takes a super row and a slab of 128 columns of B and C and
// walks the UNION of the super row's block columns, two at a time (one MFMA 16x16x32 step):
// the 32 x 128 panel of B of a step is staged once in LDS and read by all four waves, each
// of which owns four of the sixteen block rows and keeps a 64 x 128 accumulator tile in
// registers.  A B operand built from LDS is reused for the wave's four block rows.  A block
// row that has neither block of a step stores nothing for it and multiplies zeros (its loads
// are out of range): the loop has no branches.
//
// This is still the paper's scheme (Implementation section, Alg. 1): per output tile, loop over
// stored blocks and multiply-accumulate on the matrix units; the loop is merely shared by the
// block rows of a super row so that the panel of B is read once for all of them.
#include <algorithm>
#include <cstdio>
#include <mutex>
#include <type_traits>

#include <hip/hip_runtime.h>

#include "kernels.h"
#include "mfma_types.h"

namespace smat {

namespace {

constexpr uint32_t kOutOfRange = 0x80000000u;
constexpr int kRsrcFlags = 0x00020000;

__device__ __forceinline__ u32x4 buf_load16(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff)
{
    const i32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 0);
    return u32x4{static_cast<uint32_t>(v[0]), static_cast<uint32_t>(v[1]), static_cast<uint32_t>(v[2]), static_cast<uint32_t>(v[3])};
}

}  // namespace

// ---------------------------------------------------------------------------------------------
// The tile kernel: C rows of the dense super rows, 128 columns per workgroup; 4 waves per group,
// wave w owns block rows 4w..4w+3 of the super row.  With gridDim.z > 1 the steps of a tile are
// split over that many workgroups; each writes its partial 256 x 128 tile to the scratch area
// and a second kernel adds the partial tiles in a fixed order (reproducible; fp32 atomics on C
// were measured at three times the cost of the idle compute units they were meant to fill).
//
// KG = 1: one group of four waves per workgroup, two workgroups per compute unit; for super
// rows of few steps, where the start and the write of C of one workgroup overlap the loop of
// the other.  KG = 2 puts two groups of four waves into one workgroup: group 0 walks the even
// steps of the tile, group 1 the odd ones, each with its own panel buffers, and at the end
// group 1 hands its accumulators to group 0 through LDS; for long super rows, also when every
// compute unit gets only one tile.  Every variant stays within 256 registers, so that a SIMD
// holds two waves whose waits and matrix instructions overlap.
//
// DT is the operand type.  A step of the 16-bit types is two block columns (the 32 k slots of
// one MFMA 16x16x32); the 8-bit types take four (two sub-steps of 32 k slots): a block row's
// values for a step are again 1 KiB (sixteen bytes per lane, eight per sub-step), the panel of B
// is 64 rows of 128 bytes, so a step moves the same bytes as a 16-bit one and a tile has half as
// many steps.  int8 multiplies both sub-steps with one instruction (16x16x64, sixteen bytes per
// lane and operand, twice the rate); the 8-bit floats take two MFMA 16x16x32.
//
// A wave has 512 clocks of matrix work per step, while a load takes a few thousand clocks under
// load, and whatever a wave does right behind a barrier happens at the same moment in all eight
// waves of the compute unit.  So
//   * the panel of B goes from memory straight into LDS (buffer loads with the LDS modifier:
//     lane l of a wave delivers 16 bytes to M0 + 16 l, so a wave fills 1 KiB of panel rows with
//     one instruction and no register is spent on staging), into a ring of three panels, two
//     steps ahead;
//   * the block values sit in a register ring of three steps, two steps ahead;
//   * the right operand of a matrix instruction -- eight k-consecutive values of one column per
//     lane, out of a panel that holds rows of B -- comes from two transposing LDS reads
//     (ds_read_b64_tr_b16 / _b8) per group of sixteen columns, asked for one group ahead of its
//     use: no byte permutes, no registers for the panel's rows, and the first matrix instruction
//     of a step waits for two reads instead of the whole panel (a 4096 x 4096 x 2048 product:
//     bf16 70 -> 63 us; e4m3 66 -> 53 us and int8 56 -> 40 us against the kernel that staged the
//     panel through registers and built operands with permutes);
//   * every thread waits for its own loads of the step (in-order counter: all but the youngest
//     six), one barrier makes the panel visible, and the loads of the next two steps stay in
//     flight across it -- twelve KiB per wave;
//   * the six loads of a step are not issued together behind the barrier -- forty-eight loads at
//     once kept every wave waiting at its load instructions while the matrix units idled, and the
//     time of the loads and the time of the matrix instructions added up (measured by leaving out
//     one or the other) -- but one by one between the groups of matrix instructions.
// Built, measured and set aside: the panel staged through registers with operands by byte permutes
// (the first form of this kernel), with prefetch rings of two to four steps; a 256-column tile with
// 256 accumulators per lane in the accumulation registers (9 % faster than one group at N = 4096,
// slower than two); the panel read from LDS in two halves around the matrix instructions; requests
// for the lines of later steps through the scalar cache (88 us against 79 us at the time);
// transposing reads two groups ahead (65 against 63 us); a ring of four steps with the transposing reads (no
// change, hot or on flushed caches).
// The tiles are numbered so that the workgroups an XCD runs (every eighth in dispatch order) form
// compact rectangles of super rows x column slabs: the tile values of a super row and the panel rows
// of a slab then miss that XCD's L2 once and hit it for the other workgroups that walk them at the
// same time.
constexpr int kTileGroup = 4;          // super rows of a rectangle

// What the host and the kernel agree on: tile number -> (index of the super row, column slab).
struct TileOrder {
    int n_super, n_slab, per_xcd;      // per_xcd = ceil(tiles / 8)
};
// What the tile kernel needs later than its first loads (DenseTiles and DeviceBcsr have the rest).
struct TileTables {
    const int32_t* step_cols;
    const uint32_t* step_rows;
    const uint32_t* step_base;
    const int32_t* perm;
    void* scratch;
};

__device__ __forceinline__ uint32_t lds_offset_of(const void* p)
{
    return static_cast<uint32_t>(reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) const char*)p));
}

// One load straight into LDS: every lane fetches the 16 bytes at voff + soff of the buffer (zeros
// when out of range), and the wave's 64 pieces land back to back from lds_addr on (wave-uniform).
// The compiler counts it among the outstanding memory loads like any other.
typedef __attribute__((address_space(3))) void lds_void;
__device__ __forceinline__ void load_to_lds16(lds_void* lds_addr, __amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff)
{
    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, lds_addr, 16, voff, soff, 0, 0);
}

// Reads of what such loads delivered.  They are written as assembly so that the compiler does not
// see an LDS read at all: it would hold every such read back until the most recent load into LDS
// has completed (it cannot tell the ring's panels apart), which is the look-ahead this kernel is
// for.  The panel's arrival is awaited by hand and made visible by a barrier.  (None of the
// assembly statements of this kernel claims to touch memory: the compiler would then no longer
// fetch the per-step tables with scalar loads, and its vector loads would wait for everything.)
//
// Transposing read (gfx950): every lane names eight bytes (four 16-bit elements of one row); inside
// each group of sixteen lanes, lane i receives element i % 4 of the pieces named by lanes i / 4,
// i / 4 + 4, i / 4 + 8 and i / 4 + 12, in that order -- four k-consecutive elements of one column
// when those four lanes name four consecutive rows.
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
template <int OFFSET>
__device__ __forceinline__ u32x2_t lds_read_tr(uint32_t addr)
{
    u32x2_t v;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFFSET));
    return v;
}
// The same for bytes: a lane names eight bytes of a row, and lane i receives byte i % 8 of the pieces
// named by lanes i / 8, i / 8 + 2, ..., i / 8 + 14 -- eight k-consecutive bytes of one column when
// those eight lanes name eight consecutive rows.
template <int OFFSET>
__device__ __forceinline__ u32x2_t lds_read_tr8(uint32_t addr)
{
    u32x2_t v;
    asm volatile("ds_read_b64_tr_b8 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFFSET));
    return v;
}
// the two reads into lo and hi have returned once at most YOUNGER later LDS reads are outstanding
template <int YOUNGER>
__device__ __forceinline__ void lds_pair_done(u32x2_t& lo, u32x2_t& hi)
{
    asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(lo), "+v"(hi) : "n"(YOUNGER));
}

template <int DT, int KG, bool FULL = false>
__global__ __launch_bounds__(256 * KG)
__attribute__((amdgpu_waves_per_eu(2, 2)))
void spmm_tile_kernel(int n_super, int n_slab, int per_xcd, int N, const int32_t* __restrict__ super_rows,
                      const void* steps_arg, const void* __restrict__ B, const void* __restrict__ tile_vals,
                      uint32_t ldb_bytes, uint32_t K, TileTables tab, typename Elem<DT>::Out* __restrict__ C, int64_t ldc)
{
    // The fourteen words in front are what the first loads of a tile are computed from; the compiler is asked (build
    // flag) to have the dispatcher place them in scalar registers, so that a workgroup does not begin by waiting
    // for a load of its own arguments.  n_super, n_slab, per_xcd: the tile order; steps_arg: the table of the super
    // rows' first steps, or (FULL, where the tables are computed) the number of steps of every super row; K: rows of B.
    const int32_t* __restrict__ step_ptr = static_cast<const int32_t*>(steps_arg);
    const int full_steps = static_cast<int>(reinterpret_cast<uintptr_t>(steps_arg));
    constexpr uint32_t kElemBytes = Elem<DT>::ES;
    // (the rows' padding after the last row is not B's.  Said to be wave-uniform in so many words: the compiler has
    // computed it on the vector unit and then wrapped every load through the descriptor into a loop over lanes.)
    const uint32_t b_bytes = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(
        static_cast<int>(K > 0u ? (K - 1u) * ldb_bytes + static_cast<uint32_t>(N) * kElemBytes : 0u)));
    using Acc = typename Elem<DT>::Acc;
    using Out = typename Elem<DT>::Out;
    constexpr int ES = Elem<DT>::ES;               // bytes per element of A and B
    constexpr int KS = ES == 1 ? 2 : 1;            // sub-steps of 32 k slots (two block columns) per step
    constexpr int NT = 8;                          // groups of 16 columns: 128 columns per tile
    constexpr int RM = 4;                          // block rows per wave
    constexpr int RD = 3;                          // ring depth: panels in LDS, steps of block values in registers
    // per wave group, RD panels of 8 KiB: 32 rows of B x 128 columns of two bytes, or 64 rows x 128 columns of one
    // byte; the two groups' hand-over at the end needs 128 KiB
    constexpr int kLdsWords = KG == 2 ? (KG * RD * 32 * 16 > 8192 ? KG * RD * 32 * 16 : 8192) : KG * RD * 32 * 16;
    __shared__ u32x4 lds_words[kLdsWords];

    // tile of this workgroup: the XCD's share of the tile numbers is contiguous
    const int tile = static_cast<int>(blockIdx.x % 8u) * per_xcd + static_cast<int>(blockIdx.x / 8u);
    if (tile >= n_super * n_slab) return;
    const int band = tile / (kTileGroup * n_slab), in_band = tile % (kTileGroup * n_slab);
    const int band_rows = min(kTileGroup, n_super - kTileGroup * band);
    const int sidx = kTileGroup * band + in_band % band_rows;
    const int slab = in_band / band_rows;

    const int tid = threadIdx.x & 255;             // thread inside its wave group
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);             // wave inside its group
    const int kg = KG == 1 ? 0 : __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x) >> 8);
    const int i = lane & 15, g = lane >> 4;
    const int super = super_rows[sidx];
    const int n0 = slab * 128;
    const int ks = static_cast<int>(gridDim.z);    // workgroups sharing this tile's steps
    // (a matrix all of whose blocks are stored: the tables would say what can be computed, at the price of two
    // dependent round trips to memory before the first load of the tile can be issued)
    const int q_first = FULL ? sidx * full_steps : step_ptr[sidx];
    const int q_last = FULL ? q_first + full_steps : step_ptr[sidx + 1];
    const int per = (q_last - q_first + ks - 1) / ks;
    const int q0 = min(q_first + static_cast<int>(blockIdx.z) * per, q_last);
    const int q1 = min(q0 + per, q_last);
    const int nq = q1 - q0;

    const __amdgpu_buffer_rsrc_t b_rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(B), 0, static_cast<int>(b_bytes), kRsrcFlags);
    // tile values of this workgroup's steps q0..q1-1 are stored back to back
    const uint32_t first_slot = nq <= 0 ? 0u : FULL ? 16u * static_cast<uint32_t>(q0) : tab.step_base[q0];
    const uint32_t end_slot = nq <= 0 ? 0u : FULL ? 16u * static_cast<uint32_t>(q1) : tab.step_base[q1 - 1] + __popc(tab.step_rows[q1 - 1]);
    const __amdgpu_buffer_rsrc_t a_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        static_cast<uint8_t*>(const_cast<void*>(tile_vals)) + static_cast<size_t>(first_slot) * 1024, 0,
        static_cast<int>((end_slot - first_slot) * 1024u), kRsrcFlags);

    // A wave's share of a panel is two loads of 1 KiB, lane l delivering the 16 bytes at position 16 l.
    // 16-bit types: panel rows of 256 bytes, rows 0..15 the step's first block column, 16..31 its second;
    // load e brings rows 4 wave .. 4 wave + 3 of block column e, lane l the piece l & 15 of row l >> 4.
    // 8-bit types: panel rows of 128 bytes, rows 16 c .. 16 c + 15 the step's c-th block column (c < 4);
    // the wave brings block column `wave`, load e its rows 8 e .. 8 e + 7, lane l the piece l & 7 of row l >> 3.
    // (N is a multiple of the columns of a piece on this path, so a piece is all inside or all outside.)
    const int st_row = ES == 2 ? 4 * wave + (lane >> 4) : lane >> 3;
    // The piece that lands at position p of row r of the panel is piece p ^ 2 (r & 3) ^ 8 (r / 8 & 1) of that
    // row of B (8-bit: p ^ (r / 2 & 7)).  LDS has 64 banks of four bytes and serves 32 lanes of an 8-byte read
    // per clock; the 32 lanes of a transposing read name rows 8 g + e of two lane groups g -- four rows e x
    // 32 bytes each with 256-byte rows, eight rows x 16 bytes with 128-byte rows -- and with this placement
    // they hit every bank once.  (Placed for sixteen lanes only, p ^ 2 (r & 3) and p ^ (r & 7), the two
    // lane groups met in the same banks: the counters showed a bank conflict in 47 % of the LDS cycles.)
    // (16-bit: r = 16 e + 4 wave + lane / 16 for load e; 8-bit: r = 16 wave + 8 e + lane / 8, so the two loads of a
    // wave differ in the placement)
    uint32_t st_off_of[2];
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int st_piece = ES == 2 ? (lane & 15) ^ (2 * ((lane >> 4) & 3)) ^ (8 * ((wave >> 1) & 1))
                                     : (lane & 7) ^ (4 * e + (lane >> 4));
        const int st_col = n0 + (16 / ES) * st_piece;
        st_off_of[e] = st_col < N ? static_cast<uint32_t>(st_col) * ES : kOutOfRange;
    }
    const uint32_t no_row = K;
    const int nbc = static_cast<int>((K + 15u) >> 4);
    const uint32_t panels = lds_offset_of(lds_words) + static_cast<uint32_t>(kg) * (RD * 8192);   // this group's ring
    // where load e of this wave goes in panel buf
    auto lds_of_load = [&](int buf, int e) {
        return panels + static_cast<uint32_t>(buf) * 8192u + (ES == 2 ? 4096u * e + 1024u * wave : 2048u * wave + 1024u * e);
    };
    // Where this lane reads (+ 8192 per panel).  16-bit: lane (g, j) names row 8 g + j / 4 (+ 4 for the
    // second read, + 1024 bytes) and, for the group of columns 16 x .. 16 x + 15, the eight bytes of columns
    // 16 x + 4 (j % 4) ..: piece 2 x + (j % 4) / 2 of the row, which lies at position
    // (2 x + (j % 4) / 2) ^ 2 (j / 4) ^ 8 (g & 1).  8-bit: row 8 g + j / 2 of the first sub-step (the second: + 32 rows,
    // + 4096 bytes), the eight bytes of columns 16 x + 8 (j % 2) ..: half j % 2 of piece x, at position
    // x ^ (4 (g & 1) + j / 4).
    constexpr uint32_t kSecondRead = ES == 2 ? 1024u : 4096u;
    uint32_t tr_addr[8];
    {
#pragma unroll
        for (int x = 0; x < 8; ++x) {
            if constexpr (ES == 2) {
                const int e = i >> 2, qq = i & 3;
                tr_addr[x] = panels + (8 * g + e) * 256u + 32u * (x ^ e ^ (4 * (g & 1))) + 16u * (qq >> 1) + 8u * (qq & 1);
            } else {
                const int e = i >> 1, qq = i & 1;
                tr_addr[x] = panels + (8 * g + e) * 128u + 16u * (x ^ (4 * (g & 1) + (e >> 1))) + 8u * qq;
            }
        }
    }

    // What a step's loads need to know, fetched with scalar loads a step before it is used.  A
    // step past the group's last one names no block column (its panel rows read zeros) and no block
    // row (its block values read zeros).
    // (c: the block columns this wave brings into LDS -- both of a 16-bit step, or the wave's one of an 8-bit step's four)
    struct StepMeta { int c[2]; uint32_t rows, base; };
    // (The tables are written at bind time and never while a kernel runs.  Reading them through the
    // constant address space tells the compiler so: the loads stay scalar even though the loop
    // contains loads that write LDS, which it takes for writes to anything.)
    typedef __attribute__((address_space(4))) const int32_t* const_i32;
    typedef __attribute__((address_space(4))) const uint32_t* const_u32;
    const const_i32 step_cols = (const_i32)tab.step_cols;
    const const_u32 step_rows = (const_u32)tab.step_rows, step_base = (const_u32)tab.step_base;
    auto is_live = [&](int gs) { return kg + KG * gs < nq; };      // step gs of this wave group = step kg + KG * gs of the tile
    auto fetch_meta = [&](int gs) {
        const bool live = is_live(gs);
        const size_t q = static_cast<size_t>(q0 + (live ? kg + KG * gs : nq - 1));     // clamped: the loads are unconditional
        // nothing is computed from the loaded words here: they are first looked at a step later,
        // so the wave does not wait for the scalar loads
        StepMeta m;
        if constexpr (FULL) {
            // a matrix all of whose blocks are stored: step q of the super row has the block columns
            // 2q and 2q+1 (8-bit: 4q .. 4q+3) and a block of every block row -- nothing to look up (3 % of a launch)
            const int rel = static_cast<int>(q) - q_first;
            m.c[0] = 2 * KS * rel + (ES == 2 ? 0 : wave);
            m.c[1] = 2 * KS * rel + 1;
            m.rows = 0xFFFFu;
            m.base = first_slot + 16u * static_cast<uint32_t>(static_cast<int>(q) - q0);
            return m;
        }
        m.c[0] = step_cols[(2 * KS) * q + (ES == 2 ? 0 : wave)];
        m.c[1] = ES == 2 ? step_cols[(2 * KS) * q + 1] : 0;
        m.rows = step_rows[q];
        m.base = step_base[q];
        return m;
    };
    // e-th load of the wave's share of the step's panel (e = 0, 1): one load into LDS
    auto load_panel_half = [&](const StepMeta& m, bool live, int buf, int e) {
        // rows past K (ragged last block column, or no such column) are out of range: zeros
        int c = ES == 2 && e == 1 ? m.c[1] : m.c[0];
        c = live ? c : 0x7FFFFFFF;
        uint32_t row = c < nbc ? static_cast<uint32_t>(c) * 16u + (ES == 2 ? 0 : 8 * e) + st_row : no_row;
        row = row < no_row ? row : no_row;
        load_to_lds16((lds_void*)(uintptr_t)lds_of_load(buf, e), b_rsrc, __umul24(row, ldb_bytes) + st_off_of[e], 0u);
    };
    auto load_panel = [&](const StepMeta& m, bool live, int buf) {
        load_panel_half(m, live, buf, 0);
        load_panel_half(m, live, buf, 1);
    };
    // Values of the wave's r-th block row for a step.  A block row without data in the step reads
    // out of range (zeros) and multiplies zeros: no branches in the loop body.
    auto load_a_row = [&](const StepMeta& m, bool live, int r) {
        const uint32_t rows = live ? m.rows : 0u;
        const int j = RM * wave + r;
        const uint32_t slot = m.base - first_slot + __popc(rows & ((1u << j) - 1u));
        const uint32_t absent = (rows >> j & 1u) ? 0u : kOutOfRange;                      // wave-uniform
        // (the slot is wave-uniform; saying so keeps it in a scalar register whatever the pressure there)
        return buf_load16(a_rsrc, (static_cast<uint32_t>(lane) * 16u) | absent,
                          static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(slot * 1024u))));
    };
    auto load_a = [&](const StepMeta& m, bool live, u32x4 (&a)[RM]) {
#pragma unroll
        for (int r = 0; r < RM; ++r) a[r] = load_a_row(m, live, r);
    };

    Acc acc[RM][NT];
#pragma unroll
    for (int r = 0; r < RM; ++r)
#pragma unroll
        for (int x = 0; x < NT; ++x) acc[r][x] = Acc{0, 0, 0, 0};

    int32_t out_rows[RM][4];
    if constexpr (KG == 1) {
        if (ks == 1) {
#pragma unroll
            for (int r = 0; r < RM; ++r)
#pragma unroll
                for (int y = 0; y < 4; ++y)
                    out_rows[r][y] = tab.perm[(static_cast<int64_t>(super) * 16 + RM * wave + r) * 16 + 4 * g + y];
        }
    }

    if (nq > 0) {
        u32x4 a[RD][RM];
        StepMeta mt[RD];
#pragma unroll
        for (int h = 0; h < RD; ++h) mt[h] = fetch_meta(h);
        // prologue: what steps -2 and -1 of the loop would have issued, in the loop's order
#pragma unroll
        for (int h = 0; h < RD - 1; ++h) {
            load_panel(mt[h], is_live(h), h);
            load_a(mt[h], is_live(h), a[h]);
            mt[h] = fetch_meta(h + RD);
            __builtin_amdgcn_sched_barrier(0);
        }
        // steps of a group (the same count for both: they share the barriers; with an odd number of steps the
        // second group's last one multiplies zeros): whole passes of the three-step loop body, and one or two
        // steps behind the loop, so that no pass ends in steps that are not there
        const int gsteps = (nq + KG - 1) / KG;
        const int iters = gsteps / RD, rem = gsteps % RD;
        // step s of the group, s = u (mod RD): u picks the panel buffer and the register set
        auto step = [&](auto u_, int s) {
            constexpr int u = decltype(u_)::value;
            // Loads complete in order: all but the youngest six (those of step s+1) are the
            // panel and the block values of step s, and everything older.
            asm volatile("s_waitcnt vmcnt(6)");
            __builtin_amdgcn_s_barrier();
            // Every wave is past step s-1: its panel buffer and this wave's registers of that step
            // take the loads of step s+2 -- not here, though.  After the barrier all waves of the
            // compute unit are at the same point, and forty-eight loads asked for at once keep every
            // wave waiting at its load instructions while the matrix units idle (measured: the time of
            // the loads and the time of the matrix instructions added up).  The six loads go out one by
            // one between the groups of matrix instructions below.
            // Right operands by transposing reads, two per group of sixteen columns (k 0..3 and 4..7 of
            // the lane group), asked for one group ahead.  (The wait counts LDS reads, which return in
            // order; scalar loads of the tables that are still out only make it wait longer.)
            const StepMeta next = mt[(u + 2) % RD];
            const bool next_live = is_live(s + 2);
            mt[(u + 2) % RD] = fetch_meta(s + 2 + RD);
            __builtin_amdgcn_sched_barrier(0);
            u32x2_t lo[2], hi[2];
            auto read_pair = [&](int x, u32x2_t& l, u32x2_t& h) {
                if constexpr (ES == 2) {
                    l = lds_read_tr<8192 * u>(tr_addr[x]);
                    h = lds_read_tr<8192 * u + kSecondRead>(tr_addr[x]);
                } else {
                    l = lds_read_tr8<8192 * u>(tr_addr[x]);
                    h = lds_read_tr8<8192 * u + kSecondRead>(tr_addr[x]);
                }
            };
            read_pair(0, lo[0], hi[0]);
#pragma unroll
            for (int x = 0; x < NT; ++x) {
                if (x + 1 < NT) {
                    read_pair((x + 1) & 7, lo[(x + 1) & 1], hi[(x + 1) & 1]);
                    lds_pair_done<2>(lo[x & 1], hi[x & 1]);
                } else {
                    lds_pair_done<0>(lo[x & 1], hi[x & 1]);
                }
                // 16-bit: the two reads are k 0..3 and 4..7 of the lane group; 8-bit: the two sub-steps, which
                // the int8 instruction with k = 64 takes at once and the 8-bit floats one after the other
                // (the lane's block values of sub-step j are dwords 2j, 2j+1)
                const u32x4 b = u32x4{lo[x & 1][0], lo[x & 1][1], hi[x & 1][0], hi[x & 1][1]};
                // (the 8-bit forms with the result in the addend's registers, see mfma_types.h; the 8-bit floats
                // take the four block rows' first sub-step and then their second, so that no instruction waits
                // for the one before it)
                if constexpr (ES == 2) {
#pragma unroll
                    for (int r = 0; r < RM; ++r) acc[r][x] = mfma_pack<DT>(a[u][r], b, acc[r][x]);
                } else if constexpr (DT == kI8) {
#pragma unroll
                    for (int r = 0; r < RM; ++r) mfma_i8_k64_in_place(a[u][r], b, acc[r][x]);
                } else {
#pragma unroll
                    for (int r = 0; r < RM; ++r) mfma_pack8_in_place<DT>(a[u][r], b, false, acc[r][x]);
#pragma unroll
                    for (int r = 0; r < RM; ++r) mfma_pack8_in_place<DT>(a[u][r], b, true, acc[r][x]);
                }
                __builtin_amdgcn_sched_barrier(0);
                if (x < 2) {
                    load_panel_half(next, next_live, (u + 2) % RD, x);
                } else if (x < 2 + RM) {
                    a[(u + 2) % RD][x - 2] = load_a_row(next, next_live, x - 2);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            __builtin_amdgcn_sched_barrier(0);
        };
        static_assert(RD == 3, "the loop body names its three steps");
        for (int it = 0; it < iters; ++it) {
            step(std::integral_constant<int, 0>{}, RD * it);
            step(std::integral_constant<int, 1>{}, RD * it + 1);
            step(std::integral_constant<int, 2>{}, RD * it + 2);
        }
        if (rem >= 1) step(std::integral_constant<int, 0>{}, RD * iters);
        if (rem >= 2) step(std::integral_constant<int, 1>{}, RD * iters + 1);
        // nothing may still be on its way into LDS when the buffers get another use or the workgroup ends
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)");
        // the last matrix instructions written out by hand have finished before anything reads their result
        if constexpr (ES == 1) asm volatile("s_nop 15\n\ts_nop 15");
    }

    // Where the lane's rows of C' go.  One group per workgroup: already asked for before the loop (the registers are
    // there, and the stores then begin without one more trip to memory -- which a short tile on cold caches feels).
    // Two groups: asked for when the loop ends, ahead of the hand-over, which hides the trip; a lane then stores two
    // of its four block rows (group 0 the first two, group 1 the others).  (The empty statement makes the super
    // row's number a value the compiler knows only from here on, so that it cannot move these loads above the loop:
    // there the 8-bit instantiations once spilled registers inside it and ran 79 instead of 53 us.)
    if constexpr (KG == 2) {
        int super_now = super;
        asm volatile("" : "+s"(super_now));
        if (ks == 1) {
#pragma unroll
            for (int r = 0; r < RM; ++r)
                if ((r >> 1) == kg) {
#pragma unroll
                    for (int y = 0; y < 4; ++y)
                        out_rows[r][y] = tab.perm[(static_cast<int64_t>(super_now) * 16 + RM * wave + r) * 16 + 4 * g + y];
                }
        }
    }
    // acc[r][x][y] = C'[16 * (16 super + 4 wave + r) + 4g + y][n0 + 16x + i]
    auto store_block_row = [&](int r) {
        if (ks > 1) {
            // partial tile, row-major 256 x 128 words, at [(tile * ks + z)]
            const size_t tile_at = static_cast<size_t>(sidx) * n_slab + slab;
            Out* part = static_cast<Out*>(tab.scratch) + (tile_at * ks + blockIdx.z) * (256 * 128);
#pragma unroll
            for (int y = 0; y < 4; ++y) {
                Out* dst = part + (64 * wave + 16 * r + 4 * g + y) * 128 + i;
#pragma unroll
                for (int x = 0; x < NT; ++x) dst[16 * x] = acc[r][x][y];
            }
            return;
        }
        // sixteen lanes store 64 consecutive bytes of a row of C; the eight groups of columns of a lane
        // lie 64 bytes apart.  (Turning the tile over through LDS first, to store 16 bytes per lane and whole
        // rows of 512 bytes, was slower: 63.0 against 62.0 us hot, 71.5 against 68.7 us on flushed caches.)
#pragma unroll
        for (int y = 0; y < 4; ++y) {
            const int64_t out_row = out_rows[r][y];
            if (out_row < 0) continue;
            Out* dst = C + out_row * ldc + n0 + i;
#pragma unroll
            for (int x = 0; x < NT; ++x)
                if (n0 + 16 * x + i < N) dst[16 * x] = acc[r][x][y];
        }
    };
    if constexpr (KG == 2) {
        // The two groups hold partial sums of the same tile (even and odd steps).  Each hands two of its four block
        // rows per wave to the other through LDS -- group 1 its first two, group 0 its last two, 64 KiB each way --
        // and adds and stores the two it keeps: one barrier, and all eight waves store.
        __syncthreads();
        Out* handover = reinterpret_cast<Out*>(lds_words) + (kg == 0 ? 16384 : 0);      // where this group writes
        const Out* incoming = reinterpret_cast<const Out*>(lds_words) + (kg == 0 ? 0 : 16384);
#pragma unroll
        for (int rr = 0; rr < 2; ++rr)
#pragma unroll
            for (int x = 0; x < NT; ++x)
#pragma unroll
                for (int y = 0; y < 4; ++y) {
                    const Out v = kg == 0 ? acc[2 + rr][x][y] : acc[rr][x][y];
                    handover[(((wave * 2 + rr) * NT + x) * 4 + y) * 64 + lane] = v;
                }
        __syncthreads();
#pragma unroll
        for (int rr = 0; rr < 2; ++rr)
#pragma unroll
            for (int x = 0; x < NT; ++x)
#pragma unroll
                for (int y = 0; y < 4; ++y) {
                    const Out v = incoming[(((wave * 2 + rr) * NT + x) * 4 + y) * 64 + lane];
                    if (kg == 0) acc[rr][x][y] += v;
                    else acc[2 + rr][x][y] += v;
                }
        if (kg == 0) {
            store_block_row(0);
            store_block_row(1);
        } else {
            store_block_row(2);
            store_block_row(3);
        }
        return;
    }
#pragma unroll
    for (int r = 0; r < RM; ++r) store_block_row(r);
}

template <int DT, int KG>
static void launch_tile(const DeviceBcsr& d, const DenseTiles& t, int ks, const void* B, int64_t ldb,
                          void* C, int64_t ldc, int64_t N, hipStream_t s)
{
    TileOrder order;
    order.n_super = t.n;
    order.n_slab = static_cast<int>((N + 127) / 128);
    order.per_xcd = (order.n_super * order.n_slab + 7) / 8;
    dim3 grid(static_cast<unsigned>(8 * order.per_xcd), 1, static_cast<unsigned>(ks));
    const TileTables tab{t.step_cols, t.step_rows, t.step_base, d.perm, t.scratch};
    const uint32_t ldb_bytes = static_cast<uint32_t>(ldb * Elem<DT>::ES);
    auto* out = static_cast<typename Elem<DT>::Out*>(C);
    if (t.all_full)
        hipLaunchKernelGGL((spmm_tile_kernel<DT, KG, true>), grid, dim3(256 * KG), 0, s, order.n_super, order.n_slab, order.per_xcd,
                           static_cast<int>(N), t.super_rows, reinterpret_cast<const void*>(static_cast<uintptr_t>(t.full_steps)), B,
                           t.vals, ldb_bytes, static_cast<uint32_t>(d.K), tab, out, ldc);
    else
        hipLaunchKernelGGL((spmm_tile_kernel<DT, KG, false>), grid, dim3(256 * KG), 0, s, order.n_super, order.n_slab, order.per_xcd,
                           static_cast<int>(N), t.super_rows, static_cast<const void*>(t.step_ptr), B,
                           t.vals, ldb_bytes, static_cast<uint32_t>(d.K), tab, out, ldc);
}

template <typename T>
__global__ void dense_fill_kernel(DeviceBcsr d, DenseTiles t, const int64_t* __restrict__ csr_row_ptr,
                                  const int32_t* __restrict__ csr_col_idx, const uint16_t* __restrict__ csr_vals,
                                  T* __restrict__ vals_out)
{
    const int sidx = blockIdx.x;                       // which dense super row
    const int rr = threadIdx.x;                        // row inside the super row, 0..255
    const int64_t i = static_cast<int64_t>(t.super_rows[sidx]) * 256 + rr;
    if (i >= d.M) return;
    const int64_t r = d.perm[i];
    const int j = rr >> 4, ii = rr & 15;
    const int q0 = t.step_ptr[sidx], q1 = t.step_ptr[sidx + 1];
    const int cps = t.cols_per_step, ksub = cps / 2;
    const int32_t* cols = t.step_cols + static_cast<size_t>(cps) * static_cast<size_t>(q0);   // ascending; a missing last column is INT_MAX
    const int ncols = cps * (q1 - q0);
    int hint = 0;
    for (int64_t p = csr_row_ptr[r]; p < csr_row_ptr[r + 1]; ++p) {
        const int c = csr_col_idx[p];
        const int bc = c >> 4;
        int lo = hint, hi = ncols;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (cols[mid] < bc) lo = mid + 1; else hi = mid;
        }
        hint = lo;
        const size_t q = static_cast<size_t>(q0 + lo / cps);
        const uint32_t rows = t.step_rows[q];
        const size_t slot = static_cast<size_t>(t.step_base[q]) + __popc(rows & ((1u << j) - 1u));
        const int pc = (lo % cps) * 16 + (c & 15);                 // column inside the step
        const int sub = pc >> 5, g = (pc & 31) >> 3;               // sub-step, lane group
        vals_out[slot * (1024 / sizeof(T)) + static_cast<size_t>(((16 * g + ii) * ksub + sub) * 8 + (pc & 7))] = static_cast<T>(csr_vals[p]);
    }
}

int launch_dense_fill(const DeviceBcsr& d, const DenseTiles& t, const int64_t* csr_row_ptr,
                      const int32_t* csr_col_idx, const uint16_t* csr_vals, void* vals_out, int elem_bytes, void* stream)
{
    if (t.n == 0) return 0;
    if (elem_bytes == 1)
        hipLaunchKernelGGL(dense_fill_kernel<uint8_t>, dim3(static_cast<unsigned>(t.n)), dim3(256), 0,
                           static_cast<hipStream_t>(stream), d, t, csr_row_ptr, csr_col_idx, csr_vals, static_cast<uint8_t*>(vals_out));
    else
        hipLaunchKernelGGL(dense_fill_kernel<uint16_t>, dim3(static_cast<unsigned>(t.n)), dim3(256), 0,
                           static_cast<hipStream_t>(stream), d, t, csr_row_ptr, csr_col_idx, csr_vals, static_cast<uint16_t*>(vals_out));
    return static_cast<int>(hipGetLastError());
}

// Adds the ks partial tiles of every (super row, 128-column slab) in the order 0 .. ks-1 and
// writes the rows to C.  Eight workgroups per tile (32 rows each); a thread sums four groups of
// four columns and has all its loads in flight at once.
// V is the vector of four elements of C: f32x4, or i32x4 for the integer type.
template <typename V, typename Out>
__global__ __launch_bounds__(256)
void dense_reduce_kernel(DeviceBcsr d, DenseTiles t, int ks, Out* __restrict__ C, int64_t ldc, int N, int vec_store)
{
    const int super = t.super_rows[blockIdx.x];
    const int n0 = blockIdx.y * 128;
    const size_t tile = static_cast<size_t>(blockIdx.x) * gridDim.y + blockIdx.y;
    const Out* part = static_cast<const Out*>(t.scratch) + tile * ks * (256 * 128);
    V v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int e = static_cast<int>(blockIdx.z) * 1024 + j * 256 + static_cast<int>(threadIdx.x);
        v[j] = *reinterpret_cast<const V*>(part + e * 4);
    }
    for (int z = 1; z < ks; ++z)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int e = static_cast<int>(blockIdx.z) * 1024 + j * 256 + static_cast<int>(threadIdx.x);
            v[j] += *reinterpret_cast<const V*>(part + static_cast<size_t>(z) * (256 * 128) + e * 4);
        }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int e = static_cast<int>(blockIdx.z) * 1024 + j * 256 + static_cast<int>(threadIdx.x);
        const int row = e >> 5, c = (e & 31) * 4;
        const int64_t out_row = d.perm[static_cast<int64_t>(super) * 256 + row];
        if (out_row < 0 || n0 + c >= N) continue;             // N is a multiple of 8 on this path
        Out* dst = C + out_row * ldc + n0 + c;
        if (vec_store) {
            *reinterpret_cast<V*>(dst) = v[j];
        } else {
            dst[0] = v[j][0]; dst[1] = v[j][1]; dst[2] = v[j][2]; dst[3] = v[j][3];
        }
    }
}

// An area for partial tiles that belongs to the library, not to a workspace: a file-scope device
// array, one copy per GPU, present from the moment the code object is loaded until the process
// ends.  Host code never passes the array itself to a kernel -- its name is only the handle by
// which hipGetSymbolAddress finds the copy of the current device; the address is looked up once
// per device and kept.
constexpr size_t kStaticScratchBytes = size_t{16} << 20;        // 128 partial tiles of 256 x 128 words
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[kStaticScratchBytes];

int static_tile_scratch(void** area, size_t* bytes)
{
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void* addr[kMaxDevices] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return static_cast<int>(e);
    if (dev < 0 || dev >= kMaxDevices) return static_cast<int>(hipErrorInvalidDevice);
    std::lock_guard<std::mutex> lock(mu);
    if (addr[dev] == nullptr) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return static_cast<int>(e);
        if (p == nullptr) return static_cast<int>(hipErrorInvalidSymbol);
        addr[dev] = p;
    }
    *area = addr[dev];
    *bytes = kStaticScratchBytes;
    return 0;
}

// How many workgroups share the steps of a 128-column tile: as many as fit the 256 compute
// units in one round, as long as each keeps at least eight steps and the partial tiles fit the
// scratch area.
int dense_split(const DenseTiles& t, int64_t N)
{
    const int64_t tiles = static_cast<int64_t>(t.n) * ((N + 127) / 128);
    if (tiles <= 0 || tiles > 128 || t.scratch == nullptr) return 1;
    int64_t ks = std::min<int64_t>(8, 256 / tiles);
    ks = std::min<int64_t>(ks, static_cast<int64_t>(t.mean_steps / 8.0));
    ks = std::min<int64_t>(ks, static_cast<int64_t>(t.scratch_bytes / (static_cast<size_t>(tiles) * 256 * 128 * 4)));
    return ks < 2 ? 1 : static_cast<int>(ks);
}

template <int DT>
static int launch_dense_dtype(const DeviceBcsr& d, const DenseTiles& t, const void* B, int64_t ldb, void* C, int64_t ldc,
                              int64_t N, hipStream_t s, const char** variant)
{
    using Out = typename Elem<DT>::Out;
    using Acc = typename Elem<DT>::Acc;
    const int vec_store = (ldc % 4 == 0 && reinterpret_cast<uintptr_t>(C) % 16 == 0 && N % 4 == 0) ? 1 : 0;
    // long super rows: two wave groups per workgroup; short ones: one group, two workgroups per CU
    const bool deep = t.mean_steps >= 32.0;
    const int ks = dense_split(t, N);
    static thread_local char name[40];
    const char* type = DT == kF16 ? "f16" : DT == kBF16 ? "bf16" : DT == kE4M3 ? "e4m3" : DT == kE5M2 ? "e5m2" : "i8";
    if (ks > 1) snprintf(name, sizeof(name), "spmm_dense_%s_g%dk%d", type, deep ? 2 : 1, ks);
    else snprintf(name, sizeof(name), "spmm_dense_%s_g%d", type, deep ? 2 : 1);
    *variant = name;
    if (deep) launch_tile<DT, 2>(d, t, ks, B, ldb, C, ldc, N, s);
    else launch_tile<DT, 1>(d, t, ks, B, ldb, C, ldc, N, s);
    if (ks > 1)
        hipLaunchKernelGGL((dense_reduce_kernel<Acc, Out>), dim3(static_cast<unsigned>(t.n), static_cast<unsigned>((N + 127) / 128), 8),
                           dim3(256), 0, s, d, t, ks, static_cast<Out*>(C), ldc, static_cast<int>(N), vec_store);
    return static_cast<int>(hipGetLastError());
}

int launch_spmm_dense(const DeviceBcsr& d, const DenseTiles& t, int dtype, const void* B, int64_t ldb,
                      void* C, int64_t ldc, int64_t N, void* stream, const char** variant)
{
    if (t.n == 0) return 0;
    hipStream_t s = static_cast<hipStream_t>(stream);
    switch (dtype) {
    case kF16: return launch_dense_dtype<kF16>(d, t, B, ldb, C, ldc, N, s, variant);
    case kBF16: return launch_dense_dtype<kBF16>(d, t, B, ldb, C, ldc, N, s, variant);
    case kE4M3: return launch_dense_dtype<kE4M3>(d, t, B, ldb, C, ldc, N, s, variant);
    case kE5M2: return launch_dense_dtype<kE5M2>(d, t, B, ldb, C, ldc, N, s, variant);
    case kI8: return launch_dense_dtype<kI8>(d, t, B, ldb, C, ldc, N, s, variant);
    default: return static_cast<int>(hipErrorInvalidValue);
    }
}

}  // namespace smat
