// Per-row SpMM kernel templates for gfx950 (CDNA4, wave64), shared by the translation units
// that instantiate them for the 16-bit and the 8-bit operand types: the blocked SpMM of the
// paper's Implementation section (Alg. 1: per output tile, loop over the stored blocks of the
// block row and multiply-accumulate on the matrix units), written for the MFMA 16x16x32 forms
// (fp16, bf16, the two 8-bit floating-point formats with fp32 accumulation; int8 with int32).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdio>
#include <type_traits>

#include "kernels.h"
#include "mfma_types.h"
#include "pack_layout.h"

namespace smat {

// Work split: one workgroup per (block row, group of SW column slabs of 16*NT columns).  The
// group has KW*SW wavefronts: wave (ks, sl) takes packs ks, ks+KW, ... of the block row
// for slab sl, so the group streams the row's block values front to back once from HBM; the
// KW partial tiles of a slab are summed through LDS in a fixed order and scattered to the
// rows perm[16*br + 0..15] of C.
//
// One MFMA 16x16x32 multiplies a pack: the consecutive stored blocks of the block row that
// fit its 32 k slots with their occupied columns (pack_layout.h).  The left operand of lane l
// is the lane's L elements of the pack's values.  The right operand wants, per
// lane, eight k-consecutive values of one column of B, while B is row-major (n-consecutive).
// Instead of transposing through LDS, lane (g, i) loads from each B row of its k slots the NT
// consecutive columns n0 + NT*i .. n0 + NT*i + NT-1, and MFMA number t is defined to produce
// the column set { n0 + NT*i + t : i = 0..15 }.  The elements a lane feeds to MFMA t are then
// element t of its row loads (16-bit types: one byte-permute per two rows; 8-bit types: three
// per four rows), and after the NT MFMAs the lane holds, for each of its four output rows
// 4g..4g+3, NT consecutive columns of C.  The 8-bit types use the same 32-slot packs: their
// 16x16x32 instructions take eight bytes per lane where the 16-bit ones take eight halves, so
// everything below is the same walk with elements of half the size.
//
// Only occupied columns of a pack need a B row.  The layout puts them into the first
// slots of every lane group, so a block row whose packs hold at most 4*L occupied columns
// runs a loop that issues exactly L row loads per lane and pack (L = 2, 4 or 8, the row's
// "class", stored with the work order) and builds only the operand dwords they feed.  The slot table
// gives the B row of every slot; empty slots name row K, one past the end of B, for which
// the range-checked buffer load returns zeros without a memory access.  The number of loads
// per step is fixed inside a loop on purpose: the in-order load counter then lets a multiply
// wait for exactly the loads it needs while younger ones stay in flight.
//
// Entry rows (row class 3, pack_layout.h) run the L = 8 loop on packs of 32 stored entries:
// the slot table names one B row per entry and carries the entries' row numbers, the pack's
// values are the 32 entry values, and the left operand is built in registers -- lane (g, i)
// keeps the value of entry (g, kk) where that entry's row number is i.
//
// All loads of the loop are buffer loads whose wave-uniform part of the address travels in
// a scalar register, so a step spends vector ALU work only on what is per lane: one
// multiply-add per B row address and one byte-permute per operand dword.

constexpr uint32_t kOutOfRange = 0x80000000u;   // B must be smaller than 2 GiB on this path
constexpr int kRsrcFlags = 0x00020000;          // raw buffer, 32-bit data format

template <int BYTES> struct BLoad;
template <> struct BLoad<1> {
    static __device__ __forceinline__ void ld(uint32_t* r, __amdgpu_buffer_rsrc_t s, uint32_t off, uint32_t soff)
    { r[0] = static_cast<uint8_t>(__builtin_amdgcn_raw_buffer_load_b8(s, off, soff, 0)); }
};
template <> struct BLoad<2> {
    static __device__ __forceinline__ void ld(uint32_t* r, __amdgpu_buffer_rsrc_t s, uint32_t off, uint32_t soff)
    { r[0] = static_cast<uint16_t>(__builtin_amdgcn_raw_buffer_load_b16(s, off, soff, 0)); }
};
template <> struct BLoad<4> {
    static __device__ __forceinline__ void ld(uint32_t* r, __amdgpu_buffer_rsrc_t s, uint32_t off, uint32_t soff)
    { r[0] = static_cast<uint32_t>(__builtin_amdgcn_raw_buffer_load_b32(s, off, soff, 0)); }
};
template <> struct BLoad<8> {
    static __device__ __forceinline__ void ld(uint32_t* r, __amdgpu_buffer_rsrc_t s, uint32_t off, uint32_t soff)
    { i32x2 v = __builtin_amdgcn_raw_buffer_load_b64(s, off, soff, 0); r[0] = v[0]; r[1] = v[1]; }
};
template <> struct BLoad<16> {
    static __device__ __forceinline__ void ld(uint32_t* r, __amdgpu_buffer_rsrc_t s, uint32_t off, uint32_t soff)
    { i32x4 v = __builtin_amdgcn_raw_buffer_load_b128(s, off, soff, 0); r[0] = v[0]; r[1] = v[1]; r[2] = v[2]; r[3] = v[3]; }
};

// Same loads with the non-temporal hint: the block values and slot tables stream through
// once and should not push the rows of B out of the L2.
template <int BYTES> struct SLoad;
template <> struct SLoad<2> {
    static __device__ __forceinline__ void ld(uint32_t* r, __amdgpu_buffer_rsrc_t s, uint32_t off, uint32_t soff)
    { r[0] = static_cast<uint16_t>(__builtin_amdgcn_raw_buffer_load_b16(s, off, soff, 2)); }
};
template <> struct SLoad<4> {
    static __device__ __forceinline__ void ld(uint32_t* r, __amdgpu_buffer_rsrc_t s, uint32_t off, uint32_t soff)
    { r[0] = static_cast<uint32_t>(__builtin_amdgcn_raw_buffer_load_b32(s, off, soff, 2)); }
};
template <> struct SLoad<8> {
    static __device__ __forceinline__ void ld(uint32_t* r, __amdgpu_buffer_rsrc_t s, uint32_t off, uint32_t soff)
    { i32x2 v = __builtin_amdgcn_raw_buffer_load_b64(s, off, soff, 2); r[0] = v[0]; r[1] = v[1]; }
};
template <> struct SLoad<16> {
    static __device__ __forceinline__ void ld(uint32_t* r, __amdgpu_buffer_rsrc_t s, uint32_t off, uint32_t soff)
    { i32x4 v = __builtin_amdgcn_raw_buffer_load_b128(s, off, soff, 2); r[0] = v[0]; r[1] = v[1]; r[2] = v[2]; r[3] = v[3]; }
};

// 16-byte store with the non-temporal hint.  The pointer passes through an empty asm so that
// the compiler cannot merge this store with the plain one on the other side of a branch (it
// would drop the hint when it does).
template <typename T, typename V>
__device__ __forceinline__ void store_streaming(T* dst, V v)
{
    asm volatile("" : "+v"(dst));
    typedef __attribute__((address_space(1))) V global_v;               // C is device memory: a global, not a flat store
    __builtin_nontemporal_store(v, (global_v*)dst);
}

// Everything a wave needs to walk its share of a block row.
struct RowWalk {
    const uint32_t* slots;      // slot table of the row's first pack
    const uint8_t* vals;        // values of the row's first pack
    int npacks;                 // packs in the row (0 if this wave's slab is beyond N)
    int ks;                     // first pack of this wave
    int g, lane;
    uint32_t lane_off[2];       // per column chunk: byte offset of the lane's first column inside a B row
    uint32_t ldb_bytes;
    uint32_t no_row;            // the slot table's mark for an empty slot: K
    bool stream;                // block values and slot tables are read with the non-temporal hint
};

// Per-class pieces shared by the two pipelines below.
template <int NT, int L, int NCH, int DT, bool ENTRY = false>
struct PackOps {
    using Acc = typename Elem<DT>::Acc;
    static constexpr int ES = Elem<DT>::ES;
    static constexpr int LB = NT * ES;                    // bytes per B row load
    static_assert(!ENTRY || L == 8, "an entry pack has eight slots per lane group");
    static constexpr int AB = L * ES;                     // bytes of block values per lane and pack
    static constexpr int EB = 8 * ES;                     // entry rows: bytes of a lane group's eight entry values
    static constexpr uint32_t PB = ENTRY ? 64u : 64u * AB; // bytes of block values per pack
    static constexpr int ND = LB >= 4 ? LB / 4 : 1;       // dwords per B row load
    static constexpr int NQ = (AB + 3) / 4;               // operand dwords that carry data
    __amdgpu_buffer_rsrc_t slots_rsrc, vals_rsrc, none_rsrc, b_rsrc;
    uint32_t slots_voff, vals_voff, lane_off[NCH], ldb_bytes, no_row, row_match;
    int last, lane_in_wave, group_base;     // group_base: byte address, for ds_bpermute, of the lane that holds the group's entry 0
    bool stream;

    __device__ __forceinline__ PackOps(const RowWalk& w, __amdgpu_buffer_rsrc_t b)
        : b_rsrc(b), slots_voff(static_cast<uint32_t>(w.g) * 4u * L),
          vals_voff(ENTRY ? static_cast<uint32_t>(w.g) * EB : static_cast<uint32_t>(w.lane) * AB),
          ldb_bytes(w.ldb_bytes), no_row(w.no_row), row_match(static_cast<uint32_t>(w.lane & 15) * 0x11111111u),
          last(w.npacks - 1), lane_in_wave(w.lane), group_base(4 * 8 * w.g), stream(w.stream)
    {
#pragma unroll
        for (int c = 0; c < NCH; ++c) lane_off[c] = w.lane_off[c];
        slots_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(w.slots), 0, w.npacks * 16 * L, kRsrcFlags);
        vals_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(w.vals), 0, w.npacks * static_cast<int>(PB), kRsrcFlags);
        none_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(w.vals), 0, 0, kRsrcFlags);
    }
    // Loads of a pack are unconditional: a pack index past the row's end is clamped to the
    // row's last pack (a cache hit).  All of this is scalar arithmetic.
    __device__ __forceinline__ uint32_t clamp(int p) const { return static_cast<uint32_t>(p < last ? p : last); }
    // B rows of the lane group's L slots
    __device__ __forceinline__ void load_slots(int p, uint32_t (&m)[L]) const
    {
        const uint32_t soff = clamp(p) * (16u * L);
        if constexpr (L == 2) {
            if (stream) SLoad<8>::ld(m, slots_rsrc, slots_voff, soff);
            else BLoad<8>::ld(m, slots_rsrc, slots_voff, soff);
        } else {
#pragma unroll
            for (int x = 0; x < L; x += 4) {
                if (stream) SLoad<16>::ld(m + x, slots_rsrc, slots_voff + 4u * x, soff);
                else BLoad<16>::ld(m + x, slots_rsrc, slots_voff + 4u * x, soff);
            }
        }
    }
    // The same table for L = 8 with one request of four bytes per lane instead of two of sixteen: lane l fetches
    // entry l mod 32 of the pack's 32 (the memory pipeline spends its time per lane and byte asked for, also where
    // sixteen lanes ask for the same bytes: 4 clocks against 32 of the 176 a pack costs it in all), and expand_slots
    // hands every lane the eight entries of its lane group through the LDS crossbar (no LDS memory involved).
    __device__ __forceinline__ uint32_t load_slots_compact(int p) const
    {
        static_assert(L == 8, "the compact table load is for packs of 32 slots");
        const uint32_t soff = clamp(p) * 128u;
        const uint32_t voff = static_cast<uint32_t>(lane_in_wave & 31) * 4u;
        uint32_t r[1];
        if (stream) SLoad<4>::ld(r, slots_rsrc, voff, soff);
        else BLoad<4>::ld(r, slots_rsrc, voff, soff);
        return r[0];
    }
    __device__ __forceinline__ void expand_slots(uint32_t raw, uint32_t (&m)[L]) const
    {
#pragma unroll
        for (int kk = 0; kk < L; ++kk)
            m[kk] = static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute(group_base + 4 * kk, static_cast<int>(raw)));
    }
    // block values: the lane's L elements (the other operand dwords multiply nothing and stay
    // zero); `live` false (a step past the wave's last pack) reads zeros instead
    __device__ __forceinline__ u32x4 load_a(int p, bool live) const
    {
        // an entry pack is its 32 entry values (one 64-byte unit): the lane group's eight, to be
        // expanded by multiply()
        constexpr int W = ENTRY ? EB : AB;
        uint32_t r[4] = {0u, 0u, 0u, 0u};
        if (!live) BLoad<W>::ld(r, none_rsrc, vals_voff, 0u);
        else if (stream) SLoad<W>::ld(r, vals_rsrc, vals_voff, clamp(p) * PB);
        else BLoad<W>::ld(r, vals_rsrc, vals_voff, clamp(p) * PB);
        return u32x4{r[0], r[1], r[2], r[3]};
    }
    // Occupied columns fill the slots group by group, so position kk is empty in every group
    // as soon as it is empty in group 0 (lane 0).  In the sparse classes a pack therefore has
    // a wave-uniform "level": the number of leading positions that hold anything, rounded up
    // to 1, 2 or 4; only that many B rows are requested, and the multiply permutes only the
    // operand dwords they feed.  Returns the level; for an entry pack, the row numbers of the
    // lane group's entries instead (4 bits each), which multiply() needs.
    __device__ __forceinline__ int issue_b(const uint32_t (&m)[L], uint32_t (&R)[L][NCH][ND]) const
    {
        int level = L;
        if constexpr (ENTRY) {
            // the eight row numbers of the group's entries, from the top bytes of its first four
            // slots (the address arithmetic below only takes the low 24 bits of a slot)
            const uint32_t lo = __builtin_amdgcn_perm(m[1], m[0], 0x0C0C0703u);
            const uint32_t hi = __builtin_amdgcn_perm(m[3], m[2], 0x0C0C0703u);
            level = static_cast<int>(__builtin_amdgcn_perm(hi, lo, 0x05040100u));
        } else if constexpr (L == 2) {
            level = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(m[1])) == no_row ? 1 : 2;
        } else if constexpr (L == 4) {
            level = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(m[1])) == no_row ? 1
                  : static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(m[2])) == no_row ? 2 : 4;
        }
#pragma unroll
        for (int kk = 0; kk < L; ++kk)
            if (ENTRY || kk < level) {
                const uint32_t row_off = __umul24(m[kk], ldb_bytes);
#pragma unroll
                for (int c = 0; c < NCH; ++c) BLoad<LB>::ld(R[kk][c], b_rsrc, row_off + lane_off[c], 0u);
            }
        return level;
    }
    // Rows above the pack's level were not requested: their registers hold stale data and are
    // replaced by zeros (a select on a wave-uniform condition) before the permutes.
    __device__ __forceinline__ void multiply(const u32x4& a_in, const uint32_t (&R)[L][NCH][ND], int level, Acc (&acc)[NCH * NT]) const
    {
        u32x4 a = a_in;
        if constexpr (ENTRY) {
            // left operand of lane (g, i): entry value kk where the entry's row is i, else zero.
            // `miss` has a zero nibble kk exactly there.
            const uint32_t miss = static_cast<uint32_t>(level) ^ row_match;
            constexpr int PER = 4 / ES;                    // entries per operand dword
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                uint32_t keep = 0u;
                if (q < 8 / PER) {
#pragma unroll
                    for (int e = 0; e < PER; ++e)
                        if (((miss >> (4 * (PER * q + e))) & 15u) == 0u) keep |= (ES == 2 ? 0xFFFFu : 0xFFu) << (8 * ES * e);
                }
                a[q] = a_in[q] & keep;
            }
        }
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            uint32_t S[L][ND];
#pragma unroll
            for (int kk = 0; kk < L; ++kk)
#pragma unroll
                for (int x = 0; x < ND; ++x)
                    S[kk][x] = (L == 8 || kk == 0 || kk < level) ? R[kk][c][x] : 0u;
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                u32x4 b = u32x4{0u, 0u, 0u, 0u};
                if constexpr (ES == 2) {
                    // operand dword q = halves t of rows 2q and 2q+1
                    const uint32_t pick = (t & 1) ? 0x07060302u : 0x05040100u;
#pragma unroll
                    for (int q = 0; q < NQ; ++q)
                        b[q] = __builtin_amdgcn_perm(S[2 * q + 1][t >> 1], S[2 * q][t >> 1], pick);
                } else {
                    // operand dword q = bytes t of rows 4q .. 4q+3: two rows at a time into the low
                    // half of a dword (selector 0x0c gives a zero byte), then the two halves joined
                    const uint32_t pair = 0x0C0C0400u + static_cast<uint32_t>(t & 3) * 0x0101u;
                    if constexpr (L == 2) {
                        b[0] = __builtin_amdgcn_perm(S[1][t >> 2], S[0][t >> 2], pair);
                    } else {
#pragma unroll
                        for (int q = 0; q < NQ; ++q) {
                            const uint32_t lo = __builtin_amdgcn_perm(S[4 * q + 1][t >> 2], S[4 * q][t >> 2], pair);
                            const uint32_t hi = __builtin_amdgcn_perm(S[4 * q + 3][t >> 2], S[4 * q + 2][t >> 2], pair);
                            b[q] = __builtin_amdgcn_perm(hi, lo, 0x05040100u);
                        }
                    }
                }
                acc[c * NT + t] = mfma_pack<DT>(a, b, acc[c * NT + t]);
            }
        }
    }
};

// Pipeline for the dense class (L = 8), two register sets.  Per pack h: its slot table is
// requested two steps ahead, its B rows (whose addresses need it) one step ahead, its block
// values right after the multiply of pack h-2 has released their registers.  The loop body
// handles two packs and has no exit in the middle (an odd tail multiplies zeros).  The
// scheduling barriers keep every load ahead of the multiply that precedes its use, and the
// prologue issues its loads in the order the loop body leaves them in flight.
template <int NT, int KW, int L, int NCH, int DT, bool ENTRY = false>
__device__ __forceinline__ void walk_row(const RowWalk& w, __amdgpu_buffer_rsrc_t rsrc, typename Elem<DT>::Acc (&acc)[NCH * NT])
{
    using Ops = PackOps<NT, L, NCH, DT, ENTRY>;
    if (w.ks >= w.npacks) return;
    const Ops ops(w, rsrc);
    const int count = (w.npacks - w.ks + KW - 1) / KW;     // packs of this wave
    const int iters = (count + 1) >> 1;
    uint32_t R0[L][NCH][Ops::ND], R1[L][NCH][Ops::ND];
    uint32_t m[L];
    int p = w.ks;
    uint32_t raw0 = ops.load_slots_compact(p);
    __builtin_amdgcn_sched_barrier(0);
    uint32_t raw1 = ops.load_slots_compact(p + KW);
    u32x4 a0 = ops.load_a(p, true);
    ops.expand_slots(raw0, m);
    int l0 = ops.issue_b(m, R0), l1;                       // level of the pack (entry rows: its row numbers)
    __builtin_amdgcn_sched_barrier(0);
    u32x4 a1 = ops.load_a(p + KW, count > 1);
    for (int it = 0; it < iters; ++it) {
        const int h = 2 * it;                              // pack of this wave multiplied first
        raw0 = ops.load_slots_compact(p + 2 * KW);
        ops.expand_slots(raw1, m);
        l1 = ops.issue_b(m, R1);
        __builtin_amdgcn_sched_barrier(0);
        ops.multiply(a0, R0, l0, acc);
        __builtin_amdgcn_sched_barrier(0);
        a0 = ops.load_a(p + 2 * KW, h + 2 < count);
        raw1 = ops.load_slots_compact(p + 3 * KW);
        ops.expand_slots(raw0, m);
        l0 = ops.issue_b(m, R0);
        __builtin_amdgcn_sched_barrier(0);
        ops.multiply(a1, R1, l1, acc);
        __builtin_amdgcn_sched_barrier(0);
        a1 = ops.load_a(p + 3 * KW, h + 3 < count);
        p += 2 * KW;
    }
}

// Pipeline for the sparse classes (L = 2, 4), whose row buffers are small: four-slot rings.
// While pack h is multiplied, the loads in flight are the B rows and block values of packs
// h+1..h+3 and the slot tables of packs h+4..h+6 (pack x has its slot table requested at step
// x-6, its B rows and values at step x-3) -- about three packs per wave in flight.  The loop
// body is four steps without an exit; steps past the wave's last pack multiply zeros.
template <int NT, int KW, int L, int NCH, int DT>
__device__ __forceinline__ void walk_row_deep(const RowWalk& w, __amdgpu_buffer_rsrc_t rsrc, typename Elem<DT>::Acc (&acc)[NCH * NT])
{
    using Ops = PackOps<NT, L, NCH, DT>;
    static_assert(L <= 4, "the deep ring is meant for the sparse classes");
    if (w.ks >= w.npacks) return;
    const Ops ops(w, rsrc);
    const int count = (w.npacks - w.ks + KW - 1) / KW;     // packs of this wave
    const int iters = (count + 3) >> 2;
    uint32_t R[4][L][NCH][Ops::ND];
    u32x4 a[4];
    uint32_t m[4][L];
    int level[4];
    const int p0 = w.ks;
    auto pack_of = [&](int h) { return p0 + h * KW; };     // h-th pack of this wave
    // prologue = steps -6 .. -1 of the loop without their multiplies
#pragma unroll
    for (int h = 0; h < 3; ++h) {
        ops.load_slots(pack_of(h), m[h]);
        __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int h = 0; h < 3; ++h) {
        uint32_t mh[L];
#pragma unroll
        for (int x = 0; x < L; ++x) mh[x] = m[h][x];
        ops.load_slots(pack_of(h + 3), m[(h + 3) & 3]);
        __builtin_amdgcn_sched_barrier(0);
        a[h] = ops.load_a(pack_of(h), h < count);
        level[h] = ops.issue_b(mh, R[h]);
        __builtin_amdgcn_sched_barrier(0);
    }
    int h0 = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int h = h0 + u;                          // pack of this wave multiplied in this step
            // the table of pack h+6 takes the ring slot of pack h+2, whose B rows went out a step
            // ago; it is requested first: a later step waits for it and should wait for nothing younger
            uint32_t mh[L];
#pragma unroll
            for (int x = 0; x < L; ++x) mh[x] = m[(u + 3) & 3][x];
            ops.load_slots(pack_of(h + 6), m[(u + 2) & 3]);
            __builtin_amdgcn_sched_barrier(0);
            a[(u + 3) & 3] = ops.load_a(pack_of(h + 3), h + 3 < count);
            level[(u + 3) & 3] = ops.issue_b(mh, R[(u + 3) & 3]);
            __builtin_amdgcn_sched_barrier(0);
            ops.multiply(a[u], R[u], level[u], acc);
            __builtin_amdgcn_sched_barrier(0);
        }
        h0 += 4;
    }
}

// ---------------------------------------------------------------------------
// Entry rows at N = 1, 2, 4, 8, 16 (16-bit types)
// ---------------------------------------------------------------------------
// With few columns the walk above asks the memory pipeline for next to nothing per request: a
// row load of lane (g, i) is one element, a pack costs eight such requests plus two for its
// slots and values.  Here every lane fetches the whole piece of ONE row of B with one load of W
// bytes instead -- the row of "its" entry, all N columns at N <= 8 (W = 2 N, two packs per
// round, PK = 2), eight of the sixteen at N = 16 (one pack per round, PK = 1) -- plus that
// entry's slot word and value, so a round of 64 (32) entries takes three requests per lane.
// Both operands of the multiply then go through the wave's own part of LDS:
//   - the pieces, from where lane (g, i) of the multiply reads the eight elements of its column,
//     one per entry of its lane group.  The piece of entry (g, kk) lies at 16-byte (PK = 1:
//     32-byte) position 8 c + ((kk + c) mod 8), c the number of the lane group among the
//     round's eight (four): one read instruction (a fixed kk) touches every LDS bank once;
//   - the left operand as the multiply wants it, 16 bytes per lane: the lane that holds entry
//     (g, kk) with row number i' stores its value at element kk of lane (g, i')'s sixteen bytes
//     (it learns i' from the slot word of entry (g, kk / 2), a neighbour lane), and puts the
//     zero back once the round is multiplied.
//
// PK = 2: columns 0..7 of the multiply's right operand belong to the first pack of the round
// (lanes i < 8) and columns 8..15 to the second (lanes i >= 8, column i - 8).  The first pack's
// left operand accumulates into one tile, the second pack's into another, both with the same
// right operand: the first tile is right in its columns 0..7 and the second in its columns
// 8..15, the rest of each is never used, and the two halves are added at the end of the row.
//
// What this buys is bounded by the gather itself: 4.2 M random 16-byte pieces out of a 4 MB
// array take 22 us on this chip whatever the load width or cache policy (each costs the L2 a
// whole 128-byte line); the walk above needs 36.7 us for that many entries at N = 8, this one 29.
template <int PK> constexpr int narrow_lds_bytes() { return 1024 + PK * 1024; }

template <int KW, int PK, int W, int DT>
__device__ __forceinline__ void walk_entries_narrow(const RowWalk& w, __amdgpu_buffer_rsrc_t b_rsrc,
                                                    typename Elem<DT>::Acc& acc)
{
    using Acc = typename Elem<DT>::Acc;
    static_assert(Elem<DT>::ES == 2, "16-bit operand types only");
    static_assert((PK == 2 && (W == 2 || W == 4 || W == 8 || W == 16)) || (PK == 1 && W == 16),
                  "two packs of pieces of W bytes per round, or one pack of 32-byte pieces");
    constexpr int RW = W >= 4 ? W / 4 : 1;         // registers of a piece
    constexpr int AREA = narrow_lds_bytes<PK>();
    __shared__ __attribute__((aligned(16))) uint8_t narrow_lds[KW * AREA];
    const int rounds = (w.npacks + PK - 1) / PK;
    if (w.ks >= rounds) return;
    const int count = (rounds - w.ks + KW - 1) / KW;       // rounds of this wave
    uint8_t* lds_b = narrow_lds + w.ks * AREA;              // pieces of B
    uint8_t* lds_a = lds_b + 1024;                          // left operands: PK x 64 lanes x 16 bytes
    const int lane = w.lane, g = lane >> 4, i = lane & 15;

    // what this lane fetches: entry l_e of pack l_sp of the round, columns from 8 l_half on
    const int l_sp = PK == 2 ? (lane >> 3) & 1 : 0;
    const int l_e = PK == 2 ? 8 * g + (lane & 7) : lane >> 1;
    const int l_half = PK == 2 ? 0 : lane & 1;
    const int l_g = l_e >> 3, l_kk = l_e & 7;
    const int l_c = PK == 2 ? 4 * l_sp + l_g : l_g;        // lane group of the entry among the round's
    const uint32_t wr_b = PK == 2 ? static_cast<uint32_t>(8 * l_c + ((l_kk + l_c) & 7)) * 16u
                                  : static_cast<uint32_t>(8 * l_c + ((l_kk + l_c) & 7)) * 32u + 16u * l_half;
    const uint32_t l_idx = static_cast<uint32_t>(l_sp * 32 + l_e);
    const bool owner = l_half == 0;                        // one lane per entry places the value
    // the lane that holds the slot word with this entry's row number, and where the number is in it
    const int nib_from = (PK == 2 ? ((lane & ~7) | (l_kk >> 1)) : 2 * ((l_e & ~7) | (l_kk >> 1))) * 4;
    const uint32_t nib_shift = 24u + 4u * (l_kk & 1);
    const uint32_t wr_a0 = static_cast<uint32_t>(l_sp * 4 + l_g) * 256u + 2u * l_kk;
    // what this lane reads for the multiply: column rd_col / 2 of the entries of lane group rd_c
    const int rd_c = PK == 2 ? 4 * (i >> 3) + g : g;
    const uint32_t rd_col = PK == 2 ? 2u * (i & 7) : 2u * i;
    uint32_t rd_b[8];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk)
        rd_b[kk] = static_cast<uint32_t>(8 * rd_c + ((kk + rd_c) & 7)) * (PK == 2 ? 16u : 32u) + rd_col;

    const __amdgpu_buffer_rsrc_t slots_rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(w.slots), 0, w.npacks * 128, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t vals_rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(w.vals), 0, w.npacks * 64, kRsrcFlags);

#pragma unroll
    for (int x = 0; x < PK; ++x) *reinterpret_cast<u32x4*>(lds_a + x * 1024 + lane * 16) = u32x4{0u, 0u, 0u, 0u};

    // slot word and value of the lane's entry in round r (zeros past the row's last pack)
    auto load_meta = [&](int r, uint32_t& m, uint32_t& v) {
        const uint32_t idx = static_cast<uint32_t>(PK * r) * 32u + l_idx;    // beyond the tables: range-checked to zero
        BLoad<4>::ld(&m, slots_rsrc, idx * 4u, 0u);
        BLoad<2>::ld(&v, vals_rsrc, idx * 2u, 0u);
    };
    // Requests the lane's piece of B (an entry past the row's last pack names row K: zeros, no
    // access) and returns where the entry's value goes in the left operands.
    auto load_piece = [&](int r, uint32_t m, uint32_t (&P)[RW]) -> uint32_t {
        const bool valid = PK * r + l_sp < w.npacks;
        BLoad<W>::ld(P, b_rsrc, __umul24(valid ? m : w.no_row, w.ldb_bytes) + 16u * l_half, 0u);
        const uint32_t word = static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute(nib_from, static_cast<int>(m)));
        return wr_a0 + ((word >> nib_shift) & 15u) * 16u;
    };
    auto stash = [&](const uint32_t (&P)[RW], uint32_t wr_a, uint32_t v) {
        if (owner) *reinterpret_cast<uint16_t*>(lds_a + wr_a) = static_cast<uint16_t>(v);
        if constexpr (W == 16) *reinterpret_cast<u32x4*>(lds_b + wr_b) = u32x4{P[0], P[1], P[2], P[3]};
        else if constexpr (W == 8) *reinterpret_cast<u32x2*>(lds_b + wr_b) = u32x2{P[0], P[1]};
        else if constexpr (W == 4) *reinterpret_cast<uint32_t*>(lds_b + wr_b) = P[0];
        else *reinterpret_cast<uint16_t*>(lds_b + wr_b) = static_cast<uint16_t>(P[0]);
    };
    Acc acc2 = Acc{0, 0, 0, 0};
    auto multiply = [&](uint32_t wr_a) {
        u32x4 b;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t lo = *reinterpret_cast<const uint16_t*>(lds_b + rd_b[2 * q]);
            const uint32_t hi = *reinterpret_cast<const uint16_t*>(lds_b + rd_b[2 * q + 1]);
            b[q] = lo | (hi << 16);
        }
        const u32x4 a0 = *reinterpret_cast<const u32x4*>(lds_a + lane * 16);
        acc = mfma_pack<DT>(a0, b, acc);
        if constexpr (PK == 2) {
            const u32x4 a1 = *reinterpret_cast<const u32x4*>(lds_a + 1024 + lane * 16);
            acc2 = mfma_pack<DT>(a1, b, acc2);
        }
        if (owner) *reinterpret_cast<uint16_t*>(lds_a + wr_a) = 0;     // the operands start every round as zeros
    };

    // Round x of this wave: its slot words and values are requested two steps ahead, the pieces
    // they name one step ahead; all of it goes to LDS right before the multiply.  Two steps per
    // loop body, no exit in the middle (a step past the last round multiplies zeros).
    uint32_t M0, V0, M1, V1, A0, A1;
    uint32_t P0[RW], P1[RW];
    int r = w.ks;
    load_meta(r, M0, V0);
    load_meta(r + KW, M1, V1);
    __builtin_amdgcn_sched_barrier(0);
    A0 = load_piece(r, M0, P0);
    const int iters = (count + 1) >> 1;
    for (int it = 0; it < iters; ++it) {
        const uint32_t v0 = V0;
        load_meta(r + 2 * KW, M0, V0);
        __builtin_amdgcn_sched_barrier(0);
        A1 = load_piece(r + KW, M1, P1);
        __builtin_amdgcn_sched_barrier(0);
        stash(P0, A0, v0);
        __builtin_amdgcn_wave_barrier();
        multiply(A0);
        __builtin_amdgcn_sched_barrier(0);
        const uint32_t v1 = V1;
        load_meta(r + 3 * KW, M1, V1);
        __builtin_amdgcn_sched_barrier(0);
        A0 = load_piece(r + 2 * KW, M0, P0);
        __builtin_amdgcn_sched_barrier(0);
        stash(P1, A1, v1);
        __builtin_amdgcn_wave_barrier();
        multiply(A1);
        __builtin_amdgcn_sched_barrier(0);
        r += 2 * KW;
    }
    if constexpr (PK == 2) {
        // columns 8..15 of the second tile are columns 0..7 of the row's result
        const int from = ((lane + 8) & 63) * 4;
#pragma unroll
        for (int y = 0; y < 4; ++y) {
            const float mine = acc2[y];            // a scalar copy: the cast below must see one element
            acc[y] += __int_as_float(__builtin_amdgcn_ds_bpermute(from, __float_as_int(mine)));
        }
    }
}

// NARROW: 0, or 100 * PK + W of walk_entries_narrow for the entry rows (then NT = SW = NCH = 1).
template <int NT, int KW, int SW, int NCH, int LMAX, int DT, int NARROW = 0>
__global__ __launch_bounds__(KW * SW * 64)
void spmm_kernel(const int32_t* __restrict__ work, const uint32_t* __restrict__ slots, const void* __restrict__ vals,
                 const int32_t* __restrict__ perm, const void* __restrict__ B, uint32_t b_bytes, uint32_t ldb_bytes,
                 uint32_t K, typename Elem<DT>::Out* __restrict__ C, int64_t ldc, int N, int vec_store, int stream_hint)
{
    // The arguments are plain words, the ones needed first in front: the compiler is asked
    // (build flag) to have the dispatcher place the leading ones in scalar registers, so that the
    // first load of the kernel does not have to wait for a load of its own arguments.
    using Acc = typename Elem<DT>::Acc;
    using Out = typename Elem<DT>::Out;
    constexpr int ES = Elem<DT>::ES;
    constexpr int NW = 16 * NT;                    // columns per chunk (one set of NT MFMAs)
    constexpr int WC = NCH * NW;                   // columns per wave
    constexpr int WAVES = KW * SW;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform, kept in an SGPR
    const int ks = wave % KW;                      // which share of the block row
    const int sl = wave / KW;                      // which column slab of the group
    const int i = lane & 15, g = lane >> 4;
    const i32x4 rec = reinterpret_cast<const i32x4*>(work)[blockIdx.x];     // one record of the launch table
    const int br = rec[0] & 0x0FFFFFFF;
    const int cls = rec[0] >> 28;                  // 0: L = 2, 1: L = 4, 2: L = 8, 3: entry row
    const int n0 = (blockIdx.y * SW + sl) * WC;

    RowWalk w;
    w.slots = slots + static_cast<size_t>(static_cast<uint32_t>(rec[2])) * 8;        // 32 bytes of slot table per unit
    w.vals = static_cast<const uint8_t*>(vals) + static_cast<size_t>(static_cast<uint32_t>(rec[3])) * 64;            // 64 bytes per unit
    w.npacks = n0 < N ? rec[1] : 0;
    w.ks = ks;
    w.g = g;
    w.lane = lane;
    int col0[NCH];                                 // first of this lane's NT columns, per chunk
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        col0[c] = n0 + c * NW + NT * i;
        // A lane whose columns lie beyond N carries the out-of-range bit in its offset (N is a
        // multiple of NT on this path, so a lane's columns are all in or all out) -- unless one of
        // the other three lanes of its quad is inside: the memory pipeline takes a quad of lanes
        // with consecutive addresses at once and a quad with a hole lane by lane (N = 1, 2, 3, 6
        // ran 1.6 x slower than N = 4, 8).  Such a lane reads what follows column N (the row's
        // padding or the next row; past the end of B the range check returns zeros) into columns
        // of the tile that are never stored.
        w.lane_off[c] = col0[c] - NT * (i & 3) < N ? static_cast<uint32_t>(col0[c]) * ES : kOutOfRange;
    }
    w.ldb_bytes = ldb_bytes;
    w.no_row = K;
    w.stream = (stream_hint & 1) != 0;
    const bool c_stream = (stream_hint & 2) != 0;  // C is stored with the non-temporal hint

    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(B), 0, static_cast<int>(b_bytes), kRsrcFlags);

    // Where this thread's output rows go is read now, not after the loop: the epilogue then
    // starts with the addresses in registers instead of with one more trip to memory.
    constexpr int Q = NT >= 4 ? WC / 4 : WC;       // epilogue items per tile row (quads, or single columns)
    constexpr int EP = KW == 1 ? 4 : (SW * 16 * Q + WAVES * 64 - 1) / (WAVES * 64);
    int out_rows[EP];
    if constexpr (KW == 1) {
#pragma unroll
        for (int r = 0; r < 4; ++r) out_rows[r] = perm[br * 16 + 4 * g + r];
    } else {
#pragma unroll
        for (int k = 0; k < EP; ++k) {
            const int e = static_cast<int>(threadIdx.x) + k * WAVES * 64;
            out_rows[k] = e < SW * 16 * Q ? perm[br * 16 + (e / Q) % 16] : -1;
        }
    }

    Acc acc[NCH * NT];
#pragma unroll
    for (int t = 0; t < NCH * NT; ++t) acc[t] = Acc{0, 0, 0, 0};

    if constexpr (LMAX >= 8) {
        if (cls == 2) walk_row<NT, KW, 8, NCH, DT>(w, rsrc, acc);
        if (cls == kEntryClass) {
            if constexpr (NARROW != 0) {
                static_assert(NT == 1 && SW == 1 && NCH == 1, "the narrow walk covers one slab of 16 columns");
                walk_entries_narrow<KW, NARROW / 100, NARROW % 100, DT>(w, rsrc, acc[0]);
            } else {
                walk_row<NT, KW, 8, NCH, DT, true>(w, rsrc, acc);
            }
        }
    }
    if constexpr (LMAX >= 4) {
        if (cls == 1) walk_row_deep<NT, KW, 4, NCH, DT>(w, rsrc, acc);
    }
    if (cls == 0) walk_row_deep<NT, KW, 2, NCH, DT>(w, rsrc, acc);

    // acc[c*NT + t][r] = C'[4g + r][n0 + c*NW + NT*i + t]
    if constexpr (KW == 1) {
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            if (col0[c] >= N) continue;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int64_t out_row = out_rows[r];
                if (out_row < 0) continue;
                Out* dst = C + out_row * ldc + col0[c];
                if constexpr (NT >= 4) {
                    if (vec_store) {
#pragma unroll
                        for (int t = 0; t < NT; t += 4) {
                            const Acc v = Acc{acc[c * NT + t][r], acc[c * NT + t + 1][r], acc[c * NT + t + 2][r], acc[c * NT + t + 3][r]};
                            if (c_stream) store_streaming(dst + t, v);
                            else *reinterpret_cast<Acc*>(dst + t) = v;
                        }
                        continue;
                    }
                }
#pragma unroll
                for (int t = 0; t < NT; ++t) dst[t] = acc[c * NT + t][r];
            }
        }
    } else {
        constexpr int LD = WC + 4;                 // padded row of the reduction buffer (32-bit words)
        __shared__ Out red[WAVES * 16 * LD];
        Out* mine = red + wave * 16 * LD;
#pragma unroll
        for (int c = 0; c < NCH; ++c)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                Out* dst = mine + (4 * g + r) * LD + c * NW + NT * i;
                if constexpr (NT >= 4) {
#pragma unroll
                    for (int t = 0; t < NT; t += 4)
                        *reinterpret_cast<Acc*>(dst + t) =
                            Acc{acc[c * NT + t][r], acc[c * NT + t + 1][r], acc[c * NT + t + 2][r], acc[c * NT + t + 3][r]};
                } else {
#pragma unroll
                    for (int t = 0; t < NT; ++t) dst[t] = acc[c * NT + t][r];
                }
            }
        __syncthreads();
        const int nbase = blockIdx.y * SW * WC;
        if constexpr (NT >= 4) {
            // each thread sums and stores four consecutive columns
#pragma unroll
            for (int k = 0; k < EP; ++k) {
                const int e = static_cast<int>(threadIdx.x) + k * WAVES * 64;
                if (e >= SW * 16 * Q) break;
                const int s = e / (16 * Q), row = (e / Q) % 16, c = (e % Q) * 4;
                const Out* src = red + (s * KW) * 16 * LD + row * LD + c;
                Acc v = *reinterpret_cast<const Acc*>(src);
#pragma unroll
                for (int x = 1; x < KW; ++x) v += *reinterpret_cast<const Acc*>(src + x * 16 * LD);
                const int64_t out_row = out_rows[k];
                const int col = nbase + s * WC + c;
                if (out_row < 0 || col >= N) continue;
                Out* dst = C + out_row * ldc + col;
                if (vec_store) {
                    if (c_stream) store_streaming(dst, v);
                    else *reinterpret_cast<Acc*>(dst) = v;
                } else {
                    dst[0] = v[0]; dst[1] = v[1]; dst[2] = v[2]; dst[3] = v[3];
                }
            }
        } else {
#pragma unroll
            for (int k = 0; k < EP; ++k) {
                const int e = static_cast<int>(threadIdx.x) + k * WAVES * 64;
                if (e >= SW * 16 * WC) break;
                const int s = e / (16 * WC), row = (e / WC) % 16, c = e % WC;
                const Out* src = red + (s * KW) * 16 * LD + row * LD + c;
                Out v = src[0];
#pragma unroll
                for (int x = 1; x < KW; ++x) v += src[x * 16 * LD];
                const int64_t out_row = out_rows[k];
                const int col = nbase + s * WC + c;
                if (out_row >= 0 && col < N) C[out_row * ldc + col] = v;
            }
        }
    }
}

// How many workgroups of a launch a compute unit should hold at a time.  The registers of the wide
// variants allow three waves per SIMD; with block rows of about the same length, whole cache lines
// of B per row and slab and one slab per workgroup, TWO are as fast or faster: all waves walk their
// rows at about the same pace, so at any moment the chip gathers from a window of B's rows, and
// fewer rows in flight keep that window narrower for the L2s.  Measured, three -> two waves per SIMD:
// a 32768 x 32768 matrix of 2048 block rows of ~21 packs 58.3 -> 50.2 us at N = 256, 100.5 -> 75.5 at
// N = 384, 124.9 -> 99.8 at 512, 202.8 -> 151.7 at 768 (at N = 256 also ten / six / five workgroups
// per unit: 56.3 / 61.4 / 67.0 us); random matrices of 64-400 entries per row, a band and a pruned
// weight matrix on this kernel, and all of them in 8-bit types: within 2 % either way.  It loses
// where the rows differ in length (power-law degrees: 81.6 -> 87-109 us for any limit), with two
// slabs per workgroup and with rows of B off the cache lines (N = 1000: 347 -> 438 us), which is
// why the caller asks for it only in the case above.  The limit is set by asking for LDS with the
// launch that the kernel does not touch: that many bytes per workgroup that two waves per SIMD fit
// a compute unit's 160 KiB and no more.  Returns the bytes to ask for, or 0 to leave the launch alone.
struct Residency {
    int resident = 0;          // workgroups of the kernel a compute unit holds (0: not known)
    int64_t static_lds = 0;    // LDS bytes the kernel declares
};
static Residency query_residency(const void* kernel, int waves_per_group)
{
    Residency r;
    hipFuncAttributes attr;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&r.resident, kernel, waves_per_group * 64, 0) != hipSuccess ||
        hipFuncGetAttributes(&attr, kernel) != hipSuccess || r.resident <= 0) {
        (void)hipGetLastError();
        r.resident = 0;
        return r;
    }
    r.static_lds = static_cast<int64_t>(attr.sharedSizeBytes);
    return r;
}
static size_t lds_to_limit_residency(const Residency& info, int waves_per_group, int64_t groups, bool even)
{
    if (!even || groups <= 0 || info.resident <= 0) return 0;
    const int64_t resident = info.resident;
    constexpr int64_t kUnits = 256, kLdsBytes = 160 * 1024;
    const int64_t best = (8 + waves_per_group - 1) / waves_per_group;           // two waves per SIMD
    if (best >= resident || groups < kUnits * best) return 0;                   // nothing to limit, or the chip would not fill
    const int64_t per_group = kLdsBytes / best / 512 * 512;                      // best groups fit, best + 1 do not
    if (kLdsBytes / per_group != best || per_group > 64 * 1024) return 0;
    const int64_t extra = per_group - info.static_lds;
    return extra > 0 ? static_cast<size_t>(extra) : 0;
}

template <int NT, int KW, int SW, int NCH, int LMAX, int DT, int NARROW = 0>
static int launch_variant(const DeviceBcsr& d, const void* B, int64_t ldb, void* C, int64_t ldc,
                          int64_t N, hipStream_t stream, bool even_rows = false)
{
    constexpr int ES = Elem<DT>::ES;
    const int64_t per_group = 16 * NT * NCH * SW;          // columns of one workgroup
    if (d.n_order == 0) return 0;
    dim3 grid(static_cast<unsigned>(d.n_order), static_cast<unsigned>((N + per_group - 1) / per_group));
    const uint32_t b_bytes = d.K > 0 ? static_cast<uint32_t>(((d.K - 1) * ldb + N) * ES) : 0u;
    const int vec_store = (ldc % 4 == 0 && reinterpret_cast<uintptr_t>(C) % 16 == 0 && N % 4 == 0) ? 1 : 0;
    // Block values that are read once per launch (a single group per block row) and are too many
    // to stay in the 256 MB Infinity Cache between launches are streamed past the L2, which
    // then keeps the rows of B.
    int stream_hint = (grid.y == 1 && SW == 1 && static_cast<double>(d.stream_bytes) > 200e6) ? 1 : 0;
    // A B of about the size of the L2s stays there between its uses only if the write of C does
    // not push it out: then C is stored past the cache (measured: -7 % where B is 4 MiB, no gain
    // or a loss where B is 16 MiB and more).
    if (static_cast<double>(d.K) * static_cast<double>(N) * ES <= 8.0e6) stream_hint |= 2;
    // asked once per kernel and process (the devices of a process are taken to be alike)
    static const Residency info = query_residency(reinterpret_cast<const void*>(&spmm_kernel<NT, KW, SW, NCH, LMAX, DT, NARROW>), KW * SW);
    const size_t lds = lds_to_limit_residency(info, KW * SW, static_cast<int64_t>(grid.x) * grid.y, even_rows);
    hipLaunchKernelGGL((spmm_kernel<NT, KW, SW, NCH, LMAX, DT, NARROW>), grid, dim3(KW * SW * 64), lds, stream,
                       d.work, d.slots, d.vals, d.perm, B, b_bytes, static_cast<uint32_t>(ldb * ES), static_cast<uint32_t>(d.K),
                       static_cast<typename Elem<DT>::Out*>(C), ldc, static_cast<int>(N), vec_store, stream_hint);
    return static_cast<int>(hipGetLastError());
}

template <int DT>
static const char* variant_name(int nt, int kw, int sw, int nch, int lmax)
{
    static thread_local char buf[48];
    const char* type = DT == kF16 ? "f16" : DT == kBF16 ? "bf16" : DT == kE4M3 ? "e4m3" : DT == kE5M2 ? "e5m2" : "i8";
    snprintf(buf, sizeof(buf), "spmm_%s_n%dk%ds%dc%d_l%d", type, nt, kw, sw, nch, lmax);
    return buf;
}

template <int NT, int LMAX, int DT>
static int launch_shape(const DeviceBcsr& d, const void* B, int64_t ldb, void* C, int64_t ldc,
                        int64_t N, hipStream_t stream, const char** variant)
{
    constexpr int ES = Elem<DT>::ES;
    // A wave covers NCH chunks of 16*NT columns with one read of the block values; SW waves of
    // a group take neighbouring slabs of the same block row, so its block values reach HBM once
    // per group; KW waves share one block row (partial tiles summed through LDS).  Splitting a
    // row costs a pipeline fill and a reduction per extra wave, so KW is the smallest split for
    // which (a) the longest row, walked at about 0.25 us per pack and wave, stays below half of
    // what the launch needs (its streams at ~5 TB/s plus the gather of B), and (b) the launch
    // has at least two waves for every SIMD of the chip (four where the variant's registers
    // allow six resident).
    const int64_t slabs = (N + 16 * NT - 1) / (16 * NT);
    // two chunks per wave: 16-bit types only (the 8-bit types reach the same 256 bytes per row
    // with NT = 16), and the dense class has no registers to spare
    constexpr bool kTwoChunks = NT == 8 && ES == 2 && LMAX < 8;
    const int nch = (kTwoChunks && slabs >= 2) ? 2 : 1;
    const int64_t wave_slabs = (slabs + nch - 1) / nch;
    // Two waves of a group on neighbouring slabs read the block values once for both, but every
    // phase of the launch then gathers from twice as many columns of B.  Measured (three
    // workloads, N = 256 ... 1000, 16-bit and 8-bit): with full-width pieces of B (256 bytes per
    // row and slab) that start on cache lines, one slab per group is 2-14 % faster; with
    // misaligned rows (N = 1000) or narrow pieces the pair is, and so it is when the block values
    // are too many to stay in the 256 MB Infinity Cache from one pass over the block rows to the
    // next (712 MB: 683 against 744 us).
    const bool whole_lines = 16 * NT * ES >= 256 && (ldb * ES) % 128 == 0 && reinterpret_cast<uintptr_t>(B) % 128 == 0;
    const bool one_slab = whole_lines && static_cast<double>(d.stream_bytes) <= 128.0e6;
    const int sw = (wave_slabs >= 2 && !one_slab) ? 2 : 1;
    const int64_t groups = d.n_order * ((wave_slabs + sw - 1) / sw);
    const double stream_us = (static_cast<double>(d.stream_bytes) + static_cast<double>(d.M) * N * 4.0 +
                              static_cast<double>(d.K) * N * ES) / 5.0e6;
    // every named row of B is fetched once per slab, 16*NT elements of it (no less than a
    // 64-byte piece).  The compute units take in about 10 TB/s of such fills together; the
    // gather enters at twice that rate, which is where the measured choices (three workloads,
    // N = 1 ... 1000) change over.
    const double piece = 16.0 * NT * ES < 64.0 ? 64.0 : 16.0 * NT * ES;
    const double gather_us = static_cast<double>(d.b_rows) * static_cast<double>(slabs) * piece / 20.0e6;
    const double longest_us = static_cast<double>(d.max_row_packs) * 0.25;
    // the narrow variants (row loads of at most four bytes) keep six waves per SIMD resident,
    // the wide ones three
    const int64_t wave_target = NT * ES <= 4 ? 4096 : 2048;
    // (a) is for rows that stand out; where all rows are about as long, (b) alone decides
    const bool skewed = static_cast<double>(d.max_row_packs) > 2.0 * d.mean_row_packs;
    int kw = 1;
    while (kw < 8 && d.mean_row_packs >= 4.0 * kw &&
           ((skewed && longest_us / kw > 0.5 * (stream_us + gather_us)) || groups * sw * kw < wave_target)) kw *= 2;
    if (nch == 2 && kw > 4) kw = 4;
    // rows of about the same length: the launch may hold fewer workgroups per compute unit (launch_variant)
    const bool even = !skewed && d.mean_row_packs >= 16.0 && whole_lines && sw == 1;
#define SMAT_LAUNCH(KW_, SW_, NCH_)                                                             \
    do {                                                                                        \
        *variant = variant_name<DT>(NT, KW_, SW_, NCH_, LMAX);                                  \
        return launch_variant<NT, KW_, SW_, NCH_, LMAX, DT>(d, B, ldb, C, ldc, N, stream, even); \
    } while (0)
    if constexpr (kTwoChunks) {
        if (nch == 2) {
            if (sw == 2) {
                // (eight waves per workgroup leave a wave 256 registers; with packs of up to sixteen columns the
                // two-chunk walk wants some 270 and would spill inside its loop: two waves per row there)
                if constexpr (LMAX < 4) {
                    if (kw >= 4) SMAT_LAUNCH(4, 2, 2);
                }
                if (kw >= 2) SMAT_LAUNCH(2, 2, 2);
                SMAT_LAUNCH(1, 2, 2);
            }
            if (kw >= 4) SMAT_LAUNCH(4, 1, 2);
            if (kw == 2) SMAT_LAUNCH(2, 1, 2);
            SMAT_LAUNCH(1, 1, 2);
        }
    }
    if (sw == 2) {
        if (kw >= 4) SMAT_LAUNCH(4, 2, 1);
        if (kw == 2) SMAT_LAUNCH(2, 2, 1);
        SMAT_LAUNCH(1, 2, 1);
    }
    if (kw == 8) SMAT_LAUNCH(8, 1, 1);
    if (kw == 4) SMAT_LAUNCH(4, 1, 1);
    if (kw == 2) SMAT_LAUNCH(2, 1, 1);
    SMAT_LAUNCH(1, 1, 1);
#undef SMAT_LAUNCH
}

template <int NT, int DT>
static int launch_nt(const DeviceBcsr& d, const void* B, int64_t ldb, void* C, int64_t ldc,
                     int64_t N, hipStream_t stream, const char** variant)
{
    // the kernel only carries the loops (and registers) for the row classes the matrix has
    if (d.max_class >= 2) return launch_shape<NT, 8, DT>(d, B, ldb, C, ldc, N, stream, variant);
    if (d.max_class == 1) return launch_shape<NT, 4, DT>(d, B, ldb, C, ldc, N, stream, variant);
    return launch_shape<NT, 2, DT>(d, B, ldb, C, ldc, N, stream, variant);
}

// Entry of a translation unit's instantiations: all load widths of one operand type.
template <int DT>
static int launch_dtype(const DeviceBcsr& d, const void* B, int64_t ldb, void* C, int64_t ldc,
                        int64_t N, hipStream_t stream, const char** variant)
{
    constexpr int ES = Elem<DT>::ES;
    // B row loads are NT elements wide and a wave covers 16*NT columns per pass over its packs.
    // Among the widths N, ldb and the base address allow, take the one with the least
    // (passes x cost of a pass); the relative cost of a pass, 1 : 1.05 : 1.4 : 1.65 for loads of
    // 2, 4, 8 and 16 bytes, was measured with fp16 on two workloads at N = 8 ... 1000 (ties:
    // the wider load) and is taken over for the 8-bit types, whose widest load is 16 elements.
    const uintptr_t addr = reinterpret_cast<uintptr_t>(B);
    const double cost_of_bytes[17] = {0, 1.0, 1.0, 0, 1.05, 0, 0, 0, 1.4, 0, 0, 0, 0, 0, 0, 0, 1.65};
    constexpr int kWidest = 16 / ES;
    int best = 1;
    double best_cost = static_cast<double>((N + 15) / 16);
    for (int nt = 2; nt <= kWidest; nt *= 2) {
        if (N % nt != 0 || ldb % nt != 0 || addr % (ES * nt) != 0) continue;
        const double cost = static_cast<double>((N + 16 * nt - 1) / (16 * nt)) * cost_of_bytes[ES * nt];
        if (cost <= best_cost) { best = nt; best_cost = cost; }
    }
    if constexpr (ES == 1) {
        if (best == 16) return launch_nt<16, DT>(d, B, ldb, C, ldc, N, stream, variant);
    }
    switch (best) {
    case 8: return launch_nt<8, DT>(d, B, ldb, C, ldc, N, stream, variant);
    case 4: return launch_nt<4, DT>(d, B, ldb, C, ldc, N, stream, variant);
    case 2: return launch_nt<2, DT>(d, B, ldb, C, ldc, N, stream, variant);
    default: return launch_nt<1, DT>(d, B, ldb, C, ldc, N, stream, variant);
    }
}

}  // namespace smat
