// Kernel template of the block-dense SpMM path (see kernels_dense.hip for the description).
// Included by the two translation units that instantiate it with different register-file
// settings: the 128-column tile keeps its accumulators in ordinary VGPRs, the 256-column
// tile needs the accumulation registers for them.
#pragma once

#include <hip/hip_runtime.h>

#include "kernels.h"

namespace smat {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr uint32_t kOutOfRange = 0x80000000u;
constexpr int kRsrcFlags = 0x00020000;

__device__ __forceinline__ u32x4 buf_load16(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff)
{
    const i32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 0);
    return u32x4{static_cast<uint32_t>(v[0]), static_cast<uint32_t>(v[1]), static_cast<uint32_t>(v[2]), static_cast<uint32_t>(v[3])};
}

template <bool BF16>
__device__ __forceinline__ f32x4 mfma_pack(u32x4 a, u32x4 b, f32x4 c)
{
    if constexpr (BF16)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

}  // namespace

// C rows of the dense super rows, 128 columns per workgroup; 4 waves, wave w owns block rows
// 4w..4w+3 of the super row.  With gridDim.z > 1 the steps of a tile are split over that many
// workgroups; each writes its partial 256 x 128 tile to the scratch area and a second kernel
// adds the partial tiles in a fixed order (reproducible; fp32 atomics on C were measured at
// three times the cost of the idle compute units they were meant to fill).
//
// RING is the depth of the prefetch (see below).  The deep variant (4) needs more than 256
// registers and runs one workgroup per compute unit; the shallow one (2) fits two, which pays
// for super rows of few steps, where the start and the write of C of one workgroup overlap
// the loop of the other.
//
// KG = 2 puts two such groups of four waves into one workgroup: group 0 walks the even steps of
// the tile, group 1 the odd ones, each with its own panel buffers, and at the end group 1 hands
// its accumulators to group 0 through LDS.  A SIMD then holds two waves whose LDS reads,
// barrier waits and matrix instructions overlap, which one wave alone cannot do.
template <bool BF16, int RING, int NCH, int KG = 1>
__global__ __launch_bounds__(256 * KG)
__attribute__((amdgpu_waves_per_eu((KG == 1 && (RING > 2 || NCH > 1)) ? 1 : 2, (KG == 1 && (RING > 2 || NCH > 1)) ? 1 : 2)))
void spmm_dense_kernel(DeviceBcsr d, DenseTiles t, const void* __restrict__ B, uint32_t b_bytes,
                       uint32_t ldb_bytes, float* __restrict__ C, int64_t ldc, int N, int vec_store)
{
    constexpr int NT = 8;                          // columns per lane; 16 lanes cover a 128-column chunk
    constexpr int RM = 4;                          // block rows per wave
    constexpr int NS = 2 * NCH;                    // 16-byte pieces of the panel a thread stages per step
    static_assert(KG == 1 || (RING <= 3 && NCH == 1), "two wave groups: at most 256 registers, 128 columns");
    constexpr int NBUF = RING == 3 ? 3 : 2;        // panel buffers; the loop body of RING steps keeps their indices constant
    __shared__ u32x4 panel_all[KG][NBUF][32][16 * NCH];   // per wave group, buffers of 32 B rows x (128 * NCH) halves

    const int tid = threadIdx.x & 255;             // thread inside its wave group
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);             // wave inside its group
    const int kg = KG == 1 ? 0 : __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x) >> 8);
    u32x4 (*panel)[32][16 * NCH] = panel_all[kg];
    const int i = lane & 15, g = lane >> 4;
    const int sidx = blockIdx.x;
    const int super = t.super_rows[sidx];
    const int n0 = blockIdx.y * (128 * NCH);
    const int ks = static_cast<int>(gridDim.z);    // workgroups sharing this tile's steps
    const int q_first = t.step_ptr[sidx], q_last = t.step_ptr[sidx + 1];
    const int per = (q_last - q_first + ks - 1) / ks;
    const int q0 = min(q_first + static_cast<int>(blockIdx.z) * per, q_last);
    const int q1 = min(q0 + per, q_last);
    const int nq = q1 - q0;

    const __amdgpu_buffer_rsrc_t b_rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(B), 0, static_cast<int>(b_bytes), kRsrcFlags);
    // tile values of this workgroup's steps q0..q1-1 are stored back to back
    const uint32_t first_slot = nq > 0 ? t.step_base[q0] : 0u;
    const uint32_t end_slot = nq > 0 ? t.step_base[q1 - 1] + __popc(t.step_rows[q1 - 1]) : 0u;
    const __amdgpu_buffer_rsrc_t a_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t*>(t.vals) + static_cast<size_t>(first_slot) * 512, 0,
        static_cast<int>((end_slot - first_slot) * 1024u), kRsrcFlags);

    // staging of the B panel: thread tid copies, per chunk, 16 bytes of rows (tid >> 4) and 16 + (tid >> 4)
    const int st_row = tid >> 4, st_chunk = tid & 15;
    uint32_t st_off[NCH];
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int st_col = n0 + 128 * c + NT * st_chunk;
        st_off[c] = st_col < N ? static_cast<uint32_t>(st_col) * 2u : kOutOfRange;
    }
    const uint32_t no_row = static_cast<uint32_t>(d.K);
    const int nbc = static_cast<int>((d.K + 15) >> 4);

    // What a step's loads need to know, fetched with scalar loads one step before it is used:
    // a scalar load that is waited for right away costs a few hundred cycles in which the wave,
    // alone on its SIMD, does nothing.
    struct StepMeta { int c0, c1; uint32_t rows, base; };
    auto fetch_meta = [&](int q) {
        StepMeta m;
        m.c0 = t.step_cols[2 * static_cast<size_t>(q)];
        m.c1 = t.step_cols[2 * static_cast<size_t>(q) + 1];
        m.rows = t.step_rows[q];
        m.base = t.step_base[q];
        return m;
    };
    auto load_panel = [&](const StepMeta& m, u32x4 (&stage)[NS]) {
        const int c0 = m.c0, c1 = m.c1;
        // rows past K (ragged last block column, or no second column) are out of range: zeros
        uint32_t row0 = c0 < nbc ? static_cast<uint32_t>(c0) * 16u + st_row : no_row;
        uint32_t row1 = c1 < nbc ? static_cast<uint32_t>(c1) * 16u + st_row : no_row;
        row0 = row0 < no_row ? row0 : no_row;
        row1 = row1 < no_row ? row1 : no_row;
        const uint32_t off0 = __umul24(row0, ldb_bytes), off1 = __umul24(row1, ldb_bytes);
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            stage[2 * c] = buf_load16(b_rsrc, off0 + st_off[c], 0u);
            stage[2 * c + 1] = buf_load16(b_rsrc, off1 + st_off[c], 0u);
        }
    };
    auto store_panel = [&](int buf, const u32x4 (&stage)[NS]) {
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            panel[buf][st_row][16 * c + st_chunk] = stage[2 * c];
            panel[buf][16 + st_row][16 * c + st_chunk] = stage[2 * c + 1];
        }
    };
    // Values of the wave's four block rows for step q.  A block row without data in the step
    // (or any block row in a step past the last one, `live` false) reads out of range (zeros)
    // and multiplies zeros: no branches in the loop body.
    auto load_a = [&](const StepMeta& m, bool live, u32x4 (&a)[RM]) {
        const uint32_t rows = m.rows;
        const uint32_t base = m.base - first_slot;
#pragma unroll
        for (int r = 0; r < RM; ++r) {
            const int j = RM * wave + r;
            const uint32_t slot = base + __popc(rows & ((1u << j) - 1u));
            const uint32_t absent = (live && (rows >> j & 1u)) ? 0u : kOutOfRange;      // wave-uniform
            a[r] = buf_load16(a_rsrc, (static_cast<uint32_t>(lane) * 16u) | absent, slot * 1024u);
        }
    };

    f32x4 acc[RM][NCH * NT];
#pragma unroll
    for (int r = 0; r < RM; ++r)
#pragma unroll
        for (int x = 0; x < NCH * NT; ++x) acc[r][x] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Software pipeline with register rings of RING slots (no copies; the loop body is RING steps
    // without an exit; steps past the last one read zeros as block values).  While step s is
    // multiplied, the B panels and block values of the next RING-1 steps are on their way from
    // memory; the panel of step s+1 is copied into the other LDS buffer at the end of step s.
    if constexpr (NCH > 1) {
        // One step per loop pass (every accumulator is written by exactly one instruction of the
        // body, which lets it stay in one register): the panel and the values of step s+1 are
        // requested at the start of step s; the values move to the working registers at its end.
        if (nq > 0) {
            u32x4 stage[NS];
            u32x4 a_cur[RM], a_next[RM];
            auto step_of = [&](int s) { return q0 + (s < nq ? s : nq - 1); };
            StepMeta meta = fetch_meta(step_of(0));
            load_panel(meta, stage);
            load_a(meta, true, a_cur);
            meta = fetch_meta(step_of(1));
            __builtin_amdgcn_sched_barrier(0);
            store_panel(0, stage);
            __syncthreads();
            int buf = 0;
            for (int s = 0; s < nq; ++s) {
                load_panel(meta, stage);
                load_a(meta, s + 1 < nq, a_next);
                meta = fetch_meta(step_of(s + 2));
#pragma unroll
                for (int c = 0; c < NCH; ++c) {
                    u32x4 R[8];
#pragma unroll
                    for (int kk = 0; kk < 8; ++kk) R[kk] = panel[buf][8 * g + kk][16 * c + i];
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int x = 0; x < NT; ++x) {
                        const uint32_t pick = (x & 1) ? 0x07060302u : 0x05040100u;
                        u32x4 b;
#pragma unroll
                        for (int qd = 0; qd < 4; ++qd)
                            b[qd] = __builtin_amdgcn_perm(R[2 * qd + 1][x >> 1], R[2 * qd][x >> 1], pick);
#pragma unroll
                        for (int r = 0; r < RM; ++r)
                            acc[r][c * NT + x] = mfma_pack<BF16>(a_cur[r], b, acc[r][c * NT + x]);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                store_panel(buf ^ 1, stage);
#pragma unroll
                for (int r = 0; r < RM; ++r) a_cur[r] = a_next[r];
                __syncthreads();
                buf ^= 1;
            }
        }
    } else
    if (nq > 0) {
        u32x4 stage[RING][NS];
        u32x4 a[RING][RM];
        // step s of this wave group is step kg + KG * s of the tile
        auto live_step = [&](int s) { return kg + KG * s < nq; };
        auto step_of = [&](int s) { return q0 + (live_step(s) ? kg + KG * s : nq - 1); };   // clamped: a cache hit, unused
        // prologue: steps 0..RING-2 requested, panel of step 0 in LDS
#pragma unroll
        for (int h = 0; h < RING - 1; ++h) {
            const StepMeta m = fetch_meta(step_of(h));
            load_panel(m, stage[h]);
            load_a(m, live_step(h), a[h]);
            __builtin_amdgcn_sched_barrier(0);
        }
        StepMeta meta = fetch_meta(step_of(RING - 1));
        store_panel(0, stage[0]);
        __syncthreads();
        const int iters = ((nq + KG - 1) / KG + RING - 1) / RING;      // the same for both groups: they share the barriers
        int s0 = 0;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int u = 0; u < RING; ++u) {
                const int s = s0 + u;
                const int buf = u % NBUF;
                load_panel(meta, stage[(u + RING - 1) % RING]);
                load_a(meta, live_step(s + RING - 1), a[(u + RING - 1) % RING]);
                meta = fetch_meta(step_of(s + RING));
#pragma unroll
                for (int c = 0; c < NCH; ++c) {
                    // B rows of this lane's k range: row 8g + kk, columns 128c + 8i .. 128c + 8i+7
                    u32x4 R[8];
#pragma unroll
                    for (int kk = 0; kk < 8; ++kk) R[kk] = panel[buf][8 * g + kk][16 * c + i];
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int x = 0; x < NT; ++x) {
                        const uint32_t pick = (x & 1) ? 0x07060302u : 0x05040100u;
                        u32x4 b;
#pragma unroll
                        for (int qd = 0; qd < 4; ++qd)
                            b[qd] = __builtin_amdgcn_perm(R[2 * qd + 1][x >> 1], R[2 * qd][x >> 1], pick);
#pragma unroll
                        for (int r = 0; r < RM; ++r)
                            acc[r][c * NT + x] = mfma_pack<BF16>(a[u][r], b, acc[r][c * NT + x]);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                store_panel((u + 1) % NBUF, stage[(u + 1) % RING]);
                __syncthreads();
            }
            s0 += RING;
        }
    }

    if constexpr (KG == 2) {
        // group 1 hands its accumulators to group 0, two block rows per wave at a time (64 KiB)
        __shared__ float handover[4 * 2 * NT * 4 * 64];
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            if (kg == 1) {
#pragma unroll
                for (int rr = 0; rr < 2; ++rr)
#pragma unroll
                    for (int x = 0; x < NT; ++x)
#pragma unroll
                        for (int y = 0; y < 4; ++y)
                            handover[(((wave * 2 + rr) * NT + x) * 4 + y) * 64 + lane] = acc[2 * half + rr][x][y];
            }
            __syncthreads();
            if (kg == 0) {
#pragma unroll
                for (int rr = 0; rr < 2; ++rr)
#pragma unroll
                    for (int x = 0; x < NT; ++x)
#pragma unroll
                        for (int y = 0; y < 4; ++y)
                            acc[2 * half + rr][x][y] += handover[(((wave * 2 + rr) * NT + x) * 4 + y) * 64 + lane];
            }
            __syncthreads();
        }
        if (kg == 1) return;
    }

    // acc[r][c*8 + x][y] = C'[16 * (16 super + 4 wave + r) + 4g + y][n0 + 128c + 8i + x]
    if constexpr (NCH == 1) {
        if (ks > 1) {
            // partial tile, row-major 256 x 128 floats, at [(tile * ks + z)]
            const size_t tile = static_cast<size_t>(sidx) * gridDim.y + blockIdx.y;
            float* part = t.scratch + (tile * ks + blockIdx.z) * (256 * 128);
#pragma unroll
            for (int r = 0; r < RM; ++r)
#pragma unroll
                for (int y = 0; y < 4; ++y) {
                    float* dst = part + (64 * wave + 16 * r + 4 * g + y) * 128 + NT * i;
                    *reinterpret_cast<f32x4*>(dst) = f32x4{acc[r][0][y], acc[r][1][y], acc[r][2][y], acc[r][3][y]};
                    *reinterpret_cast<f32x4*>(dst + 4) = f32x4{acc[r][4][y], acc[r][5][y], acc[r][6][y], acc[r][7][y]};
                }
            return;
        }
    }
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int col0 = n0 + 128 * c + NT * i;
        if (col0 >= N) continue;
#pragma unroll
        for (int r = 0; r < RM; ++r) {
            const int64_t br = static_cast<int64_t>(super) * 16 + RM * wave + r;
#pragma unroll
            for (int y = 0; y < 4; ++y) {
                const int64_t out_row = d.perm[br * 16 + 4 * g + y];
                if (out_row < 0) continue;
                float* dst = C + out_row * ldc + col0;
                if (vec_store) {
                    *reinterpret_cast<f32x4*>(dst) = f32x4{acc[r][c * NT][y], acc[r][c * NT + 1][y], acc[r][c * NT + 2][y], acc[r][c * NT + 3][y]};
                    *reinterpret_cast<f32x4*>(dst + 4) = f32x4{acc[r][c * NT + 4][y], acc[r][c * NT + 5][y], acc[r][c * NT + 6][y], acc[r][c * NT + 7][y]};
                } else {
#pragma unroll
                    for (int x = 0; x < NT; ++x) dst[x] = acc[r][c * NT + x][y];
                }
            }
        }
    }
}

template <bool BF16, int RING, int NCH = 1, int KG = 1>
static void launch_dense_tile(const DeviceBcsr& d, const DenseTiles& t, int ks, const void* B, uint32_t b_bytes, int64_t ldb,
                              float* C, int64_t ldc, int64_t N, int vec_store, hipStream_t s)
{
    dim3 grid(static_cast<unsigned>(t.n), static_cast<unsigned>((N + 128 * NCH - 1) / (128 * NCH)), static_cast<unsigned>(ks));
    hipLaunchKernelGGL((spmm_dense_kernel<BF16, RING, NCH, KG>), grid, dim3(256 * KG), 0, s, d, t, B, b_bytes,
                       static_cast<uint32_t>(ldb * 2), C, ldc, static_cast<int>(N), vec_store);
}

}  // namespace smat
