// HIP kernels for gfx950: the SpMM path for block-dense parts of the matrix.
//
// Where sixteen consecutive block rows (a "super row", 256 rows of A') share most of their
// block columns, multiplying every block row on its own makes each wave fetch the same rows
// of B again.  Here one workgroup takes a super row and a slab of 128 columns of B and C and
// walks the UNION of the super row's block columns, two at a time (one MFMA 16x16x32 step):
// the 32 x 128 panel of B of a step is staged once in LDS and read by all four waves, each
// of which owns four of the sixteen block rows and keeps a 64 x 128 accumulator tile in
// registers.  A B operand built from LDS is reused for the wave's four block rows.  Block
// rows that have neither block of a step skip its MFMAs (their values are not stored).
//
// This is still the paper's scheme (Implementation section, Alg. 1): per output tile, loop over
// stored blocks and multiply-accumulate on the matrix units; the loop is merely shared by the
// block rows of a super row so that the panel of B is read once for all of them.
#include "kernels.h"

#include <hip/hip_runtime.h>

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
__device__ __forceinline__ f32x4 mfma_pair(u32x4 a, u32x4 b, f32x4 c)
{
    if constexpr (BF16)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

}  // namespace

// Scatter of the CSR values into the tile layout: one thread per row of a dense super row.
// A tile step q holds, for every block row of the super row that has one of the step's two
// block columns, 1 KiB: lane l = 16 g + i owns halves [8 l, 8 l + 8) = row i, columns 8g..8g+7 of
// the 32 columns of the step (first block column: 0..15, second: 16..31).
__global__ void dense_fill_kernel(DeviceBcsr d, DenseTiles t, const int64_t* __restrict__ csr_row_ptr,
                                  const int32_t* __restrict__ csr_col_idx, const uint16_t* __restrict__ csr_vals,
                                  uint16_t* __restrict__ vals_out)
{
    const int sidx = blockIdx.x;                       // which dense super row
    const int rr = threadIdx.x;                        // row inside the super row, 0..255
    const int64_t i = static_cast<int64_t>(t.super_rows[sidx]) * 256 + rr;
    if (i >= d.M) return;
    const int64_t r = d.perm[i];
    const int j = rr >> 4, ii = rr & 15;
    const int q0 = t.step_ptr[sidx], q1 = t.step_ptr[sidx + 1];
    const int32_t* cols = t.step_cols + 2 * static_cast<size_t>(q0);   // ascending; a missing last column is INT_MAX
    const int ncols = 2 * (q1 - q0);
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
        const size_t q = static_cast<size_t>(q0 + (lo >> 1));
        const uint32_t rows = t.step_rows[q];
        const size_t slot = static_cast<size_t>(t.step_base[q]) + __popc(rows & ((1u << j) - 1u));
        const int pc = (lo & 1) * 16 + (c & 15);
        vals_out[slot * 512 + static_cast<size_t>((16 * (pc >> 3) + ii) * 8 + (pc & 7))] = csr_vals[p];
    }
}

int launch_dense_fill(const DeviceBcsr& d, const DenseTiles& t, const int64_t* csr_row_ptr,
                      const int32_t* csr_col_idx, const uint16_t* csr_vals, uint16_t* vals_out, void* stream)
{
    if (t.n == 0) return 0;
    hipLaunchKernelGGL(dense_fill_kernel, dim3(static_cast<unsigned>(t.n)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), d, t, csr_row_ptr, csr_col_idx, csr_vals, vals_out);
    return static_cast<int>(hipGetLastError());
}

// C rows of the dense super rows, 128 columns per workgroup; 4 waves, wave w owns block rows
// 4w..4w+3 of the super row.
template <bool BF16>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void spmm_dense_kernel(DeviceBcsr d, DenseTiles t, const void* __restrict__ B, uint32_t b_bytes,
                       uint32_t ldb_bytes, float* __restrict__ C, int64_t ldc, int N, int vec_store)
{
    constexpr int NT = 8;                          // columns per lane; 16 lanes cover the 128-column slab
    constexpr int RM = 4;                          // block rows per wave
    __shared__ u32x4 panel[2][32][16];             // two buffers of 32 B rows x 128 halves (8 KiB each)

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i = lane & 15, g = lane >> 4;
    const int sidx = blockIdx.x;
    const int super = t.super_rows[sidx];
    const int n0 = blockIdx.y * 128;
    const int q0 = t.step_ptr[sidx], q1 = t.step_ptr[sidx + 1];
    const int nq = q1 - q0;

    const __amdgpu_buffer_rsrc_t b_rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(B), 0, static_cast<int>(b_bytes), kRsrcFlags);
    // tile values of this super row: steps q0..q1-1 are stored back to back
    const uint32_t first_slot = nq > 0 ? t.step_base[q0] : 0u;
    const uint32_t end_slot = nq > 0 ? t.step_base[q1 - 1] + __popc(t.step_rows[q1 - 1]) : 0u;
    const __amdgpu_buffer_rsrc_t a_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t*>(t.vals) + static_cast<size_t>(first_slot) * 512, 0,
        static_cast<int>((end_slot - first_slot) * 1024u), kRsrcFlags);

    // staging of the B panel: thread tid copies 16 bytes of rows (tid >> 4) and 16 + (tid >> 4)
    const int st_row = tid >> 4, st_chunk = tid & 15;
    const int st_col = n0 + NT * st_chunk;
    const uint32_t st_off = st_col < N ? static_cast<uint32_t>(st_col) * 2u : kOutOfRange;
    const uint32_t no_row = static_cast<uint32_t>(d.K);
    const int nbc = static_cast<int>((d.K + 15) >> 4);

    auto b_row = [&](int bc) -> uint32_t {         // first B row of a block column, or "no row"
        return bc < nbc ? static_cast<uint32_t>(bc) * 16u : no_row;
    };
    auto load_panel = [&](int q, u32x4 (&stage)[2]) {
        const int c0 = t.step_cols[2 * static_cast<size_t>(q)], c1 = t.step_cols[2 * static_cast<size_t>(q) + 1];
        const uint32_t r0 = b_row(c0), r1 = b_row(c1);
        // rows past K (ragged last block column, or no second column) are out of range: zeros
        const uint32_t row0 = r0 == no_row ? no_row : r0 + st_row;
        const uint32_t row1 = r1 == no_row ? no_row : r1 + st_row;
        stage[0] = buf_load16(b_rsrc, __umul24(row0 < no_row ? row0 : no_row, ldb_bytes) + st_off, 0u);
        stage[1] = buf_load16(b_rsrc, __umul24(row1 < no_row ? row1 : no_row, ldb_bytes) + st_off, 0u);
    };
    // Values of the wave's four block rows for step q.  A block row without data in the step
    // (or any block row in a step past the last one, `live` false) reads out of range (zeros)
    // and multiplies zeros: no branches in the loop body.
    auto load_a = [&](int q, bool live, u32x4 (&a)[RM]) {
        const uint32_t rows = t.step_rows[q];
        const uint32_t base = t.step_base[q] - first_slot;
#pragma unroll
        for (int r = 0; r < RM; ++r) {
            const int j = RM * wave + r;
            const uint32_t slot = base + __popc(rows & ((1u << j) - 1u));
            const uint32_t absent = (live && (rows >> j & 1u)) ? 0u : kOutOfRange;      // wave-uniform
            a[r] = buf_load16(a_rsrc, (static_cast<uint32_t>(lane) * 16u) | absent, slot * 1024u);
        }
    };

    f32x4 acc[RM][NT];
#pragma unroll
    for (int r = 0; r < RM; ++r)
#pragma unroll
        for (int x = 0; x < NT; ++x) acc[r][x] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Software pipeline, four-slot register rings (no copies, loop body of four steps without
    // an exit; steps past the last one read zeros as block values).  While step s is multiplied, the B panels of steps
    // s+2 and s+3 and the block values of steps s+1..s+3 are on their way from memory; the panel
    // of step s+1 is copied into the other LDS buffer at the end of step s.
    if (nq > 0) {
        u32x4 stage[4][2];
        u32x4 a[4][RM];
        auto step_of = [&](int s) { return q0 + (s < nq ? s : nq - 1); };   // clamped: a cache hit, unused
        // prologue: steps 0..2 requested, panel of step 0 in LDS
        load_panel(step_of(0), stage[0]);
        load_a(step_of(0), true, a[0]);
        __builtin_amdgcn_sched_barrier(0);
        load_panel(step_of(1), stage[1]);
        load_a(step_of(1), 1 < nq, a[1]);
        __builtin_amdgcn_sched_barrier(0);
        load_panel(step_of(2), stage[2]);
        load_a(step_of(2), 2 < nq, a[2]);
        __builtin_amdgcn_sched_barrier(0);
        panel[0][st_row][st_chunk] = stage[0][0];
        panel[0][16 + st_row][st_chunk] = stage[0][1];
        __syncthreads();
        const int iters = (nq + 3) >> 2;
        int s0 = 0;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int s = s0 + u;
                const int buf = u & 1;
                load_panel(step_of(s + 3), stage[(u + 3) & 3]);
                load_a(step_of(s + 3), s + 3 < nq, a[(u + 3) & 3]);
                // B rows of this lane's k range: row 8g + kk, columns 8i .. 8i+7
                u32x4 R[8];
#pragma unroll
                for (int kk = 0; kk < 8; ++kk) R[kk] = panel[buf][8 * g + kk][i];
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int x = 0; x < NT; ++x) {
                    const uint32_t pick = (x & 1) ? 0x07060302u : 0x05040100u;
                    u32x4 b;
#pragma unroll
                    for (int qd = 0; qd < 4; ++qd)
                        b[qd] = __builtin_amdgcn_perm(R[2 * qd + 1][x >> 1], R[2 * qd][x >> 1], pick);
#pragma unroll
                    for (int r = 0; r < RM; ++r) acc[r][x] = mfma_pair<BF16>(a[u][r], b, acc[r][x]);
                }
                __builtin_amdgcn_sched_barrier(0);
                panel[buf ^ 1][st_row][st_chunk] = stage[(u + 1) & 3][0];
                panel[buf ^ 1][16 + st_row][st_chunk] = stage[(u + 1) & 3][1];
                __syncthreads();
            }
            s0 += 4;
        }
    }

    // acc[r][x][y] = C'[16 * (16 super + 4 wave + r) + 4g + y][n0 + 8i + x]
    const int col0 = n0 + NT * i;
    if (col0 < N) {
#pragma unroll
        for (int r = 0; r < RM; ++r) {
            const int64_t br = static_cast<int64_t>(super) * 16 + RM * wave + r;
            if (br >= d.nbr) continue;
#pragma unroll
            for (int y = 0; y < 4; ++y) {
                const int64_t out_row = d.perm[br * 16 + 4 * g + y];
                if (out_row < 0) continue;
                float* dst = C + out_row * ldc + col0;
                if (vec_store) {
                    *reinterpret_cast<f32x4*>(dst) = f32x4{acc[r][0][y], acc[r][1][y], acc[r][2][y], acc[r][3][y]};
                    *reinterpret_cast<f32x4*>(dst + 4) = f32x4{acc[r][4][y], acc[r][5][y], acc[r][6][y], acc[r][7][y]};
                } else {
#pragma unroll
                    for (int x = 0; x < NT; ++x) dst[x] = acc[r][x][y];
                }
            }
        }
    }
}

int launch_spmm_dense(const DeviceBcsr& d, const DenseTiles& t, bool bf16, const void* B, int64_t ldb,
                      float* C, int64_t ldc, int64_t N, void* stream)
{
    if (t.n == 0) return 0;
    dim3 grid(static_cast<unsigned>(t.n), static_cast<unsigned>((N + 127) / 128));
    const uint32_t b_bytes = d.K > 0 ? static_cast<uint32_t>(((d.K - 1) * ldb + N) * 2) : 0u;
    const int vec_store = (ldc % 4 == 0 && reinterpret_cast<uintptr_t>(C) % 16 == 0 && N % 4 == 0) ? 1 : 0;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (bf16)
        hipLaunchKernelGGL(spmm_dense_kernel<true>, grid, dim3(256), 0, s, d, t, B, b_bytes,
                           static_cast<uint32_t>(ldb * 2), C, ldc, static_cast<int>(N), vec_store);
    else
        hipLaunchKernelGGL(spmm_dense_kernel<false>, grid, dim3(256), 0, s, d, t, B, b_bytes,
                           static_cast<uint32_t>(ldb * 2), C, ldc, static_cast<int>(N), vec_store);
    return static_cast<int>(hipGetLastError());
}

}  // namespace smat
