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
#include <algorithm>
#include <cstdio>

#include "dense_kernel.inc.h"

namespace smat {

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

// Adds the ks partial tiles of every (super row, 128-column slab) in the order 0 .. ks-1 and
// writes the rows to C.  Eight workgroups per tile (32 rows each); a thread sums four groups of
// four columns and has all its loads in flight at once.
__global__ __launch_bounds__(256)
void dense_reduce_kernel(DeviceBcsr d, DenseTiles t, int ks, float* __restrict__ C, int64_t ldc, int N, int vec_store)
{
    const int super = t.super_rows[blockIdx.x];
    const int n0 = blockIdx.y * 128;
    const size_t tile = static_cast<size_t>(blockIdx.x) * gridDim.y + blockIdx.y;
    const float* part = t.scratch + tile * ks * (256 * 128);
    f32x4 v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int e = static_cast<int>(blockIdx.z) * 1024 + j * 256 + static_cast<int>(threadIdx.x);
        v[j] = *reinterpret_cast<const f32x4*>(part + e * 4);
    }
    for (int z = 1; z < ks; ++z)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int e = static_cast<int>(blockIdx.z) * 1024 + j * 256 + static_cast<int>(threadIdx.x);
            v[j] += *reinterpret_cast<const f32x4*>(part + static_cast<size_t>(z) * (256 * 128) + e * 4);
        }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int e = static_cast<int>(blockIdx.z) * 1024 + j * 256 + static_cast<int>(threadIdx.x);
        const int row = e >> 5, c = (e & 31) * 4;
        const int64_t out_row = d.perm[static_cast<int64_t>(super) * 256 + row];
        if (out_row < 0 || n0 + c >= N) continue;             // N is a multiple of 8 on this path
        float* dst = C + out_row * ldc + n0 + c;
        if (vec_store) {
            *reinterpret_cast<f32x4*>(dst) = v[j];
        } else {
            dst[0] = v[j][0]; dst[1] = v[j][1]; dst[2] = v[j][2]; dst[3] = v[j][3];
        }
    }
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

// 256-column tiles, compiled in kernels_dense_wide.hip
void launch_dense_wide(const DeviceBcsr& d, const DenseTiles& t, bool bf16, const void* B, uint32_t b_bytes,
                       int64_t ldb, float* C, int64_t ldc, int64_t N, int vec_store, void* stream);

int launch_spmm_dense(const DeviceBcsr& d, const DenseTiles& t, bool bf16, const void* B, int64_t ldb,
                      float* C, int64_t ldc, int64_t N, void* stream, const char** variant)
{
    if (t.n == 0) return 0;
    const uint32_t b_bytes = d.K > 0 ? static_cast<uint32_t>(((d.K - 1) * ldb + N) * 2) : 0u;
    const int vec_store = (ldc % 4 == 0 && reinterpret_cast<uintptr_t>(C) % 16 == 0 && N % 4 == 0) ? 1 : 0;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // Tile width: 256 columns when the super rows are long (the loop, not its start and end,
    // is what counts) and there are enough wide tiles for every compute unit; the wide tile
    // moves a third fewer bytes per matrix instruction (measured: 9 % faster at N = 4096,
    // slower at N = 2048 where it leaves half of the chip idle).
    const bool deep = t.mean_steps >= 32.0;
    const bool wide = deep && static_cast<int64_t>(t.n) * ((N + 255) / 256) >= 240;
    const int ks = wide ? 1 : dense_split(t, N);
    static thread_local char name[40];
    if (wide) snprintf(name, sizeof(name), "spmm_dense_%s_w", bf16 ? "bf16" : "f16");
    else if (ks > 1) snprintf(name, sizeof(name), "spmm_dense_%s_g%dk%d", bf16 ? "bf16" : "f16", deep ? 2 : 1, ks);
    else snprintf(name, sizeof(name), "spmm_dense_%s_g%d", bf16 ? "bf16" : "f16", deep ? 2 : 1);
    *variant = name;
    if (wide) {
        launch_dense_wide(d, t, bf16, B, b_bytes, ldb, C, ldc, N, vec_store, stream);
    } else if (bf16) {
        if (deep) launch_dense_tile<true, 2, 1, 2>(d, t, ks, B, b_bytes, ldb, C, ldc, N, vec_store, s);
        else launch_dense_tile<true, 2>(d, t, ks, B, b_bytes, ldb, C, ldc, N, vec_store, s);
    } else {
        if (deep) launch_dense_tile<false, 2, 1, 2>(d, t, ks, B, b_bytes, ldb, C, ldc, N, vec_store, s);
        else launch_dense_tile<false, 2>(d, t, ks, B, b_bytes, ldb, C, ldc, N, vec_store, s);
    }
    if (ks > 1)
        hipLaunchKernelGGL(dense_reduce_kernel, dim3(static_cast<unsigned>(t.n), static_cast<unsigned>((N + 127) / 128), 8), dim3(256), 0, s,
                           d, t, ks, C, ldc, static_cast<int>(N), vec_store);
    return static_cast<int>(hipGetLastError());
}

}  // namespace smat
