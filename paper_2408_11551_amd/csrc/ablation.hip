// Ablation kernels: the same product C = A * B computed from the canonical BCSR arrays (rowPtr,
// col, 256 values per block) with fewer of the optimisations, after the paper's figure of
// measured against modelled time (Performance model section; Implementation section, steps B
// and T): visiting every block of the grid and looking its presence up, iterating over the
// stored blocks only (B), and multiplying a block with one matrix instruction (T).  They exist
// to be timed next to the library's kernel; nothing else calls them.  One wavefront per
// (block row, 16 output columns), no software pipelining, no staging.
#include <hip/hip_runtime.h>

#include "kernels.h"

namespace smat {

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef short i16x4 __attribute__((ext_vector_type(4)));

template <bool BF16>
__device__ __forceinline__ float to_float(uint16_t bits)
{
    if constexpr (BF16) return __uint_as_float(static_cast<uint32_t>(bits) << 16);
    else return static_cast<float>(__builtin_bit_cast(_Float16, bits));
}

// lane (g, n): rows 4g .. 4g+3 of the block row, output column n0 + n
template <bool BF16>
__device__ __forceinline__ void store_tile(const CanonicalBcsr& m, int br, int g, int col, int N,
                                           const float (&acc)[4], float* __restrict__ C, int64_t ldc)
{
    if (col >= N) return;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int64_t out_row = m.perm[br * 16 + 4 * g + r];
        if (out_row >= 0) C[out_row * ldc + col] = acc[r];
    }
}

// Levels 0 and 1: scalar multiply-adds.  BY_PTR = false walks all block columns and asks the
// dense block map whether the block exists; BY_PTR = true walks rowPtr / col.
template <bool BF16, bool BY_PTR>
__global__ __launch_bounds__(64)
void ablation_scalar_kernel(CanonicalBcsr m, const uint16_t* __restrict__ B, int64_t ldb,
                            float* __restrict__ C, int64_t ldc, int N)
{
    const int lane = threadIdx.x, n = lane & 15, g = lane >> 4;
    const int br = blockIdx.x;
    const int col = blockIdx.y * 16 + n;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    auto multiply_block = [&](int64_t blk, int64_t bc) {
        const uint16_t* v = m.vals + blk * 256;
        for (int k = 0; k < 16; ++k) {
            const int64_t b_row = bc * 16 + k;
            const float b = (col < N && b_row < m.K) ? to_float<BF16>(B[b_row * ldb + col]) : 0.f;
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[r] = fmaf(to_float<BF16>(v[(4 * g + r) * 16 + k]), b, acc[r]);
        }
    };
    if constexpr (BY_PTR) {
        for (int blk = m.row_ptr[br]; blk < m.row_ptr[br + 1]; ++blk) multiply_block(blk, m.col_idx[blk]);
    } else {
        for (int64_t bc = 0; bc < m.nbc; ++bc) {
            const int blk = m.block_map[static_cast<int64_t>(br) * m.nbc + bc];
            if (blk >= 0) multiply_block(blk, bc);
        }
    }
    store_tile<BF16>(m, br, g, col, N, acc, C, ldc);
}

// Level 2: rowPtr / col iteration and one MFMA 16x16x16 per stored block.  Lane (g, i) holds
// A[i][4g .. 4g+3] (eight contiguous bytes of the row-major block) and B[4g .. 4g+3][n0 + i]
// (four 2-byte loads); the result has rows 4g .. 4g+3 of column n0 + i.
template <bool BF16>
__global__ __launch_bounds__(64)
void ablation_mfma_kernel(CanonicalBcsr m, const uint16_t* __restrict__ B, int64_t ldb,
                          float* __restrict__ C, int64_t ldc, int N)
{
    const int lane = threadIdx.x, i = lane & 15, g = lane >> 4;
    const int br = blockIdx.x;
    const int col = blockIdx.y * 16 + i;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int blk = m.row_ptr[br]; blk < m.row_ptr[br + 1]; ++blk) {
        const int64_t bc = m.col_idx[blk];
        const uint16_t* v = m.vals + static_cast<int64_t>(blk) * 256 + i * 16 + 4 * g;
        i16x4 a, b;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            a[j] = static_cast<short>(v[j]);
            const int64_t b_row = bc * 16 + 4 * g + j;
            b[j] = (col < N && b_row < m.K) ? static_cast<short>(B[b_row * ldb + col]) : short{0};
        }
        if constexpr (BF16) acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, b, acc, 0, 0, 0);
        else acc = __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(f16x4, a), __builtin_bit_cast(f16x4, b), acc, 0, 0, 0);
    }
    const float out[4] = {acc[0], acc[1], acc[2], acc[3]};
    store_tile<BF16>(m, br, g, col, N, out, C, ldc);
}

}  // namespace

int launch_ablation(const CanonicalBcsr& m, int level, bool bf16, const void* B, int64_t ldb, float* C,
                    int64_t ldc, int64_t N, void* stream)
{
    if (m.nbr == 0 || N == 0) return 0;
    const dim3 grid(static_cast<unsigned>(m.nbr), static_cast<unsigned>((N + 15) / 16));
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint16_t* b = static_cast<const uint16_t*>(B);
    const int n = static_cast<int>(N);
#define SMAT_ABLATE(KERNEL) hipLaunchKernelGGL(KERNEL, grid, dim3(64), 0, s, m, b, ldb, C, ldc, n)
    if (level == 0) { if (bf16) SMAT_ABLATE((ablation_scalar_kernel<true, false>)); else SMAT_ABLATE((ablation_scalar_kernel<false, false>)); }
    else if (level == 1) { if (bf16) SMAT_ABLATE((ablation_scalar_kernel<true, true>)); else SMAT_ABLATE((ablation_scalar_kernel<false, true>)); }
    else { if (bf16) SMAT_ABLATE(ablation_mfma_kernel<true>); else SMAT_ABLATE(ablation_mfma_kernel<false>); }
#undef SMAT_ABLATE
    return static_cast<int>(hipGetLastError());
}

}  // namespace smat
