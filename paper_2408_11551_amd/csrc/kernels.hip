// HIP kernels for gfx950 (CDNA4, wave64): device-side BCSR value fill and the
// blocked SpMM of the paper's Implementation section (Alg. 1: per output tile,
// loop over the stored blocks of the block row and multiply-accumulate on the
// matrix units).  Written for MFMA 16x16x32 with fp32 accumulation.
#include "kernels.h"

#include <hip/hip_runtime.h>

namespace smat {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x2 __attribute__((ext_vector_type(2)));

// ---------------------------------------------------------------------------
// bind-time kernels
// ---------------------------------------------------------------------------
__global__ void fill_zero_kernel(u32x4* dst, size_t n16)
{
    const size_t stride = static_cast<size_t>(gridDim.x) * blockDim.x;
    for (size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n16; i += stride)
        dst[i] = u32x4{0u, 0u, 0u, 0u};
}

int launch_fill_zero(void* dst, size_t n16, void* stream)
{
    if (n16 == 0) return 0;
    const int threads = 256;
    const size_t want = (n16 + threads - 1) / threads;
    const int blocks = static_cast<int>(want < 8192 ? want : 8192);
    hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks), dim3(threads), 0, static_cast<hipStream_t>(stream),
                       static_cast<u32x4*>(dst), n16);
    return static_cast<int>(hipGetLastError());
}

// One thread per row of A' = P A: walks the row's CSR entries, finds each entry's block in
// the block row by binary search over the ascending block columns and stores the value at
// its place in the two-half-panel layout.
__global__ void bcsr_fill_kernel(DeviceBcsr d, const int64_t* __restrict__ csr_row_ptr,
                                 const int32_t* __restrict__ csr_col_idx,
                                 const uint16_t* __restrict__ csr_vals, uint16_t* __restrict__ vals_out)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;   // new row
    if (i >= d.M) return;
    const int64_t r = d.perm[i];
    const int64_t br = i >> 4;
    const int rr = static_cast<int>(i & 15);
    const int lo0 = d.row_ptr[br], hi0 = d.row_ptr[br + 1];
    int hint = lo0;
    for (int64_t p = csr_row_ptr[r]; p < csr_row_ptr[r + 1]; ++p) {
        const int c = csr_col_idx[p];
        const int bc = c >> 4;
        int lo = hint, hi = hi0;                     // columns ascend, so the slot never moves back
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (d.meta[2 * mid] < bc) lo = mid + 1; else hi = mid;
        }
        hint = lo;
        const int cc = c & 15;
        vals_out[static_cast<size_t>(lo) * 256 + static_cast<size_t>(((cc >> 3) * 16 + rr) * 8 + (cc & 7))] = csr_vals[p];
    }
}

int launch_bcsr_fill(const DeviceBcsr& d, const int64_t* csr_row_ptr, const int32_t* csr_col_idx,
                     const uint16_t* csr_vals, uint16_t* vals_out, void* stream)
{
    if (d.M == 0) return 0;
    const int threads = 256;
    const int blocks = static_cast<int>((d.M + threads - 1) / threads);
    hipLaunchKernelGGL(bcsr_fill_kernel, dim3(blocks), dim3(threads), 0, static_cast<hipStream_t>(stream),
                       d, csr_row_ptr, csr_col_idx, csr_vals, vals_out);
    return static_cast<int>(hipGetLastError());
}

// ---------------------------------------------------------------------------
// SpMM
// ---------------------------------------------------------------------------
//
// Work split: one workgroup of WAVES wavefronts per (block row, slab of 16*NT columns of
// B and C).  Wave w of the group takes block pairs w, w+WAVES, ... of the block row, so
// that the group as a whole streams the row's block values front to back; the partial
// 16 x (16*NT) tiles are summed through LDS in a fixed order and scattered to the rows
// perm[16*br + 0..15] of C.
//
// One MFMA 16x16x32 multiplies TWO stored blocks: k = 0..15 is the first block of the pair,
// k = 16..31 the second.  Lane l = 16*g + i supplies, as the left operand, row i of the
// pair's k range 8g..8g+7, which is the 16 bytes at offset 16*l of the pair in the
// two-half-panel layout.  The right operand wants, per lane, eight k-consecutive values of
// one column of B, while B is row-major (n-consecutive).  Instead of transposing through
// LDS, lane (g, i) loads from each of its eight B rows the NT consecutive columns
// n0 + NT*i .. n0 + NT*i + NT-1, and MFMA number t is defined to produce the column set
// { n0 + NT*i + t : i = 0..15 }.  The eight halves a lane feeds to MFMA t are then half t
// of its eight row loads (one byte-permute per two halves), and after the NT MFMAs the lane
// holds, for each of its four output rows 4g..4g+3, NT consecutive columns of C.
//
// B rows whose column in the block is empty (bit clear in the occupancy mask) are not
// fetched: their buffer-load offset is pushed out of range, which makes the hardware
// return zeros without touching memory.

constexpr uint32_t kOutOfRange = 0x80000000u;   // B must be smaller than 2 GiB on this path

template <int BYTES> struct BLoad;
template <> struct BLoad<2> {
    static __device__ __forceinline__ void ld(uint32_t* r, __amdgpu_buffer_rsrc_t s, uint32_t off)
    { r[0] = static_cast<uint16_t>(__builtin_amdgcn_raw_buffer_load_b16(s, off, 0, 0)); }
};
template <> struct BLoad<4> {
    static __device__ __forceinline__ void ld(uint32_t* r, __amdgpu_buffer_rsrc_t s, uint32_t off)
    { r[0] = static_cast<uint32_t>(__builtin_amdgcn_raw_buffer_load_b32(s, off, 0, 0)); }
};
template <> struct BLoad<8> {
    static __device__ __forceinline__ void ld(uint32_t* r, __amdgpu_buffer_rsrc_t s, uint32_t off)
    { i32x2 v = __builtin_amdgcn_raw_buffer_load_b64(s, off, 0, 0); r[0] = v[0]; r[1] = v[1]; }
};
template <> struct BLoad<16> {
    static __device__ __forceinline__ void ld(uint32_t* r, __amdgpu_buffer_rsrc_t s, uint32_t off)
    { i32x4 v = __builtin_amdgcn_raw_buffer_load_b128(s, off, 0, 0); r[0] = v[0]; r[1] = v[1]; r[2] = v[2]; r[3] = v[3]; }
};

template <bool BF16>
__device__ __forceinline__ f32x4 mfma_pair(u32x4 a, u32x4 b, f32x4 c)
{
    if constexpr (BF16)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

template <int NT, int WAVES, bool BF16>
__global__ __launch_bounds__(WAVES * 64)
void spmm_kernel(DeviceBcsr d, const void* __restrict__ B, uint32_t b_bytes, uint32_t ldb_bytes,
                 float* __restrict__ C, int64_t ldc, int N)
{
    constexpr int NW = 16 * NT;                    // columns per workgroup
    constexpr int ND = NT >= 2 ? NT / 2 : 1;       // dwords per B row load
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int i = lane & 15, g = lane >> 4;
    const int br = d.order[blockIdx.x];
    const int n0 = blockIdx.y * NW;
    const int start = d.row_ptr[br], end = d.row_ptr[br + 1];
    const int npairs = (end - start + 1) >> 1;
    const int col0 = n0 + NT * i;                  // first of this lane's NT columns
    const bool col_ok = col0 < N;                  // N is a multiple of NT on this path

    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(B), 0, static_cast<int>(b_bytes), 0x00020000);

    f32x4 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};

    for (int p = wave; p < npairs; p += WAVES) {
        const int blk = start + 2 * p + (g >> 1);
        const bool valid = blk < end;
        int bcol = 0;
        uint32_t mask = 0;
        u32x4 a = u32x4{0u, 0u, 0u, 0u};
        if (valid) {
            const i32x2 m = *reinterpret_cast<const i32x2*>(d.meta + 2 * static_cast<size_t>(blk));
            bcol = m[0];
            mask = static_cast<uint32_t>(m[1]);
            a = *reinterpret_cast<const u32x4*>(d.vals + static_cast<size_t>(blk) * 256 + ((g & 1) * 16 + i) * 8);
        }
        const uint32_t bits = col_ok ? ((mask >> (8 * (g & 1))) & 0xFFu) : 0u;
        const uint32_t row0 = static_cast<uint32_t>(bcol) * 16u + 8u * (g & 1);
        const uint32_t off0 = row0 * ldb_bytes + static_cast<uint32_t>(col0) * 2u;

        uint32_t R[8][ND];
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            const uint32_t off = ((bits >> kk) & 1u) ? off0 + kk * ldb_bytes : kOutOfRange;
            BLoad<2 * NT>::ld(R[kk], rsrc, off);
        }
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const uint32_t sel = (t & 1) ? 0x07060302u : 0x05040100u;
            u32x4 b;
#pragma unroll
            for (int q = 0; q < 4; ++q)
                b[q] = __builtin_amdgcn_perm(R[2 * q + 1][t >> 1], R[2 * q][t >> 1], sel);
            acc[t] = mfma_pair<BF16>(a, b, acc[t]);
        }
    }

    // acc[t][r] = C'[4g + r][n0 + NT*i + t]
    if constexpr (WAVES == 1) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int64_t out_row = d.perm[br * 16 + 4 * g + r];
            if (out_row < 0 || !col_ok) continue;
            float* dst = C + out_row * ldc + col0;
#pragma unroll
            for (int t = 0; t < NT; ++t) dst[t] = acc[t][r];
        }
    } else {
        __shared__ float red[WAVES][16][NW + 4];
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int t = 0; t < NT; ++t) red[wave][4 * g + r][NT * i + t] = acc[t][r];
        __syncthreads();
        for (int e = threadIdx.x; e < 16 * NW; e += WAVES * 64) {
            const int row = e / NW, c = e % NW;
            float s = red[0][row][c];
#pragma unroll
            for (int w = 1; w < WAVES; ++w) s += red[w][row][c];
            const int64_t out_row = d.perm[br * 16 + row];
            if (out_row >= 0 && n0 + c < N) C[out_row * ldc + n0 + c] = s;
        }
    }
}

template <int NT, int WAVES, bool BF16>
static int launch_variant(const DeviceBcsr& d, const void* B, int64_t ldb, float* C, int64_t ldc,
                          int64_t N, hipStream_t stream)
{
    const int64_t slabs = (N + 16 * NT - 1) / (16 * NT);
    dim3 grid(static_cast<unsigned>(d.nbr), static_cast<unsigned>(slabs));
    const uint32_t b_bytes = d.K > 0 ? static_cast<uint32_t>(((d.K - 1) * ldb + N) * 2) : 0u;
    hipLaunchKernelGGL((spmm_kernel<NT, WAVES, BF16>), grid, dim3(WAVES * 64), 0, stream,
                       d, B, b_bytes, static_cast<uint32_t>(ldb * 2), C, ldc, static_cast<int>(N));
    return static_cast<int>(hipGetLastError());
}

template <int NT, bool BF16>
static int launch_nt(const DeviceBcsr& d, const void* B, int64_t ldb, float* C, int64_t ldc,
                     int64_t N, hipStream_t stream, const char** variant)
{
    // short block rows: one wave per tile, no LDS reduction; long rows: split over four waves
    if (d.mean_row_blocks < 12.0 && d.max_row_blocks < 64) {
        *variant = BF16 ? "spmm_bf16_w1" : "spmm_f16_w1";
        return launch_variant<NT, 1, BF16>(d, B, ldb, C, ldc, N, stream);
    }
    *variant = BF16 ? "spmm_bf16_w4" : "spmm_f16_w4";
    return launch_variant<NT, 4, BF16>(d, B, ldb, C, ldc, N, stream);
}

template <bool BF16>
static int launch_dtype(const DeviceBcsr& d, const void* B, int64_t ldb, float* C, int64_t ldc,
                        int64_t N, hipStream_t stream, const char** variant)
{
    // widest B row load (2*NT bytes) that N, ldb and the base address allow
    const uintptr_t addr = reinterpret_cast<uintptr_t>(B);
    auto fits = [&](int nt) { return N % nt == 0 && ldb % nt == 0 && addr % (2 * nt) == 0; };
    if (fits(8)) return launch_nt<8, BF16>(d, B, ldb, C, ldc, N, stream, variant);
    if (fits(4)) return launch_nt<4, BF16>(d, B, ldb, C, ldc, N, stream, variant);
    if (fits(2)) return launch_nt<2, BF16>(d, B, ldb, C, ldc, N, stream, variant);
    return launch_nt<1, BF16>(d, B, ldb, C, ldc, N, stream, variant);
}

int launch_spmm(const DeviceBcsr& d, bool bf16, const void* B, int64_t ldb, float* C, int64_t ldc,
                int64_t N, void* stream, const char** variant)
{
    hipStream_t s = static_cast<hipStream_t>(stream);
    return bf16 ? launch_dtype<true>(d, B, ldb, C, ldc, N, s, variant)
                : launch_dtype<false>(d, B, ldb, C, ldc, N, s, variant);
}

}  // namespace smat
