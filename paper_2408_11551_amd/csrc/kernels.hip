// HIP kernels for gfx950 (CDNA4, wave64): device-side BCSR value fill and the 16-bit
// instantiations (fp16, bf16) of the per-row SpMM kernel (spmm_rows.h); the 8-bit ones are
// in kernels_8bit.hip.
#include "spmm_rows.h"

namespace smat {

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
// its slot in the block's pack (pack_layout.h); in an entry row the value goes to the slot with
// the entry's number instead.  The CSR values arrive as 16-bit words; T is the stored element
// (the 8-bit types keep the low byte).
template <typename T>
__global__ void bcsr_fill_kernel(DeviceBcsr d, const int64_t* __restrict__ csr_row_ptr,
                                 const int32_t* __restrict__ csr_col_idx,
                                 const uint16_t* __restrict__ csr_vals, T* __restrict__ vals_out)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;   // new row
    if (i >= d.M) return;
    const int64_t r = d.perm[i];
    const int64_t br = i >> 4;
    const int rr = static_cast<int>(i & 15);
    const int lo0 = d.blk_ptr[br], hi0 = d.blk_ptr[br + 1];
    const int npacks = d.pack_ptr[br + 1] - d.pack_ptr[br];
    if (npacks == 0) return;
    const int cls = d.row_class[br];
    T* row_vals = vals_out + static_cast<size_t>(d.vals_off[br]) * (64 / sizeof(T));
    if (cls == kEntryClass) {
        // entry row: the entries of the block row are numbered by column, then by row; an
        // entry's number is the count of those before it, row by row of the block row
        const int64_t j0 = br << 4, j1 = (j0 + 16 < d.M) ? j0 + 16 : d.M;
        for (int64_t p = csr_row_ptr[r]; p < csr_row_ptr[r + 1]; ++p) {
            const int c = csr_col_idx[p];
            int64_t e = 0;
            for (int64_t j = j0; j < j1; ++j) {
                const int64_t rj = d.perm[j];
                const int64_t first = csr_row_ptr[rj];
                const int below = j < i ? c + 1 : c;       // columns that come before (c, this row) in row j
                int64_t lo = first, hi = csr_row_ptr[rj + 1];
                while (lo < hi) {
                    const int64_t mid = (lo + hi) >> 1;
                    if (csr_col_idx[mid] < below) lo = mid + 1; else hi = mid;
                }
                e += lo - first;
            }
            const int rank = static_cast<int>(e & 31);
            row_vals[static_cast<size_t>(e >> 5) * (64 / sizeof(T)) + entry_elem_index(slot_group(rank), slot_pos(rank))] =
                static_cast<T>(csr_vals[p]);
        }
        return;
    }
    const int L = 2 << cls;
    int hint = lo0;
    for (int64_t p = csr_row_ptr[r]; p < csr_row_ptr[r + 1]; ++p) {
        const int c = csr_col_idx[p];
        const int bc = c >> 4;
        int lo = hint, hi = hi0;                     // columns ascend, so the block never moves back
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (d.blk_col[mid] < bc) lo = mid + 1; else hi = mid;
        }
        hint = lo;
        const uint32_t meta = d.blk_meta[lo];
        const int rank = static_cast<int>(meta >> 16) + __popc(meta & 0xFFFFu & ((1u << (c & 15)) - 1u));
        row_vals[static_cast<size_t>(d.blk_pack[lo]) * pack_elems(L) + pack_elem_index(L, rr, slot_group(rank), slot_pos(rank))] =
            static_cast<T>(csr_vals[p]);
    }
}

int launch_bcsr_fill(const DeviceBcsr& d, const int64_t* csr_row_ptr, const int32_t* csr_col_idx,
                     const uint16_t* csr_vals, void* vals_out, int elem_bytes, void* stream)
{
    if (d.M == 0) return 0;
    const int threads = 256;
    const int blocks = static_cast<int>((d.M + threads - 1) / threads);
    if (elem_bytes == 1)
        hipLaunchKernelGGL(bcsr_fill_kernel<uint8_t>, dim3(blocks), dim3(threads), 0, static_cast<hipStream_t>(stream),
                           d, csr_row_ptr, csr_col_idx, csr_vals, static_cast<uint8_t*>(vals_out));
    else
        hipLaunchKernelGGL(bcsr_fill_kernel<uint16_t>, dim3(blocks), dim3(threads), 0, static_cast<hipStream_t>(stream),
                           d, csr_row_ptr, csr_col_idx, csr_vals, static_cast<uint16_t*>(vals_out));
    return static_cast<int>(hipGetLastError());
}

int launch_spmm(const DeviceBcsr& d, int dtype, const void* B, int64_t ldb, void* C, int64_t ldc,
                int64_t N, void* stream, const char** variant)
{
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int narrow = launch_spmm_narrow(d, dtype, B, ldb, C, ldc, N, stream, variant);
    if (narrow != kNotNarrow) return narrow;
    switch (dtype) {
    case kF16: return launch_dtype<kF16>(d, B, ldb, C, ldc, N, s, variant);
    case kBF16: return launch_dtype<kBF16>(d, B, ldb, C, ldc, N, s, variant);
    case kE4M3: return launch_spmm_e4m3(d, B, ldb, C, ldc, N, stream, variant);
    case kE5M2: return launch_spmm_e5m2(d, B, ldb, C, ldc, N, stream, variant);
    case kI8: return launch_spmm_i8(d, B, ldb, C, ldc, N, stream, variant);
    default: return static_cast<int>(hipErrorInvalidValue);
    }
}

}  // namespace smat
