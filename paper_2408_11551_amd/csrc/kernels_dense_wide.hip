// The 256-column tile of the block-dense SpMM path (kernels_dense.hip describes the path).
// A workgroup of four waves holds a 256 x 256 tile of C: 256 accumulator registers per lane,
// which only fit next to the operands when they live in the accumulation registers, so this
// file is compiled with the compiler's default placement of MFMA results while the 128-column
// tiles are compiled with results in ordinary VGPRs.  The wide tile fetches a third fewer
// bytes from the L2 per matrix instruction (per step 16 KiB of block values and 16 KiB of B
// for 64 instructions per wave instead of 16 + 8 for 32).
#include "dense_kernel.inc.h"

namespace smat {

void launch_dense_wide(const DeviceBcsr& d, const DenseTiles& t, bool bf16, const void* B, uint32_t b_bytes,
                       int64_t ldb, float* C, int64_t ldc, int64_t N, int vec_store, void* stream)
{
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (bf16) launch_dense_tile<true, 2, 2>(d, t, 1, B, b_bytes, ldb, C, ldc, N, vec_store, s);
    else launch_dense_tile<false, 2, 2>(d, t, 1, B, b_bytes, ldb, C, ldc, N, vec_store, s);
}

}  // namespace smat
