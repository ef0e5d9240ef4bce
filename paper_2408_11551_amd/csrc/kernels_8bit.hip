// Instantiations of the per-row SpMM kernel (spmm_rows.h) for the 8-bit operand types of the
// gfx950 matrix units: the two 8-bit floating-point formats (fp32 accumulation, C in fp32) and
// int8 (int32 accumulation, C in int32).
#include "spmm_rows.h"

namespace smat {

int launch_spmm_8bit(const DeviceBcsr& d, int dtype, const void* B, int64_t ldb, void* C, int64_t ldc,
                     int64_t N, void* stream, const char** variant)
{
    hipStream_t s = static_cast<hipStream_t>(stream);
    switch (dtype) {
    case kE4M3: return launch_dtype<kE4M3>(d, B, ldb, C, ldc, N, s, variant);
    case kE5M2: return launch_dtype<kE5M2>(d, B, ldb, C, ldc, N, s, variant);
    case kI8: return launch_dtype<kI8>(d, B, ldb, C, ldc, N, s, variant);
    default: return static_cast<int>(hipErrorInvalidValue);
    }
}

}  // namespace smat
