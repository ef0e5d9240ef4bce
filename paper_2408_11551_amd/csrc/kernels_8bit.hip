// Instantiations of the per-row SpMM kernel (spmm_rows.h) for the 8-bit operand types of the
// gfx950 matrix units: the two 8-bit floating-point formats (fp32 accumulation, C in fp32) and
// int8 (int32 accumulation, C in int32).  With the macro SMAT_8BIT_DT (the number of one type in
// smat_dtype_t: 2, 3 or 4) the file yields that type only; the build compiles it once per type
// so that the three sets of kernels build side by side.  Without the macro it yields all three.
#include "spmm_rows.h"

namespace smat {

#define SMAT_8BIT_ENTRY(NAME, DT)                                                                       \
    int NAME(const DeviceBcsr& d, const void* B, int64_t ldb, void* C, int64_t ldc, int64_t N,          \
             void* stream, const char** variant)                                                        \
    {                                                                                                   \
        return launch_dtype<DT>(d, B, ldb, C, ldc, N, static_cast<hipStream_t>(stream), variant);       \
    }

#if !defined(SMAT_8BIT_DT) || SMAT_8BIT_DT == 2
SMAT_8BIT_ENTRY(launch_spmm_e4m3, kE4M3)
#endif
#if !defined(SMAT_8BIT_DT) || SMAT_8BIT_DT == 3
SMAT_8BIT_ENTRY(launch_spmm_e5m2, kE5M2)
#endif
#if !defined(SMAT_8BIT_DT) || SMAT_8BIT_DT == 4
SMAT_8BIT_ENTRY(launch_spmm_i8, kI8)
#endif

}  // namespace smat
