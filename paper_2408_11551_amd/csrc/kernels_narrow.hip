// Instantiations of the per-row SpMM kernel (spmm_rows.h) whose entry rows take the walk for
// N = 1, 2, 4, 8, 16 (walk_entries_narrow): fp16 and bf16, one or two packs per round, pieces of B
// of 2, 4, 8 or 16 bytes, one, two or four waves per block row.
#include "spmm_rows.h"

namespace smat {

template <int DT, int PK, int W>
static int launch_narrow_shape(const DeviceBcsr& d, const void* B, int64_t ldb, void* C, int64_t ldc,
                               int64_t N, hipStream_t stream, const char** variant)
{
    // Waves per block row as for the other variants (launch_shape), counted in rounds of PK packs.
    const double mean_rounds = d.mean_row_packs / PK;
    const double longest_us = static_cast<double>(d.max_row_packs) / PK * 0.25;
    const double stream_us = (static_cast<double>(d.stream_bytes) + static_cast<double>(d.M) * N * 4.0 +
                              static_cast<double>(d.K) * N * 2.0) / 5.0e6;
    const double gather_us = static_cast<double>(d.b_rows) * 64.0 / 20.0e6;
    const bool skewed = static_cast<double>(d.max_row_packs) > 2.0 * d.mean_row_packs;
    int kw = 1;
    while (kw < 4 && mean_rounds >= 4.0 * kw &&
           ((skewed && longest_us / kw > 0.5 * (stream_us + gather_us)) || d.n_order * kw < 4096)) kw *= 2;
    static thread_local char name[48];
    snprintf(name, sizeof(name), "spmm_%s_t%dw%dk%d", DT == kF16 ? "f16" : "bf16", PK == 2 ? 8 : 16, W, kw);
    *variant = name;
    if (kw == 4) return launch_variant<1, 4, 1, 1, 8, DT, 100 * PK + W>(d, B, ldb, C, ldc, N, stream);
    if (kw == 2) return launch_variant<1, 2, 1, 1, 8, DT, 100 * PK + W>(d, B, ldb, C, ldc, N, stream);
    return launch_variant<1, 1, 1, 1, 8, DT, 100 * PK + W>(d, B, ldb, C, ldc, N, stream);
}

template <int DT>
static int launch_narrow_dtype(const DeviceBcsr& d, const void* B, int64_t ldb, void* C, int64_t ldc,
                               int64_t N, hipStream_t stream, const char** variant)
{
    // One load per piece: the piece (all N columns, or eight of sixteen) is 2, 4, 8 or 16 bytes
    // and every row of B starts on a multiple of that.  Nothing past column N is read.
    const uintptr_t addr = reinterpret_cast<uintptr_t>(B);
    const int64_t piece = N == 16 ? 16 : 2 * N;
    if ((ldb * 2) % piece != 0 || addr % piece != 0) return kNotNarrow;
    switch (N) {
    case 1: return launch_narrow_shape<DT, 2, 2>(d, B, ldb, C, ldc, N, stream, variant);
    case 2: return launch_narrow_shape<DT, 2, 4>(d, B, ldb, C, ldc, N, stream, variant);
    case 4: return launch_narrow_shape<DT, 2, 8>(d, B, ldb, C, ldc, N, stream, variant);
    case 8: return launch_narrow_shape<DT, 2, 16>(d, B, ldb, C, ldc, N, stream, variant);
    case 16: return launch_narrow_shape<DT, 1, 16>(d, B, ldb, C, ldc, N, stream, variant);
    default: return kNotNarrow;
    }
}

int launch_spmm_narrow(const DeviceBcsr& d, int dtype, const void* B, int64_t ldb, void* C, int64_t ldc,
                       int64_t N, void* stream, const char** variant)
{
    if (N < 1 || N > 16 || d.max_class != kEntryClass || d.n_order == 0) return kNotNarrow;
    // A row's first result takes one more trip through LDS here than in the general walk, which
    // a small launch (one or two rounds per wave, the chip not full) feels: 6.5 against 4.8 us at
    // 8.9 k packs; from 35 k packs on this walk is the faster one (10.0 against 13.1 us).
    if (d.n_packs < 24576) return kNotNarrow;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (dtype == kF16) return launch_narrow_dtype<kF16>(d, B, ldb, C, ldc, N, s, variant);
    if (dtype == kBF16) return launch_narrow_dtype<kBF16>(d, B, ldb, C, ldc, N, s, variant);
    return kNotNarrow;
}

}  // namespace smat
