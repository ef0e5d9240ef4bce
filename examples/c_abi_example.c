/*
 * The library used from plain C, with no Python and no PyTorch in the process: device memory comes
 * from hipMalloc, everything else goes through include/smat.h.
 *
 *   gcc -std=c11 -O2 -D__HIP_PLATFORM_AMD__ examples/c_abi_example.c -Iinclude -I/opt/rocm/include \
 *       -Lpaper_2408_11551_amd -lsmat -L/opt/rocm/lib -lamdhip64 -Wl,-rpath,'$ORIGIN' -Wl,-rpath,/opt/rocm/lib \
 *       -o paper_2408_11551_amd/c_abi_example            (paper_2408_11551_amd/build.py does this)
 *   paper_2408_11551_amd/c_abi_example [M K N nnz_per_row]
 *
 * Builds a random CSR matrix with small integer values (exact in fp16 and in fp32 sums), multiplies
 * it by a small-integer B on the GPU and compares every element of C with a plain loop on the host.
 * Prints "OK" and exits 0 when they are equal.
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "smat.h"

#define CHECK_HIP(call)                                                                       \
    do {                                                                                      \
        hipError_t e_ = (call);                                                               \
        if (e_ != hipSuccess) {                                                               \
            fprintf(stderr, "%s: %s\n", #call, hipGetErrorString(e_));                        \
            return 2;                                                                         \
        }                                                                                     \
    } while (0)
#define CHECK_SMAT(call)                                                                      \
    do {                                                                                      \
        smat_status_t s_ = (call);                                                            \
        if (s_ != SMAT_OK) {                                                                  \
            fprintf(stderr, "%s: status %d: %s\n", #call, (int)s_, smat_last_error());        \
            return 3;                                                                         \
        }                                                                                     \
    } while (0)

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t next_u32(void)
{
    rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
    return (uint32_t)(rng_state >> 33);
}

/* fp16 bit pattern of a small integer -8 .. 8 (exactly representable) */
static uint16_t half_of_small_int(int v)
{
    uint16_t sign = 0;
    int e = 0;
    if (v == 0) return 0;
    if (v < 0) { sign = 0x8000u; v = -v; }
    while ((v >> (e + 1)) != 0) ++e;                        /* v = 1.m * 2^e */
    return (uint16_t)(sign | (uint16_t)((e + 15) << 10) | (uint16_t)(((v << (10 - e)) & 0x3FF)));
}

static int cmp_i32(const void* a, const void* b)
{
    const int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
    return (x > y) - (x < y);
}

int main(int argc, char** argv)
{
    const int64_t M = argc > 1 ? atoll(argv[1]) : 1000;
    const int64_t K = argc > 2 ? atoll(argv[2]) : 777;
    const int64_t N = argc > 3 ? atoll(argv[3]) : 40;
    const int per_row = argc > 4 ? atoi(argv[4]) : 9;
    if (M < 1 || K < per_row || N < 1 || per_row < 1) { fprintf(stderr, "bad sizes\n"); return 1; }

    /* CSR with per_row distinct ascending columns in every row, values -4 .. 4 without 0 */
    int64_t* row_ptr = (int64_t*)malloc((size_t)(M + 1) * sizeof(int64_t));
    int32_t* col_idx = (int32_t*)malloc((size_t)M * per_row * sizeof(int32_t));
    uint16_t* a_bits = (uint16_t*)malloc((size_t)M * per_row * sizeof(uint16_t));
    int* a_int = (int*)malloc((size_t)M * per_row * sizeof(int));
    for (int64_t r = 0; r <= M; ++r) row_ptr[r] = r * per_row;
    for (int64_t r = 0; r < M; ++r) {
        int32_t* c = col_idx + r * per_row;
        int have = 0;
        while (have < per_row) {
            const int32_t cand = (int32_t)(next_u32() % (uint32_t)K);
            int dup = 0;
            for (int j = 0; j < have; ++j) dup |= c[j] == cand;
            if (!dup) c[have++] = cand;
        }
        qsort(c, (size_t)per_row, sizeof(int32_t), cmp_i32);
        for (int j = 0; j < per_row; ++j) {
            int v = (int)(next_u32() % 4u) + 1;
            if (next_u32() & 1u) v = -v;
            a_int[r * per_row + j] = v;
            a_bits[r * per_row + j] = half_of_small_int(v);
        }
    }
    int* b_int = (int*)malloc((size_t)K * N * sizeof(int));
    uint16_t* b_bits = (uint16_t*)malloc((size_t)K * N * sizeof(uint16_t));
    for (int64_t i = 0; i < K * N; ++i) {
        b_int[i] = (int)(next_u32() % 9u) - 4;
        b_bits[i] = half_of_small_int(b_int[i]);
    }

    /* preprocess on the host, bind to device memory of our own, multiply */
    smat_handle_t* h = NULL;
    CHECK_SMAT(smat_preprocess(M, K, row_ptr, col_idx, a_bits, SMAT_F16, NULL, &h));
    int64_t nbr = 0, n_blocks = 0, n_packs = 0;
    CHECK_SMAT(smat_get_info(h, &nbr, &n_blocks, NULL, NULL));
    CHECK_SMAT(smat_get_layout_info(h, &n_packs, NULL, NULL, NULL));
    size_t ws_bytes = 0;
    CHECK_SMAT(smat_device_bytes(h, &ws_bytes));
    void *ws = NULL, *dB = NULL, *dC = NULL;
    hipStream_t stream;
    CHECK_HIP(hipStreamCreate(&stream));
    CHECK_HIP(hipMalloc(&ws, ws_bytes));
    CHECK_HIP(hipMalloc(&dB, (size_t)K * N * 2));
    CHECK_HIP(hipMalloc(&dC, (size_t)M * N * 4));
    CHECK_HIP(hipMemcpy(dB, b_bits, (size_t)K * N * 2, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemset(dC, 0xFF, (size_t)M * N * 4));
    CHECK_SMAT(smat_bind_device(h, ws, ws_bytes, stream));
    CHECK_SMAT(smat_spmm(h, dB, N, dC, N, N, stream));
    CHECK_HIP(hipStreamSynchronize(stream));
    float* c = (float*)malloc((size_t)M * N * sizeof(float));
    CHECK_HIP(hipMemcpy(c, dC, (size_t)M * N * 4, hipMemcpyDeviceToHost));

    /* the definition, in integers */
    int64_t wrong = 0;
    for (int64_t r = 0; r < M; ++r)
        for (int64_t n = 0; n < N; ++n) {
            long sum = 0;
            for (int j = 0; j < per_row; ++j) sum += (long)a_int[r * per_row + j] * b_int[(int64_t)col_idx[r * per_row + j] * N + n];
            if (c[r * N + n] != (float)sum) ++wrong;
        }
    printf("M=%lld K=%lld N=%lld nnz=%lld blocks=%lld packs=%lld kernel=%s wrong=%lld\n", (long long)M, (long long)K,
           (long long)N, (long long)(M * per_row), (long long)n_blocks, (long long)n_packs, smat_last_kernel(), (long long)wrong);
    smat_destroy(h);
    CHECK_HIP(hipFree(ws));
    CHECK_HIP(hipFree(dB));
    CHECK_HIP(hipFree(dC));
    CHECK_HIP(hipStreamDestroy(stream));
    free(row_ptr); free(col_idx); free(a_bits); free(a_int); free(b_int); free(b_bits); free(c);
    if (wrong) { printf("MISMATCH\n"); return 4; }
    printf("OK\n");
    return 0;
}
