// Five small kernels that measure what this GPU delivers for the access patterns the SpMM
// kernels consist of, so that the figures quoted next to the rooflines can be reproduced:
// a streaming read, two random gathers of rows (the ways rows of B are fetched), a
// register-resident MFMA loop, and the step of the tile kernel put together piece by piece.  They compute nothing of the method.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <type_traits>

#include "../../include/smat_bench.h"

namespace {

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void lds_void;

// every thread reads eight 16-byte words per pass; a wave covers eight contiguous KiB
__global__ __launch_bounds__(256) void probe_read_kernel(const u32x4* __restrict__ src, size_t n16, uint32_t* sink)
{
    const size_t wave = (static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x) >> 6;
    const size_t nwaves = (static_cast<size_t>(gridDim.x) * blockDim.x) >> 6;
    const int lane = threadIdx.x & 63;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (size_t base = wave * 512; base + 512 <= n16; base += nwaves * 512) {
        u32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = src[base + u * 64 + lane];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u];
    }
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x12345678u) sink[0] = 1u;   // never true for the probe's data; keeps the loads
}

// Every wave reads the same window of `chunks` x 8 KiB once, beginning at a chunk of its own and wrapping
// round: the window stays in every XCD's L2 (if it is small enough) while a compute unit's waves, each at
// another place of it, get nothing out of the 32 KiB L1 -- what the L2s deliver to the L1s for plain
// 16-byte loads of whole lines.
__global__ __launch_bounds__(256) void probe_read_window_kernel(const u32x4* __restrict__ src, uint32_t chunks, uint32_t* sink)
{
    const uint32_t wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    u32x4 acc = {0u, 0u, 0u, 0u};
    uint32_t at = (wave * 37u) % chunks;
    for (uint32_t c = 0; c < chunks; ++c) {
        const u32x4* from = src + static_cast<size_t>(at) * 512;
        u32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = from[u * 64 + lane];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u];
        at = at + 1 == chunks ? 0u : at + 1;
    }
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x12345678u) sink[0] = 1u;
}

// One wave per workgroup walks `packs` groups of 32 row numbers; lane (g, i) loads VEC bytes at
// offset VEC * i of rows idx[8 g + kk], kk = 0..7 -- eight loads in flight per group, four rows
// per load, as in the SpMM kernel with VEC / 2 columns per lane.
template <int VEC>
__global__ __launch_bounds__(64) void probe_gather_kernel(const unsigned char* __restrict__ table, uint32_t row_bytes,
                                                          const uint32_t* __restrict__ idx, int packs, uint32_t* sink)
{
    const int lane = threadIdx.x, g = lane >> 4, i = lane & 15;
    const uint32_t* my = idx + static_cast<size_t>(blockIdx.x) * packs * 32;
    uint32_t acc = 0u;
    for (int p = 0; p < packs; ++p) {
        uint32_t v[8][VEC / 4];
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            const unsigned char* at = table + static_cast<size_t>(my[p * 32 + 8 * g + kk]) * row_bytes + VEC * i;
            if constexpr (VEC == 8) { const u32x2 t = *reinterpret_cast<const u32x2*>(at); v[kk][0] = t[0]; v[kk][1] = t[1]; }
            else { const u32x4 t = *reinterpret_cast<const u32x4*>(at); v[kk][0] = t[0]; v[kk][1] = t[1]; v[kk][2] = t[2]; v[kk][3] = t[3]; }
        }
#pragma unroll
        for (int kk = 0; kk < 8; ++kk)
#pragma unroll
            for (int x = 0; x < VEC / 4; ++x) acc ^= v[kk][x];
    }
    if (acc == 0x12345678u) sink[0] = 1u;
}

// One wave per workgroup; every lane fetches per_lane pieces of VEC bytes, piece x of lane l from
// the start of row idx[(wave * per_lane + x) * 64 + l], four loads in flight per lane.
template <int VEC>
__global__ __launch_bounds__(64) void probe_pieces_kernel(const unsigned char* __restrict__ table, uint32_t row_bytes,
                                                          const uint32_t* __restrict__ idx, int per_lane, uint32_t* sink)
{
    const uint32_t* my = idx + static_cast<size_t>(blockIdx.x) * per_lane * 64 + threadIdx.x;
    uint32_t acc = 0u;
    for (int x = 0; x < per_lane; x += 4) {
        uint32_t v[4][VEC >= 4 ? VEC / 4 : 1];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const unsigned char* at = table + static_cast<size_t>(my[(x + u) * 64]) * row_bytes;
            if constexpr (VEC == 2) v[u][0] = *reinterpret_cast<const uint16_t*>(at);
            else if constexpr (VEC == 4) v[u][0] = *reinterpret_cast<const uint32_t*>(at);
            else if constexpr (VEC == 8) { const u32x2 t = *reinterpret_cast<const u32x2*>(at); v[u][0] = t[0]; v[u][1] = t[1]; }
            else { const u32x4 t = *reinterpret_cast<const u32x4*>(at); v[u][0] = t[0]; v[u][1] = t[1]; v[u][2] = t[2]; v[u][3] = t[3]; }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int y = 0; y < (VEC >= 4 ? VEC / 4 : 1); ++y) acc ^= v[u][y];
    }
    if ((acc & 0xFFFFu) == 0x5678u) sink[0] = 1u;              // never true for the probe's data; keeps the loads
}

// 16 independent accumulators per wave, operands in registers: nothing but MFMA 16x16x32
__global__ __launch_bounds__(256) void probe_mfma_kernel(int iters, float* sink)
{
    f32x4 acc[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) acc[k] = f32x4{0.f, 0.f, 0.f, 0.f};
    f16x8 a, b;
#pragma unroll
    for (int k = 0; k < 8; ++k) { a[k] = static_cast<_Float16>(threadIdx.x & 3); b[k] = static_cast<_Float16>(k & 1); }
    for (int it = 0; it < iters; ++it)
#pragma unroll
        for (int k = 0; k < 16; ++k) acc[k] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, acc[k], 0, 0, 0);
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < 16; ++k) s += acc[k][0];
    if (s == -1.f) sink[0] = s;
}

// The step of the tile kernel (kernels_dense.hip, 16-bit operands) on data that never leaves the L1: two
// groups of four waves, per wave and step 32 MFMA 16x16x32 (four block rows x eight groups of 16
// columns) whose right operands are built with four byte permutes each.  PARTS adds the rest of a
// step bit by bit: 1 = the four 1 KiB loads of block values into a register ring of three, 2 = the
// eight 16-byte LDS reads of the panel, 4 = the barrier, 8 = the two 1 KiB loads straight into LDS,
// 16 = all loads of a step issued together behind the barrier instead of one after each group of
// matrix instructions, 32 = the right operands by transposing LDS reads, two per group of sixteen
// columns and one group ahead, instead of the eight reads of the panel and the permutes (as the
// kernel does now; replaces part 2).  The rate it reaches says what the structure of the step costs when memory
// costs nothing.
template <int OFFSET>
__device__ __forceinline__ u32x4 probe_lds_read16(uint32_t addr)
{
    u32x4 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFFSET));
    return v;
}
__device__ __forceinline__ void probe_lds_reads_done(u32x4 (&R)[8])
{
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(R[0]), "+v"(R[1]), "+v"(R[2]), "+v"(R[3]), "+v"(R[4]), "+v"(R[5]), "+v"(R[6]), "+v"(R[7]));
}
template <int OFFSET>
__device__ __forceinline__ u32x2 probe_lds_read_tr(uint32_t addr)
{
    u32x2 v;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFFSET));
    return v;
}
template <int YOUNGER>
__device__ __forceinline__ void probe_lds_pair_done(u32x2& lo, u32x2& hi)
{
    asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(lo), "+v"(hi) : "n"(YOUNGER));
}
__device__ __forceinline__ u32x4 probe_ld16(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff)
{
    const i32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 0);
    return u32x4{static_cast<uint32_t>(v[0]), static_cast<uint32_t>(v[1]), static_cast<uint32_t>(v[2]), static_cast<uint32_t>(v[3])};
}

constexpr uint32_t kTileStepBytes = 1u << 20;      // what the probe reads from (all of it stays in the L1/L2)

template <int PARTS>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2)))
void probe_tile_step_kernel(int steps, const u32x4* __restrict__ src, float* sink)
{
    __shared__ u32x4 lds[2 * 3 * 512];             // per group a ring of three 8 KiB panels
    const int lane = threadIdx.x & 63, wave = (threadIdx.x >> 6) & 3, kg = threadIdx.x >> 8;
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<u32x4*>(src), 0, static_cast<int>(kTileStepBytes), 0x00020000);
    for (int k = threadIdx.x; k < 2 * 3 * 512; k += 512) lds[k] = u32x4{0u, 0u, 0u, 0u};
    __syncthreads();
    const uint32_t lds_base =
        static_cast<uint32_t>(reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) const char*)lds)) + kg * 3 * 8192;
    const uint32_t rd = lds_base + (lane >> 4) * 2048 + (lane & 15) * 16;
    uint32_t tr[8];                                // transposing reads: where lane (g, j) reads for column group x
    {
        const int g = lane >> 4, j = lane & 15, e = j >> 2, q = j & 3;
        for (int x = 0; x < 8; ++x) tr[x] = lds_base + (8 * g + e) * 256 + 32 * (x ^ e ^ (4 * (g & 1))) + 16 * (q >> 1) + 8 * (q & 1);
    }
    u32x4 a[3][4];
    for (int u = 0; u < 3; ++u)
        for (int r = 0; r < 4; ++r) a[u][r] = probe_ld16(rs, lane * 16, (wave * 4 + r) * 1024);
    u32x4 fixed[8];
    for (int k = 0; k < 8; ++k) fixed[k] = probe_ld16(rs, lane * 16, 16384 + k * 1024);
    f32x4 acc[4][8];
    for (int r = 0; r < 4; ++r)
        for (int x = 0; x < 8; ++x) acc[r][x] = f32x4{0.f, 0.f, 0.f, 0.f};
    auto step = [&](auto uc, int s) {
        constexpr int u = decltype(uc)::value;
        // the loads of this step's data were issued two steps ago: all but the youngest step's have to be back
        if constexpr ((PARTS & 9) == 9) asm volatile("s_waitcnt vmcnt(6)");
        else if constexpr (PARTS & 8) asm volatile("s_waitcnt vmcnt(2)");
        else if constexpr (PARTS & 1) asm volatile("s_waitcnt vmcnt(4)");
        if constexpr (PARTS & 4) __builtin_amdgcn_s_barrier();
        const uint32_t soff = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(((s & 7) * 16 + wave * 4) * 1024));
        auto issue = [&](int x) {
            if constexpr (PARTS & 8)
                if (x < 2)
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_void*)(uintptr_t)(lds_base + ((u + 2) % 3) * 8192 + x * 4096 + wave * 1024),
                                                             16, lane * 16, 32768 + wave * 1024 + x * 4096, 0, 0);
            if constexpr (PARTS & 1)
                if (x >= 2 && x < 6) a[(u + 2) % 3][x - 2] = probe_ld16(rs, lane * 16, soff + (x - 2) * 1024);
        };
        if constexpr (PARTS & 32) {
            u32x2 lo[2], hi[2];
            lo[0] = probe_lds_read_tr<8192 * u>(tr[0]);
            hi[0] = probe_lds_read_tr<8192 * u + 1024>(tr[0]);
#pragma unroll
            for (int x = 0; x < 8; ++x) {
                if (x < 7) {
                    lo[(x + 1) & 1] = probe_lds_read_tr<8192 * u>(tr[(x + 1) & 7]);
                    hi[(x + 1) & 1] = probe_lds_read_tr<8192 * u + 1024>(tr[(x + 1) & 7]);
                    probe_lds_pair_done<2>(lo[x & 1], hi[x & 1]);
                } else {
                    probe_lds_pair_done<0>(lo[x & 1], hi[x & 1]);
                }
                const u32x4 b = u32x4{lo[x & 1][0], lo[x & 1][1], hi[x & 1][0], hi[x & 1][1]};
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    acc[r][x] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a[u][r]), __builtin_bit_cast(bf16x8, b), acc[r][x], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (x < 6) issue(x);
                __builtin_amdgcn_sched_barrier(0);
            }
            return;
        }
        u32x4 R[8];
        if constexpr (PARTS & 2) {
            const uint32_t p = rd + u * 8192;
            R[0] = probe_lds_read16<0>(p); R[1] = probe_lds_read16<256>(p); R[2] = probe_lds_read16<512>(p); R[3] = probe_lds_read16<768>(p);
            R[4] = probe_lds_read16<1024>(p); R[5] = probe_lds_read16<1280>(p); R[6] = probe_lds_read16<1536>(p); R[7] = probe_lds_read16<1792>(p);
            probe_lds_reads_done(R);
        } else {
#pragma unroll
            for (int k = 0; k < 8; ++k) R[k] = fixed[k];
        }
        if constexpr (PARTS & 16) {
            for (int x = 0; x < 6; ++x) issue(x);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int x = 0; x < 8; ++x) {
            const uint32_t pick = (x & 1) ? 0x07060302u : 0x05040100u;
            u32x4 b;
#pragma unroll
            for (int q = 0; q < 4; ++q) b[q] = __builtin_amdgcn_perm(R[2 * q + 1][x >> 1], R[2 * q][x >> 1], pick);
#pragma unroll
            for (int r = 0; r < 4; ++r)
                acc[r][x] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a[u][r]), __builtin_bit_cast(bf16x8, b), acc[r][x], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (!(PARTS & 16)) {
                if (x < 6) issue(x);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };
    for (int s = 0; s < steps; s += 3) {           // every wave runs the same number of steps: the barriers match
        step(std::integral_constant<int, 0>{}, s);
        step(std::integral_constant<int, 1>{}, s + 1);
        step(std::integral_constant<int, 2>{}, s + 2);
    }
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)");
    float sum = 0.f;
    for (int r = 0; r < 4; ++r)
        for (int x = 0; x < 8; ++x) sum += acc[r][x][0] + acc[r][x][3];
    if (sum == -1.2345f) sink[0] = sum;
}

}  // namespace

extern "C" {

smat_status_t smat_probe_read(const void* dev_buf, size_t bytes, void* dev_sink, void* stream)
{
    if (!dev_buf || !dev_sink || bytes < 8192) return SMAT_ERR_INVALID_ARG;
    hipLaunchKernelGGL(probe_read_kernel, dim3(4096), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const u32x4*>(dev_buf), bytes / 16, static_cast<uint32_t*>(dev_sink));
    return hipGetLastError() == hipSuccess ? SMAT_OK : SMAT_ERR_HIP;
}

smat_status_t smat_probe_read_window(const void* dev_buf, size_t window_bytes, int waves, void* dev_sink, void* stream)
{
    if (!dev_buf || !dev_sink || window_bytes < 8192 || window_bytes % 8192 != 0 || window_bytes > (size_t{1} << 30) ||
        waves < 4 || waves % 4 != 0)
        return SMAT_ERR_INVALID_ARG;
    hipLaunchKernelGGL(probe_read_window_kernel, dim3(static_cast<unsigned>(waves / 4)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const u32x4*>(dev_buf), static_cast<uint32_t>(window_bytes / 8192), static_cast<uint32_t*>(dev_sink));
    return hipGetLastError() == hipSuccess ? SMAT_OK : SMAT_ERR_HIP;
}

smat_status_t smat_probe_gather(const void* dev_table, uint32_t row_bytes, const uint32_t* dev_idx, int waves, int packs,
                                int bytes_per_lane, void* dev_sink, void* stream)
{
    if (!dev_table || !dev_idx || !dev_sink || waves <= 0 || packs <= 0) return SMAT_ERR_INVALID_ARG;
    if ((bytes_per_lane != 8 && bytes_per_lane != 16) || row_bytes < 16u * static_cast<uint32_t>(bytes_per_lane))
        return SMAT_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (bytes_per_lane == 8)
        hipLaunchKernelGGL(probe_gather_kernel<8>, dim3(waves), dim3(64), 0, s, static_cast<const unsigned char*>(dev_table),
                           row_bytes, dev_idx, packs, static_cast<uint32_t*>(dev_sink));
    else
        hipLaunchKernelGGL(probe_gather_kernel<16>, dim3(waves), dim3(64), 0, s, static_cast<const unsigned char*>(dev_table),
                           row_bytes, dev_idx, packs, static_cast<uint32_t*>(dev_sink));
    return hipGetLastError() == hipSuccess ? SMAT_OK : SMAT_ERR_HIP;
}

smat_status_t smat_probe_pieces(const void* dev_table, uint32_t row_bytes, const uint32_t* dev_idx, int waves, int per_lane,
                                int bytes_per_lane, void* dev_sink, void* stream)
{
    if (!dev_table || !dev_idx || !dev_sink || waves <= 0 || per_lane <= 0 || per_lane % 4 != 0) return SMAT_ERR_INVALID_ARG;
    const int v = bytes_per_lane;
    if ((v != 2 && v != 4 && v != 8 && v != 16) || row_bytes < static_cast<uint32_t>(v) || row_bytes % static_cast<uint32_t>(v) != 0)
        return SMAT_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const unsigned char* table = static_cast<const unsigned char*>(dev_table);
    uint32_t* sink = static_cast<uint32_t*>(dev_sink);
    if (v == 2) hipLaunchKernelGGL(probe_pieces_kernel<2>, dim3(waves), dim3(64), 0, s, table, row_bytes, dev_idx, per_lane, sink);
    else if (v == 4) hipLaunchKernelGGL(probe_pieces_kernel<4>, dim3(waves), dim3(64), 0, s, table, row_bytes, dev_idx, per_lane, sink);
    else if (v == 8) hipLaunchKernelGGL(probe_pieces_kernel<8>, dim3(waves), dim3(64), 0, s, table, row_bytes, dev_idx, per_lane, sink);
    else hipLaunchKernelGGL(probe_pieces_kernel<16>, dim3(waves), dim3(64), 0, s, table, row_bytes, dev_idx, per_lane, sink);
    return hipGetLastError() == hipSuccess ? SMAT_OK : SMAT_ERR_HIP;
}

smat_status_t smat_probe_tile_step(int workgroups, int steps, int parts, const void* dev_buf, size_t bytes, void* dev_sink,
                                   void* stream)
{
    if (workgroups <= 0 || steps <= 0 || steps % 3 != 0 || !dev_buf || !dev_sink || bytes < kTileStepBytes)
        return SMAT_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const u32x4* src = static_cast<const u32x4*>(dev_buf);
    float* sink = static_cast<float*>(dev_sink);
#define SMAT_TILE_STEP(P) \
    case P: hipLaunchKernelGGL(probe_tile_step_kernel<P>, dim3(workgroups), dim3(512), 0, s, steps, src, sink); break
    switch (parts) {
    SMAT_TILE_STEP(0); SMAT_TILE_STEP(1); SMAT_TILE_STEP(2); SMAT_TILE_STEP(3); SMAT_TILE_STEP(6); SMAT_TILE_STEP(7);
    SMAT_TILE_STEP(12); SMAT_TILE_STEP(14); SMAT_TILE_STEP(15); SMAT_TILE_STEP(31);
    SMAT_TILE_STEP(32); SMAT_TILE_STEP(36); SMAT_TILE_STEP(37); SMAT_TILE_STEP(45);
    default: return SMAT_ERR_INVALID_ARG;
    }
#undef SMAT_TILE_STEP
    return hipGetLastError() == hipSuccess ? SMAT_OK : SMAT_ERR_HIP;
}

smat_status_t smat_probe_mfma(int workgroups, int iters, void* dev_sink, void* stream)
{
    if (workgroups <= 0 || iters <= 0 || !dev_sink) return SMAT_ERR_INVALID_ARG;
    hipLaunchKernelGGL(probe_mfma_kernel, dim3(workgroups), dim3(256), 0, static_cast<hipStream_t>(stream), iters,
                       static_cast<float*>(dev_sink));
    return hipGetLastError() == hipSuccess ? SMAT_OK : SMAT_ERR_HIP;
}

}  // extern "C"
