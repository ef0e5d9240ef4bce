// Four small kernels that measure what this GPU delivers for the access patterns the SpMM
// kernels consist of, so that the figures quoted next to the rooflines can be reproduced:
// a streaming read, two random gathers of rows (the ways rows of B are fetched), and a
// register-resident MFMA loop.  They compute nothing of the method.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "../../include/smat_bench.h"

namespace {

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

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

}  // namespace

extern "C" {

smat_status_t smat_probe_read(const void* dev_buf, size_t bytes, void* dev_sink, void* stream)
{
    if (!dev_buf || !dev_sink || bytes < 8192) return SMAT_ERR_INVALID_ARG;
    hipLaunchKernelGGL(probe_read_kernel, dim3(4096), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const u32x4*>(dev_buf), bytes / 16, static_cast<uint32_t*>(dev_sink));
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

smat_status_t smat_probe_mfma(int workgroups, int iters, void* dev_sink, void* stream)
{
    if (workgroups <= 0 || iters <= 0 || !dev_sink) return SMAT_ERR_INVALID_ARG;
    hipLaunchKernelGGL(probe_mfma_kernel, dim3(workgroups), dim3(256), 0, static_cast<hipStream_t>(stream), iters,
                       static_cast<float*>(dev_sink));
    return hipGetLastError() == hipSuccess ? SMAT_OK : SMAT_ERR_HIP;
}

}  // extern "C"
