// Measurement kernels: the ceilings a benchmark prints beside the library's own figures, measured on
// the same device in the same run.  None of them is part of the hot path.
//   copy  - a plain device copy, 16 bytes per lane, a contiguous 16 KB piece per workgroup (read + write traffic)
//   read  - a plain streaming read, 16 bytes per lane, a contiguous slice per workgroup (what a small-token pass is bound by)
//   mfma  - a loop of independent v_mfma_f32_32x32x16_bf16 on registers (what a fused GEMM is bound by), once on
//           constant operands and once on operands that change with every instruction and hold pseudo-random
//           bf16 values of order one: the chip's power management slows the matrix pipe down by what the data
//           toggles, so the second figure is the ceiling of a GEMM on real data
#include "../../include/lowra.h"
#include "lowra_dev.h"

namespace lowra {

// Access patterns chosen by measurement (1 GiB, this chip): a workgroup that copies ONE contiguous 16 KB piece with
// its four loads per lane in flight together reaches 6.3-6.4 TB/s (read + write) where a grid-stride loop of 8192
// workgroups reached 5.0-5.2 and the runtime's device-to-device copy 5.1; a workgroup that streams one contiguous
// slice (1/2048 of the buffer, eight loads per lane in flight) reads at 7.0 TB/s where the grid-stride loop read
// at 5.5-6.0.
__global__ __launch_bounds__(256) void measure_copy_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n16) {
    const size_t base = (size_t)blockIdx.x * 1024 + threadIdx.x;
    u32x4_t v[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const size_t o = base + (size_t)q * 256;
        v[q] = o < n16 ? __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(src + o)) : u32x4_t{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const size_t o = base + (size_t)q * 256;
        if (o < n16) __builtin_nontemporal_store(v[q], reinterpret_cast<u32x4_t*>(dst + o));
    }
}

__global__ __launch_bounds__(256) void measure_read_kernel(const uint4* __restrict__ src, size_t n16, uint32_t* __restrict__ out) {
    const size_t per = (n16 + gridDim.x - 1) / gridDim.x, lo = per * blockIdx.x, hi = lo + per < n16 ? lo + per : n16;
    uint32_t acc = 0;
    for (size_t o = lo + threadIdx.x; o < hi; o += 256 * 8) {
        // eight loads in flight per lane and pass
        u32x4_t v[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const size_t idx = o + (size_t)q * 256;
            v[q] = idx < hi ? __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(src + idx)) : u32x4_t{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) acc ^= v[q].x ^ v[q].y ^ v[q].z ^ v[q].w;
    }
    if (acc == 0x9e3779b9u) out[0] = acc;       // keeps the loads alive; practically never taken
}

__global__ __launch_bounds__(256) void measure_mfma_kernel(int iters, float* __restrict__ out) {
    const bf16x8_t a = {1, 1, 1, 1, 1, 1, 1, 1}, b = {1, 1, 1, 1, 1, 1, 1, 1};
    floatx16_t acc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int t = 0; t < 4; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[t], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int t = 0; t < 4; ++t) s += acc[t][0];
    if (s == -1.0f) out[0] = s;                 // keeps the loop alive; never taken
}

// The same loop on operands of pseudo-random bf16 values (sign and mantissa from a hash of lane, wavefront and
// index; magnitudes in [0.5, 2)): four A and four B fragments per lane, every MFMA takes another pair.
__device__ __forceinline__ uint32_t measure_hash(uint32_t x) {
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}
__device__ __forceinline__ bf16x8_t measure_random_frag(uint32_t key) {
    uint32_t w[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const uint32_t h = measure_hash(key * 4u + (uint32_t)q);
        // two bf16: sign and 7 mantissa bits random, exponent 126 or 127
        const uint32_t lo = (h & 0x80ffu) | 0x3f00u, hi = ((h >> 16) & 0x80ffu) | 0x3f00u;
        w[q] = lo | (hi << 16);
    }
    return __builtin_bit_cast(bf16x8_t, make_uint4(w[0], w[1], w[2], w[3]));
}
__global__ __launch_bounds__(256) void measure_mfma_random_kernel(int iters, uint32_t seed, float* __restrict__ out) {
    bf16x8_t a[4], b[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        a[u] = measure_random_frag(seed + (uint32_t)((blockIdx.x * 256 + threadIdx.x) * 8 + u));
        b[u] = measure_random_frag(seed + (uint32_t)((blockIdx.x * 256 + threadIdx.x) * 8 + 4 + u));
    }
    floatx16_t acc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.0f;
    for (int it = 0; it < iters; it += 4) {                     // 16 MFMAs per pass = 4 per iteration counted
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int t = 0; t < 4; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(u + t) & 3], b[u], acc[t], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int t = 0; t < 4; ++t) s += acc[t][0];
    if (s == -1.0f) out[0] = s;                 // keeps the loop alive; practically never taken
}

}  // namespace lowra

extern "C" {

lowra_status lowra_measure_copy(void* dst, const void* src, size_t bytes, void* stream) {
    if (!dst || !src || bytes % 16 != 0) return LOWRA_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src)) & 15u) return LOWRA_MISALIGNED;
    if (bytes == 0) return LOWRA_OK;
    const size_t n16 = bytes / 16;
    if ((n16 + 1023) / 1024 > 0x7fffffffu) return LOWRA_UNSUPPORTED;
    lowra::measure_copy_kernel<<<dim3((unsigned)((n16 + 1023) / 1024)), dim3(256), 0, static_cast<hipStream_t>(stream)>>>(
        static_cast<uint4*>(dst), static_cast<const uint4*>(src), n16);
    return hipGetLastError() == hipSuccess ? LOWRA_OK : LOWRA_HIP_ERROR;
}

lowra_status lowra_measure_read(const void* src, size_t bytes, void* out4, void* stream) {
    if (!src || !out4 || bytes % 16 != 0) return LOWRA_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(src) & 15u) return LOWRA_MISALIGNED;
    if (bytes == 0) return LOWRA_OK;
    lowra::measure_read_kernel<<<dim3(2048), dim3(256), 0, static_cast<hipStream_t>(stream)>>>(
        static_cast<const uint4*>(src), bytes / 16, static_cast<uint32_t*>(out4));
    return hipGetLastError() == hipSuccess ? LOWRA_OK : LOWRA_HIP_ERROR;
}

lowra_status lowra_measure_mfma(int workgroups, int iterations, void* out4, double* flops_out, void* stream) {
    if (workgroups <= 0 || iterations <= 0 || !out4) return LOWRA_INVALID_ARG;
    lowra::measure_mfma_kernel<<<dim3(workgroups), dim3(256), 0, static_cast<hipStream_t>(stream)>>>(iterations, static_cast<float*>(out4));
    if (flops_out) *flops_out = (double)workgroups * 4.0 * iterations * 4.0 * 2.0 * 32 * 32 * 16;
    return hipGetLastError() == hipSuccess ? LOWRA_OK : LOWRA_HIP_ERROR;
}

lowra_status lowra_measure_mfma_random(int workgroups, int iterations, void* out4, double* flops_out, void* stream) {
    if (workgroups <= 0 || iterations <= 0 || iterations % 4 != 0 || !out4) return LOWRA_INVALID_ARG;
    lowra::measure_mfma_random_kernel<<<dim3(workgroups), dim3(256), 0, static_cast<hipStream_t>(stream)>>>(iterations, 0x2502u, static_cast<float*>(out4));
    if (flops_out) *flops_out = (double)workgroups * 4.0 * iterations * 4.0 * 2.0 * 32 * 32 * 16;
    return hipGetLastError() == hipSuccess ? LOWRA_OK : LOWRA_HIP_ERROR;
}

}  // extern "C"
