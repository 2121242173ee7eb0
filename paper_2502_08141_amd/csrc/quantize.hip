// Quantize kernel (paper App. A.1): per 64-element group absmax, normalise, bin every weight
// against its channel's sorted thresholds, bit-pack the codes at the channel's width.
//
// Mapping: one workgroup per output channel (the unit that owns a width and a table, Sec. 4.1).
// A lane owns 8 consecutive weights (two 16-byte loads), so a group is 8 adjacent lanes: the
// absmax is an in-lane max plus three cross-lane steps, and the lane's 8 codes form exactly
// 1, 2 or 4 whole bytes of the row's bit stream -- no cross-lane packing.  HBM-read bound:
// 4 B/weight in, bits/8 + 1/16 B/weight out.
#include "lowra_host.h"

namespace lowra {

template <int BITS>
__device__ __forceinline__ void quantize_row(const float* __restrict__ w, const float* __restrict__ thr,
                                             uint8_t* __restrict__ row, float* __restrict__ am, int K) {
    constexpr int NT = (1 << BITS) - 1;
    float T[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) T[j] = thr[j];   // channel-uniform: scalar loads

    const int units = K >> 3;
    for (int u = threadIdx.x; u < units; u += blockDim.x) {
        const float4 v0 = reinterpret_cast<const float4*>(w)[2 * u];
        const float4 v1 = reinterpret_cast<const float4*>(w)[2 * u + 1];
        const float v[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
        float a = 0.0f;
#pragma unroll
        for (int i = 0; i < 8; ++i) a = fmaxf(a, fabsf(v[i]));
        // the 8 lanes of a group are all active together (K/8 is a multiple of 8)
        a = fmaxf(a, __shfl_xor(a, 1));
        a = fmaxf(a, __shfl_xor(a, 2));
        a = fmaxf(a, __shfl_xor(a, 4));
        const float inv = (a == 0.0f) ? 0.0f : 1.0f / a;   // IEEE division, once per group
        uint32_t c = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float un = v[i] * inv;
            uint32_t code = 0;
#pragma unroll
            for (int j = 0; j < NT; ++j) code += (T[j] < un) ? 1u : 0u;
            c |= code << (i * BITS);
        }
        if (BITS == 1) row[u] = (uint8_t)c;
        else if (BITS == 2) reinterpret_cast<uint16_t*>(row)[u] = (uint16_t)c;
        else reinterpret_cast<uint32_t*>(row)[u] = c;
        if ((u & 7) == 0) am[u >> 3] = a;
    }
}

__global__ __launch_bounds__(256) void quantize_kernel(const RowInfo* __restrict__ rows,
                                                       const float* __restrict__ W,
                                                       const float* __restrict__ thresholds,
                                                       uint8_t* __restrict__ packed,
                                                       float* __restrict__ absmax, int K) {
    const int n = blockIdx.x;
    const RowInfo ri = rows[n];
    const float* w = W + (size_t)n * K;
    const float* thr = thresholds + (size_t)ri.cb() * kTableStride;
    uint8_t* row = packed + ri.offset;
    float* am = absmax + (size_t)n * (K / kGroup);
    switch (ri.bits()) {
        case 1: quantize_row<1>(w, thr, row, am, K); break;
        case 2: quantize_row<2>(w, thr, row, am, K); break;
        default: quantize_row<4>(w, thr, row, am, K); break;
    }
}

hipError_t launch_quantize(const lowra_layout& L, const float* W, const float* thresholds,
                           uint8_t* packed, float* absmax, hipStream_t st) {
    if (L.N == 0) return hipSuccess;
    quantize_kernel<<<dim3(L.N), dim3(256), 0, st>>>(L.d_rows, W, thresholds, packed, absmax, L.K);
    return hipGetLastError();
}

}  // namespace lowra
