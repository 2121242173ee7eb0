// Dequantize kernel (paper App. A.2): find the row's slice of the packed buffer from its
// precision, unpack 1/2/4-bit codes, look each up in the channel's mapping table, multiply by
// the group's absmax, store bf16 (round-to-nearest-even) or fp32.
//
// Mapping: one workgroup per output channel; the channel's 16-entry table sits in LDS (16
// consecutive banks: any mix of codes is conflict-free).  A lane decodes 8 consecutive weights
// from 1, 2 or 4 bytes and issues one 16-byte store, so a wavefront writes 1 KB contiguous.
// HBM-write bound: 2 B/weight out, bits/8 + 1/16 B/weight in.
#include "lowra_host.h"

namespace lowra {

template <bool F32>
__global__ __launch_bounds__(256) void dequantize_kernel(const RowInfo* __restrict__ rows,
                                                         const uint8_t* __restrict__ packed,
                                                         const float* __restrict__ absmax,
                                                         const float* __restrict__ mappings,
                                                         void* __restrict__ out, int K) {
    __shared__ float tab[kTableStride];
    const int n = blockIdx.x;
    const RowInfo ri = rows[n];
    const int bits = ri.bits();
    if (threadIdx.x < kTableStride)
        tab[threadIdx.x] = mappings[(size_t)ri.cb() * kTableStride + threadIdx.x];
    __syncthreads();
    const uint8_t* row = packed + ri.offset;
    const float* am = absmax + (size_t)n * (K / kGroup);
    const int units = K >> 3;
    const uint32_t mask = (1u << bits) - 1u;
    for (int u = threadIdx.x; u < units; u += blockDim.x) {
        const uint32_t c = load_codes8(row, u, bits);
        const float a = am[u >> 3];
        if (F32) {
            float w[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) w[i] = tab[(c >> (i * bits)) & mask] * a;
            float4* o = reinterpret_cast<float4*>(static_cast<float*>(out) + (size_t)n * K) + 2 * u;
            o[0] = make_float4(w[0], w[1], w[2], w[3]);
            o[1] = make_float4(w[4], w[5], w[6], w[7]);
        } else {
            uint4* o = reinterpret_cast<uint4*>(static_cast<uint16_t*>(out) + (size_t)n * K) + u;
            *o = decode8_bf16(c, bits, tab, a);
        }
    }
}

hipError_t launch_dequantize(const lowra_layout& L, const uint8_t* packed, const float* absmax,
                             const float* mappings, int out_dtype, void* out, hipStream_t st) {
    if (L.N == 0) return hipSuccess;
    if (out_dtype == 1)
        dequantize_kernel<true><<<dim3(L.N), dim3(256), 0, st>>>(L.d_rows, packed, absmax, mappings, out, L.K);
    else
        dequantize_kernel<false><<<dim3(L.N), dim3(256), 0, st>>>(L.d_rows, packed, absmax, mappings, out, L.K);
    return hipGetLastError();
}

}  // namespace lowra
