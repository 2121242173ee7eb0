// Dequantize kernel (paper App. A.2): find the row's slice of the packed buffer from its
// precision, unpack 1/2/4-bit codes, look each up in the channel's mapping table, multiply by
// the group's absmax, store bf16 (round-to-nearest-even) or fp32.
//
// Mapping: a workgroup owns kDeqRows consecutive output channels and requests their records, then
// the codes, scales and mapping tables of all of them, before it decodes anything: the dependent
// chain record -> codes -> store is paid once per 32 KB of output (K = 4096) instead of once per
// row.  The 16-entry tables sit in LDS (16 consecutive banks: any mix of codes is conflict-free).
// A lane decodes 8 consecutive weights from 1, 2 or 4 bytes and issues one 16-byte store, so a
// wavefront writes 1 KB contiguous.  HBM-write bound: 2 B/weight out, bits/8 + 1/16 B/weight in.
#include "lowra_host.h"

namespace lowra {

#ifndef LOWRA_DEQ_ROWS
#define LOWRA_DEQ_ROWS 2
#endif
constexpr int kDeqRows = LOWRA_DEQ_ROWS;   // channels per workgroup
constexpr int kDeqUnits = 2;               // 8-weight units per lane, row and pass

template <bool F32, int R>
__global__ __launch_bounds__(256) void dequantize_kernel(const RowInfo* __restrict__ rows,
                                                         const uint8_t* __restrict__ packed,
                                                         const void* __restrict__ absmax,
                                                         const float* __restrict__ mappings,
                                                         void* __restrict__ out, int K, int N, int scale_bf16) {
    constexpr int UU = kDeqUnits;
    static_assert(R * kTableStride <= 256, "one lane per table entry");
    __shared__ float tab[R][kTableStride];
    const int units = K >> 3, G = K / kGroup;
    const int tid = threadIdx.x, n0 = blockIdx.x * R;
    RowInfo ri[R];
#pragma unroll
    for (int j = 0; j < R; ++j) ri[j] = rows[min(n0 + j, N - 1)];       // past the last channel: a valid record, never stored
    float m = 0.0f;
#pragma unroll
    for (int j = 0; j < R; ++j)
        if ((tid >> 4) == j) m = mappings[(size_t)ri[j].cb() * kTableStride + (tid & (kTableStride - 1))];
    for (int base = 0; base < units; base += 256 * UU) {
        uint32_t c[R][UU];
        float a[R][UU];
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const uint8_t* row = packed + ri[j].offset;
            const size_t am0 = (size_t)min(n0 + j, N - 1) * G;
            const int bits = ri[j].bits();
#pragma unroll
            for (int q = 0; q < UU; ++q) {
                const int u = min(base + tid + q * 256, units - 1);          // past the row's end: in bounds, never decoded
                c[j][q] = load_codes8(row, u, bits);
                a[j][q] = scale_bf16 ? bf16_bits_to_float(static_cast<const uint16_t*>(absmax)[am0 + (u >> 3)])
                                     : static_cast<const float*>(absmax)[am0 + (u >> 3)];
            }
        }
        if (base == 0) {
            if (tid < R * kTableStride) tab[tid >> 4][tid & (kTableStride - 1)] = m;
            __syncthreads();
        }
#pragma unroll
        for (int j = 0; j < R; ++j) {
            if (n0 + j >= N) break;
            const int n = n0 + j, bits = ri[j].bits();
            const float* t = tab[j];
#pragma unroll
            for (int q = 0; q < UU; ++q) {
                const int u = base + tid + q * 256;
                if (u < units) {
                    if (F32) {
                        const uint32_t mask = (1u << bits) - 1u;
                        float w[8];
#pragma unroll
                        for (int i = 0; i < 8; ++i) w[i] = t[(c[j][q] >> (i * bits)) & mask] * a[j][q];
                        float4* o = reinterpret_cast<float4*>(static_cast<float*>(out) + (size_t)n * K) + 2 * u;
                        store16_stream(o, make_float4(w[0], w[1], w[2], w[3]));
                        store16_stream(o + 1, make_float4(w[4], w[5], w[6], w[7]));
                    } else {
                        uint4* o = reinterpret_cast<uint4*>(static_cast<uint16_t*>(out) + (size_t)n * K) + u;
                        store16_stream(o, decode8_bf16(c[j][q], bits, t, a[j][q]));
                    }
                }
            }
        }
    }
}

hipError_t launch_dequantize(const lowra_layout& L, const uint8_t* packed, const void* absmax,
                             const float* mappings, int out_dtype, void* out, hipStream_t st) {
    if (L.N == 0) return hipSuccess;
    const int grid = (L.N + kDeqRows - 1) / kDeqRows;
    KernelTimer timer(st);
    if (out_dtype == 1)
        dequantize_kernel<true, kDeqRows><<<dim3(grid), dim3(256), 0, st>>>(L.d_rows, packed, absmax, mappings, out, L.K, L.N, L.scale_bf16 ? 1 : 0);
    else
        dequantize_kernel<false, kDeqRows><<<dim3(grid), dim3(256), 0, st>>>(L.d_rows, packed, absmax, mappings, out, L.K, L.N, L.scale_bf16 ? 1 : 0);
    return hipGetLastError();
}

}  // namespace lowra
