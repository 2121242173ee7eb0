// Quantize kernel (paper App. A.1): per 64-element group absmax, normalise, bin every weight
// against its channel's sorted thresholds, bit-pack the codes at the channel's width.
//
// Mapping: one workgroup per output channel (the unit that owns a width and a table, Sec. 4.1).
// A lane ends up owning 8 consecutive weights, so a group is 8 lanes: the absmax is an in-lane
// max plus three cross-lane steps, and the lane's 8 codes form exactly 1, 2 or 4 whole bytes of
// the row's bit stream -- no cross-lane packing.  HBM-read bound: 4 B/weight in,
// bits/8 + 1/16 B/weight out.
#include "lowra_host.h"

namespace lowra {

template <int CTRL>
__device__ __forceinline__ float dpp_f32(float x) {
    const int v = __builtin_bit_cast(int, x);
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(v, v, CTRL, 0xf, 0xf, true));
}
constexpr int kDppSwapPairs = 0xB1;   // quad_perm [1,0,3,2]: lanes 2j <-> 2j+1
constexpr int kDppXor2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppRor4 = 0x124;       // row_ror:4 (within 16 lanes)
constexpr int kDppRor8 = 0x128;       // row_ror:8

// One unit = 8 consecutive weights held by one lane: absmax of its 64-wide group, codes, packed
// bytes.  The 8 units of a group sit in 8 lanes of equal parity inside one 16-lane row.
// scale_bf16: the group scale is rounded to bf16 right after the maximum (nearest even; a maximum that would round to
// infinity keeps the largest finite bf16), and that value normalises the group and is what is stored, 2 bytes per group.
// 4-bit rows find the code -- the number of thresholds strictly below the weight -- by bisection over the sorted
// thresholds (the last two steps read the threshold from `thr_l`, the row's 15 thresholds in LDS: 16 consecutive
// banks, conflict-free for any mix of indices) instead of 15 compares.
template <int BITS>
__device__ __forceinline__ void quantize_unit(const float4& v0, const float4& v1, const float (&T)[15], const float* thr_l,
                                              uint8_t* __restrict__ row, void* __restrict__ am, int u, bool valid,
                                              bool scale_bf16) {
    constexpr int NT = (1 << BITS) - 1;
    const float v[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
    float a = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) a = fmaxf(a, fabsf(v[i]));
    a = fmaxf(a, dpp_f32<kDppXor2>(a));     // lanes l, l^2
    a = fmaxf(a, dpp_f32<kDppRor4>(a));     // quads q, q+1
    a = fmaxf(a, dpp_f32<kDppRor8>(a));     // all four quads of the row, same parity
    uint32_t a16 = 0;
    if (scale_bf16) {
        a16 = pack_bf16x2(a, 0.0f) & 0xffffu;
        if (a16 == 0x7f80u) a16 = 0x7f7fu;
        a = bf16_bits_to_float(a16);
    }
    const float inv = (a == 0.0f) ? 0.0f : 1.0f / a;   // IEEE division, once per group
    uint32_t c = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const float un = v[i] * inv;
        uint32_t code = 0;
        if (BITS == 4) {
            const uint32_t b3 = (T[7] < un) ? 1u : 0u;
            code = 2u * b3 + (((b3 ? T[11] : T[3]) < un) ? 1u : 0u);
            code = 2u * code + ((thr_l[4u * code + 1u] < un) ? 1u : 0u);
            code = 2u * code + ((thr_l[2u * code] < un) ? 1u : 0u);
        } else {
#pragma unroll
            for (int j = 0; j < NT; ++j) code += (T[j] < un) ? 1u : 0u;
        }
        c |= code << (i * BITS);
    }
    if (valid) {
        if (BITS == 1) row[u] = (uint8_t)c;
        else if (BITS == 2) reinterpret_cast<uint16_t*>(row)[u] = (uint16_t)c;
        else reinterpret_cast<uint32_t*>(row)[u] = c;
        if ((u & 7) == 0) {
            if (scale_bf16) static_cast<uint16_t*>(am)[u >> 3] = (uint16_t)a16;
            else static_cast<float*>(am)[u >> 3] = a;
        }
    }
}

// One workgroup per channel.  A wavefront covers 64 units (2 KB of weights) per pass with two
// fully coalesced 16-byte loads per lane (lane l reads bytes [16 l, 16 l + 16) of each KB), then
// neighbouring lanes trade halves so that lane 2j holds unit j and lane 2j+1 holds unit 32 + j.
// The weights of two passes (a whole row of K = 4096) are requested before anything else: they
// do not depend on the row record.
__device__ __forceinline__ void quantize_row(const RowInfo* __restrict__ rows,
                                             const float* __restrict__ W,
                                             const float* __restrict__ thresholds,
                                             uint8_t* __restrict__ packed,
                                             void* __restrict__ absmax, const int K, const int scale_bf16, const int n) {
    constexpr int U = 2;                                  // passes requested together
    __shared__ float thr_l[16];
    const float4* w4 = reinterpret_cast<const float4*>(W + (size_t)n * K);
    const int units = K >> 3, last4 = 2 * units - 1;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const bool odd = lane & 1;
    float4 x0[U], x1[U];
    auto fetch = [&](int base) {                          // past the row's end: clamped, in bounds, never stored
#pragma unroll
        for (int q = 0; q < U; ++q) {
            const int f = 2 * (base + q * 256 + wave * 64) + lane;
            x0[q] = load16_stream(w4 + min(f, last4)); x1[q] = load16_stream(w4 + min(f + 64, last4));
        }
    };
    fetch(0);
    const RowInfo ri = rows[n];
    const float* thr = thresholds + (size_t)ri.cb() * kTableStride;
    uint8_t* row = packed + ri.offset;
    void* am = scale_bf16 ? static_cast<void*>(static_cast<uint16_t*>(absmax) + (size_t)n * (K / kGroup))
                          : static_cast<void*>(static_cast<float*>(absmax) + (size_t)n * (K / kGroup));
    const bool sb16 = scale_bf16 != 0;
    const int bits = ri.bits();
    float T[15];
#pragma unroll
    for (int j = 0; j < 15; ++j) T[j] = thr[j];           // channel-uniform scalar loads; a table row always holds 16 floats
    if (bits == 4) {                                      // uniform over the workgroup
        if (threadIdx.x < 16) thr_l[threadIdx.x] = thr[threadIdx.x];
        __syncthreads();
    }
    for (int base = 0; base < units; base += U * 256) {
        if (base > 0) fetch(base);
#pragma unroll
        for (int q = 0; q < U; ++q) {
            // lane 2j sends the second unit's first half and gets the first unit's second half
            const float4 send = odd ? x0[q] : x1[q];
            float4 recv;
            recv.x = dpp_f32<kDppSwapPairs>(send.x); recv.y = dpp_f32<kDppSwapPairs>(send.y);
            recv.z = dpp_f32<kDppSwapPairs>(send.z); recv.w = dpp_f32<kDppSwapPairs>(send.w);
            const float4 v0 = odd ? recv : x0[q], v1 = odd ? x1[q] : recv;
            const int u = base + q * 256 + wave * 64 + (lane >> 1) + (odd ? 32 : 0);
            const bool valid = u < units;                 // units is a multiple of 8: a group is valid as a whole
            switch (bits) {
                case 1: quantize_unit<1>(v0, v1, T, thr_l, row, am, u, valid, sb16); break;
                case 2: quantize_unit<2>(v0, v1, T, thr_l, row, am, u, valid, sb16); break;
                default: quantize_unit<4>(v0, v1, T, thr_l, row, am, u, valid, sb16); break;
            }
        }
    }
}

__global__ __launch_bounds__(256) void quantize_kernel(const RowInfo* __restrict__ rows,
                                                       const float* __restrict__ W,
                                                       const float* __restrict__ thresholds,
                                                       uint8_t* __restrict__ packed,
                                                       void* __restrict__ absmax, int K, int scale_bf16) {
    quantize_row(rows, W, thresholds, packed, absmax, K, scale_bf16, (int)blockIdx.x);
}

// Several matrices in one launch (a decoder layer's seven, say): the workgroups of matrix m are
// [first[m], first[m + 1]).  Between two launches on a stream lie 2-3 us in which nothing streams -- a tenth of
// the time of a 4096 x 4096 matrix.  The descriptors travel as kernel arguments: no device table, no copy.
struct QuantizeBatch {
    const RowInfo* rows[kQuantizeBatchMax]; const float* W[kQuantizeBatchMax]; const float* thresholds[kQuantizeBatchMax];
    uint8_t* packed[kQuantizeBatchMax]; void* absmax[kQuantizeBatchMax];
    int K[kQuantizeBatchMax], scale_bf16[kQuantizeBatchMax], first[kQuantizeBatchMax + 1];
    int count;
};
__global__ __launch_bounds__(256) void quantize_batch_kernel(const QuantizeBatch b) {
    int m = 0;
#pragma unroll
    for (int q = 1; q < kQuantizeBatchMax; ++q)
        if (q < b.count && (int)blockIdx.x >= b.first[q]) m = q;         // uniform
    quantize_row(b.rows[m], b.W[m], b.thresholds[m], b.packed[m], b.absmax[m], b.K[m], b.scale_bf16[m], (int)blockIdx.x - b.first[m]);
}

hipError_t launch_quantize(const lowra_layout& L, const float* W, const float* thresholds,
                           uint8_t* packed, void* absmax, hipStream_t st) {
    if (L.N == 0) return hipSuccess;
    KernelTimer timer(st);
    quantize_kernel<<<dim3(L.N), dim3(256), 0, st>>>(L.d_rows, W, thresholds, packed, absmax, L.K, L.scale_bf16 ? 1 : 0);
    return hipGetLastError();
}

// count matrices, kQuantizeBatchMax per launch; matrices without channels are skipped
hipError_t launch_quantize_batch(int count, const lowra_layout* const* layouts, const float* const* W,
                                 const float* const* thresholds, uint8_t* const* packed, void* const* absmax, hipStream_t st) {
    KernelTimer timer(st);
    int i = 0;
    while (i < count) {
        QuantizeBatch b{};
        int rows = 0;
        for (; i < count && b.count < kQuantizeBatchMax; ++i) {
            const lowra_layout& L = *layouts[i];
            if (L.N == 0) continue;
            if ((long long)rows + L.N > 0x7fffffffLL) break;               // the grid's limit: the next launch takes it
            const int m = b.count++;
            b.rows[m] = L.d_rows; b.W[m] = W[i]; b.thresholds[m] = thresholds[i]; b.packed[m] = packed[i]; b.absmax[m] = absmax[i];
            b.K[m] = L.K; b.scale_bf16[m] = L.scale_bf16 ? 1 : 0; b.first[m] = rows;
            rows += L.N;
        }
        if (b.count == 0) continue;
        b.first[b.count] = rows;
        quantize_batch_kernel<<<dim3(rows), dim3(256), 0, st>>>(b);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace lowra
