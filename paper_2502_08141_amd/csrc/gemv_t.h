// Partial sums of the rank-r intermediate of the small-token kernels, shared by both of them.
#pragma once
#include "gemm_common.h"

namespace lowra {

// ---------------------------------------------------------------------------------------------
// t partials:  tp[b][m][j] = sum over the 256 columns of block b of x[m][k] A[j][k]     (fp32)
// One wavefront per block; lane (i, kg) owns columns 64 kg .. 64 kg + 63 of the block for token i
// (operand B) and for ranks i + 16 c (operand A): 128 contiguous bytes per lane and row.
__device__ __forceinline__ void t_partial_body(const uint16_t* __restrict__ x, int M, int K,
                                               const uint16_t* __restrict__ A, int r, int RT,
                                               float* __restrict__ tp, const int b) {
    const int lane = threadIdx.x, i = lane & 15, kg = lane >> 4;
    const int kbase = b * 256 + kg * 64;
    const bool k_ok = kbase < K;                                  // K is a multiple of 64: a run is in or out as a whole
    const bf16x8_t zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
    bf16x8_t xf[8];
    const uint16_t* xr = x + (size_t)min(i, M - 1) * K + (k_ok ? kbase : 0);
#pragma unroll
    for (int j = 0; j < 8; ++j) xf[j] = (k_ok && i < M) ? *reinterpret_cast<const bf16x8_t*>(xr + 8 * j) : zero8;
    for (int c = 0; c < RT / 16; ++c) {
        const int jr = c * 16 + i;
        const uint16_t* ar = A + (size_t)min(jr, r - 1) * K + (k_ok ? kbase : 0);
        bf16x8_t af[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) af[j] = (k_ok && jr < r) ? *reinterpret_cast<const bf16x8_t*>(ar + 8 * j) : zero8;
        floatx4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int j = 0; j < 8; ++j) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[j], xf[j], acc, 0, 0, 0);
        // lane (i, kg) holds D[rank 16 c + 4 kg + v][token i]
#pragma unroll
        for (int v = 0; v < 4; ++v) tp[((size_t)b * 16 + i) * RT + c * 16 + 4 * kg + v] = acc[v];
    }
}


}  // namespace lowra
