// Rank-r side products of the LoRA term (Sec. 2.1): t = s x A^T (forward) and u = s dY B (input
// gradient), plus the small operand re-layouts they need.  Bandwidth-bound on reading x / dY once.
#include "gemm_common.h"

namespace lowra {

// out[m][j] = bf16( s * sum_c P[m][c] Q[j][c] ), j < 32 CT (rows j >= r of Q count as zero).
// One workgroup per 32 token rows; 8 wavefronts split the contraction (wave w takes 16-wide
// steps w, w+8, ...), four steps of loads in flight per wavefront, partial tiles meet in LDS.
template <int CT>
__global__ __launch_bounds__(512) void skinny_nt_kernel(const uint16_t* __restrict__ P, int ldp, int M,
                                                       const uint16_t* __restrict__ Q, int ldq, int r,
                                                       int Kc, float s, uint16_t* __restrict__ out) {
    extern __shared__ __align__(16) uint8_t smem[];
    float* red = reinterpret_cast<float*>(smem);   // [8][32][CT*32]
    constexpr int RP = CT * 32, U = 4;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 31, kg = lane >> 5;
    const int m = blockIdx.x * 32 + i;
    const bool m_ok = m < M;
    floatx16_t acc[CT];
#pragma unroll
    for (int c = 0; c < CT; ++c)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[c][v] = 0.0f;
    const bf16x8_t zero = {0, 0, 0, 0, 0, 0, 0, 0};
    const uint16_t* prow = P + (size_t)(m_ok ? m : 0) * ldp;
    for (int kb = wave * 16; kb < Kc; kb += 128 * U) {   // wavefront-uniform trip count: MFMA reads every lane
        const int k0 = kb + kg * 8;
        bf16x8_t a[U], b[U][CT];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int kk = k0 + u * 128;
            const bool kin = kk < Kc;
            a[u] = (m_ok && kin) ? *reinterpret_cast<const bf16x8_t*>(prow + kk) : zero;
#pragma unroll
            for (int c = 0; c < CT; ++c) {
                const int j = c * 32 + i;
                b[u][c] = (j < r && kin) ? *reinterpret_cast<const bf16x8_t*>(Q + (size_t)j * ldq + kk) : zero;
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int c = 0; c < CT; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[u], b[u][c], acc[c], 0, 0, 0);
    }
#pragma unroll
    for (int c = 0; c < CT; ++c)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = 8 * (v >> 2) + 4 * kg + (v & 3);
            red[(wave * 32 + row) * RP + c * 32 + i] = acc[c][v];
        }
    __syncthreads();
    for (int idx = threadIdx.x; idx < 32 * RP; idx += 512) {
        const int row = idx / RP, col = idx % RP;
        float v = 0.0f;
#pragma unroll
        for (int w = 0; w < 8; ++w) v += red[(w * 32 + row) * RP + col];
        const int mo = blockIdx.x * 32 + row;
        if (mo < M) out[(size_t)mo * RP + col] = (uint16_t)(pack_bf16x2(v * s, 0.0f) & 0xffffu);
    }
}

// dst [R, CP] = src [R, c] padded with zero columns.
__global__ void pad_cols_kernel(const uint16_t* __restrict__ src, int R, int c, uint16_t* __restrict__ dst, int CP) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)R * CP) return;
    const int row = (int)(idx / CP), col = (int)(idx % CP);
    dst[idx] = col < c ? src[(size_t)row * c + col] : (uint16_t)0;
}
// dst [c, R] = transpose of src [R, c]; 32 x 32 tiles through LDS so both sides are coalesced.
__global__ __launch_bounds__(256) void transpose_kernel(const uint16_t* __restrict__ src, int R, int c,
                                                        uint16_t* __restrict__ dst) {
    __shared__ uint16_t tile[32][33];
    const int r0 = blockIdx.x * 32, c0 = blockIdx.y * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    for (int y = ty; y < 32; y += 8) {
        const int rr = r0 + y, cc = c0 + tx;
        tile[y][tx] = (rr < R && cc < c) ? src[(size_t)rr * c + cc] : (uint16_t)0;
    }
    __syncthreads();
    for (int y = ty; y < 32; y += 8) {
        const int cc = c0 + y, rr = r0 + tx;
        if (cc < c && rr < R) dst[(size_t)cc * R + rr] = tile[tx][y];
    }
}

hipError_t launch_skinny(const uint16_t* P, int ldp, int M, const uint16_t* Q, int ldq, int r, int Kc,
                         float s, uint16_t* out, int RP, hipStream_t st) {
    const dim3 grid((M + 31) / 32), block(512);
    const size_t sh = (size_t)8 * 32 * RP * sizeof(float);
    if (RP == 64) {
        static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(skinny_nt_kernel<2>),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, 8 * 32 * 64 * 4);
        if (attr != hipSuccess) return attr;
        skinny_nt_kernel<2><<<grid, block, sh, st>>>(P, ldp, M, Q, ldq, r, Kc, s, out);
    } else {
        static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(skinny_nt_kernel<4>),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, 8 * 32 * 128 * 4);
        if (attr != hipSuccess) return attr;
        skinny_nt_kernel<4><<<grid, block, sh, st>>>(P, ldp, M, Q, ldq, r, Kc, s, out);
    }
    return hipGetLastError();
}
hipError_t launch_pad_cols(const uint16_t* src, int R, int c, uint16_t* dst, int CP, hipStream_t st) {
    const size_t tot = (size_t)R * CP;
    pad_cols_kernel<<<dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, st>>>(src, R, c, dst, CP);
    return hipGetLastError();
}
hipError_t launch_transpose(const uint16_t* src, int R, int c, uint16_t* dst, hipStream_t st) {
    transpose_kernel<<<dim3((R + 31) / 32, (c + 31) / 32), dim3(256), 0, st>>>(src, R, c, dst);
    return hipGetLastError();
}

}  // namespace lowra
