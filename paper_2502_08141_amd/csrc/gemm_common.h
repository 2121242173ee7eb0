// Shared pieces of the fused dequant-GEMM kernels (forward and input gradient).
//
// Workgroup tile: 256 x 256 outputs, 64-deep contraction steps, 4 wavefronts (2 x 2), each
// owning 128 x 128 outputs = 4 x 4 tiles of v_mfma_f32_32x32x16_bf16 (256 accumulator registers).
// LDS holds two stages of (activation tile, weight tile), each tile 256 rows x 64 bf16 = 128 B
// per row with the 16-byte chunk index XOR-swizzled by (row>>1)&7: row-wise 16-byte writes and
// the MFMA operand reads (16 consecutive rows, same chunk) both spread over all 64 banks.
#pragma once
#include "lowra_host.h"

namespace lowra {

constexpr int BM = 256;        // token rows per workgroup
constexpr int BN = 256;        // output columns per workgroup
constexpr int BK = 64;         // contraction depth per step
constexpr int NTHREADS = 256;
constexpr int ROWB = 128;                 // bytes per LDS row
constexpr int TILEB = 256 * ROWB;         // one operand tile: 32 KB
constexpr int STAGEB = 2 * TILEB;         // activation tile + weight tile
constexpr int TAB_LD = 17;                // floats per LDS table row (odd stride spreads rows over banks)

struct GemmParams {
    const RowInfo* rows;
    const uint16_t* tile_order;  // forward: per 256-row tile, local rows sorted by width
    const uint8_t* packed;
    const float* absmax;
    const float* mappings;
    const uint16_t* act;         // x [M,K] or dY [M,N]
    const uint16_t* ext_act;     // s * rank-r intermediate [M,RP]
    const uint16_t* ext_w;       // B padded [N,RP] (fwd) or A^T padded [K,RP] (bwd)
    uint16_t* out;               // y [M,N] or dX [M,K]
    int M, N, K, G, RP;
};

__device__ __forceinline__ uint4 zero4() { return make_uint4(0, 0, 0, 0); }
__device__ __forceinline__ int swz_off(int row, int chunk) { return row * ROWB + ((chunk ^ ((row >> 1) & 7)) << 4); }

// XCD-aware tile order: workgroups are dealt round-robin over the 8 XCDs, so each XCD gets a
// contiguous run of logical tiles; with the output-column tile varying fastest the workgroups
// that share an L2 also share their activation rows.
__device__ __forceinline__ int xcd_tile(int bid, int nblk) {
    const int per = nblk >> 3, rem = nblk & 7;
    const int xcd = bid & 7, idx = bid >> 3;
    return xcd * per + (xcd < rem ? xcd : rem) + idx;
}

// epilogue: accumulator (row = 8 (v/4) + 4 (lane/32) + v%4, col = lane%32) -> bf16
__device__ __forceinline__ void store_out(const floatx16_t (&acc)[4][4], uint16_t* out, int ld, int rows_valid,
                                          int cols_valid, int row0, int col0) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
#pragma unroll
    for (int tm = 0; tm < 4; ++tm)
#pragma unroll
        for (int tn = 0; tn < 4; ++tn) {
            const int col = col0 + wn * 128 + tn * 32 + (lane & 31);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = row0 + wm * 128 + tm * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                if (row < rows_valid && col < cols_valid)
                    out[(size_t)row * ld + col] = (uint16_t)(pack_bf16x2(acc[tm][tn][v], 0.0f) & 0xffffu);
            }
        }
}

}  // namespace lowra
