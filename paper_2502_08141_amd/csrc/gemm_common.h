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
    const SortedRow* gemm_rows;  // forward: row records in the per-tile order below
    const uint16_t* tile_order;  // forward: per 256-row tile, the local rows in processing order (natural, 4-bit rows last)
    const uint8_t* packed;
    const float* absmax;
    const float* mappings;
    const uint16_t* act;         // x [M,K] or dY [M,N]
    const uint16_t* ext_act;     // s * rank-r intermediate [M,RP]
    const uint16_t* ext_w;       // fwd: LoRA B with rows of RP entries [N,RP]
    const uint16_t* lora_A;      // bwd: LoRA A [r,K]
    int lora_r;
    uint16_t* out;               // y [M,N] or dX [M,K]
    int M, N, K, G, RP;
    int any4;                    // the matrix holds 4-bit rows
    int C;                       // number of codebooks
    // input gradient only.  ld_act = row length of act (the matrix's N).  The output tiles from `split_first` on (the
    // last, short round of workgroups; all tiles when the grid is at most half the chip) have their contraction over
    // the channels split between `splits` workgroups: split s takes rows [s rows_per_split, ...) and leaves an fp32
    // partial tile in split_out [splits][tiles - split_first][256][256]
    int ld_act, splits, rows_per_split, split_first;
    float* split_out;
};

// plan of a split input gradient (gemm_bwd_split_plan): workgroups per split tile, rows of the matrix per split,
// first split tile, number of split tiles
struct BwdSplitPlan { int splits, rows_per_split, first, tail; };

struct GemvParams {
    const SortedRow* sorted_rows;
    const uint8_t* packed;
    size_t packed_bytes;
    const float* absmax;
    const float* mappings;
    const uint16_t* x;       // [M,K]
    const uint16_t* A;       // LoRA A [r,K] (null when r == 0)
    const uint16_t* B;       // LoRA B [N,r]
    float* tp;               // workspace: partial sums of x A^T, [ceil(K/256)][16][RT] fp32
    uint16_t* y;             // [M,N]
    float s;
    int M, N, K, G, r, RT;   // RT = r rounded up to 16 (0 when r == 0)
    int xbufs;               // activation buffers per wavefront in LDS (set by the launcher)
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

// the same accumulators as fp32 (partial tiles of a split contraction)
__device__ __forceinline__ void store_out_f32(const floatx16_t (&acc)[4][4], float* out, int ld, int rows_valid,
                                              int cols_valid, int row0, int col0) {
    // (the thread index is taken afresh here: sharing its pieces with the kernel's prologue kept them alive, and
    // spilled, across the whole kernel)
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
#pragma unroll
    for (int tm = 0; tm < 4; ++tm)
#pragma unroll
        for (int tn = 0; tn < 4; ++tn) {
            const int col = col0 + wn * 128 + tn * 32 + (lane & 31);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = row0 + wm * 128 + tm * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                if (row < rows_valid && col < cols_valid) out[(size_t)row * ld + col] = acc[tm][tn][v];
            }
        }
}

// A pointer that the compiler knows to lie in global memory.  Kernel arguments are known to; a pointer that a kernel
// reads out of a descriptor in memory is generic to it, and generic loads and stores count on the vector-memory and
// the LDS counter at once: every use then waits for ALL outstanding transfers of both kinds.
template <class T> using gptr = T __attribute__((address_space(1)))*;
template <class T> __device__ __forceinline__ gptr<T> as_global(T* p) { return (gptr<T>)p; }
// 8- and 16-byte accesses through such a pointer (the runtime's vector classes bind to generic references only)
typedef unsigned int g_u32x2_t __attribute__((ext_vector_type(2)));
typedef unsigned int g_u32x4_t __attribute__((ext_vector_type(4)));
typedef float g_f32x4_t __attribute__((ext_vector_type(4)));
template <class T> __device__ __forceinline__ uint2 gload_u2(gptr<T> p) { const g_u32x2_t v = *(gptr<const g_u32x2_t>)p; return make_uint2(v.x, v.y); }
template <class T> __device__ __forceinline__ uint4 gload_u4(gptr<T> p) { const g_u32x4_t v = *(gptr<const g_u32x4_t>)p; return make_uint4(v.x, v.y, v.z, v.w); }
template <class T> __device__ __forceinline__ float4 gload_f4(gptr<T> p) { const g_f32x4_t v = *(gptr<const g_f32x4_t>)p; return make_float4(v.x, v.y, v.z, v.w); }
template <class T> __device__ __forceinline__ void gstore_u2(gptr<T> p, uint2 v) { *(gptr<g_u32x2_t>)p = g_u32x2_t{v.x, v.y}; }

// compute units of the current device (asked once; 256 if the runtime does not say)
static inline int device_compute_units() {
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) v = 256;
        cus = v;
    }
    return cus;
}

typedef __attribute__((address_space(1))) const void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

// Global -> LDS DMA of 16 bytes per lane (global_load_lds_dwordx4): lane l's data lands at LDS
// address lds_base + 16 l (lds_base wavefront-uniform).  Issued as inline assembly on purpose:
// the compiler orders every LDS access it cannot disambiguate behind an outstanding DMA it knows
// about and would wait for the transfer in the middle of a step.  The price is that the compiler
// does not count these transfers: every step ends with dma_wait_all() before its barrier.
__device__ __forceinline__ void dma16(const void* gaddr, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 : : "v"(gaddr), "s"(__builtin_amdgcn_readfirstlane(lds_base)) : "memory");
}
// 4 bytes per lane: lane l's dword lands at lds_base + 4 l
__device__ __forceinline__ void dma4(const void* gaddr, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off"
                 : : "v"(gaddr), "s"(__builtin_amdgcn_readfirstlane(lds_base)) : "memory");
}
// Same transfers with the address split into a wavefront-uniform 64-bit base (scalar registers) and a
// 32-bit per-lane byte offset, and the LDS base already uniform: no vector arithmetic per transfer.
__device__ __forceinline__ void dma16_s(const void* sbase, uint32_t voff, uint32_t lds_base_uniform) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 : : "v"(voff), "s"(sbase), "s"(lds_base_uniform) : "memory");
}
__device__ __forceinline__ void dma4_s(const void* sbase, uint32_t voff, uint32_t lds_base_uniform) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
                 : : "v"(voff), "s"(sbase), "s"(lds_base_uniform) : "memory");
}
__device__ __forceinline__ void dma_wait_all() { asm volatile("s_waitcnt vmcnt(0)" : : : "memory"); }

// 8 one-bit codes (low byte of c) -> 8 bf16 through the byte table Q = [lo0, lo1, hi0, hi1]
__device__ __forceinline__ uint4 decode8_w1(uint32_t c, uint32_t Q) {
    uint32_t d[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t q = __builtin_amdgcn_ubfe(c, 2 * j, 2);
        d[j] = __builtin_amdgcn_perm(Q, Q, (__umul24(q, 0x808101u) & 0x01010101u) | 0x02000200u);
    }
    return make_uint4(d[0], d[1], d[2], d[3]);
}
// 8 two-bit codes (low 16 bits of c) -> 8 bf16 through TL = low bytes, TH = high bytes of the 4 levels
__device__ __forceinline__ uint4 decode8_w2(uint32_t c, uint32_t TL, uint32_t TH) {
    uint32_t d[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t q = __builtin_amdgcn_ubfe(c, 4 * j, 4);
        d[j] = __builtin_amdgcn_perm(TH, TL, (__umul24(q, 0x404101u) & 0x03030303u) | 0x04000400u);
    }
    return make_uint4(d[0], d[1], d[2], d[3]);
}

}  // namespace lowra
