// Dequant-fused frozen-base LoRA linear on gfx950 MFMA (bf16 in, fp32 accumulate).
//
//   forward        y  = x  What^T + s (x A^T) B^T        (Sec. 2.1 LoRA form, Sec. 3 step P5)
//   input gradient dX = dY What   + s (dY B) A           (the base is frozen: no dW, Sec. 3)
//
// What is never written to HBM: every workgroup decodes the slice of the packed codes it needs
// (App. A.2: unpack, per-channel table lookup, multiply by the group absmax, round to bf16 -- the
// same arithmetic as the stand-alone dequantize kernel) straight into the LDS tile that feeds
// v_mfma_f32_32x32x16_bf16.  The LoRA term rides in the same kernel as a K-extension: the
// contraction runs over [x | s x A^T] against [What | B] (forward) and over [dY | s dY B]
// against [What ; A] (backward), with the rank-r intermediate produced by a small MFMA kernel.
//
// Tile: 256 x 256 outputs per workgroup, 64-deep contraction steps, 4 wavefronts in a 2 x 2
// grid, each owning 128 x 128 = 4 x 4 MFMA tiles (256 accumulator registers).
#include <cstdlib>

#include "gemm_common.h"

namespace lowra {

hipError_t launch_gemm_fwd(const GemmParams& p, hipStream_t st);

constexpr int LDS_LD = 72;   // bf16 per LDS row of the backward kernel: 64 + 8 pad

// ---- activation tile: 256 rows x 64 bf16, thread -> (16-byte chunk = tid&7, rows tid>>3 + 32 i)
__device__ __forceinline__ void load_act_tile(uint4 (&ra)[8], const uint16_t* src, int ld, int rows_valid,
                                              int row0, int col0, int cols_valid) {
    const int chunk = threadIdx.x & 7;
    const int col = col0 + chunk * 8;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int m = row0 + (threadIdx.x >> 3) + 32 * i;
        ra[i] = (m < rows_valid && col < cols_valid)
                    ? *reinterpret_cast<const uint4*>(src + (size_t)m * ld + col)
                    : zero4();
    }
}
__device__ __forceinline__ void store_act_tile(uint16_t* sA, const uint4 (&ra)[8]) {
    const int chunk = threadIdx.x & 7;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int row = (threadIdx.x >> 3) + 32 * i;
        *reinterpret_cast<uint4*>(sA + row * LDS_LD + chunk * 8) = ra[i];
    }
}

// ---- the MFMA part of one 64-deep step
__device__ __forceinline__ void mma_step(const uint16_t* sA, const uint16_t* sB, floatx16_t (&acc)[4][4]) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const uint16_t* pa = sA + (wm * 128 + (lane & 31)) * LDS_LD + (lane >> 5) * 8;
    const uint16_t* pb = sB + (wn * 128 + (lane & 31)) * LDS_LD + (lane >> 5) * 8;
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
        bf16x8_t a[4], b[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            a[t] = *reinterpret_cast<const bf16x8_t*>(pa + t * 32 * LDS_LD + kk * 16);
            b[t] = *reinterpret_cast<const bf16x8_t*>(pb + t * 32 * LDS_LD + kk * 16);
        }
#pragma unroll
        for (int tm = 0; tm < 4; ++tm)
#pragma unroll
            for (int tn = 0; tn < 4; ++tn)
                acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[tm], b[tn], acc[tm][tn], 0, 0, 0);
    }
}

// =====================================================================================
// backward: contraction over output channels n.  Thread (rb = tid&7, kc = tid>>3) decodes an
// 8 (rows n) x 8 (columns k) block per step and writes it transposed, so the LDS tile is
// [k][n] with n contiguous, the order the MFMA operand wants.
// =====================================================================================
__global__ __launch_bounds__(NTHREADS) void linear_bwd_kernel(GemmParams p) {
    extern __shared__ __align__(16) uint8_t smem[];
    uint16_t* sA = reinterpret_cast<uint16_t*>(smem);
    uint16_t* sB = sA + BM * LDS_LD;
    float* sT = reinterpret_cast<float*>(sB + BN * LDS_LD);   // [64][TAB_LD]

    const int tid = threadIdx.x;
    const int k0 = blockIdx.x * BN, m0 = blockIdx.y * BM;
    const int rb = tid & 7, kc = tid >> 3;
    const int kcol = k0 + kc * 8;                   // my 8 output columns
    const bool k_ok = kcol < p.K;
    const int nt_main = (p.N + BK - 1) / BK, nt_all = nt_main + p.RP / BK;
    const int trow = tid >> 2, tpart = tid & 3;     // table staging: 64 rows x 4 float4

    uint4 ra[8];
    RowInfo rin[8], rin_t;                          // row records one step ahead of the codes
    uint32_t rcode[8], rbits[8];
    float rsc[8];
    float4 rtab = make_float4(0, 0, 0, 0);

    auto load_rows = [&](int nt) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int n = nt * BK + rb * 8 + i;
            rin[i].offset = 0; rin[i].bits_cb = 1;
            if (nt < nt_main && n < p.N) rin[i] = p.rows[n];
        }
        const int n = nt * BK + trow;
        rin_t.offset = 0; rin_t.bits_cb = 1;
        if (nt < nt_main && n < p.N) rin_t = p.rows[n];
    };
    auto load_tile = [&](int nt) {   // uses rin / rin_t loaded for this nt
        if (nt < nt_main) {
            load_act_tile(ra, p.act, p.N, p.M, m0, nt * BK, p.N);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int n = nt * BK + rb * 8 + i;
                const bool ok = k_ok && n < p.N;
                rbits[i] = rin[i].bits();
                rcode[i] = ok ? load_codes8(p.packed + rin[i].offset, kcol >> 3, rin[i].bits()) : 0u;
                rsc[i] = ok ? p.absmax[(size_t)n * p.G + (kcol >> 6)] : 0.0f;
            }
            const int n = nt * BK + trow;
            rtab = (n < p.N) ? reinterpret_cast<const float4*>(p.mappings + (size_t)rin_t.cb() * kTableStride)[tpart]
                             : make_float4(0, 0, 0, 0);
        } else {
            load_act_tile(ra, p.ext_act, p.RP, p.M, m0, (nt - nt_main) * BK, p.RP);
        }
    };
    auto store_tile = [&](int nt) {
        store_act_tile(sA, ra);
        if (nt < nt_main) {
            float* t = sT + trow * TAB_LD + tpart * 4;
            t[0] = rtab.x; t[1] = rtab.y; t[2] = rtab.z; t[3] = rtab.w;
            __syncthreads();
            float w[8][8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float* tab = sT + (rb * 8 + i) * TAB_LD;
                const uint32_t b = rbits[i], mask = (1u << b) - 1u;
#pragma unroll
                for (int j = 0; j < 8; ++j) w[i][j] = tab[(rcode[i] >> (j * b)) & mask] * rsc[i];
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                uint4 v;
                v.x = pack_bf16x2(w[0][j], w[1][j]);
                v.y = pack_bf16x2(w[2][j], w[3][j]);
                v.z = pack_bf16x2(w[4][j], w[5][j]);
                v.w = pack_bf16x2(w[6][j], w[7][j]);
                *reinterpret_cast<uint4*>(sB + (kc * 8 + j) * LDS_LD + rb * 8) = v;
            }
        } else {   // LoRA extension: LDS row k_local = tid holds A^T[k0 + tid][64 padded ranks]
            const int k = k0 + tid;
            const uint4* s = reinterpret_cast<const uint4*>(p.ext_w + (size_t)(k < p.K ? k : 0) * p.RP + (nt - nt_main) * BK);
            uint4* dst = reinterpret_cast<uint4*>(sB + tid * LDS_LD);
#pragma unroll
            for (int i = 0; i < 8; ++i) dst[i] = (k < p.K) ? s[i] : zero4();
        }
    };

    floatx16_t acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    load_rows(0);
    load_tile(0);
    load_rows(1);
    for (int nt = 0; nt < nt_all; ++nt) {
        store_tile(nt);
        __syncthreads();
        if (nt + 1 < nt_all) {
            load_tile(nt + 1);
            load_rows(nt + 2);
        }
        mma_step(sA, sB, acc);
        __syncthreads();
    }
    store_out(acc, p.out, p.K, p.M, p.K, m0, k0);
}

// =====================================================================================
// rank-r side products and operand preparation
// =====================================================================================
// out[m][j] = bf16( s * sum_c P[m][c] Q[j][c] ), j < RP (rows j >= r of Q count as zero).
// One workgroup per 32 token rows; its 4 wavefronts split the contraction and meet in LDS.
template <int CT>
__global__ __launch_bounds__(NTHREADS) void skinny_nt_kernel(const uint16_t* __restrict__ P, int ldp, int M,
                                                            const uint16_t* __restrict__ Q, int ldq, int r,
                                                            int Kc, float s, uint16_t* __restrict__ out) {
    extern __shared__ __align__(16) uint8_t smem[];
    float* red = reinterpret_cast<float*>(smem);   // [4][32][CT*32]
    constexpr int RP = CT * 32;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 31, kg = lane >> 5;
    const int m = blockIdx.x * 32 + i;
    floatx16_t acc[CT];
#pragma unroll
    for (int c = 0; c < CT; ++c)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[c][v] = 0.0f;
    const bf16x8_t zero = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll 2
    for (int k = wave * 16; k < Kc; k += 64) {
        const int kk = k + kg * 8;
        const bool kin = kk < Kc;
        const bf16x8_t a = (m < M && kin) ? *reinterpret_cast<const bf16x8_t*>(P + (size_t)m * ldp + kk) : zero;
#pragma unroll
        for (int c = 0; c < CT; ++c) {
            const int j = c * 32 + i;
            const bf16x8_t b = (j < r && kin) ? *reinterpret_cast<const bf16x8_t*>(Q + (size_t)j * ldq + kk) : zero;
            acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[c], 0, 0, 0);
        }
    }
#pragma unroll
    for (int c = 0; c < CT; ++c)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = 8 * (v >> 2) + 4 * kg + (v & 3);
            red[(wave * 32 + row) * RP + c * 32 + i] = acc[c][v];
        }
    __syncthreads();
    for (int idx = threadIdx.x; idx < 32 * RP; idx += NTHREADS) {
        const int row = idx / RP, col = idx % RP;
        const float v = red[(0 * 32 + row) * RP + col] + red[(1 * 32 + row) * RP + col] +
                        red[(2 * 32 + row) * RP + col] + red[(3 * 32 + row) * RP + col];
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
// dst [DR, DC]: dst[a][b] = src[b][a] for a < c, b < R, else 0  (src is [R, c]).
__global__ void transpose_pad_kernel(const uint16_t* __restrict__ src, int R, int c, uint16_t* __restrict__ dst,
                                     int DR, int DC) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)DR * DC) return;
    const int a = (int)(idx / DC), b = (int)(idx % DC);
    dst[idx] = (a < c && b < R) ? src[(size_t)b * c + a] : (uint16_t)0;
}

// measurement hook (lowra_set_kernel_timer): events recorded around the dominant kernel only
static hipEvent_t g_timer_start = nullptr, g_timer_stop = nullptr;
void set_kernel_timer(hipEvent_t start, hipEvent_t stop) { g_timer_start = start; g_timer_stop = stop; }
struct KernelTimer {
    hipStream_t st;
    explicit KernelTimer(hipStream_t s) : st(s) { if (g_timer_start) (void)hipEventRecord(g_timer_start, st); }
    ~KernelTimer() { if (g_timer_stop) (void)hipEventRecord(g_timer_stop, st); }
};

static inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }
static inline int round_up(int v, int m) { return (v + m - 1) / m * m; }

size_t linear_workspace_bytes(const lowra_layout& L, int op, int M, int r) {
    if (r <= 0) return 0;
    const size_t RP = (size_t)round_up(r, BK);
    const size_t t = align256((size_t)M * RP * 2);
    if (op == 0) return t + align256((size_t)L.N * RP * 2);
    return t + align256(RP * (size_t)L.N * 2) + align256((size_t)L.K * RP * 2);
}

static hipError_t launch_skinny(const uint16_t* P, int ldp, int M, const uint16_t* Q, int ldq, int r, int Kc,
                                float s, uint16_t* out, int RP, hipStream_t st) {
    const dim3 grid((M + 31) / 32), block(NTHREADS);
    const size_t sh = (size_t)4 * 32 * RP * sizeof(float);
    if (RP == 64) skinny_nt_kernel<2><<<grid, block, sh, st>>>(P, ldp, M, Q, ldq, r, Kc, s, out);
    else skinny_nt_kernel<4><<<grid, block, sh, st>>>(P, ldp, M, Q, ldq, r, Kc, s, out);
    return hipGetLastError();
}

static constexpr size_t kGemmSmem = (size_t)(BM + BN) * LDS_LD * 2 + (size_t)BN * TAB_LD * 4;

static hipError_t ensure_smem_attr() {
    static hipError_t st = [] {
        return hipFuncSetAttribute(reinterpret_cast<const void*>(linear_bwd_kernel),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)kGemmSmem);
    }();
    return st;
}

hipError_t launch_linear_fwd(const lowra_layout& L, const LinearArgs& a, int path, hipStream_t st) {
    (void)path;
    if (a.M == 0 || L.N == 0) return hipSuccess;
    hipError_t e = ensure_smem_attr();
    if (e != hipSuccess) return e;
    const int RP = a.r > 0 ? round_up(a.r, BK) : 0;
    uint16_t* ws_t = static_cast<uint16_t*>(a.workspace);
    uint16_t* ws_b = RP ? reinterpret_cast<uint16_t*>(static_cast<uint8_t*>(a.workspace) + align256((size_t)a.M * RP * 2)) : nullptr;
    if (RP) {
        e = launch_skinny(a.act, L.K, a.M, a.A, L.K, a.r, L.K, a.s, ws_t, RP, st);
        if (e != hipSuccess) return e;
        const size_t tot = (size_t)L.N * RP;
        pad_cols_kernel<<<dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, st>>>(a.B, L.N, a.r, ws_b, RP);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    GemmParams p;
    p.rows = L.d_rows; p.tile_order = L.d_tile_order; p.packed = a.packed; p.absmax = a.absmax;
    p.mappings = a.mappings; p.act = a.act; p.ext_act = ws_t; p.ext_w = ws_b; p.out = a.out;
    p.M = a.M; p.N = L.N; p.K = L.K; p.G = L.G; p.RP = RP;
    KernelTimer timer(st);
    return launch_gemm_fwd(p, st);
}

hipError_t launch_linear_bwd_input(const lowra_layout& L, const LinearArgs& a, int path, hipStream_t st) {
    (void)path;
    if (a.M == 0) return hipSuccess;
    hipError_t e = ensure_smem_attr();
    if (e != hipSuccess) return e;
    const int RP = a.r > 0 ? round_up(a.r, BK) : 0;
    uint8_t* ws = static_cast<uint8_t*>(a.workspace);
    uint16_t* ws_u = reinterpret_cast<uint16_t*>(ws);
    uint16_t* ws_bt = RP ? reinterpret_cast<uint16_t*>(ws + align256((size_t)a.M * RP * 2)) : nullptr;
    uint16_t* ws_at = RP ? reinterpret_cast<uint16_t*>(ws + align256((size_t)a.M * RP * 2) + align256((size_t)RP * L.N * 2)) : nullptr;
    if (RP) {
        size_t tot = (size_t)RP * L.N;   // B^T padded: [RP, N]
        transpose_pad_kernel<<<dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, st>>>(a.B, L.N, a.r, ws_bt, RP, L.N);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        tot = (size_t)L.K * RP;          // A^T padded: [K, RP]
        transpose_pad_kernel<<<dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, st>>>(a.A, a.r, L.K, ws_at, L.K, RP);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        e = launch_skinny(a.act, L.N, a.M, ws_bt, L.N, a.r, L.N, a.s, ws_u, RP, st);
        if (e != hipSuccess) return e;
    }
    GemmParams p;
    p.rows = L.d_rows; p.tile_order = nullptr; p.packed = a.packed; p.absmax = a.absmax;
    p.mappings = a.mappings; p.act = a.act; p.ext_act = ws_u; p.ext_w = ws_at; p.out = a.out;
    p.M = a.M; p.N = L.N; p.K = L.K; p.G = L.G; p.RP = RP;
    const dim3 grid((L.K + BN - 1) / BN, (a.M + BM - 1) / BM);
    KernelTimer timer(st);
    linear_bwd_kernel<<<grid, dim3(NTHREADS), kGemmSmem, st>>>(p);
    return hipGetLastError();
}

}  // namespace lowra
