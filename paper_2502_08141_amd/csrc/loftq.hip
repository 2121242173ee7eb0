// Alternating low-rank initialisation of the adapter (Sec. 4.1, "Using LoftQ as low-rank
// initializer"; App. D): starting from B A = 0, every step quantizes the residual W - B A with the
// layer's widths and tables and then fits B A to what the quantized weights miss, E = W - What.
//
// The paper takes the rank-r fit from an SVD.  Here it is a block power (subspace) iteration, which
// only needs products with E and E^T -- the two tall-skinny kernels this library already has:
//   Y = E A^T   [N, r]   (lora_side.hip, contraction over the input features)
//   Z = Y^T E   [r, K]   (adapter_grads.hip, contraction over the channels)
//   A <- rows of Z made orthonormal (Gram matrix, Cholesky factor, triangular solve: below)
// and, after the last round, B = E A^T, so that B A is the projection of E onto the row space
// found.  The start is a random A the caller passes in; later steps start from the previous
// step's A, whose row space hardly moves between steps.  E, Y, A and B are bf16 (B and A are what
// the linear calls consume), Z and the orthonormalisation are fp32 / fp64.
#include <algorithm>

#include "gemm_common.h"

namespace lowra {

hipError_t launch_skinny(const uint16_t* P, int ldp, int M, const uint16_t* Q, int ldq, int r, int Kc,
                         float s, uint16_t* out, int RP, hipStream_t st);
size_t tn_partial_bytes(int C, int M, int RP);
hipError_t launch_tn_skinny(const uint16_t* P, int C, int M, const uint16_t* Q, int RP, int r, int transposed,
                            float* partial, float* out, hipStream_t st);

constexpr int LQ_RP = 64;      // rank padded to the side products' row length
constexpr int LQ_GCH = 128;    // columns of Z per partial Gram matrix

// ---- F = W - Y At^T: Y [N][64] bf16 (B, padded with zero columns), At [K][64] bf16 (A^T, padded)
// A wavefront owns 32 channels x 128 input features: its 32 x 64 piece of Y stays in registers,
// each 32 x 32 tile is 4 MFMAs, W is read and F written in 128-byte segments, 4 side by side per row.
__global__ __launch_bounds__(256) void residual_kernel(const float* __restrict__ W, const uint16_t* __restrict__ Y,
                                                       const uint16_t* __restrict__ At, float* __restrict__ F, int N, int K) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 31, h = lane >> 5;
    const int n0 = blockIdx.x * 32;
    const int kbase = blockIdx.y * 512 + wave * 128;
    if (kbase >= K) return;                                        // whole wavefront; the kernel has no barrier
    const int nrow = min(n0 + i, N - 1);                           // rows past N: a valid row, never stored
    bf16x8_t yf[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) yf[kk] = *reinterpret_cast<const bf16x8_t*>(Y + (size_t)nrow * LQ_RP + 16 * kk + 8 * h);
    // K is a multiple of 64: a 32-wide tile is in or out as a whole
    floatx16_t acc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.0f;
        const int kr = min(kbase + 32 * t + i, K - 1);               // a tile past K: valid rows of At, result unused
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const bf16x8_t af = *reinterpret_cast<const bf16x8_t*>(At + (size_t)kr * LQ_RP + 16 * kk + 8 * h);
            acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(yf[kk], af, acc[t], 0, 0, 0);
        }
    }
    // acc[t][v] = (Y At^T)[n0 + 8 (v/4) + 4 h + v%4][kbase + 32 t + i]: row by row, the wavefront's 4 tiles side by side
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int n = n0 + 8 * (v >> 2) + 4 * h + (v & 3);
        if (n < N) {
            float w[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) w[t] = kbase + 32 * t < K ? W[(size_t)n * K + kbase + 32 * t + i] : 0.0f;
#pragma unroll
            for (int t = 0; t < 4; ++t)
                if (kbase + 32 * t < K) F[(size_t)n * K + kbase + 32 * t + i] = w[t] - acc[t][v];
        }
    }
}

// ---- E = bf16(W - What), What decoded on the fly (App. A.2: table level times the group's absmax, fp32):
// one workgroup per channel, 8 weights per lane and pass; nothing but E is written.
__global__ __launch_bounds__(256) void residual_of_decode_kernel(const RowInfo* __restrict__ rows, const uint8_t* __restrict__ packed,
                                                                 const float* __restrict__ absmax, const float* __restrict__ mappings,
                                                                 const float* __restrict__ W, uint16_t* __restrict__ E, int K) {
    __shared__ float tab[kTableStride];
    const int n = blockIdx.x, tid = threadIdx.x, units = K >> 3;
    const RowInfo ri = rows[n];
    const int bits = ri.bits();
    if (tid < kTableStride) tab[tid] = mappings[(size_t)ri.cb() * kTableStride + tid];
    __syncthreads();
    const uint8_t* row = packed + ri.offset;
    const float* am = absmax + (size_t)n * (K / kGroup);
    const float4* w4 = reinterpret_cast<const float4*>(W + (size_t)n * K);
    uint4* e4 = reinterpret_cast<uint4*>(E + (size_t)n * K);
    const uint32_t mask = (1u << bits) - 1u;
    for (int base = 0; base < units; base += 512) {
        uint32_t c[2];
        float a[2];
        float4 w[2][2];
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int u = min(base + tid + q * 256, units - 1);          // past the row's end: in bounds, never stored
            c[q] = load_codes8(row, u, bits);
            a[q] = am[u >> 3];
            w[q][0] = w4[2 * u]; w[q][1] = w4[2 * u + 1];
        }
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int u = base + tid + q * 256;
            if (u < units) {
                float d[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) d[i] = tab[(c[q] >> (i * bits)) & mask] * a[q];
                e4[u] = make_uint4(pack_bf16x2(w[q][0].x - d[0], w[q][0].y - d[1]), pack_bf16x2(w[q][0].z - d[2], w[q][0].w - d[3]),
                                   pack_bf16x2(w[q][1].x - d[4], w[q][1].y - d[5]), pack_bf16x2(w[q][1].z - d[6], w[q][1].w - d[7]));
            }
        }
    }
}

// ---- partial Gram matrices of Z [r][K]: the sum over a chunk's columns of Z[i][k] Z[j][k] (fp64), kept block by block:
// Gp[chunk][16 bj + bi][4 u + v] is entry (4 bi + u, 4 bj + v), so that the thread of the factorisation that owns a
// 4 x 4 block reads one 128-byte line per chunk.  Only the blocks on and below the diagonal are written or read.
// One workgroup per (chunk, band of 16 rows): the contraction is bound by a compute unit's fp64 rate, so the 64 x 64
// outputs of a chunk are dealt over four workgroups.  Wavefront w takes the chunk's columns [32 w, 32 w + 32), lane
// (bi, bj) the 4 x 4 block of rows 16 band + 4 bi.., columns 4 bj.. ; the four wavefronts' sums meet in LDS and are
// added in wavefront order.
__global__ __launch_bounds__(256) void gram_kernel(const float* __restrict__ Z, int K, int r, double* __restrict__ Gp) {
    constexpr int ZS = 68;                                           // row stride of zt: 16-byte aligned rows
    __shared__ __align__(16) float zt[LQ_GCH * ZS];                  // zt[k][i], the chunk transposed
    __shared__ double comb[3][16][64];                               // [wavefront - 1][element][lane]
    const int chunk = blockIdx.x >> 2, band = blockIdx.x & 3;
    const int c0 = chunk * LQ_GCH, tid = threadIdx.x;
    const int lc = (tid & 31) * 4;                                   // my four columns of a row
#pragma unroll
    for (int p = 0; p < 8; ++p) {
        const int i = (tid >> 5) + 8 * p;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (i < r) {
            const float* src = Z + (size_t)i * K + c0 + lc;
            if (c0 + lc < K) v = *reinterpret_cast<const float4*>(src);      // K is a multiple of 64
        }
        zt[(lc + 0) * ZS + i] = v.x; zt[(lc + 1) * ZS + i] = v.y; zt[(lc + 2) * ZS + i] = v.z; zt[(lc + 3) * ZS + i] = v.w;
    }
    __syncthreads();
    const int wave = tid >> 6, lane = tid & 63, bi = lane >> 4, bj = lane & 15;
    const int row0 = 16 * band + 4 * bi;
    double g[4][4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) g[u][v] = 0.0;
    if (4 * bj <= row0) {                                            // blocks above the diagonal: nothing to do
        const float* za = zt + (32 * wave) * ZS + row0;
        const float* zb = zt + (32 * wave) * ZS + 4 * bj;
#pragma unroll 4
        for (int k = 0; k < 32; ++k) {
            const float4 a4 = *reinterpret_cast<const float4*>(za + k * ZS);
            const float4 b4 = *reinterpret_cast<const float4*>(zb + k * ZS);
            const double a[4] = {a4.x, a4.y, a4.z, a4.w}, b[4] = {b4.x, b4.y, b4.z, b4.w};
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int v = 0; v < 4; ++v) g[u][v] = fma(a[u], b[v], g[u][v]);
        }
    }
    if (wave > 0) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int v = 0; v < 4; ++v) comb[wave - 1][4 * u + v][lane] = g[u][v];
    }
    __syncthreads();
    if (wave == 0 && 4 * bj <= row0) {
        double* out = Gp + (size_t)chunk * 4096 + (16 * bj + 4 * band + bi) * 16;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            double4 o;
            o.x = ((g[u][0] + comb[0][4 * u + 0][lane]) + comb[1][4 * u + 0][lane]) + comb[2][4 * u + 0][lane];
            o.y = ((g[u][1] + comb[0][4 * u + 1][lane]) + comb[1][4 * u + 1][lane]) + comb[2][4 * u + 1][lane];
            o.z = ((g[u][2] + comb[0][4 * u + 2][lane]) + comb[1][4 * u + 2][lane]) + comb[2][4 * u + 2][lane];
            o.w = ((g[u][3] + comb[0][4 * u + 3][lane]) + comb[1][4 * u + 3][lane]) + comb[2][4 * u + 3][lane];
            *reinterpret_cast<double4*>(out + 4 * u) = o;
        }
    }
}

// ---- G = the sum of the partial matrices, entry by entry in chunk order, in the same block-by-block layout.  A kernel
// of its own because one compute unit fetches about 30 GB/s: the 0.5 MB of partial matrices took the factorisation's
// single workgroup 18 us, half of its time; spread over the chip the sum is a microsecond.
__global__ __launch_bounds__(64) void gram_sum_kernel(const double* __restrict__ Gp, int chunks, double* __restrict__ G) {
    const int e = blockIdx.x * 64 + threadIdx.x;                     // entry 4 u + v of block 16 bj + bi
    const int bj = e >> 8, bi = (e >> 4) & 15;
    if (bj > bi) return;
    double sum = 0.0;
    for (int c0 = 0; c0 < chunks; c0 += 16) {
        double part[16];
#pragma unroll
        for (int q = 0; q < 16; ++q) part[q] = Gp[(size_t)(c0 + q < chunks ? c0 + q : chunks - 1) * 4096 + e];
#pragma unroll
        for (int q = 0; q < 16; ++q)
            if (c0 + q < chunks) sum += part[q];
    }
    G[e] = sum;
}

// ---- G = L L^T (fp64, one workgroup).  Output Lf fp32 [64][64]: L below the
// diagonal, 1 / L[i][i] on it, zero elsewhere.  A pivot that vanishes (a row of Z inside the span of
// the earlier ones, a row >= r, or Z = 0) gets a zero column and a zero reciprocal: that row of A
// comes out zero and the rest stays orthonormal.
// Thread (bi, bj) keeps the 4 x 4 block of rows 4 bi.., columns 4 bj.. in registers for the whole
// right-looking factorisation (blocks above the diagonal hold nothing of use), which goes by panels of four
// columns: the sixteen owners of a panel -- neighbouring lanes of one wavefront, the diagonal block among them,
// so that its ten entries reach them by lane reads -- factor the diagonal block (every lane the same
// arithmetic) and solve their own four rows against it, then publish the four columns through LDS (double
// buffered: ONE barrier per panel); every thread whose block lies right of the panel, on or below the diagonal,
// subtracts the rank-4 product.  Published rows up to the panel's last are zero, so that this update needs no
// test per entry, and what it writes above the diagonal of a diagonal block is never read.
// 1 / d for d > 0 from the hardware's approximation and two Newton steps (about 1e-15 relative), 1 / sqrt(d) with
// one step (about 1e-13; the factor is rounded to fp32 afterwards): the library's correctly rounded division and
// square root are some forty instructions each, and four square roots sit on the critical path of every panel.
__device__ __forceinline__ double lq_rcp(double d) {
    double r = __builtin_amdgcn_rcp(d);
    r = r * fma(-d, r, 2.0);
    return r * fma(-d, r, 2.0);
}
__device__ __forceinline__ double lq_rsqrt(double d) {
    const double r = __builtin_amdgcn_rsq(d);
    return r * fma(-0.5 * d * r, r, 1.5);
}

// v of lane `lane` (the same for the whole wavefront) as a wavefront-uniform value
__device__ __forceinline__ double lq_readlane(double v, int lane) {
    const unsigned long long b = (unsigned long long)__double_as_longlong(v);
    const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)b, lane);
    const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(b >> 32), lane);
    return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}

__global__ __launch_bounds__(256) void chol_kernel(const double* __restrict__ G, float* __restrict__ Lf) {
    __shared__ __align__(16) double col[2][4][64];                   // [buffer][column of the panel][row]
    __shared__ double diag[64];
    // the sixteen owners of a block column are sixteen neighbouring lanes of one wavefront
    const int tid = threadIdx.x, bj = tid >> 4, bi = tid & 15;
    double g[4][4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) g[u][v] = 0.0;
    if (bj <= bi) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const double4 row = *reinterpret_cast<const double4*>(G + tid * 16 + 4 * u);
            g[u][0] = row.x; g[u][1] = row.y; g[u][2] = row.z; g[u][3] = row.w;
        }
    }
    if (bi == bj) {
#pragma unroll
        for (int u = 0; u < 4; ++u) diag[4 * bi + u] = g[u][u];
    }
    __syncthreads();
    double maxdiag = 0.0;
    for (int i = 0; i < 64; ++i) maxdiag = fmax(maxdiag, diag[i]);
    const double tiny = 1e-12 * maxdiag;
    for (int jb = 0; jb < 16; ++jb) {
        const int buf = jb & 1;
        // the diagonal block sits with thread (bi = jb, bj = jb), lane 16 (jb % 4) + jb of the owners' wavefront
        const int src = 16 * (jb & 3) + jb;
        double d[4][4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int v = 0; v <= u; ++v) d[u][v] = lq_readlane(g[u][v], src);
        if (bj == jb) {
            // L of the diagonal block, column by column; is[v] = 1 / L[v][v], or zero for a pivot that vanishes
            double is[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                double pv = d[v][v];
#pragma unroll
                for (int w = 0; w < v; ++w) pv = fma(-d[v][w], d[v][w], pv);
                is[v] = pv > tiny ? lq_rsqrt(pv) : 0.0;
                d[v][v] = pv * is[v];
#pragma unroll
                for (int u = v + 1; u < 4; ++u) {
                    double x = d[u][v];
#pragma unroll
                    for (int w = 0; w < v; ++w) x = fma(-d[u][w], d[v][w], x);
                    d[u][v] = x * is[v];
                }
            }
            // my four rows against it: y L^T = x, entry by entry; for the diagonal block itself this repeats the
            // factorisation (its entries on and below the diagonal are the ones kept)
            double y[4][4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    double x = g[u][v];
#pragma unroll
                    for (int w = 0; w < v; ++w) x = fma(-y[u][w], d[v][w], x);
                    y[u][v] = x * is[v];
                }
            // (entries above the diagonal, which this also overwrites, are never read)
            const bool below = bi > jb;                              // rows up to the panel's last are published as zero
#pragma unroll
            for (int v = 0; v < 4; ++v) {
#pragma unroll
                for (int u = 0; u < 4; ++u) g[u][v] = y[u][v];
                double2* dst = reinterpret_cast<double2*>(&col[buf][v][4 * bi]);
                if (below) { dst[0] = make_double2(y[0][v], y[1][v]); dst[1] = make_double2(y[2][v], y[3][v]); }
                else { dst[0] = make_double2(0.0, 0.0); dst[1] = make_double2(0.0, 0.0); }
            }
        }
        __syncthreads();
        if (bj <= jb || bi < bj) continue;                           // finished columns and blocks above the diagonal: nothing to update
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const double2 la = *reinterpret_cast<const double2*>(&col[buf][w][4 * bi]), lb = *reinterpret_cast<const double2*>(&col[buf][w][4 * bi + 2]);
            const double2 ka = *reinterpret_cast<const double2*>(&col[buf][w][4 * bj]), kb = *reinterpret_cast<const double2*>(&col[buf][w][4 * bj + 2]);
            const double li[4] = {la.x, la.y, lb.x, lb.y}, lk[4] = {ka.x, ka.y, kb.x, kb.y};
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int v = 0; v < 4; ++v) g[u][v] = fma(-li[u], lk[v], g[u][v]);
        }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        float o[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int i = 4 * bi + u, k = 4 * bj + v;
            o[v] = 0.0f;
            if (k < i) o[v] = (float)g[u][v];
            if (k == i) o[v] = g[u][v] > 0.0 ? (float)lq_rcp(g[u][v]) : 0.0f;
        }
        *reinterpret_cast<float4*>(Lf + (4 * bi + u) * 64 + 4 * bj) = make_float4(o[0], o[1], o[2], o[3]);
    }
}

// ---- A = L^-1 Z by forward substitution: orthonormal rows, written as bf16 [64][K] (rows >= r zero) and
// transposed, At [K][64].  One workgroup of eight wavefronts per 64 columns of Z, a lane per column, wavefront w
// the rows 8 w .. 8 w + 7.  In stage jb wavefront jb solves its 8 x 8 triangle and publishes its eight rows
// through LDS; the wavefronts below take that block's contribution off their rows (eight independent chains of
// multiply-adds) -- one column per lane alone would be a single chain of 2016 dependent operations per wavefront.
// L comes from LDS with the same address in every lane; a wavefront fetches the block of the next stage before it
// waits at the barrier.
constexpr int LQ_APPLY_THREADS = 512;
__global__ __launch_bounds__(LQ_APPLY_THREADS) void apply_kernel(const float* __restrict__ Z, const float* __restrict__ Lf, int K, int r,
                                                                 uint16_t* __restrict__ A, uint16_t* __restrict__ At) {
    __shared__ __align__(16) float Ls[64 * 64];
    __shared__ float as[64][64];                                     // as[row][lane]: finished rows of A
    const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int k = blockIdx.x * 64 + lane;
    const bool live = k < K;
    float s[8];
#pragma unroll
    for (int ii = 0; ii < 8; ++ii) s[ii] = (live && 8 * w + ii < r) ? Z[(size_t)(8 * w + ii) * K + k] : 0.0f;
#pragma unroll
    for (int q = 0; q < 2; ++q)
        reinterpret_cast<float4*>(Ls)[q * LQ_APPLY_THREADS + threadIdx.x] = reinterpret_cast<const float4*>(Lf)[q * LQ_APPLY_THREADS + threadIdx.x];
    __syncthreads();
    float ld[8][8], lb[8][8];                                        // my rows of L: the triangle's block, the current stage's block
    auto fetch = [&](float (&dst)[8][8], int cb) {
#pragma unroll
        for (int ii = 0; ii < 8; ++ii) {
            const float4 l0 = *reinterpret_cast<const float4*>(&Ls[(8 * w + ii) * 64 + 8 * cb]);
            const float4 l1 = *reinterpret_cast<const float4*>(&Ls[(8 * w + ii) * 64 + 8 * cb + 4]);
            dst[ii][0] = l0.x; dst[ii][1] = l0.y; dst[ii][2] = l0.z; dst[ii][3] = l0.w;
            dst[ii][4] = l1.x; dst[ii][5] = l1.y; dst[ii][6] = l1.z; dst[ii][7] = l1.w;
        }
    };
    fetch(ld, w);
    if (w > 0) fetch(lb, 0);
    for (int jb = 0; jb < 8; ++jb) {
        if (w == jb) {
            uint32_t pk[4];
#pragma unroll
            for (int ii = 0; ii < 8; ++ii) {
#pragma unroll
                for (int jj = 0; jj < ii; ++jj) s[ii] = fmaf(-ld[ii][jj], s[jj], s[ii]);
                s[ii] *= ld[ii][ii];                                 // the diagonal holds 1 / L[i][i]
                as[8 * w + ii][lane] = s[ii];
                const uint32_t b = pack_bf16x2(s[ii], 0.0f) & 0xffffu;
                if (live) A[(size_t)(8 * w + ii) * K + k] = (uint16_t)b;
                if (ii & 1) pk[ii >> 1] |= b << 16; else pk[ii >> 1] = b;
            }
            if (live) reinterpret_cast<uint4*>(At + (size_t)k * LQ_RP)[w] = make_uint4(pk[0], pk[1], pk[2], pk[3]);
        }
        __syncthreads();
        if (w > jb) {
            float aj[8];
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) aj[jj] = as[8 * jb + jj][lane];
#pragma unroll
            for (int jj = 0; jj < 8; ++jj)
#pragma unroll
                for (int ii = 0; ii < 8; ++ii) s[ii] = fmaf(-lb[ii][jj], aj[jj], s[ii]);
            if (jb + 1 < w) fetch(lb, jb + 1);
        }
    }
}

// dst [rows][cols] = src [rows][ld] restricted to its first `cols` columns
__global__ __launch_bounds__(256) void copy_cols_kernel(const uint16_t* __restrict__ src, int ld, size_t rows, int cols, uint16_t* __restrict__ dst) {
    const size_t tot = rows * (size_t)cols;
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < tot; e += (size_t)gridDim.x * 256)
        dst[e] = src[(e / cols) * ld + (e % cols)];
}

static inline size_t lq_align(size_t v) { return (v + 255) & ~(size_t)255; }

struct LoftqWs {
    size_t F, E, Y, Z, partial, Gp, G, Lf, A, At, total;
};
static LoftqWs loftq_ws(int N, int K) {
    LoftqWs w;
    size_t o = 0;
    w.F = o; o += lq_align((size_t)N * K * 4);
    w.E = o; o += lq_align((size_t)N * K * 2);
    w.Y = o; o += lq_align((size_t)N * LQ_RP * 2);
    w.Z = o; o += lq_align((size_t)LQ_RP * K * 4);
    w.partial = o; o += lq_align(tn_partial_bytes(K, N, LQ_RP));
    w.Gp = o; o += lq_align((size_t)((K + LQ_GCH - 1) / LQ_GCH) * 4096 * sizeof(double));
    w.G = o; o += lq_align(4096 * sizeof(double));
    w.Lf = o; o += lq_align(4096 * sizeof(float));
    w.A = o; o += lq_align((size_t)LQ_RP * K * 2);
    w.At = o; o += lq_align((size_t)K * LQ_RP * 2);
    w.total = o;
    return w;
}
size_t loftq_workspace_bytes(const lowra_layout& L, int r) { return r > 0 ? loftq_ws(L.N, L.K).total : 0; }

static unsigned lq_grid(size_t items) { return (unsigned)std::min<size_t>((items + 255) / 256, 16384); }

hipError_t launch_loftq(const lowra_layout& L, const float* W, const float* thresholds, const float* mappings, int r, int steps,
                        int iters, const uint16_t* omega, uint8_t* packed, float* absmax, uint16_t* A_out, uint16_t* B_out,
                        void* workspace, hipStream_t st) {
    const int N = L.N, K = L.K;
    hipError_t e;
    if (r == 0) return launch_quantize(L, W, thresholds, packed, absmax, st);      // nothing to fit: plain quantization
    const LoftqWs o = loftq_ws(N, K);
    uint8_t* ws = static_cast<uint8_t*>(workspace);
    float* F = reinterpret_cast<float*>(ws + o.F);
    uint16_t* E = reinterpret_cast<uint16_t*>(ws + o.E);
    uint16_t* Y = reinterpret_cast<uint16_t*>(ws + o.Y);
    float* Z = reinterpret_cast<float*>(ws + o.Z);
    float* partial = reinterpret_cast<float*>(ws + o.partial);
    double* Gp = reinterpret_cast<double*>(ws + o.Gp);
    double* G = reinterpret_cast<double*>(ws + o.G);
    float* Lf = reinterpret_cast<float*>(ws + o.Lf);
    uint16_t* A = reinterpret_cast<uint16_t*>(ws + o.A);
    uint16_t* At = reinterpret_cast<uint16_t*>(ws + o.At);
    const int chunks = (K + LQ_GCH - 1) / LQ_GCH;
    for (int t = 0; t < steps; ++t) {
        const float* src = W;
        if (t > 0) {                                                 // residual of the previous step's factors
            residual_kernel<<<dim3((N + 31) / 32, (K + 511) / 512), dim3(256), 0, st>>>(W, Y, At, F, N, K);
            if ((e = hipGetLastError()) != hipSuccess) return e;
            src = F;
        }
        if ((e = launch_quantize(L, src, thresholds, packed, absmax, st)) != hipSuccess) return e;
        residual_of_decode_kernel<<<dim3(N), dim3(256), 0, st>>>(L.d_rows, packed, absmax, mappings, W, E, K);   // E = W - What
        if ((e = hipGetLastError()) != hipSuccess) return e;
        const uint16_t* Aq = t == 0 ? omega : A;
        for (int it = 0; it < iters; ++it) {
            if ((e = launch_skinny(E, K, N, Aq, K, r, K, 1.0f, Y, LQ_RP, st)) != hipSuccess) return e;              // Y = E A^T
            if ((e = launch_tn_skinny(E, K, N, Y, LQ_RP, r, 1, partial, Z, st)) != hipSuccess) return e;            // Z = Y^T E
            gram_kernel<<<dim3(4 * chunks), dim3(256), 0, st>>>(Z, K, r, Gp);
            gram_sum_kernel<<<dim3(64), dim3(64), 0, st>>>(Gp, chunks, G);
            chol_kernel<<<dim3(1), dim3(256), 0, st>>>(G, Lf);
            apply_kernel<<<dim3((K + 63) / 64), dim3(LQ_APPLY_THREADS), 0, st>>>(Z, Lf, K, r, A, At);
            if ((e = hipGetLastError()) != hipSuccess) return e;
            Aq = A;
        }
        if ((e = launch_skinny(E, K, N, A, K, r, K, 1.0f, Y, LQ_RP, st)) != hipSuccess) return e;                  // B = E A^T
    }
    copy_cols_kernel<<<dim3(lq_grid((size_t)r * K)), dim3(256), 0, st>>>(A, K, (size_t)r, K, A_out);
    copy_cols_kernel<<<dim3(lq_grid((size_t)N * r)), dim3(256), 0, st>>>(Y, LQ_RP, (size_t)N, r, B_out);
    return hipGetLastError();
}

}  // namespace lowra
