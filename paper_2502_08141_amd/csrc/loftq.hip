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

// ---- partial Gram matrices of Z [r][K]: Gp[chunk][i][j] = sum over the chunk's columns of Z[i][k] Z[j][k] (fp64)
__global__ __launch_bounds__(256) void gram_kernel(const float* __restrict__ Z, int K, int r, double* __restrict__ Gp) {
    __shared__ float zt[64][LQ_GCH + 1];
    const int c0 = blockIdx.x * LQ_GCH;
    for (int e = threadIdx.x; e < 64 * LQ_GCH; e += 256) {
        const int i = e / LQ_GCH, k = e % LQ_GCH;
        zt[i][k] = (i < r && c0 + k < K) ? Z[(size_t)i * K + c0 + k] : 0.0f;
    }
    __syncthreads();
    const int bi = threadIdx.x >> 4, bj = threadIdx.x & 15;        // my 4 x 4 block of the 64 x 64 matrix
    double g[4][4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) g[u][v] = 0.0;
    for (int k = 0; k < LQ_GCH; ++k) {
        float a[4], b[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) { a[u] = zt[4 * bi + u][k]; b[u] = zt[4 * bj + u][k]; }
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int v = 0; v < 4; ++v) g[u][v] += (double)a[u] * (double)b[v];
    }
    double* out = Gp + (size_t)blockIdx.x * 4096;
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) out[(4 * bi + u) * 64 + 4 * bj + v] = g[u][v];
}

// ---- G = sum of the partials = L L^T (fp64, one workgroup).  Output Lf fp32 [64][64]: L below the
// diagonal, 1 / L[i][i] on it, zero elsewhere.  A pivot that vanishes (a row of Z inside the span of
// the earlier ones, a row >= r, or Z = 0) gets a zero column and a zero reciprocal: that row of A
// comes out zero and the rest stays orthonormal.
// Thread (bi, bj) keeps the 4 x 4 block of rows 4 bi.., columns 4 bj.. in registers for the whole
// right-looking factorisation; per step only the pivot column travels through LDS (double buffered:
// one barrier per step).
// 1 / d and 1 / sqrt(d) for d > 0 from the hardware's approximations and two Newton steps each (about 1e-15
// relative): the library's correctly rounded division and square root are some forty instructions each, on the
// critical path of every one of the factorisation's 64 steps.
__device__ __forceinline__ double lq_rcp(double d) {
    double r = __builtin_amdgcn_rcp(d);
    r = r * (2.0 - d * r);
    return r * (2.0 - d * r);
}
__device__ __forceinline__ double lq_rsqrt(double d) {
    double r = __builtin_amdgcn_rsq(d);
    r = r * (1.5 - 0.5 * d * r * r);
    return r * (1.5 - 0.5 * d * r * r);
}

__global__ __launch_bounds__(256) void chol_kernel(const double* __restrict__ Gp, int chunks, float* __restrict__ Lf) {
    __shared__ double col[2][64];
    __shared__ double diag[64];
    const int tid = threadIdx.x, bi = tid >> 4, bj = tid & 15;
    double g[4][4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) g[u][v] = 0.0;
    // the partial matrices, eight at a time with all their loads in flight together (one dependent round trip per
    // partial matrix made this sum half of the kernel's time); the order of the additions stays c = 0, 1, 2, ...
    for (int c0 = 0; c0 < chunks; c0 += 8) {
        double part[8][4][4];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int c = c0 + q < chunks ? c0 + q : chunks - 1;    // past the end: a valid matrix again, not added
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const double4 row = *reinterpret_cast<const double4*>(Gp + (size_t)c * 4096 + (4 * bi + u) * 64 + 4 * bj);
                part[q][u][0] = row.x; part[q][u][1] = row.y; part[q][u][2] = row.z; part[q][u][3] = row.w;
            }
        }
#pragma unroll
        for (int q = 0; q < 8; ++q)
            if (c0 + q < chunks) {
#pragma unroll
                for (int u = 0; u < 4; ++u)
#pragma unroll
                    for (int v = 0; v < 4; ++v) g[u][v] += part[q][u][v];
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
#pragma unroll
        for (int jo = 0; jo < 4; ++jo) {
            const int j = 4 * jb + jo, buf = jo & 1;
            if (bj == jb) {                                          // the owners of column j publish it
#pragma unroll
                for (int u = 0; u < 4; ++u) col[buf][4 * bi + u] = g[u][jo];
            }
            __syncthreads();
            const double d = col[buf][j];
            const bool ok = d > tiny;
            const double inv = ok ? lq_rcp(d) : 0.0;
            double ci[4], ck[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) { ci[u] = col[buf][4 * bi + u]; ck[u] = col[buf][4 * bj + u]; }
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int i = 4 * bi + u, k = 4 * bj + v;
                    if (k > j && i >= k) g[u][v] -= ci[u] * ck[v] * inv;
                }
            if (bj == jb) {
                const double isq = ok ? lq_rsqrt(d) : 0.0;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int i = 4 * bi + u;
                    if (i >= j) g[u][jo] = i == j ? d * isq : ci[u] * isq;
                }
            }
        }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int i = 4 * bi + u, k = 4 * bj + v;
            float o = 0.0f;
            if (k < i) o = (float)g[u][v];
            if (k == i) o = g[u][v] > 0.0 ? (float)(1.0 / g[u][v]) : 0.0f;
            Lf[i * 64 + k] = o;
        }
}

// ---- A = L^-1 Z by forward substitution, one column of Z per thread: orthonormal rows, written as
// bf16 [64][K] (rows >= r zero) and transposed, At [K][64]
__global__ __launch_bounds__(256) void apply_kernel(const float* __restrict__ Z, const float* __restrict__ Lf, int K, int r,
                                                    uint16_t* __restrict__ A, uint16_t* __restrict__ At) {
    __shared__ float Ls[64 * 64];
    for (int e = threadIdx.x; e < 4096; e += 256) Ls[e] = Lf[e];
    __syncthreads();
    const int k = blockIdx.x * 256 + threadIdx.x;
    if (k >= K) return;
    float a[64];
#pragma unroll
    for (int j = 0; j < 64; ++j) a[j] = j < r ? Z[(size_t)j * K + k] : 0.0f;
    uint32_t w[32];
#pragma unroll
    for (int i = 0; i < 64; ++i) {
        float s = a[i];
#pragma unroll
        for (int j = 0; j < i; ++j) s -= Ls[i * 64 + j] * a[j];
        a[i] = s * Ls[i * 64 + i];
        const uint32_t b = pack_bf16x2(a[i], 0.0f) & 0xffffu;
        A[(size_t)i * K + k] = (uint16_t)b;
        if (i & 1) w[i >> 1] |= b << 16; else w[i >> 1] = b;
    }
    uint4* dst = reinterpret_cast<uint4*>(At + (size_t)k * LQ_RP);
#pragma unroll
    for (int q = 0; q < 8; ++q) dst[q] = make_uint4(w[4 * q], w[4 * q + 1], w[4 * q + 2], w[4 * q + 3]);
}

// dst [rows][cols] = src [rows][ld] restricted to its first `cols` columns
__global__ __launch_bounds__(256) void copy_cols_kernel(const uint16_t* __restrict__ src, int ld, size_t rows, int cols, uint16_t* __restrict__ dst) {
    const size_t tot = rows * (size_t)cols;
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < tot; e += (size_t)gridDim.x * 256)
        dst[e] = src[(e / cols) * ld + (e % cols)];
}

static inline size_t lq_align(size_t v) { return (v + 255) & ~(size_t)255; }

struct LoftqWs {
    size_t F, E, Y, Z, partial, Gp, Lf, A, At, total;
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
            gram_kernel<<<dim3(chunks), dim3(256), 0, st>>>(Z, K, r, Gp);
            chol_kernel<<<dim3(1), dim3(256), 0, st>>>(Gp, chunks, Lf);
            apply_kernel<<<dim3((K + 255) / 256), dim3(256), 0, st>>>(Z, Lf, K, r, A, At);
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
