// Adapter gradients of the LoRA linear (Sec. 2.1; only the low-rank tensors are trained, Sec. 3):
//   dB[n,j] = sum_m dY[m,n] (s t)[m,j],  t = x A^T          dA[j,k] = sum_m (s u)[m,j] x[m,k],  u = dY B
// Both are "tall-skinny, contraction over the tokens": out[c][j] = sum_m P[m][c] Q[m][j] with P the
// big row-major activation matrix (dY or x, read once: HBM bound, 2 B per element) and Q the small
// rank-r intermediate [M][RP] that lora_side.hip already produces for the forward and the input
// gradient.
//
// Mapping: a workgroup owns 64 columns of P and a chunk of tokens; its 4 wavefronts take a quarter
// of the chunk each.  A wavefront stages [64 tokens][64 columns] of P and [64 tokens][RP] of Q in
// LDS by global->LDS DMA (double buffered, private to the wavefront: no barrier in the loop) and
// gets both MFMA operands -- 8 consecutive tokens of one column -- with transposing LDS reads
// (ds_read_b64_tr_b16), exactly as the input-gradient GEMM reads its weight tile.  The four partial
// tiles are added in LDS and written as fp32 partial sums per token chunk; a second small kernel
// adds the chunks in a fixed order and writes dB [N][r] or, transposed, dA [r][K].
#include <algorithm>

#include "gemm_common.h"

namespace lowra {

typedef short ag_v4i16_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) ag_v4i16_t* ag_lds_v4i16_ptr;

constexpr int AG_COLS = 64;                 // columns of P per workgroup
constexpr int AG_MT = 64;                   // tokens per stage
constexpr int AG_ROWB = 128;                // bytes per LDS row: 64 bf16
constexpr int AG_TILEB = AG_MT * AG_ROWB;   // 8 KB: one [64][64] bf16 tile

// 16-byte chunk c (0..7) of row r of a [64][64] bf16 tile: rows r and r+2 would share their banks,
// so the chunk's bit 2 is flipped on every other pair of rows.
__device__ __forceinline__ int ag_off(int r, int c) { return r * AG_ROWB + ((c ^ (((r >> 1) & 1) << 2)) << 4); }

// One product out = P^T Q of a launch: `tiles` column tiles x `chunks` token chunks = `nwg` workgroups.  A launch
// carries two (the adapter gradients' dB and dA: the second fills the compute units the first leaves idle, and
// no launch gap lies between them) or one (nwg of the second = 0).
struct TnProb {
    const uint16_t* P; const uint16_t* Q;
    float* partial; float* direct;       // direct: the result itself (single chunk), else null
    int C, chunk_rows, transposed, tiles, nwg;
};

template <int RT>   // RT = RP / 64: 64-wide tiles of Q
__global__ __launch_bounds__(256) void tn_skinny_kernel(const TnProb pa, const TnProb pb, int M, int r) {
    extern __shared__ __align__(16) uint8_t ag_smem[];
    constexpr int RP = RT * 64;
    constexpr int STAGEB_ = (1 + RT) * AG_TILEB;            // P tile + Q tiles
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lptr_t)ag_smem;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const bool second = (int)blockIdx.x >= pa.nwg;            // uniform: the fields below stay in scalar registers
    const uint16_t* __restrict__ P = second ? pb.P : pa.P;
    const uint16_t* __restrict__ Q = second ? pb.Q : pa.Q;
    float* __restrict__ partial = second ? pb.partial : pa.partial;
    float* __restrict__ direct = second ? pb.direct : pa.direct;
    const int C = second ? pb.C : pa.C, chunk_rows = second ? pb.chunk_rows : pa.chunk_rows;
    const int transposed = second ? pb.transposed : pa.transposed, tiles = second ? pb.tiles : pa.tiles;
    const int widx = (int)blockIdx.x - (second ? pa.nwg : 0);
    const int chunk = widx / tiles;
    const int c0 = (widx - chunk * tiles) * AG_COLS;
    const int m_lo = chunk * chunk_rows + wave * (chunk_rows / 4);
    const int m_hi = min(m_lo + chunk_rows / 4, M);
    const int nst = m_hi > m_lo ? (m_hi - m_lo + AG_MT - 1) / AG_MT : 0;
    uint8_t* wbase = ag_smem + wave * 2 * STAGEB_;
    const uint32_t wlds = lds0 + wave * 2 * STAGEB_;

    // DMA lane mapping: one instruction = 8 rows x 128 B; lane -> row 8 i + lane/8, physical chunk lane%8
    const int drow = lane >> 3, dch = lane & 7;
    const int last_chunk = C / 8 - 1;                         // C is a multiple of 8
    auto stage_in = [&](int st, int buf) {
        const int m0 = m_lo + st * AG_MT;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int r = 8 * i + drow;
            const int m = min(m0 + r, M - 1);                 // past the end: a valid row, its Q row is zeroed below
            const int lc = dch ^ (((r >> 1) & 1) << 2);       // logical chunk landing on my physical chunk
            const int gc = min(c0 / 8 + lc, last_chunk);      // past the last column: duplicates, never stored
            dma16(reinterpret_cast<const uint8_t*>(P) + ((size_t)m * C + (size_t)gc * 8) * 2, wlds + buf * STAGEB_ + i * 1024);
#pragma unroll
            for (int t = 0; t < RT; ++t)
                dma16(reinterpret_cast<const uint8_t*>(Q) + ((size_t)m * RP + (size_t)(t * 8 + lc) * 8) * 2,
                      wlds + buf * STAGEB_ + (1 + t) * AG_TILEB + i * 1024);
        }
    };

    floatx16_t acc[2][2 * RT];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2 * RT; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;

    // transposing read: lane -> (row 16 kk + 8 fkg + 4 eb + L/4, 8 bytes at column 32 tn + 16 grp + 4 (L%4))
    const int L = lane & 15, grp = (lane >> 4) & 1, fkg = lane >> 5;
    auto frag = [&](const uint8_t* tile, int kk, int tn) -> bf16x8_t {
        typedef short v8i16_t __attribute__((ext_vector_type(8)));
        ag_v4i16_t h[2];
#pragma unroll
        for (int eb = 0; eb < 2; ++eb) {
            const int row = kk * 16 + fkg * 8 + eb * 4 + (L >> 2);
            const int ch = tn * 4 + grp * 2 + ((L & 3) >> 1);
            const uint32_t a = lds0 + (uint32_t)(tile - ag_smem) + ag_off(row, ch) + (L & 1) * 8;
            h[eb] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((ag_lds_v4i16_ptr)(uintptr_t)a);
        }
        const v8i16_t v = {h[0][0], h[0][1], h[0][2], h[0][3], h[1][0], h[1][1], h[1][2], h[1][3]};
        return __builtin_bit_cast(bf16x8_t, v);
    };

    if (nst > 0) stage_in(0, 0);
    for (int st = 0; st < nst; ++st) {
        const int buf = st & 1;
        dma_wait_all();                                       // my stage has landed (transfers are private to the wavefront)
        if (st + 1 < nst) stage_in(st + 1, buf ^ 1);
        uint8_t* tp = wbase + buf * STAGEB_;
        // rows past the last token: zero their Q rows (P holds a valid, finite row there)
        const int valid = m_hi - (m_lo + st * AG_MT);
        if (valid < AG_MT) {
            for (int e = lane; e < AG_MT * 8 * RT; e += 64) {
                const int t = e / (AG_MT * 8), r = (e / 8) % AG_MT, c = e % 8;
                if (r >= valid) *reinterpret_cast<uint4*>(tp + (1 + t) * AG_TILEB + r * AG_ROWB + c * 16) = zero4();
            }
        }
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            bf16x8_t fp[2], fq[2 * RT];
#pragma unroll
            for (int tn = 0; tn < 2; ++tn) fp[tn] = frag(tp, kk, tn);
#pragma unroll
            for (int tq = 0; tq < 2 * RT; ++tq) fq[tq] = frag(tp + (1 + (tq >> 1)) * AG_TILEB, kk, tq & 1);
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < 2 * RT; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fp[a], fq[b], acc[a][b], 0, 0, 0);
        }
    }
    dma_wait_all();
    __syncthreads();
    // ---- sum of the four wavefronts in LDS ([64 cols][RP + 1] fp32 per wavefront: the odd stride keeps reads along
    // the columns off one bank), then the chunk's partial tile -- or, with a single chunk, the result itself
    constexpr int RS = RP + 1;
    float* red = reinterpret_cast<float*>(ag_smem) + wave * AG_COLS * RS;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2 * RT; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int col = 32 * a + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3), rk = 32 * b + (lane & 31);
                red[col * RS + rk] = acc[a][b][v];
            }
    __syncthreads();
    const float* r0 = reinterpret_cast<const float*>(ag_smem);
    auto sum4 = [&](int col, int rk) {
        const int o = col * RS + rk;
        return r0[o] + r0[AG_COLS * RS + o] + r0[2 * AG_COLS * RS + o] + r0[3 * AG_COLS * RS + o];
    };
    if (direct == nullptr) {
        float* out = partial + ((size_t)chunk * C) * RP;
        for (int e = threadIdx.x; e < AG_COLS * RP; e += 256) {
            const int col = e / RP, rk = e % RP;
            if (c0 + col < C) out[(size_t)(c0 + col) * RP + rk] = sum4(col, rk);
        }
    } else if (!transposed) {                                  // out [C][r]
        for (int e = threadIdx.x; e < AG_COLS * RP; e += 256) {
            const int col = e / RP, rk = e % RP;
            if (c0 + col < C && rk < r) direct[(size_t)(c0 + col) * r + rk] = sum4(col, rk);
        }
    } else {                                                   // out [r][C]: the stores run along the columns
        for (int e = threadIdx.x; e < AG_COLS * RP; e += 256) {
            const int rk = e / AG_COLS, col = e % AG_COLS;
            if (c0 + col < C && rk < r) direct[(size_t)rk * C + c0 + col] = sum4(col, rk);
        }
    }
}

// out[c][j] = sum over chunks of partial[chunk][c][j], j < r
__global__ __launch_bounds__(256) void tn_reduce_kernel(const float* __restrict__ partial, int nchunks, int C, int RP, int r,
                                                        float* __restrict__ out) {
    const size_t tot = (size_t)C * r;
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < tot; e += (size_t)gridDim.x * 256) {
        const int c = (int)(e / r), j = (int)(e % r);
        float s = 0.0f;
        for (int k = 0; k < nchunks; ++k) s += partial[((size_t)k * C + c) * RP + j];
        out[e] = s;
    }
}
// The same sum written transposed, out[j][c]: a workgroup takes 16 columns c, reads their partial rows as they lie
// (64 ranks = 256 contiguous bytes per column), and turns the tile through LDS so that the stores run along c too.
constexpr int AG_RT_COLS = 16;
__global__ __launch_bounds__(256) void tn_reduce_t_kernel(const float* __restrict__ partial, int nchunks, int C, int r,
                                                          float* __restrict__ out) {
    __shared__ float tile[AG_RT_COLS][65];
    const int c0 = blockIdx.x * AG_RT_COLS, tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    float s[AG_RT_COLS / 4];
#pragma unroll
    for (int q = 0; q < AG_RT_COLS / 4; ++q) s[q] = 0.0f;
    for (int k = 0; k < nchunks; ++k) {                       // fixed order; thread (tx, ty): rank tx of columns c0 + ty + 4 q
#pragma unroll
        for (int q = 0; q < AG_RT_COLS / 4; ++q) {
            const int c = min(c0 + ty + 4 * q, C - 1);        // past the last column: a valid address, never stored
            s[q] += partial[((size_t)k * C + c) * 64 + tx];
        }
    }
#pragma unroll
    for (int q = 0; q < AG_RT_COLS / 4; ++q) tile[ty + 4 * q][tx] = s[q];
    __syncthreads();
    const int cl = threadIdx.x & (AG_RT_COLS - 1);
    if (c0 + cl < C)
        for (int j = threadIdx.x / AG_RT_COLS; j < r; j += 256 / AG_RT_COLS) out[(size_t)j * C + c0 + cl] = tile[cl][j];
}

// Token chunks: about one workgroup per compute unit -- the fp32 partial tiles of every further chunk are written,
// read again and summed, which costs more than idle units (measured on config 3: 172 column tiles run faster as
// 172 workgroups than as 344 or 688; 64 column tiles fastest as 4 chunks, 256 workgroups).  A single chunk writes
// the result itself.
struct TnPlan { int chunks, chunk_rows; };
// other_tiles: column tiles of the product that shares the launch (they take that many compute units)
static TnPlan tn_plan(int C, int M, int other_tiles = 0) {
    const int col_tiles = (C + AG_COLS - 1) / AG_COLS;
    const int cus = std::max(device_compute_units() - other_tiles, device_compute_units() / 4);
    const int max_chunks = std::max(1, std::min(8, (M + 255) / 256));
    const int best = std::max(1, std::min(max_chunks, (cus + col_tiles / 2) / col_tiles));
    int chunk_rows = ((M + best - 1) / best + 255) / 256 * 256;
    return TnPlan{(M + chunk_rows - 1) / chunk_rows, chunk_rows};
}
static size_t tn_partial_bytes_beside(int C, int M, int RP, int other_tiles) { return (size_t)tn_plan(C, M, other_tiles).chunks * C * RP * sizeof(float); }
size_t tn_partial_bytes(int C, int M, int RP) { return tn_partial_bytes_beside(C, M, RP, 0); }

// out = P^T Q: P [M][C] bf16, Q [M][RP] bf16 (RP = 64), out fp32 [C][r] or [r][C]; one product or two in one launch
struct TnCall { const uint16_t* P; int C; const uint16_t* Q; int transposed; float* partial; float* out; int other_tiles; };
static TnProb tn_prob(const TnCall& c, int M) {
    const TnPlan pl = tn_plan(c.C, M, c.other_tiles);
    const int tiles = (c.C + AG_COLS - 1) / AG_COLS;
    return TnProb{c.P, c.Q, c.partial, pl.chunks == 1 ? c.out : nullptr, c.C, pl.chunk_rows, c.transposed, tiles, tiles * pl.chunks};
}
static hipError_t tn_finish(const TnCall& c, int M, int r, hipStream_t st) {      // the chunk sum, where there are chunks
    const TnPlan pl = tn_plan(c.C, M, c.other_tiles);
    if (pl.chunks == 1) return hipSuccess;
    const size_t tot = (size_t)c.C * r;
    if (c.transposed) tn_reduce_t_kernel<<<dim3((unsigned)((c.C + AG_RT_COLS - 1) / AG_RT_COLS)), dim3(256), 0, st>>>(c.partial, pl.chunks, c.C, r, c.out);
    else tn_reduce_kernel<<<dim3((unsigned)std::min<size_t>((tot + 255) / 256, 4096)), dim3(256), 0, st>>>(c.partial, pl.chunks, c.C, 64, r, c.out);
    return hipGetLastError();
}
static hipError_t launch_tn(const TnCall* c0, const TnCall* c1, int M, int r, hipStream_t st) {
    const size_t sh = std::max((size_t)4 * 2 * 2 * AG_TILEB, (size_t)4 * AG_COLS * (64 + 1) * sizeof(float));
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(tn_skinny_kernel<1>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (attr != hipSuccess) return attr;
    const TnProb pa = tn_prob(*c0, M);
    TnProb pb = pa;
    pb.nwg = 0;
    if (c1) pb = tn_prob(*c1, M);
    tn_skinny_kernel<1><<<dim3(pa.nwg + pb.nwg), dim3(256), sh, st>>>(pa, pb, M, r);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if ((e = tn_finish(*c0, M, r, st)) != hipSuccess) return e;
    return c1 ? tn_finish(*c1, M, r, st) : hipSuccess;
}
hipError_t launch_tn_skinny(const uint16_t* P, int C, int M, const uint16_t* Q, int RP, int r, int transposed,
                            float* partial, float* out, hipStream_t st) {
    if (RP != 64) return hipErrorInvalidValue;                 // two Q tiles per stage would not fit the staging area
    const TnCall c{P, C, Q, transposed, partial, out, 0};
    return launch_tn(&c, nullptr, M, r, st);
}

// No tokens: both gradients are zero (the reduction over zero chunks writes exactly that; a kernel
// rather than a memset, so the call can be captured into a graph).
hipError_t launch_zero_grads(int N, int K, int r, float* dA, float* dB, hipStream_t st) {
    const size_t ta = (size_t)r * K, tb = (size_t)N * r;
    if (ta) tn_reduce_kernel<<<dim3((unsigned)std::min<size_t>((ta + 255) / 256, 4096)), dim3(256), 0, st>>>(nullptr, 0, K, 64, r, dA);
    if (tb) tn_reduce_kernel<<<dim3((unsigned)std::min<size_t>((tb + 255) / 256, 4096)), dim3(256), 0, st>>>(nullptr, 0, N, 64, r, dB);
    return hipGetLastError();
}

// ---- the whole gradient call
hipError_t launch_skinny_ws(const uint16_t* P, int ldp, int M, const uint16_t* Q, int ldq, int r, int Kc,
                            float s, uint16_t* out, int RP, float* scratch, hipStream_t st);
size_t skinny_scratch_bytes(int M, int Kc, int RP);
hipError_t launch_skinny_qt(const uint16_t* P, int ldp, int M, const uint16_t* Qt, int Kc, float s, uint16_t* out,
                            float* scratch, hipStream_t st);
hipError_t launch_transpose(const uint16_t* src, int R, int c, uint16_t* dst, hipStream_t st);

static inline size_t ag_align(size_t v) { return (v + 255) & ~(size_t)255; }
constexpr int kGradRP = 64;

// workspace: [ s t : M x 64 ][ s u : M x 64 ][ B^T : r x N ][ fp32 partial tiles of dB, then of dA; the side products' partial sums use the same region before ]
size_t adapter_grads_workspace_bytes(const lowra_layout& L, int M, int r) {
    if (r <= 0 || M <= 0) return 0;
    const size_t tu = ag_align((size_t)M * kGradRP * 2);
    return 2 * tu + ag_align((size_t)r * L.N * 2) +
           ag_align(std::max(ag_align(tn_partial_bytes_beside(L.N, M, kGradRP, (L.K + AG_COLS - 1) / AG_COLS)) + tn_partial_bytes_beside(L.K, M, kGradRP, (L.N + AG_COLS - 1) / AG_COLS),
                             std::max(skinny_scratch_bytes(M, L.K, kGradRP), skinny_scratch_bytes(M, L.N, kGradRP))));
}

hipError_t launch_adapter_grads_from_side(const lowra_layout& L, const uint16_t* x, const uint16_t* dY, int M, int r,
                                          const uint16_t* ts, const uint16_t* us, float* dA, float* dB, void* workspace, hipStream_t st);

hipError_t launch_adapter_grads(const lowra_layout& L, const uint16_t* x, const uint16_t* dY, int M, const uint16_t* A,
                                const uint16_t* B, int r, float s, float* dA, float* dB, void* workspace, hipStream_t st) {
    uint8_t* ws = static_cast<uint8_t*>(workspace);
    const size_t tu = ag_align((size_t)M * kGradRP * 2);
    uint16_t* ts = reinterpret_cast<uint16_t*>(ws);
    uint16_t* us = reinterpret_cast<uint16_t*>(ws + tu);
    uint16_t* bt = reinterpret_cast<uint16_t*>(ws + 2 * tu);
    float* partial = reinterpret_cast<float*>(ws + 2 * tu + ag_align((size_t)r * L.N * 2));   // scratch of the side products, then the partial tiles
    hipError_t e;
    if ((e = launch_skinny_ws(x, L.K, M, A, L.K, r, L.K, s, ts, kGradRP, partial, st)) != hipSuccess) return e;       // s t = s x A^T
    if (r == 64) {                                                                                      // s u = s dY B, B read in place
        if ((e = launch_skinny_qt(dY, L.N, M, B, L.N, s, us, partial, st)) != hipSuccess) return e;
    } else {
        if ((e = launch_transpose(B, L.N, r, bt, st)) != hipSuccess) return e;                          // B^T [r, N]
        if ((e = launch_skinny_ws(dY, L.N, M, bt, L.N, r, L.N, s, us, kGradRP, partial, st)) != hipSuccess) return e;
    }
    return launch_adapter_grads_from_side(L, x, dY, M, r, ts, us, dA, dB, workspace, st);
}

// The two token contractions alone, from intermediates that already exist (s t and s u as bf16 [M][64]): x and dY are
// read once.  The partial tiles sit where the whole call keeps them.
hipError_t launch_adapter_grads_from_side(const lowra_layout& L, const uint16_t* x, const uint16_t* dY, int M, int r,
                                          const uint16_t* ts, const uint16_t* us, float* dA, float* dB, void* workspace, hipStream_t st) {
    const size_t tu = ag_align((size_t)M * kGradRP * 2);
    float* partial = reinterpret_cast<float*>(static_cast<uint8_t*>(workspace) + 2 * tu + ag_align((size_t)r * L.N * 2));
    float* partial_a = reinterpret_cast<float*>(reinterpret_cast<uint8_t*>(partial) + ag_align(tn_partial_bytes_beside(L.N, M, kGradRP, (L.K + AG_COLS - 1) / AG_COLS)));
    const int tiles_n = (L.N + AG_COLS - 1) / AG_COLS, tiles_k = (L.K + AG_COLS - 1) / AG_COLS;
    const TnCall db{dY, L.N, ts, 0, partial, dB, tiles_k};    // dB = dY^T (s t)
    const TnCall da{x, L.K, us, 1, partial_a, dA, tiles_n};   // dA = (s u)^T x
    KernelTimer timer(st);
    return launch_tn(&db, &da, M, r, st);
}

}  // namespace lowra
