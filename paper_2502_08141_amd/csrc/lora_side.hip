// Rank-r side products of the LoRA term (Sec. 2.1): t = s x A^T (forward) and u = s dY B (input
// gradient), plus the small operand re-layouts they need.  Bandwidth-bound on reading x / dY once.
#include <algorithm>

#include "gemm_common.h"

#ifndef LOWRA_SKINNY_TALL
#define LOWRA_SKINNY_TALL 1   // 0: tall inputs use the 16-row kernel too
#endif

namespace lowra {

// Wait until at most `newer` batches of NIW transfers each are still outstanding (0 <= newer <= MAXN <= 5).
template <int NIW, int MAXN>
__device__ __forceinline__ void wait_newer(int newer) {
    static_assert(MAXN <= 5 && MAXN * NIW <= 63, "wait count does not fit the counter");
    switch (newer) {
        case 0: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
        case 1: asm volatile("s_waitcnt vmcnt(%0)" :: "n"(NIW) : "memory"); break;
        case 2: asm volatile("s_waitcnt vmcnt(%0)" :: "n"(MAXN >= 2 ? 2 * NIW : 0) : "memory"); break;
        case 3: asm volatile("s_waitcnt vmcnt(%0)" :: "n"(MAXN >= 3 ? 3 * NIW : 0) : "memory"); break;
        case 4: asm volatile("s_waitcnt vmcnt(%0)" :: "n"(MAXN >= 4 ? 4 * NIW : 0) : "memory"); break;
        default: asm volatile("s_waitcnt vmcnt(%0)" :: "n"(MAXN >= 5 ? 5 * NIW : 0) : "memory"); break;
    }
}

// out[m][j] = bf16( s * sum_c P[m][c] Q[j][c] ), j < 16 CT (rows j >= r of Q count as zero).
//
// One workgroup per 16 PT token rows and one slice of the contraction (grid.y).  PT = 1 with a single
// slice: M = 4096 fills all 256 compute units.  Tall inputs take PT = 4 and split the contraction
// instead: every stage carries all of Q's rows next to the workgroup's rows of P, so Q -- re-read
// from L2 by every workgroup -- is 80 % of what a stage moves at PT = 1 and 50 % at PT = 4; the
// slices leave unscaled fp32 partial sums that skinny_sum_kernel adds.  Both operands are
// row-major with the contraction index contiguous, while an MFMA lane wants 16 bytes of ITS OWN
// row: loading operands straight into registers would make every lane a separate 16-byte request.
// So the workgroup streams [16 PT rows of P | 16 CT rows of Q], KW columns at a time, through a ring
// of RING LDS stages by global->LDS DMA (four adjacent lanes fetch 64 contiguous bytes).  Moving
// a stage keeps the vector memory pipe busy about as long as multiplying one keeps the LDS and
// matrix pipes busy, so the two jobs belong to different wavefronts: wavefronts [NC, 2 NC) issue
// the transfers of stage it+RING-1 and wait for stage it+1 while wavefronts [0, NC) multiply stage it
// (wavefront w takes columns [KW w / NC, KW (w+1) / NC), v_mfma_f32_16x16x32_bf16); one barrier
// per stage hands the buffers over.  LDS rows hold KW bf16; 16-byte chunk c of row r sits at
// c ^ (r & 15), which makes the operand reads (16 rows, same chunk) conflict-free.
// QT: Q is given transposed, [Kc][64] row-major with rank 64 (LoRA B as the caller holds it): a stage's
// 128 contraction rows of 128 bytes are one contiguous 16 KB block, moved as it lies (16-byte chunk c
// of row n at chunk c ^ (n & 7)) and read with transposing LDS reads -- two ds_read_b64_tr_b16 give a
// lane the 8 consecutive contraction elements of its column.
typedef short sk_v4i16_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) sk_v4i16_t* sk_lds_v4i16_ptr;

template <int CT, int KW, int NC, int RING, int PT = 1, bool QT = false>
__global__ __launch_bounds__(128 * NC) void skinny_nt_kernel(const uint16_t* __restrict__ P, int ldp, int M,
                                                            const uint16_t* __restrict__ Q, int ldq, int r,
                                                            int Kc, float s, uint16_t* __restrict__ out,
                                                            float* __restrict__ partial, int kslice) {
    extern __shared__ __align__(16) uint8_t smem[];
    constexpr int RP = CT * 16, PR = PT * 16, ROWS = PR + RP, ROWBYTES = KW * 2, CPR = KW / 8;   // chunks per row
    constexpr int STAGE = ROWS * ROWBYTES, RPI = 1024 / ROWBYTES;                   // rows per DMA instruction
    constexpr int NI = ROWS / RPI, NIW = NI / NC;                                   // instructions per stage / per issuing wavefront
    constexpr int USTEPS = KW / NC / 32;                                            // 32-wide MFMA steps per multiplying wavefront and stage
    static_assert(KW % (32 * NC) == 0 && NI % NC == 0 && RING >= 3 && RING <= 7 && PR % RPI == 0, "stage split / ring depth");
    static_assert(!QT || (CT == 4 && KW == 128), "the transposed operand is laid out for rank 64 and 128-column stages");
    static_assert(PR % (NC * RPI) == 0, "an issuing wavefront's t-th instruction is P for all of them or for none");
    const uint32_t smem_lds = (uint32_t)(uintptr_t)(lptr_t)smem;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const bool mover = wave >= NC;
    const int sw = mover ? wave - NC : wave;
    const int i = lane & 15, kg = lane >> 4;
    const int m0 = blockIdx.x * PR;
    const int kbeg = blockIdx.y * kslice, kend = min(kbeg + kslice, Kc);     // my slice of the contraction (kslice: a multiple of KW)
    const int nst = (kend - kbeg + KW - 1) / KW;

    floatx4_t acc[PT][CT];
#pragma unroll
    for (int p = 0; p < PT; ++p)
#pragma unroll
        for (int c = 0; c < CT; ++c) acc[p][c] = floatx4_t{0.0f, 0.0f, 0.0f, 0.0f};

    if (mover) {
        // instruction q = sw + NC t moves rows [q RPI, (q+1) RPI) of the stage: [0, PR) from P, the rest from Q
        uint32_t voff[NIW], lc16[NIW];
        const uint32_t kmax_byte = (uint32_t)(Kc - 8) * 2u;
#pragma unroll
        for (int t = 0; t < NIW; ++t) {
            const int row = (sw + NC * t) * RPI + lane / CPR;
            lc16[t] = (uint32_t)((lane % CPR) ^ (row & 15)) * 16u;   // logical chunk landing on my physical chunk
            voff[t] = row < PR ? (uint32_t)min(m0 + row, M - 1) * (uint32_t)ldp * 2u
                               : (uint32_t)min(row - PR, r - 1) * (uint32_t)ldq * 2u;
            if (QT && row >= PR) {                                   // transposed Q: 8 contraction rows of 128 B per instruction
                const int nloc = 8 * ((sw + NC * t) - PR / RPI) + (lane >> 3);
                voff[t] = (uint32_t)nloc;                            // my row within the stage
                lc16[t] = (uint32_t)((lane & 7) ^ (nloc & 7)) * 16u;
            }
        }
        auto issue_stage = [&](int st) {
            const uint32_t kb2 = (uint32_t)(kbeg + st * KW) * 2u;
#pragma unroll
            for (int t = 0; t < NIW; ++t) {
                const int q = sw + NC * t;                           // uniform
                const bool from_p = t * NC * RPI < PR;               // known at compile time: PR is a multiple of NC RPI
                // columns past Kc: any valid bytes, zeroed at the read
                if (QT && !from_p)
                    dma16_s(Q, (uint32_t)min(kbeg + st * KW + (int)voff[t], Kc - 1) * 128u + lc16[t], smem_lds + (st % RING) * STAGE + q * 1024);
                else if (from_p)
                    dma16_s(P, voff[t] + min(kb2 + lc16[t], kmax_byte), smem_lds + (st % RING) * STAGE + q * 1024);
                else
                    dma16_s(Q, voff[t] + min(kb2 + lc16[t], kmax_byte), smem_lds + (st % RING) * STAGE + q * 1024);
            }
        };
        for (int st = 0; st < RING - 1 && st < nst; ++st) issue_stage(st);
        wait_newer<NIW, RING - 2>(min(RING - 2, nst - 1));
        __syncthreads();                                             // stage 0 is there
        for (int it = 0; it < nst; ++it) {
            if (it + RING - 1 < nst) issue_stage(it + RING - 1);
            wait_newer<NIW, RING - 2>(max(0, min(RING - 2, nst - 2 - it)));   // stage it+1 has landed
            __syncthreads();
        }
    } else {
        const bf16x8_t zero = {0, 0, 0, 0, 0, 0, 0, 0};
        __syncthreads();
        for (int it = 0; it < nst; ++it) {
            const uint8_t* sb = smem + (it % RING) * STAGE;
#pragma unroll
            for (int u = 0; u < USTEPS; ++u) {
                const int cl = (KW / NC / 8) * sw + 4 * u + kg;      // logical chunk of my 8 columns
                const bool kin = kbeg + it * KW + cl * 8 < kend;
                const int pc = (cl ^ i) << 4;
                bf16x8_t a[PT];
#pragma unroll
                for (int p = 0; p < PT; ++p) {
                    a[p] = *reinterpret_cast<const bf16x8_t*>(sb + (16 * p + i) * ROWBYTES + pc);
                    if (!kin || m0 + 16 * p + i >= M) a[p] = zero;
                }
#pragma unroll
                for (int c = 0; c < CT; ++c) {
                    bf16x8_t b;
                    if (QT) {
                        typedef short v8i16_t __attribute__((ext_vector_type(8)));
                        sk_v4i16_t h[2];
#pragma unroll
                        for (int eb = 0; eb < 2; ++eb) {
                            const int nr = (KW / NC) * sw + 32 * u + 8 * kg + 4 * eb + (i >> 2);     // contraction row within the stage
                            const int ch = 2 * c + ((i & 3) >> 1);
                            const uint32_t ad = smem_lds + (it % RING) * STAGE + PR * ROWBYTES + nr * 128 + ((ch ^ (nr & 7)) << 4) + (i & 1) * 8;
                            h[eb] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((sk_lds_v4i16_ptr)(uintptr_t)ad);
                        }
                        const v8i16_t v = {h[0][0], h[0][1], h[0][2], h[0][3], h[1][0], h[1][1], h[1][2], h[1][3]};
                        b = __builtin_bit_cast(bf16x8_t, v);
                    } else {
                        b = *reinterpret_cast<const bf16x8_t*>(sb + (PR + 16 * c + i) * ROWBYTES + pc);
                    }
                    if (!kin || 16 * c + i >= r) b = zero;
#pragma unroll
                    for (int p = 0; p < PT; ++p) acc[p][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[p], b, acc[p][c], 0, 0, 0);
                }
            }
            __syncthreads();                                         // stage it is free again, stage it+1 is there
        }
    }
    // lane (i, kg) of a multiplying wavefront holds out[16 p + 4 kg + v][16 c + i]
    float* red = reinterpret_cast<float*>(smem);   // [NC][PR][RP]
    if (!mover) {
#pragma unroll
        for (int p = 0; p < PT; ++p)
#pragma unroll
            for (int c = 0; c < CT; ++c)
#pragma unroll
                for (int v = 0; v < 4; ++v) red[(sw * PR + 16 * p + 4 * kg + v) * RP + c * 16 + i] = acc[p][c][v];
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < PR * RP; idx += 128 * NC) {
        const int row = idx / RP, col = idx % RP;
        float v = 0.0f;
#pragma unroll
        for (int w = 0; w < NC; ++w) v += red[(w * PR + row) * RP + col];
        const int mo = m0 + row;
        if (mo < M) {
            if (partial) partial[((size_t)blockIdx.y * M + mo) * RP + col] = v;          // one slice: unscaled, summed later
            else out[(size_t)mo * RP + col] = (uint16_t)(pack_bf16x2(v * s, 0.0f) & 0xffffu);
        }
    }
}

// out = bf16(s * sum over the slices of partial [slices][M x RP])
__global__ __launch_bounds__(256) void skinny_sum_kernel(const float4* __restrict__ partial, int slices, size_t n4, float s,
                                                         uint2* __restrict__ out) {
    const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= n4) return;
    float4 v = partial[e];
    for (int q = 1; q < slices; ++q) {
        const float4 w = partial[(size_t)q * n4 + e];
        v.x += w.x; v.y += w.y; v.z += w.z; v.w += w.w;
    }
    out[e] = make_uint2(pack_bf16x2(v.x * s, v.y * s), pack_bf16x2(v.z * s, v.w * s));
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

// Tall inputs (at least 64 workgroups of 64 rows) with a long contraction (>= 8192) take the 64-row kernel
// with the contraction split so that about one workgroup per compute unit results; they need
// `scratch` for the slices' fp32 partial sums.
struct SkinnyPlan { int slices, kslice; };
static SkinnyPlan skinny_plan(int M, int Kc, int RP) {
    const int blocks = (M + 63) / 64;
    if (!LOWRA_SKINNY_TALL || RP != 64 || blocks < 64 || Kc < 8192) return SkinnyPlan{1, 0};   // shorter contractions: the extra kernel that adds the slices costs what the split saves
    int slices = std::max(1, std::min(8, 256 / blocks));
    int kslice = ((Kc + slices - 1) / slices + 127) / 128 * 128;
    if (kslice < 512) return SkinnyPlan{1, 0};
    slices = (Kc + kslice - 1) / kslice;
    return slices > 1 ? SkinnyPlan{slices, kslice} : SkinnyPlan{1, 0};
}
size_t skinny_scratch_bytes(int M, int Kc, int RP) {
    const SkinnyPlan pl = skinny_plan(M, Kc, RP);
    return pl.slices > 1 ? (size_t)pl.slices * M * RP * sizeof(float) : 0;
}

template <bool QT>
static hipError_t launch_skinny_any(const uint16_t* P, int ldp, int M, const uint16_t* Q, int ldq, int r, int Kc,
                                    float s, uint16_t* out, int RP, float* scratch, hipStream_t st) {
    // the kernel addresses P rows with 32-bit byte offsets: very tall inputs go in slabs of rows
    const long long max_rows = ((1LL << 31) / ((long long)ldp * 2)) & ~63LL;
    if (max_rows < 64 || (long long)r * ldq * 2 >= (1LL << 31) || (QT && (RP != 64 || (long long)Kc * 128 >= (1LL << 32)))) return hipErrorInvalidValue;
    const SkinnyPlan pl = scratch && M <= max_rows ? skinny_plan(M, Kc, RP) : SkinnyPlan{1, 0};
    // One slice: every workgroup brings in all of Q next to its rows of P, and a compute unit fetches at a fixed rate
    // (about 55 GB/s), so a workgroup costs (its rows + Q's rows) and the call costs that times the rounds its
    // workgroups need on the chip.  64-row workgroups win once the 16-row ones need several rounds
    // (11008 rows: 1 x 128 against 3 x 80).
    if (pl.slices == 1 && RP == 64 && M <= max_rows) {
        const long long cus = device_compute_units();
        const long long cost16 = ((M + 15) / 16 + cus - 1) / cus * (16 + 64), cost64 = ((M + 63) / 64 + cus - 1) / cus * (64 + 64);
        if (LOWRA_SKINNY_TALL && cost64 < cost16) {
            constexpr int sh = 4 * (64 + 64) * 128 * 2;
            static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(skinny_nt_kernel<4, 128, 4, 4, 4, QT>),
                                                         hipFuncAttributeMaxDynamicSharedMemorySize, sh);
            if (attr != hipSuccess) return attr;
            skinny_nt_kernel<4, 128, 4, 4, 4, QT><<<dim3((M + 63) / 64, 1), dim3(512), sh, st>>>(P, ldp, M, Q, ldq, r, Kc, s, out, nullptr, Kc);
            return hipGetLastError();
        }
    }
    if (pl.slices > 1) {
        constexpr int sh = 4 * (64 + 64) * 128 * 2;
        static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(skinny_nt_kernel<4, 128, 4, 4, 4, QT>),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, sh);
        if (attr != hipSuccess) return attr;
        skinny_nt_kernel<4, 128, 4, 4, 4, QT><<<dim3((M + 63) / 64, pl.slices), dim3(512), sh, st>>>(P, ldp, M, Q, ldq, r, Kc, s, out, scratch, pl.kslice);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        const size_t n4 = (size_t)M * RP / 4;
        skinny_sum_kernel<<<dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, st>>>(reinterpret_cast<const float4*>(scratch), pl.slices, n4, s,
                                                                                   reinterpret_cast<uint2*>(out));
        return hipGetLastError();
    }
    for (long long mb = 0; mb < M; mb += max_rows) {
        const int rows = (int)std::min<long long>(max_rows, M - mb);
        const uint16_t* Pb = P + (size_t)mb * ldp;
        uint16_t* ob = out + (size_t)mb * RP;
        const dim3 grid((rows + 15) / 16);
        if (RP == 64) {
            constexpr int sh = 7 * (16 + 64) * 128 * 2;
            static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(skinny_nt_kernel<4, 128, 4, 7, 1, QT>),
                                                         hipFuncAttributeMaxDynamicSharedMemorySize, sh);
            if (attr != hipSuccess) return attr;
            skinny_nt_kernel<4, 128, 4, 7, 1, QT><<<grid, dim3(512), sh, st>>>(Pb, ldp, rows, Q, ldq, r, Kc, s, ob, nullptr, Kc);
        } else if (!QT) {
            constexpr int sh = 4 * (16 + 128) * 128 * 2;
            static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(skinny_nt_kernel<8, 128, 4, 4>),
                                                         hipFuncAttributeMaxDynamicSharedMemorySize, sh);
            if (attr != hipSuccess) return attr;
            skinny_nt_kernel<8, 128, 4, 4><<<grid, dim3(512), sh, st>>>(Pb, ldp, rows, Q, ldq, r, Kc, s, ob, nullptr, Kc);
        }
    }
    return hipGetLastError();
}
hipError_t launch_skinny_ws(const uint16_t* P, int ldp, int M, const uint16_t* Q, int ldq, int r, int Kc,
                            float s, uint16_t* out, int RP, float* scratch, hipStream_t st) {
    return launch_skinny_any<false>(P, ldp, M, Q, ldq, r, Kc, s, out, RP, scratch, st);
}
// out[m][j] = bf16( s * sum_c P[m][c] Qt[c][j] ) with Qt [Kc][64] row-major (rank exactly 64): no transposed copy needed
hipError_t launch_skinny_qt(const uint16_t* P, int ldp, int M, const uint16_t* Qt, int Kc, float s, uint16_t* out,
                            float* scratch, hipStream_t st) {
    return launch_skinny_any<true>(P, ldp, M, Qt, 64, 64, Kc, s, out, 64, scratch, st);
}
hipError_t launch_skinny(const uint16_t* P, int ldp, int M, const uint16_t* Q, int ldq, int r, int Kc,
                         float s, uint16_t* out, int RP, hipStream_t st) {
    return launch_skinny_ws(P, ldp, M, Q, ldq, r, Kc, s, out, RP, nullptr, st);
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
