// Small-token forward (M <= 16):  y = x What^T + (s x A^T) B^T, streaming the packed codes once.
//
// Bandwidth-bound: per weight the method moves bits/8 + 1/16 bytes (codes + fp32 group scale), a
// whole Llama-sized matrix is a few MB, about what the chip must have outstanding to cover one HBM
// round trip.  So every wavefront issues ALL its loads of codes and scales before it touches the
// first result, and every load is as wide as the layout allows.
//
// Workgroup = 16 output channels (one MFMA tile, walked in the width-sorted order of their 256-row
// tile so a wavefront mostly sees one width) x all of K.  Its W wavefronts split K in
// blocks of 256: in a block, lane (i, kg) of v_mfma_f32_16x16x32_bf16 owns ONE 64-wide group of
// channel i -- group 4 blk + kg, i.e. a contiguous run of the packed row (8/16/32 bytes, one or two
// 16-byte loads) and one absmax.  The MFMA contraction index is therefore permuted (step j of a
// block multiplies k = 256 blk + 64 kg + 8 j .. + 8), which is free as long as the activations are
// read with the same permutation.  The group's levels times its absmax are rounded to bf16 once
// per group (App. A.2) and the codes decode in registers exactly as in the GEMM kernels; 4-bit rows
// look their 16 levels up in LDS.
//
// The activations of a block (16 tokens x 256 columns, 8 KB, the same for every workgroup: L2)
// come by global->LDS DMA, one round (one block per wavefront) ahead, into a buffer private to
// the wavefront, so that no operand load of x ever is a per-lane request and no round needs a barrier.
//
// The rank-r term needs t = s x A^T first: a small kernel writes partial sums of t per 256-column
// block; every workgroup of the main kernel adds them up (a few KB from L2) and multiplies
// [B rows] [t]^T with one more MFMA per 32 ranks.
#include <algorithm>

#include "gemm_common.h"

namespace lowra {

constexpr int GV_XROW = 512;                 // bytes per token row of a staged activation block (256 bf16)
constexpr int GV_XPIECE = 16 * GV_XROW;      // 8 KB per block
constexpr int GV_MAXR = 8;                   // blocks (rounds) per multiplying wavefront at most

// ---------------------------------------------------------------------------------------------
// t partials:  tp[b][m][j] = sum over the 256 columns of block b of x[m][k] A[j][k]     (fp32)
// One wavefront per block; lane (i, kg) owns columns 64 kg .. 64 kg + 63 of the block for token i
// (operand B) and for ranks i + 16 c (operand A): 128 contiguous bytes per lane and row.
__global__ __launch_bounds__(64) void gemv_t_partial_kernel(const uint16_t* __restrict__ x, int M, int K,
                                                           const uint16_t* __restrict__ A, int r, int RT,
                                                           float* __restrict__ tp) {
    const int lane = threadIdx.x, i = lane & 15, kg = lane >> 4;
    const int b = blockIdx.x;
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

// ---------------------------------------------------------------------------------------------
template <int W, int PER>
__global__ __launch_bounds__(W * 64) void gemv_fwd_kernel(GemvParams p) {
    extern __shared__ __align__(16) uint8_t gv_smem[];
    // LDS: [W][16][17] partial results | 4-bit levels [16][17] | channel numbers [16] | t (bf16 [16][RT]) |
    //      [2 buffers][W pieces][rows2 KB] activations (rows2 = pairs of token rows)
    constexpr int PART0 = 0, STAB0 = PART0 + W * 16 * 17 * 4, NL0 = STAB0 + 16 * 17 * 4, T0 = NL0 + 64;
    const int rows2 = (min(p.M, 16) + 1) >> 1;
    const int XPIECE = rows2 * 1024, XBUF = W * XPIECE;
    const int X0 = T0 + 16 * p.RT * 2;
    int* n_lds = reinterpret_cast<int*>(gv_smem + NL0);
    float (*part)[16][17] = reinterpret_cast<float (*)[16][17]>(gv_smem + PART0);
    float (*stab)[17] = reinterpret_cast<float (*)[17]>(gv_smem + STAB0);
    uint16_t* t_lds = reinterpret_cast<uint16_t*>(gv_smem + T0);
    const uint32_t smem_lds = (uint32_t)(uintptr_t)(lptr_t)gv_smem;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int i = lane & 15, kg = lane >> 4;
    const int row0 = blockIdx.x * 16;
    const int nblk = (p.G + 3) >> 2;                               // blocks of 4 groups
    const int per = (nblk + W - 1) / W;                            // rounds: blocks per wavefront (<= PER)

    {
        // One DMA instruction moves 2 token rows x 512 B of my block of round q into buffer q & 1;
        // chunk c of token row m lands at chunk c ^ (m & 15).
        const int tok = lane >> 5;
        auto issue_x = [&](int q) {
            const int blk = min(wave * per + q, nblk - 1);
            for (int pr = 0; pr < rows2; ++pr) {                    // uniform
                const int m = min(2 * pr + tok, p.M - 1);
                const int lc = (lane & 31) ^ ((2 * pr + tok) & 15);
                const uint32_t col = min((uint32_t)blk * 256u + (uint32_t)lc * 8u, (uint32_t)p.K - 8u);   // past K: unused
                dma16_s(p.x, ((uint32_t)m * (uint32_t)p.K + col) * 2u,
                        smem_lds + X0 + (q & 1) * XBUF + wave * XPIECE + pr * 1024);
            }
        };
        issue_x(0);

        const SortedRow rec = p.sorted_rows[row0 + i];
        const int bits = (int)(rec.bits_cb & 0xffu);
        const bool row_ok = rec.n >= 0;                            // padding rows are recorded as 1-bit rows
        const int nc = row_ok ? rec.n : 0;
        const uint8_t* rowp = p.packed + rec.offset;
        const uint8_t* pend16 = p.packed + p.packed_bytes - 16;
        const float* mrow = p.mappings + (size_t)(rec.bits_cb >> 8) * kTableStride;
        const float4 lv = *reinterpret_cast<const float4*>(mrow);
        const bool two = bits == 2, four = bits == 4;
        const bool small = row_ok && !four;
        const float l0 = small ? lv.x : 0.0f, l1 = small ? lv.y : 0.0f;
        const float l2 = (small && two) ? lv.z : 0.0f, l3 = (small && two) ? lv.w : 0.0f;

        // every load of codes and scales of all my rounds, back to back
        const bool wave_has4 = __builtin_amdgcn_ballot_w64(four) != 0;
        uint4 ca[PER], cb[PER];
        float sc[PER];
        bool hi8[PER];
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            const int blk = wave * per + q;
            const int g = min(4 * blk + kg, p.G - 1);              // clamped: groups past the row get a zero scale below
            const uint8_t* a0 = rowp + (size_t)g * 8 * bits;
            const uint8_t* a0c = a0 < pend16 ? a0 : pend16;         // a 1-bit group is 8 B: its 16-byte load may be pulled back
            hi8[q] = a0 != a0c;                                     // ... then the group sits in the upper 8 bytes
            const uint8_t* a1 = four ? a0 + 16 : a0c;
            if (q < per) {                                          // uniform
                ca[q] = *reinterpret_cast<const uint4*>(a0c);
                cb[q] = wave_has4 ? *reinterpret_cast<const uint4*>(a1) : zero4();
                sc[q] = p.absmax[(size_t)nc * p.G + g];
            } else {
                ca[q] = cb[q] = zero4(); sc[q] = 0.0f;
            }
        }

        // my fragment of B for the first 32 ranks, asked for with everything else; my channel number for the final store
        bf16x8_t bfr0 = {0, 0, 0, 0, 0, 0, 0, 0};
        if (wave == 0 && p.RT > 0 && (p.r & 7) == 0 && row_ok && kg * 8 < p.r)
            bfr0 = *reinterpret_cast<const bf16x8_t*>(p.B + (size_t)nc * p.r + kg * 8);
        if (wave == 0 && kg == 0) n_lds[i] = rec.n;

        // ---- t = s * sum of the partials (bf16, [16][RT]), by all multipliers; 4-bit levels by wavefront 0
        if (p.RT > 0) {
            for (int o = threadIdx.x; o < 16 * p.RT; o += W * 64) {
                float v = 0.0f;
                for (int b0 = 0; b0 < nblk; b0 += 16) {             // 16 loads in flight, not one after the other
                    float tmp[16];
#pragma unroll
                    for (int u = 0; u < 16; ++u) tmp[u] = p.tp[(size_t)min(b0 + u, nblk - 1) * 16 * p.RT + o];
#pragma unroll
                    for (int u = 0; u < 16; ++u) v += b0 + u < nblk ? tmp[u] : 0.0f;
                }
                t_lds[o] = (uint16_t)(pack_bf16x2(v * p.s, 0.0f) & 0xffffu);
            }
        }
        if (wave == 0 && kg == 0 && four && row_ok) {
            const float4* m4 = reinterpret_cast<const float4*>(mrow);
            const float4 t0 = m4[0], t1 = m4[1], t2 = m4[2], t3 = m4[3];
            const float tv[16] = {t0.x, t0.y, t0.z, t0.w, t1.x, t1.y, t1.z, t1.w, t2.x, t2.y, t2.z, t2.w, t3.x, t3.y, t3.z, t3.w};
#pragma unroll
            for (int e = 0; e < 16; ++e) stab[i][e] = tv[e];
        }
        __syncthreads();                                           // t, levels

        // per-lane constants of the unified 1-/2-bit decode
        const uint32_t fw = two ? 4u : 2u;
        const uint32_t MUL = two ? 0x404101u : 0x808101u, MASK = two ? 0x03030303u : 0x01010101u;
        const uint32_t ORC = two ? 0x04000400u : 0x02000200u;
        const uint32_t selL = two ? 0x06040200u : 0x03010200u, selH = two ? 0x07050301u : 0x03010200u;
        const uint32_t selE = two ? 0x07060504u : 0x0c010c00u;     // 16-bit slots of two steps from a dword (its lower / upper half for 1-bit rows)
        const uint32_t selO = two ? 0x07060504u : 0x0c030c02u;
        const float* my_tab = &stab[i][0];

        floatx4_t tot = {0.0f, 0.0f, 0.0f, 0.0f};
        const bf16x8_t zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            if (q < per) {                                          // uniform
                // my block of this round has landed (so has everything else I asked for); ask for the next
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                if (q + 1 < per) issue_x(q + 1);
                const int blk = wave * per + q;
                const bool g_ok = row_ok && blk < nblk && 4 * blk + kg < p.G;
                const float a = g_ok ? sc[q] : 0.0f;
                // my group's codes: a 1-bit row uses 8 of the 16 bytes it loaded
                const bool up = hi8[q] && !two && !four;
                const uint32_t c0 = up ? ca[q].z : ca[q].x, c1 = up ? ca[q].w : ca[q].y;
                // one 16-bit slot per step (8 codes), two steps per register
                uint32_t xs[4];
                const uint32_t s1 = two ? c1 : c0, s2 = two ? ca[q].z : c1, s3 = two ? ca[q].w : c1;
                xs[0] = __builtin_amdgcn_perm(c0, c0, selE);
                xs[1] = __builtin_amdgcn_perm(s1, s1, selO);
                xs[2] = __builtin_amdgcn_perm(s2, s2, selE);
                xs[3] = __builtin_amdgcn_perm(s3, s3, selO);
                const uint32_t P01 = pack_bf16x2(l0 * a, l1 * a), P23 = pack_bf16x2(l2 * a, l3 * a);
                const uint32_t SL = __builtin_amdgcn_perm(P23, P01, selL), SH = __builtin_amdgcn_perm(P23, P01, selH);
                const uint32_t c4[8] = {ca[q].x, ca[q].y, ca[q].z, ca[q].w, cb[q].x, cb[q].y, cb[q].z, cb[q].w};
                const uint8_t* xp = gv_smem + X0 + (q & 1) * XBUF + wave * XPIECE + min(i, p.M - 1) * GV_XROW;
                bf16x8_t xf[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    xf[j] = *reinterpret_cast<const bf16x8_t*>(xp + (((8 * kg + j) ^ i) << 4));
                    if (i >= p.M) xf[j] = zero8;
                }
                // weights are the rows, tokens the columns: lane (i, kg) gets y[token i][channel 4 kg + v]
                if (!wave_has4) {                                   // uniform; the usual case, branch-free inside
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        uint32_t d[4];
#pragma unroll
                        for (int pp = 0; pp < 4; ++pp) {
                            const uint32_t cq = __builtin_amdgcn_ubfe(xs[j >> 1], 16u * (j & 1) + pp * fw, fw);
                            d[pp] = __builtin_amdgcn_perm(SH, SL, (__umul24(cq, MUL) & MASK) | ORC);
                        }
                        tot = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, make_uint4(d[0], d[1], d[2], d[3])), xf[j], tot, 0, 0, 0);
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        uint32_t d[4];
                        if (!four) {
#pragma unroll
                            for (int pp = 0; pp < 4; ++pp) {
                                const uint32_t cq = __builtin_amdgcn_ubfe(xs[j >> 1], 16u * (j & 1) + pp * fw, fw);
                                d[pp] = __builtin_amdgcn_perm(SH, SL, (__umul24(cq, MUL) & MASK) | ORC);
                            }
                        } else {
#pragma unroll
                            for (int pp = 0; pp < 4; ++pp) {
                                const uint32_t byte = (c4[j] >> (8 * pp)) & 0xffu;
                                d[pp] = pack_bf16x2(my_tab[byte & 15u] * a, my_tab[byte >> 4] * a);
                            }
                        }
                        tot = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, make_uint4(d[0], d[1], d[2], d[3])), xf[j], tot, 0, 0, 0);
                    }
                }
            }
        }
        // ---- rank-r term (wavefront 0): [B rows] x [t]
        if (wave == 0 && p.RT > 0) {
            for (int e0 = 0; e0 < p.RT; e0 += 32) {
                const int j0 = e0 + kg * 8;
                bf16x8_t tf = zero8, bfr = zero8;
                if (j0 < p.RT && i < p.M) tf = *reinterpret_cast<const bf16x8_t*>(t_lds + i * p.RT + j0);
                if (row_ok && j0 < p.r) {
                    const uint16_t* br = p.B + (size_t)nc * p.r + j0;
                    if ((p.r & 7) == 0) {
                        bfr = e0 == 0 ? bfr0 : *reinterpret_cast<const bf16x8_t*>(br);
                    } else {
                        uint32_t tmp[8];
#pragma unroll
                        for (int e = 0; e < 8; ++e) tmp[e] = j0 + e < p.r ? (uint32_t)br[e] : 0u;
                        bfr = __builtin_bit_cast(bf16x8_t, make_uint4(tmp[0] | (tmp[1] << 16), tmp[2] | (tmp[3] << 16),
                                                                         tmp[4] | (tmp[5] << 16), tmp[6] | (tmp[7] << 16)));
                    }
                }
                tot = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bfr, tf, tot, 0, 0, 0);
            }
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) part[wave][4 * kg + v][i] = tot[v];     // [channel][token]
    }
    __syncthreads();

    // reduce over wavefronts, store bf16
    for (int o = threadIdx.x; o < 256; o += W * 64) {
        const int rl = o >> 4, m = o & 15;
        const int n = n_lds[rl];
        if (m < p.M && n >= 0) {
            float v = 0.0f;
#pragma unroll
            for (int w = 0; w < W; ++w) v += part[w][rl][m];
            p.y[(size_t)m * p.N + n] = (uint16_t)(pack_bf16x2(v, 0.0f) & 0xffffu);
        }
    }
}

template <int W, int PER>
static hipError_t launch_one(const GemvParams& p, hipStream_t st) {
    constexpr int fixed = W * 16 * 17 * 4 + 16 * 17 * 4 + 64;
    static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(gemv_fwd_kernel<W, PER>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, fixed + 16 * 128 * 2 + 2 * W * GV_XPIECE);
    if (attr != hipSuccess) return attr;
    const int rows2 = (std::min(p.M, 16) + 1) / 2;
    const size_t sh = (size_t)fixed + (size_t)16 * p.RT * 2 + (size_t)2 * W * rows2 * 1024;
    const dim3 grid((p.N + 15) / 16);
    gemv_fwd_kernel<W, PER><<<grid, dim3(W * 64), sh, st>>>(p);
    return hipGetLastError();
}

// 8 wavefronts x GV_MAXR rounds x 256 columns
bool gemv_fwd_fits(int K) { return (K + 255) / 256 <= 8 * GV_MAXR; }

hipError_t launch_gemv_fwd(const GemvParams& p, hipStream_t st) {
    const int nblk = (p.G + 3) / 4;
    if (p.RT > 0) {
        gemv_t_partial_kernel<<<dim3(nblk), dim3(64), 0, st>>>(p.x, p.M, p.K, p.A, p.r, p.RT, p.tp);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    // rounds per wavefront fix the register footprint, so the kernel is compiled for a few depths
    if (nblk <= 4) return launch_one<4, 1>(p, st);
    if (nblk <= 8) return launch_one<4, 2>(p, st);
    if (nblk <= 16) return launch_one<8, 2>(p, st);      // K <= 4096
    if (nblk <= 32) return launch_one<8, 4>(p, st);
    if (nblk <= 48) return launch_one<8, 6>(p, st);      // K = 11008
    return launch_one<8, 8>(p, st);
}

}  // namespace lowra
