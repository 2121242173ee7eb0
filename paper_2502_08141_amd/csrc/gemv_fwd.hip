// Small-token forward (M <= 16):  y = x What^T + (s x A^T) B^T, streaming the packed codes once.
//
// Bandwidth-bound: per weight the method moves bits/8 + 1/16 bytes (codes + fp32 group scale), a
// whole Llama-sized matrix is a few MB, about what the chip must have outstanding to cover one HBM
// round trip.  So every wavefront issues ALL its loads of codes and scales before it touches the
// first result, and every load is as wide as the layout allows.
//
// Workgroup = 16 output channels (one MFMA tile, walked in the width-sorted order of their 256-row
// tile so a wavefront mostly sees one width) x all of K.  Its wavefronts split K in blocks of 256.
// In a block, lane (i, kg) LOADS one whole 64-wide group of channel i -- group 4 blk + kg, a
// contiguous run of the packed row (8/16/32 bytes, one or two 16-byte loads) -- and the four scales
// of the block.  v_mfma_f32_16x16x32_bf16 step (g, h) then contracts k = 64 g + 32 h + 8 kg + e, so
// both steps of a group see ONE group in all four kg lanes: the lanes of a channel trade pieces of
// their groups first (a 4 x 4 dword transpose with v_permlane32_swap / v_permlane16_swap).
//
// Decode: two codes (2, 4 or 8 bits) index the channel's pair table in LDS, whose entry is the two
// UNSCALED levels as bf16 (App. A.2's lookup); the absmax multiplies the fp32 dot product of the
// group instead of every weight -- the same sum in another order, with one bf16 rounding per level
// instead of per product.  One table read per two weights for every width, no per-group set-up.
// Tokens are the MFMA rows and channels its columns, so a lane's results belong to its own channel.
//
// The activations of a block (16 tokens x 256 columns, 8 KB, the same for every workgroup: L2)
// come by global->LDS DMA into buffers private to the wavefront -- all rounds at once when they
// fit, else one round ahead -- so that no operand load of x ever is a per-lane request and no
// round needs a barrier.
//
// The rank-r term needs t = s x A^T first: a small kernel writes partial sums of t per 256-column
// block; every workgroup of the main kernel adds them up (a few KB from L2) and multiplies
// [B rows] [t]^T with one more MFMA per 32 ranks.
#include <algorithm>

#include "gemm_common.h"
#include "gemv_t.h"

#ifndef LOWRA_BATCH_SMALL_WG
#define LOWRA_BATCH_SMALL_WG 1
#endif

namespace lowra {

constexpr int GV_XROW = 512;                 // bytes per token row of a staged activation block (256 bf16)
constexpr int GV_MAXR = 8;                   // blocks (rounds) per multiplying wavefront at most
constexpr int GV_TABROW = 1024 + 16;         // bytes per channel of the pair tables: 256 entries, rows skewed by 4 banks

__global__ __launch_bounds__(64) void gemv_t_partial_kernel(const uint16_t* __restrict__ x, int M, int K,
                                                           const uint16_t* __restrict__ A, int r, int RT,
                                                           float* __restrict__ tp) {
    t_partial_body(x, M, K, A, r, RT, tp, blockIdx.x);
}

// the same for every matrix of a batch in one launch: workgroup = one 256-column block of one matrix.
// owner[id] names the matrix of workgroup id and first[m] its first workgroup: two dependent scalar
// loads (a search over the prefix sums would be a chain of eight).
__global__ __launch_bounds__(64) void gemv_t_partial_batch_kernel(const GemvParams* __restrict__ descs, const int* __restrict__ blk0,
                                                                 const int* __restrict__ owner) {
    const int m = owner[blockIdx.x];
    const GemvParams& p = descs[m];
    t_partial_body(p.x, p.M, p.K, p.A, p.r, p.RT, p.tp, (int)blockIdx.x - blk0[m]);
}

// ---------------------------------------------------------------------------------------------
typedef unsigned int uint2v_t __attribute__((ext_vector_type(2)));

// 4 x 4 transpose of dwords over the four lanes (i, kg = 0..3) of a channel: lane kg ends up with
// z[kg] of lanes 0, 1, 2, 3.  v_permlane32_swap trades the upper half of the first register for
// the lower half of the second, v_permlane16_swap the odd 16-lane rows for the even ones.
__device__ __forceinline__ void transpose4(uint32_t (&z)[4]) {
    const uint2v_t p02 = __builtin_amdgcn_permlane32_swap(z[0], z[2], false, false);
    const uint2v_t p13 = __builtin_amdgcn_permlane32_swap(z[1], z[3], false, false);
    const uint2v_t r01 = __builtin_amdgcn_permlane16_swap(p02.x, p13.x, false, false);
    const uint2v_t r23 = __builtin_amdgcn_permlane16_swap(p02.y, p13.y, false, false);
    z[0] = r01.x; z[1] = r01.y; z[2] = r23.x; z[3] = r23.y;
}

template <int W, int PER>
__device__ __forceinline__ void gemv_body(const GemvParams& p, const int strip) {
    extern __shared__ __align__(16) uint8_t gv_smem[];
    // LDS: pair tables [16 channels][GV_TABROW bytes] | channel numbers [16] | t (bf16 [16][RT]) |
    //      [xbufs buffers][W pieces][rows2 KB] activations (rows2 = pairs of token rows; xbufs = all
    //      rounds when they fit, else 2).  After its last round a wavefront reuses the head of its
    //      piece of buffer 0 for its partial results [16 channels][16 tokens].
    constexpr int TAB0 = 0, NL0 = TAB0 + 16 * GV_TABROW, T0 = NL0 + 64;
    const int rows2 = (min(p.M, 16) + 1) >> 1;
    const int XPIECE = rows2 * 1024, XBUF = W * XPIECE;
    const int X0 = T0 + 16 * p.RT * 2;
    int* n_lds = reinterpret_cast<int*>(gv_smem + NL0);
    uint16_t* t_lds = reinterpret_cast<uint16_t*>(gv_smem + T0);
    const uint32_t smem_lds = (uint32_t)(uintptr_t)(lptr_t)gv_smem;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int i = lane & 15, kg = lane >> 4;
    const int row0 = strip * 16;
    const int nblk = (p.G + 3) >> 2;                               // blocks of 4 groups
    const int per = (nblk + W - 1) / W;                            // rounds: blocks per wavefront (<= PER)

    {
        // One DMA instruction moves 2 token rows x 512 B of my block of round q into that round's
        // buffer; chunk c of token row m lands at chunk c ^ (m & 15).
        const int tok = lane >> 5;
        const bool x_all = p.xbufs >= per;                         // every round has a buffer of its own: all asked for at once
        auto xbuf_of = [&](int q) { return x_all ? q : (q & 1); };
        auto issue_x = [&](int q) {
            const int blk = min(wave * per + q, nblk - 1);
            for (int pr = 0; pr < rows2; ++pr) {                    // uniform
                const int m = min(2 * pr + tok, p.M - 1);
                const int lc = (lane & 31) ^ ((2 * pr + tok) & 15);
                const uint32_t col = min((uint32_t)blk * 256u + (uint32_t)lc * 8u, (uint32_t)p.K - 8u);   // past K: unused
                dma16_s(p.x, ((uint32_t)m * (uint32_t)p.K + col) * 2u,
                        smem_lds + X0 + xbuf_of(q) * XBUF + wave * XPIECE + pr * 1024);
            }
        };
        if (x_all) {
            for (int q = 0; q < per; ++q) issue_x(q);                // uniform
        } else {
            issue_x(0);
        }

        const SortedRow rec = p.sorted_rows[row0 + i];
        const int bits = (int)(rec.bits_cb & 0xffu);
        const bool row_ok = rec.n >= 0;                            // padding rows are recorded as 1-bit rows
        const int nc = row_ok ? rec.n : 0;
        const uint8_t* rowp = p.packed + rec.offset;
        const uint8_t* pend16 = p.packed + p.packed_bytes - 16;
        const float* mrow = p.mappings + (size_t)(rec.bits_cb >> 8) * kTableStride;
        const bool two = bits == 2, four = bits == 4;

        // levels for my entries of my channel's pair table: entry e = two codes (low, high) -> two bf16
        constexpr int NE = 256 / (4 * W);
        const int nent = 1 << (2 * bits);
        const uint32_t cmask = (1u << bits) - 1u;
        float tlo[NE], thi[NE];
#pragma unroll
        for (int j = 0; j < NE; ++j) {
            const int e = (int)(threadIdx.x >> 4) + 4 * W * j;
            const bool e_ok = row_ok && e < nent;
            tlo[j] = e_ok ? mrow[e & cmask] : 0.0f;
            thi[j] = e_ok ? mrow[e >> bits] : 0.0f;
        }

        // every load of codes and scales of all my rounds, back to back
        const bool wave_has4 = __builtin_amdgcn_ballot_w64(four) != 0;
        const bool vec_sc = (p.G & 3) == 0;                          // a block's four scales are one aligned 16-byte load
        uint4 ca[PER], cb[PER];
        float4 sc[PER];
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
                const float* ar = p.absmax + (size_t)nc * p.G;
                if (vec_sc) {
                    sc[q] = *reinterpret_cast<const float4*>(ar + min(4 * blk, p.G - 4));
                } else {
                    sc[q].x = ar[min(4 * blk, p.G - 1)]; sc[q].y = ar[min(4 * blk + 1, p.G - 1)];
                    sc[q].z = ar[min(4 * blk + 2, p.G - 1)]; sc[q].w = ar[min(4 * blk + 3, p.G - 1)];
                }
            } else {
                ca[q] = cb[q] = zero4(); sc[q] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            }
        }

        // my fragment of B for the first 32 ranks, asked for with everything else; my channel number for the final store
        bf16x8_t bfr0 = {0, 0, 0, 0, 0, 0, 0, 0};
        if (wave == 0 && p.RT > 0 && (p.r & 7) == 0 && row_ok && kg * 8 < p.r)
            bfr0 = *reinterpret_cast<const bf16x8_t*>(p.B + (size_t)nc * p.r + kg * 8);
        if (wave == 0 && kg == 0) n_lds[i] = rec.n;

        // my channel's pair table (unscaled levels; the group scale multiplies the group's dot product)
        uint8_t* tabp = gv_smem + TAB0 + i * GV_TABROW;
#pragma unroll
        for (int j = 0; j < NE; ++j) {
            const int e = (int)(threadIdx.x >> 4) + 4 * W * j;
            if (row_ok && e < nent) *reinterpret_cast<uint32_t*>(tabp + 4 * e) = pack_bf16x2(tlo[j], thi[j]);
        }

        // ---- t = s * sum of the partials (bf16, [16][RT]), by all wavefronts
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
        __syncthreads();                                           // t, pair tables

        const uint32_t fw2 = 2u * (uint32_t)bits;                  // bits of one table index (two codes)
        floatx4_t tot = {0.0f, 0.0f, 0.0f, 0.0f};
        const bf16x8_t zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            if (q < per) {                                          // uniform
                // my block of this round has landed (so has everything else I asked for); ask for the next
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                if (!x_all && q + 1 < per) issue_x(q + 1);
                const int blk = wave * per + q;
                const bool b_ok = row_ok && blk < nblk;
                const float a4[4] = {(b_ok && 4 * blk < p.G) ? sc[q].x : 0.0f, (b_ok && 4 * blk + 1 < p.G) ? sc[q].y : 0.0f,
                                     (b_ok && 4 * blk + 2 < p.G) ? sc[q].z : 0.0f, (b_ok && 4 * blk + 3 < p.G) ? sc[q].w : 0.0f};
                // I loaded group kg of my channel; MFMA step (g, h) wants from me the 8 codes
                // k = 64 g + 32 h + 8 kg .. + 8 of group g: piece kg of each half of the group goes
                // to lane kg of the lane that loaded it
                const bool up = hi8[q] && !two && !four;
                const uint32_t c0 = up ? ca[q].z : ca[q].x, c1 = up ? ca[q].w : ca[q].y;     // a 1-bit row uses 8 of its 16 bytes
                const uint32_t D[8] = {ca[q].x, ca[q].y, ca[q].z, ca[q].w, cb[q].x, cb[q].y, cb[q].z, cb[q].w};
                uint32_t za[4], zb[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const uint32_t a2 = D[k >> 1] >> (16 * (k & 1)), b2 = D[2 + (k >> 1)] >> (16 * (k & 1));
                    const uint32_t a1 = c0 >> (8 * k), b1 = c1 >> (8 * k);
                    za[k] = four ? D[k] : (two ? a2 : a1);
                    zb[k] = four ? D[4 + k] : (two ? b2 : b1);
                }
                transpose4(za);
                transpose4(zb);
                const uint8_t* xp = gv_smem + X0 + xbuf_of(q) * XBUF + wave * XPIECE + min(i, p.M - 1) * GV_XROW;
                // tokens are the rows, channels the columns: lane (i, kg) gets y[token 4 kg + v][channel i].
                // Token rows past M repeat row M - 1 and are never stored.
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    floatx4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const uint32_t cs = h ? zb[g] : za[g];
                        uint32_t d[4];
#pragma unroll
                        for (int pp = 0; pp < 4; ++pp)
                            d[pp] = *reinterpret_cast<const uint32_t*>(tabp + 4u * __builtin_amdgcn_ubfe(cs, pp * fw2, fw2));
                        const bf16x8_t xf = *reinterpret_cast<const bf16x8_t*>(xp + (((8 * g + 4 * h + kg) ^ i) << 4));
                        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xf, __builtin_bit_cast(bf16x8_t, make_uint4(d[0], d[1], d[2], d[3])), acc, 0, 0, 0);
                    }
#pragma unroll
                    for (int v = 0; v < 4; ++v) tot[v] += a4[g] * acc[v];
                }
            }
        }
        // ---- rank-r term (wavefront 0): [t] x [B rows]
        if (wave == 0 && p.RT > 0) {
            for (int e0 = 0; e0 < p.RT; e0 += 32) {
                const int j0 = e0 + kg * 8;
                bf16x8_t tf = zero8, bfr = zero8;
                if (j0 < p.RT) tf = *reinterpret_cast<const bf16x8_t*>(t_lds + i * p.RT + j0);
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
                tot = __builtin_amdgcn_mfma_f32_16x16x32_bf16(tf, bfr, tot, 0, 0, 0);
            }
        }
        // my piece of buffer 0 is dead (all my rounds are done, all transfers have landed)
        float* part = reinterpret_cast<float*>(gv_smem + X0 + wave * XPIECE);
        *reinterpret_cast<float4*>(part + i * 16 + 4 * kg) = make_float4(tot[0], tot[1], tot[2], tot[3]);   // [channel][token]
    }
    __syncthreads();

    // reduce over wavefronts, store bf16
    for (int o = threadIdx.x; o < 256; o += W * 64) {
        const int rl = o >> 4, m = o & 15;
        const int n = n_lds[rl];
        if (m < p.M && n >= 0) {
            float v = 0.0f;
#pragma unroll
            for (int w = 0; w < W; ++w) v += reinterpret_cast<const float*>(gv_smem + X0 + w * XPIECE)[o];
            p.y[(size_t)m * p.N + n] = (uint16_t)(pack_bf16x2(v, 0.0f) & 0xffffu);
        }
    }
}

template <int W, int PER>
__global__ __launch_bounds__(W * 64) void gemv_fwd_kernel(GemvParams p) {
    gemv_body<W, PER>(p, blockIdx.x);
}
// every matrix of a batch that takes this instantiation, in one launch: workgroup = one 16-channel strip of one matrix
template <int W, int PER>
__global__ __launch_bounds__(W * 64) void gemv_fwd_batch_kernel(const GemvParams* __restrict__ descs, const int* __restrict__ strip0,
                                                                const int* __restrict__ owner) {
    const int m = owner[blockIdx.x];
    const GemvParams p = descs[m];
    gemv_body<W, PER>(p, (int)blockIdx.x - strip0[m]);
}

// LDS bytes of an instantiation for this matrix (0: does not fit); sets the number of activation buffers
template <int W, int PER>
static size_t gemv_lds(GemvParams& p) {
    constexpr int fixed = 16 * GV_TABROW + 64;
    constexpr int kMaxLds = 160 * 1024;
    const int rows2 = (std::min(p.M, 16) + 1) / 2;
    const int nblk = (p.G + 3) / 4, per = (nblk + W - 1) / W;
    const size_t base = (size_t)fixed + (size_t)16 * p.RT * 2, xbuf = (size_t)W * rows2 * 1024;
    p.xbufs = base + per * xbuf <= (size_t)kMaxLds ? per : 2;     // a buffer per round when they fit
    const size_t sh = base + (size_t)p.xbufs * xbuf;
    return sh > (size_t)kMaxLds ? 0 : sh;
}
template <int W, int PER>
static hipError_t gemv_attr() {
    static hipError_t a0 = hipFuncSetAttribute(reinterpret_cast<const void*>(gemv_fwd_kernel<W, PER>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    static hipError_t a1 = hipFuncSetAttribute(reinterpret_cast<const void*>(gemv_fwd_batch_kernel<W, PER>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    return a0 != hipSuccess ? a0 : a1;
}
template <int W, int PER>
static hipError_t launch_one(GemvParams p, hipStream_t st) {
    const hipError_t attr = gemv_attr<W, PER>();
    if (attr != hipSuccess) return attr;
    const size_t sh = gemv_lds<W, PER>(p);
    if (sh == 0) return hipErrorInvalidValue;
    const dim3 grid((p.N + 15) / 16);
    gemv_fwd_kernel<W, PER><<<grid, dim3(W * 64), sh, st>>>(p);
    return hipGetLastError();
}

static int compute_units_cached() {
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) v = 256;
        cus = v;
    }
    return cus;
}

// 8 wavefronts x GV_MAXR rounds x 256 columns
bool gemv_fwd_fits(int K) { return (K + 255) / 256 <= 8 * GV_MAXR; }

// The instantiation a matrix takes.  Rounds per wavefront fix the register footprint, so the kernel is
// compiled for a few depths; 16 wavefronts (4 per SIMD hide the LDS and decode latencies better)
// whenever their activation buffers fit; with more strips than compute units two 8-wavefront
// workgroups per unit (when their buffers fit twice) overlap one strip's loads with the other's
// arithmetic.
struct GemvChoice { int W, PER; };
static GemvChoice gemv_choose(const GemvParams& p, bool many_strips = false) {
    const int nblk = (p.G + 3) / 4;
    const int rows2 = (std::min(p.M, 16) + 1) / 2;
    const bool fit16 = (size_t)16 * GV_TABROW + 64 + (size_t)16 * p.RT * 2 +
                       (size_t)std::min((nblk + 15) / 16, 2) * 16 * rows2 * 1024 <= (size_t)160 * 1024;
    const int nstrips = (p.N + 15) / 16;
    const size_t lds8 = (size_t)16 * GV_TABROW + 64 + (size_t)16 * p.RT * 2 + (size_t)std::min((nblk + 7) / 8, 2) * 8 * rows2 * 1024;
    const bool pair8 = (many_strips || nstrips > compute_units_cached()) && 2 * lds8 <= (size_t)150 * 1024 && nblk <= 16;
    if (fit16 && !pair8) {
        if (nblk <= 16) return {16, 1};     // K <= 4096
        if (nblk <= 32) return {16, 2};
        if (nblk <= 48) return {16, 3};     // K = 11008
        if (nblk <= 64) return {16, 4};
    }
    if (nblk <= 4) return {4, 1};
    if (nblk <= 8) return {4, 2};
    if (nblk <= 16) return {8, 2};          // K <= 4096
    if (nblk <= 32) return {8, 4};
    if (nblk <= 48) return {8, 6};          // K = 11008
    return {8, 8};
}
// calls f.template operator()<W, PER>() for the chosen instantiation
template <typename F>
static hipError_t gemv_dispatch(GemvChoice c, F&& f) {
    if (c.W == 16 && c.PER == 1) return f.template operator()<16, 1>();
    if (c.W == 16 && c.PER == 2) return f.template operator()<16, 2>();
    if (c.W == 16 && c.PER == 3) return f.template operator()<16, 3>();
    if (c.W == 16 && c.PER == 4) return f.template operator()<16, 4>();
    if (c.W == 4 && c.PER == 1) return f.template operator()<4, 1>();
    if (c.W == 4 && c.PER == 2) return f.template operator()<4, 2>();
    if (c.W == 8 && c.PER == 2) return f.template operator()<8, 2>();
    if (c.W == 8 && c.PER == 4) return f.template operator()<8, 4>();
    if (c.W == 8 && c.PER == 6) return f.template operator()<8, 6>();
    if (c.W == 8 && c.PER == 8) return f.template operator()<8, 8>();
    return hipErrorInvalidValue;
}
struct LaunchSingle {
    const GemvParams& p; hipStream_t st;
    template <int W, int PER> hipError_t operator()() const { return launch_one<W, PER>(p, st); }
};

hipError_t launch_gemv_fwd(const GemvParams& p, hipStream_t st) {
    const int nblk = (p.G + 3) / 4;
    if (p.RT > 0) {
        gemv_t_partial_kernel<<<dim3(nblk), dim3(64), 0, st>>>(p.x, p.M, p.K, p.A, p.r, p.RT, p.tp);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return gemv_dispatch(gemv_choose(p), LaunchSingle{p, st});
}

// ---- several matrices in one launch per instantiation.  The descriptors (every pointer of every matrix)
// are fixed when the batch is built and live in device memory; a run is one launch of the partial-sum
// kernel over all matrices that have a LoRA term and one launch of the main kernel per group of
// matrices that take the same instantiation with the same LDS size.
struct PrepareDesc {
    GemvParams& p; size_t& sh;
    template <int W, int PER> hipError_t operator()() const {
        const hipError_t attr = gemv_attr<W, PER>();
        if (attr != hipSuccess) return attr;
        sh = gemv_lds<W, PER>(p);
        return sh ? hipSuccess : hipErrorInvalidValue;
    }
};
struct LaunchGroup {
    const GemvBatchGroup& g; hipStream_t st;
    template <int W, int PER> hipError_t operator()() const {
        gemv_fwd_batch_kernel<W, PER><<<dim3(g.nstrips), dim3(W * 64), g.sh, st>>>(g.d_descs, g.d_strip0, g.d_owner);
        return hipGetLastError();
    }
};

void gemv_batch_free(lowra_fwd_batch& b) {
    for (auto& g : b.groups) { (void)hipFree(g.d_descs); (void)hipFree(g.d_strip0); (void)hipFree(g.d_owner); }
    b.groups.clear();
    (void)hipFree(b.d_tdescs); (void)hipFree(b.d_blk0); (void)hipFree(b.d_towner);
    b.d_tdescs = nullptr; b.d_blk0 = nullptr; b.d_towner = nullptr;
}

template <typename T>
static hipError_t to_device(const std::vector<T>& v, T** out) {
    hipError_t e = hipMalloc(reinterpret_cast<void**>(out), v.size() * sizeof(T));
    if (e != hipSuccess) return e;
    return hipMemcpy(*out, v.data(), v.size() * sizeof(T), hipMemcpyHostToDevice);
}

hipError_t gemv_batch_build(std::vector<GemvParams>& items, lowra_fwd_batch& b) {
    hipError_t e;
    struct Key { int W, PER; size_t sh; };
    std::vector<Key> keys;
    std::vector<std::vector<GemvParams>> members;
    for (auto& p : items) {
        const GemvChoice c = gemv_choose(p, LOWRA_BATCH_SMALL_WG != 0);
        size_t sh = 0;
        if ((e = gemv_dispatch(c, PrepareDesc{p, sh})) != hipSuccess) return e;
        size_t k = 0;
        while (k < keys.size() && !(keys[k].W == c.W && keys[k].PER == c.PER && keys[k].sh == sh)) ++k;
        if (k == keys.size()) { keys.push_back(Key{c.W, c.PER, sh}); members.emplace_back(); }
        members[k].push_back(p);
    }
    for (size_t k = 0; k < keys.size(); ++k) {
        GemvBatchGroup g{};
        g.W = keys[k].W; g.PER = keys[k].PER; g.sh = keys[k].sh; g.nmat = (int)members[k].size();
        std::vector<int> strip0(members[k].size() + 1, 0);
        for (size_t m = 0; m < members[k].size(); ++m) strip0[m + 1] = strip0[m] + (members[k][m].N + 15) / 16;
        g.nstrips = strip0.back();
        std::vector<int> owner((size_t)g.nstrips);
        for (size_t m = 0; m < members[k].size(); ++m)
            for (int w = strip0[m]; w < strip0[m + 1]; ++w) owner[(size_t)w] = (int)m;
        b.groups.push_back(g);                                       // pushed first so that a failure below is freed with the rest
        if ((e = to_device(members[k], &b.groups.back().d_descs)) != hipSuccess) return e;
        if ((e = to_device(strip0, &b.groups.back().d_strip0)) != hipSuccess) return e;
        if ((e = to_device(owner, &b.groups.back().d_owner)) != hipSuccess) return e;
    }
    std::vector<GemvParams> tdescs;
    std::vector<int> blk0(1, 0);
    for (auto& p : items)
        if (p.RT > 0) { tdescs.push_back(p); blk0.push_back(blk0.back() + (p.G + 3) / 4); }
    b.nt = (int)tdescs.size(); b.nblk_total = blk0.back();
    if (b.nt > 0) {
        std::vector<int> owner((size_t)b.nblk_total);
        for (int m = 0; m < b.nt; ++m)
            for (int w = blk0[(size_t)m]; w < blk0[(size_t)m + 1]; ++w) owner[(size_t)w] = m;
        if ((e = to_device(tdescs, &b.d_tdescs)) != hipSuccess) return e;
        if ((e = to_device(blk0, &b.d_blk0)) != hipSuccess) return e;
        if ((e = to_device(owner, &b.d_towner)) != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t gemv_batch_run(const lowra_fwd_batch& b, hipStream_t st) {
    if (b.nt > 0) {
        gemv_t_partial_batch_kernel<<<dim3(b.nblk_total), dim3(64), 0, st>>>(b.d_tdescs, b.d_blk0, b.d_towner);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (b.groups.empty()) return hipSuccess;
    KernelTimer timer(st);
    for (const auto& g : b.groups) {
        const hipError_t e = gemv_dispatch(GemvChoice{g.W, g.PER}, LaunchGroup{g, st});
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace lowra
