// Streaming small-token forward (M <= 16):  y = x What^T + (s x A^T) B^T over one or many matrices,
// as ONE persistent launch that keeps the memory system full.
//
// Bandwidth-bound: per weight the method moves bits/8 + 1/16 bytes (codes + fp32 group scale).  A
// compute unit has to keep tens of KB of loads in flight all the time to cover the memory latency, so
// nothing here waits for a load it has just issued:
//
//  * One workgroup (16 wavefronts) per compute unit walks a contiguous range of UNITS.  A unit is 16 bytes
//    of codes per lane for a 16-channel strip of one K-chunk (up to 4096 columns) of one matrix: a whole
//    strip at 1 or 2 bits, one half (the first or the second 32 codes of every 64-wide group) of a 4-bit
//    strip.  Wavefront w owns the 256 columns [256 w, 256 w + 256) of the chunk for every strip, so its
//    activations (the MFMA operand of x) stay in REGISTERS for the whole chunk -- LDS carries no activations.
//  * The codes and scales of a unit travel global -> LDS (global_load_lds) into a ring private to the
//    wavefront, GS_D units before they are used; the row records (byte offset, channel) they depend on
//    travel the same way 2 GS_D units ahead.  The transfers are invisible to the compiler on purpose: it
//    would otherwise wait for all of them at every loop-carried copy.  Every transfer is issued on every
//    pass (past the last unit: to the same address again), so "the transfers of unit j have landed" is
//    one s_waitcnt vmcnt(3 GS_D - 2), a constant.
//  * Strips come in the layout's class-sorted order: all 16 rows of a strip have one width and one
//    table, so a wavefront runs one instruction stream per strip (uniform branch on the width).
//  * Lane (i, kg) receives 16 contiguous bytes of channel i; v_mfma_f32_16x16x32_bf16 step (g, h) contracts
//    k = 64 g + 32 h + 8 kg + e, so the four lanes of a channel first trade pieces (4 x 4 dword transpose,
//    v_permlane32/16_swap) and all lanes of an MFMA step then sit in ONE group: the group scale multiplies
//    the fp32 result of the group's steps instead of every weight (the same sum in another order).
//  * Decode (App. A.2's table lookup): a nibble or byte of codes indexes a table of UNSCALED bf16 levels
//    in LDS that is replicated per lane (1- and 2-bit: bank-conflict free; 4-bit: 16 copies), one
//    shift and one and-or per lookup: 4 weights per lookup at 1 bit, 2 at 2 and 4 bits.
//  * The 16 partial results of a strip meet in LDS (two alternating slots, one barrier per strip); one
//    wavefront, a different one per strip, adds them in a fixed order, applies the rank-r term
//    ([t] [B rows]^T, one MFMA) and stores.  Long rows (K > 4096) are cut into chunks whose fp32
//    partial outputs a small kernel adds afterwards.
//
// Used when every 16-row strip can have one class (at most 4 (width, table) classes per matrix), K is
// a multiple of 256 and the rank is a multiple of 8 up to 32; other shapes take the general kernel.
#include <algorithm>
#include <vector>

#include "gemm_common.h"
#include "gemv_t.h"

#ifndef GS_EXP
#define GS_EXP 0      // measurement variants (bit flags), 0 in the product: 1 no stores, 2 no barrier / reduction, 4 no decode, 8 no transfers of codes and scales
#endif

namespace lowra {

constexpr int GS_W = 16;                 // wavefronts per workgroup = 256-column blocks per K-chunk
constexpr int GS_THREADS = GS_W * 64;
#ifndef GS_DEPTH
#define GS_DEPTH 3
#endif
constexpr int GS_D = GS_DEPTH;           // units whose codes are in flight per wavefront
constexpr int GS_MAXSEG = 4;             // K-chunks of one row at most (K <= 16384)
constexpr int GS_T4B = 16384, GS_T12B = 4096;   // bytes of a 4-bit table (256 entries x 16 copies x 4 B) and of a 1- or 2-bit table
constexpr int GS_REDB = GS_W * 64 * 16;  // one reduction slot: a float4 per lane and wavefront
constexpr int GS_TROW = 32;              // bf16 per token row of t in LDS (rank padded to 32)
constexpr int GS_SLOTB = 1024 + 256;     // ring slot: 16 B of codes per lane, then 4 scales per channel
constexpr int GS_RECB = 256;             // record slot: 16 records of 8 bytes (fetched twice: 64 lanes x 4 B)
constexpr int GS_WAVEB = GS_D * GS_SLOTB + (GS_D + 1) * GS_RECB + 1024;   // per wavefront: ring, record ring, B fragment

// One (matrix, K-chunk): everything a workgroup needs to stream its strips.
struct GsSeg {
    const GvRow* rows;       // [nstrips * 16] class-sorted row records
    const uint8_t* packed;
    const float* absmax;
    const uint16_t* x;       // [M][K] bf16
    const uint16_t* B;       // [N][r] bf16; null when this chunk carries no rank-r term
    const float* tp;         // partial sums of x A^T: [nblk_all][16][RT] fp32
    void* out;               // y [M][N] bf16, or this chunk's fp32 partial [M][N]
    int N, K, G, M;
    int nstrips;
    int first4;              // first strip of the 4-bit classes (nstrips when there is none): those strips are two units each
    int kblk0, nblk;         // first 256-column block of the chunk, and how many (1..16)
    int nblk_all;            // 256-column blocks of the whole row
    int out_fp32;
    int r, RT;
    float s;
    int cls_end[kGvMaxClasses];
    int cls_bits_cb[kGvMaxClasses];   // width | LDS byte offset of the class's table << 8
    int first_unit;          // index of this segment's first unit in the launch's unit list
    int nunits;              // nstrips + (nstrips - first4)
};

struct GsTabs {
    int nslot;                     // codebooks (table rows of `mappings`) with a table in LDS
    int bits[kGvMaxClasses];       // width of codebook c (0: unused)
    int off[kGvMaxClasses];        // byte offset of its table in LDS
    int bytes;                     // table region, rounded up to 1 KB
};

typedef unsigned int gs_uint2v_t __attribute__((ext_vector_type(2)));

// 4 x 4 transpose of dwords over the four lanes (i, kg = 0..3) of a channel: afterwards z[j] of lane kg is
// what z[kg] of lane j was.
__device__ __forceinline__ void gs_transpose4(uint32_t (&z)[4]) {
    const gs_uint2v_t p02 = __builtin_amdgcn_permlane32_swap(z[0], z[2], false, false);
    const gs_uint2v_t p13 = __builtin_amdgcn_permlane32_swap(z[1], z[3], false, false);
    const gs_uint2v_t r01 = __builtin_amdgcn_permlane16_swap(p02.x, p13.x, false, false);
    const gs_uint2v_t r23 = __builtin_amdgcn_permlane16_swap(p02.y, p13.y, false, false);
    z[0] = r01.x; z[1] = r01.y; z[2] = r23.x; z[3] = r23.y;
}

__device__ __forceinline__ void gs_lds_barrier() {
    // LDS traffic of this wavefront done, then the barrier; outstanding global -> LDS transfers keep flying
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}
// every transfer of this wavefront except the newest `N` has landed (they complete in order)
template <int N>
__device__ __forceinline__ void gs_wait_transfers() {
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}
// my LDS reads have returned (their slot may now be refilled)
__device__ __forceinline__ void gs_wait_lds() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

// The descriptors are read-only for the whole launch: reading them through the constant address space lets
// the compiler use scalar loads, so a segment's fields live in scalar registers.
typedef const __attribute__((address_space(4))) GsSeg* gs_cseg_t;
typedef const __attribute__((address_space(4))) int* gs_cint_t;

// The fields of a segment that a stage keeps in scalar registers: plain local variables, loaded one by one
// (a struct copy would end up in private memory).
#define GS_LOAD_ISSUE(p)                                                                                          \
    do {                                                                                                          \
        iPacked = (p)->packed; iAbsmax = (p)->absmax; iB = (p)->B; iG = (p)->G; iKblk0 = (p)->kblk0; iNblk = (p)->nblk; \
        iNstrips = (p)->nstrips; iFirst4 = (p)->first4; iR = (p)->r;                                              \
        iE0 = (p)->cls_end[0]; iE1 = (p)->cls_end[1]; iE2 = (p)->cls_end[2];                                      \
        iC0 = (p)->cls_bits_cb[0]; iC1 = (p)->cls_bits_cb[1]; iC2 = (p)->cls_bits_cb[2]; iC3 = (p)->cls_bits_cb[3];   \
    } while (0)
#define GS_LOAD_MATH(p)                                                                                           \
    do {                                                                                                          \
        mX = (p)->x; mB = (p)->B; mTp = (p)->tp; mOut = (p)->out; mN = (p)->N; mK = (p)->K; mM = (p)->M;          \
        mNstrips = (p)->nstrips; mFirst4 = (p)->first4; mKblk0 = (p)->kblk0; mNblk = (p)->nblk;                   \
        mNblkAll = (p)->nblk_all; mOutFp32 = (p)->out_fp32; mRT = (p)->RT; mS = (p)->s;                           \
        mE0 = (p)->cls_end[0]; mE1 = (p)->cls_end[1]; mE2 = (p)->cls_end[2];                                      \
        mC0 = (p)->cls_bits_cb[0]; mC1 = (p)->cls_bits_cb[1]; mC2 = (p)->cls_bits_cb[2]; mC3 = (p)->cls_bits_cb[3];   \
    } while (0)
// one unit forward: a 4-bit strip is two units (halves 0 and 1)
#define GS_ADVANCE(strip, half, first4)                   \
    do {                                                  \
        if ((strip) >= (first4) && (half) == 0) (half) = 1; \
        else { (half) = 0; ++(strip); }                   \
    } while (0)

__global__ __launch_bounds__(GS_THREADS) void gemv_stream_kernel(const GsSeg* __restrict__ segs_g, const int* __restrict__ wg_first_g,
                                                                 const int* __restrict__ wg_seg_g, const float* __restrict__ mappings,
                                                                 const GsTabs tabs) {
    const gs_cseg_t segs = reinterpret_cast<gs_cseg_t>(reinterpret_cast<uintptr_t>(segs_g));
    const gs_cint_t wg_first = reinterpret_cast<gs_cint_t>(reinterpret_cast<uintptr_t>(wg_first_g));
    const gs_cint_t wg_seg = reinterpret_cast<gs_cint_t>(reinterpret_cast<uintptr_t>(wg_seg_g));
    extern __shared__ __align__(16) uint8_t gs_smem[];
    // LDS: [tables: tabs.bytes] [reduction slots: 2 x GS_REDB] [t: 2 x 16 x GS_TROW bf16] [per wavefront: GS_WAVEB]
    const int RED0 = tabs.bytes, T0 = RED0 + 2 * GS_REDB, WV0 = T0 + 2 * 16 * GS_TROW * 2;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int i = lane & 15, kg = lane >> 4;
    const uint32_t smem_lds = (uint32_t)(uintptr_t)(lptr_t)gs_smem;
    // my wavefront's private LDS: ring slots, record slots, B fragment
    const int RING0 = WV0 + wave * GS_WAVEB, REC0 = RING0 + GS_D * GS_SLOTB, BF0 = REC0 + (GS_D + 1) * GS_RECB;

    // ---- tables of unscaled bf16 levels, one per codebook
#pragma unroll
    for (int c = 0; c < kGvMaxClasses; ++c) {                       // static indices: `tabs` stays in scalar registers
        if (c >= tabs.nslot) break;
        const float* mrow = mappings + (size_t)c * kTableStride;
        uint8_t* tb = gs_smem + tabs.off[c];
        if (tabs.bits[c] == 1) {          // nibble of 4 codes -> 4 bf16 (8 B); copy q of 32 at e * 256 + 8 q
            const float l0 = mrow[0], l1 = mrow[1];
            for (int idx = threadIdx.x; idx < 16 * 32; idx += GS_THREADS) {
                const int e = idx >> 5, q = idx & 31;
                *reinterpret_cast<uint2*>(tb + e * 256 + 8 * q) =
                    make_uint2(pack_bf16x2((e & 1) ? l1 : l0, (e & 2) ? l1 : l0), pack_bf16x2((e & 4) ? l1 : l0, (e & 8) ? l1 : l0));
            }
        } else if (tabs.bits[c] == 2) {   // nibble of 2 codes -> 2 bf16 (4 B); copy q of 64 at e * 256 + 4 q
            for (int idx = threadIdx.x; idx < 16 * 64; idx += GS_THREADS) {
                const int e = idx >> 6, q = idx & 63;
                *reinterpret_cast<uint32_t*>(tb + e * 256 + 4 * q) = pack_bf16x2(mrow[e & 3], mrow[e >> 2]);
            }
        } else if (tabs.bits[c] == 4) {   // byte of 2 codes -> 2 bf16 (4 B); copy q of 16 at e * 64 + 4 q
            for (int idx = threadIdx.x; idx < 256 * 16; idx += GS_THREADS) {
                const int e = idx >> 4, q = idx & 15;
                *reinterpret_cast<uint32_t*>(tb + e * 64 + 4 * q) = pack_bf16x2(mrow[e & 15], mrow[e >> 4]);
            }
        }
    }
    // the record slots start as a valid record (offset 0, no channel): the first requests read them before any has landed
    for (int o = lane; o < (GS_D + 1) * GS_RECB / 8; o += 64)
        *reinterpret_cast<uint2*>(gs_smem + REC0 + 8 * o) = make_uint2(0u, 0xffffffffu);
    __syncthreads();

    const int u0 = wg_first[blockIdx.x], n = wg_first[blockIdx.x + 1] - u0;
    if (n <= 0) return;                                             // whole workgroup

    // ---- three cursors over the same unit list: records (2 GS_D ahead), codes and scales (GS_D ahead), arithmetic
    const int seg0 = wg_seg[blockIdx.x];
    int strip0, half0;
    {
        const int local = u0 - segs[seg0].first_unit, f4 = segs[seg0].first4;
        strip0 = local <= f4 ? local : f4 + ((local - f4) >> 1);
        half0 = local <= f4 ? 0 : ((local - f4) & 1);
    }
    int segR = seg0, stripR = strip0, halfR = half0, nstripsR = segs[seg0].nstrips, first4R = segs[seg0].first4;
    const GvRow* rowsR = segs[seg0].rows;

    int segI = seg0, stripI = strip0, halfI = half0;
    const uint8_t* iPacked; const float* iAbsmax; const uint16_t* iB;
    int iG, iKblk0, iNblk, iNstrips, iFirst4, iR, iE0, iE1, iE2, iC0, iC1, iC2, iC3;
    GS_LOAD_ISSUE(segs + segI);

    int segC = seg0, stripC = strip0, halfC = half0;
    const uint16_t* mX; const uint16_t* mB; const float* mTp; void* mOut;
    int mN, mK, mM, mNstrips, mFirst4, mKblk0, mNblk, mNblkAll, mOutFp32, mRT, mE0, mE1, mE2, mC0, mC1, mC2, mC3;
    float mS;
    GS_LOAD_MATH(segs + segC);
    bool freshC = true;                                             // the arithmetic enters a new segment

    int nred = -1;                                                  // channel of my lanes in the strip I will reduce next
    int nstrip_done = 0;                                            // strips finished by this workgroup: picks the slot and the reducer
    int red_id_I = 0;                                               // the same count, GS_D units ahead (who reduces the strip being requested)
    bf16x8_t xr[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) xr[q] = bf16x8_t{0, 0, 0, 0, 0, 0, 0, 0};
    floatx4_t tot = {0.0f, 0.0f, 0.0f, 0.0f};

    const uint32_t lb1 = 8u * (lane & 31), lb2 = 4u * lane, lb4 = 4u * (lane & 15);

    for (int j = -2 * GS_D; j < n; ++j) {
        // ================= request: the row records of unit j + 2 GS_D (past the last unit: the same again).
        // Lane l fetches dword l & 31 of the strip's 16 records (128 contiguous bytes).
        {
            const int slot = (j + 2 * GS_D) % (GS_D + 1);
            dma4(reinterpret_cast<const uint32_t*>(rowsR + (size_t)stripR * 16) + (lane & 31), smem_lds + REC0 + slot * GS_RECB);
            if (j + 2 * GS_D + 1 < n) {                             // uniform
                GS_ADVANCE(stripR, halfR, first4R);
                if (stripR == nstripsR) {
                    stripR = 0; ++segR;
                    rowsR = segs[segR].rows; nstripsR = segs[segR].nstrips; first4R = segs[segR].first4;
                }
            }
        }

        if (j >= 0) {                                               // uniform
            // ================= arithmetic of unit j
            if (freshC) {
                freshC = false;
                // my activations: x[token i][256 (kblk0 + wave) + 64 g + 32 h + 8 kg ..], zero past M or past the chunk
                const bool ok = wave < mNblk && i < mM;
                const uint16_t* xp = mX + (size_t)min(i, mM - 1) * mK + (size_t)(mKblk0 + min(wave, mNblk - 1)) * 256 + 8 * kg;
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    const bf16x8_t v = *reinterpret_cast<const bf16x8_t*>(xp + 32 * q);
                    xr[q] = ok ? v : bf16x8_t{0, 0, 0, 0, 0, 0, 0, 0};
                }
                // t = s * sum of the partials, bf16 [16][GS_TROW], into the buffer of this segment's parity
                if (mB) {
                    uint16_t* t_lds = reinterpret_cast<uint16_t*>(gs_smem + T0 + (segC & 1) * 16 * GS_TROW * 2);
                    for (int o = threadIdx.x; o < 16 * GS_TROW; o += GS_THREADS) {
                        const int m = o / GS_TROW, jr = o % GS_TROW;
                        float v = 0.0f;
                        if (jr < mRT)
                            for (int b = 0; b < mNblkAll; ++b) v += mTp[((size_t)b * 16 + m) * mRT + jr];
                        t_lds[o] = (uint16_t)(pack_bf16x2(v * mS, 0.0f) & 0xffffu);
                    }
                }
            }
            int c = mC0;                                            // width | table offset << 8 of the strip's class
            c = stripC >= mE0 ? mC1 : c;
            c = stripC >= mE1 ? mC2 : c;
            c = stripC >= mE2 ? mC3 : c;
            const int bits = c & 0xff;
            const uint32_t toff = (uint32_t)(c >> 8);

            // the transfers of unit j (issued GS_D passes ago) have landed: after them came GS_D - 1 passes
            // of 3 transfers each and this pass's record request
            gs_wait_transfers<3 * GS_D - 2>();
            const uint8_t* slot = gs_smem + RING0 + (j % GS_D) * GS_SLOTB;
            const uint4 cq = *reinterpret_cast<const uint4*>(slot + 16 * lane);
            const float4 sq = *reinterpret_cast<const float4*>(slot + 1024 + 16 * i);
            const float a4[4] = {sq.x, sq.y, sq.z, sq.w};
            if (GS_EXP & 4) {
                tot[0] += a4[0] * __builtin_bit_cast(float, cq.x); tot[1] += a4[1] * __builtin_bit_cast(float, cq.y);
                tot[2] += a4[2] * __builtin_bit_cast(float, cq.z); tot[3] += a4[3] * __builtin_bit_cast(float, cq.w);
            } else if (bits == 2) {
                // I hold group kg of my channel: codes 16 d .. 16 d + 15 in dword d
                const uint32_t tb = lb2 + toff;
                uint32_t z[4];
                z[0] = __builtin_amdgcn_perm(cq.z, cq.x, 0x05040100u);
                z[1] = __builtin_amdgcn_perm(cq.z, cq.x, 0x07060302u);
                z[2] = __builtin_amdgcn_perm(cq.w, cq.y, 0x05040100u);
                z[3] = __builtin_amdgcn_perm(cq.w, cq.y, 0x07060302u);
                gs_transpose4(z);
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    floatx4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        uint32_t d[4];
#pragma unroll
                        for (int p = 0; p < 4; ++p) {
                            const int q = 4 * h + p;                                   // nibble of z[g]: codes 2 p, 2 p + 1 of half h
                            const uint32_t sh = q < 2 ? z[g] << (8 - 4 * q) : z[g] >> (4 * q - 8);
                            d[p] = *reinterpret_cast<const uint32_t*>(gs_smem + ((sh & 0xF00u) | tb));
                        }
                        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xr[2 * g + h], __builtin_bit_cast(bf16x8_t, make_uint4(d[0], d[1], d[2], d[3])), acc, 0, 0, 0);
                    }
#pragma unroll
                    for (int v = 0; v < 4; ++v) tot[v] += a4[g] * acc[v];
                }
            } else if (bits == 1) {
                // I hold the pair of groups (kg & ~1, kg | 1) of my channel: mine is the low or the high 8 bytes
                // (bitwise choice, so that it cannot become an indexed access)
                const uint32_t tb = lb1 + toff;
                const uint32_t odd_mask = 0u - (uint32_t)(kg & 1);
                const uint32_t d0 = (cq.z & odd_mask) | (cq.x & ~odd_mask), d1 = (cq.w & odd_mask) | (cq.y & ~odd_mask);
                uint32_t z[4];
                z[0] = __builtin_amdgcn_perm(d1, d0, 0x0c0c0400u);
                z[1] = __builtin_amdgcn_perm(d1, d0, 0x0c0c0501u);
                z[2] = __builtin_amdgcn_perm(d1, d0, 0x0c0c0602u);
                z[3] = __builtin_amdgcn_perm(d1, d0, 0x0c0c0703u);
                gs_transpose4(z);
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    floatx4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        uint2 d[2];
#pragma unroll
                        for (int p = 0; p < 2; ++p) {
                            const int q = 2 * h + p;                                   // nibble of z[g]: codes 4 p .. 4 p + 3 of half h
                            const uint32_t sh = q < 2 ? z[g] << (8 - 4 * q) : z[g] >> (4 * q - 8);
                            d[p] = *reinterpret_cast<const uint2*>(gs_smem + ((sh & 0xF00u) | tb));
                        }
                        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xr[2 * g + h], __builtin_bit_cast(bf16x8_t, make_uint4(d[0].x, d[0].y, d[1].x, d[1].y)), acc, 0, 0, 0);
                    }
#pragma unroll
                    for (int v = 0; v < 4; ++v) tot[v] += a4[g] * acc[v];
                }
            } else {
                // half halfC of group kg of my channel: dword d = its codes 8 d .. 8 d + 7, the piece of lane d
                const uint32_t tb = lb4 + toff;
                uint32_t z[4] = {cq.x, cq.y, cq.z, cq.w};
                gs_transpose4(z);
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    uint32_t d[4];
#pragma unroll
                    for (int p = 0; p < 4; ++p) {                                      // byte p: codes 2 p, 2 p + 1
                        const uint32_t sh = p == 0 ? z[g] << 6 : z[g] >> (8 * p - 6);
                        d[p] = *reinterpret_cast<const uint32_t*>(gs_smem + ((sh & 0x3FC0u) | tb));
                    }
                    const bf16x8_t wv = __builtin_bit_cast(bf16x8_t, make_uint4(d[0], d[1], d[2], d[3]));
                    floatx4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
                    if (halfC == 0) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xr[2 * g], wv, acc, 0, 0, 0);
                    else acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xr[2 * g + 1], wv, acc, 0, 0, 0);
#pragma unroll
                    for (int v = 0; v < 4; ++v) tot[v] += a4[g] * acc[v];
                }
            }
        }

        // ================= request: codes and scales of unit j + GS_D, into the slot the arithmetic above just
        // emptied (its record landed long ago).  Issued on every pass, see the head of the file.
        {
            const bool validI = j + GS_D >= 0 && j + GS_D < n;      // uniform
            int c = iC0;
            c = stripI >= iE0 ? iC1 : c;
            c = stripI >= iE1 ? iC2 : c;
            c = stripI >= iE2 ? iC3 : c;
            const int bits = c & 0xff;
            // the records of unit j + GS_D were requested GS_D passes ago, before 3 GS_D other transfers (a no-op after
            // the arithmetic's wait; needed in the first passes, which have no arithmetic)
            gs_wait_transfers<3 * GS_D>();
            const uint8_t* recs_u = gs_smem + REC0 + ((j + GS_D + 2 * (GS_D + 1)) % (GS_D + 1)) * GS_RECB;
            const uint2 rc = *reinterpret_cast<const uint2*>(recs_u + 8 * i);          // my channel's record
            const uint2 rs = *reinterpret_cast<const uint2*>(recs_u + 8 * (lane >> 2)); // the record of the channel whose scale I fetch
            const int kb = iKblk0 + min(wave, iNblk - 1);           // a wavefront past the chunk's end: the last block again (unused)
            // codes: 16 bytes per lane.  2 bits: group kg.  4 bits: half halfI of group kg.  1 bit: the aligned pair of
            // groups that holds group kg (a group is 8 bytes; rows are 32-byte aligned).
            const uint32_t goff = bits == 2 ? (uint32_t)(4 * kb + kg) * 16u
                                : bits == 4 ? (uint32_t)(4 * kb + kg) * 32u + 16u * (uint32_t)halfI
                                            : (uint32_t)(4 * kb + 2 * (kg >> 1)) * 8u;
            const uint8_t* cp = iPacked + rc.x + goff;
            const float* sp = iAbsmax + (size_t)max((int)rs.y, 0) * iG + 4 * kb + (lane & 3);
            gs_wait_lds();                                          // the slot's old contents are in registers
            if (validI && (red_id_I & (GS_W - 1)) == wave && iB) {  // uniform: I will reduce that strip: its B rows, 16 bytes per lane
                const int nn = max((int)rc.y, 0);
                dma16(iB + (size_t)nn * iR + 8 * min(kg, max(iR / 8 - 1, 0)), smem_lds + BF0);
            }
            if (validI && (red_id_I & (GS_W - 1)) == wave) nred = (int)rc.y;
            const uint32_t slot_lds = smem_lds + RING0 + ((j + 3 * GS_D) % GS_D) * GS_SLOTB;
            if (!(GS_EXP & 8)) {
                dma16(cp, slot_lds);
                dma4(sp, slot_lds + 1024);
            }
            if (validI) {
                const bool last_of_strip = bits != 4 || halfI == 1;
                if (last_of_strip) ++red_id_I;
                if (j + GS_D + 1 < n) {
                    GS_ADVANCE(stripI, halfI, iFirst4);
                    if (stripI == iNstrips) { stripI = 0; ++segI; GS_LOAD_ISSUE(segs + segI); }
                }
            }
        }

        if (j >= 0) {
            // ================= end of a strip: the 16 partial results meet; wavefront (strip count) mod 16 adds and stores
            int c = mC0;
            c = stripC >= mE0 ? mC1 : c;
            c = stripC >= mE1 ? mC2 : c;
            c = stripC >= mE2 ? mC3 : c;
            const bool last_of_strip = (c & 0xff) != 4 || halfC == 1;
            if (last_of_strip) {                                    // uniform
                const int slot = nstrip_done & 1;
                *reinterpret_cast<float4*>(gs_smem + RED0 + slot * GS_REDB + (wave * 64 + lane) * 16) = make_float4(tot[0], tot[1], tot[2], tot[3]);
                tot = floatx4_t{0.0f, 0.0f, 0.0f, 0.0f};
                if (!(GS_EXP & 2)) gs_lds_barrier();
                if (!(GS_EXP & 2) && (nstrip_done & (GS_W - 1)) == wave) {           // uniform
                    const uint8_t* red = gs_smem + RED0 + slot * GS_REDB + lane * 16;
                    floatx4_t sum = {0.0f, 0.0f, 0.0f, 0.0f};
                    for (int w = 0; w < mNblk; ++w) {               // fixed order
                        const float4 v = *reinterpret_cast<const float4*>(red + w * 1024);
                        sum[0] += v.x; sum[1] += v.y; sum[2] += v.z; sum[3] += v.w;
                    }
                    if (mB) {
                        const uint16_t* t_lds = reinterpret_cast<const uint16_t*>(gs_smem + T0 + (segC & 1) * 16 * GS_TROW * 2);
                        const bf16x8_t tf = *reinterpret_cast<const bf16x8_t*>(t_lds + i * GS_TROW + 8 * kg);
                        uint4 bq = *reinterpret_cast<const uint4*>(gs_smem + BF0 + 16 * lane);
                        if (nred < 0 || 8 * kg >= mRT) bq = make_uint4(0u, 0u, 0u, 0u);   // t is zero past the rank, B rows are r long: nothing past it is read
                        sum = __builtin_amdgcn_mfma_f32_16x16x32_bf16(tf, __builtin_bit_cast(bf16x8_t, bq), sum, 0, 0, 0);
                    }
                    if (nred >= 0 && !(GS_EXP & 1)) {
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            const int m = 4 * kg + v;
                            if (m < mM) {
                                const size_t o = (size_t)m * mN + nred;
                                if (mOutFp32) static_cast<float*>(mOut)[o] = sum[v];
                                else static_cast<uint16_t*>(mOut)[o] = (uint16_t)(pack_bf16x2(sum[v], 0.0f) & 0xffffu);
                            }
                        }
                    }
                }
                ++nstrip_done;
            }
            if (j + 1 < n) {
                GS_ADVANCE(stripC, halfC, mFirst4);
                if (stripC == mNstrips) { stripC = 0; ++segC; freshC = true; GS_LOAD_MATH(segs + segC); }
            }
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                // nothing of mine may land in LDS after I am gone
}

// y = bf16(sum of the chunks' fp32 partial outputs), for every matrix that was cut into chunks
struct GsSum { const float* part; uint16_t* y; int count; int nchunks; };
__global__ __launch_bounds__(256) void gemv_stream_sum_kernel(const GsSum* __restrict__ sums, int per_item_blocks) {
    const GsSum d = sums[blockIdx.x / per_item_blocks];
    for (int o = (blockIdx.x % per_item_blocks) * 256 + threadIdx.x; o < d.count; o += per_item_blocks * 256) {
        float v = 0.0f;
        for (int c = 0; c < d.nchunks; ++c) v += d.part[(size_t)c * d.count + o];
        d.y[o] = (uint16_t)(pack_bf16x2(v, 0.0f) & 0xffffu);
    }
}

// ---- partial sums of x A^T for every matrix with a rank-r term: workgroup = one 256-column block of one matrix
struct GsTItem { const uint16_t* x; const uint16_t* A; float* tp; int M, K, r, RT, blk0; };
__global__ __launch_bounds__(64) void gemv_stream_t_kernel(const GsTItem* __restrict__ items, const int* __restrict__ owner) {
    const GsTItem it = items[owner[blockIdx.x]];
    t_partial_body(it.x, it.M, it.K, it.A, it.r, it.RT, it.tp, (int)blockIdx.x - it.blk0);
}

// ---- one matrix, descriptors written on the device (the call must not copy from the host: it may be captured)
struct GsSingle {
    GsSeg segs[GS_MAXSEG];
    GsSum sum;
    int nseg, nwg, nblk_all;
    const uint16_t* A;
    GsSeg* d_segs; int* d_wg_first; int* d_wg_seg; GsSum* d_sum;
};
__global__ __launch_bounds__(64) void gemv_stream_prep_kernel(const GsSingle a) {
    if ((int)blockIdx.x < a.nblk_all && a.segs[0].RT > 0)
        t_partial_body(a.segs[0].x, a.segs[0].M, a.segs[0].K, a.A, a.segs[0].r, a.segs[0].RT, const_cast<float*>(a.segs[0].tp), blockIdx.x);
    if (blockIdx.x == 0) {
        const int per = a.segs[0].nunits, f4 = a.segs[0].first4, units = a.nseg * per;
        for (int b = threadIdx.x; b <= a.nwg; b += 64) {
            int u = (int)((long long)b * units / a.nwg);
            const int local = u % per;
            if (b < a.nwg && local > f4 && ((local - f4) & 1)) ++u;      // never between the two units of a 4-bit strip
            a.d_wg_first[b] = u;
            if (b < a.nwg) a.d_wg_seg[b] = min(u / per, a.nseg - 1);
        }
        if (threadIdx.x == 0) {
#pragma unroll
            for (int c = 0; c < GS_MAXSEG; ++c)
                if (c < a.nseg) a.d_segs[c] = a.segs[c];
            *a.d_sum = a.sum;
        }
    }
}

// =============================================================================================== host side
static inline size_t gs_align(size_t v) { return (v + 255) & ~(size_t)255; }
static inline int gs_round_up(int v, int m) { return (v + m - 1) / m * m; }

bool gemv_stream_supported(const lowra_layout& L, int M, int r) {
    return M >= 1 && M <= 16 && L.gv_nstrips > 0 && L.K % 256 == 0 && L.K >= 1024 && L.K <= GS_MAXSEG * GS_W * 256 &&
           L.C <= kGvMaxClasses && r >= 0 && r <= 32 && r % 8 == 0 && L.N > 0;
}

static int gs_nchunks(const lowra_layout& L) { return (L.K / 256 + GS_W - 1) / GS_W; }
// first strip of the 4-bit classes (classes are sorted by width): those strips count as two units
static int gs_first4(const lowra_layout& L) {
    int f = L.gv_nstrips;
    for (int c = kGvMaxClasses - 1; c >= 0; --c)
        if (c < L.gv_nclasses && (L.gv_cls_bits_cb[c] & 0xff) == 4) f = c == 0 ? 0 : L.gv_cls_end[c - 1];
    return f;
}
static int gs_units_per_seg(const lowra_layout& L) { return 2 * L.gv_nstrips - gs_first4(L); }

// table offsets: 4-bit tables first (their lookup needs a 16 KB aligned base), then the 4 KB ones
static GsTabs gs_tabs(const std::vector<uint8_t>& cb_bits) {
    GsTabs t{};
    t.nslot = (int)cb_bits.size();
    int off = 0;
    for (int c = 0; c < t.nslot; ++c) { t.bits[c] = cb_bits[(size_t)c]; if (t.bits[c] == 4) { t.off[c] = off; off += GS_T4B; } }
    for (int c = 0; c < t.nslot; ++c) if (t.bits[c] != 4) { t.off[c] = off; off += GS_T12B; }
    t.bytes = (off + 1023) & ~1023;
    return t;
}
static size_t gs_lds_bytes(const GsTabs& t) { return (size_t)t.bytes + 2 * GS_REDB + 2 * 16 * GS_TROW * 2 + (size_t)GS_W * GS_WAVEB; }

static hipError_t gs_attr() {
    static hipError_t a = hipFuncSetAttribute(reinterpret_cast<const void*>(gemv_stream_kernel),
                                              hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    return a;
}

static int gs_compute_units() {
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) v = 256;
        cus = v;
    }
    return cus;
}

// the segments (K-chunks) of one matrix; `part`: fp32 [nchunks][M][N] when there is more than one chunk
static int gs_make_segs(const lowra_layout& L, const uint8_t* packed, const float* absmax, const uint16_t* x, const uint16_t* B,
                        const float* tp, uint16_t* y, float* part, int M, int r, float s, GsSeg* out) {
    const int nblk_all = L.K / 256, nch = gs_nchunks(L);
    const GsTabs tabs = gs_tabs(L.cb_bits);
    for (int c = 0; c < nch; ++c) {
        GsSeg& g = out[c];
        g = GsSeg{};
        g.rows = L.d_gv_rows; g.packed = packed; g.absmax = absmax; g.x = x;
        g.B = (c == 0 && r > 0) ? B : nullptr;
        g.tp = tp;
        g.out = nch > 1 ? static_cast<void*>(part + (size_t)c * M * L.N) : static_cast<void*>(y);
        g.N = L.N; g.K = L.K; g.G = L.G; g.M = M; g.nstrips = L.gv_nstrips;
        g.first4 = gs_first4(L); g.nunits = gs_units_per_seg(L);
        g.kblk0 = c * GS_W; g.nblk = std::min(GS_W, nblk_all - c * GS_W); g.nblk_all = nblk_all;
        g.out_fp32 = nch > 1; g.r = r; g.RT = r > 0 ? gs_round_up(r, 16) : 0; g.s = s;
        for (int q = 0; q < kGvMaxClasses; ++q) {
            g.cls_end[q] = L.gv_cls_end[q];
            g.cls_bits_cb[q] = (L.gv_cls_bits_cb[q] & 0xff) | (tabs.off[(L.gv_cls_bits_cb[q] >> 8) & (kGvMaxClasses - 1)] << 8);
        }
    }
    return nch;
}

// workspace of a single call: [descriptors: segments | sum | wg_first | wg_seg][tp][fp32 partial outputs of the chunks]
constexpr size_t GS_DESC_BYTES = 16384, GS_DESC_SUM = 1024, GS_DESC_FIRST = 2048, GS_DESC_SEG = 8192;
constexpr int GS_MAXWG = 1024;
size_t gemv_stream_workspace_bytes(const lowra_layout& L, int M, int r) {
    const size_t tp = r > 0 ? gs_align((size_t)(L.K / 256) * 16 * gs_round_up(r, 16) * sizeof(float)) : 0;
    const size_t part = gs_nchunks(L) > 1 ? gs_align((size_t)gs_nchunks(L) * M * L.N * sizeof(float)) : 0;
    return GS_DESC_BYTES + tp + part;
}

hipError_t launch_gemv_stream(const lowra_layout& L, const LinearArgs& a, hipStream_t st) {
    hipError_t e = gs_attr();
    if (e != hipSuccess) return e;
    const GsTabs tabs = gs_tabs(L.cb_bits);
    uint8_t* ws = static_cast<uint8_t*>(a.workspace);
    const int nwg = std::min(std::min(gs_compute_units(), GS_MAXWG), gs_nchunks(L) * L.gv_nstrips);   // at least one strip each
    static_assert(GS_MAXSEG * sizeof(GsSeg) <= GS_DESC_SUM && GS_DESC_SUM + sizeof(GsSum) <= GS_DESC_FIRST &&
                  GS_DESC_FIRST + (GS_MAXWG + 1) * sizeof(int) <= GS_DESC_SEG && GS_DESC_SEG + GS_MAXWG * sizeof(int) <= GS_DESC_BYTES,
                  "descriptor area");
    if (nwg > GS_MAXWG) return hipErrorInvalidValue;
    GsSingle sg{};
    sg.d_segs = reinterpret_cast<GsSeg*>(ws);
    sg.d_sum = reinterpret_cast<GsSum*>(ws + GS_DESC_SUM);
    sg.d_wg_first = reinterpret_cast<int*>(ws + GS_DESC_FIRST);
    sg.d_wg_seg = reinterpret_cast<int*>(ws + GS_DESC_SEG);
    const size_t tpb = a.r > 0 ? gs_align((size_t)(L.K / 256) * 16 * gs_round_up(a.r, 16) * sizeof(float)) : 0;
    float* tp = reinterpret_cast<float*>(ws + GS_DESC_BYTES);
    float* part = reinterpret_cast<float*>(ws + GS_DESC_BYTES + tpb);
    sg.nseg = gs_make_segs(L, a.packed, a.absmax, a.act, a.B, tp, a.out, part, a.M, a.r, a.s, sg.segs);
    for (int c = 0; c < sg.nseg; ++c) sg.segs[c].first_unit = c * gs_units_per_seg(L);
    sg.nwg = nwg; sg.nblk_all = L.K / 256; sg.A = a.A;
    sg.sum = GsSum{part, a.out, a.M * L.N, sg.nseg};
    gemv_stream_prep_kernel<<<dim3(a.r > 0 ? sg.nblk_all : 1), dim3(64), 0, st>>>(sg);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    gemv_stream_kernel<<<dim3(nwg), dim3(GS_THREADS), gs_lds_bytes(tabs), st>>>(sg.d_segs, sg.d_wg_first, sg.d_wg_seg, a.mappings, tabs);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (sg.nseg > 1) {
        const int blocks = std::min(64, (a.M * L.N + 255) / 256);
        gemv_stream_sum_kernel<<<dim3(blocks), dim3(256), 0, st>>>(sg.d_sum, blocks);
        e = hipGetLastError();
    }
    return e;
}

// ---- a batch: descriptors built once on the host
template <typename T>
static hipError_t gs_to_device(const std::vector<T>& v, T** out) {
    if (v.empty()) { *out = nullptr; return hipSuccess; }
    hipError_t e = hipMalloc(reinterpret_cast<void**>(out), v.size() * sizeof(T));
    if (e != hipSuccess) return e;
    return hipMemcpy(*out, v.data(), v.size() * sizeof(T), hipMemcpyHostToDevice);
}

size_t gemv_stream_batch_item_ws(const lowra_layout& L, int r) {      // tp + chunk partials (for 16 tokens)
    const size_t tp = r > 0 ? gs_align((size_t)(L.K / 256) * 16 * gs_round_up(r, 16) * sizeof(float)) : 0;
    const size_t part = gs_nchunks(L) > 1 ? gs_align((size_t)gs_nchunks(L) * 16 * L.N * sizeof(float)) : 0;
    return tp + part;
}

void gemv_stream_batch_free(GsBatch& b) {
    (void)hipFree(b.d_segs); (void)hipFree(b.d_wg_first); (void)hipFree(b.d_wg_seg); (void)hipFree(b.d_sums);
    (void)hipFree(b.d_titems); (void)hipFree(b.d_towner);
    b = GsBatch{};
}

hipError_t gemv_stream_batch_build(const std::vector<GsBatchItem>& items, const float* mappings, int M, int r, float s, GsBatch& b) {
    if (items.empty()) return hipSuccess;
    std::vector<GsSeg> segs;
    std::vector<GsSum> sums;
    std::vector<GsTItem> titems;
    std::vector<int> towner;
    std::vector<double> unit_cost;                                   // bytes of codes and scales per unit
    std::vector<char> pair_second;                                   // the unit is the second half of a 4-bit strip
    constexpr double kUnitFixedCost = 4096.0;
    int units = 0;
    for (const GsBatchItem& it : items) {
        const lowra_layout& L = *it.L;
        const size_t tpb = r > 0 ? gs_align((size_t)(L.K / 256) * 16 * gs_round_up(r, 16) * sizeof(float)) : 0;
        float* tp = reinterpret_cast<float*>(it.ws);
        float* part = reinterpret_cast<float*>(it.ws + tpb);
        GsSeg tmp[GS_MAXSEG];
        const int nch = gs_make_segs(L, it.packed, it.absmax, it.x, it.B, tp, it.y, part, M, r, s, tmp);
        for (int c = 0; c < nch; ++c) {
            tmp[c].first_unit = units;
            segs.push_back(tmp[c]);
            for (int sidx = 0; sidx < L.gv_nstrips; ++sidx) {
                int cls = L.gv_cls_bits_cb[0];
                for (int q = 0; q + 1 < kGvMaxClasses; ++q) if (sidx >= L.gv_cls_end[q]) cls = L.gv_cls_bits_cb[q + 1];
                const int b = cls & 0xff;
                // bytes of codes and scales of a unit, plus a constant for its fixed work
                const double cost = 16.0 * tmp[c].nblk * (b == 1 ? 32.0 + 16.0 : 64.0 + 16.0) + kUnitFixedCost;
                unit_cost.push_back(cost);
                pair_second.push_back(0);
                if (b == 4) { unit_cost.push_back(cost); pair_second.push_back(1); }
            }
            units += tmp[c].nunits;
        }
        if (nch > 1) sums.push_back(GsSum{part, it.y, M * L.N, nch});
        if (r > 0) {
            const int blk0 = (int)towner.size();
            titems.push_back(GsTItem{it.x, it.A, tp, M, L.K, r, gs_round_up(r, 16), blk0});
            towner.insert(towner.end(), (size_t)(L.K / 256), (int)titems.size() - 1);
        }
    }
    // contiguous unit ranges of (nearly) equal bytes
    const int nwg = std::min(gs_compute_units(), units);
    double total = 0.0;
    for (double c : unit_cost) total += c;
    std::vector<int> wg_first((size_t)nwg + 1, units), wg_seg((size_t)nwg, 0);
    {
        double acc = 0.0;
        int w = 0;
        wg_first[0] = 0;
        for (int u = 0; u < units; ++u) {
            while (w + 1 < nwg && acc >= total * (w + 1) / nwg && !pair_second[(size_t)u]) wg_first[(size_t)++w] = u;
            acc += unit_cost[(size_t)u];
        }
        while (w + 1 < nwg) wg_first[(size_t)++w] = units;
        wg_first[(size_t)nwg] = units;
        size_t sg = 0;
        for (int q = 0; q < nwg; ++q) {
            while (sg + 1 < segs.size() && segs[sg + 1].first_unit <= wg_first[(size_t)q]) ++sg;
            wg_seg[(size_t)q] = (int)sg;
        }
    }
    b.nwg = nwg; b.nsums = (int)sums.size(); b.nt_blocks = (int)towner.size(); b.mappings = mappings;
    b.max_count = 0;
    for (const GsSum& q : sums) b.max_count = std::max(b.max_count, q.count);
    b.cb_bits = items[0].L->cb_bits;
    hipError_t e;
    if ((e = gs_to_device(segs, reinterpret_cast<GsSeg**>(&b.d_segs))) != hipSuccess) return e;
    if ((e = gs_to_device(wg_first, &b.d_wg_first)) != hipSuccess) return e;
    if ((e = gs_to_device(wg_seg, &b.d_wg_seg)) != hipSuccess) return e;
    if ((e = gs_to_device(sums, reinterpret_cast<GsSum**>(&b.d_sums))) != hipSuccess) return e;
    if ((e = gs_to_device(titems, reinterpret_cast<GsTItem**>(&b.d_titems))) != hipSuccess) return e;
    if ((e = gs_to_device(towner, &b.d_towner)) != hipSuccess) return e;
    return gs_attr();
}

hipError_t gemv_stream_batch_run(const GsBatch& b, hipStream_t st) {
    if (b.nwg == 0) return hipSuccess;
    hipError_t e;
    if (b.nt_blocks > 0) {
        gemv_stream_t_kernel<<<dim3(b.nt_blocks), dim3(64), 0, st>>>(static_cast<const GsTItem*>(b.d_titems), b.d_towner);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    const GsTabs tabs = gs_tabs(b.cb_bits);
    {
        KernelTimer timer(st);
        gemv_stream_kernel<<<dim3(b.nwg), dim3(GS_THREADS), gs_lds_bytes(tabs), st>>>(static_cast<const GsSeg*>(b.d_segs), b.d_wg_first,
                                                                                      b.d_wg_seg, b.mappings, tabs);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    if (b.nsums > 0) {
        const int blocks = std::min(64, (b.max_count + 255) / 256);
        gemv_stream_sum_kernel<<<dim3(b.nsums * blocks), dim3(256), 0, st>>>(static_cast<const GsSum*>(b.d_sums), blocks);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace lowra
