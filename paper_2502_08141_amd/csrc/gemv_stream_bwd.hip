// Streaming small-token input gradient (M <= 16):  dX = dY What + (s dY B) A over one or many matrices
// (Sec. 4.1 for What; the base weights are frozen, so this is the only gradient that flows through them).
//
// The same stream of units as the forward kernel (16-channel class-sorted strips, 16 bytes of codes per lane
// and unit, global -> LDS rings private to each wavefront), but the contraction now runs over the CHANNELS:
//
//  * Wavefront w owns the 256 columns [256 w, 256 w + 256) of the K-chunk and keeps dX for them in
//    registers (16 tiles of 16 tokens x 16 columns) across ALL the units of a run -- the wavefronts never
//    meet: no barrier, no reduction per unit.
//  * v_mfma_f32_16x16x16_bf16 wants, per lane, four consecutive contraction indices (channels) of one column,
//    while a byte of codes decodes into the levels of consecutive columns of one channel.  Lane (c, nq) looks
//    up byte c of channels nq, nq + 4, nq + 8, nq + 12 (one byte read and one table read each; the order of the
//    contraction index is free as long as both operands agree) and transposes the 4 x 4
//    block of bf16 in registers (v_perm_b32).  A tile's 16 columns are then {f(c, e)}: 64 g + 4 c + e at one
//    and two bits, 64 g + 32 h + 2 c + e for half h of a 4-bit strip.  All columns of a tile share a group,
//    so the group scale (which depends on the channel, the contraction index) multiplies the dY operand:
//    bf16(dY[m][n] absmax[n][g]), four products per lane and group.
//  * dY arrives gathered into strip order ([strip][token][16 channels], zero for padding rows and past M) by
//    a small kernel before, which also forms the partial sums of u = dY B.
//  * A run (consecutive units of one workgroup in one K-chunk with one column mapping) ends with a store
//    of the accumulators into a partial slot [M][2048] fp32; a last kernel adds the slots of each chunk in
//    a fixed order, adds s u A and rounds to bf16.
#include <cmath>
#include <cstddef>

#include "gemv_stream.h"

namespace lowra {

#ifndef GB_EXP
#define GB_EXP 0      // measurement variants (bit flags), 0 in the product: 1 no dY transfers, 2 no scale transfers, 4 no code transfers
#endif
#ifndef GB_SYNC
#define GB_SYNC 16     // a workgroup barrier every so many units keeps its wavefronts on the same cache lines (0: never)
#endif
#ifndef GB_WAVES
#define GB_WAVES 16
#endif
#ifndef GB_DEPTH
#define GB_DEPTH 2
#endif
constexpr int GB_W = GB_WAVES;           // wavefronts per workgroup = 256-column blocks per K-chunk
constexpr int GB_THREADS = GB_W * 64;
constexpr int GB_MAXSEG = 64 / GB_W;     // K-chunks of one row at most (K <= 16384)
constexpr int GB_D = GB_DEPTH;                 // units whose codes are in flight per wavefront (the ring has GB_D + 1 slots)
constexpr int GB_CODEB = 1024, GB_SCALEB = 256, GB_DYB = 512;
constexpr int GB_SLOTB = GB_CODEB + GB_SCALEB + GB_DYB;
constexpr int GB_WAVEB = (GB_D + 1) * (GB_SLOTB + GS_RECB);   // per wavefront: ring, record ring
constexpr int GB_CHUNK = GB_W * 256;     // columns of a K-chunk = floats per token row of a partial slot
constexpr int GB_MAXWG = 256;
constexpr int GB_PRE_WAVES = 16;
constexpr int GB_PRE_U = 4;              // strips a set-up wavefront handles at a time
constexpr int GB_MAXPRE = 16;           // set-up workgroups per matrix at most (a batch runs the same number for every matrix)
static_assert(GS_MAXTAB * GS_TABB + GB_W * GB_WAVEB <= 160 * 1024, "LDS budget");

typedef short gb_bf16x4_t __attribute__((ext_vector_type(4)));

// One (matrix, K-chunk)
struct GbSeg {
    const GvRow* rows;       // [nstrips * 16] class-sorted row records
    const uint8_t* packed;
    const float* absmax;
    const uint16_t* dys;     // [nstrips][16 tokens][16 channels] bf16: dY in strip order (entry 4 q + v of a token: channel q + 4 v)
    int G;
    int kblk0, nblk;         // first 256-column block of the chunk, and how many (1..16)
    int pad;
};
typedef const __attribute__((address_space(4))) GbSeg* gb_cseg_t;

#define GB_LOAD_ISSUE(p)                                                                                          \
    do {                                                                                                          \
        iPacked = (p)->packed; iDys = reinterpret_cast<const uint8_t*>((p)->dys); iG4 = (sb16 ? 2 : 4) * (p)->G;  \
        iKb32 = 32 * ((p)->kblk0 + min(wave, (p)->nblk - 1)); /* past the chunk's end: the last block again (unused) */ \
        iScaleBase = reinterpret_cast<const uint8_t*>((p)->absmax) + (size_t)(iKb32 >> (sb16 ? 2 : 1));           \
    } while (0)

__device__ __forceinline__ gb_bf16x4_t gb_pack4(float a, float b, float c, float d) {
    return __builtin_bit_cast(gb_bf16x4_t, make_uint2(pack_bf16x2(a, b), pack_bf16x2(c, d)));
}
// the 4 x 4 block lv[channel v] = (levels of 4 consecutive columns) -> w[column e] = (levels of the 4 channels)
__device__ __forceinline__ void gb_transpose4x4(const uint2 (&lv)[4], gb_bf16x4_t (&w)[4]) {
    w[0] = __builtin_bit_cast(gb_bf16x4_t, make_uint2(__builtin_amdgcn_perm(lv[1].x, lv[0].x, 0x05040100u), __builtin_amdgcn_perm(lv[3].x, lv[2].x, 0x05040100u)));
    w[1] = __builtin_bit_cast(gb_bf16x4_t, make_uint2(__builtin_amdgcn_perm(lv[1].x, lv[0].x, 0x07060302u), __builtin_amdgcn_perm(lv[3].x, lv[2].x, 0x07060302u)));
    w[2] = __builtin_bit_cast(gb_bf16x4_t, make_uint2(__builtin_amdgcn_perm(lv[1].y, lv[0].y, 0x05040100u), __builtin_amdgcn_perm(lv[3].y, lv[2].y, 0x05040100u)));
    w[3] = __builtin_bit_cast(gb_bf16x4_t, make_uint2(__builtin_amdgcn_perm(lv[1].y, lv[0].y, 0x07060302u), __builtin_amdgcn_perm(lv[3].y, lv[2].y, 0x07060302u)));
}

// ---- LDS access by 32-bit address (the arithmetic works on addresses it builds with one instruction each)
typedef const __attribute__((address_space(3))) uint8_t* gb_l8_t;
typedef const __attribute__((address_space(3))) uint32_t* gb_l32_t;
typedef unsigned int gb_u32x2_t __attribute__((ext_vector_type(2)));
typedef const __attribute__((address_space(3))) gb_u32x2_t* gb_l64_t;
typedef const __attribute__((address_space(3))) floatx4_t* gb_l128_t;
__device__ __forceinline__ uint32_t gb_lds_u8(uint32_t a) { return *(gb_l8_t)(uintptr_t)a; }
__device__ __forceinline__ uint32_t gb_lds_b32(uint32_t a) { return *(gb_l32_t)(uintptr_t)a; }
__device__ __forceinline__ uint2 gb_lds_b64(uint32_t a) { const gb_u32x2_t v = *(gb_l64_t)(uintptr_t)a; return make_uint2(v.x, v.y); }
__device__ __forceinline__ float4 gb_lds_b128(uint32_t a) { const floatx4_t v = *(gb_l128_t)(uintptr_t)a; return make_float4(v[0], v[1], v[2], v[3]); }
// (byte << 6) | rest: the table entry of a byte of codes (v_lshl_or_b32)
__device__ __forceinline__ uint32_t gb_entry(uint32_t byte, uint32_t rest) { return (byte << 6) | rest; }

// operand of dY for the four groups: lane (token c, channels nq + 4 v), times the channels' group scales
__device__ __forceinline__ void gb_scaled_dy(const uint32_t slot, const int c, const int nq, const bool sb16, gb_bf16x4_t (&a)[4]) {
    const uint2 dyq = gb_lds_b64(slot + GB_CODEB + GB_SCALEB + 32 * c + 8 * nq);
    float sc[4][4];
    if (sb16) {                                                     // uniform: 8 bytes of bf16 scales per channel
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const uint2 h = gb_lds_b64(slot + GB_CODEB + 8 * nq + 32 * v);
            sc[v][0] = bf16_bits_to_float(h.x & 0xffffu); sc[v][1] = __builtin_bit_cast(float, h.x & 0xffff0000u);
            sc[v][2] = bf16_bits_to_float(h.y & 0xffffu); sc[v][3] = __builtin_bit_cast(float, h.y & 0xffff0000u);
        }
    } else {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const float4 q = gb_lds_b128(slot + GB_CODEB + 16 * nq + 64 * v);
            sc[v][0] = q.x; sc[v][1] = q.y; sc[v][2] = q.z; sc[v][3] = q.w;
        }
    }
    const float dyf[4] = {bf16_bits_to_float(dyq.x & 0xffffu), __builtin_bit_cast(float, dyq.x & 0xffff0000u),
                          bf16_bits_to_float(dyq.y & 0xffffu), __builtin_bit_cast(float, dyq.y & 0xffff0000u)};
#pragma unroll
    for (int g = 0; g < 4; ++g) a[g] = gb_pack4(dyf[0] * sc[0][g], dyf[1] * sc[1][g], dyf[2] * sc[2][g], dyf[3] * sc[3][g]);
}

// One unit at one or two bits.  Group g of channel n sits at 16 (16 g + n) (two bits; byte c = columns 64 g + 4 c .. + 3) or
// in the pair of groups at 16 (32 (g / 2) + n) + 8 (g % 2) (one bit; the low or high four codes of byte c / 2 are those
// columns): the two widths differ in a shift, four offsets and the lane's table copy, all selected without a branch.
__device__ __forceinline__ void gb_unit_low(const uint32_t slot, const bool one, const uint32_t tbv, const int lane, const bool sb16, floatx4_t (&acc)[16]) {
    const int c = lane & 15, nq = lane >> 4;
    gb_bf16x4_t a[4];
    gb_scaled_dy(slot, c, nq, sb16, a);
    const uint32_t cb = slot + 16 * nq + (c >> (one ? 1 : 0));
    uint32_t byte[4][4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const uint32_t cg = cb + (one ? 512 * (g >> 1) + 8 * (g & 1) : 256 * g);
#pragma unroll
        for (int v = 0; v < 4; ++v) byte[g][v] = gb_lds_u8(cg + 64 * v);
    }
    uint2 lv[4][4];
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int v = 0; v < 4; ++v) lv[g][v] = gb_lds_b64(gb_entry(byte[g][v], tbv));
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        gb_bf16x4_t w[4];
        gb_transpose4x4(lv[g], w);
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[4 * g + e] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a[g], w[e], acc[4 * g + e], 0, 0, 0);
    }
}

// One half (HALF) of a 4-bit strip: half HALF of group g of channel n at 16 (16 g + n); byte c = columns 64 g + 32 HALF + 2 c, + 1
template <int HALF>
__device__ __forceinline__ void gb_unit_four(const uint32_t slot, const uint32_t tbv, const int lane, const bool sb16, floatx4_t (&acc)[16]) {
    const int c = lane & 15, nq = lane >> 4;
    gb_bf16x4_t a[4];
    gb_scaled_dy(slot, c, nq, sb16, a);
    const uint32_t cb = slot + 16 * nq + c;
    uint32_t byte[4][4];
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int v = 0; v < 4; ++v) byte[g][v] = gb_lds_u8(cb + 256 * g + 64 * v);
    uint32_t lv[4][4];
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int v = 0; v < 4; ++v) lv[g][v] = gb_lds_b32(gb_entry(byte[g][v], tbv));
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const gb_bf16x4_t w0 = __builtin_bit_cast(gb_bf16x4_t, make_uint2(__builtin_amdgcn_perm(lv[g][1], lv[g][0], 0x05040100u), __builtin_amdgcn_perm(lv[g][3], lv[g][2], 0x05040100u)));
        const gb_bf16x4_t w1 = __builtin_bit_cast(gb_bf16x4_t, make_uint2(__builtin_amdgcn_perm(lv[g][1], lv[g][0], 0x07060302u), __builtin_amdgcn_perm(lv[g][3], lv[g][2], 0x07060302u)));
        acc[4 * g + 2 * HALF + 0] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a[g], w0, acc[4 * g + 2 * HALF + 0], 0, 0, 0);
        acc[4 * g + 2 * HALF + 1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a[g], w1, acc[4 * g + 2 * HALF + 1], 0, 0, 0);
    }
}

__global__ __launch_bounds__(GB_THREADS) void gemv_stream_bwd_kernel(const GbSeg* __restrict__ segs_g, const GsUnit* __restrict__ units_g,
                                                                     const int* __restrict__ wg_first_g, const int* __restrict__ wg_slot0_g,
                                                                     const float* __restrict__ mappings, const GsTabs tabs,
                                                                     float* __restrict__ part, const int M) {
    const gb_cseg_t segs = reinterpret_cast<gb_cseg_t>(reinterpret_cast<uintptr_t>(segs_g));
    const gs_cunit_t units = reinterpret_cast<gs_cunit_t>(reinterpret_cast<uintptr_t>(units_g));
    const gs_cint_t wg_first = reinterpret_cast<gs_cint_t>(reinterpret_cast<uintptr_t>(wg_first_g));
    const gs_cint_t wg_slot0 = reinterpret_cast<gs_cint_t>(reinterpret_cast<uintptr_t>(wg_slot0_g));
    extern __shared__ __align__(16) uint8_t gb_smem[];
    // LDS: [tables: nslot x GS_TABB] [per wavefront: ring of GB_D + 1 slots, record ring of GB_D + 1 slots]
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int i = lane & 15, kg = lane >> 4;
    const uint32_t smem_lds = (uint32_t)(uintptr_t)(lptr_t)gb_smem;
    const int RING0 = tabs.nslot * GS_TABB + wave * GB_WAVEB, REC0 = RING0 + (GB_D + 1) * GB_SLOTB;

    gs_fill_tables(gb_smem, mappings, tabs);
    // the record slots start as a valid record (offset 0, no channel): the first requests read them before any has landed
    for (int o = lane; o < (GB_D + 1) * GS_RECB / 8; o += 64)
        *reinterpret_cast<uint2*>(gb_smem + REC0 + 8 * o) = make_uint2(0u, 0xffffffffu);
    __syncthreads();

    const int u0 = wg_first[blockIdx.x], n = wg_first[blockIdx.x + 1] - u0;
    if (n <= 0) return;                                             // whole workgroup
    const gs_cunit_t myunits = units + u0;
    int slot = wg_slot0[blockIdx.x];                                // partial slot of my current run

    // ---- three stages walk the same unit list: records (2 GB_D ahead), codes / scales / dY (GB_D ahead), arithmetic.
    // A stage past the end of the list (or before its start) repeats the last (first) unit: same transfers, no effect.
    GsUnit uR = gs_load_unit(myunits), uI = uR, uC = uR;
    int segR = (int)uR.seg, segI = (int)uI.seg, segC = (int)uC.seg;
    const uint8_t* rowsR = reinterpret_cast<const uint8_t*>(segs[segR].rows);
    const uint8_t* iPacked; const uint8_t* iScaleBase; const uint8_t* iDys;
    int iG4, iKb32;
    const bool sb16 = tabs.scale_bf16 != 0;                         // uniform
    GB_LOAD_ISSUE(segs + segI);
    int mNblk = segs[segC].nblk;

    floatx4_t acc[16];
#pragma unroll
    for (int q = 0; q < 16; ++q) acc[q] = floatx4_t{0.0f, 0.0f, 0.0f, 0.0f};

    // per-lane constants of the requests and of the table reads
    const uint32_t code_lane1 = 16u * (kg >> 1), code_lane2 = 16u * kg, code_lane4 = 32u * kg;
    // scales: fp32, lane l fetches group l % 4 of channel l / 4; bf16, lane l < 32 fetches dword l % 2 of channel l / 2
    const uint32_t rec_voff = 4u * (lane & 31), scale_lane = sb16 ? 4u * (lane & 1) : 4u * (lane & 3), dy_voff = 16u * (lane & 31);
    const uint32_t rec_mine = 8u * i, rec_scale = sb16 ? 8u * ((lane & 31) >> 1) : 8u * (lane >> 2);
    const uint32_t tb1 = smem_lds + 16u * (lane & 3) + 8u * (lane & 1), tb2 = smem_lds + 8u * (lane & 7), tb4 = smem_lds + 4u * (lane & 15);
    const uint32_t ring_begin = smem_lds + RING0, ring_end = ring_begin + (GB_D + 1) * GB_SLOTB;
    const uint32_t rec_begin = smem_lds + REC0, rec_end = rec_begin + (GB_D + 1) * GS_RECB;
    uint32_t ringW = ring_begin, ringRd = ring_begin + GB_SLOTB;    // the slot filled now (unit j + GB_D) and the one unit j sits in
    uint32_t recW = rec_begin, recRd = rec_begin + GS_RECB;         // same for the records of units j + 2 GB_D and j + GB_D

    // One pass: the requests of the units ahead, then the arithmetic of unit J in the instruction stream MODE names
    // (0: none yet, 1: one or two bits, 2 / 3: first / second half of a 4-bit strip).  ENDS: whether unit J ends a run
    // (last unit, or the next one sits in another chunk or has the other column mapping).  A macro: as a lambda the
    // captured state (the accumulators above all) ended up in private memory.
#define GB_PASS(MODE, J, ENDS)                                                                                  \
    do {                                                                                                          \
        /* the next pass's units, asked for now (scalar loads), used after this pass */                               \
        const GsUnit nR = gs_load_unit(myunits + min((J) + 1 + 2 * GB_D, n - 1));                                     \
        const GsUnit nI = gs_load_unit(myunits + min(max((J) + 1 + GB_D, 0), n - 1));                                 \
        const GsUnit nC = gs_load_unit(myunits + min(max((J) + 1, 0), n - 1));                                        \
                                                                                                                      \
        /* ================= request: the row records of unit j + 2 GB_D (lane l < 32: dword l of the strip's 16 records) */ \
        if (GB_SYNC > 0 && (((J) + 2 * GB_D) % GB_SYNC) == 0) __builtin_amdgcn_s_barrier();                           \
        gs_dma4_low32(gs_uniform(rowsR + uR.rows_off), rec_voff, recW);                                               \
        recW = recW + GS_RECB == rec_end ? rec_begin : recW + GS_RECB;                                                \
                                                                                                                      \
        /* The transfers of unit j (issued GB_D passes ago) have landed: after them came GB_D - 1 passes of 4 transfers */ \
        /* each and this pass's record request.  The records of unit j + GB_D are older still. */                     \
        gs_wait_transfers<4 * GB_D - 3>();                                                                            \
        const uint2 rc = gb_lds_b64(recRd + rec_mine);              /* my channel's record */                         \
        const uint2 rs = gb_lds_b64(recRd + rec_scale);             /* the record of the channel whose scale I fetch */ \
        recRd = recRd + GS_RECB == rec_end ? rec_begin : recRd + GS_RECB;                                             \
                                                                                                                      \
        /* ================= request: codes, scales and dY fragment of unit j + GB_D, into the slot that the previous */ \
        /* pass read (its LDS reads have returned: waited for below).  Issued on every pass. */                       \
        {                                                                                                             \
            const int bits = (int)(uI.flags & 15u), halfI = (int)((uI.flags >> 4) & 1u);                              \
            /* codes: 16 bytes per lane.  2 bits: group kg.  4 bits: half halfI of group kg.  1 bit: the aligned pair of */ \
            /* groups that holds group kg (a group is 8 bytes; rows are 32-byte aligned). */                          \
            const uint8_t* cbase = iPacked + (size_t)(iKb32 * bits + 16 * halfI);                                     \
            gs_wait_lds();                                                                                            \
            const uint32_t cvoff = rc.x + (bits == 2 ? code_lane2 : bits == 4 ? code_lane4 : code_lane1);             \
            const uint32_t svoff = (uint32_t)max((int)rs.y, 0) * (uint32_t)iG4 + scale_lane;                          \
            if (!(GB_EXP & 4)) dma16_s(gs_uniform(cbase), cvoff, ringW);                                              \
            if (!(GB_EXP & 2)) {                                                                                      \
                if (sb16) gs_dma4_low32(gs_uniform(iScaleBase), svoff, ringW + GB_CODEB);                             \
                else dma4_s(gs_uniform(iScaleBase), svoff, ringW + GB_CODEB);                                         \
            }                                                                                                         \
            if (!(GB_EXP & 1)) gs_dma16_low32(gs_uniform(iDys + 4u * uI.rows_off), dy_voff, ringW + GB_CODEB + GB_SCALEB);   /* 512 bytes per strip, 128 of records */ \
            ringW = ringW + GB_SLOTB == ring_end ? ring_begin : ringW + GB_SLOTB;                                     \
        }                                                                                                             \
                                                                                                                      \
        /* ================= arithmetic of unit j */                                                                  \
        ENDS = false;                                                                                                 \
        if (MODE != 0) {                                                                                              \
            const uint32_t toff = ((uC.flags >> 6) & 3u) * (uint32_t)GS_TABB;                                         \
            if (MODE == 1) {                                                                                          \
                const bool one = (uC.flags & 15u) == 1u;                                                              \
                gb_unit_low(ringRd, one, (one ? tb1 : tb2) + toff, lane, sb16, acc);                                        \
            } else if (MODE == 2) {                                                                                   \
                gb_unit_four<0>(ringRd, tb4 + toff, lane, sb16, acc);                                                       \
            } else {                                                                                                  \
                gb_unit_four<1>(ringRd, tb4 + toff, lane, sb16, acc);                                                       \
            }                                                                                                         \
            ENDS = (J) == n - 1 || nC.seg != uC.seg || ((nC.flags & 15u) == 4u) != (MODE != 1);                       \
        }                                                                                                             \
        ringRd = ringRd + GB_SLOTB == ring_end ? ring_begin : ringRd + GB_SLOTB;                                      \
                                                                                                                      \
        /* ================= the next pass's units and, where they change, segments */                                \
        uR = nR; uI = nI; uC = nC;                                                                                    \
        if ((int)uR.seg != segR) { segR = (int)uR.seg; rowsR = reinterpret_cast<const uint8_t*>(segs[segR].rows); }   \
        if ((int)uI.seg != segI) { segI = (int)uI.seg; GB_LOAD_ISSUE(segs + segI); }                                  \
        if ((int)uC.seg != segC) { segC = (int)uC.seg; mNblk = segs[segC].nblk; }                                     \
    } while (0)

    // The end of a run: my 16 x 256 block of its partial slot (the chunk of the run is the one the arithmetic stage was in
    // before the last pass moved on: `nblk` was read before).
#define GB_FLUSH(FOUR, NBLK)                                                                                    \
    do {                                                                                                          \
        if (wave < (NBLK)) {                                                                                          \
            float* dst = part + (size_t)slot * ((size_t)M * GB_CHUNK) + 256 * wave;                                   \
_Pragma("unroll")                                                                                                     \
            for (int v = 0; v < 4; ++v) {                                                                             \
                const int m = 4 * kg + v;                           /* result rows of my lanes: tokens 4 kg .. 4 kg + 3, column role i */ \
                if (m < M) {                                                                                          \
                    float* row = dst + (size_t)m * GB_CHUNK;                                                          \
                    if (!(FOUR)) {                                                                                    \
_Pragma("unroll")                                                                                                     \
                        for (int g = 0; g < 4; ++g)                                                                   \
                            *reinterpret_cast<float4*>(row + 64 * g + 4 * i) = make_float4(acc[4 * g][v], acc[4 * g + 1][v], acc[4 * g + 2][v], acc[4 * g + 3][v]); \
                    } else {                                                                                          \
_Pragma("unroll")                                                                                                     \
                        for (int g = 0; g < 4; ++g) {                                                                 \
                            *reinterpret_cast<float2*>(row + 64 * g + 2 * i) = make_float2(acc[4 * g][v], acc[4 * g + 1][v]); \
                            *reinterpret_cast<float2*>(row + 64 * g + 32 + 2 * i) = make_float2(acc[4 * g + 2][v], acc[4 * g + 3][v]); \
                        }                                                                                             \
                    }                                                                                                 \
                }                                                                                                     \
            }                                                                                                         \
        }                                                                                                             \
_Pragma("unroll")                                                                                                     \
        for (int q = 0; q < 16; ++q) acc[q] = floatx4_t{0.0f, 0.0f, 0.0f, 0.0f};                                      \
        ++slot;                                                                                                       \
    } while (0)

    int j = -2 * GB_D;
    bool ends = false;
    for (; j < 0; ++j) GB_PASS(0, j, ends);
    while (j < n) {                                                 // uniform: one run per round
        const int nblk = mNblk;
        if ((uC.flags & 15u) != 4u) {
            do { GB_PASS(1, j, ends); ++j; } while (!ends);
            GB_FLUSH(false, nblk);
        } else {                                                    // the two halves of a strip are consecutive units of one workgroup
            do { GB_PASS(2, j, ends); GB_PASS(3, j + 1, ends); j += 2; } while (!ends);
            GB_FLUSH(true, nblk);
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                // nothing of mine may land in LDS after I am gone
}

// ---- before: dY gathered into strip order, and partial sums of u = dY B (one per workgroup), for one matrix.
// Lane (m, nq) handles token m and the strip's channels nq + 4 v (v = 0..3): its 8 bytes are the MFMA operand, here and
// in the streaming kernel (whose four lanes of a column then read four neighbouring 16-byte rows of codes at a time:
// all LDS banks, no conflict).
struct GbPre {
    const GvRow* rows; const uint16_t* dY; const uint16_t* B;
    uint16_t* dys;           // [nstrips][16][16] bf16 (out)
    float* upart;            // [P][16][GS_TROW] fp32 (out), only when r > 0
    int N, M, r, nstrips;
};
__device__ __forceinline__ void gb_pre_body(const GbPre& it, const int p, const int P) {
    __shared__ float red[GB_PRE_WAVES][16 * GS_TROW];
    // per wavefront: a strip's dY fragment [16 tokens][16 entries] and its rows of B [16 rows][GS_TROW] (bf16), on
    // their way from the lanes that fetch them to the lanes whose MFMA operands they are
    __shared__ __align__(16) uint16_t xch[GB_PRE_WAVES][16 * 16 + 16 * GS_TROW];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, m = lane & 15, nq = lane >> 4;
    // As a loader, lane l is row l % 16 of the strip: it reads the row's record, its channel's dY of tokens
    // l / 16 + 4 u, and 16 bytes (ranks 8 (l / 16) ..) of its row of B -- one load instruction per strip for the
    // records, one per four tokens for dY, one for B, where one lane per operand element took thirteen, and the
    // kernel's time was their address processing.  Ranks that are no multiple of 8 keep the element-wise loads of B.
    const int entry = 4 * (m & 3) + (m >> 2);                     // where row m's channel sits among a token's 16 entries
    uint16_t* T = xch[wave];
    uint16_t* Bt = T + 256;
    const bool vec_b = it.r > 0 && (it.r & 7) == 0;
    const auto rows = as_global(it.rows);
    const auto dY = as_global(it.dY), B = as_global(it.B);
    const auto dys = as_global(it.dys);
    const auto upart = as_global(it.upart);
    floatx4_t au[2] = {{0.0f, 0.0f, 0.0f, 0.0f}, {0.0f, 0.0f, 0.0f, 0.0f}};
    // GB_PRE_U strips per pass, every load of a stage requested before the first is used: a wavefront's time is a
    // chain of dependent round trips (records -> dY and B -> product), not bytes
    for (int s0 = p * GB_PRE_WAVES + wave; s0 < it.nstrips; s0 += GB_PRE_WAVES * P * GB_PRE_U) {
        int n[GB_PRE_U];
#pragma unroll
        for (int q = 0; q < GB_PRE_U; ++q) {
            const int strip = s0 + q * GB_PRE_WAVES * P;
            n[q] = strip < it.nstrips ? rows[strip * 16 + m].n : -1;     // uniform condition
        }
        uint32_t dv[GB_PRE_U][4];
        uint4 bq[GB_PRE_U];
        uint32_t bv[GB_PRE_U][2][4];
#pragma unroll
        for (int q = 0; q < GB_PRE_U; ++q) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int mm = nq + 4 * u;
                dv[q][u] = (mm < it.M && n[q] >= 0) ? dY[(size_t)mm * it.N + n[q]] : 0u;
            }
            bq[q] = zero4();
            if (vec_b) {
                if (8 * nq < it.r && n[q] >= 0) bq[q] = gload_u4(B + (size_t)n[q] * it.r + 8 * nq);
            } else if (it.r > 0) {
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int ch = __shfl(n[q], nq + 4 * v);        // the channel of row nq + 4 v
#pragma unroll
                    for (int jt = 0; jt < 2; ++jt) {
                        const int jr = 16 * jt + m;                 // my column of B in this tile
                        bv[q][jt][v] = (jr < it.r && ch >= 0) ? B[(size_t)ch * it.r + jr] : 0u;
                    }
                }
            }
        }
#pragma unroll
        for (int q = 0; q < GB_PRE_U; ++q) {
            const int strip = s0 + q * GB_PRE_WAVES * P;
            if (strip >= it.nstrips) break;
#pragma unroll
            for (int u = 0; u < 4; ++u) T[(nq + 4 * u) * 16 + entry] = (uint16_t)dv[q][u];
            if (vec_b) *reinterpret_cast<uint4*>(Bt + m * GS_TROW + 8 * nq) = bq[q];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            const uint2 frag = *reinterpret_cast<const uint2*>(T + m * 16 + 4 * nq);
            gstore_u2(dys + (size_t)strip * 256 + m * 16 + 4 * nq, frag);
            if (it.r > 0) {
#pragma unroll
                for (int jt = 0; jt < 2; ++jt) {
                    uint32_t b[4];
#pragma unroll
                    for (int v = 0; v < 4; ++v) b[v] = vec_b ? (uint32_t)Bt[(nq + 4 * v) * GS_TROW + 16 * jt + m] : bv[q][jt][v];
                    au[jt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(gb_bf16x4_t, frag),
                                                                       __builtin_bit_cast(gb_bf16x4_t, make_uint2(b[0] | (b[1] << 16), b[2] | (b[3] << 16))),
                                                                       au[jt], 0, 0, 0);
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();                        // the next strip overwrites T and Bt
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
    }
    if (it.r > 0) {
        // lane (j, nq) holds u[token 4 nq + v][rank 16 jt + j]
#pragma unroll
        for (int jt = 0; jt < 2; ++jt)
#pragma unroll
            for (int v = 0; v < 4; ++v) red[wave][(4 * nq + v) * GS_TROW + 16 * jt + m] = au[jt][v];
        __syncthreads();
        for (int o = threadIdx.x; o < 16 * GS_TROW; o += GB_PRE_WAVES * 64) {
            float s = 0.0f;
#pragma unroll
            for (int w = 0; w < GB_PRE_WAVES; ++w) s += red[w][o];  // fixed order
            upart[(size_t)p * 16 * GS_TROW + o] = s;
        }
    }
}

// ---- after: dX = bf16(sum of the chunk's partial slots + s u A), for one matrix
struct GbItem {
    const float* part; const float* upart; const uint16_t* A; uint16_t* dX;
    int slot0[GB_MAXSEG], nslots[GB_MAXSEG];
    int M, K, r, nup;        // nup: partial sums of u
    float s;
    int pad;
};
// Few slots per chunk (a batch: a workgroup's range covers whole chunks): one thread per quad of columns adds
// them all, for every token (MT: the tokens rounded up), so that A is read once per quad and not once per token.
template <int MT>
__device__ __forceinline__ void gb_sum_flat_body(const GbItem* __restrict__ it, const int blk, const int nblk) {
    __shared__ float u[16 * GS_TROW];
    const int M = it->M, K = it->K, r = it->r;
    const auto part = as_global(it->part), upart = as_global(it->upart);
    const auto A = as_global(it->A);
    const auto dX = as_global(it->dX);
    if (r > 0) {
        for (int o = threadIdx.x; o < 16 * GS_TROW; o += blockDim.x) {
            float v = 0.0f;
            for (int p = 0; p < it->nup; ++p) v += upart[(size_t)p * 16 * GS_TROW + o];
            u[o] = v * it->s;
        }
        __syncthreads();
    }
    const size_t slot_stride = (size_t)M * GB_CHUNK;
    const int quads = K / 4;                                        // K is a multiple of 256
    for (int o = blk * blockDim.x + threadIdx.x; o < quads; o += nblk * blockDim.x) {
        const int k = 4 * o, chunk = k / GB_CHUNK, kc = k % GB_CHUNK;
        const auto src = part + (size_t)it->slot0[chunk] * slot_stride + kc;
        float4 v[MT];
#pragma unroll
        for (int m = 0; m < MT; ++m) v[m] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        for (int q = 0; q < it->nslots[chunk]; ++q) {               // fixed order
#pragma unroll
            for (int m = 0; m < MT; ++m)
                if (m < M) {
                    const float4 t = gload_f4(src + (size_t)q * slot_stride + (size_t)m * GB_CHUNK);
                    v[m].x += t.x; v[m].y += t.y; v[m].z += t.z; v[m].w += t.w;
                }
        }
        for (int j = 0; j < r; ++j) {
            const uint2 a = gload_u2(A + (size_t)j * K + k);
            const float a0 = bf16_bits_to_float(a.x & 0xffffu), a1 = bf16_bits_to_float(a.x >> 16);
            const float a2 = bf16_bits_to_float(a.y & 0xffffu), a3 = bf16_bits_to_float(a.y >> 16);
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                const float uj = u[m * GS_TROW + j];
                v[m].x += uj * a0; v[m].y += uj * a1; v[m].z += uj * a2; v[m].w += uj * a3;
            }
        }
#pragma unroll
        for (int m = 0; m < MT; ++m)
            if (m < M) gstore_u2(dX + (size_t)m * K + k, make_uint2(pack_bf16x2(v[m].x, v[m].y), pack_bf16x2(v[m].z, v[m].w)));
    }
}

// Many slots per chunk (one matrix spread over all workgroups): a workgroup of 256 threads takes tiles of 16 quads
// (64 consecutive columns of one token): thread (ql, sl) adds the slots sl, sl + 16, ... and the ranks sl, sl + 16
// of quad ql; the 16 partial sums of a quad meet in LDS and are added in order (a fixed assignment: the result does
// not depend on timing).
__device__ __forceinline__ void gb_sum_body(const GbItem* __restrict__ it, const int blk, const int nblk) {
    __shared__ float u[GS_TROW];
    __shared__ float4 red[16][16];
    const int M = it->M, K = it->K, r = it->r;
    const auto part = as_global(it->part), upart = as_global(it->upart);
    const auto A = as_global(it->A);
    const auto dX = as_global(it->dX);
    const int ql = threadIdx.x & 15, sl = threadIdx.x >> 4;
    const size_t slot_stride = (size_t)M * GB_CHUNK;
    const int tiles = M * K / 64;                                   // K is a multiple of 256
    for (int tile = blk; tile < tiles; tile += nblk) {              // uniform
        const int m = (64 * tile) / K, k = (64 * tile) % K + 4 * ql, chunk = k / GB_CHUNK, kc = k % GB_CHUNK;
        if (r > 0 && threadIdx.x < GS_TROW) {
            float v = 0.0f;
            for (int p = 0; p < it->nup; ++p) v += upart[(size_t)p * 16 * GS_TROW + m * GS_TROW + threadIdx.x];
            u[threadIdx.x] = v * it->s;
        }
        __syncthreads();
        const auto src = part + (size_t)it->slot0[chunk] * slot_stride + (size_t)m * GB_CHUNK + kc;
        const int ns = it->nslots[chunk];
        float4 v = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        for (int q = sl; q < ns; q += 16) {
            const float4 t = gload_f4(src + (size_t)q * slot_stride);
            v.x += t.x; v.y += t.y; v.z += t.z; v.w += t.w;
        }
        for (int j = sl; j < r; j += 16) {
            const uint2 a = gload_u2(A + (size_t)j * K + k);
            const float uj = u[j];
            v.x += uj * bf16_bits_to_float(a.x & 0xffffu); v.y += uj * bf16_bits_to_float(a.x >> 16);
            v.z += uj * bf16_bits_to_float(a.y & 0xffffu); v.w += uj * bf16_bits_to_float(a.y >> 16);
        }
        red[sl][ql] = v;
        __syncthreads();
        if (sl == 0) {
            float4 t = red[0][ql];
#pragma unroll
            for (int w = 1; w < 16; ++w) { const float4 q = red[w][ql]; t.x += q.x; t.y += q.y; t.z += q.z; t.w += q.w; }
            gstore_u2(dX + (size_t)m * K + k, make_uint2(pack_bf16x2(t.x, t.y), pack_bf16x2(t.z, t.w)));
        }
    }
}

__global__ __launch_bounds__(GB_PRE_WAVES * 64) void gemv_stream_bwd_pre_kernel(const GbPre* __restrict__ items, int P) {
    const GbPre it = items[blockIdx.x / P];                       // a copy: the body's stores cannot alias it
    gb_pre_body(it, blockIdx.x % P, P);
}
__global__ __launch_bounds__(256) void gemv_stream_bwd_sum_kernel(const GbItem* __restrict__ items, int per_item_blocks) {
    gb_sum_body(items + blockIdx.x / per_item_blocks, blockIdx.x % per_item_blocks, per_item_blocks);
}
template <int MT>
__global__ __launch_bounds__(256) void gemv_stream_bwd_sum_flat_kernel(const GbItem* __restrict__ items, int per_item_blocks) {
    gb_sum_flat_body<MT>(items + blockIdx.x / per_item_blocks, blockIdx.x % per_item_blocks, per_item_blocks);
}

// ---- one matrix: the small tables travel as kernel arguments and the set-up kernel writes them (and the units)
// to the workspace, so that the call copies nothing from the host and may be captured.
struct GbSingle {
    GbSeg segs[GB_MAXSEG];
    GbPre pre;
    GbItem item;
    int nseg, nwg, P;
    int per, f4, nstrips;    // units per chunk, first 4-bit strip, strips
    int cls_end[kGvMaxClasses], cls_bits_cb[kGvMaxClasses];
    int wg_first[GB_MAXWG + 1], wg_slot0[GB_MAXWG + 1];
    GbSeg* d_segs; GsUnit* d_units; int* d_wg_first; int* d_wg_slot0; GbItem* d_item;
};
__global__ __launch_bounds__(GB_PRE_WAVES * 64) void gemv_stream_bwd_pre_single_kernel(const GbSingle a) {
    gb_pre_body(a.pre, blockIdx.x, a.P);
    // the descriptors and the unit table, spread over the workgroups
    const int tid = blockIdx.x * blockDim.x + threadIdx.x, nthreads = gridDim.x * blockDim.x;
    // (the two tables are read straight from the kernel-argument segment: indexing the by-value struct with a
    // run-time index would copy it to private memory first)
    const __attribute__((address_space(4))) uint8_t* ka = (const __attribute__((address_space(4))) uint8_t*)__builtin_amdgcn_kernarg_segment_ptr();
    const gs_cint_t k_first = reinterpret_cast<gs_cint_t>(ka + offsetof(GbSingle, wg_first));
    const gs_cint_t k_slot0 = reinterpret_cast<gs_cint_t>(ka + offsetof(GbSingle, wg_slot0));
    for (int b = tid; b <= a.nwg; b += nthreads) { a.d_wg_first[b] = k_first[b]; a.d_wg_slot0[b] = k_slot0[b]; }
    for (int o = tid; o < a.nseg * a.nstrips; o += nthreads) {
        const int c = o / a.nstrips, sidx = o % a.nstrips;
        int cls = a.cls_bits_cb[0];
#pragma unroll
        for (int q = 0; q + 1 < kGvMaxClasses; ++q) cls = sidx >= a.cls_end[q] ? a.cls_bits_cb[q + 1] : cls;
        const int bits = cls & 0xff, tab = cls >> 8;
        GsUnit* dst = a.d_units + (size_t)c * a.per + (sidx < a.f4 ? sidx : a.f4 + 2 * (sidx - a.f4));
        if (bits == 4) {
            dst[0] = GsUnit{(uint32_t)sidx * 128u, (uint32_t)c, gs_unit_flags(4, 0, 0, tab, o), 0u};
            dst[1] = GsUnit{(uint32_t)sidx * 128u, (uint32_t)c, gs_unit_flags(4, 1, 1, tab, o), 0u};
        } else {
            dst[0] = GsUnit{(uint32_t)sidx * 128u, (uint32_t)c, gs_unit_flags(bits, 0, 1, tab, o), 0u};
        }
    }
    if (tid == 0) {
#pragma unroll
        for (int c = 0; c < GB_MAXSEG; ++c)
            if (c < a.nseg) a.d_segs[c] = a.segs[c];
        *a.d_item = a.item;
    }
}

// =============================================================================================== host side
bool gemv_stream_bwd_supported(const lowra_layout& L, int M, int r) {
    return M >= 1 && M <= 16 && gs_layout_supported(L) && r >= 0 && r <= GS_TROW;
}

static int gb_nchunks(const lowra_layout& L) { return gs_nchunks(L, GB_W); }
int gemv_stream_bwd_nchunks(const lowra_layout& L) { return gb_nchunks(L); }

static size_t gb_lds_bytes(const GsTabs& t) { return (size_t)t.nslot * GS_TABB + (size_t)GB_W * GB_WAVEB; }
static hipError_t gb_attr() {
    static hipError_t a = gs_prepare_kernel(reinterpret_cast<const void*>(gemv_stream_bwd_kernel));
    return a;
}

// the K-chunks of one matrix
static int gb_make_segs(const lowra_layout& L, const uint8_t* packed, const float* absmax, const uint16_t* dys, GbSeg* out) {
    const int nblk_all = L.K / 256, nch = gb_nchunks(L);
    for (int c = 0; c < nch; ++c) {
        GbSeg& g = out[c];
        g = GbSeg{};
        g.rows = L.d_gv_rows; g.packed = packed; g.absmax = absmax; g.dys = dys; g.G = L.G;
        g.kblk0 = c * GB_W; g.nblk = std::min(GB_W, nblk_all - c * GB_W);
    }
    return nch;
}

static size_t gb_dys_bytes(const lowra_layout& L) { return gs_align((size_t)L.gv_nstrips * 512); }
static int gb_pre_blocks(const lowra_layout& L) { return std::max(1, std::min(GB_MAXPRE, L.gv_nstrips / (GB_PRE_WAVES * GB_PRE_U))); }
static size_t gb_upart_bytes(int r) { return r > 0 ? (size_t)GB_MAXPRE * 16 * GS_TROW * sizeof(float) : 0; }
static size_t gb_matrix_bytes(const lowra_layout& L) { return L.packed_bytes + (size_t)L.N * L.G * (L.scale_bf16 ? 2 : 4); }

// Workgroups of a single call.  A workgroup streams about 10 GB/s, and every workgroup writes (and the last kernel
// reads back, at some 4 TB/s) M x 2048 floats per run: the sum of the two times is least near
// sqrt(matrix bytes / (40 M)) workgroups.
static int gb_single_nwg(const lowra_layout& L, int M) {
    const int units = gb_nchunks(L) * gs_units_per_seg(L);
    const int best = (int)std::sqrt((double)gb_matrix_bytes(L) / (40.0 * M));
    return std::max(1, std::min(std::min(std::min(gs_compute_units(), GB_MAXWG), std::max(8, best)), units / 2));
}

// workspace of a single call: [descriptors][units][dY in strip order][partial sums of u][partial slots]
constexpr size_t GB_DESC_BYTES = 4096, GB_DESC_ITEM = 512, GB_DESC_FIRST = 1024, GB_DESC_SLOT0 = 2560;
static_assert(GB_MAXSEG * sizeof(GbSeg) <= GB_DESC_ITEM && GB_DESC_ITEM + sizeof(GbItem) <= GB_DESC_FIRST &&
              GB_DESC_FIRST + (GB_MAXWG + 1) * sizeof(int) <= GB_DESC_SLOT0 && GB_DESC_SLOT0 + (GB_MAXWG + 1) * sizeof(int) <= GB_DESC_BYTES, "descriptor area");
static_assert(sizeof(GbSingle) <= 4096, "kernel arguments");
static size_t gb_units_bytes(const lowra_layout& L) { return gs_align((size_t)gb_nchunks(L) * gs_units_per_seg(L) * sizeof(GsUnit)); }
size_t gemv_stream_bwd_workspace_bytes(const lowra_layout& L, int M, int r) {
    const size_t slots = (size_t)gb_single_nwg(L, M) + 2 * (size_t)gb_nchunks(L);
    return GB_DESC_BYTES + gb_units_bytes(L) + gb_dys_bytes(L) + gb_upart_bytes(r) + gs_align(slots * M * GB_CHUNK * sizeof(float));
}

// Runs of a unit list: unit u is in chunk u / per; units at or past f4 within a chunk are 4-bit halves.  Numbers the
// runs of every workgroup (wg_slot0) and of every chunk (slot0, nslots).  Returns the number of runs.
static int gb_number_runs(int nwg, const int* wg_first, int per, int f4, int nseg, int* wg_slot0, int* slot0, int* nslots) {
    for (int c = 0; c < nseg; ++c) { slot0[c] = 0; nslots[c] = 0; }
    int slot = 0;
    for (int b = 0; b < nwg; ++b) {
        wg_slot0[b] = slot;
        for (int u = wg_first[b]; u < wg_first[b + 1];) {
            const int c = u / per, local = u % per;
            const int run_end = local < f4 ? c * per + f4 : (c + 1) * per;
            if (nslots[c]++ == 0) slot0[c] = slot;
            ++slot;
            u = std::min(run_end, wg_first[b + 1]);
        }
    }
    wg_slot0[nwg] = slot;
    return slot;
}

hipError_t launch_gemv_stream_bwd(const lowra_layout& L, const LinearArgs& a, hipStream_t st) {
    hipError_t e = gb_attr();
    if (e != hipSuccess) return e;
    const GsTabs tabs = gs_tabs(L.cb_bits, L.scale_bf16);
    uint8_t* ws = static_cast<uint8_t*>(a.workspace);
    GbSingle sg{};
    sg.d_segs = reinterpret_cast<GbSeg*>(ws);
    sg.d_item = reinterpret_cast<GbItem*>(ws + GB_DESC_ITEM);
    sg.d_wg_first = reinterpret_cast<int*>(ws + GB_DESC_FIRST);
    sg.d_wg_slot0 = reinterpret_cast<int*>(ws + GB_DESC_SLOT0);
    sg.d_units = reinterpret_cast<GsUnit*>(ws + GB_DESC_BYTES);
    uint16_t* dys = reinterpret_cast<uint16_t*>(ws + GB_DESC_BYTES + gb_units_bytes(L));
    float* upart = reinterpret_cast<float*>(ws + GB_DESC_BYTES + gb_units_bytes(L) + gb_dys_bytes(L));
    float* part = reinterpret_cast<float*>(ws + GB_DESC_BYTES + gb_units_bytes(L) + gb_dys_bytes(L) + gb_upart_bytes(a.r));
    sg.nseg = gb_make_segs(L, a.packed, a.absmax, dys, sg.segs);
    sg.nwg = gb_single_nwg(L, a.M);
    sg.P = gb_pre_blocks(L);
    sg.per = gs_units_per_seg(L); sg.f4 = gs_first4(L); sg.nstrips = L.gv_nstrips;
    for (int q = 0; q < kGvMaxClasses; ++q) { sg.cls_end[q] = L.gv_cls_end[q]; sg.cls_bits_cb[q] = L.gv_cls_bits_cb[q]; }
    const int total = sg.nseg * sg.per;
    for (int b = 0; b <= sg.nwg; ++b) {
        int u = (int)((long long)b * total / sg.nwg);
        const int local = u % sg.per;
        if (b < sg.nwg && local > sg.f4 && ((local - sg.f4) & 1)) ++u;      // never between the two units of a 4-bit strip
        sg.wg_first[b] = u;
    }
    sg.pre = GbPre{L.d_gv_rows, a.act, a.B, dys, upart, L.N, a.M, a.r, L.gv_nstrips};
    sg.item = GbItem{};
    sg.item.part = part; sg.item.upart = upart; sg.item.A = a.A; sg.item.dX = a.out;
    sg.item.M = a.M; sg.item.K = L.K; sg.item.r = a.r; sg.item.nup = sg.P; sg.item.s = a.s;
    gb_number_runs(sg.nwg, sg.wg_first, sg.per, sg.f4, sg.nseg, sg.wg_slot0, sg.item.slot0, sg.item.nslots);
    gemv_stream_bwd_pre_single_kernel<<<dim3(sg.P), dim3(GB_PRE_WAVES * 64), 0, st>>>(sg);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    gemv_stream_bwd_kernel<<<dim3(sg.nwg), dim3(GB_THREADS), gb_lds_bytes(tabs), st>>>(sg.d_segs, sg.d_units, sg.d_wg_first, sg.d_wg_slot0,
                                                                                       a.mappings, tabs, part, a.M);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    const int blocks = std::max(1, std::min(2 * gs_compute_units(), a.M * L.K / 64));
    gemv_stream_bwd_sum_kernel<<<dim3(blocks), dim3(256), 0, st>>>(sg.d_item, blocks);
    return hipGetLastError();
}

// ---- a batch: descriptors built once on the host
// per matrix: [dY in strip order][partial sums of u]; the partial slots of the whole batch follow the matrices' pieces
size_t gemv_stream_bwd_batch_item_ws(const lowra_layout& L, int r) { return gb_dys_bytes(L) + gb_upart_bytes(r); }
// upper bound of the batch's partial slots: one per workgroup plus two per chunk
size_t gemv_stream_bwd_batch_slots_ws(int nchunks_total, int M) {
    return gs_align(((size_t)GB_MAXWG + 2 * (size_t)nchunks_total) * M * GB_CHUNK * sizeof(float));
}

void gemv_stream_bwd_batch_free(GbBatch& b) {
    (void)hipFree(b.d_segs); (void)hipFree(b.d_wg_first); (void)hipFree(b.d_wg_slot0); (void)hipFree(b.d_units);
    (void)hipFree(b.d_pre); (void)hipFree(b.d_items);
    b = GbBatch{};
}

hipError_t gemv_stream_bwd_batch_build(const std::vector<GbBatchItem>& items, const float* mappings, int M, int r, float s,
                                       float* part, GbBatch& b) {
    if (items.empty()) return hipSuccess;
    std::vector<GbSeg> segs;
    std::vector<GsUnit> unitv;
    std::vector<double> unit_cost;                                   // bytes of codes, scales and dY per unit, plus a constant
    std::vector<char> pair_second;                                   // the unit is the second half of a 4-bit strip
    std::vector<GbPre> pres;
    std::vector<GbItem> sums;
    constexpr double kUnitFixedCost = 16384.0;
    int max_p = 1;
    for (const GbBatchItem& it : items) max_p = std::max(max_p, gb_pre_blocks(*it.L));
    // the set-up workgroups of all matrices should be resident together (two of 16 wavefronts per compute unit): a
    // wavefront's time is a chain of round trips per pass, and a second round of workgroups repeats it
    max_p = std::max(1, std::min(max_p, 2 * gs_compute_units() / (int)std::max<size_t>(items.size(), 1)));
    int strip_seq = 0;
    for (const GbBatchItem& it : items) {
        const lowra_layout& L = *it.L;
        uint16_t* dys = reinterpret_cast<uint16_t*>(it.ws);
        float* upart = reinterpret_cast<float*>(it.ws + gb_dys_bytes(L));
        GbSeg tmp[GB_MAXSEG];
        const int nch = gb_make_segs(L, it.packed, it.absmax, dys, tmp);
        for (int c = 0; c < nch; ++c) {
            segs.push_back(tmp[c]);
            const uint32_t seg_index = (uint32_t)segs.size() - 1u;
            for (int sidx = 0; sidx < L.gv_nstrips; ++sidx) {
                const int cls = gs_strip_class(L, sidx), bw = cls & 0xff, tab = cls >> 8;
                const double cost = 16.0 * tmp[c].nblk * (bw == 1 ? 32.0 + 16.0 : 64.0 + 16.0) + kUnitFixedCost;
                unit_cost.push_back(cost); pair_second.push_back(0);
                unitv.push_back(GsUnit{(uint32_t)sidx * 128u, seg_index, gs_unit_flags(bw, 0, bw != 4, tab, strip_seq), 0u});
                if (bw == 4) {
                    unit_cost.push_back(cost); pair_second.push_back(1);
                    unitv.push_back(GsUnit{(uint32_t)sidx * 128u, seg_index, gs_unit_flags(4, 1, 1, tab, strip_seq), 0u});
                }
                ++strip_seq;
            }
        }
        GbPre pre{L.d_gv_rows, it.dY, it.B, dys, upart, L.N, M, r, L.gv_nstrips};
        pres.push_back(pre);
        GbItem sum{};
        sum.part = part; sum.upart = upart; sum.A = it.A; sum.dX = it.dX;
        sum.M = M; sum.K = L.K; sum.r = r; sum.nup = max_p; sum.s = s;   // every matrix runs max_p set-up workgroups (idle ones write zero sums)
        sums.push_back(sum);
    }
    // contiguous unit ranges of (nearly) equal cost, never between the two units of a 4-bit strip
    const int units = (int)unitv.size();
    const int nwg = std::min(std::min(gs_compute_units(), GB_MAXWG), units);
    double total = 0.0;
    for (double c : unit_cost) total += c;
    std::vector<int> wg_first((size_t)nwg + 1, units), wg_slot0((size_t)nwg + 1, 0);
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
    }
    // number the runs: a new one at every workgroup start, chunk start and change of the column mapping
    std::vector<int> seg_slot0(segs.size(), 0), seg_nslots(segs.size(), 0);
    int slot = 0;
    for (int w = 0; w < nwg; ++w) {
        wg_slot0[(size_t)w] = slot;
        for (int u = wg_first[(size_t)w]; u < wg_first[(size_t)w + 1]; ++u) {
            const bool fresh = u == wg_first[(size_t)w] || unitv[(size_t)u].seg != unitv[(size_t)u - 1].seg ||
                               ((unitv[(size_t)u].flags & 15u) == 4u) != ((unitv[(size_t)u - 1].flags & 15u) == 4u);
            if (fresh) {
                const size_t sg = unitv[(size_t)u].seg;
                if (seg_nslots[sg]++ == 0) seg_slot0[sg] = slot;
                ++slot;
            }
        }
    }
    wg_slot0[(size_t)nwg] = slot;
    {
        size_t sg = 0;
        for (size_t q = 0; q < items.size(); ++q)
            for (int c = 0; c < gb_nchunks(*items[q].L); ++c, ++sg) { sums[q].slot0[c] = seg_slot0[sg]; sums[q].nslots[c] = seg_nslots[sg]; }
    }
    b.nwg = nwg; b.nitems = (int)items.size(); b.P = max_p; b.M = M; b.mappings = mappings; b.part = part; b.nslots = slot;
    b.max_quads = 0; b.max_nslots = 0;
    for (const GbItem& q : sums) b.max_quads = std::max(b.max_quads, q.M * q.K / 4);
    for (int q : seg_nslots) b.max_nslots = std::max(b.max_nslots, q);
    b.cb_bits = items[0].L->cb_bits;
    b.scale_bf16 = items[0].L->scale_bf16;
    hipError_t e;
    if ((e = gs_to_device(segs, reinterpret_cast<GbSeg**>(&b.d_segs))) != hipSuccess) return e;
    if ((e = gs_to_device(wg_first, &b.d_wg_first)) != hipSuccess) return e;
    if ((e = gs_to_device(wg_slot0, &b.d_wg_slot0)) != hipSuccess) return e;
    if ((e = gs_to_device(unitv, reinterpret_cast<GsUnit**>(&b.d_units))) != hipSuccess) return e;
    if ((e = gs_to_device(pres, reinterpret_cast<GbPre**>(&b.d_pre))) != hipSuccess) return e;
    if ((e = gs_to_device(sums, reinterpret_cast<GbItem**>(&b.d_items))) != hipSuccess) return e;
    return gb_attr();
}

hipError_t gemv_stream_bwd_batch_run(const GbBatch& b, hipStream_t st) {
    if (b.nwg == 0) return hipSuccess;
    hipError_t e;
    gemv_stream_bwd_pre_kernel<<<dim3(b.nitems * b.P), dim3(GB_PRE_WAVES * 64), 0, st>>>(static_cast<const GbPre*>(b.d_pre), b.P);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    const GsTabs tabs = gs_tabs(b.cb_bits, b.scale_bf16);
    {
        KernelTimer timer(st);
        gemv_stream_bwd_kernel<<<dim3(b.nwg), dim3(GB_THREADS), gb_lds_bytes(tabs), st>>>(static_cast<const GbSeg*>(b.d_segs), static_cast<const GsUnit*>(b.d_units),
                                                                                          b.d_wg_first, b.d_wg_slot0, b.mappings, tabs, b.part, b.M);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    if (b.max_nslots <= 8) {
        const int blocks = std::max(1, std::min(64, b.max_quads / b.M / 256));      // quads of columns per matrix
        const GbItem* items = static_cast<const GbItem*>(b.d_items);
        if (b.M == 1) gemv_stream_bwd_sum_flat_kernel<1><<<dim3(b.nitems * blocks), dim3(256), 0, st>>>(items, blocks);
        else if (b.M <= 4) gemv_stream_bwd_sum_flat_kernel<4><<<dim3(b.nitems * blocks), dim3(256), 0, st>>>(items, blocks);
        else gemv_stream_bwd_sum_flat_kernel<16><<<dim3(b.nitems * blocks), dim3(256), 0, st>>>(items, blocks);
    } else {
        const int blocks = std::max(1, std::min(64, b.max_quads / 16));
        gemv_stream_bwd_sum_kernel<<<dim3(b.nitems * blocks), dim3(256), 0, st>>>(static_cast<const GbItem*>(b.d_items), blocks);
    }
    return hipGetLastError();
}

}  // namespace lowra
