// Streaming small-token forward (M <= 16):  y = x What^T + (s x A^T) B^T over one or many matrices,
// as ONE persistent launch that keeps the memory system full.
//
// Bandwidth-bound: per weight the method moves bits/8 + 1/16 bytes (codes + fp32 group scale).  A
// compute unit has to keep tens of KB of loads in flight all the time to cover the memory latency, and at
// 8 TB/s it has about 2000 cycles per 20 KB strip for all 16 wavefronts together: every instruction per
// unit counts.
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
//    one s_waitcnt vmcnt with a constant count.
//  * Strips come in the layout's class-sorted order: all 16 rows of a strip have one width and one
//    table, so a wavefront runs one instruction stream per strip (uniform branch on the width).
//  * Lane (i, kg) receives 16 contiguous bytes of channel i; v_mfma_f32_16x16x32_bf16 step (g, h) contracts
//    k = 64 g + 32 h + 8 kg + e, so the four lanes of a channel first trade pieces (4 x 4 dword transpose,
//    v_permlane32/16_swap) and all lanes of an MFMA step then sit in ONE group: the group scale multiplies
//    the fp32 result of the group's steps instead of every weight (the same sum in another order).
//  * Decode (App. A.2's table lookup): ONE BYTE of codes (8, 4 or 2 of them) indexes a table of the
//    unscaled bf16 levels of all its codes (16, 8 or 4 bytes), 256 entries of 64 bytes holding 4, 8 or 16
//    copies so that neighbouring lanes read different banks: one shift, one and-or and one LDS read per byte.
//  * The rank-r term rides as one more MFMA step of wavefront 0: [t] against the strip's B rows, which
//    arrive through a ring like the codes; t = s x A^T comes from a small kernel before.
//  * The 16 partial results of a strip meet in LDS (two alternating slots, one barrier per strip); one
//    wavefront, a different one per strip, adds them in a fixed order and stores.  Long rows (K > 4096)
//    are cut into chunks whose fp32 partial outputs a small kernel adds afterwards.
//
// Used when every 16-row strip can have one class (at most 4 (width, table) classes and 3 tables per
// matrix), K is a multiple of 256 and the rank is a multiple of 8 up to 32; other shapes take the
// general kernel.
#include "gemv_stream.h"

#ifndef GS_EXP
#define GS_EXP 0      // measurement variants (bit flags), 0 in the product: 1 no stores, 2 no barrier / reduction, 4 no decode, 8 no transfers of codes and scales
#endif
#ifndef GS_DEPTH
#define GS_DEPTH 3
#endif

namespace lowra {

constexpr int GS_D = GS_DEPTH;           // units whose codes are in flight per wavefront
constexpr int GS_REDB = GS_W * 64 * 16;  // one reduction slot: a float4 per lane and wavefront
constexpr int GS_SLOTB = 1024 + 256;     // ring slot: 16 B of codes per lane, then 4 scales per channel
constexpr int GS_NREC = GS_D + 1;        // record slots per wavefront: written 2 GS_D units ahead, read GS_D ahead
constexpr int GS_WAVEB = GS_D * GS_SLOTB + GS_NREC * GS_RECB;   // per wavefront: ring, record ring
constexpr int GS_LORAB = GS_D * 1024;    // wavefront 0: ring of B fragments, 16 B per lane

// One (matrix, K-chunk): everything a workgroup needs to stream its strips.
struct GsSeg {
    const GvRow* rows;       // [nstrips * 16] class-sorted row records
    const uint8_t* packed;
    const float* absmax;
    const uint16_t* x;       // [M][K] bf16
    const uint16_t* B;       // [N][r] bf16; null when this chunk carries no rank-r term
    const uint16_t* t;       // s x A^T as bf16 [16][GS_TROW], zero past M and past r
    void* out;               // y [M][N] bf16, or this chunk's fp32 partial [M][N]
    int N, K, G, M;
    int nstrips;
    int first4;              // first strip of the 4-bit classes (nstrips when there is none): those strips are two units each
    int kblk0, nblk;         // first 256-column block of the chunk, and how many (1..16)
    int out_fp32;
    int r;
    int cls_end[kGvMaxClasses];
    int cls_bits_cb[kGvMaxClasses];   // width | table index << 8 of class c
    int first_unit;          // index of this segment's first unit in the launch's unit list
    int seq0;                // sequence number of its first strip in the launch (picks the reducing wavefront and the reduction slot)
    int nunits;              // nstrips + (nstrips - first4)
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

// The descriptors are read-only for the whole launch: reading them through the constant address space lets
// the compiler use scalar loads, so a segment's fields live in scalar registers.
typedef const __attribute__((address_space(4))) GsSeg* gs_cseg_t;

// The arithmetic of one unit: decode my 16 bytes of codes (cq) and contract them with my activations.
// ONE: a single token, so only row 0 of the MFMA result is ever used.
template <bool ONE, int bits>
__device__ __forceinline__ void gs_unit(const uint8_t* __restrict__ smem, const int half, const uint32_t toff,
                                        const uint4 cq, const float4 sq, const bf16x8_t (&xr)[8], const int lane, floatx4_t& tot) {
    const int kg = lane >> 4;
    const float a4[4] = {sq.x, sq.y, sq.z, sq.w};
    if (GS_EXP & 4) {
        tot[0] += a4[0] * __builtin_bit_cast(float, cq.x) + a4[1] * __builtin_bit_cast(float, cq.y);
        return;
    }
    if constexpr (bits == 2) {
        // I hold group kg of my channel: codes 16 d .. 16 d + 15 in dword d.  Piece (h, kg') = 16 bits.
        const uint32_t tb = 8u * (lane & 7) + toff;
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
                const uint2 d0 = *reinterpret_cast<const uint2*>(smem + gs_entry(z[g], 2 * h, tb));       // codes 0..3 of my 8
                const uint2 d1 = *reinterpret_cast<const uint2*>(smem + gs_entry(z[g], 2 * h + 1, tb));   // codes 4..7
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xr[2 * g + h], __builtin_bit_cast(bf16x8_t, make_uint4(d0.x, d0.y, d1.x, d1.y)), acc, 0, 0, 0);
            }
            tot[0] += a4[g] * acc[0];
            if (!ONE) { tot[1] += a4[g] * acc[1]; tot[2] += a4[g] * acc[2]; tot[3] += a4[g] * acc[3]; }
        }
    } else if constexpr (bits == 1) {
        // I hold the pair of groups (kg & ~1, kg | 1) of my channel: mine is the low or the high 8 bytes
        // (bitwise choice, so that it cannot become an indexed access).  Piece (h, kg') = 1 byte.
        const uint32_t tb = 16u * (lane & 3) + toff;
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
                const uint4 d = *reinterpret_cast<const uint4*>(smem + gs_entry(z[g], h, tb));
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xr[2 * g + h], __builtin_bit_cast(bf16x8_t, d), acc, 0, 0, 0);
            }
            tot[0] += a4[g] * acc[0];
            if (!ONE) { tot[1] += a4[g] * acc[1]; tot[2] += a4[g] * acc[2]; tot[3] += a4[g] * acc[3]; }
        }
    } else {
        // half `half` of group kg of my channel: dword d = its codes 8 d .. 8 d + 7, the piece of lane d
        const uint32_t tb = 4u * (lane & 15) + toff;
        uint32_t z[4] = {cq.x, cq.y, cq.z, cq.w};
        gs_transpose4(z);
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            uint32_t d[4];
#pragma unroll
            for (int p = 0; p < 4; ++p) d[p] = *reinterpret_cast<const uint32_t*>(smem + gs_entry(z[g], p, tb));   // byte p: codes 2 p, 2 p + 1
            const bf16x8_t wv = __builtin_bit_cast(bf16x8_t, make_uint4(d[0], d[1], d[2], d[3]));
            floatx4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
            if (half == 0) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xr[2 * g], wv, acc, 0, 0, 0);
            else acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xr[2 * g + 1], wv, acc, 0, 0, 0);
            tot[0] += a4[g] * acc[0];
            if (!ONE) { tot[1] += a4[g] * acc[1]; tot[2] += a4[g] * acc[2]; tot[3] += a4[g] * acc[3]; }
        }
    }
}

template <bool ONE, bool SB16>
__global__ __launch_bounds__(GS_THREADS) void gemv_stream_kernel(const GsSeg* __restrict__ segs_g, const GsUnit* __restrict__ units_g,
                                                                 const int* __restrict__ wg_first_g, const float* __restrict__ mappings,
                                                                 const GsTabs tabs) {
    // the descriptors are read-only for the whole launch: read through the constant address space (scalar loads)
    const gs_cseg_t segs = reinterpret_cast<gs_cseg_t>(reinterpret_cast<uintptr_t>(segs_g));
    const gs_cunit_t units = reinterpret_cast<gs_cunit_t>(reinterpret_cast<uintptr_t>(units_g));
    const gs_cint_t wg_first = reinterpret_cast<gs_cint_t>(reinterpret_cast<uintptr_t>(wg_first_g));
    extern __shared__ __align__(16) uint8_t gs_smem[];
    // LDS: [tables: nslot x GS_TABB] [reduction slots: 2 x GS_REDB] [per wavefront: GS_WAVEB] [wavefront 0: GS_LORAB]
    const int RED0 = tabs.nslot * GS_TABB, WV0 = RED0 + 2 * GS_REDB, LORA0 = WV0 + GS_W * GS_WAVEB;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int i = lane & 15, kg = lane >> 4;
    const uint32_t smem_lds = (uint32_t)(uintptr_t)(lptr_t)gs_smem;
    const int RING0 = WV0 + wave * GS_WAVEB, REC0 = RING0 + GS_D * GS_SLOTB;

    gs_fill_tables(gs_smem, mappings, tabs);
    // the record slots start as a valid record (offset 0, no channel): the first requests read them before any has landed
    for (int o = lane; o < GS_NREC * GS_RECB / 8; o += 64)
        *reinterpret_cast<uint2*>(gs_smem + REC0 + 8 * o) = make_uint2(0u, 0xffffffffu);
    __syncthreads();

    const int u0 = wg_first[blockIdx.x], n = wg_first[blockIdx.x + 1] - u0;
    if (n <= 0) return;                                             // whole workgroup

    // ---- three stages walk the same units: records (2 GS_D ahead), codes and scales (GS_D ahead), arithmetic.
    // A stage past the end of the range stays on the last unit: same transfers, no effect.
    GS_CUR_DECL(R); GS_CUR_DECL(I); GS_CUR_DECL(C);
    {
        const int seg0 = (int)units[u0].seg, lu0 = u0 - segs[seg0].first_unit;
        GS_CUR_SEEK(R, seg0, lu0); GS_CUR_SEEK(I, seg0, lu0); GS_CUR_SEEK(C, seg0, lu0);
        leftR = leftI = leftC = n - 1;
        (void)tabR; (void)tabI; (void)stripI;
    }
    // what a stage keeps of its segment: plain local variables in scalar registers
    const uint8_t* rowsR = reinterpret_cast<const uint8_t*>(segs[segR].rows);
    const uint8_t* iPacked; const uint8_t* iScaleBase; const uint16_t* iB;
    int iG4, iKb32, iR;
    const uint16_t* mX; const uint16_t* mB; const uint16_t* mT; void* mOut;
    int mN, mK, mM, mKblk0, mNblk, mOutFp32, mSeq0;
#define GS_SEG_ISSUE(p)                                                                                           \
    do {                                                                                                          \
        iPacked = (p)->packed; iB = (p)->B; iR = (p)->r; iG4 = (SB16 ? 2 : 4) * (p)->G;                       \
        iKb32 = 32 * ((p)->kblk0 + min(wave, (p)->nblk - 1)); /* past the chunk's end: the last block again (unused) */ \
        iScaleBase = reinterpret_cast<const uint8_t*>((p)->absmax) + (size_t)(iKb32 >> (SB16 ? 2 : 1));           \
    } while (0)
#define GS_SEG_MATH(p)                                                                                            \
    do {                                                                                                          \
        mX = (p)->x; mB = (p)->B; mT = (p)->t; mOut = (p)->out; mN = (p)->N; mK = (p)->K; mM = (p)->M;            \
        mKblk0 = (p)->kblk0; mNblk = (p)->nblk; mOutFp32 = (p)->out_fp32; mSeq0 = (p)->seq0;                      \
    } while (0)
    GS_SEG_ISSUE(segs + segI);
    GS_SEG_MATH(segs + segC);

    // channel of my row (lane i) in the strips of the last GS_D requests: read with the records when a unit's codes are
    // asked for, used GS_D passes later by the wavefront that adds the strip up and stores it
    static_assert(GS_D == 3, "the channel numbers travel through a three-deep register queue");
    int nfifo0 = -1, nfifo1 = -1, nfifo2 = -1;
    bf16x8_t xr[8];
    bf16x8_t tf = bf16x8_t{0, 0, 0, 0, 0, 0, 0, 0};                 // wavefront 0: t[token i][8 kg ..]
    floatx4_t tot = {0.0f, 0.0f, 0.0f, 0.0f};

    // my activations: x[token i][256 (kblk0 + wave) + 64 g + 32 h + 8 kg ..], zero past M or past the chunk; wavefront 0:
    // its fragment of t.  These loads are the compiler's own: they are back before the next transfers are counted.
#define GS_LOAD_X()                                                                                               \
    do {                                                                                                          \
        const bool x_ok = wave < mNblk && i < mM;                                                                 \
        const uint16_t* xp = mX + (size_t)min(i, mM - 1) * mK + (size_t)(mKblk0 + min(wave, mNblk - 1)) * 256 + 8 * kg; \
        _Pragma("unroll") for (int q = 0; q < 8; ++q) {                                                           \
            const bf16x8_t v = *reinterpret_cast<const bf16x8_t*>(xp + 32 * q);                                   \
            xr[q] = x_ok ? v : bf16x8_t{0, 0, 0, 0, 0, 0, 0, 0};                                                  \
        }                                                                                                         \
        tf = bf16x8_t{0, 0, 0, 0, 0, 0, 0, 0};                                                                    \
        if (wave == 0 && mB) tf = *reinterpret_cast<const bf16x8_t*>(mT + i * GS_TROW + 8 * kg);                  \
        __builtin_amdgcn_s_waitcnt(0x0F70);                                                                       \
    } while (0)

    // per-lane constants of the requests
    const uint32_t code_lane1 = 16u * (kg >> 1), code_lane2 = 16u * kg, code_lane4 = 32u * kg;
    // scales: fp32, lane l fetches group l % 4 of channel l / 4 (16 bytes per channel); bf16, lane l < 32 fetches
    // dword l % 2 of channel l / 2 (8 bytes per channel)
    const uint32_t rec_voff = 4u * (lane & 31), scale_lane = SB16 ? 4u * (lane & 1) : 4u * (lane & 3);
    const uint32_t rec_mine = 8u * i, rec_scale = SB16 ? 8u * ((lane & 31) >> 1) : 8u * (lane >> 2);
    const uint32_t ring_begin = smem_lds + RING0, ring_end = ring_begin + GS_D * GS_SLOTB;
    const uint32_t lora_begin = smem_lds + LORA0, lora_end = lora_begin + GS_LORAB;
    const uint32_t rec_begin = smem_lds + REC0, rec_end = rec_begin + GS_NREC * GS_RECB;
    uint32_t ring_slot = ring_begin;                                // ring slot of unit j (and of unit j + GS_D, which refills it)
    uint32_t lora_slot = lora_begin;
    uint32_t recW = rec_begin;                                      // record slots of units j + 2 GS_D (written) ...
    uint32_t recRd = rec_begin + (GS_NREC - GS_D) * GS_RECB;        // ... and j + GS_D (read): written GS_D passes ago

    // One pass (BITS: the width of the C cursor's unit, 0 while there is no arithmetic yet):
    //  * request the row records of the R cursor's unit (2 GS_D ahead): lane l < 32 fetches dword l of the strip's 16
    //    records (128 contiguous bytes);
    //  * wait: the transfers of unit j (issued GS_D passes ago) have landed -- after them came GS_D - 1 passes of 3
    //    transfers each (4 for wavefront 0) and this pass's record request; the records of unit j + GS_D are older still;
    //  * read everything this pass needs from the rings at once: my codes and scales (unit j), the records of unit
    //    j + GS_D, wavefront 0's B fragment;
    //  * request the codes and scales of the I cursor's unit into the slot just read (codes: 16 bytes per lane -- 2 bits:
    //    group kg; 4 bits: half of group kg; 1 bit: the aligned pair of groups that holds group kg), wavefront 0 also the
    //    strip's B rows (no rank-r term: the codes again, so that the count of transfers stays the same);
    //  * contract unit j; at the end of a strip the 16 partial results meet in LDS, and wavefront (strip number) mod 16
    //    adds them in a fixed order and stores.  It reads all 16 slots at once (a wavefront past the chunk's end
    //    contributed zeros): with one dependent LDS round trip per slot this wavefront was late for the next strip's
    //    barrier by 16 round trips, on every strip.  (Every wavefront adding one channel of every strip, with a
    //    sum across lanes, was slower: 0.71 against 0.60 ms for the whole set at one token.);
    //  * move the three cursors on (GS_CUR_STEP: no tests; the run around the passes settles them afterwards).
#define GS_PASS(BITS)                                                                                                                                            \
    do {                                                                                                                                                   \
            gs_dma4_low32(rowsR + (size_t)(uint32_t)stripR * GS_RECB, rec_voff, recW);                                                                               \
            recW = gs_ring_next(recW, GS_RECB, rec_begin, rec_end);                                                                                        \
            GS_CUR_STEP(R, advR, t4R);                                                                     \
            if (wave == 0) gs_wait_transfers<4 * GS_D - 3>();                                                                                              \
            else gs_wait_transfers<3 * GS_D - 2>();                                                                                                        \
            const uint8_t* slot = gs_smem + (ring_slot - smem_lds);                                                                                        \
            uint4 cq = make_uint4(0u, 0u, 0u, 0u);                                                                                                         \
            float4 sq = make_float4(0.0f, 0.0f, 0.0f, 0.0f);                                                                                               \
            uint2 sh = make_uint2(0u, 0u);                                                                                                                 \
            if (BITS) {                                                                                                                                    \
                cq = *reinterpret_cast<const uint4*>(slot + 16 * lane);                                                                                    \
                if (SB16) sh = *reinterpret_cast<const uint2*>(slot + 1024 + 8 * i);                                                                       \
                else sq = *reinterpret_cast<const float4*>(slot + 1024 + 16 * i);                                                                          \
            }                                                                                                                                              \
            const uint8_t* recs = gs_smem + (recRd - smem_lds);                                                                                            \
            recRd = gs_ring_next(recRd, GS_RECB, rec_begin, rec_end);                                                                                      \
            const uint2 rc = *reinterpret_cast<const uint2*>(recs + rec_mine);                                                                             \
            const uint2 rs = *reinterpret_cast<const uint2*>(recs + rec_scale);                                                                            \
            uint4 bq = make_uint4(0u, 0u, 0u, 0u);                                                                                                         \
            const int n_now = nfifo0; (void)n_now;                                                                                                         \
            if (BITS && wave == 0) bq = *reinterpret_cast<const uint4*>(gs_smem + (lora_slot - smem_lds) + 16 * lane);                                     \
            {                                                                                                                                              \
                const uint8_t* cbase = iPacked + (size_t)(iKb32 * bitsI + 16 * halfI);                                                                     \
                gs_wait_lds();                                                                                                                             \
                const uint32_t cvoff = rc.x + (bitsI == 2 ? code_lane2 : bitsI == 4 ? code_lane4 : code_lane1);                                            \
                const uint32_t svoff = (uint32_t)max((int)rs.y, 0) * (uint32_t)iG4 + scale_lane;                                                           \
                if (wave == 0) {                                                                                                                           \
                    const uint8_t* bbase = iB ? reinterpret_cast<const uint8_t*>(iB) : cbase;                                                              \
                    const uint32_t bvoff = iB ? ((uint32_t)max((int)rc.y, 0) * (uint32_t)iR + 8u * (uint32_t)min(kg, max(iR / 8 - 1, 0))) * 2u : cvoff;    \
                    dma16_s(bbase, bvoff, lora_slot);                                                                                                      \
                    lora_slot = gs_ring_next(lora_slot, 1024, lora_begin, lora_end);                                                                       \
                }                                                                                                                                          \
                nfifo0 = nfifo1; nfifo1 = nfifo2; nfifo2 = (int)rc.y;                                                                                      \
                if (!(GS_EXP & 8)) {                                                                                                                       \
                    dma16_s(cbase, cvoff, ring_slot);                                                                                                      \
                    if (SB16) gs_dma4_low32(iScaleBase, svoff, ring_slot + 1024);                                                                          \
                    else dma4_s(iScaleBase, svoff, ring_slot + 1024);                                                                                      \
                }                                                                                                                                          \
                ring_slot = gs_ring_next(ring_slot, GS_SLOTB, ring_begin, ring_end);                                                                       \
                GS_CUR_STEP(I, advI, t4I);                                                                                                 \
            }                                                                                                                                              \
            if (BITS != 0) {                                                                                                                               \
                if (SB16) sq = make_float4(bf16_bits_to_float(sh.x & 0xffffu), __builtin_bit_cast(float, sh.x & 0xffff0000u),                              \
                                           bf16_bits_to_float(sh.y & 0xffffu), __builtin_bit_cast(float, sh.y & 0xffff0000u));                             \
                const bool last = BITS != 4 || halfC != 0;                                                                                                 \
                gs_unit<ONE, (BITS) ? (BITS) : 1>(gs_smem, halfC, (uint32_t)tabC * (uint32_t)GS_TABB, cq, sq, xr, lane, tot);                              \
                if (last) {                                                                                                                                \
                    if (wave == 0 && mB)                                                                                                                   \
                        tot = __builtin_amdgcn_mfma_f32_16x16x32_bf16(tf, __builtin_bit_cast(bf16x8_t, bq), tot, 0, 0, 0);                                 \
                    const int seq = mSeq0 + stripC;                                                                                                        \
                    const int rslot = seq & 1;                                                                                                             \
                    *reinterpret_cast<float4*>(gs_smem + RED0 + rslot * GS_REDB + (wave * 64 + lane) * 16) = make_float4(tot[0], tot[1], tot[2], tot[3]);  \
                    tot = floatx4_t{0.0f, 0.0f, 0.0f, 0.0f};                                                                                               \
                    if (!(GS_EXP & 2)) gs_lds_barrier();                                                                                                   \
                    if (!(GS_EXP & 2) && (seq & (GS_W - 1)) == wave) {                                                                                     \
                        const uint8_t* red = gs_smem + RED0 + rslot * GS_REDB + lane * 16;                                                                 \
                        floatx4_t sum = {0.0f, 0.0f, 0.0f, 0.0f};                                                                                          \
                        if (ONE) {                                                                                                                         \
                            float r1[GS_W];                                                                                                                \
    _Pragma("unroll")                                                                                                                                      \
                            for (int w = 0; w < GS_W; ++w) r1[w] = *reinterpret_cast<const float*>(red + w * 1024);                                        \
    _Pragma("unroll")                                                                                                                                      \
                            for (int w = 0; w < GS_W; ++w) sum[0] += r1[w];                                                                                \
                        } else {                                                                                                                           \
    _Pragma("nounroll")                                                                                                                                    \
                            for (int h = 0; h < 4; ++h) {                                                                                                  \
                                float4 rv[GS_W / 4];                                                                                                       \
    _Pragma("unroll")                                                                                                                                      \
                                for (int w = 0; w < GS_W / 4; ++w) rv[w] = *reinterpret_cast<const float4*>(red + (h * (GS_W / 4) + w) * 1024);            \
    _Pragma("unroll")                                                                                                                                      \
                                for (int w = 0; w < GS_W / 4; ++w) { sum[0] += rv[w].x; sum[1] += rv[w].y; sum[2] += rv[w].z; sum[3] += rv[w].w; }         \
                            }                                                                                                                              \
                        }                                                                                                                                  \
                        if (n_now >= 0 && !(GS_EXP & 1)) {                                                                                                 \
    _Pragma("unroll")                                                                                                                                      \
                            for (int v = 0; v < (ONE ? 1 : 4); ++v) {                                                                                      \
                                const int m = 4 * kg + v;                                                                                                  \
                                if (m < mM) {                                                                                                              \
                                    const size_t o = (size_t)m * mN + n_now;                                                                               \
                                    if (mOutFp32) static_cast<float*>(mOut)[o] = sum[v];                                                                   \
                                    else static_cast<uint16_t*>(mOut)[o] = (uint16_t)(pack_bf16x2(sum[v], 0.0f) & 0xffffu);                                \
                                }                                                                                                                          \
                            }                                                                                                                              \
                        }                                                                                                                                  \
                    }                                                                                                                                      \
                }                                                                                                                                          \
            }                                                                                                                                              \
            if (BITS == 4) GS_CUR_STEP(C, 1, 1); else if (BITS != 0) GS_CUR_STEP(C, 1, 0);                    \
    } while (0)

    // A run of TOTAL passes with the arithmetic of width BITS (0: none; else the C cursor stays inside its class for
    // the whole run, which the caller sees to), cut into pieces in which the R and I cursors stay inside theirs.
    // HOLD_I: the I cursor does not move (the first GS_D passes: no record has landed yet).
#define GS_RUN(BITS, TOTAL, HOLD_I)                                                                               \
    for (int todo = (TOTAL); todo > 0;) {                                                                         \
        const int advR = leftR > 0 ? 1 : 0, advI = (!(HOLD_I) && leftI > 0) ? 1 : 0;                              \
        const int t4R = bitsR == 4 ? advR : 0, t4I = bitsI == 4 ? advI : 0;                                       \
        int cnt = todo;                                                                                           \
        if (advR) cnt = min(cnt, min(endR - luR, leftR));                                                         \
        if (advI) cnt = min(cnt, min(endI - luI, leftI));                                                         \
        for (int k = 0; k < cnt; ++k) GS_PASS(BITS);                                                              \
        todo -= cnt;                                                                                              \
        if (advR) GS_CUR_SETTLE(R, cnt, rowsR = reinterpret_cast<const uint8_t*>(segs[segR].rows));               \
        if (advI) GS_CUR_SETTLE(I, cnt, GS_SEG_ISSUE(segs + segI));                                               \
    }

    // ---- the first 2 GS_D passes only ask
    GS_RUN(0, GS_D, true);
    GS_RUN(0, GS_D, false);
    GS_LOAD_X();
    // ---- then class by class of the arithmetic's cursor: one instruction stream per width
    for (int done = 0; done < n;) {
        const int cnt_c = min(endC - luC, n - done);
        const int seg_before = segC;
        if (bitsC == 1) GS_RUN(1, cnt_c, false)
        else if (bitsC == 2) GS_RUN(2, cnt_c, false)
        else GS_RUN(4, cnt_c, false)
        done += cnt_c;
        if (done < n) {
            GS_CUR_SETTLE(C, cnt_c, (void)0);
            if (segC != seg_before) { GS_SEG_MATH(segs + segC); GS_LOAD_X(); }
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                // nothing of mine may land in LDS after I am gone
#undef GS_SEG_ISSUE
#undef GS_SEG_MATH
#undef GS_LOAD_X
#undef GS_PASS
#undef GS_RUN
}

// y = bf16(sum of the chunks' fp32 partial outputs), for every matrix that was cut into chunks
struct GsSum { const float* part; uint16_t* y; int count; int nchunks; };
__global__ __launch_bounds__(256) void gemv_stream_sum_kernel(const GsSum* __restrict__ sums, int per_item_blocks) {
    const GsSum d = sums[blockIdx.x / per_item_blocks];
    const auto part = as_global(d.part);
    const auto y = as_global(d.y);
    for (int o = (blockIdx.x % per_item_blocks) * 256 + threadIdx.x; o < d.count; o += per_item_blocks * 256) {
        float v = 0.0f;
        for (int c = 0; c < d.nchunks; ++c) v += part[(size_t)c * d.count + o];
        y[o] = (uint16_t)(pack_bf16x2(v, 0.0f) & 0xffffu);
    }
}

// ---- t = s x A^T as bf16 [16][GS_TROW] (zero past M and past r): one workgroup of 16 wavefronts per matrix.
// Wavefront w takes the 256-column blocks w, w + 16, ...: MFMA step q of a block contracts columns 32 q + 8 kg + e
// of lane (i, kg), token i (operand B) against ranks i + 16 c (operand A), so one load instruction fetches 64
// contiguous bytes of each of its 16 rows (with 128 contiguous bytes per lane every instruction touched 64
// cache lines); the wavefronts' partial sums meet in LDS and are added in a fixed order.
struct GsTItem { const uint16_t* x; const uint16_t* A; uint16_t* t; int M, K, r; float s; };
__device__ __forceinline__ void gs_t_body(const GsTItem it) {
    __shared__ float tsum[GS_W][16][GS_TROW];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, i = lane & 15, kg = lane >> 4;
    const bf16x8_t zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
    floatx4_t acc[2] = {{0.0f, 0.0f, 0.0f, 0.0f}, {0.0f, 0.0f, 0.0f, 0.0f}};
    const int nblk = it.K / 256;
    for (int b = wave; b < nblk; b += GS_W) {
        const int kbase = b * 256 + kg * 8;
        // the block's loads are requested before the first is used: the rows are clamped to valid ones and what
        // lies past M or r is zeroed afterwards (a load under a condition is not moved above it).  The kernel is
        // a chain of round trips to cold memory either way -- descriptor, then a wavefront's one to three blocks
        // in turn: 20 us whether it runs one matrix or 224 (23.5 us with the conditional loads).
        typedef gptr<const bf16x8_t> gld_t;                          // the pointers come out of a descriptor in memory
        bf16x8_t xf[8], af[2][8];
        const uint16_t* xrow = it.x + (size_t)min(i, it.M - 1) * it.K + kbase;
#pragma unroll
        for (int q = 0; q < 8; ++q) xf[q] = *(gld_t)(xrow + 32 * q);
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const uint16_t* arow = it.A + (size_t)min(c * 16 + i, it.r - 1) * it.K + kbase;
#pragma unroll
            for (int q = 0; q < 8; ++q) af[c][q] = *(gld_t)(arow + 32 * q);
        }
#pragma unroll
        for (int q = 0; q < 8; ++q)
            if (i >= it.M) xf[q] = zero8;
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                if (c * 16 + i >= it.r) af[c][q] = zero8;
                acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[c][q], xf[q], acc[c], 0, 0, 0);
            }
    }
    // lane (i, kg) holds D[rank 16 c + 4 kg + v][token i]
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int v = 0; v < 4; ++v) tsum[wave][i][16 * c + 4 * kg + v] = acc[c][v];
    __syncthreads();
    for (int o = threadIdx.x; o < 16 * GS_TROW; o += GS_THREADS) {
        float v = 0.0f;
        for (int w = 0; w < GS_W; ++w) v += tsum[w][o / GS_TROW][o % GS_TROW];
        as_global(it.t)[o] = (uint16_t)(pack_bf16x2(v * it.s, 0.0f) & 0xffffu);
    }
}
__global__ __launch_bounds__(GS_THREADS) void gemv_stream_t_kernel(const GsTItem* __restrict__ items) { gs_t_body(items[blockIdx.x]); }

// ---- one matrix, descriptors written on the device (the call must not copy from the host: it may be captured)
struct GsSingle {
    GsSeg segs[GS_MAXSEG];
    GsSum sum;
    GsTItem titem;
    int nseg, nwg;
    GsSeg* d_segs; GsUnit* d_units; int* d_wg_first; GsSum* d_sum;
};
__global__ __launch_bounds__(GS_THREADS) void gemv_stream_prep_kernel(const GsSingle a) {
    if (a.titem.r > 0) gs_t_body(a.titem);
    const int per = a.segs[0].nunits, f4 = a.segs[0].first4, nstrips = a.segs[0].nstrips, total = a.nseg * per;
    for (int b = threadIdx.x; b <= a.nwg; b += GS_THREADS) {
        int u = (int)((long long)b * total / a.nwg);
        const int local = u % per;
        if (b < a.nwg && local > f4 && ((local - f4) & 1)) ++u;      // never between the two units of a 4-bit strip
        a.d_wg_first[b] = u;
    }
    for (int o = threadIdx.x; o < a.nseg * nstrips; o += GS_THREADS) {
        const int c = o / nstrips, sidx = o % nstrips;
        int cls = a.segs[0].cls_bits_cb[0];
#pragma unroll
        for (int q = 0; q + 1 < kGvMaxClasses; ++q) cls = sidx >= a.segs[0].cls_end[q] ? a.segs[0].cls_bits_cb[q + 1] : cls;
        const int bits = cls & 0xff, tab = cls >> 8;
        GsUnit* dst = a.d_units + (size_t)c * per + (sidx < f4 ? sidx : f4 + 2 * (sidx - f4));
        if (bits == 4) {
            dst[0] = GsUnit{(uint32_t)sidx * 128u, (uint32_t)c, gs_unit_flags(4, 0, 0, tab, o), 0u};
            dst[1] = GsUnit{(uint32_t)sidx * 128u, (uint32_t)c, gs_unit_flags(4, 1, 1, tab, o), 0u};
        } else {
            dst[0] = GsUnit{(uint32_t)sidx * 128u, (uint32_t)c, gs_unit_flags(bits, 0, 1, tab, o), 0u};
        }
    }
    if (threadIdx.x == 0) {
#pragma unroll
        for (int c = 0; c < GS_MAXSEG; ++c)
            if (c < a.nseg) a.d_segs[c] = a.segs[c];
        *a.d_sum = a.sum;
    }
}

// =============================================================================================== host side
bool gemv_stream_supported(const lowra_layout& L, int M, int r) {
    return M >= 1 && M <= 16 && gs_layout_supported(L) && r >= 0 && r <= 32 && r % 8 == 0;
}

static size_t gs_lds_bytes(const GsTabs& t) { return (size_t)t.nslot * GS_TABB + 2 * GS_REDB + (size_t)GS_W * GS_WAVEB + GS_LORAB; }
static_assert(GS_MAXTAB * GS_TABB + 2 * GS_REDB + GS_W * GS_WAVEB + GS_LORAB <= 160 * 1024, "LDS budget");

static hipError_t gs_attr() {
    static hipError_t a = gs_prepare_kernel(reinterpret_cast<const void*>(gemv_stream_kernel<true, false>));
    static hipError_t b = gs_prepare_kernel(reinterpret_cast<const void*>(gemv_stream_kernel<false, false>));
    static hipError_t c = gs_prepare_kernel(reinterpret_cast<const void*>(gemv_stream_kernel<true, true>));
    static hipError_t d = gs_prepare_kernel(reinterpret_cast<const void*>(gemv_stream_kernel<false, true>));
    return a != hipSuccess ? a : b != hipSuccess ? b : c != hipSuccess ? c : d;
}

static void gs_launch_main(bool one, const GsTabs& tabs, int nwg, const GsSeg* segs, const GsUnit* units, const int* wg_first,
                           const float* mappings, hipStream_t st) {
    const dim3 grid(nwg), block(GS_THREADS);
    const size_t lds = gs_lds_bytes(tabs);
    if (tabs.scale_bf16) {
        if (one) gemv_stream_kernel<true, true><<<grid, block, lds, st>>>(segs, units, wg_first, mappings, tabs);
        else gemv_stream_kernel<false, true><<<grid, block, lds, st>>>(segs, units, wg_first, mappings, tabs);
    } else {
        if (one) gemv_stream_kernel<true, false><<<grid, block, lds, st>>>(segs, units, wg_first, mappings, tabs);
        else gemv_stream_kernel<false, false><<<grid, block, lds, st>>>(segs, units, wg_first, mappings, tabs);
    }
}

// the segments (K-chunks) of one matrix; `part`: fp32 [nchunks][M][N] when there is more than one chunk
static int gs_make_segs(const lowra_layout& L, const uint8_t* packed, const float* absmax, const uint16_t* x, const uint16_t* B,
                        const uint16_t* t, uint16_t* y, float* part, int M, int r, GsSeg* out) {
    const int nblk_all = L.K / 256, nch = gs_nchunks(L);
    for (int c = 0; c < nch; ++c) {
        GsSeg& g = out[c];
        g = GsSeg{};
        g.rows = L.d_gv_rows; g.packed = packed; g.absmax = absmax; g.x = x;
        g.B = (c == 0 && r > 0) ? B : nullptr;
        g.t = t;
        g.out = nch > 1 ? static_cast<void*>(part + (size_t)c * M * L.N) : static_cast<void*>(y);
        g.N = L.N; g.K = L.K; g.G = L.G; g.M = M; g.nstrips = L.gv_nstrips;
        g.first4 = gs_first4(L); g.nunits = gs_units_per_seg(L);
        g.kblk0 = c * GS_W; g.nblk = std::min(GS_W, nblk_all - c * GS_W);
        g.out_fp32 = nch > 1; g.r = r;
        for (int q = 0; q < kGvMaxClasses; ++q) {
            g.cls_end[q] = L.gv_cls_end[q];
            g.cls_bits_cb[q] = L.gv_cls_bits_cb[q];
        }
    }
    return nch;
}

// workspace of a single call: [descriptors: segments | sum | wg_first][units][t][fp32 partial outputs of the chunks]
constexpr size_t GS_DESC_BYTES = 8192, GS_DESC_SUM = 1024, GS_DESC_FIRST = 2048;
constexpr int GS_MAXWG = 1024;
constexpr size_t GS_TBYTES = 16 * GS_TROW * 2;
static size_t gs_units_bytes(const lowra_layout& L) { return gs_align((size_t)gs_nchunks(L) * gs_units_per_seg(L) * sizeof(GsUnit)); }
size_t gemv_stream_workspace_bytes(const lowra_layout& L, int M, int r) {
    const size_t part = gs_nchunks(L) > 1 ? gs_align((size_t)gs_nchunks(L) * M * L.N * sizeof(float)) : 0;
    return GS_DESC_BYTES + gs_units_bytes(L) + (r > 0 ? GS_TBYTES : 0) + part;
}

hipError_t launch_gemv_stream(const lowra_layout& L, const LinearArgs& a, hipStream_t st) {
    hipError_t e = gs_attr();
    if (e != hipSuccess) return e;
    const GsTabs tabs = gs_tabs(L.cb_bits, L.scale_bf16);
    uint8_t* ws = static_cast<uint8_t*>(a.workspace);
    const int nwg = std::min(std::min(gs_compute_units(), GS_MAXWG), gs_nchunks(L) * L.gv_nstrips);   // at least one strip each
    static_assert(GS_MAXSEG * sizeof(GsSeg) <= GS_DESC_SUM && GS_DESC_SUM + sizeof(GsSum) <= GS_DESC_FIRST &&
                  GS_DESC_FIRST + (GS_MAXWG + 1) * sizeof(int) <= GS_DESC_BYTES, "descriptor area");
    GsSingle sg{};
    sg.d_segs = reinterpret_cast<GsSeg*>(ws);
    sg.d_sum = reinterpret_cast<GsSum*>(ws + GS_DESC_SUM);
    sg.d_wg_first = reinterpret_cast<int*>(ws + GS_DESC_FIRST);
    sg.d_units = reinterpret_cast<GsUnit*>(ws + GS_DESC_BYTES);
    uint16_t* t = reinterpret_cast<uint16_t*>(ws + GS_DESC_BYTES + gs_units_bytes(L));
    float* part = reinterpret_cast<float*>(ws + GS_DESC_BYTES + gs_units_bytes(L) + (a.r > 0 ? GS_TBYTES : 0));
    sg.nseg = gs_make_segs(L, a.packed, a.absmax, a.act, a.B, t, a.out, part, a.M, a.r, sg.segs);
    for (int c = 0; c < sg.nseg; ++c) { sg.segs[c].first_unit = c * gs_units_per_seg(L); sg.segs[c].seq0 = c * L.gv_nstrips; }
    sg.nwg = nwg;
    sg.titem = GsTItem{a.act, a.A, t, a.M, L.K, a.r, a.s};
    sg.sum = GsSum{part, a.out, a.M * L.N, sg.nseg};
    gemv_stream_prep_kernel<<<dim3(1), dim3(GS_THREADS), 0, st>>>(sg);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    gs_launch_main(a.M == 1, tabs, nwg, sg.d_segs, sg.d_units, sg.d_wg_first, a.mappings, st);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (sg.nseg > 1) {
        const int blocks = std::min(64, (a.M * L.N + 255) / 256);
        gemv_stream_sum_kernel<<<dim3(blocks), dim3(256), 0, st>>>(sg.d_sum, blocks);
        e = hipGetLastError();
    }
    return e;
}

// ---- a batch: descriptors built once on the host
size_t gemv_stream_batch_item_ws(const lowra_layout& L, int r) {      // t + chunk partials (for 16 tokens)
    const size_t part = gs_nchunks(L) > 1 ? gs_align((size_t)gs_nchunks(L) * 16 * L.N * sizeof(float)) : 0;
    return (r > 0 ? GS_TBYTES : 0) + part;
}

void gemv_stream_batch_free(GsBatch& b) {
    (void)hipFree(b.d_segs); (void)hipFree(b.d_wg_first); (void)hipFree(b.d_units); (void)hipFree(b.d_sums);
    (void)hipFree(b.d_titems);
    b = GsBatch{};
}

hipError_t gemv_stream_batch_build(const std::vector<GsBatchItem>& items, const float* mappings, int M, int r, float s, GsBatch& b) {
    if (items.empty()) return hipSuccess;
    std::vector<GsSeg> segs;
    std::vector<GsSum> sums;
    std::vector<GsTItem> titems;
    std::vector<GsUnit> unitv;
    std::vector<double> unit_cost;                                   // bytes of codes and scales per unit, plus a constant
    std::vector<char> pair_second;                                   // the unit is the second half of a 4-bit strip
    int strip_seq = 0;
#ifndef GS_FIXED_COST
#define GS_FIXED_COST 65536.0
#endif
    constexpr double kUnitFixedCost = GS_FIXED_COST;
    int units = 0;
    for (const GsBatchItem& it : items) {
        const lowra_layout& L = *it.L;
        uint16_t* t = reinterpret_cast<uint16_t*>(it.ws);
        float* part = reinterpret_cast<float*>(it.ws + (r > 0 ? GS_TBYTES : 0));
        GsSeg tmp[GS_MAXSEG];
        const int nch = gs_make_segs(L, it.packed, it.absmax, it.x, it.B, t, it.y, part, M, r, tmp);
        for (int c = 0; c < nch; ++c) {
            tmp[c].first_unit = units;
            tmp[c].seq0 = strip_seq;
            segs.push_back(tmp[c]);
            for (int sidx = 0; sidx < L.gv_nstrips; ++sidx) {
                int cls = L.gv_cls_bits_cb[0];
                for (int q = 0; q + 1 < kGvMaxClasses; ++q) if (sidx >= L.gv_cls_end[q]) cls = L.gv_cls_bits_cb[q + 1];
                const int bw = cls & 0xff, tab = cls >> 8;
                const double cost = 16.0 * tmp[c].nblk * (bw == 1 ? 32.0 + 16.0 : 64.0 + 16.0) + kUnitFixedCost;
                const uint32_t seg_index = (uint32_t)segs.size() - 1u;
                unit_cost.push_back(cost);
                pair_second.push_back(0);
                unitv.push_back(GsUnit{(uint32_t)sidx * 128u, seg_index, gs_unit_flags(bw, 0, bw != 4, tab, strip_seq), 0u});
                if (bw == 4) {
                    unit_cost.push_back(cost); pair_second.push_back(1);
                    unitv.push_back(GsUnit{(uint32_t)sidx * 128u, seg_index, gs_unit_flags(4, 1, 1, tab, strip_seq), 0u});
                }
                ++strip_seq;
            }
            units += tmp[c].nunits;
        }
        if (nch > 1) sums.push_back(GsSum{part, it.y, M * L.N, nch});
        if (r > 0) titems.push_back(GsTItem{it.x, it.A, t, M, L.K, r, s});
    }
    // contiguous unit ranges of (nearly) equal cost, never between the two units of a 4-bit strip
    const int nwg = std::min(gs_compute_units(), units);
    double total = 0.0;
    for (double c : unit_cost) total += c;
    std::vector<int> wg_first((size_t)nwg + 1, units);
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
    b.nwg = nwg; b.nsums = (int)sums.size(); b.nt = (int)titems.size(); b.mappings = mappings; b.M = M;
    b.max_count = 0;
    for (const GsSum& q : sums) b.max_count = std::max(b.max_count, q.count);
    b.cb_bits = items[0].L->cb_bits;
    b.scale_bf16 = items[0].L->scale_bf16;
    hipError_t e;
    if ((e = gs_to_device(segs, reinterpret_cast<GsSeg**>(&b.d_segs))) != hipSuccess) return e;
    if ((e = gs_to_device(wg_first, &b.d_wg_first)) != hipSuccess) return e;
    if ((e = gs_to_device(unitv, reinterpret_cast<GsUnit**>(&b.d_units))) != hipSuccess) return e;
    if ((e = gs_to_device(sums, reinterpret_cast<GsSum**>(&b.d_sums))) != hipSuccess) return e;
    if ((e = gs_to_device(titems, reinterpret_cast<GsTItem**>(&b.d_titems))) != hipSuccess) return e;
    return gs_attr();
}

hipError_t gemv_stream_batch_run(const GsBatch& b, hipStream_t st) {
    if (b.nwg == 0) return hipSuccess;
    hipError_t e;
    if (b.nt > 0) {
        gemv_stream_t_kernel<<<dim3(b.nt), dim3(GS_THREADS), 0, st>>>(static_cast<const GsTItem*>(b.d_titems));
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    const GsTabs tabs = gs_tabs(b.cb_bits, b.scale_bf16);
    {
        KernelTimer timer(st);
        gs_launch_main(b.M == 1, tabs, b.nwg, static_cast<const GsSeg*>(b.d_segs), static_cast<const GsUnit*>(b.d_units), b.d_wg_first, b.mappings, st);
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
