// Forward fused dequant-GEMM:  y = [x | s x A^T] [What | B]^T   (Sec. 2.1 LoRA form; App. A.2 decode)
//
// Thread t of a workgroup owns one weight row of the 256-row tile (rows of equal width sit on
// adjacent lanes, see tile_order) and decodes its 64 codes of the next contraction step into the
// LDS weight tile while the MFMAs of the current step run.  One barrier per step, two LDS stages.
//
// Decode of 1- and 2-bit rows uses no table memory and one instruction stream for both widths:
// the row's 2 or 4 levels times the group absmax are rounded to bf16 once per step (the same
// multiply and rounding as App. A.2, applied to 2^b values instead of 64 weights), their low and
// high bytes form the 8-byte source of v_perm_b32, and a pair of codes becomes the 4-byte selector
// with one bit-field extract, one 24-bit multiply that spreads the bits, and one and-or.  Width
// only changes per-lane constants.  Wavefronts that hold a 4-bit row take a slower step that
// looks the 16 levels up in an LDS table.
#include <cstdlib>

#include "gemm_common.h"

namespace lowra {

constexpr size_t kFwdSmem = 2 * STAGEB + (size_t)BN * TAB_LD * 4;

template <int DBG>
__global__ __launch_bounds__(NTHREADS) void linear_fwd_kernel(GemmParams p) {
    extern __shared__ __align__(16) uint8_t smem[];
    float* sT = reinterpret_cast<float*>(smem + 2 * STAGEB);
    const uint32_t smem_lds = (uint32_t)(uintptr_t)(lptr_t)smem;
    auto lds_of = [&](const uint8_t* q) -> uint32_t { return smem_lds + (uint32_t)(q - smem); };   // LDS byte address of the dynamic segment

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tiles_n = (p.N + BN - 1) / BN;
    const int tile = xcd_tile(blockIdx.x, gridDim.x);
    const int n0 = (tile % tiles_n) * BN, m0 = (tile / tiles_n) * BM;

    // ---- my weight row
    const int lr = p.tile_order[n0 + tid];
    const int n = n0 + lr;
    const bool row_ok = n < p.N;
    const int nc = row_ok ? n : p.N - 1;                 // clamped: loads stay in bounds, levels are zeroed
    const RowInfo ri = p.rows[nc];
    const int bits = ri.bits();
    const uint8_t* rowp = p.packed + ri.offset;
    const float* amp = p.absmax + (size_t)nc * p.G;
    const float* mrow = p.mappings + (size_t)ri.cb() * kTableStride;
    float lev[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) lev[q] = (row_ok && q < (1 << bits)) ? mrow[q] : 0.0f;
    float* tab = sT + lr * TAB_LD;
    if (bits == 4) {
#pragma unroll
        for (int q = 0; q < 16; ++q) tab[q] = row_ok ? mrow[q] : 0.0f;
    }
    const bool wave_fast = __builtin_amdgcn_ballot_w64(bits == 4) == 0;

    // per-lane constants of the unified 1-/2-bit decode
    const bool two = bits == 2;
    const uint32_t fw = two ? 4u : 2u;                      // bits per pair of codes
    const uint32_t MUL = two ? 0x404101u : 0x808101u;       // spreads the pair's bits to byte lanes
    const uint32_t MASK = two ? 0x03030303u : 0x01010101u;
    const uint32_t ORC = two ? 0x04000400u : 0x02000200u;   // high-byte entries sit after the low-byte ones
    const uint32_t selL = two ? 0x06040200u : 0x03010200u;
    const uint32_t selH = two ? 0x07050301u : 0x03010200u;
    const uint32_t selN0 = two ? 0x03020100u : 0x0c010c00u; // code stream -> one 16-bit slot per 8 codes
    const uint32_t selN1 = two ? 0x07060504u : 0x0c030c02u;
    const uint32_t selN2 = two ? 0x07060504u : 0x0c010c00u;
    const int cstride = 8 * bits;                            // code bytes per step
    const int c2off = two ? 8 : 0;                           // 1-bit rows re-read their 8 bytes

    // ---- activation tile: global -> LDS DMA (global_load_lds_dwordx4), no registers in between.
    // One instruction fills 8 LDS rows (64 lanes x 16 B, linear in LDS); wavefront w owns rows
    // [64 w, 64 w + 64).  The LDS side is linear, so the chunk swizzle is applied to the global
    // address: the lane that lands on physical chunk l&7 of row r fetches logical chunk
    // (l&7) ^ ((r>>1)&7).  Rows past M are clamped to the last row (never stored back).
    const int m_last = p.M - 1 - m0;
    uint32_t a_row_c[8], a_chunk_b[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int r = wave * 64 + 8 * i + (lane >> 3);
        a_row_c[i] = (uint32_t)(r < m_last ? r : m_last);
        a_chunk_b[i] = (uint32_t)(((lane & 7) ^ ((r >> 1) & 7)) * 16);
    }
    uint32_t a_voff_main[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) a_voff_main[i] = a_row_c[i] * (uint32_t)p.K * 2u + a_chunk_b[i];

    const int kt_main = p.K / BK, kt_all = kt_main + p.RP / BK;
    uint32_t rc[8];
    float rscale = 0.0f;

    auto dma_act_main = [&](int kt, uint8_t* sdst) {
        const uint8_t* base = reinterpret_cast<const uint8_t*>(p.act + (size_t)m0 * p.K + (size_t)kt * BK);
#pragma unroll
        for (int i = 0; i < 8; ++i)
            dma16(base + a_voff_main[i], lds_of(sdst) + wave * 8192 + i * 1024);
    };
    auto dma_act_any = [&](int kt, uint8_t* sdst) {
        if (kt < kt_main) {
            dma_act_main(kt, sdst);
        } else {
            const uint8_t* base = reinterpret_cast<const uint8_t*>(p.ext_act + (size_t)m0 * p.RP + (size_t)(kt - kt_main) * BK);
#pragma unroll
            for (int i = 0; i < 8; ++i)
                dma16(base + a_row_c[i] * (uint32_t)p.RP * 2u + a_chunk_b[i], lds_of(sdst) + wave * 8192 + i * 1024);
        }
    };
    auto load_codes_fast = [&](int kt) {      // 1-/2-bit rows only
        const uint8_t* cp = rowp + (size_t)kt * cstride;
        const uint2 c0 = *reinterpret_cast<const uint2*>(cp);
        const uint2 c1 = *reinterpret_cast<const uint2*>(cp + c2off);
        rc[0] = c0.x; rc[1] = c0.y; rc[2] = c1.x; rc[3] = c1.y;
        rscale = amp[kt];
    };
    auto load_codes_any = [&](int kt) {
        if (kt < kt_main) {
            const uint2* cp = reinterpret_cast<const uint2*>(rowp + (size_t)kt * cstride);
            const uint2 c0 = cp[0];
            rc[0] = c0.x; rc[1] = c0.y;
            if (bits >= 2) { const uint2 c1 = cp[1]; rc[2] = c1.x; rc[3] = c1.y; }
            if (bits == 4) {
                const uint2 c2 = cp[2], c3 = cp[3];
                rc[4] = c2.x; rc[5] = c2.y; rc[6] = c3.x; rc[7] = c3.y;
            }
            rscale = amp[kt];
        }
    };
    // generic decode of chunks [c_lo, c_hi) of step kt into the weight tile at bdst (branches allowed)
    auto store_b_any = [&](int kt, uint8_t* bdst, int c_lo, int c_hi, const uint32_t (&codes)[8], float a) {
        if (kt < kt_main) {
            if (bits == 1) {
                const uint32_t P01 = pack_bf16x2(lev[0] * a, lev[1] * a);
                const uint32_t Q = __builtin_amdgcn_perm(P01, P01, 0x03010200u);
#pragma unroll
                for (int i = c_lo; i < c_hi; ++i)
                    *reinterpret_cast<uint4*>(bdst + swz_off(lr, i)) = decode8_w1(codes[i >> 2] >> (8 * (i & 3)), Q);
            } else if (bits == 2) {
                const uint32_t P01 = pack_bf16x2(lev[0] * a, lev[1] * a), P23 = pack_bf16x2(lev[2] * a, lev[3] * a);
                const uint32_t TL = __builtin_amdgcn_perm(P23, P01, 0x06040200u);
                const uint32_t TH = __builtin_amdgcn_perm(P23, P01, 0x07050301u);
#pragma unroll
                for (int i = c_lo; i < c_hi; ++i)
                    *reinterpret_cast<uint4*>(bdst + swz_off(lr, i)) = decode8_w2(codes[i >> 1] >> (16 * (i & 1)), TL, TH);
            } else {
#pragma unroll
                for (int i = c_lo; i < c_hi; ++i)
                    *reinterpret_cast<uint4*>(bdst + swz_off(lr, i)) = decode8_bf16(codes[i], 4, tab, a);
            }
        } else {
            const uint4* s = reinterpret_cast<const uint4*>(p.ext_w + (size_t)nc * p.RP + (kt - kt_main) * BK);
#pragma unroll
            for (int i = c_lo; i < c_hi; ++i) *reinterpret_cast<uint4*>(bdst + swz_off(lr, i)) = row_ok ? s[i] : zero4();
        }
    };

    // ---- MFMA operand addressing
    const int wm = wave >> 1, wn = wave & 1;
    const int fi = lane & 31, fkg = lane >> 5, fsw = (fi >> 1) & 7;
    const int a_base = (wm * 128 + fi) * ROWB, b_base = TILEB + (wn * 128 + fi) * ROWB;
    int koff[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) koff[kk] = ((2 * kk + fkg) ^ fsw) << 4;
    int b_soff[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) b_soff[i] = TILEB + swz_off(lr, i);

    floatx16_t acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    auto load_frags = [&](const uint8_t* sbase, int kk, bf16x8_t (&fa)[4], bf16x8_t (&fb)[4]) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            fa[t] = *reinterpret_cast<const bf16x8_t*>(sbase + a_base + t * 32 * ROWB + koff[kk]);
            fb[t] = *reinterpret_cast<const bf16x8_t*>(sbase + b_base + t * 32 * ROWB + koff[kk]);
        }
    };
    auto mma16 = [&](const bf16x8_t (&fa)[4], const bf16x8_t (&fb)[4]) {
#pragma unroll
        for (int tm = 0; tm < 4; ++tm)
#pragma unroll
            for (int tn = 0; tn < 4; ++tn)
                acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[tm], fb[tn], acc[tm][tn], 0, 0, 0);
    };

    // Fast step (1-/2-bit wavefront; steps kt+1 and kt+2 are ordinary weight steps): no branches.
    // Fast step (1-/2-bit wavefront; steps kt+1 and kt+2 are ordinary weight steps): no branches,
    // and the issue order is fixed by hand.  Each of the 64 MFMAs (8 passes = 32 cycles in the
    // matrix pipe) is followed by a slot of independent work that issues in its shadow: two decode
    // instructions, and in some slots one LDS operand read for the next sub-step, one DMA of the
    // next activation tile, the code loads of step kt+2 or an LDS write of a finished chunk.
    uint32_t boff[2][4];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int j = 0; j < 4; ++j) boff[h][j] = 16u * h + j * fw;
    auto fast_step = [&](int kt) {
        const uint8_t* sbase = smem + (kt & 1) * STAGEB;
        uint8_t* nbase = smem + ((kt & 1) ^ 1) * STAGEB;
        bf16x8_t fa[2][4], fb[2][4];
        load_frags(sbase, 0, fa[0], fb[0]);
        // while those reads fly: scaled levels of step kt+1 as byte tables, codes as one 16-bit slot per chunk
        const uint32_t P01 = pack_bf16x2(lev[0] * rscale, lev[1] * rscale);
        const uint32_t P23 = pack_bf16x2(lev[2] * rscale, lev[3] * rscale);
        const uint32_t SL = __builtin_amdgcn_perm(P23, P01, selL), SH = __builtin_amdgcn_perm(P23, P01, selH);
        uint32_t x[4];
        x[0] = __builtin_amdgcn_perm(rc[1], rc[0], selN0);
        x[1] = __builtin_amdgcn_perm(rc[1], rc[0], selN1);
        x[2] = __builtin_amdgcn_perm(rc[2], rc[1], selN2);
        x[3] = __builtin_amdgcn_perm(rc[3], rc[1], selN1);
        const uint8_t* dma_base = reinterpret_cast<const uint8_t*>(p.act + (size_t)m0 * p.K + (size_t)(kt + 1) * BK);
        const uint32_t nlds = smem_lds + ((kt & 1) ^ 1) * STAGEB;
        __builtin_amdgcn_sched_barrier(0);
        uint32_t d[2][4], t = 0;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
#pragma unroll
            for (int g = 0; g < 16; ++g) {
                const int tm = g >> 2, tn = g & 3;
                acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[kk & 1][tm], fb[kk & 1][tn], acc[tm][tn], 0, 0, 0);
                if (kk < 3 && g < 8 && !(DBG & 8)) {
                    if (g < 4)
                        fa[(kk + 1) & 1][g] = *reinterpret_cast<const bf16x8_t*>(sbase + a_base + g * 32 * ROWB + koff[kk + 1]);
                    else
                        fb[(kk + 1) & 1][g - 4] = *reinterpret_cast<const bf16x8_t*>(sbase + b_base + (g - 4) * 32 * ROWB + koff[kk + 1]);
                }
                {
                    const int pr = g >> 1, i = 2 * kk + (pr >> 2), j = pr & 3;
                    if (DBG & 2) {
                    } else if ((g & 1) == 0) {
                        t = __umul24(__builtin_amdgcn_ubfe(x[i >> 1], boff[i & 1][j], fw), MUL);
                    } else {
                        d[pr >> 2][j] = __builtin_amdgcn_perm(SH, SL, (t & MASK) | ORC);
                    }
                    if (DBG & 4) {
                    } else if (g == 7) *reinterpret_cast<uint4*>(nbase + b_soff[2 * kk]) = make_uint4(d[0][0], d[0][1], d[0][2], d[0][3]);
                    if (!(DBG & 4) && g == 15) *reinterpret_cast<uint4*>(nbase + b_soff[2 * kk + 1]) = make_uint4(d[1][0], d[1][1], d[1][2], d[1][3]);
                }
                if (kk == 0 && g < 8 && !(DBG & 1))
                    dma16(dma_base + a_voff_main[g], lds_of(nbase) + wave * 8192 + g * 1024);
                if (kk == 0 && g == 8) load_codes_fast(kt + 2);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        dma_wait_all();
        __syncthreads();
    };
    // General step: any width, LoRA extension steps, end of the contraction.
    auto slow_step = [&](int kt) {
        const uint8_t* sbase = smem + (kt & 1) * STAGEB;
        uint8_t* nbase = smem + ((kt & 1) ^ 1) * STAGEB;
        const bool has_next = kt + 1 < kt_all;
        bf16x8_t fa[2][4], fb[2][4];
        load_frags(sbase, 0, fa[0], fb[0]);
        uint32_t codes[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) codes[i] = rc[i];
        const float a = rscale;
        if (has_next) dma_act_any(kt + 1, nbase);
        if (kt + 2 < kt_all) load_codes_any(kt + 2);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            if (kk < 3) load_frags(sbase, kk + 1, fa[(kk + 1) & 1], fb[(kk + 1) & 1]);
            if (has_next) store_b_any(kt + 1, nbase + TILEB, 2 * kk, 2 * kk + 2, codes, a);
            mma16(fa[kk & 1], fb[kk & 1]);
        }
        dma_wait_all();
        __syncthreads();
    };

    // ---- prologue: step 0 into stage 0, step 1 in registers
    dma_act_any(0, smem);
    load_codes_any(0);
    {
        uint32_t codes[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) codes[i] = rc[i];
        store_b_any(0, smem + TILEB, 0, 8, codes, rscale);
    }
    if (kt_all > 1) load_codes_any(1);
    dma_wait_all();
    __syncthreads();

    int kt = 0;
    if (wave_fast) {
        for (; kt + 2 < kt_main; ++kt) fast_step(kt);
    } else {
        for (; kt + 2 < kt_main; ++kt) slow_step(kt);
    }
    for (; kt < kt_all; ++kt) slow_step(kt);

    store_out(acc, p.out, p.N, p.M, p.N, m0, n0);
}

hipError_t launch_gemm_fwd(const GemmParams& p, hipStream_t st) {
    static const int dbg = getenv("LOWRA_DBG") ? atoi(getenv("LOWRA_DBG")) : 0;
    const dim3 grid(((p.N + BN - 1) / BN) * ((p.M + BM - 1) / BM));
#define LAUNCH(D) case D: { static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(linear_fwd_kernel<D>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)kFwdSmem); if (attr != hipSuccess) return attr; linear_fwd_kernel<D><<<grid, dim3(NTHREADS), kFwdSmem, st>>>(p); break; }
    switch (dbg) { LAUNCH(0) LAUNCH(1) LAUNCH(2) LAUNCH(4) LAUNCH(6) LAUNCH(7) LAUNCH(8) LAUNCH(15) default: return hipErrorInvalidValue; }
    return hipGetLastError();
}

}  // namespace lowra
