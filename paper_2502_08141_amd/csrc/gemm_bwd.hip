// Input-gradient fused dequant-GEMM:  dX = [dY | s dY B] [What ; A]   (the base is frozen: no dW, Sec. 3)
//
// The contraction runs over output channels n while the codes are packed along k, so the MFMA
// operand of What wants 8 consecutive n for one k -- the transpose of what a packed row yields.
// The kernel keeps the decode exactly as in the forward kernel (a thread decodes 64 consecutive
// k of ONE row: one width, one table, one absmax per step) and stores the weight tile in LDS as
// [n][k]; the transposition happens in the LDS read: ds_read_b64_tr_b16 hands each lane of a
// 16-lane group four consecutive-n values of its own k column when lane r of the group points
// at row n0 + r/4, k offset 4 (r%4).  No second, transposed copy of the codes exists anywhere.
//
// Tile: 256 (tokens) x 256 (k) outputs, 64 channels per step.  Thread = (row lane, k-quarter
// wave): wavefront w decodes group k0/64 + w of the step's 64 rows.
//
// Fast steps (no 4-bit row in the matrix, K a multiple of 256) never load a row's codes with one
// lane per row: 64 lanes x 8 bytes from 64 different rows would cost 64 cache-line requests per
// instruction.  Instead wavefront w moves the 64 contiguous code bytes (the tile's four groups) of
// rows 16 w .. 16 w + 15 and their four absmax with one DMA each (4 lanes per row), three steps
// ahead, into a small LDS staging area; a step later each thread reads its own 16 bytes back,
// builds the byte tables of its row in the last slots of the step, and decodes one step later.

#include <algorithm>
#include <type_traits>

#include "gemm_common.h"

namespace lowra {

typedef short v4i16_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) v4i16_t* lds_v4i16_ptr;

constexpr int BROWB = 512;   // bytes per LDS row of the weight tile: 256 k x bf16
constexpr int CSTAGE0 = 2 * STAGEB;            // staged codes: 2 buffers x 64 rows x 64 B
constexpr int ASTAGE0 = CSTAGE0 + 2 * 4096;    // staged absmax: 2 buffers x 64 rows x 4 groups x 4 B
constexpr int kLutBooks = 64;                  // codebooks the lookup decode keeps in LDS (16 fp32 levels each)
constexpr int TABL0 = ASTAGE0 + 2 * 1024;
constexpr int kRowTabB = BK * kTableStride * 4; // with more codebooks than that: the tables of a step's 64 rows, 64 B each, two buffers
constexpr size_t kBwdSmem = TABL0 + 2 * kRowTabB;
static_assert(kLutBooks * kTableStride * 4 <= 2 * kRowTabB, "either table scheme fits the region");

// LDS byte offset of 16-byte chunk c (0..31) of weight-tile row r.  The low four bits of the chunk
// index are XOR-swizzled with the row: row bits 0-1 move chunk bits 2-3, row bits 2-3 move chunk
// bits 0-1.  A 16-byte store instruction (16 consecutive rows, one chunk) then lands on 16
// different chunk positions = all 64 banks, and so does half a transposing read (4 consecutive
// rows x 4 consecutive chunks, the other row bits fixed).
__device__ __forceinline__ int bswz(int r, int c) { return r * BROWB + ((c ^ (((r & 3) << 2) | ((r >> 2) & 3))) << 4); }

struct LutRegs {          // the same for the lookup decode (any width): the group's codes, absmax, codebook address
    uint32_t rc[8];
    float scale;
    uint32_t tb;
    uint32_t bits;
};

struct RowRegs {          // what a thread needs to decode its row's group for one step
    uint32_t rc[4];
    float scale;
    float lev[4];
    int bits;
};

// LUT: the instantiation for matrices with 4-bit rows (every step a general step with the lookup decode)
template <bool LUT>
__global__ __launch_bounds__(NTHREADS) void linear_bwd_kernel(GemmParams p_in) {
    extern __shared__ __align__(16) uint8_t smem[];
    const uint32_t smem_lds = (uint32_t)(uintptr_t)(lptr_t)smem;
    auto lds_of = [&](const uint8_t* q) -> uint32_t { return smem_lds + (uint32_t)(q - smem); };

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform, and known to be
    GemmParams p = p_in;
    const int tiles_k = (p.K + BN - 1) / BN;
    const int ntiles = tiles_k * ((p.M + BM - 1) / BM);
    // The grid: the whole tiles first, then `splits` workgroups for each of the tiles from p.split_first on (launched
    // last, so that they fill the last, short round together).
    int tile, split = 0, nsplit = 1;
    if ((int)blockIdx.x < p.split_first || p.splits <= 1) {
        tile = xcd_tile(blockIdx.x, p.splits > 1 ? p.split_first : (int)gridDim.x);
    } else {
        const int ntail = ntiles - p.split_first;
        const int w = xcd_tile((int)blockIdx.x - p.split_first, ntail * p.splits);
        // (a division by a run-time value is vector arithmetic: back into scalar registers, these live to the last store)
        split = __builtin_amdgcn_readfirstlane(w / ntail);
        tile = p.split_first + w - split * ntail;
        nsplit = p.splits;
    }
    const int k0 = (tile % tiles_k) * BN, m0 = (tile / tiles_k) * BM;
    // A split of the contraction is the same problem on a run of the matrix's rows: the records, the scales and the
    // columns of dY start at the run's first row; only the last split carries the ragged end and the rank-r steps.
    if (nsplit > 1) {
        const int rows_lo = split * p.rows_per_split;
        p.rows += rows_lo;
        p.absmax += (size_t)rows_lo * p.G;
        p.act += rows_lo;
        if (split + 1 < nsplit) { p.N = p.rows_per_split; p.RP = 0; }
        else p.N -= rows_lo;
    }

    // ---- my slice of the weight tile: row `lane` of the step, group k0/64 + wave
    const int kcol = k0 + wave * 64;
    const bool g_ok = kcol < p.K;
    const int g = (g_ok ? kcol : 0) >> 6;
    const int nt_full = p.N / BK;                      // steps whose 64 rows all exist
    const int nt_main = (p.N + BK - 1) / BK, nt_all = nt_main + p.RP / BK;

    // all codebooks into LDS for the lookup decode (visible after the prologue's barrier).  With more codebooks than
    // fit (the paper's own data model: one table set per output channel, Sec. 4.1) the tables of a step's 64 rows are
    // staged instead, two steps ahead of their decode: wavefront w fetches levels 4 w .. 4 w + 3 of row `lane`.
    const bool per_row = LUT && p.C > kLutBooks;
    if (LUT && !per_row)
        for (int e = tid; e < p.C * kTableStride; e += NTHREADS) reinterpret_cast<float*>(smem + TABL0)[e] = p.mappings[e];
    float4 lvq = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    auto load_row_table = [&](int nt, const RowInfo& ri) {            // my quarter of the table of row `lane` of step nt
        const int n = nt * BK + lane;
        lvq = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        if (nt < nt_main && n < p.N) lvq = *reinterpret_cast<const float4*>(p.mappings + (size_t)ri.cb() * kTableStride + 4 * wave);
    };
    auto store_row_table = [&](int nt) {
        *reinterpret_cast<float4*>(smem + TABL0 + (nt & 1) * kRowTabB + lane * (kTableStride * 4) + 16 * wave) = lvq;
    };

    // ---- activation tile dY[m0.., n-step] by DMA, as in the forward kernel (row length N)
    const int m_last = p.M - 1 - m0;
    auto a_row_c = [&](int i) -> uint32_t {
        const int r = wave * 64 + 8 * i + (lane >> 3);
        return (uint32_t)(r < m_last ? r : m_last);
    };
    auto a_chunk = [&](int i) -> uint32_t {
        const int r = wave * 64 + 8 * i + (lane >> 3);
        return (uint32_t)((lane & 7) ^ ((r >> 1) & 7));
    };
    uint32_t a_voff_main[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) a_voff_main[i] = a_row_c(i) * (uint32_t)p.ld_act * 2u + a_chunk(i) * 16u;

    auto dma_act_any = [&](int nt, uint8_t* sdst) {
        if (nt < nt_full) {
            const uint8_t* base = reinterpret_cast<const uint8_t*>(p.act + (size_t)m0 * p.ld_act + (size_t)nt * BK);
#pragma unroll
            for (int i = 0; i < 8; ++i)
                dma16(base + a_voff_main[i], lds_of(sdst) + wave * 8192 + i * 1024);
        } else if (nt < nt_main) {
            // ragged last step: chunks past N are clamped onto the last valid chunk (their weights are zero)
            const uint8_t* base = reinterpret_cast<const uint8_t*>(p.act + (size_t)m0 * p.ld_act);
            const int last_chunk = p.N / 8 - 1;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                int ch = nt * 8 + (int)a_chunk(i);
                ch = ch < last_chunk ? ch : last_chunk;
                dma16(base + a_row_c(i) * (uint32_t)p.ld_act * 2u + (uint32_t)ch * 16u, lds_of(sdst) + wave * 8192 + i * 1024);
            }
        } else {
            const uint8_t* base = reinterpret_cast<const uint8_t*>(p.ext_act + (size_t)m0 * p.RP + (size_t)(nt - nt_main) * BK);
#pragma unroll
            for (int i = 0; i < 8; ++i)
                dma16(base + a_row_c(i) * (uint32_t)p.RP * 2u + a_chunk(i) * 16u, lds_of(sdst) + wave * 8192 + i * 1024);
        }
    };

    // ---- per-step row pipeline: record (3 steps ahead) -> codes/scale/levels (2 ahead) -> decode (1 ahead)
    auto load_rowinfo = [&](int nt) -> RowInfo {
        const int n = nt * BK + lane;
        RowInfo ri;
        ri.offset = 0; ri.bits_cb = 1;
        if (nt < nt_main && n < p.N) ri = p.rows[n];
        return ri;
    };
    auto load_rowregs = [&](int nt, const RowInfo& ri, RowRegs& d) {
        const int n = nt * BK + lane;
        const bool ok = g_ok && nt < nt_main && n < p.N;
        const int bits = ri.bits();
        d.bits = bits;
        if (ok && bits != 4) {
            const uint8_t* cp = p.packed + ri.offset + (size_t)g * 8 * bits;
            const uint2 c0 = *reinterpret_cast<const uint2*>(cp);
            const uint2 c1 = *reinterpret_cast<const uint2*>(cp + (bits == 2 ? 8 : 0));
            d.rc[0] = c0.x; d.rc[1] = c0.y; d.rc[2] = c1.x; d.rc[3] = c1.y;
            d.scale = p.absmax[(size_t)n * p.G + g];
            const float4 lv = *reinterpret_cast<const float4*>(p.mappings + (size_t)ri.cb() * kTableStride);
            d.lev[0] = lv.x; d.lev[1] = lv.y; d.lev[2] = bits == 2 ? lv.z : 0.0f; d.lev[3] = bits == 2 ? lv.w : 0.0f;
        } else {
            d.rc[0] = d.rc[1] = d.rc[2] = d.rc[3] = 0u;
            d.scale = ok ? p.absmax[(size_t)n * p.G + g] : 0.0f;
            d.lev[0] = d.lev[1] = d.lev[2] = d.lev[3] = 0.0f;
        }
    };
    // fast variant: rows exist, widths are 1 or 2 (checked by the caller), no branches
    auto load_rowregs_fast = [&](int nt, const RowInfo& ri, RowRegs& d) {
        const int n = nt * BK + lane;
        const int bits = ri.bits();
        d.bits = bits;
        const uint8_t* cp = p.packed + ri.offset + (size_t)g * 8 * bits;
        const uint2 c0 = *reinterpret_cast<const uint2*>(cp);
        const uint2 c1 = *reinterpret_cast<const uint2*>(cp + (bits == 2 ? 8 : 0));
        d.rc[0] = c0.x; d.rc[1] = c0.y; d.rc[2] = c1.x; d.rc[3] = c1.y;
        d.scale = p.absmax[(size_t)n * p.G + g];            // g is clamped; a k-quarter past K gets zero levels
        const float4 lv = *reinterpret_cast<const float4*>(p.mappings + (size_t)ri.cb() * kTableStride);
        d.lev[0] = g_ok ? lv.x : 0.0f; d.lev[1] = g_ok ? lv.y : 0.0f;
        d.lev[2] = (g_ok && bits == 2) ? lv.z : 0.0f; d.lev[3] = (g_ok && bits == 2) ? lv.w : 0.0f;
    };

    // generic decode of my 64 weights of step nt into the weight tile (any width, LoRA rows): branches allowed
    auto store_b_any = [&](int nt, uint8_t* bdst, int c_lo, int c_hi, const RowRegs& d, const RowInfo& ri_cur) {
        const int row = lane;
        if (nt < nt_main) {
            const int n = nt * BK + lane;
            const bool ok = g_ok && n < p.N;
            if (!ok) {
#pragma unroll
                for (int i = c_lo; i < c_hi; ++i) *reinterpret_cast<uint4*>(bdst + bswz(row, wave * 8 + i)) = zero4();
            } else if (d.bits == 1) {
                const uint32_t P01 = pack_bf16x2(d.lev[0] * d.scale, d.lev[1] * d.scale);
                const uint32_t Q = __builtin_amdgcn_perm(P01, P01, 0x03010200u);
#pragma unroll
                for (int i = c_lo; i < c_hi; ++i)
                    *reinterpret_cast<uint4*>(bdst + bswz(row, wave * 8 + i)) = decode8_w1(d.rc[i >> 2] >> (8 * (i & 3)), Q);
            } else if (d.bits == 2) {
                const uint32_t P01 = pack_bf16x2(d.lev[0] * d.scale, d.lev[1] * d.scale);
                const uint32_t P23 = pack_bf16x2(d.lev[2] * d.scale, d.lev[3] * d.scale);
                const uint32_t TL = __builtin_amdgcn_perm(P23, P01, 0x06040200u);
                const uint32_t TH = __builtin_amdgcn_perm(P23, P01, 0x07050301u);
#pragma unroll
                for (int i = c_lo; i < c_hi; ++i)
                    *reinterpret_cast<uint4*>(bdst + bswz(row, wave * 8 + i)) = decode8_w2(d.rc[i >> 1] >> (16 * (i & 1)), TL, TH);
            } else {
                // 4-bit row: codes and the 16-level table straight from global memory (slow path)
                const uint32_t* cp = reinterpret_cast<const uint32_t*>(p.packed + ri_cur.offset + (size_t)g * 32);
                const float* tab = p.mappings + (size_t)ri_cur.cb() * kTableStride;
#pragma unroll
                for (int i = c_lo; i < c_hi; ++i)
                    *reinterpret_cast<uint4*>(bdst + bswz(row, wave * 8 + i)) = decode8_bf16(cp[i], 4, tab, d.scale);
            }
        } else {
            // LoRA extension: row j of A (rank index), my 64 k columns
            const int j = (nt - nt_main) * BK + lane;
            const bool ok = g_ok && j < p.lora_r;
            const uint4* s = reinterpret_cast<const uint4*>(p.lora_A + (size_t)(ok ? j : 0) * p.K + (g_ok ? kcol : 0));
#pragma unroll
            for (int i = c_lo; i < c_hi; ++i) *reinterpret_cast<uint4*>(bdst + bswz(row, wave * 8 + i)) = ok ? s[i] : zero4();
        }
    };

    // Lookup decode for matrices with 4-bit rows: one instruction stream for every width, so the
    // rows of a step (any mix of widths) do not serialise three branches.  Every code indexes its
    // codebook's fp32 levels in LDS (16 consecutive banks: conflict-free whatever the codes); the
    // level times the group's absmax is rounded to bf16 (App. A.2 as written).  A missing row has
    // zero codes and a zero absmax.
    auto load_lutregs = [&](int nt, const RowInfo& ri, LutRegs& d) {
        const int n = nt * BK + lane;
        const bool ok = g_ok && nt < nt_main && n < p.N;
        const int bits = ri.bits();
        d.bits = (uint32_t)bits;
        d.tb = per_row ? (uint32_t)TABL0 + (uint32_t)((nt & 1) * kRowTabB + lane * (kTableStride * 4))
                       : (uint32_t)TABL0 + (uint32_t)min(ri.cb(), kLutBooks - 1) * (kTableStride * 4);
        uint2 c[4] = {make_uint2(0u, 0u), make_uint2(0u, 0u), make_uint2(0u, 0u), make_uint2(0u, 0u)};
        d.scale = 0.0f;
        if (ok) {
            const uint2* cp = reinterpret_cast<const uint2*>(p.packed + ri.offset + (size_t)g * 8 * bits);
            c[0] = cp[0];
            if (bits >= 2) c[1] = cp[1];
            if (bits == 4) { c[2] = cp[2]; c[3] = cp[3]; }
            d.scale = p.absmax[(size_t)n * p.G + g];
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) { d.rc[2 * i] = c[i].x; d.rc[2 * i + 1] = c[i].y; }
    };
    // the same for a step whose 64 rows all exist: 32-bit offsets from wavefront-uniform bases, no per-lane bounds
    auto load_lutregs_full = [&](int nt, const RowInfo& ri, LutRegs& d) {
        const uint32_t n = (uint32_t)(nt * BK + lane);
        const uint32_t bits = (uint32_t)ri.bits();
        d.bits = bits;
        d.tb = per_row ? (uint32_t)TABL0 + (uint32_t)((nt & 1) * kRowTabB + lane * (kTableStride * 4))
                       : (uint32_t)TABL0 + (uint32_t)min(ri.cb(), kLutBooks - 1) * (kTableStride * 4);
        uint2 c[4] = {make_uint2(0u, 0u), make_uint2(0u, 0u), make_uint2(0u, 0u), make_uint2(0u, 0u)};
        d.scale = 0.0f;
        if (g_ok) {                                                   // uniform
            const uint8_t* cp = p.packed + (ri.offset + (uint32_t)g * 8u * bits);
            c[0] = *reinterpret_cast<const uint2*>(cp);
            if (bits >= 2u) c[1] = *reinterpret_cast<const uint2*>(cp + 8);
            if (bits == 4u) { c[2] = *reinterpret_cast<const uint2*>(cp + 16); c[3] = *reinterpret_cast<const uint2*>(cp + 24); }
            d.scale = p.absmax[n * (uint32_t)p.G + (uint32_t)g];
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) { d.rc[2 * i] = c[i].x; d.rc[2 * i + 1] = c[i].y; }
    };
    auto store_b_lut = [&](uint8_t* bdst, int c_lo, int c_hi, const LutRegs& d) {      // rows of the matrix (branch-free)
        const int row = lane;
        const bool w4 = d.bits == 4u, w2 = d.bits == 2u;
#pragma unroll
        for (int i = c_lo; i < c_hi; ++i) {
            // my 8 codes of chunk i: dword i (4-bit), half (i&1) of dword i/2 (2-bit), byte i (1-bit)
            const uint32_t c4 = d.rc[i], c2 = d.rc[i >> 1] >> (16 * (i & 1)), c1 = d.rc[i >> 2] >> (8 * (i & 3));
            const uint32_t c21 = w2 ? c2 : c1;
            const uint32_t cw = w4 ? c4 : c21;
            float w[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t idx = __builtin_amdgcn_ubfe(cw, (uint32_t)e * d.bits, d.bits);
                w[e] = *reinterpret_cast<const float*>(smem + d.tb + 4u * idx) * d.scale;
            }
            *reinterpret_cast<uint4*>(bdst + bswz(row, wave * 8 + i)) =
                make_uint4(pack_bf16x2(w[0], w[1]), pack_bf16x2(w[2], w[3]), pack_bf16x2(w[4], w[5]), pack_bf16x2(w[6], w[7]));
        }
    };
    auto store_b_lora = [&](int nt, uint8_t* bdst, int c_lo, int c_hi) {       // LoRA extension: row j of A (rank index), my 64 k columns
        const int row = lane;
        const int j = (nt - nt_main) * BK + lane;
        const bool ok = g_ok && j < p.lora_r;
        const uint4* s = reinterpret_cast<const uint4*>(p.lora_A + (size_t)(ok ? j : 0) * p.K + (g_ok ? kcol : 0));
#pragma unroll
        for (int i = c_lo; i < c_hi; ++i) *reinterpret_cast<uint4*>(bdst + bswz(row, wave * 8 + i)) = ok ? s[i] : zero4();
    };

    // ---- MFMA operand addressing
    const int wm = wave >> 1, wn = wave & 1;
    const int fi = lane & 31, fkg = lane >> 5, fsw = (fi >> 1) & 7;
    const int a_base = (wm * 128 + fi) * ROWB;
    int koff[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) koff[kk] = ((2 * kk + fkg) ^ fsw) << 4;
    // transposing reads of the weight tile: lane -> (row n_base + (L>>2), 8 bytes at k = col_base + 4 (L&3))
    int tr_off[2][4];   // [eb][tn], + kk * 16 * BROWB
    {
        const int L = lane & 15, grp = (lane >> 4) & 1;
#pragma unroll
        for (int eb = 0; eb < 2; ++eb)
#pragma unroll
            for (int tn = 0; tn < 4; ++tn) {
                const int row = fkg * 8 + eb * 4 + (L >> 2);
                const int c = wn * 16 + tn * 4 + grp * 2 + ((L & 3) >> 1);
                tr_off[eb][tn] = TILEB + bswz(row, c) + (L & 1) * 8;
            }
    }
    int b_soff[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) b_soff[i] = TILEB + bswz(lane, wave * 8 + i);

    floatx16_t acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    auto read_a = [&](const uint8_t* sbase, int kk, int t) -> bf16x8_t {
        return *reinterpret_cast<const bf16x8_t*>(sbase + a_base + t * 32 * ROWB + koff[kk]);
    };
    auto read_b_half = [&](uint32_t slds, int kk, int tn, int eb) -> v4i16_t {
        return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16_ptr)(uintptr_t)(slds + tr_off[eb][tn] + kk * 16 * BROWB));
    };
    auto join = [](v4i16_t lo, v4i16_t hi) -> bf16x8_t {
        typedef short v8i16_t __attribute__((ext_vector_type(8)));
        const v8i16_t v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        return __builtin_bit_cast(bf16x8_t, v);
    };
    auto load_frags = [&](const uint8_t* sbase, uint32_t slds, int kk, bf16x8_t (&fa)[4], bf16x8_t (&fb)[4]) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            fa[t] = read_a(sbase, kk, t);
            fb[t] = join(read_b_half(slds, kk, t, 0), read_b_half(slds, kk, t, 1));
        }
    };

    RowRegs D;          // decode inputs of step kt+1
    RowInfo R, Rcur;    // R: record of step kt+2; Rcur: record the D registers were loaded with

    // ---- fast path state (see the head of the file).  Step s: rows 64 s + lane (my row) and
    // 64 s + 16 w + lane/4 (the row whose bytes I move).  Step indices past the last full step are
    // clamped: the pipeline then fetches rows again that it never decodes.
    const int fetch_row = wave * 16 + (lane >> 2), fetch_c = lane & 3;
    const uint32_t gbyte0 = (uint32_t)k0 >> 3;                 // byte offset of the tile's first group in a 1-bit row
    const uint32_t cst_lds = smem_lds + CSTAGE0 + wave * 1024, ast_lds = smem_lds + ASTAGE0 + wave * 256;
    uint32_t SL = 0, SH = 0, x[4] = {0u, 0u, 0u, 0u}, fw = 2, MUL = 0, MASK = 0, ORC = 0;        // tables of tile kt+1
    uint32_t SLn = 0, SHn = 0, xn[4] = {0u, 0u, 0u, 0u}, fwn = 2, MULn = 0, MASKn = 0, ORCn = 0;  // ... of tile kt+2
    uint32_t rcn[4] = {0u, 0u, 0u, 0u};
    float scalen = 0.0f, lev2[4] = {0.0f, 0.0f, 0.0f, 0.0f}, lev3[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    int bits2 = 1;
    RowInfo R3, R4, R5, Rf4, Rf5;
    R3.offset = R4.offset = R5.offset = Rf4.offset = Rf5.offset = 0;
    R3.bits_cb = R4.bits_cb = R5.bits_cb = Rf4.bits_cb = Rf5.bits_cb = 1;
    bf16x8_t fa[2][4], fb[2][4];     // MFMA operands, [slice parity][tile]; slice 0 of a step is read during the step before
    auto step_c = [&](int st) { return min(st, nt_full - 1); };
    auto fetch_codes_dma = [&](int st, const RowInfo& rf) {      // codes and absmax of step st into buffer st & 1
        const uint32_t fb = (uint32_t)rf.bits();
        const uint32_t row_bytes = (uint32_t)p.K * fb >> 3;
        const uint32_t off = min(gbyte0 * fb + 16u * fetch_c, row_bytes - 16u);   // a 1-bit row has only 32 B here
        dma16_s(p.packed, rf.offset + off, cst_lds + (st & 1) * 4096);
        dma4_s(p.absmax, (uint32_t)(((size_t)step_c(st) * BK + fetch_row) * p.G + (k0 >> 6) + fetch_c) * 4u, ast_lds + (st & 1) * 1024);
    };
    auto read_staged = [&](int st, bool two_) {
        const uint8_t* cs = smem + CSTAGE0 + (st & 1) * 4096 + lane * 64 + ((two_ ? wave : wave >> 1) << 4);
        const uint4 c = *reinterpret_cast<const uint4*>(cs);
        rcn[0] = c.x; rcn[1] = c.y; rcn[2] = c.z; rcn[3] = c.w;
        scalen = *reinterpret_cast<const float*>(smem + ASTAGE0 + (st & 1) * 1024 + lane * 16 + wave * 4);
    };
    // byte tables and 16-bit code slots of the row (bits2, lev2, rcn, scalen) into the "next" set,
    // in 11 parts of about two instructions
    uint32_t tP01 = 0, tP23 = 0, tsl = 0, tsh = 0, tn0 = 0, tn1 = 0, tn2 = 0, tlo = 0, thi = 0;
    float tl[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    auto tables_part = [&](int part) {
        const bool two = bits2 == 2;
        switch (part) {
            case 0: fwn = two ? 4u : 2u; MULn = two ? 0x404101u : 0x808101u; break;
            case 1: MASKn = two ? 0x03030303u : 0x01010101u; ORCn = two ? 0x04000400u : 0x02000200u; break;
            case 2: tsl = two ? 0x06040200u : 0x03010200u; tsh = two ? 0x07050301u : 0x03010200u; break;
            case 3: tn0 = two ? 0x03020100u : 0x0c010c00u; tn1 = two ? 0x07060504u : 0x0c030c02u; break;
            case 4: tn2 = two ? 0x07060504u : 0x0c010c00u; tl[0] = lev2[0] * scalen; break;
            case 5: tl[1] = lev2[1] * scalen; tl[2] = lev2[2] * scalen; break;
            case 6: tl[3] = lev2[3] * scalen; tP01 = pack_bf16x2(tl[0], tl[1]); break;
            case 7: tP23 = pack_bf16x2(tl[2], tl[3]);
                    tlo = (!two && (wave & 1)) ? rcn[2] : rcn[0]; break;     // a 1-bit row read the 16 B of two groups
            case 8: thi = (!two && (wave & 1)) ? rcn[3] : rcn[1]; SLn = __builtin_amdgcn_perm(tP23, tP01, tsl); break;
            case 9: SHn = __builtin_amdgcn_perm(tP23, tP01, tsh); xn[0] = __builtin_amdgcn_perm(thi, tlo, tn0); break;
            case 10: xn[1] = __builtin_amdgcn_perm(thi, tlo, tn1); xn[2] = __builtin_amdgcn_perm(rcn[2], thi, tn2); break;
            default: xn[3] = __builtin_amdgcn_perm(rcn[3], thi, tn1); break;
        }
    };
    auto rotate_tables = [&]() {
        SL = SLn; SH = SHn; fw = fwn; MUL = MULn; MASK = MASKn; ORC = ORCn;
#pragma unroll
        for (int i = 0; i < 4; ++i) x[i] = xn[i];
    };

    // Fast step kt <= nt_full - 2 (tile kt+1 is a full step).  The step's ONE barrier sits at slot
    // 48 of 64, not at its end, so that nothing waits at a step boundary:
    //   slots  0..47  decode chunks 2..7 of weight tile kt+1 (tables "current"), read the staged
    //                 codes of step kt+2 (slot 20) and build its tables (slots 32..43, "next");
    //   slot   48     all transfers landed + barrier: tile kt+1 (activations and weights) is
    //                 published, stage kt&1 is free; the next tables become current;
    //   slots 48..63  read the operands of (tile kt+1, slice 0); decode chunks 0..1 of weight tile
    //                 kt+2 and start the DMA of activation tile kt+2 into stage kt&1; start the
    //                 staged code transfer of step kt+4.
    // Entry: operands of (tile kt, slice 0) in fa[0]/fb[0]; chunks 0..1 of weight tile kt+1 stored;
    // tables of tile kt+1 current; lev2/bits2 of step kt+2, its staged codes landed; R3 = record of
    // step kt+3, R4/Rf4 of step kt+4 (the pipeline advances at the barrier).  Step indices past the
    // last full step are clamped.
    auto fast_step = [&](auto PAR_, int kt) {          // PAR = kt & 1 at compile time: the stage addresses fold into offsets
        constexpr int PAR = decltype(PAR_)::value;
        const uint8_t* sbase = smem + PAR * STAGEB;
        const uint32_t slds = smem_lds + PAR * STAGEB;
        uint8_t* nbase = smem + (PAR ^ 1) * STAGEB;
        const uint32_t nlds = smem_lds + (PAR ^ 1) * STAGEB;
        v4i16_t hlo = {0, 0, 0, 0};
        uint32_t fw2 = fw * 2, fw3 = fw * 3;
        const uint8_t* dma_base = reinterpret_cast<const uint8_t*>(p.act + (size_t)m0 * p.ld_act + (size_t)step_c(kt + 2) * BK);
        const uint32_t dma_lds = slds + wave * 8192;
        const uint8_t* dma_base1 = reinterpret_cast<const uint8_t*>(p.act + (size_t)m0 * p.ld_act + (size_t)step_c(kt + 1) * BK);
        const uint32_t dma_lds1 = nlds + wave * 8192;
        const int s5 = step_c(kt + 5);
        __builtin_amdgcn_sched_barrier(0);
        uint32_t d[2][4], t = 0;
        RowInfo rf_use = Rf4;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
#pragma unroll
            for (int gslot = 0; gslot < 16; ++gslot) {
                const int tm = gslot >> 2, tn = gslot & 3;
                if (kk == 3 && gslot == 0) {
                    // everything asked for so far has landed; tile kt+1 is complete for every wavefront.
                    // (vmcnt(0) through the builtin, so that the compiler knows its own loads are done too:
                    // otherwise it waits again at the loop's end, behind the transfers issued below)
                    __builtin_amdgcn_s_waitcnt(0x0F70);
                    __syncthreads();
                    rotate_tables();
                    fw2 = fw * 2; fw3 = fw * 3;
                    // the row pipeline advances here, where every load has landed anyway (at the end of
                    // the step a register move would wait for the transfers issued after the barrier)
                    rf_use = Rf4;
#pragma unroll
                    for (int i = 0; i < 4; ++i) lev2[i] = lev3[i];
                    bits2 = R3.bits();
                    R3 = R4; R4 = R5; Rf4 = Rf5;
                    __builtin_amdgcn_sched_barrier(0);
                }
                acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[kk & 1][tm], fb[kk & 1][tn], acc[tm][tn], 0, 0, 0);
                // operands of the next slice: of this tile, or (after the barrier) slice 0 of tile kt+1
                {
                    const uint8_t* rb = kk < 3 ? sbase : nbase;
                    const uint32_t rl = kk < 3 ? slds : nlds;
                    const int nk = (kk + 1) & 3;
                    if (gslot < 4) fa[(kk + 1) & 1][gslot] = read_a(rb, nk, gslot);
                    else if (gslot < 12) {
                        const int q = (gslot - 4) >> 1;
                        if (((gslot - 4) & 1) == 0) hlo = read_b_half(rl, nk, q, 0);
                        else fb[(kk + 1) & 1][q] = join(hlo, read_b_half(rl, nk, q, 1));
                    }
                }
                {
                    // chunk i of the thread's 8: sections 0..2 decode chunks 2..7 of tile kt+1, section 3 chunks 0..1 of tile kt+2
                    const int pr = gslot >> 1, i = (kk < 3 ? 2 * kk + 2 : 0) + (pr >> 2), j = pr & 3;
                    uint8_t* wbase = kk < 3 ? nbase : const_cast<uint8_t*>(sbase);
                    if ((gslot & 1) == 0) {
                        const uint32_t off = 16u * (i & 1) + (j == 0 ? 0u : j == 1 ? fw : j == 2 ? fw2 : fw3);
                        t = __umul24(__builtin_amdgcn_ubfe(x[i >> 1], off, fw), MUL);
                    } else {
                        d[pr >> 2][j] = __builtin_amdgcn_perm(SH, SL, (t & MASK) | ORC);
                    }
                    // a chunk is stored one slot after its last pair was looked up
                    const int i0c = kk < 3 ? 2 * kk + 2 : 0;
                    if (gslot == 8) *reinterpret_cast<uint4*>(wbase + b_soff[i0c]) = make_uint4(d[0][0], d[0][1], d[0][2], d[0][3]);
                    if (gslot == 15) *reinterpret_cast<uint4*>(wbase + b_soff[i0c + 1]) = make_uint4(d[1][0], d[1][1], d[1][2], d[1][3]);
                }
                // records of step kt+5 and levels of step kt+3 first (nothing else is in flight yet)
                if (kk == 0 && gslot == 1) {
                    R5 = p.rows[s5 * BK + lane];
                    Rf5 = p.rows[s5 * BK + fetch_row];
                    // (levels 2 and 3 of a 1-bit row are never selected: no masking, so nothing here waits for the load)
                    const float4 lv = *reinterpret_cast<const float4*>(p.mappings + (size_t)R3.cb() * kTableStride);
                    lev3[0] = lv.x; lev3[1] = lv.y; lev3[2] = lv.z; lev3[3] = lv.w;
                }
                if (kk == 1 && gslot == 4) read_staged(kt + 2, bits2 == 2);
                if (kk == 2 && gslot < 12) tables_part(gslot);
                // activation tiles, one transfer every 6 slots: transfers 3..7 of tile kt+1 (its stage was
                // freed at the previous barrier) early in the step, transfers 0..2 of tile kt+2 after the
                // barrier into the stage just freed; then the staged codes and absmax of step kt+4
                if (kk < 2 && (kk * 16 + gslot) % 6 == 3 && (kk * 16 + gslot) / 6 < 5)
                    dma16_s(dma_base1, a_voff_main[3 + (kk * 16 + gslot) / 6], dma_lds1 + (3 + (kk * 16 + gslot) / 6) * 1024);
                if (kk == 3 && gslot % 6 == 1 && gslot / 6 < 3)
                    dma16_s(dma_base, a_voff_main[gslot / 6], dma_lds + (gslot / 6) * 1024);
                if (kk == 3 && gslot == 10) fetch_codes_dma(kt + 4, rf_use);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };
    // General step.
    auto slow_step = [&](int kt) {
        const uint8_t* sbase = smem + (kt & 1) * STAGEB;
        const uint32_t slds = smem_lds + (kt & 1) * STAGEB;
        uint8_t* nbase = smem + ((kt & 1) ^ 1) * STAGEB;
        const bool has_next = kt + 1 < nt_all;
        bf16x8_t fa[2][4], fb[2][4];
        load_frags(sbase, slds, 0, fa[0], fb[0]);
        const RowRegs Dc = D;
        const RowInfo Rc = Rcur;
        if (has_next) dma_act_any(kt + 1, nbase);
        if (kt + 2 < nt_all) {
            Rcur = R;
            load_rowregs(kt + 2, R, D);
            R = load_rowinfo(kt + 3);
        }
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            if (kk < 3) load_frags(sbase, slds, kk + 1, fa[(kk + 1) & 1], fb[(kk + 1) & 1]);
            if (has_next) store_b_any(kt + 1, nbase + TILEB, 2 * kk, 2 * kk + 2, Dc, Rc);
#pragma unroll
            for (int tm = 0; tm < 4; ++tm)
#pragma unroll
                for (int tn = 0; tn < 4; ++tn)
                    acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[kk & 1][tm], fb[kk & 1][tn], acc[tm][tn], 0, 0, 0);
        }
        dma_wait_all();
        __syncthreads();
    };

    // General step with the lookup decode, one body for every step so that the decode can be
    // spread over the MFMAs without a branch inside.
    LutRegs DL;
    // FULL: steps kt + 1 .. kt + 3 are steps whose 64 rows all exist (the bulk of a matrix): the transfers and loads
    // for the steps ahead then need no bounds, no branches and no per-lane 64-bit addresses.
    // PAR: kt & 1 at compile time (the stage addresses then fold into the LDS instructions' offsets), or -1.
    auto slow_step_lut = [&](auto FULL_, auto PAR_, int kt) {
        constexpr bool FULL = decltype(FULL_)::value;
        constexpr int PAR = decltype(PAR_)::value;
        const int par = PAR >= 0 ? PAR : (kt & 1);
        const uint8_t* sbase = smem + par * STAGEB;
        const uint32_t slds = smem_lds + par * STAGEB;
        uint8_t* nbase = smem + (par ^ 1) * STAGEB;
        const bool has_next = FULL || kt + 1 < nt_all;
        bf16x8_t fa[2][4], fb[2][4];
        load_frags(sbase, slds, 0, fa[0], fb[0]);
        const LutRegs Dc = DL;             // registers of step kt+1: zero codes and absmax when it holds no rows of the matrix
        if constexpr (FULL) {
            const uint16_t* base = p.act + (size_t)m0 * p.ld_act + (size_t)(kt + 1) * BK;
            const uint32_t dst = smem_lds + (par ^ 1) * STAGEB + wave * 8192;
#pragma unroll
            for (int i = 0; i < 8; ++i) dma16_s(base, a_voff_main[i], dst + i * 1024);
        } else {
            if (has_next) dma_act_any(kt + 1, nbase);
        }
        const bool stage_table = per_row && (FULL || kt + 2 < nt_all);
        if constexpr (FULL) {
            load_lutregs_full(kt + 2, R, DL);
            if (per_row) lvq = *reinterpret_cast<const float4*>(p.mappings + (size_t)R.cb() * kTableStride + 4 * wave);
            R = p.rows[(kt + 3) * BK + lane];
        } else if (kt + 2 < nt_all) {
            load_lutregs(kt + 2, R, DL);
            if (per_row) load_row_table(kt + 2, R);
            R = load_rowinfo(kt + 3);
        }
        // Slot schedule of a slice (16 MFMAs) for its two chunks of 8 weights: slots 0-3 and 4-7
        // extract the codes, form the table addresses and start the LDS reads of chunk 0 and
        // chunk 1 (two weights per slot); slots 8-11 and 12-15 multiply by the absmax, pack
        // (two weights per slot) and store the chunk -- every table read has 8 slots to land.
        const bool w4 = Dc.bits == 4u, w2 = Dc.bits == 2u;
        const uint32_t eb1 = Dc.bits, eb2 = 2u * Dc.bits, eb3 = 3u * Dc.bits, eb4 = 4u * Dc.bits, eb5 = 5u * Dc.bits,
                       eb6 = 6u * Dc.bits, eb7 = 7u * Dc.bits;
        const uint32_t r0 = Dc.rc[0], r1 = Dc.rc[1], r2 = Dc.rc[2], r3 = Dc.rc[3], r4 = Dc.rc[4], r5 = Dc.rc[5], r6 = Dc.rc[6], r7 = Dc.rc[7];
        const uint32_t tbl = Dc.tb, wbits = Dc.bits;
        const float ascale = Dc.scale;
        uint32_t cw0 = 0, cw1 = 0, pk0 = 0, pk1 = 0, pk2 = 0;
        float v0 = 0, v1 = 0, v2 = 0, v3 = 0, v4 = 0, v5 = 0, v6 = 0, v7 = 0, u0 = 0, u1 = 0, u2 = 0, u3 = 0, u4 = 0, u5 = 0, u6 = 0, u7 = 0;
        auto code_word = [&](auto I_) __attribute__((always_inline)) -> uint32_t {           // chunk i: dword i (4-bit), half (i&1) of dword i/2 (2-bit), byte i (1-bit)
            constexpr int i = decltype(I_)::value;
            const uint32_t q4 = i == 0 ? r0 : i == 1 ? r1 : i == 2 ? r2 : i == 3 ? r3 : i == 4 ? r4 : i == 5 ? r5 : i == 6 ? r6 : r7;
            const uint32_t q2 = ((i >> 1) == 0 ? r0 : (i >> 1) == 1 ? r1 : (i >> 1) == 2 ? r2 : r3) >> (16 * (i & 1));
            const uint32_t q1 = ((i >> 2) == 0 ? r0 : r1) >> (8 * (i & 3));
            const uint32_t q21 = w2 ? q2 : q1;
            return w4 ? q4 : q21;
        };
        auto look = [&](uint32_t cw, uint32_t ofs) __attribute__((always_inline)) -> float {
            return *reinterpret_cast<const float*>(smem + tbl + 4u * __builtin_amdgcn_ubfe(cw, ofs, wbits));
        };
        auto slot = [&](auto KK_, auto SL_) __attribute__((always_inline)) {
            constexpr int kk = decltype(KK_)::value, sl = decltype(SL_)::value, tm = sl >> 2, tn = sl & 3;
            acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[kk & 1][tm], fb[kk & 1][tn], acc[tm][tn], 0, 0, 0);
            if constexpr (sl == 0) { v0 = look(cw0, 0u); v1 = look(cw0, eb1); }
            if constexpr (sl == 1) { v2 = look(cw0, eb2); v3 = look(cw0, eb3); }
            if constexpr (sl == 2) { v4 = look(cw0, eb4); v5 = look(cw0, eb5); }
            if constexpr (sl == 3) { v6 = look(cw0, eb6); v7 = look(cw0, eb7); }
            if constexpr (sl == 4) { u0 = look(cw1, 0u); u1 = look(cw1, eb1); }
            if constexpr (sl == 5) { u2 = look(cw1, eb2); u3 = look(cw1, eb3); }
            if constexpr (sl == 6) { u4 = look(cw1, eb4); u5 = look(cw1, eb5); }
            if constexpr (sl == 7) { u6 = look(cw1, eb6); u7 = look(cw1, eb7); }
            if constexpr (sl == 8) pk0 = pack_bf16x2(v0 * ascale, v1 * ascale);
            if constexpr (sl == 9) pk1 = pack_bf16x2(v2 * ascale, v3 * ascale);
            if constexpr (sl == 10) pk2 = pack_bf16x2(v4 * ascale, v5 * ascale);
            if constexpr (sl == 11)
                *reinterpret_cast<uint4*>(nbase + b_soff[2 * kk]) =
                    make_uint4(pk0, pk1, pk2, pack_bf16x2(v6 * ascale, v7 * ascale));
            if constexpr (sl == 12) pk0 = pack_bf16x2(u0 * ascale, u1 * ascale);
            if constexpr (sl == 13) pk1 = pack_bf16x2(u2 * ascale, u3 * ascale);
            if constexpr (sl == 14) pk2 = pack_bf16x2(u4 * ascale, u5 * ascale);
            if constexpr (sl == 15)
                *reinterpret_cast<uint4*>(nbase + b_soff[2 * kk + 1]) =
                    make_uint4(pk0, pk1, pk2, pack_bf16x2(u6 * ascale, u7 * ascale));
            __builtin_amdgcn_sched_barrier(0);
        };
        auto slice = [&](auto KK_) __attribute__((always_inline)) {
            constexpr int kk = decltype(KK_)::value;
            if (kk < 3) load_frags(sbase, slds, kk + 1, fa[(kk + 1) & 1], fb[(kk + 1) & 1]);
            cw0 = code_word(std::integral_constant<int, 2 * kk>{});
            cw1 = code_word(std::integral_constant<int, 2 * kk + 1>{});
            __builtin_amdgcn_sched_barrier(0);
            slot(KK_, std::integral_constant<int, 0>{}); slot(KK_, std::integral_constant<int, 1>{});
            slot(KK_, std::integral_constant<int, 2>{}); slot(KK_, std::integral_constant<int, 3>{});
            slot(KK_, std::integral_constant<int, 4>{}); slot(KK_, std::integral_constant<int, 5>{});
            slot(KK_, std::integral_constant<int, 6>{}); slot(KK_, std::integral_constant<int, 7>{});
            slot(KK_, std::integral_constant<int, 8>{}); slot(KK_, std::integral_constant<int, 9>{});
            slot(KK_, std::integral_constant<int, 10>{}); slot(KK_, std::integral_constant<int, 11>{});
            slot(KK_, std::integral_constant<int, 12>{}); slot(KK_, std::integral_constant<int, 13>{});
            slot(KK_, std::integral_constant<int, 14>{}); slot(KK_, std::integral_constant<int, 15>{});
        };
        slice(std::integral_constant<int, 0>{}); slice(std::integral_constant<int, 1>{});
        slice(std::integral_constant<int, 2>{}); slice(std::integral_constant<int, 3>{});
        // a LoRA step (rows of A) overwrites the zeros the decode stored; past the last step the
        // zeros land in a stage nobody reads again
        if (!FULL && has_next && kt + 1 >= nt_main) store_b_lora(kt + 1, nbase + TILEB, 0, 8);
        // the table buffer of step kt + 2 was last read by the decode of step kt, one barrier ago
        if (stage_table) store_row_table(kt + 2);
        dma_wait_all();
        __syncthreads();
    };

    // ---- matrices with 4-bit rows: every step is a general step with the lookup decode
    if constexpr (LUT) {
        dma_act_any(0, smem);
        Rcur = load_rowinfo(0);
        load_lutregs(0, Rcur, DL);
        if (per_row) {                            // step 0's tables are needed right away
            load_row_table(0, Rcur);
            store_row_table(0);
            __syncthreads();
        }
        R = load_rowinfo(1);
        store_b_lut(smem + TILEB, 0, 8, DL);      // N >= 1: step 0 holds rows of the matrix
        if (nt_all > 1) {
            load_lutregs(1, R, DL);
            if (per_row) { load_row_table(1, R); store_row_table(1); }
            R = load_rowinfo(2);
        }
        dma_wait_all();
        __syncthreads();
        int kt = 0;
        for (; kt + 4 < nt_full; kt += 2) {                        // kt is even here
            slow_step_lut(std::true_type{}, std::integral_constant<int, 0>{}, kt);
            slow_step_lut(std::true_type{}, std::integral_constant<int, 1>{}, kt + 1);
        }
        for (; kt < nt_all; ++kt) slow_step_lut(std::false_type{}, std::integral_constant<int, -1>{}, kt);
        if (nsplit > 1) store_out_f32(acc, p.split_out + ((size_t)split * (ntiles - p.split_first) + (tile - p.split_first)) * (BM * BN), BN, BM, BN, 0, 0);
        else store_out(acc, p.out, p.K, p.M, p.K, m0, k0);
        return;
    }

    // ---- prologue: step 0 into stage 0; registers of step 1; record of step 2
    dma_act_any(0, smem);
    Rcur = load_rowinfo(0);
    load_rowregs(0, Rcur, D);
    R = load_rowinfo(1);
    store_b_any(0, smem + TILEB, 0, 8, D, Rcur);
    if (nt_all > 1) {
        Rcur = R;
        load_rowregs(1, R, D);
        R = load_rowinfo(2);
    }
    dma_wait_all();
    __syncthreads();

    int kt = 0;
    if (!p.any4 && (p.K & 255) == 0 && nt_full >= 8) {
        // fill the fast pipeline with plain loads (tile 0 is complete in stage 0 already)
        {
            RowRegs D1;
            const RowInfo r1 = p.rows[BK + lane];
            load_rowregs_fast(1, r1, D1);
            // chunks 0..1 of weight tile 1, and its tables as the current set
            store_b_any(1, smem + STAGEB + TILEB, 0, 2, D1, r1);
            bits2 = D1.bits; scalen = D1.scale;
#pragma unroll
            for (int i = 0; i < 4; ++i) { lev2[i] = D1.lev[i]; rcn[i] = D1.rc[i]; }
            for (int part = 0; part < 12; ++part) tables_part(part);    // (wave & 1 picks either copy of a 1-bit row's 8 bytes)
            rotate_tables();
            // activation tile 1
            {
                const uint8_t* base = reinterpret_cast<const uint8_t*>(p.act + (size_t)m0 * p.ld_act + (size_t)BK);
#pragma unroll
                for (int i = 0; i < 8; ++i) dma16_s(base, a_voff_main[i], smem_lds + STAGEB + wave * 8192 + i * 1024);
            }
            // step 2: levels, width, staged codes; step 3: staged codes, record; step 4: records
            const RowInfo r2 = p.rows[2 * BK + lane];
            const float4 lv = *reinterpret_cast<const float4*>(p.mappings + (size_t)r2.cb() * kTableStride);
            bits2 = r2.bits();
            lev2[0] = lv.x; lev2[1] = lv.y; lev2[2] = lv.z; lev2[3] = lv.w;
            fetch_codes_dma(2, p.rows[2 * BK + fetch_row]);
            fetch_codes_dma(3, p.rows[3 * BK + fetch_row]);
            R3 = p.rows[3 * BK + lane];
            R4 = p.rows[step_c(4) * BK + lane];
            Rf4 = p.rows[step_c(4) * BK + fetch_row];
            dma_wait_all();
            __builtin_amdgcn_s_waitcnt(0x0F70);
            __syncthreads();
            load_frags(smem, smem_lds, 0, fa[0], fb[0]);
        }
        for (; kt + 2 <= nt_full - 1; kt += 2) {          // kt is even here
            fast_step(std::integral_constant<int, 0>{}, kt);
            fast_step(std::integral_constant<int, 1>{}, kt + 1);
        }
        if (kt < nt_full - 1) { fast_step(std::integral_constant<int, 0>{}, kt); ++kt; }
        // hand over to the general steps: everything in flight lands, their registers of step kt+1, record of step kt+2
        dma_wait_all();
        __syncthreads();
        if (kt + 1 < nt_all) {
            Rcur = load_rowinfo(kt + 1);
            load_rowregs(kt + 1, Rcur, D);
            R = load_rowinfo(kt + 2);
        }
    }
    for (; kt < nt_all; ++kt) slow_step(kt);

    if (nsplit > 1) store_out_f32(acc, p.split_out + ((size_t)split * (ntiles - p.split_first) + (tile - p.split_first)) * (BM * BN), BN, BM, BN, 0, 0);
        else store_out(acc, p.out, p.K, p.M, p.K, m0, k0);
}

// dX tile = bf16(sum of its splits' partial tiles, in split order): eight workgroups per split tile, 8 outputs per thread
__global__ __launch_bounds__(256) void split_sum_kernel(const float* __restrict__ part, int splits, int ntail, int first_tile,
                                                        int tiles_k, int M, int K, uint16_t* __restrict__ out) {
    constexpr int PIECES = 8;                                      // workgroups per tile: 32 rows each
    const int tt = blockIdx.x / PIECES, piece = blockIdx.x % PIECES;
    const int tile = first_tile + tt;
    const int k0 = (tile % tiles_k) * BN, m0 = (tile / tiles_k) * BM;
    for (int o = piece * (BM * BN / 8 / PIECES) + threadIdx.x; o < (piece + 1) * (BM * BN / 8 / PIECES); o += 256) {
        const int r = o / (BN / 8), c = (o % (BN / 8)) * 8;
        if (m0 + r >= M || k0 + c >= K) continue;                  // K is a multiple of 64: eight columns are in or out together
        float4 a = make_float4(0.0f, 0.0f, 0.0f, 0.0f), b = a;
        for (int s = 0; s < splits; ++s) {
            const float4* src = reinterpret_cast<const float4*>(part + ((size_t)s * ntail + tt) * (BM * BN) + (size_t)r * BN + c);
            const float4 u = src[0], v = src[1];
            a.x += u.x; a.y += u.y; a.z += u.z; a.w += u.w; b.x += v.x; b.y += v.y; b.z += v.z; b.w += v.w;
        }
        *reinterpret_cast<uint4*>(out + (size_t)(m0 + r) * K + k0 + c) =
            make_uint4(pack_bf16x2(a.x, a.y), pack_bf16x2(a.z, a.w), pack_bf16x2(b.x, b.y), pack_bf16x2(b.z, b.w));
    }
}

hipError_t launch_gemm_bwd(const GemmParams& p, hipStream_t st) {
    static const hipError_t attr0 = hipFuncSetAttribute(reinterpret_cast<const void*>(linear_bwd_kernel<false>),
                                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)kBwdSmem);
    static const hipError_t attr1 = hipFuncSetAttribute(reinterpret_cast<const void*>(linear_bwd_kernel<true>),
                                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)kBwdSmem);
    if (attr0 != hipSuccess) return attr0;
    if (attr1 != hipSuccess) return attr1;
    const int tiles_k = (p.K + BN - 1) / BN, ntiles = tiles_k * ((p.M + BM - 1) / BM);
    const int ntail = p.splits > 1 ? ntiles - p.split_first : 0;
    const dim3 grid(p.splits > 1 ? p.split_first + ntail * p.splits : ntiles);
    if (p.any4)
        linear_bwd_kernel<true><<<grid, dim3(NTHREADS), kBwdSmem, st>>>(p);
    else
        linear_bwd_kernel<false><<<grid, dim3(NTHREADS), kBwdSmem, st>>>(p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || p.splits <= 1) return e;
    split_sum_kernel<<<dim3(ntail * 8), dim3(256), 0, st>>>(p.split_out, p.splits, ntail, p.split_first, tiles_k, p.M, p.K, p.out);
    return hipGetLastError();
}

// Which output tiles of the input gradient share their contraction, and between how many workgroups: the tiles of the
// last round of workgroups when that round would fill at most half of the compute units (all tiles when there is
// only such a round), between as many workgroups as fill them, at most 4, each with at least 8 contraction steps.
BwdSplitPlan gemm_bwd_split_plan(int N, int K, int M) {
    const int tiles = ((K + BN - 1) / BN) * ((M + BM - 1) / BM), cus = device_compute_units();
    const int steps = (N + BK - 1) / BK;
    BwdSplitPlan pl{1, 0, tiles, 0};
    const int tail = tiles % cus;
    if (tail == 0 || 2 * tail > cus) return pl;
    const int s = std::min(std::min(4, cus / tail), steps / 8);
    if (s < 2) return pl;
    pl.splits = s;
    pl.rows_per_split = (steps + s - 1) / s * BK;
    pl.first = tiles - tail;
    pl.tail = tail;
    return pl;
}

}  // namespace lowra
