// Forward fused dequant-GEMM:  y = [x | s x A^T] [What | B]^T   (Sec. 2.1 LoRA form; App. A.2 decode)
//
// 256 x 256 outputs per workgroup; wavefront w owns 64 output channels x all 256 token rows
// (2 x 8 tiles of v_mfma_f32_32x32x16_bf16, weights as the A operand, activations as the B
// operand).  One contraction step is one 64-wide absmax group.
//
// The dequantized weights never touch LDS.  An MFMA lane (row i, k-half h) needs, per 16-deep MFMA
// slice, the 8 consecutive weights W[i][16 kk + 8 h ..] of its own row: exactly one byte (1-bit
// rows) or two bytes (2-bit rows) of the packed stream.  Each lane therefore decodes the operand
// registers of its two rows itself, one slice ahead of the MFMAs that consume them, two plain
// ALU instructions per MFMA slot.  Only the activations are staged: 4 LDS stages of 256 rows x
// 64 bf16, filled by global->LDS DMA three steps ahead, one barrier per 64 MFMAs.
//
// 1- and 2-bit rows decode without table memory and with one instruction stream for both widths:
// the row's 2 or 4 levels times the group absmax are rounded to bf16 once per group (the multiply
// and rounding of App. A.2 on 2^b values instead of 64 weights), their low and high bytes form the
// 8-byte source of v_perm_b32, and a pair of codes becomes the 4-byte selector with one bit-field
// extract, one 24-bit multiply that spreads the bits, and one and-or.  Width only changes per-lane
// constants.  The codes and absmax of a group travel global -> LDS -> registers three steps ahead.
// Wavefronts that hold a 4-bit row, contractions whose group count is odd or not a multiple of
// four (their last steps) and the LoRA extension take a general step with the same barrier protocol.
#include <algorithm>
#include <type_traits>

#include "gemm_common.h"

namespace lowra {

// ---- the schedule of global -> LDS transfers inside one 64-slot weight step, shared by the two instruction
// streams (fast and lookup): which slots issue one.  The step's closing wait counts them.
constexpr bool slot_issues_activation(int S, int TM) { return S % 6 == 1 && S / 6 < TM; }   // activation tile j + 3: TM transfers per wavefront
constexpr int slot_requests_codes(int S) { return S == 56 ? 0 : S == 58 ? 1 : -1; }   // row 0 / row 1 of group j + 3 (slots without an LDS read)
constexpr int slot_requests_scale(int S) { return S == 60 ? 0 : S == 62 ? 1 : -1; }
// The fast path reads the landed codes of group j + 1 back at these slots and then builds its tables in twelve
// one-instruction pieces per row, spread over slots that carry little else (a wavefront alone on its SIMD hides about
// four plain-ALU instructions behind an MFMA, no more): slot -> piece of row 0 / row 1, -1: none.  All pieces are
// done before slot 48, where the decode turns to the next group.
constexpr int kFetchSlot[2] = {8, 10};
constexpr int kTablePieceSlot[2][12] = {{12, 14, 15, 16, 17, 18, 21, 22, 23, 24, 26, 27},
                                        {28, 29, 30, 32, 33, 34, 40, 41, 42, 44, 45, 46}};
constexpr int slot_table_piece(int S, int R) {
    for (int q = 0; q < 12; ++q) if (kTablePieceSlot[R][q] == S) return q;
    return -1;
}
constexpr int step_transfers(int TM) {
    int n = 0;
    for (int S = 0; S < 64; ++S) n += (slot_issues_activation(S, TM) ? 1 : 0) + (slot_requests_codes(S) >= 0 ? 1 : 0) + (slot_requests_scale(S) >= 0 ? 1 : 0);
    return n;
}
static_assert(step_transfers(8) == 8 + 2 + 2 && step_transfers(6) == 6 + 2 + 2 && step_transfers(4) == 4 + 2 + 2,
              "a step refills one activation tile (TM transfers per wavefront) and asks for two rows of codes and scales");
static_assert(step_transfers(8) < 64, "s_waitcnt vmcnt holds 6 bits");
// The 64 slots of a step carry 8 TM MFMAs: 2 TM per 16-slot section (one 16-deep slice), every slot at TM = 8, three of
// four at TM = 6, every other one at TM = 4.  Slot s of a section -> index of its MFMA in the slice, or -1.
constexpr int slot_mfma(int s, int TM) {
    return TM == 8 ? s : TM == 6 ? (s % 4 == 3 ? -1 : s - s / 4) : TM == 4 ? (s % 2 ? -1 : s / 2) : -1;
}

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

#ifndef LOWRA_FWD_COST6
#define LOWRA_FWD_COST6 0.80
#endif
#ifndef LOWRA_FWD_COST4
#define LOWRA_FWD_COST4 0.62
#endif

constexpr int KS = 64;                     // contraction depth per step: one absmax group
constexpr int AROWB = 128;                 // bytes per LDS activation row: 64 bf16 = 8 chunks of 16 B
constexpr int ASTAGEB = 256 * AROWB;       // 32 KB per stage
constexpr int NSTAGE = 4;
constexpr int CBUFB = 4 * 2 * 1024;        // one code buffer: 4 wavefronts x 2 rows x 64 lanes x 16 B
constexpr int SBUFB = 4 * 2 * 256;         // one absmax buffer: 4 wavefronts x 2 rows x 64 lanes x 4 B
constexpr int CBUF0 = NSTAGE * ASTAGEB, SBUF0 = CBUF0 + 2 * CBUFB;
constexpr int EPI_LD = 512;                // bytes per staged output row; 16-byte chunk c of row r sits at chunk c ^ (r & 31)
constexpr int kLutBooks = 64;              // codebooks the lookup path keeps in LDS (16 fp32 levels each)
constexpr int TAB0 = SBUF0 + 2 * SBUFB;
constexpr size_t kFwdSmem = 159 * 1024;    // nearly all of it (the workgroup vote takes a few bytes of its own): what follows TAB0 holds the lookup path's tables
constexpr int kRowTabBudget = (int)kFwdSmem - TAB0 - 16;   // with more codebooks than kLutBooks: per-row tables of the tile (the last 16 bytes: the wavefronts' sizes)
static_assert(kLutBooks * kTableStride * 4 <= kRowTabBudget, "either table scheme fits the region");
static_assert(256 * EPI_LD <= (int)kFwdSmem, "the output tile is staged in the same LDS");

template <int V> using int_c = std::integral_constant<int, V>;

// Pair q (0..31) of a step's decode stream: section q>>3 of the step builds the operands of MFMA
// slice (q>>3)+1 (slice 4 = slice 0 of the next step); 4 pairs per row, row 0 first.  q = -1 is
// the last pair of the previous step's stream: it belongs to this step's slice 0.
struct PairInfo { int row, jp, buf, xreg, half, next_set; };
__host__ __device__ constexpr PairInfo pair_info(int q) {
    if (q < 0) return PairInfo{1, 3, 0, 0, 0, 0};
    const int tkk = (q >> 3) + 1;
    return PairInfo{(q >> 2) & 1, q & 3, tkk & 1, (tkk & 3) >> 1, tkk & 1, tkk == 4 ? 1 : 0};
}

// One output tile: channels [n0, n0 + 256) x token rows [m0, m0 + 32 TM).
template <int TM>
__device__ __forceinline__ void fwd_tile(const GemmParams& p, const int n0, const int m0, uint8_t* smem) {
    static_assert(TM == 8 || TM == 6 || TM == 4, "token tiles of 256, 192 or 128 rows");
    constexpr int kStepTransfers = step_transfers(TM);
    constexpr int WROWS = 8 * TM;            // token rows a wavefront moves per activation tile (8 per transfer)
    const uint32_t smem_lds = (uint32_t)(uintptr_t)(lptr_t)smem;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform, and known to be
    const int fi = lane & 31, fkg = lane >> 5;
    const int G = p.G;

    // ---- activation tile: global -> LDS DMA, 8 rows x 128 B per instruction, wavefront w owns rows
    // [64 w, 64 w + 64).  LDS is filled linearly, so the chunk swizzle is applied to the global
    // address: the lane landing on physical chunk l&7 of row r fetches logical chunk (l&7)^((r>>1)&7).
    const int m_last = p.M - 1 - m0;
    auto a_voff_of = [&](int i, int ld_elems) -> uint32_t {
        const int r = wave * WROWS + 8 * i + (lane >> 3);
        const int rcl = r < m_last ? r : m_last;              // rows past M are clamped (never stored back)
        return (uint32_t)rcl * (uint32_t)ld_elems * 2u + (uint32_t)(((lane & 7) ^ ((r >> 1) & 7)) << 4);
    };
    uint32_t a_voff[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) a_voff[i] = a_voff_of(i, p.K);
    const uint16_t* act0 = p.act + (size_t)m0 * p.K;
    auto dma_act = [&](int jt, int stage) {
        const uint32_t dst = smem_lds + stage * ASTAGEB + wave * (WROWS * AROWB);
        const uint16_t* base = act0 + (size_t)jt * KS;
#pragma unroll
        for (int i = 0; i < TM; ++i) dma16_s(base, a_voff[i], dst + i * 1024);
    };

    // the first three activation tiles start before anything else: their latency hides the
    // dependent loads of the row records below
    dma_act(0, 0);
    dma_act(min(1, G - 1), 1);
    dma_act(min(2, G - 1), 2);

    // ---- my two weight rows: positions 64 w + 32 R + fi of the tile's row order.  With a handful
    // of shared codebooks the levels are fetched before the row records arrive and picked afterwards,
    // which takes one global round trip out of the prologue.
    constexpr int kFewBooks = 4;
    float4 book[kFewBooks];
    const bool few = p.C <= kFewBooks;
#pragma unroll
    for (int c = 0; c < kFewBooks; ++c)
        book[c] = *reinterpret_cast<const float4*>(p.mappings + (size_t)(c < p.C ? c : 0) * kTableStride);
    // all codebooks into LDS for the lookup path (visible after the prologue's barriers)
    if (p.C <= kLutBooks)
        for (int e = tid; e < p.C * kTableStride; e += NTHREADS) reinterpret_cast<float*>(smem + TAB0)[e] = p.mappings[e];
    SortedRow rec[2];
#pragma unroll
    for (int R = 0; R < 2; ++R) rec[R] = p.gemm_rows[n0 + wave * 64 + R * 32 + fi];
    int lr[2], nrow[2], bits[2];
    bool row_ok[2], two[2];
    uint32_t rowoff[2], amoff[2];
    float lev[2][4];
    uint32_t MUL[2], MASK[2], ORC[2], fwid[2], selL[2], selH[2], selX[2], boff[2][2][4];
#pragma unroll
    for (int R = 0; R < 2; ++R) {
        row_ok[R] = rec[R].n >= 0;
        lr[R] = row_ok[R] ? rec[R].n - n0 : rec[R].pad;
        nrow[R] = row_ok[R] ? rec[R].n : p.N - 1;           // clamped: loads stay in bounds, levels are zeroed
        bits[R] = (int)(rec[R].bits_cb & 0xffu);
        const int cbi = (int)(rec[R].bits_cb >> 8);
        rowoff[R] = rec[R].offset;                           // a padding entry points at row 0 as a 1-bit row: in bounds
        amoff[R] = (uint32_t)nrow[R] * (uint32_t)G * 4u;
        float4 lv4;
        if (few) {
            lv4 = book[0];
#pragma unroll
            for (int c = 1; c < kFewBooks; ++c) if (cbi == c) lv4 = book[c];
        } else {
            lv4 = *reinterpret_cast<const float4*>(p.mappings + (size_t)cbi * kTableStride);
        }
        const float lvv[4] = {lv4.x, lv4.y, lv4.z, lv4.w};
#pragma unroll
        for (int q = 0; q < 4; ++q) lev[R][q] = (row_ok[R] && q < (1 << bits[R])) ? lvv[q] : 0.0f;
        // per-lane constants of the unified 1-/2-bit decode
        two[R] = bits[R] == 2;
        fwid[R] = two[R] ? 4u : 2u;                           // bits per pair of codes
        MUL[R] = two[R] ? 0x404101u : 0x808101u;              // spreads the pair's bits to byte lanes
        MASK[R] = two[R] ? 0x03030303u : 0x01010101u;
        ORC[R] = two[R] ? 0x04000400u : 0x02000200u;          // high-byte entries sit after the low-byte ones
        selL[R] = two[R] ? 0x06040200u : 0x03010200u;
        selH[R] = two[R] ? 0x07050301u : 0x03010200u;
        // my 8 codes of slice kk are byte 2 kk + h of a 1-bit group, half-word h of dword kk of a
        // 2-bit group; they are gathered as one 16-bit slot per slice, two slices per register
        selX[R] = two[R] ? (fkg ? 0x07060302u : 0x05040100u) : (fkg ? 0x0c030c01u : 0x0c020c00u);
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int jq = 0; jq < 4; ++jq) boff[R][h][jq] = 16u * h + jq * fwid[R];
    }
    // per-lane constants of the lookup path (any width).  Its wavefronts contract a step in the
    // order k = 32 h + 8 kk + e (h = my k-half, kk = slice): my 32 codes of a group are then one
    // contiguous run -- 16 bytes of a 4-bit row, dwords 2h, 2h+1 of a 2-bit group, dword h of a
    // 1-bit group -- and the activations are read with the same permutation.
    bool one[2], four[2];
    uint32_t rq_shift[2], rq_mul[2], rq_add[2];           // the codes' request: byte offset = ((group >> shift) * mul) + add
    uint32_t ibv[2][8], bwv[2], tbase[2], shv[2][4];
#pragma unroll
    for (int R = 0; R < 2; ++R) {
        one[R] = bits[R] == 1; four[R] = bits[R] == 4;
        rq_shift[R] = one[R] ? 1u : 0u;
        rq_mul[R] = four[R] ? 32u : 16u;
        rq_add[R] = rowoff[R] + (four[R] ? 16u * (uint32_t)fkg : 0u);
        bwv[R] = (uint32_t)bits[R];
#pragma unroll
        for (int i = 0; i < 8; ++i) ibv[R][i] = (uint32_t)(i * bits[R]);        // bit offset of code i in a slice's code word
        tbase[R] = (uint32_t)TAB0 + (uint32_t)min((int)(rec[R].bits_cb >> 8), kLutBooks - 1) * (kTableStride * 4);   // (more codebooks: set below)
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) shv[R][kk] = four[R] ? 0u : (two[R] ? 16u * (kk & 1) : 8u * kk);   // the word's shift in its dword
    }
    int kofl[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) kofl[kk] = fi * AROWB + (((4 * fkg + kk) ^ ((fi >> 1) & 7)) << 4);
    const bool wave_has4 = __builtin_amdgcn_ballot_w64(bits[0] == 4 || bits[1] == 4) != 0;
    // More codebooks than the shared table region holds (the paper's own data model: one table set per output
    // channel, Sec. 4.1): a wavefront that needs the lookup path keeps the tables of ITS 64 rows in LDS, 64 bytes
    // for a 4-bit row and 16 for a narrower one, packed in row order behind those of the wavefronts before it.
    // A wavefront whose tables do not fit any more (a tile with more than about 70 % 4-bit rows) takes the general step.
    const bool per_row = p.C > kLutBooks;
    bool row_tables_fit = true;
    if (per_row) {
        const uint64_t low = 0xffffffffull;
        const uint64_t b0 = __builtin_amdgcn_ballot_w64(bits[0] == 4) & low, b1 = __builtin_amdgcn_ballot_w64(bits[1] == 4) & low;
        const int n4 = __builtin_popcountll(b0) + __builtin_popcountll(b1);
        const int my_size = wave_has4 ? n4 * 64 + (64 - n4) * 16 : 0;
        int* sizes = reinterpret_cast<int*>(smem + TAB0 + kRowTabBudget);
        if (lane == 0) sizes[wave] = my_size;
        __syncthreads();
        int base = 0;
        for (int w = 0; w < wave; ++w) base += sizes[w];
        row_tables_fit = base + my_size <= kRowTabBudget;
        if (wave_has4 && row_tables_fit) {
            const uint64_t below = (1ull << fi) - 1ull;
#pragma unroll
            for (int R = 0; R < 2; ++R) {
                const int before4 = (R ? __builtin_popcountll(b0) : 0) + __builtin_popcountll((R ? b1 : b0) & below);
                const int before = 32 * R + fi;
                const uint32_t off = (uint32_t)(base + before4 * 64 + (before - before4) * 16);
                tbase[R] = (uint32_t)TAB0 + off;
                if (fkg == 0) {                               // one lane per row writes its levels
                    const float4* src = reinterpret_cast<const float4*>(p.mappings + (size_t)(rec[R].bits_cb >> 8) * kTableStride);
                    float4* dst = reinterpret_cast<float4*>(smem + TAB0 + off);
                    dst[0] = src[0];
                    if (bits[R] == 4) { dst[1] = src[1]; dst[2] = src[2]; dst[3] = src[3]; }
                }
            }
        }
    }
    const bool natural = __syncthreads_and(lr[0] == wave * 64 + fi && lr[1] == wave * 64 + 32 + fi) != 0;
    const bool pipe_ok = (G & 1) == 0 && G >= 4;
    const bool wave_fast = pipe_ok && !wave_has4;
    const bool wave_lut = pipe_ok && wave_has4 && row_tables_fit;

    // ---- MFMA operand addressing: lane (fi, fkg) reads 8 bf16 of token row 32 tm + fi
    int kofs[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) kofs[kk] = fi * AROWB + (((2 * kk + fkg) ^ ((fi >> 1) & 7)) << 4);

    floatx16_t acc[2][TM];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int jt = 0; jt < TM; ++jt)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][jt][v] = 0.0f;

    bf16x8_t fact[2][TM];             // activation operands, [slice parity][token tile]
    uint32_t fwd[2][2][4];            // weight operands,     [slice parity][row][pair]
#pragma unroll
    for (int i = 0; i < 16; ++i) (&fwd[0][0][0])[i] = 0u;
    auto wfrag = [&](int buf, int R) -> bf16x8_t {
        const u32x4_t v = {fwd[buf][R][0], fwd[buf][R][1], fwd[buf][R][2], fwd[buf][R][3]};
        return __builtin_bit_cast(bf16x8_t, v);
    };
    auto load_fact = [&](int stage, int kk, bf16x8_t (&f)[TM]) {
        const uint8_t* sbase = smem + stage * ASTAGEB + kofs[kk];
#pragma unroll
        for (int t = 0; t < TM; ++t) f[t] = *reinterpret_cast<const bf16x8_t*>(sbase + t * 32 * AROWB);
    };
    auto mma16 = [&](const bf16x8_t& w0, const bf16x8_t& w1, const bf16x8_t (&f)[TM]) {
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) acc[0][tm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w0, f[tm], acc[0][tm], 0, 0, 0);
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) acc[1][tm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w1, f[tm], acc[1][tm], 0, 0, 0);
    };

    // General step j (branches allowed): same barrier protocol as the fast step, nothing prefetched.
    auto slow_step = [&](int js) {
        if (js + 3 < G) dma_act(js + 3, (js + 3) & 3);
        float a[2];
        const uint8_t* cp[2];
        const float* tab[2];
#pragma unroll
        for (int R = 0; R < 2; ++R) {
            a[R] = row_ok[R] ? p.absmax[(size_t)nrow[R] * G + js] : 0.0f;
            cp[R] = p.packed + rowoff[R] + (size_t)js * (8 * bits[R]);
            tab[R] = p.mappings + (size_t)p.rows[nrow[R]].cb() * kTableStride;
        }
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            load_fact(js & 3, kk, fact[0]);
            bf16x8_t w[2];
#pragma unroll
            for (int R = 0; R < 2; ++R)
                w[R] = __builtin_bit_cast(bf16x8_t, decode8_bf16(load_codes8(cp[R], 2 * kk + fkg, bits[R]), bits[R], tab[R], a[R]));
            mma16(w[0], w[1], fact[0]);
        }
        dma_wait_all();
        __syncthreads();
    };

    // ---- fast path state.  Two table sets: group g uses set g & 1, so the set of the next group
    // is built while the current one is still in use.  The codes (16 B per row: a whole 2-bit
    // group, or the aligned pair of 1-bit groups that holds the wanted one) and the absmax of a
    // future group travel global -> LDS by DMA and are read back by the lane that asked for
    // them: the compiler never has a register load of its own outstanding next to the untracked
    // DMAs (it would wait for ALL of them before the first use).  Both lanes of a row fetch alike.
    uint32_t rc[2][4] = {{0u, 0u, 0u, 0u}, {0u, 0u, 0u, 0u}};
    float rscale[2] = {0.0f, 0.0f};
    uint32_t SL[2][2] = {{0u, 0u}, {0u, 0u}}, SH[2][2] = {{0u, 0u}, {0u, 0u}};   // [set][row]
    uint32_t x[2][2][2] = {{{0u, 0u}, {0u, 0u}}, {{0u, 0u}, {0u, 0u}}};          // [set][row][slices 0-1 | 2-3]
    const uint32_t cb_lds = smem_lds + CBUF0 + wave * 2048, sb_lds = smem_lds + SBUF0 + wave * 512;
    const uint8_t* cb_mine = smem + CBUF0 + wave * 2048 + lane * 16;
    const uint8_t* sb_mine = smem + SBUF0 + wave * 512 + lane * 4;
    auto request_codes = [&](int g, int buf, int R) __attribute__((always_inline)) {     // g clamped to the row: a late request fetches unused bytes
        const int gc = min(g, G - 1);
        // 2-bit rows: the whole group; 1-bit rows: the aligned pair of groups; 4-bit rows: my half of
        // the group's 32 bytes (the lookup path's contraction order makes it one run)
        // = rowoff + (4 bits: 32 g + 16 fkg; 2 bits: 16 g; 1 bit: 16 (g / 2)), from per-lane constants: a shift and a multiply-add
        dma16_s(p.packed, __umul24((uint32_t)gc >> rq_shift[R], rq_mul[R]) + rq_add[R], cb_lds + buf * CBUFB + R * 1024);
    };
    auto request_scale = [&](int g, int buf, int R) __attribute__((always_inline)) {
        const int gc = min(g, G - 1);
        dma4_s(p.absmax + gc, amoff[R], sb_lds + buf * SBUFB + R * 256);
    };
    auto fetch_codes = [&](int buf, int R) {
        const uint4 c = *reinterpret_cast<const uint4*>(cb_mine + buf * CBUFB + R * 1024);
        rc[R][0] = c.x; rc[R][1] = c.y; rc[R][2] = c.z; rc[R][3] = c.w;
        rscale[R] = *reinterpret_cast<const float*>(sb_mine + buf * SBUFB + R * 256);
    };
    // Tables of the fetched group for row R into set SET, in 6 parts of about two instructions.
    // ODD: the group's index is odd, so a 1-bit row finds it in the upper 8 of its 16 bytes.
    float tl[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    uint32_t P01 = 0, P23 = 0;
    uint32_t xa0 = 0, xa2 = 0;
    auto tables_piece = [&](auto SET_, auto ODD_, auto R_, auto PIECE_) __attribute__((always_inline)) {
        constexpr int SET = decltype(SET_)::value, R = decltype(R_)::value, PIECE = decltype(PIECE_)::value;
        constexpr bool ODD = decltype(ODD_)::value != 0;
        if constexpr (PIECE >= 0 && PIECE < 4) tl[PIECE] = lev[R][PIECE] * rscale[R];
        if constexpr (PIECE == 4) P01 = pack_bf16x2(tl[0], tl[1]);
        if constexpr (PIECE == 5) P23 = pack_bf16x2(tl[2], tl[3]);
        if constexpr (PIECE == 6) SL[SET][R] = __builtin_amdgcn_perm(P23, P01, selL[R]);
        if constexpr (PIECE == 7) SH[SET][R] = __builtin_amdgcn_perm(P23, P01, selH[R]);
        if constexpr (PIECE == 8) xa0 = (ODD && !two[R]) ? rc[R][2] : rc[R][0];
        if constexpr (PIECE == 9) x[SET][R][0] = __builtin_amdgcn_perm(rc[R][1], xa0, selX[R]);
        if constexpr (PIECE == 10) xa2 = two[R] ? rc[R][2] : (ODD ? rc[R][3] : rc[R][1]);
        if constexpr (PIECE == 11) x[SET][R][1] = __builtin_amdgcn_perm(rc[R][3], xa2, selX[R]);
    };
    auto tables_all = [&](auto SET_, auto ODD_, auto R_) {
        tables_piece(SET_, ODD_, R_, int_c<0>{}); tables_piece(SET_, ODD_, R_, int_c<1>{}); tables_piece(SET_, ODD_, R_, int_c<2>{});
        tables_piece(SET_, ODD_, R_, int_c<3>{}); tables_piece(SET_, ODD_, R_, int_c<4>{}); tables_piece(SET_, ODD_, R_, int_c<5>{});
        tables_piece(SET_, ODD_, R_, int_c<6>{}); tables_piece(SET_, ODD_, R_, int_c<7>{}); tables_piece(SET_, ODD_, R_, int_c<8>{});
        tables_piece(SET_, ODD_, R_, int_c<9>{}); tables_piece(SET_, ODD_, R_, int_c<10>{}); tables_piece(SET_, ODD_, R_, int_c<11>{});
    };

    // decode pipeline registers, carried from slot to slot (and across steps)
    uint32_t t0 = 0, t1 = 0;

    // One slot of the fast step (compile-time position S of 64): an MFMA and the independent work
    // that issues in its shadow; the two decode instructions of a slot belong to different code
    // pairs, so neither waits for the other.
    auto fast_slot = [&](auto SJ_, auto S_, int jd, const uint16_t* dma_base) {
        constexpr int SJ = decltype(SJ_)::value, S = decltype(S_)::value;
        constexpr int ST = SJ & 3, ST1 = (SJ + 1) & 3, ST3 = (SJ + 3) & 3;
        constexpr int CUR = SJ & 1, NXT = CUR ^ 1;             // table sets; NXT is also the code buffer of groups j+1 and j+3
        constexpr int kk = S >> 4, s = S & 15, mi = slot_mfma(s, TM);
        if constexpr (mi >= 0) {
            constexpr int tn = mi / TM, tm = mi % TM;
            acc[tn][tm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wfrag(kk & 1, tn), fact[kk & 1][tm], acc[tn][tm], 0, 0, 0);
        }
        // activation operands of the next slice (slice 0 of the next step after slice 3)
        if constexpr (s < TM) {
            const uint8_t* src = smem + (kk < 3 ? ST : ST1) * ASTAGEB;
            fact[(kk + 1) & 1][s] = *reinterpret_cast<const bf16x8_t*>(src + kofs[(kk + 1) & 3] + s * 32 * AROWB);
        }
        // One wait for the slice's eight operand reads (issued eight slots ago: long landed) instead of the eight partial
        // waits the compiler would put in front of the next slice's MFMAs: a wavefront alone on its SIMD pays for every
        // instruction it issues beside an MFMA.
        if constexpr (s == 15) __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0)
        // decode, software-pipelined over the 32 code pairs of the step: pair q = S/2 starts
        // (extract, spread) while pair q-1 finishes (select bytes, look up)
        {
            constexpr PairInfo cur = pair_info(S >> 1), prv = pair_info((S >> 1) - 1);
            constexpr int cset = cur.next_set ? NXT : CUR, pset = prv.next_set ? NXT : CUR;
            if ((S & 1) == 0) {
                t1 = (t0 & MASK[prv.row]) | ORC[prv.row];
                t0 = __builtin_amdgcn_ubfe(x[cset][cur.row][cur.xreg], boff[cur.row][cur.half][cur.jp], fwid[cur.row]);
            } else {
                fwd[prv.buf][prv.row][prv.jp] = __builtin_amdgcn_perm(SH[pset][prv.row], SL[pset][prv.row], t1);
                t0 = __umul24(t0, MUL[cur.row]);
            }
        }
        // activation tile j+3, one transfer every 6 slots
        if constexpr (slot_issues_activation(S, TM)) dma16_s(dma_base, a_voff[S / 6], smem_lds + ST3 * ASTAGEB + wave * (WROWS * AROWB) + (S / 6) * 1024);
        // group j+1: read back (landed one step ago), build its tables; then ask for group j+3
        if constexpr (S == kFetchSlot[0]) fetch_codes(NXT, 0);
        if constexpr (S == kFetchSlot[1]) fetch_codes(NXT, 1);
        if constexpr (slot_table_piece(S, 0) >= 0) tables_piece(int_c<NXT>{}, int_c<NXT>{}, int_c<0>{}, int_c<slot_table_piece(S, 0)>{});
        if constexpr (slot_table_piece(S, 1) >= 0) tables_piece(int_c<NXT>{}, int_c<NXT>{}, int_c<1>{}, int_c<slot_table_piece(S, 1)>{});
        if constexpr (slot_requests_codes(S) >= 0) request_codes(jd + 3, NXT, slot_requests_codes(S));
        if constexpr (slot_requests_scale(S) >= 0) request_scale(jd + 3, NXT, slot_requests_scale(S));
        __builtin_amdgcn_sched_barrier(0);
    };
    auto fast_slots = [&](auto SJ_, int jd, const uint16_t* dma_base, auto... Ss) {
        (fast_slot(SJ_, Ss, jd, dma_base), ...);
    };
    // Fast step j (compile-time SJ = j mod 4 fixes stage, table set and group parity).  Entry:
    // activation tiles j, j+1 visible and j+2 landing, operands of slice 0 in fact[0] / fwd[0]
    // (row 1's last pair still in the decode pipeline), tables of group j in set j&1, codes of
    // group j+1 landed, codes of group j+2 in flight.  Near the end of the contraction the tile and
    // group indices it works ahead on are clamped: the step then refills LDS nobody reads again
    // and builds tables nobody uses, and stays branch-free.
    auto fast_step = [&](auto SJ_, int jd) {
        const uint16_t* dma_base = act0 + (size_t)min(jd + 3, G - 1) * KS;
        __builtin_amdgcn_sched_barrier(0);
        fast_slots(SJ_, jd, dma_base, int_c<0>{}, int_c<1>{}, int_c<2>{}, int_c<3>{}, int_c<4>{}, int_c<5>{}, int_c<6>{}, int_c<7>{},
                   int_c<8>{}, int_c<9>{}, int_c<10>{}, int_c<11>{}, int_c<12>{}, int_c<13>{}, int_c<14>{}, int_c<15>{},
                   int_c<16>{}, int_c<17>{}, int_c<18>{}, int_c<19>{}, int_c<20>{}, int_c<21>{}, int_c<22>{}, int_c<23>{},
                   int_c<24>{}, int_c<25>{}, int_c<26>{}, int_c<27>{}, int_c<28>{}, int_c<29>{}, int_c<30>{}, int_c<31>{},
                   int_c<32>{}, int_c<33>{}, int_c<34>{}, int_c<35>{}, int_c<36>{}, int_c<37>{}, int_c<38>{}, int_c<39>{},
                   int_c<40>{}, int_c<41>{}, int_c<42>{}, int_c<43>{}, int_c<44>{}, int_c<45>{}, int_c<46>{}, int_c<47>{},
                   int_c<48>{}, int_c<49>{}, int_c<50>{}, int_c<51>{}, int_c<52>{}, int_c<53>{}, int_c<54>{}, int_c<55>{},
                   int_c<56>{}, int_c<57>{}, int_c<58>{}, int_c<59>{}, int_c<60>{}, int_c<61>{}, int_c<62>{}, int_c<63>{});
        // Everything started before this step must have landed before the barrier publishes it:
        // the transfers younger than that are exactly the ones issued in this step.
        asm volatile("s_waitcnt vmcnt(%0)" : : "n"(kStepTransfers) : "memory");
        __syncthreads();
    };

    // ---- lookup path, for wavefronts that hold a 4-bit row: every code (any width) indexes its
    // codebook's fp32 levels in LDS (16 consecutive banks: conflict-free whatever the codes), the
    // level is multiplied by the group's absmax and rounded to bf16 (App. A.2 as written).  One
    // weight per MFMA slot, in a pipeline carried from slot to slot and step to step:
    // extract (slot S) -> address (S+1) -> LDS read (S+2) -> multiply (S+6) -> pack a pair (S+7).
    // Weight S of a step's stream belongs to section S/16 (operands of slice S/16 + 1; section 3
    // builds slice 0 of the next step from the next group), row (S/8)&1, code S&7 of the slice.
    uint32_t lrc[2][2][4] = {{{0u, 0u, 0u, 0u}, {0u, 0u, 0u, 0u}}, {{0u, 0u, 0u, 0u}, {0u, 0u, 0u, 0u}}};   // [set][row]
    float lsc[2][2] = {{0.0f, 0.0f}, {0.0f, 0.0f}};
    uint32_t csh[2] = {0u, 0u}, craw = 0u, craw1 = 0u, craw2 = 0u, e_reg = 0u, ad_reg = tbase[0];
    float vring[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f}, pm[2] = {0.0f, 0.0f};
    auto fetch_lut = [&](auto BUF_, auto SET_, auto R_) __attribute__((always_inline)) {
        constexpr int BUF = decltype(BUF_)::value, SET = decltype(SET_)::value, R = decltype(R_)::value;
        const uint4 c = *reinterpret_cast<const uint4*>(cb_mine + BUF * CBUFB + R * 1024);
        lrc[SET][R][0] = c.x; lrc[SET][R][1] = c.y; lrc[SET][R][2] = c.z; lrc[SET][R][3] = c.w;
        const float a = *reinterpret_cast<const float*>(sb_mine + BUF * SBUFB + R * 256);
        lsc[SET][R] = row_ok[R] ? a : 0.0f;
    };
    // the decode work of slot S of a step whose group sits in set CUR (= its parity)
    auto lut_decode = [&](auto CUR_, auto S_) __attribute__((always_inline)) {
        constexpr int CUR = decltype(CUR_)::value, NXT = CUR ^ 1, S = decltype(S_)::value;
        {   // pack the pair (S-8, S-7)
            constexpr int w = (S - 7) & 63, i = w & 7;
            if constexpr ((i & 1) == 1) {
                constexpr int R = (w >> 3) & 1, tk = ((w >> 4) + 1) & 3;
                fwd[tk & 1][R][i >> 1] = pack_bf16x2(pm[0], pm[1]);
            }
        }
        {   // multiply weight S-6 by its group's absmax (a weight of the previous step's section 3 used that step's next set)
            constexpr int w = (S - 6) & 63, R = (w >> 3) & 1;
            constexpr int set = (S - 6 >= 0 && (w >> 4) == 3) ? NXT : CUR;
            pm[w & 1] = vring[w & 7] * lsc[set][R];
        }
        {   // LDS read of weight S-2, address of weight S-1, extraction of weight S
            constexpr int w2 = (S - 2) & 63, w1 = (S - 1) & 63;
            vring[w2 & 7] = *reinterpret_cast<const float*>(smem + ad_reg);
            ad_reg = (e_reg << 2) + tbase[(w1 >> 3) & 1];
            e_reg = __builtin_amdgcn_ubfe(csh[(S >> 3) & 1], ibv[(S >> 3) & 1][S & 7], bwv[(S >> 3) & 1]);
        }
        // code words: row 1's for this section at positions 5-7, row 0's for the next section at 13-15
        constexpr int sec = S >> 4, pos = S & 15;
        if constexpr (pos >= 5 && pos <= 7) {
            constexpr int tk = (sec + 1) & 3, set = sec == 3 ? NXT : CUR;
            if constexpr (pos == 5) {
                const uint32_t h2 = lrc[set][1][2 + (tk >> 1)], l2 = lrc[set][1][tk >> 1];
                const uint32_t h1 = lrc[set][1][2 * set + 1], l1 = lrc[set][1][2 * set];
                craw2 = fkg ? h2 : l2;
                craw1 = fkg ? h1 : l1;
            } else if constexpr (pos == 6) {
                const uint32_t c4 = lrc[set][1][tk], c21 = two[1] ? craw2 : craw1;
                craw = four[1] ? c4 : c21;
            } else {
                csh[1] = craw >> shv[1][tk];
            }
        }
        if constexpr (pos >= 13) {
            constexpr int nsec = (sec + 1) & 3;
            constexpr int tk = (nsec + 1) & 3, set = (sec == 3 || nsec == 3) ? NXT : CUR;   // after section 3: the next step's group
            if constexpr (pos == 13) {
                const uint32_t h2 = lrc[set][0][2 + (tk >> 1)], l2 = lrc[set][0][tk >> 1];
                const uint32_t h1 = lrc[set][0][2 * set + 1], l1 = lrc[set][0][2 * set];
                craw2 = fkg ? h2 : l2;
                craw1 = fkg ? h1 : l1;
            } else if constexpr (pos == 14) {
                const uint32_t c4 = lrc[set][0][tk], c21 = two[0] ? craw2 : craw1;
                craw = four[0] ? c4 : c21;
            } else {
                csh[0] = craw >> shv[0][tk];
            }
        }
    };
    auto lut_slot = [&](auto CUR_, auto S_, int jd, const uint16_t* dma_base, int st_cur, int st_nxt, uint32_t st3_lds) __attribute__((always_inline)) {
        constexpr int CUR = decltype(CUR_)::value, NXT = CUR ^ 1, S = decltype(S_)::value;
        constexpr int kk = S >> 4, s = S & 15, mi = slot_mfma(s, TM);
        if constexpr (mi >= 0) {
            constexpr int tn = mi / TM, tm = mi % TM;
            acc[tn][tm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wfrag(kk & 1, tn), fact[kk & 1][tm], acc[tn][tm], 0, 0, 0);
        }
        if constexpr (s < TM) {
            const uint8_t* src = smem + (kk < 3 ? st_cur : st_nxt);
            fact[(kk + 1) & 1][s] = *reinterpret_cast<const bf16x8_t*>(src + kofl[(kk + 1) & 3] + s * 32 * AROWB);
        }
        lut_decode(CUR_, S_);
        if constexpr (slot_issues_activation(S, TM)) dma16_s(dma_base, a_voff[S / 6], st3_lds + wave * (WROWS * AROWB) + (S / 6) * 1024);
        if (S == 20) fetch_lut(int_c<NXT>{}, int_c<NXT>{}, int_c<0>{});
        if (S == 24) fetch_lut(int_c<NXT>{}, int_c<NXT>{}, int_c<1>{});
        if constexpr (slot_requests_codes(S) >= 0) request_codes(jd + 3, NXT, slot_requests_codes(S));
        if constexpr (slot_requests_scale(S) >= 0) request_scale(jd + 3, NXT, slot_requests_scale(S));
        __builtin_amdgcn_sched_barrier(0);
    };
    auto lut_slots = [&](auto CUR_, int jd, const uint16_t* dma_base, int st_cur, int st_nxt, uint32_t st3_lds, auto... Ss) __attribute__((always_inline)) {
        (lut_slot(CUR_, Ss, jd, dma_base, st_cur, st_nxt, st3_lds), ...);
    };
    // Lookup step j (compile-time parity): same entry state, transfers and barrier as the fast step.
    auto lut_step = [&](auto CUR_, int jd) __attribute__((always_inline)) {
        const uint16_t* dma_base = act0 + (size_t)min(jd + 3, G - 1) * KS;
        const int st_cur = (jd & 3) * ASTAGEB, st_nxt = ((jd + 1) & 3) * ASTAGEB;
        const uint32_t st3_lds = smem_lds + ((jd + 3) & 3) * ASTAGEB;
        __builtin_amdgcn_sched_barrier(0);
        lut_slots(CUR_, jd, dma_base, st_cur, st_nxt, st3_lds, int_c<0>{}, int_c<1>{}, int_c<2>{}, int_c<3>{}, int_c<4>{}, int_c<5>{}, int_c<6>{}, int_c<7>{},
                  int_c<8>{}, int_c<9>{}, int_c<10>{}, int_c<11>{}, int_c<12>{}, int_c<13>{}, int_c<14>{}, int_c<15>{},
                  int_c<16>{}, int_c<17>{}, int_c<18>{}, int_c<19>{}, int_c<20>{}, int_c<21>{}, int_c<22>{}, int_c<23>{},
                  int_c<24>{}, int_c<25>{}, int_c<26>{}, int_c<27>{}, int_c<28>{}, int_c<29>{}, int_c<30>{}, int_c<31>{},
                  int_c<32>{}, int_c<33>{}, int_c<34>{}, int_c<35>{}, int_c<36>{}, int_c<37>{}, int_c<38>{}, int_c<39>{},
                  int_c<40>{}, int_c<41>{}, int_c<42>{}, int_c<43>{}, int_c<44>{}, int_c<45>{}, int_c<46>{}, int_c<47>{},
                  int_c<48>{}, int_c<49>{}, int_c<50>{}, int_c<51>{}, int_c<52>{}, int_c<53>{}, int_c<54>{}, int_c<55>{},
                  int_c<56>{}, int_c<57>{}, int_c<58>{}, int_c<59>{}, int_c<60>{}, int_c<61>{}, int_c<62>{}, int_c<63>{});
        asm volatile("s_waitcnt vmcnt(%0)" : : "n"(kStepTransfers) : "memory");
        __syncthreads();
    };
    auto lut_prime = [&](auto... Ss) __attribute__((always_inline)) { (lut_decode(int_c<1>{}, Ss), ...); };

    // ---- prologue: codes of groups 0 and 1; activation tiles 0..2 complete
    int j = 0;
    if (wave_fast || wave_lut) {
        request_codes(0, 0, 0); request_codes(0, 0, 1); request_scale(0, 0, 0); request_scale(0, 0, 1);
        request_codes(1, 1, 0); request_codes(1, 1, 1); request_scale(1, 1, 0); request_scale(1, 1, 1);
    }
    dma_wait_all();
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0), told to the compiler: nothing of the prologue is pending in the loop
    __syncthreads();

    // ---- weight steps
    if (wave_fast) {
        // tables of group 0 (set 0), operands of (step 0, slice 0); codes of group 2 requested
        fetch_codes(0, 0); fetch_codes(0, 1);
        tables_all(int_c<0>{}, int_c<0>{}, int_c<0>{});
        tables_all(int_c<0>{}, int_c<0>{}, int_c<1>{});
        request_codes(2, 0, 0); request_codes(2, 0, 1); request_scale(2, 0, 0); request_scale(2, 0, 1);
#pragma unroll
        for (int R = 0; R < 2; ++R)
#pragma unroll
            for (int jp = 0; jp < 4; ++jp) {
                const uint32_t q = __builtin_amdgcn_ubfe(x[0][R][0], boff[R][0][jp], fwid[R]);
                if (R == 1 && jp == 3) t0 = __umul24(q, MUL[R]);   // the pipeline's pending pair: finished in slots 0, 1 of step 0
                else fwd[0][R][jp] = __builtin_amdgcn_perm(SH[0][R], SL[0][R], (__umul24(q, MUL[R]) & MASK[R]) | ORC[R]);
            }
        load_fact(0, 0, fact[0]);
        for (; j + 4 <= G; j += 4) {
            fast_step(int_c<0>{}, j);
            fast_step(int_c<1>{}, j + 1);
            fast_step(int_c<2>{}, j + 2);
            fast_step(int_c<3>{}, j + 3);
        }
        if (j + 2 <= G) {                  // G is even: at most one pair of steps is left
            fast_step(int_c<0>{}, j);
            fast_step(int_c<1>{}, j + 1);
            j += 2;
        }
        dma_wait_all();
    } else if (wave_lut) {
        // group 0 into set 0; codes of group 2 requested; operands of (step 0, slice 0): the decode
        // half of the last 19 slots of a step whose next set is set 0
        fetch_lut(int_c<0>{}, int_c<0>{}, int_c<0>{}); fetch_lut(int_c<0>{}, int_c<0>{}, int_c<1>{});
        request_codes(2, 0, 0); request_codes(2, 0, 1); request_scale(2, 0, 0); request_scale(2, 0, 1);
        lut_prime(int_c<45>{}, int_c<46>{}, int_c<47>{}, int_c<48>{}, int_c<49>{}, int_c<50>{}, int_c<51>{}, int_c<52>{}, int_c<53>{}, int_c<54>{},
                  int_c<55>{}, int_c<56>{}, int_c<57>{}, int_c<58>{}, int_c<59>{}, int_c<60>{}, int_c<61>{}, int_c<62>{}, int_c<63>{});
#pragma unroll
        for (int t = 0; t < TM; ++t) fact[0][t] = *reinterpret_cast<const bf16x8_t*>(smem + kofl[0] + t * 32 * AROWB);
        for (; j + 2 <= G; j += 2) {       // G is even
            lut_step(int_c<0>{}, j);
            lut_step(int_c<1>{}, j + 1);
        }
        dma_wait_all();
    }
    for (; j < G; ++j) slow_step(j);

    // ---- LoRA steps: all RP/64 (<= 2) tiles of s t are staged at once; B rows are plain bf16
    if (p.RP) {
        const int ne = p.RP / KS;
        uint32_t e_voff[TM];
#pragma unroll
        for (int i = 0; i < TM; ++i) e_voff[i] = a_voff_of(i, p.RP);
        for (int e = 0; e < ne; ++e) {
            const uint16_t* base = p.ext_act + (size_t)m0 * p.RP + (size_t)e * KS;
            const uint32_t dst = smem_lds + e * ASTAGEB + wave * (WROWS * AROWB);
#pragma unroll
            for (int i = 0; i < TM; ++i) dma16_s(base, e_voff[i], dst + i * 1024);
        }
        // the rows of B for the first 64 ranks go straight into operand registers, asked for before the wait
        bf16x8_t wB[4][2];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
#pragma unroll
            for (int R = 0; R < 2; ++R)
                wB[kk][R] = *reinterpret_cast<const bf16x8_t*>(p.ext_w + (size_t)nrow[R] * p.RP + kk * 16 + fkg * 8);
        dma_wait_all();
        __syncthreads();
        for (int e = 0; e < ne; ++e)
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                load_fact(e, kk, fact[0]);
                bf16x8_t w[2];
#pragma unroll
                for (int R = 0; R < 2; ++R)
                    w[R] = e == 0 ? wB[kk][R]
                                  : *reinterpret_cast<const bf16x8_t*>(p.ext_w + (size_t)nrow[R] * p.RP + e * KS + kk * 16 + fkg * 8);
                mma16(w[0], w[1], fact[0]);
            }
    }

    // ---- epilogue: the tile goes through LDS so that every global store is 16 contiguous bytes.
    // Accumulator register v of tile (tn, tm): channel position 32 tn + 8 (v/4) + 4 fkg + v%4 of my
    // 64, token row 32 tm + fi.  In natural row order four registers are four adjacent columns.
    __syncthreads();
    if (natural) {
#pragma unroll
        for (int tn = 0; tn < 2; ++tn)
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int vq = 0; vq < 4; ++vq) {
                    uint2 v;
                    v.x = pack_bf16x2(acc[tn][tm][4 * vq], acc[tn][tm][4 * vq + 1]);
                    v.y = pack_bf16x2(acc[tn][tm][4 * vq + 2], acc[tn][tm][4 * vq + 3]);
                    *reinterpret_cast<uint2*>(smem + (32 * tm + fi) * EPI_LD + (((wave * 8 + 4 * tn + vq) ^ fi) << 4) + 8 * fkg) = v;
                }
    } else {
#pragma unroll
        for (int tn = 0; tn < 2; ++tn)
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
                const uint2 o = *reinterpret_cast<const uint2*>(p.tile_order + n0 + wave * 64 + 32 * tn + 8 * vq + 4 * fkg);
                const int col[4] = {(int)(o.x & 0xffffu), (int)(o.x >> 16), (int)(o.y & 0xffffu), (int)(o.y >> 16)};
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        *reinterpret_cast<uint16_t*>(smem + (32 * tm + fi) * EPI_LD + (((col[e] >> 3) ^ fi) << 4) + (col[e] & 7) * 2) =
                            (uint16_t)(pack_bf16x2(acc[tn][tm][4 * vq + e], 0.0f) & 0xffffu);
            }
    }
    __syncthreads();
    {
        const int c = tid & 31, r0 = tid >> 5;
        const bool col_ok = n0 + 8 * c < p.N;                  // N is a multiple of 8: a chunk is in or out as a whole
#pragma unroll 4
        for (int it = 0; it < 4 * TM; ++it) {
            const int r = it * 8 + r0;
            if (col_ok && m0 + r < p.M)
                *reinterpret_cast<uint4*>(p.out + (size_t)(m0 + r) * p.N + n0 + 8 * c) =
                    *reinterpret_cast<const uint4*>(smem + r * EPI_LD + ((c ^ (r & 31)) << 4));
        }
    }
}

// ---- tiling of the output.  Region A: the first cols_a 256-channel columns in token tiles of 32 TMA rows; region B:
// the other columns in tiles of 32 TMB rows.  A compute unit holds one workgroup, so a launch runs in rounds; a
// second, lower tile height for the last columns lets the last round be a short one that every compute unit takes
// part in (11008 x 4096 outputs on 256 units: 512 tiles of 256 rows, then 242 of 192, instead of 688 of 256 in
// three rounds with the last one 69 % full).  Region A's workgroups come first in launch order.
struct FwdPlan {
    int cols_a, cols_b;       // 256-channel columns of each region
    int tiles_a;              // workgroups of region A
};

template <int TMA, int TMB>
__global__ __launch_bounds__(NTHREADS) void linear_fwd_kernel(GemmParams p, FwdPlan plan) {
    extern __shared__ __align__(16) uint8_t smem[];
    const int bid = blockIdx.x;
    if (TMA == TMB || bid < plan.tiles_a) {              // uniform
        const int tile = xcd_tile(bid, TMA == TMB ? (int)gridDim.x : plan.tiles_a);
        fwd_tile<TMA>(p, (tile % plan.cols_a) * BN, (tile / plan.cols_a) * (32 * TMA), smem);
    } else if constexpr (TMA != TMB) {
        const int tile = xcd_tile(bid - plan.tiles_a, (int)gridDim.x - plan.tiles_a);
        fwd_tile<TMB>(p, (plan.cols_a + tile % plan.cols_b) * BN, (tile / plan.cols_b) * (32 * TMB), smem);
    }
}

// Relative duration of a tile by height (measured on 11008 x 4096, 4096 tokens): a lower tile decodes the same
// weights for fewer MFMAs and pays the same prologue and epilogue latencies.
static double tile_cost(int TM) { return TM == 8 ? 1.0 : TM == 6 ? LOWRA_FWD_COST6 : LOWRA_FWD_COST4; }

// Finish time of `ta` tiles of cost ca followed by `tb` tiles of cost cb on `P` compute units, every tile going to the
// unit that is free first (launch order).
static double plan_makespan(long ta, double ca, long tb, double cb, int P) {
    const long full = ta / P, rem = ta % P;
    // two groups of units after region A: `rem` of them busy until (full + 1) ca, the others until full ca
    double t_early = full * ca, t_late = (full + (rem ? 1 : 0)) * ca;
    long n_early = P - rem, n_late = rem;
    double end = ta ? (rem ? t_late : t_early) : 0.0;
    while (tb > 0) {
        const bool early = n_late == 0 || t_early <= t_late;
        double& t = early ? t_early : t_late;
        const long n = early ? n_early : n_late, take = tb < n ? tb : n;
        t += cb;
        if (t > end) end = t;
        if (take < n) break;                                           // the rest of the group stays idle
        tb -= take;
    }
    return end;
}

struct FwdChoice { int tma, tmb, cols_a; };
static FwdChoice plan_fwd(int N, int M, int forced, int units = 0) {
    const int cols = (N + BN - 1) / BN;
    if (forced >= 0) return FwdChoice{(forced >> 8) & 15, (forced >> 4) & 15, std::min(forced >> 12, cols)};
    const int P = units > 0 ? units : device_compute_units();
    static const int pairs[][2] = {{8, 8}, {6, 6}, {4, 4}, {8, 6}, {8, 4}, {6, 4}};
    FwdChoice best{8, 8, cols};
    double best_t = 1e300;                                         // ties: the first plan in this order (measured: a tie-break by total work picks worse plans)
    for (const auto& pr : pairs) {
        const long ma = (M + 32 * pr[0] - 1) / (32 * pr[0]), mb = (M + 32 * pr[1] - 1) / (32 * pr[1]);
        const int lo = pr[0] == pr[1] ? cols : 1, hi = pr[0] == pr[1] ? cols : cols - 1;
        for (int ca = lo; ca <= hi; ++ca) {
            const double t = plan_makespan(ma * ca, tile_cost(pr[0]), mb * (cols - ca), tile_cost(pr[1]), P);
            if (t < best_t * (1.0 - 1e-9)) { best_t = t; best = FwdChoice{pr[0], pr[1], ca}; }
        }
    }
    return best;
}

template <int TMA, int TMB>
static hipError_t launch_fwd_variant(const GemmParams& p, const FwdChoice& c, hipStream_t st) {
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(linear_fwd_kernel<TMA, TMB>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)kFwdSmem);
    if (attr != hipSuccess) return attr;
    const int cols = (p.N + BN - 1) / BN;
    FwdPlan plan;
    plan.cols_a = TMA == TMB ? cols : c.cols_a;
    plan.cols_b = cols - plan.cols_a;
    plan.tiles_a = plan.cols_a * ((p.M + 32 * TMA - 1) / (32 * TMA));
    const int tiles_b = plan.cols_b * ((p.M + 32 * TMB - 1) / (32 * TMB));
    linear_fwd_kernel<TMA, TMB><<<dim3(plan.tiles_a + tiles_b), dim3(NTHREADS), kFwdSmem, st>>>(p, plan);
    return hipGetLastError();
}

// the planner's choice for N channels, M tokens and `units` compute units, as token-tile heights and column count
void plan_fwd_tiling(int N, int M, int units, int* rows_a, int* rows_b, int* cols_a) {
    const FwdChoice c = plan_fwd(N, M, -1, units);
    const int cols = (N + BN - 1) / BN;
    *rows_a = 32 * c.tma; *rows_b = 32 * c.tmb; *cols_a = c.tma == c.tmb ? cols : c.cols_a;
}

// `tiling`: -1 lets the planner choose; else TMA << 8 | TMB << 4 | cols_a << 12 (test and measurement hook)
hipError_t launch_gemm_fwd(const GemmParams& p, int tiling, hipStream_t st) {
    const FwdChoice c = plan_fwd(p.N, p.M, tiling);
    const int key = c.tma * 10 + c.tmb;
    const bool split = c.tma != c.tmb && c.cols_a > 0 && c.cols_a < (p.N + BN - 1) / BN;
    if (!split) {
        const int tm = c.tma != c.tmb && c.cols_a == 0 ? c.tmb : c.tma;
        if (tm == 8) return launch_fwd_variant<8, 8>(p, c, st);
        if (tm == 6) return launch_fwd_variant<6, 6>(p, c, st);
        if (tm == 4) return launch_fwd_variant<4, 4>(p, c, st);
        return hipErrorInvalidValue;
    }
    if (key == 86) return launch_fwd_variant<8, 6>(p, c, st);
    if (key == 84) return launch_fwd_variant<8, 4>(p, c, st);
    if (key == 64) return launch_fwd_variant<6, 4>(p, c, st);
    return hipErrorInvalidValue;
}

}  // namespace lowra
