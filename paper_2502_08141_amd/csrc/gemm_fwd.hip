// Forward fused dequant-GEMM:  y = [x | s x A^T] [What | B]^T   (Sec. 2.1 LoRA form; App. A.2 decode)
//
// 256 x 256 outputs per workgroup, 4 wavefronts of 128 x 128 (v_mfma_f32_32x32x16_bf16), 32-deep
// contraction steps, FOUR LDS stages.  During step j a wavefront
//   * runs the 32 MFMAs of tile j (operands of its first half were read during step j-1),
//   * decodes its weight row's 32 codes of tile j+2 into stage (j+2)%4,
//   * starts the DMA of activation tile j+3 into stage (j+3)%4.
// The barrier that ends step j publishes tile j+2, which nobody reads before step j+1's second
// half, so the MFMA stream does not stall on it and every DMA has two steps to land.
//
// Thread t owns one weight row of the 256-row tile (rows of equal width sit on adjacent lanes, see
// tile_order).  1- and 2-bit rows decode without table memory and with one instruction stream for
// both widths: the row's 2 or 4 levels times the group absmax are rounded to bf16 once per group
// (the multiply and rounding of App. A.2 on 2^b values instead of 64 weights), their low and high
// bytes form the 8-byte source of v_perm_b32, and a pair of codes becomes the 4-byte selector with
// one bit-field extract, one 24-bit multiply that spreads the bits, and one and-or.  Width only
// changes per-lane constants.  Wavefronts that hold a 4-bit row, the ragged ends of the
// contraction and the LoRA extension steps take a general (slower) step with the same protocol.
#include <cstdlib>
#include <type_traits>

#include "gemm_common.h"

namespace lowra {

constexpr int KS = 32;                     // contraction depth per step
constexpr int FROWB = 64;                  // bytes per LDS row: 32 bf16 = 4 chunks of 16 B
constexpr int FTILEB = 256 * FROWB;        // 16 KB per operand tile
constexpr int FSTAGEB = 2 * FTILEB;        // activation tile + weight tile
constexpr int NSTAGE = 4;
constexpr int CODEB = 256 * 16 + 256 * 4;   // per-thread staging of the next group's codes (16 B) and absmax (4 B)
constexpr size_t kFwdSmem = (size_t)NSTAGE * FSTAGEB + (size_t)BN * TAB_LD * 4 + CODEB;

// 16 consecutive rows at one logical chunk hit 16 distinct 16-byte bank groups
__device__ __forceinline__ int fswz(int row, int chunk) { return row * FROWB + ((chunk ^ ((row >> 2) & 3)) << 4); }

template <int SLOT> using slot_c = std::integral_constant<int, SLOT>;

template <int DBG>
__global__ __launch_bounds__(NTHREADS) void linear_fwd_kernel(GemmParams p) {
    extern __shared__ __align__(16) uint8_t smem[];
    float* sT = reinterpret_cast<float*>(smem + NSTAGE * FSTAGEB);
    const uint32_t smem_lds = (uint32_t)(uintptr_t)(lptr_t)smem;

    uint64_t tm_begin = 0;
    if (DBG & 64) asm volatile("s_memtime %0\n\ts_waitcnt lgkmcnt(0)" : "=s"(tm_begin) :: "memory");
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform, and known to be
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
    const bool m_full = m0 + BM <= p.M && n0 + BN <= p.N;   // the fast path assumes a full output tile
    // the fast path also fetches 1-bit codes as aligned 16-byte pairs of groups: G must be even
    const bool wave_fast = __builtin_amdgcn_ballot_w64(bits == 4) == 0 && m_full && (p.G & 1) == 0;

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
    const int cstride = 8 * bits;                            // code bytes per 64-wide group
    uint32_t boff[2][4];                                     // bit offsets of pair j in the low / high 16-bit slot
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int j = 0; j < 4; ++j) boff[h][j] = 16u * h + j * fw;

    // ---- activation tile: global -> LDS DMA, 16 rows x 64 B per instruction, wavefront w owns rows
    // [64 w, 64 w + 64).  LDS is filled linearly, so the chunk swizzle is applied to the global
    // address: the lane landing on physical chunk l&3 of row r fetches logical chunk (l&3)^((r>>2)&3).
    const int m_last = p.M - 1 - m0;
    auto a_row_c = [&](int i) -> uint32_t {
        const int r = wave * 64 + 16 * i + (lane >> 2);
        return (uint32_t)(r < m_last ? r : m_last);          // rows past M are clamped (never stored back)
    };
    const uint32_t a_chunk_b = (uint32_t)(((lane & 3) ^ ((lane >> 4) & 3)) * 16);
    uint32_t a_voff[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) a_voff[i] = a_row_c(i) * (uint32_t)p.K * 2u + a_chunk_b;

    const int st_main = p.K / KS, st_all = st_main + p.RP / KS;


    auto dma_act_any = [&](int j, int stage) {
        const uint32_t dst = smem_lds + stage * FSTAGEB + wave * 4096;
        if (j < st_main) {
            const uint8_t* base = reinterpret_cast<const uint8_t*>(p.act + (size_t)m0 * p.K + (size_t)j * KS);
#pragma unroll
            for (int i = 0; i < 4; ++i) dma16(base + a_voff[i], dst + i * 1024);
        } else {
            const uint8_t* base = reinterpret_cast<const uint8_t*>(p.ext_act + (size_t)m0 * p.RP + (size_t)(j - st_main) * KS);
#pragma unroll
            for (int i = 0; i < 4; ++i) dma16(base + a_row_c(i) * (uint32_t)p.RP * 2u + a_chunk_b, dst + i * 1024);
        }
    };
    // general decode of my row's 32 weights of tile j into the weight tile of `stage` (any width, LoRA rows)
    auto store_b_any = [&](int j, int stage) {
        uint8_t* bdst = smem + stage * FSTAGEB + FTILEB;
        if (j < st_main) {
            const int g = j >> 1, half = j & 1;
            const float a = amp[g];
            const uint32_t* cp = reinterpret_cast<const uint32_t*>(rowp + (size_t)g * cstride + half * (cstride / 2));
            if (bits == 1) {
                const uint32_t P01 = pack_bf16x2(lev[0] * a, lev[1] * a);
                const uint32_t Q = __builtin_amdgcn_perm(P01, P01, 0x03010200u);
                const uint32_t c = cp[0];
#pragma unroll
                for (int i = 0; i < 4; ++i) *reinterpret_cast<uint4*>(bdst + fswz(lr, i)) = decode8_w1(c >> (8 * i), Q);
            } else if (bits == 2) {
                const uint32_t P01 = pack_bf16x2(lev[0] * a, lev[1] * a), P23 = pack_bf16x2(lev[2] * a, lev[3] * a);
                const uint32_t TL = __builtin_amdgcn_perm(P23, P01, 0x06040200u);
                const uint32_t TH = __builtin_amdgcn_perm(P23, P01, 0x07050301u);
                const uint32_t c0 = cp[0], c1 = cp[1];
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    *reinterpret_cast<uint4*>(bdst + fswz(lr, i)) = decode8_w2((i < 2 ? c0 : c1) >> (16 * (i & 1)), TL, TH);
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) *reinterpret_cast<uint4*>(bdst + fswz(lr, i)) = decode8_bf16(cp[i], 4, tab, a);
            }
        } else {
            // LoRA rows are plain bf16: thread t copies natural row t (the fast path fills them by DMA in the same order)
            const int nr = n0 + tid < p.N ? n0 + tid : p.N - 1;
            const uint4* s = reinterpret_cast<const uint4*>(p.ext_w + (size_t)nr * p.RP + (j - st_main) * KS);
#pragma unroll
            for (int i = 0; i < 4; ++i) *reinterpret_cast<uint4*>(bdst + fswz(tid, i)) = s[i];
        }
    };

    // ---- MFMA operand addressing
    const int wm = wave >> 1, wn = wave & 1;
    const int fi = lane & 31, fkg = lane >> 5, fsw = (fi >> 2) & 3;
    const int a_base = (wm * 128 + fi) * FROWB, b_base = FTILEB + (wn * 128 + fi) * FROWB;
    int koff[2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) koff[kk] = ((2 * kk + fkg) ^ fsw) << 4;
    int b_soff[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) b_soff[i] = FTILEB + fswz(lr, i);

    floatx16_t acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    bf16x8_t fa[2][4], fb[2][4];     // [half of the step][tile]
    auto load_frags = [&](int stage, int kk, bf16x8_t (&a)[4], bf16x8_t (&b)[4]) {
        const uint8_t* sbase = smem + stage * FSTAGEB;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            a[t] = *reinterpret_cast<const bf16x8_t*>(sbase + a_base + t * 32 * FROWB + koff[kk]);
            b[t] = *reinterpret_cast<const bf16x8_t*>(sbase + b_base + t * 32 * FROWB + koff[kk]);
        }
    };
    auto mma16 = [&](const bf16x8_t (&a)[4], const bf16x8_t (&b)[4]) {
#pragma unroll
        for (int tm = 0; tm < 4; ++tm)
#pragma unroll
            for (int tn = 0; tn < 4; ++tn)
                acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[tm], b[tn], acc[tm][tn], 0, 0, 0);
    };

    // General step j (branches allowed): same protocol as the fast step, nothing prefetched.
    auto slow_step = [&](int j) {
        if (j + 3 < st_main) dma_act_any(j + 3, (j + 3) & 3);
        load_frags(j & 3, 0, fa[0], fb[0]);
        load_frags(j & 3, 1, fa[1], fb[1]);
        if (j + 2 < st_main) store_b_any(j + 2, (j + 2) & 3);
        mma16(fa[0], fb[0]);
        mma16(fa[1], fb[1]);
        dma_wait_all();
        __syncthreads();
    };

    // ---- fast path state: codes of the group after next in flight, byte tables of the next group.
    // Two table sets: group g uses set g & 1, so the set of the next group is built while the
    // last pairs of the current one are still being looked up.
    uint32_t rc[4] = {0u, 0u, 0u, 0u};
    float rscale = 0.0f;
    uint32_t SL[2] = {0u, 0u}, SH[2] = {0u, 0u}, x[2][4] = {{0u, 0u, 0u, 0u}, {0u, 0u, 0u, 0u}};
    // The codes (16 B) and absmax of a future group travel global -> LDS by DMA as well, so that
    // the compiler never has a register load of its own outstanding next to the untracked DMAs
    // (it would wait for ALL of them before the first use).  A thread reads back its own 20 bytes.
    // A 2-bit row fetches exactly its group; a 1-bit row (8 B per group) fetches the aligned pair
    // of groups that holds it and picks its half when the tables are made.
    uint8_t* cbuf = smem + NSTAGE * FSTAGEB + BN * TAB_LD * 4;
    const uint32_t cbuf_lds = smem_lds + NSTAGE * FSTAGEB + BN * TAB_LD * 4 + wave * 1024;
    const uint32_t abuf_lds = smem_lds + NSTAGE * FSTAGEB + BN * TAB_LD * 4 + 4096 + wave * 256;
    const uint32_t am_voff = (uint32_t)nc * (uint32_t)p.G * 4u;
    auto request_codes = [&](int g) {            // g is clamped to the row: a late request fetches unused bytes
        const int gc = min(g, p.G - 1);
        const uint32_t voff = ri.offset + (uint32_t)(two ? gc : gc >> 1) * 16u;
        dma16_s(p.packed, voff, cbuf_lds);
        dma4_s(p.absmax + gc, am_voff, abuf_lds);
    };
    auto fetch_codes = [&]() {
        const uint4 c = *reinterpret_cast<const uint4*>(cbuf + tid * 16);
        rc[0] = c.x; rc[1] = c.y; rc[2] = c.z; rc[3] = c.w;
        rscale = *reinterpret_cast<const float*>(cbuf + 4096 + tid * 4);
    };
    // scaled levels as byte tables; codes as one 16-bit slot per chunk of 8.  ODD: the fetched group
    // has an odd index, so a 1-bit row finds it in the upper 8 of its 16 bytes.
    auto make_tables = [&](auto SET_, auto ODD_) {
        constexpr int SET = decltype(SET_)::value;
        constexpr bool ODD = decltype(ODD_)::value != 0;
        const uint32_t P01 = pack_bf16x2(lev[0] * rscale, lev[1] * rscale);
        const uint32_t P23 = pack_bf16x2(lev[2] * rscale, lev[3] * rscale);
        SL[SET] = __builtin_amdgcn_perm(P23, P01, selL);
        SH[SET] = __builtin_amdgcn_perm(P23, P01, selH);
        const uint32_t lo = (ODD && !two) ? rc[2] : rc[0];
        const uint32_t hi = (ODD && !two) ? rc[3] : rc[1];
        x[SET][0] = __builtin_amdgcn_perm(hi, lo, selN0);
        x[SET][1] = __builtin_amdgcn_perm(hi, lo, selN1);
        x[SET][2] = __builtin_amdgcn_perm(rc[2], hi, selN2);
        x[SET][3] = __builtin_amdgcn_perm(rc[3], hi, selN1);
    };

    // Fast step j (compile-time SJ = j mod 4 fixes the stages).  Entry: tiles j, j+1 visible,
    // operands of (j, first half) in fa[0]/fb[0], tables of the group of tile j+2 in set TS.
    // Near the end of the contraction the tile indices it works ahead on are clamped to the last
    // weight tile: the step then refills stages nobody reads again, and stays branch-free.
    // Every MFMA is followed by a slot of independent work that issues in its shadow; the two
    // decode instructions of a slot belong to different code pairs, so neither waits for the other.
    uint32_t tm_issue = 0, tm_lds = 0, tm_vm = 0, tm_bar = 0;
    uint64_t tm_prev = 0, tm_start = 0, tm_mid = 0;
    auto fast_step = [&](auto SJ_, int j) {
        constexpr int SJ = decltype(SJ_)::value;
        constexpr int ST = SJ & 3, ST1 = (SJ + 1) & 3, ST2 = (SJ + 2) & 3, ST3 = (SJ + 3) & 3;
        const uint8_t* s_cur = smem + ST * FSTAGEB;
        const uint8_t* s_nxt = smem + ST1 * FSTAGEB;
        uint8_t* s_dec = smem + ST2 * FSTAGEB;
        const uint32_t dma_dst = smem_lds + ST3 * FSTAGEB + wave * 4096;
        const uint8_t* dma_base = reinterpret_cast<const uint8_t*>(p.act + (size_t)m0 * p.K + (size_t)min(j + 3, st_main - 1) * KS);
        constexpr int XH = (SJ & 1) * 2;           // x[TS][XH], x[TS][XH+1] hold this tile's 4 chunks
        constexpr int TS = ((SJ >> 1) & 1) ^ 1;    // tiles j+2, j+3 of steps 0,1 belong to an odd group
        uint32_t t0 = 0, t1 = 0, d[4];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int s = 0; s < 32; ++s) {
            const int kk = s >> 4, g = s & 15, tm = g >> 2, tn = g & 3;
            acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[kk][tm], fb[kk][tn], acc[tm][tn], 0, 0, 0);
            // operand reads: second half of this step, then first half of the next step
            if (g < 8 && !(DBG & 8)) {
                const uint8_t* src = kk == 0 ? s_cur : s_nxt;
                const int ko = koff[kk == 0 ? 1 : 0];
                if (g < 4) fa[kk ^ 1][g] = *reinterpret_cast<const bf16x8_t*>(src + a_base + g * 32 * FROWB + ko);
                else fb[kk ^ 1][g - 4] = *reinterpret_cast<const bf16x8_t*>(src + b_base + (g - 4) * 32 * FROWB + ko);
            }
            // decode, software-pipelined over the 16 code pairs of the tile: pair pr = s/2 starts
            // (extract, spread) while pair pr-1 finishes (select bytes, look up)
            if (!(DBG & 2)) {
                const int pr = s >> 1;
                if ((s & 1) == 0) {
                    if (pr > 0) t1 = (t0 & MASK) | ORC;
                    t0 = __builtin_amdgcn_ubfe(x[TS][XH + (pr >> 3)], boff[(pr >> 2) & 1][pr & 3], fw);
                } else {
                    if (pr > 0) d[(pr - 1) & 3] = __builtin_amdgcn_perm(SH[TS], SL[TS], t1);
                    t0 = __umul24(t0, MUL);
                }
                if (s == 31) {
                    t1 = (t0 & MASK) | ORC;
                    d[3] = __builtin_amdgcn_perm(SH[TS], SL[TS], t1);
                }
                // chunk c is complete once pair 4c+3 is looked up (slot 8c+9)
                if (!(DBG & 4) && (s == 9 || s == 17 || s == 25 || s == 31))
                    *reinterpret_cast<uint4*>(s_dec + b_soff[s == 31 ? 3 : (s - 9) >> 3]) = make_uint4(d[0], d[1], d[2], d[3]);
            }
            if (!(DBG & 1) && (s == 1 || s == 3 || s == 5 || s == 7)) dma16_s(dma_base, a_voff[s >> 1], dma_dst + (s >> 1) * 1024);
            if ((SJ & 1) == 1 && s == 24) fetch_codes();                // requested two steps ago, landed one step ago
            if ((SJ & 1) == 1 && s == 28) make_tables(slot_c<TS ^ 1>{}, slot_c<(SJ == 3)>{});   // the group decoded next
            if ((SJ & 1) == 1 && s == 29) request_codes((j + 5) >> 1);  // the group after that
            __builtin_amdgcn_sched_barrier(0);
        }
        // Everything started before this step must have landed before the barrier publishes tile
        // j+2: the transfers younger than that are exactly the ones issued in this step.
        if (DBG & 64) {
            uint64_t tX, tA, tB, tC;
            asm volatile("s_memtime %0" : "=s"(tX) :: "memory");
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_memtime %0\n\ts_waitcnt lgkmcnt(0)" : "=s"(tA) :: "memory");
            if ((SJ & 1) == 0) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
            else asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
            asm volatile("s_memtime %0\n\ts_waitcnt lgkmcnt(0)" : "=s"(tB) :: "memory");
            __syncthreads();
            asm volatile("s_memtime %0\n\ts_waitcnt lgkmcnt(0)" : "=s"(tC) :: "memory");
            tm_issue += (uint32_t)(tX - tm_prev);
            tm_lds += (uint32_t)(tA - tX);
            tm_vm += (uint32_t)(tB - tA);
            tm_bar += (uint32_t)(tC - tB);
            tm_prev = tC;
        } else {
        if ((SJ & 1) == 0) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
        __syncthreads();
        }
    };

    // ---- prologue: tiles 0 and 1 complete, DMA of tile 2 started
    dma_act_any(0, 0);
    dma_act_any(1, 1);                       // K >= 64: there are at least two weight tiles
    if (st_main > 2) dma_act_any(2, 2);
    store_b_any(0, 0);
    store_b_any(1, 1);
    dma_wait_all();
    __syncthreads();

    // ---- weight steps
    int j = 0;
    if (wave_fast && st_main >= 16) {
        // tables for the group of tiles 2,3; codes of the group of tiles 4,5 requested
        request_codes(1);
        dma_wait_all();
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0), told to the compiler: nothing of the prologue is pending in the loop
        fetch_codes();
        make_tables(slot_c<1>{}, slot_c<1>{});
        request_codes(2);
        load_frags(0, 0, fa[0], fb[0]);
        if (DBG & 64) { asm volatile("s_memtime %0\n\ts_waitcnt lgkmcnt(0)" : "=s"(tm_prev) :: "memory"); tm_mid = tm_prev; }
        for (; j + 4 <= st_main; j += 4) {
            fast_step(slot_c<0>{}, j);
            fast_step(slot_c<1>{}, j + 1);
            fast_step(slot_c<2>{}, j + 2);
            fast_step(slot_c<3>{}, j + 3);
        }
        dma_wait_all();
    }
    for (; j < st_main; ++j) slow_step(j);

    // ---- LoRA steps: all RP/32 (<= 4) tiles of [t | B] are staged at once, then multiplied
    if (p.RP) {
        const int ne = p.RP / KS;
        for (int e = 0; e < ne; ++e) {
            dma_act_any(st_main + e, e);
            store_b_any(st_main + e, e);
        }
        dma_wait_all();
        __syncthreads();
        for (int e = 0; e < ne; ++e) {
            load_frags(e, 0, fa[0], fb[0]);
            load_frags(e, 1, fa[1], fb[1]);
            mma16(fa[0], fb[0]);
            mma16(fa[1], fb[1]);
        }
    }

    if ((DBG & 64) && tile == 0) {
        uint64_t tE;
        asm volatile("s_memtime %0\n\ts_waitcnt lgkmcnt(0)" : "=s"(tE) :: "memory");
        if (lane == 0) {
            uint32_t* o = reinterpret_cast<uint32_t*>(p.out) + wave * 8;
            o[0] = tm_issue; o[1] = tm_lds; o[2] = tm_vm; o[3] = tm_bar;
            o[4] = (uint32_t)(tm_mid - tm_begin); o[5] = (uint32_t)(tm_prev - tm_mid); o[6] = (uint32_t)(tE - tm_prev); o[7] = 0;
        }
    } else
    if (DBG & 32) {   // timing ablation: keep the MFMAs alive without the epilogue stores
        float sum = 0.0f;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int jj = 0; jj < 4; ++jj)
#pragma unroll
                for (int v = 0; v < 16; ++v) sum += acc[i][jj][v];
        if (sum == 12345.678f) p.out[0] = 1;
    } else {
        store_out(acc, p.out, p.N, p.M, p.N, m0, n0);
    }
}

hipError_t launch_gemm_fwd(const GemmParams& p, hipStream_t st) {
    static const int dbg = getenv("LOWRA_DBG") ? atoi(getenv("LOWRA_DBG")) : 0;
    const dim3 grid(((p.N + BN - 1) / BN) * ((p.M + BM - 1) / BM));
#define LAUNCH(D) case D: { static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(linear_fwd_kernel<D>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)kFwdSmem); if (attr != hipSuccess) return attr; linear_fwd_kernel<D><<<grid, dim3(NTHREADS), kFwdSmem, st>>>(p); break; }
    switch (dbg) { LAUNCH(0) LAUNCH(1) LAUNCH(2) LAUNCH(7) LAUNCH(32) LAUNCH(39) LAUNCH(47) LAUNCH(64) LAUNCH(65) LAUNCH(66) LAUNCH(68) LAUNCH(72) LAUNCH(71) LAUNCH(79) default: return hipErrorInvalidValue; }
    return hipGetLastError();
}

}  // namespace lowra
