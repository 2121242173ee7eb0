// Pieces shared by the streaming small-token kernels (forward and input gradient): the unit table, the
// decode tables in LDS, the global -> LDS transfer helpers and the host-side strip bookkeeping.
#pragma once
#include <algorithm>
#include <vector>

#include "gemm_common.h"

namespace lowra {

constexpr int GS_W = 16;                 // wavefronts per workgroup = 256-column blocks per K-chunk
constexpr int GS_THREADS = GS_W * 64;
constexpr int GS_MAXSEG = 4;             // K-chunks of one row at most (K <= 16384)
constexpr int GS_MAXTAB = 3;             // decode tables (codebooks) in LDS
constexpr int GS_TABB = 16384;           // bytes of one decode table: 256 entries x 64 bytes
constexpr int GS_TROW = 32;              // entries per token row of the rank-r intermediate (rank padded to 32)
constexpr int GS_RECB = 128;             // record slot: 16 records of 8 bytes

struct GsTabs {
    int nslot;                     // codebooks (table rows of `mappings`) with a table in LDS
    int bits[GS_MAXTAB];           // width of codebook c
    int scale_bf16;                // the group scales are bf16 (8 bytes per channel and 256 columns) instead of fp32 (16)
};

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
// a pointer the caller knows to be wavefront-uniform, forced into scalar registers
__device__ __forceinline__ const void* gs_uniform(const void* p) {
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<const void*>(((uint64_t)hi << 32) | lo);
}
// 4 bytes per lane, the low 32 lanes only: lane l's dword lands at lds_base + 4 l
__device__ __forceinline__ void gs_dma4_low32(const void* sbase, uint32_t voff, uint32_t lds_base_uniform) {
    uint64_t saved;
    asm volatile("s_mov_b64 %0, exec\n\ts_mov_b64 exec, 0xffffffff\n\ts_mov_b32 m0, %3\n\ts_nop 0\n\t"
                 "global_load_lds_dword %1, %2\n\ts_mov_b64 exec, %0"
                 : "=&s"(saved) : "v"(voff), "s"(sbase), "s"(lds_base_uniform) : "memory");
}
// 16 bytes per lane, the low 32 lanes only: lane l's 16 bytes land at lds_base + 16 l
__device__ __forceinline__ void gs_dma16_low32(const void* sbase, uint32_t voff, uint32_t lds_base_uniform) {
    uint64_t saved;
    asm volatile("s_mov_b64 %0, exec\n\ts_mov_b64 exec, 0xffffffff\n\ts_mov_b32 m0, %3\n\ts_nop 0\n\t"
                 "global_load_lds_dwordx4 %1, %2\n\ts_mov_b64 exec, %0"
                 : "=&s"(saved) : "v"(voff), "s"(sbase), "s"(lds_base_uniform) : "memory");
}

// Descriptors are read-only for a whole launch: reading them through the constant address space lets the
// compiler use scalar loads.
typedef const __attribute__((address_space(4))) int* gs_cint_t;

// One unit of the launch's work list, built once (on the host for a batch, by the set-up kernel for a single
// call): the control flow of the streaming loop is a table read, not arithmetic.
struct GsUnit {
    uint32_t rows_off;       // byte offset of the strip's 16 records in its segment's record array
    uint32_t seg;            // segment of the unit
    uint32_t flags;          // width (bits 0-3) | half << 4 | ends its strip << 5 | table index << 6 | (strip sequence number & 31) << 8
    uint32_t pad;
};
typedef const __attribute__((address_space(4))) GsUnit* gs_cunit_t;
__device__ __forceinline__ GsUnit gs_load_unit(gs_cunit_t p) {
    GsUnit u;
    u.rows_off = p->rows_off; u.seg = p->seg; u.flags = p->flags; u.pad = 0u;
    return u;
}
__host__ __device__ inline uint32_t gs_unit_flags(int bits, int half, int last, int tab, int strip_seq) {
    return (uint32_t)bits | ((uint32_t)half << 4) | ((uint32_t)last << 5) | ((uint32_t)tab << 6) | (((uint32_t)strip_seq & 31u) << 8);
}

// LDS address of the table entry of byte p of zz: (byte << 6) | lane's copy | table
__device__ __forceinline__ uint32_t gs_entry(uint32_t zz, int p, uint32_t tb) {
    const uint32_t sh = p == 0 ? zz << 6 : zz >> (8 * p - 6);
    return (sh & 0x3FC0u) | tb;
}

// Tables of unscaled bf16 levels (App. A.2's lookup, one byte of codes at a time), one per codebook at
// smem + c * GS_TABB: entry e (a byte holding 8, 4 or 2 codes) at e * 64 holds the levels of all its codes
// (16, 8 or 4 bytes) in 4, 8 or 16 copies, so that neighbouring lanes read different banks.  All threads of
// the workgroup call it; the caller synchronises afterwards.
__device__ __forceinline__ void gs_fill_tables(uint8_t* smem, const float* __restrict__ mappings, const GsTabs& tabs) {
#pragma unroll
    for (int c = 0; c < GS_MAXTAB; ++c) {                           // static indices: `tabs` stays in scalar registers
        if (c >= tabs.nslot) break;
        const float* mrow = mappings + (size_t)c * kTableStride;
        uint8_t* tb = smem + c * GS_TABB;
        if (tabs.bits[c] == 1) {          // 8 codes -> 8 bf16 (16 B), 4 copies
            const float l0 = mrow[0], l1 = mrow[1];
            for (int idx = threadIdx.x; idx < 256 * 4; idx += blockDim.x) {
                const int e = idx >> 2, q = idx & 3;
                *reinterpret_cast<uint4*>(tb + e * 64 + 16 * q) =
                    make_uint4(pack_bf16x2((e & 1) ? l1 : l0, (e & 2) ? l1 : l0), pack_bf16x2((e & 4) ? l1 : l0, (e & 8) ? l1 : l0),
                               pack_bf16x2((e & 16) ? l1 : l0, (e & 32) ? l1 : l0), pack_bf16x2((e & 64) ? l1 : l0, (e & 128) ? l1 : l0));
            }
        } else if (tabs.bits[c] == 2) {   // 4 codes -> 4 bf16 (8 B), 8 copies
            for (int idx = threadIdx.x; idx < 256 * 8; idx += blockDim.x) {
                const int e = idx >> 3, q = idx & 7;
                *reinterpret_cast<uint2*>(tb + e * 64 + 8 * q) =
                    make_uint2(pack_bf16x2(mrow[e & 3], mrow[(e >> 2) & 3]), pack_bf16x2(mrow[(e >> 4) & 3], mrow[e >> 6]));
            }
        } else {                          // 2 codes -> 2 bf16 (4 B), 16 copies
            for (int idx = threadIdx.x; idx < 256 * 16; idx += blockDim.x) {
                const int e = idx >> 4, q = idx & 15;
                *reinterpret_cast<uint32_t*>(tb + e * 64 + 4 * q) = pack_bf16x2(mrow[e & 15], mrow[e >> 4]);
            }
        }
    }
}

// A cursor over the units of a workgroup's range.  The units of a segment come class by class (classes are sorted by
// width, the 4-bit ones last, two units per strip), so a cursor is (segment, unit within it) plus what follows from
// them; it changes class or segment only at the end of a class, and everything between is arithmetic on scalar
// registers: the loop reads no work list.  The fields are plain local variables named by a suffix (a struct, or a
// lambda that captures them, ends up in private memory):
//   seg, lu (unit within the segment), end (unit where the current class ends), left (units after this one in the
//   workgroup's range; 0: the cursor stays), bits, tab (width and table of the class), strip, half (of a 4-bit strip)
#define GS_CUR_DECL(X) int seg##X, lu##X, end##X, left##X, bits##X, tab##X, strip##X, half##X
// unit index of strip boundary s in a segment whose 4-bit strips start at f4
__device__ __forceinline__ int gs_unit_of_strip(int s, int f4) { return s <= f4 ? s : 2 * s - f4; }
// cursor X := unit LU of segment SEG (the first half of its strip)
#define GS_CUR_SEEK(X, SEG, LU)                                                                                   \
    do {                                                                                                          \
        const int seek_seg = (SEG), seek_lu = (LU);                                                               \
        const auto seek_p = segs + seek_seg;   /* a segment pointer in the constant address space */                                                                 \
        const int seek_f4 = seek_p->first4;                                                                       \
        const int e0 = gs_unit_of_strip(seek_p->cls_end[0], seek_f4), e1 = gs_unit_of_strip(seek_p->cls_end[1], seek_f4),   \
                  e2 = gs_unit_of_strip(seek_p->cls_end[2], seek_f4), e3 = gs_unit_of_strip(seek_p->cls_end[3], seek_f4);   \
        const int c0 = seek_p->cls_bits_cb[0], c1 = seek_p->cls_bits_cb[1], c2 = seek_p->cls_bits_cb[2], c3 = seek_p->cls_bits_cb[3]; \
        const int seek_cls = seek_lu < e0 ? c0 : seek_lu < e1 ? c1 : seek_lu < e2 ? c2 : c3;                     \
        seg##X = seek_seg; lu##X = seek_lu; half##X = 0;                                                          \
        end##X = seek_lu < e0 ? e0 : seek_lu < e1 ? e1 : seek_lu < e2 ? e2 : e3;                                  \
        strip##X = seek_lu <= seek_f4 ? seek_lu : seek_f4 + ((seek_lu - seek_f4) >> 1);                           \
        bits##X = seek_cls & 0xff; tab##X = seek_cls >> 8;                                                        \
    } while (0)
// Inside a run of passes a cursor moves without any test: its unit counter and its end-of-class test are settled
// after the run (GS_CUR_SETTLE), whose length the caller limits to what is left of the cursor's class.
// One pass of cursor X: ADV (0 / 1: the cursor moves), T4 (0 / 1: it moves through a 4-bit class).
#define GS_CUR_STEP(X, ADV, T4)                                                                                   \
    do {                                                                                                          \
        half##X ^= (T4);                                                                                          \
        strip##X += (ADV) - ((T4) & half##X);                                                                     \
    } while (0)
// after CNT passes in which cursor X moved: on to the next class or segment where its class ended
#define GS_CUR_SETTLE(X, CNT, ON_SEG)                                                                             \
    do {                                                                                                          \
        lu##X += (CNT); left##X -= (CNT);                                                                         \
        if (lu##X == end##X) {                                                                                    \
            if (lu##X == segs[seg##X].nunits) { GS_CUR_SEEK(X, seg##X + 1, 0); ON_SEG; }                          \
            else GS_CUR_SEEK(X, seg##X, lu##X);                                                                   \
        }                                                                                                         \
    } while (0)

// ring pointer one slot on
__device__ __forceinline__ uint32_t gs_ring_next(uint32_t p, uint32_t slot_bytes, uint32_t begin, uint32_t end) {
    return p + slot_bytes == end ? begin : p + slot_bytes;
}

// =============================================================================================== host side
static inline size_t gs_align(size_t v) { return (v + 255) & ~(size_t)255; }
static inline int gs_nchunks(const lowra_layout& L, int waves = GS_W) { return (L.K / 256 + waves - 1) / waves; }
// first strip of the 4-bit classes (classes are sorted by width): those strips count as two units
static inline int gs_first4(const lowra_layout& L) {
    int f = L.gv_nstrips;
    for (int c = kGvMaxClasses - 1; c >= 0; --c)
        if (c < L.gv_nclasses && (L.gv_cls_bits_cb[c] & 0xff) == 4) f = c == 0 ? 0 : L.gv_cls_end[c - 1];
    return f;
}
static inline int gs_units_per_seg(const lowra_layout& L) { return 2 * L.gv_nstrips - gs_first4(L); }
// width | table << 8 of strip `sidx`
static inline int gs_strip_class(const lowra_layout& L, int sidx) {
    int cls = L.gv_cls_bits_cb[0];
    for (int q = 0; q + 1 < kGvMaxClasses; ++q) if (sidx >= L.gv_cls_end[q]) cls = L.gv_cls_bits_cb[q + 1];
    return cls;
}

// one table of GS_TABB bytes per codebook, at c * GS_TABB (the lookup needs a 16 KB aligned base)
static inline GsTabs gs_tabs(const std::vector<uint8_t>& cb_bits, bool scale_bf16) {
    GsTabs t{};
    t.scale_bf16 = scale_bf16 ? 1 : 0;
    t.nslot = (int)std::min<size_t>(cb_bits.size(), GS_MAXTAB);
    for (int c = 0; c < t.nslot; ++c) t.bits[c] = cb_bits[(size_t)c];
    return t;
}

static inline int gs_compute_units() { return device_compute_units(); }

template <typename T>
static inline hipError_t gs_to_device(const std::vector<T>& v, T** out) {
    if (v.empty()) { *out = nullptr; return hipSuccess; }
    hipError_t e = hipMalloc(reinterpret_cast<void**>(out), v.size() * sizeof(T));
    if (e != hipSuccess) return e;
    return hipMemcpy(*out, v.data(), v.size() * sizeof(T), hipMemcpyHostToDevice);
}

// A streaming kernel counts its own global -> LDS transfers (s_waitcnt vmcnt with a constant): a register spill
// would put private-memory traffic of the compiler's into the same counter.  Refuse to run a build that has any,
// and allow the kernel the whole LDS.
static inline hipError_t gs_prepare_kernel(const void* kernel) {
    hipFuncAttributes fa;
    hipError_t e = hipFuncGetAttributes(&fa, kernel);
    if (e != hipSuccess) return e;
    if (fa.localSizeBytes != 0) return hipErrorInvalidDeviceFunction;
    return hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
}

// The streaming kernels take a matrix whose 16-row strips each have one class (at most 4 (width, table)
// classes and 3 tables), with K a multiple of 256 from 1024 to 16384.
static inline bool gs_layout_supported(const lowra_layout& L) {
    return L.gv_nstrips > 0 && L.K % 256 == 0 && L.K >= 1024 && L.K <= GS_MAXSEG * GS_W * 256 && L.C <= GS_MAXTAB && L.N > 0;
}

}  // namespace lowra
