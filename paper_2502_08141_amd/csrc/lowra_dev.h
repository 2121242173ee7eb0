// Device-side helpers shared by the LowRA HIP kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lowra {

constexpr int kGroup = 64;        // elements per absmax group (Sec. 4.1, groupwise normalization)
constexpr int kTableStride = 16;  // floats per table row: the 16 levels of a 4-bit codebook

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx2_t __attribute__((ext_vector_type(2)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));
typedef float floatx16_t __attribute__((ext_vector_type(16)));

// Per-channel record the layout uploads: byte offset of the row in the packed buffer,
// and width | codebook index << 8.
struct RowInfo {
    uint32_t offset;
    uint32_t bits_cb;
    __device__ __forceinline__ int bits() const { return (int)(bits_cb & 0xffu); }
    __device__ __forceinline__ int cb() const { return (int)(bits_cb >> 8); }
};

// Row record in the per-256-row-tile width-sorted order the small-token kernel walks: one 16-byte
// load gives everything needed to find and decode a row (n < 0 marks padding past the last row).
struct SortedRow {
    uint32_t offset;
    uint32_t bits_cb;
    int32_t n;
    int32_t pad;
};

// Row record of the streaming small-token kernel's class-sorted order (n < 0 marks a padding row; its
// offset is that of a real row of the same class, so loads through it stay in bounds).
struct GvRow {
    uint32_t offset;
    int32_t n;
};
constexpr int kGvMaxClasses = 4;

// Two fp32 -> packed bf16 pair, round to nearest even (v_cvt_pk_bf16_f32); lo lands in bits 0-15.
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    floatx2_t v = {lo, hi};
    bf16x2_t h = __builtin_convertvector(v, bf16x2_t);
    return __builtin_bit_cast(uint32_t, h);
}

__device__ __forceinline__ float bf16_bits_to_float(uint32_t h16) {
    return __builtin_bit_cast(float, h16 << 16);
}

// Decode 8 consecutive codes of width `bits` held in the low 8*bits bits of `c`
// (App. A.2: unpack, table lookup, multiply by absmax) into 8 bf16, packed as 4 dwords.
// `tab` points at the channel's mapping row (LDS or registers-backed memory).
__device__ __forceinline__ uint4 decode8_bf16(uint32_t c, int bits, const float* tab, float a) {
    const uint32_t mask = (1u << bits) - 1u;
    float w[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) w[i] = tab[(c >> (i * bits)) & mask] * a;
    uint4 r;
    r.x = pack_bf16x2(w[0], w[1]);
    r.y = pack_bf16x2(w[2], w[3]);
    r.z = pack_bf16x2(w[4], w[5]);
    r.w = pack_bf16x2(w[6], w[7]);
    return r;
}

// Streaming accesses: data read or written exactly once goes past the caches' usual retention
// (nontemporal hint), so it does not push out what other wavefronts will read again.
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void store16_stream(void* p, uint4 v) {
    __builtin_nontemporal_store(u32x4_t{v.x, v.y, v.z, v.w}, reinterpret_cast<u32x4_t*>(p));
}
__device__ __forceinline__ void store16_stream(void* p, float4 v) {
    __builtin_nontemporal_store(f32x4_t{v.x, v.y, v.z, v.w}, reinterpret_cast<f32x4_t*>(p));
}
__device__ __forceinline__ float4 load16_stream(const float4* p) {
    const f32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}

// Load the 8*bits bits of codes that cover elements [8u, 8u+8) of a packed row.
__device__ __forceinline__ uint32_t load_codes8(const uint8_t* row, int u, int bits) {
    if (bits == 1) return row[u];
    if (bits == 2) return reinterpret_cast<const uint16_t*>(row)[u];
    return reinterpret_cast<const uint32_t*>(row)[u];
}

// ---- cross-lane helpers of the reduction kernels (learner, error table)
template <int CTRL>
__device__ __forceinline__ float dpp_max_f32(float x) {
    const int v = __builtin_bit_cast(int, x);
    return fmaxf(x, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(v, v, CTRL, 0xf, 0xf, true)));
}
template <int CTRL>
__device__ __forceinline__ double dpp_add_f64(double x) {
    const long long v = __builtin_bit_cast(long long, x);
    const int lo = (int)(v & 0xffffffffll), hi = (int)(v >> 32);
    const int lo2 = __builtin_amdgcn_update_dpp(lo, lo, CTRL, 0xf, 0xf, true);
    const int hi2 = __builtin_amdgcn_update_dpp(hi, hi, CTRL, 0xf, 0xf, true);
    return x + __builtin_bit_cast(double, ((long long)hi2 << 32) | (unsigned int)lo2);
}
// sum over the 64 lanes of a wavefront, every lane gets the result (fixed order)
__device__ __forceinline__ double wave_sum(double x) {
    x = dpp_add_f64<0xB1>(x);      // quad_perm [1,0,3,2]
    x = dpp_add_f64<0x4E>(x);      // quad_perm [2,3,0,1]
    x = dpp_add_f64<0x124>(x);     // row_ror:4
    x = dpp_add_f64<0x128>(x);     // row_ror:8
    x += __shfl_xor(x, 16);
    x += __shfl_xor(x, 32);
    return x;
}

}  // namespace lowra
