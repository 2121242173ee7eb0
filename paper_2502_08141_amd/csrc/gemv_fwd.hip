// Small-token forward (M <= 16):  y = [x | s x A^T] [What | B]^T, streaming the packed codes once.
//
// Bandwidth-bound: per weight the method moves bits/8 + 1/16 bytes (codes + fp32 group scale),
// so the arithmetic has to stay out of the way and the loads have to be in flight all at once:
// a whole Llama-sized matrix is only a few MB, about what the chip must have outstanding to
// cover one HBM round trip.  Every wavefront therefore issues ALL its loads for a chunk of the
// contraction (codes, group scales, levels, activations) before it touches the first result.
//
// Products run on v_mfma_f32_16x16x32_bf16 with the tokens padded to 16: a lane decodes 8 codes
// of its own weight row straight into the operand registers (no LDS round trip) and, because the
// result column of a lane is that same row, applies the group absmax to the partial sums once per
// 64-wide group instead of to every weight:  y[m,n] = sum_g a[n,g] sum_{k in g} x[m,k] M[c].
//
// Workgroup = 16 NT output channels (NT MFMA tiles, walked in the width-sorted order of their
// 256-row tile so a wavefront sees one width) x all of K; its W wavefronts split K and meet in LDS.
#include "gemm_common.h"

namespace lowra {

typedef float floatx4v_t __attribute__((ext_vector_type(4)));

constexpr int GV_CHUNK = 16;      // 32-wide steps a wavefront has in flight at once

template <int W, int NT>
__global__ __launch_bounds__(W * 64) void gemv_fwd_kernel(GemvParams p) {
    extern __shared__ __align__(16) uint8_t gv_smem[];
    constexpr int ROWS = NT * 16;
    float (*part)[ROWS][17] = reinterpret_cast<float (*)[ROWS][17]>(gv_smem);                               // [wave][row][token]
    float (*stab)[16][TAB_LD] = reinterpret_cast<float (*)[16][TAB_LD]>(gv_smem + (size_t)W * ROWS * 17 * 4);  // 4-bit rows: 16 levels
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 15, kg = lane >> 4;
    const int row0 = blockIdx.x * ROWS;

    // my rows (operand row i of each tile; also the result column I accumulate)
    SortedRow rec[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) rec[nt] = p.sorted_rows[row0 + nt * 16 + i];

    const int steps_all = p.K / 32;
    const int s_begin = wave * p.steps_per_wave;
    const int s_end = min(s_begin + p.steps_per_wave, steps_all);

    floatx4v_t tot[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) tot[nt] = floatx4v_t{0.0f, 0.0f, 0.0f, 0.0f};

    for (int s0 = s_begin; s0 < s_end; s0 += GV_CHUNK) {
        const int ns = min(GV_CHUNK, s_end - s0);               // even: slices start and end on group borders
        // ---- issue every load of this chunk
        // (addresses past the slice are clamped onto its last step instead of being predicated, so
        // nothing below branches and the loads go out back to back; the extra values are never used)
        bf16x8_t xf[GV_CHUNK];
        const bf16x8_t zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
        const uint16_t* xrow = p.x + (size_t)(i < p.M ? i : 0) * p.K + kg * 8;
#pragma unroll
        for (int s = 0; s < GV_CHUNK; ++s) {
            const int sg = s0 + (s < ns ? s : ns - 1);
            xf[s] = *reinterpret_cast<const bf16x8_t*>(xrow + (size_t)sg * 32);
        }
        uint32_t codes[NT][GV_CHUNK];
        float sc[NT][GV_CHUNK / 2];
        float4 lv[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int bits = (int)(rec[nt].bits_cb & 0xffu);
            const uint8_t* rowp = p.packed + rec[nt].offset;
            const float* amp = p.absmax + (size_t)(rec[nt].n < 0 ? 0 : rec[nt].n) * p.G + (s0 >> 1);
            lv[nt] = *reinterpret_cast<const float4*>(p.mappings + (size_t)(rec[nt].bits_cb >> 8) * kTableStride);
#pragma unroll
            for (int s = 0; s < GV_CHUNK; ++s) {
                const int sg = s0 + (s < ns ? s : ns - 1);
                const int unit = sg * 4 + kg;
                // width-specific load sizes without a branch: 1, 2 or 4 bytes of an aligned dword
                const uint32_t byte_off = (uint32_t)unit * (uint32_t)bits;
                const uint32_t dw = *reinterpret_cast<const uint32_t*>(rowp + (byte_off & ~3u));
                codes[nt][s] = dw >> ((byte_off & 3u) * 8u);
            }
#pragma unroll
            for (int g = 0; g < GV_CHUNK / 2; ++g) sc[nt][g] = amp[2 * g < ns ? g : 0];
        }
        if (i >= p.M) {
#pragma unroll
            for (int s = 0; s < GV_CHUNK; ++s) xf[s] = zero8;
        }
        // ---- consume
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int bits = (int)(rec[nt].bits_cb & 0xffu);
            const bool row_ok = rec[nt].n >= 0;
            const bool any4 = __builtin_amdgcn_ballot_w64(bits == 4) != 0;
            const bool two = bits == 2;
            const bool small = row_ok && bits != 4;
            const float l0 = small ? lv[nt].x : 0.0f, l1 = small ? lv[nt].y : 0.0f;
            const float l2 = (small && two) ? lv[nt].z : 0.0f, l3 = (small && two) ? lv[nt].w : 0.0f;
            const uint32_t P01 = pack_bf16x2(l0, l1), P23 = pack_bf16x2(l2, l3);
            const uint32_t SL = __builtin_amdgcn_perm(P23, P01, two ? 0x06040200u : 0x03010200u);
            const uint32_t SH = __builtin_amdgcn_perm(P23, P01, two ? 0x07050301u : 0x03010200u);
            const uint32_t fw = two ? 4u : 2u;
            const uint32_t MUL = two ? 0x404101u : 0x808101u, MASK = two ? 0x03030303u : 0x01010101u;
            const uint32_t ORC = two ? 0x04000400u : 0x02000200u;
            if (any4) {
                // 16 levels of a 4-bit row -> LDS table; four 16-byte loads in flight together
                const float4* mrow = reinterpret_cast<const float4*>(p.mappings + (size_t)(rec[nt].bits_cb >> 8) * kTableStride);
                const float4 t0 = mrow[0], t1 = mrow[1], t2 = mrow[2], t3 = mrow[3];
                if (kg == 0) {
                    const bool use = row_ok && bits == 4;
                    float* dst = &stab[wave][i][0];
                    const float tv[16] = {t0.x, t0.y, t0.z, t0.w, t1.x, t1.y, t1.z, t1.w, t2.x, t2.y, t2.z, t2.w, t3.x, t3.y, t3.z, t3.w};
#pragma unroll
                    for (int q = 0; q < 16; ++q) dst[q] = use ? tv[q] : 0.0f;
                }
                // the table is written and read by lanes of this wavefront only
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            }
            floatx4v_t grp = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int s = 0; s < GV_CHUNK; ++s) {
                if (s < ns) {
                    const uint32_t c = codes[nt][s];
                    bf16x8_t wf;
                    if (!any4) {
                        uint32_t d[4];
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const uint32_t q = __builtin_amdgcn_ubfe(c, j * fw, fw);
                            d[j] = __builtin_amdgcn_perm(SH, SL, (__umul24(q, MUL) & MASK) | ORC);
                        }
                        wf = __builtin_bit_cast(bf16x8_t, make_uint4(d[0], d[1], d[2], d[3]));
                    } else {
                        uint4 dv;
                        if (bits == 4) dv = decode8_bf16(c, 4, &stab[wave][i][0], 1.0f);
                        else if (bits == 2) dv = decode8_w2(c, SL, SH);
                        else dv = decode8_w1(c, SL);
                        wf = __builtin_bit_cast(bf16x8_t, dv);
                    }
                    // tokens are the rows, weight rows the columns: lane (i, kg) gets y[4 kg + v][row i]
                    const floatx4v_t zero4v = {0.0f, 0.0f, 0.0f, 0.0f};
                    grp = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xf[s], wf, ((s & 1) == 0) ? zero4v : grp, 0, 0, 0);
                    if (s & 1) {   // steps come in pairs: one 64-wide group done
#pragma unroll
                        for (int v = 0; v < 4; ++v) tot[nt][v] += sc[nt][s >> 1] * grp[v];
                    }
                }
            }
        }
    }
    // LoRA term as an extension of the contraction: [x | t] against [What | B], t = s x A^T.
    // B comes with rows of RP entries (zero past r), so 16-byte operand loads are always in bounds.
    if (wave == 0 && p.RP > 0) {
        for (int e0 = 0; e0 < p.RP; e0 += 32) {
            const bf16x8_t zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
            bf16x8_t tf = *reinterpret_cast<const bf16x8_t*>(p.t + (size_t)(i < p.M ? i : 0) * p.RP + e0 + kg * 8);
            if (i >= p.M) tf = zero8;
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const int n = rec[nt].n;
                bf16x8_t bfr = *reinterpret_cast<const bf16x8_t*>(p.B + (size_t)(n < 0 ? 0 : n) * p.RP + e0 + kg * 8);
                if (n < 0) bfr = zero8;
                tot[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(tf, bfr, tot[nt], 0, 0, 0);
            }
        }
    }
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int v = 0; v < 4; ++v) part[wave][nt * 16 + i][4 * kg + v] = tot[nt][v];
    __syncthreads();

    // reduce over wavefronts, store bf16
    for (int o = threadIdx.x; o < ROWS * 16; o += W * 64) {
        const int rl = o >> 4, m = o & 15;
        const int n = p.sorted_rows[row0 + rl].n;
        if (m < p.M && n >= 0) {
            float v = 0.0f;
#pragma unroll
            for (int w = 0; w < W; ++w) v += part[w][rl][m];
            p.y[(size_t)m * p.N + n] = (uint16_t)(pack_bf16x2(v, 0.0f) & 0xffffu);
        }
    }
}

template <int W, int NT>
static hipError_t launch_one(const GemvParams& p, hipStream_t st) {
    constexpr size_t sh = (size_t)W * (NT * 16 * 17 + 16 * TAB_LD) * sizeof(float);
    static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(gemv_fwd_kernel<W, NT>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)sh);
    if (attr != hipSuccess) return attr;
    const dim3 grid((p.N + NT * 16 - 1) / (NT * 16));
    gemv_fwd_kernel<W, NT><<<grid, dim3(W * 64), sh, st>>>(p);
    return hipGetLastError();
}

hipError_t launch_gemv_fwd(const GemvParams& p0, hipStream_t st) {
    GemvParams p = p0;
    const int steps_all = p.K / 32;
    const bool wide = steps_all > 8 * GV_CHUNK;      // K > 4096: 16 wavefronts split the contraction
    const int W = wide ? 16 : 8;
    int per = (steps_all + W - 1) / W;
    per += per & 1;
    p.steps_per_wave = per;
    // more tokens -> more rows per workgroup, so the activations are re-read by fewer workgroups
    const bool two_tiles = p.M > 4;
    if (wide) return two_tiles ? launch_one<16, 2>(p, st) : launch_one<16, 1>(p, st);
    return two_tiles ? launch_one<8, 2>(p, st) : launch_one<8, 1>(p, st);
}

}  // namespace lowra
