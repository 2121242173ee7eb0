// Small-token forward (M <= 16):  y = [x | s x A^T] [What | B]^T, streaming the packed codes once.
//
// Bandwidth-bound: per weight the method moves bits/8 + 1/16 bytes (codes + fp32 group scale),
// so the arithmetic has to stay out of the way.  The tokens are padded to 16 and the products
// run on v_mfma_f32_16x16x32_bf16 with the WEIGHTS as the row operand: a lane decodes 8 codes of
// its own row straight into the operand registers (no LDS round trip), the activations sit in
// registers for the whole kernel, and the group absmax is applied to the 16x16 partial sums once
// per 64-wide group instead of to every weight:  y[m,n] = sum_g a[n,g] sum_{k in g} x[m,k] M[c].
//
// Workgroup = 64 output channels (4 MFMA row tiles, taken in the width-sorted order of their
// 256-row tile so a wavefront sees one width) x all of K; its wavefronts split K and meet in LDS.
#include "gemm_common.h"

namespace lowra {

typedef float floatx4v_t __attribute__((ext_vector_type(4)));

constexpr int GV_ROWS = 64;          // output channels per workgroup
constexpr int GV_MAXSTEPS = 32;      // activation fragments a wavefront keeps in registers

template <int W>
__global__ __launch_bounds__(W * 64) void gemv_fwd_kernel(GemvParams p) {
    extern __shared__ __align__(16) uint8_t gv_smem[];
    float (*part)[GV_ROWS][17] = reinterpret_cast<float (*)[GV_ROWS][17]>(gv_smem);                  // [wave][row][token] partial sums (+1 pad)
    float (*stab)[16][TAB_LD] = reinterpret_cast<float (*)[16][TAB_LD]>(gv_smem + (size_t)W * GV_ROWS * 17 * 4);  // 4-bit rows: 16 levels
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 15, kg = lane >> 4;
    const int row0 = blockIdx.x * GV_ROWS;

    const int steps_all = p.K / 32;
    const int s_lo = wave * p.steps_per_wave;
    const int nsteps = min(p.steps_per_wave, max(steps_all - s_lo, 0));

    // activations of my K slice: lane (token i, kg) holds x[i][32 (s_lo+s) + 8 kg .. +8)
    bf16x8_t xf[GV_MAXSTEPS];
    const bf16x8_t zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int s = 0; s < GV_MAXSTEPS; ++s) {
        xf[s] = zero8;
        if (s < nsteps && i < p.M)
            xf[s] = *reinterpret_cast<const bf16x8_t*>(p.x + (size_t)i * p.K + (size_t)(s_lo + s) * 32 + kg * 8);
    }

    for (int nt = 0; nt < GV_ROWS / 16; ++nt) {
        // my row of this 16-row tile (operand row i) and the 4 rows whose sums I accumulate
        const int idx = row0 + nt * 16 + i;
        const int tile0 = idx & ~255;
        const int n = tile0 + p.tile_order[idx];
        const bool row_ok = n < p.N;
        const int nc = row_ok ? n : p.N - 1;
        const RowInfo ri = p.rows[nc];
        const int bits = ri.bits();
        const uint8_t* rowp = p.packed + ri.offset;
        const float* mrow = p.mappings + (size_t)ri.cb() * kTableStride;
        const float* amp[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int idv = row0 + nt * 16 + 4 * kg + v;
            const int nv = (idv & ~255) + p.tile_order[idv];
            amp[v] = p.absmax + (size_t)(nv < p.N ? nv : p.N - 1) * p.G;
        }
        const bool any4 = __builtin_amdgcn_ballot_w64(bits == 4) != 0;

        // unscaled levels of my row as byte tables (1-/2-bit), or as an LDS table (4-bit)
        float lev[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) lev[q] = (row_ok && q < (1 << bits) && bits != 4) ? mrow[q] : 0.0f;
        const bool two = bits == 2;
        const uint32_t P01 = pack_bf16x2(lev[0], lev[1]), P23 = pack_bf16x2(lev[2], lev[3]);
        const uint32_t SL = __builtin_amdgcn_perm(P23, P01, two ? 0x06040200u : 0x03010200u);
        const uint32_t SH = __builtin_amdgcn_perm(P23, P01, two ? 0x07050301u : 0x03010200u);
        const uint32_t fw = two ? 4u : 2u;
        const uint32_t MUL = two ? 0x404101u : 0x808101u, MASK = two ? 0x03030303u : 0x01010101u;
        const uint32_t ORC = two ? 0x04000400u : 0x02000200u;
        if (any4) {
            if (kg == 0) {
#pragma unroll
                for (int q = 0; q < 16; ++q) stab[wave][i][q] = (row_ok && bits == 4) ? mrow[q] : 0.0f;
            }
            // the table is written and read by lanes of this wavefront only
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }

        floatx4v_t tot = {0.0f, 0.0f, 0.0f, 0.0f}, grp = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int s = 0; s < GV_MAXSTEPS; ++s) {
            if (s < nsteps) {
                const int unit = (s_lo + s) * 4 + kg;            // which 8 codes of the row
                const uint32_t c = load_codes8(rowp, unit, bits);
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
                const floatx4v_t zero4v = {0.0f, 0.0f, 0.0f, 0.0f};
                grp = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf, xf[s], ((s & 1) == 0) ? zero4v : grp, 0, 0, 0);
                if (s & 1) {   // steps come in pairs: one 64-wide group done
                    const int g = (s_lo + s) >> 1;
#pragma unroll
                    for (int v = 0; v < 4; ++v) tot[v] += amp[v][g] * grp[v];
                }
            }
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) part[wave][nt * 16 + 4 * kg + v][i] = tot[v];
    }
    __syncthreads();

    // reduce over wavefronts, add the LoRA term, store bf16
    for (int o = threadIdx.x; o < GV_ROWS * 16; o += W * 64) {
        const int rl = o >> 4, m = o & 15;
        const int idx = row0 + rl;
        const int n = (idx & ~255) + p.tile_order[idx];
        if (m < p.M && n < p.N) {
            float v = 0.0f;
#pragma unroll
            for (int w = 0; w < W; ++w) v += part[w][rl][m];
            for (int j = 0; j < p.r; ++j)
                v += bf16_bits_to_float(p.t[(size_t)m * p.RP + j]) * bf16_bits_to_float(p.B[(size_t)n * p.r + j]);
            p.y[(size_t)m * p.N + n] = (uint16_t)(pack_bf16x2(v, 0.0f) & 0xffffu);
        }
    }
}

hipError_t launch_gemv_fwd(const GemvParams& p0, hipStream_t st) {
    GemvParams p = p0;
    const int steps_all = p.K / 32;
    const int W = (steps_all + 8 * GV_MAXSTEPS - 1) / (8 * GV_MAXSTEPS) > 1 ? 16 : 8;
    int per = (steps_all + W - 1) / W;
    per += per & 1;
    if (per > GV_MAXSTEPS) return hipErrorInvalidValue;     // K > 16384: the caller falls back to the GEMM path
    p.steps_per_wave = per;
    const dim3 grid((p.N + GV_ROWS - 1) / GV_ROWS);
    const size_t sh = (size_t)W * (GV_ROWS * 17 + 16 * TAB_LD) * sizeof(float);
    if (W == 8) {
        gemv_fwd_kernel<8><<<grid, dim3(8 * 64), sh, st>>>(p);
    } else {
        static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(gemv_fwd_kernel<16>),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, 16 * (GV_ROWS * 17 + 16 * TAB_LD) * 4);
        if (attr != hipSuccess) return attr;
        gemv_fwd_kernel<16><<<grid, dim3(16 * 64), sh, st>>>(p);
    }
    return hipGetLastError();
}

}  // namespace lowra
