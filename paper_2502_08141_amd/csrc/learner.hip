// Mapping/threshold learner (paper Sec. 5 "Weighted Lloyd's for LoRA Quantization", App. G):
// per output channel, weighted Lloyd-Max on the normalised weights u = w * (1/absmax) with the
// block's absmax as the weight of each of its 64 elements, started from given tables.
//   E-step  bin = number of thresholds strictly below u        (the quantizer's binning, App. A.1)
//   M-step  level_j = sum_bin_j a u / sum_bin_j a  (App. G; an empty bin keeps its level),
//           threshold_j = midpoint of levels j and j+1         (Sec. 5)
//   mse_t   = sum a (u - level(bin))^2 / sum a, for the initial tables (t = 0) and after each
//           iteration with that iteration's binning; stop after `iters` iterations or when the mse
//           does not go down (Sec. 5).
//
// Mapping: one workgroup per channel.  The row is read from HBM once (4 B/weight, the pass's
// algorithmic traffic) and stays in REGISTERS: a thread owns 8 consecutive weights of each of its
// NP 64-wide blocks' eighths (a block is 8 adjacent lanes), normalised exactly as in the quantize
// kernel.  Every iteration bins them against the thresholds and forms, per bin, sum a and sum a u
// in the thread's own column of a [bin][thread] table in LDS (written once per iteration for 1- and
// 2-bit rows, read-modify-write per element for 4-bit rows; no atomics, no bank conflicts, a fixed
// order).  The 16 x 2 column sums are then reduced by the four wavefronts in fp64, and one
// wavefront updates the tables.  The squared error never needs a second pass: sum a (u - m)^2 over
// a bin is sum a u^2 - 2 m sum a u + m^2 sum a.
//
// 1- and 2-bit rows: the 8 weights of an eighth share their block's absmax, so the thread counts
// them per bin and sums their u per bin, and multiplies by the absmax once per eighth.  With sorted
// thresholds bin j is "below threshold j but not below j - 1": the counts and sums are kept per
// THRESHOLD (number, and sum of u, of the weights above it) and the bins are their differences --
// exact for the counts, a difference of sums of at most 8 values in [-1, 1] for the others.
// 4-bit rows find the bin by bisection (thresholds in LDS).
#include "lowra_host.h"

namespace lowra {

constexpr int kLearnThreads = 256;
constexpr int kLearnMaxK = 16384;          // the row lives in registers: K / 256 per thread

// E-step of one thread for a 1- or 2-bit row: sums of a and a u per bin into column `tid` of
// col [2][nlmax][256] (nlmax = levels of the matrix's widest row).  uu[p] = my 8 normalised weights
// of pass p, aa[p] their block's absmax (0 for a pass past the row), us[p] the sum of the 8.
template <int BITS, int NP>
__device__ __forceinline__ void estep_narrow(const float* T_l, const float (&uu)[NP][8], const float (&aa)[NP], const float (&us)[NP],
                                             float* col, int tid, int nlmax) {
    constexpr int NL = 1 << BITS, NT = NL - 1;
    float T[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) T[j] = T_l[j];
    float s0[NL], s1[NL];
#pragma unroll
    for (int j = 0; j < NL; ++j) { s0[j] = 0.0f; s1[j] = 0.0f; }
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        int cnt[NT];
        float q[NT];
#pragma unroll
        for (int j = 0; j < NT; ++j) { cnt[j] = 0; q[j] = 0.0f; }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
#pragma unroll
            for (int j = 0; j < NT; ++j) {
                const bool above = T[j] < uu[p][i];
                cnt[j] += above ? 1 : 0;
                q[j] += above ? uu[p][i] : 0.0f;
            }
        }
        // bin 0: not above threshold 0; bin j: above j - 1 and not above j; last bin: above the last
        s0[0] += aa[p] * (float)(8 - cnt[0]);
        s1[0] += aa[p] * (us[p] - q[0]);
#pragma unroll
        for (int j = 1; j < NT; ++j) {
            s0[j] += aa[p] * (float)(cnt[j - 1] - cnt[j]);
            s1[j] += aa[p] * (q[j - 1] - q[j]);
        }
        s0[NT] += aa[p] * (float)cnt[NT - 1];
        s1[NT] += aa[p] * q[NT - 1];
    }
#pragma unroll
    for (int j = 0; j < NL; ++j) { col[j * kLearnThreads + tid] = s0[j]; col[(nlmax + j) * kLearnThreads + tid] = s1[j]; }
}

// the bin of u among 15 ascending thresholds in LDS: the number of thresholds strictly below u, by bisection
__device__ __forceinline__ int bin4(const float* T_l, float t3, float t7, float t11, float u) {
    const int b3 = (t7 < u) ? 1 : 0;
    int c = 2 * b3 + (((b3 ? t11 : t3) < u) ? 1 : 0);
    c = 2 * c + ((T_l[4 * c + 1] < u) ? 1 : 0);
    return 2 * c + ((T_l[2 * c] < u) ? 1 : 0);
}

// E-step of one thread for a 4-bit row: adds into its column of the table in LDS
template <int NP>
__device__ __forceinline__ void estep_wide(const float* T_l, const float (&uu)[NP][8], const float (&aa)[NP], float* col, int tid, int nlmax) {
    const float t3 = T_l[3], t7 = T_l[7], t11 = T_l[11];
#pragma unroll
    for (int j = 0; j < 16; ++j) { col[j * kLearnThreads + tid] = 0.0f; col[(nlmax + j) * kLearnThreads + tid] = 0.0f; }
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        if (aa[p] == 0.0f) continue;                               // a pass past the row, or a block of zeros: adds nothing
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int c = bin4(T_l, t3, t7, t11, uu[p][i]);
            col[c * kLearnThreads + tid] += aa[p];
            col[(nlmax + c) * kLearnThreads + tid] += aa[p] * uu[p][i];
        }
    }
}

// (short rows: 8 wavefronts per SIMD, so that one row's serial phases pass under the others' loads and binning)
template <int NP>
__global__ __launch_bounds__(kLearnThreads, NP <= 2 ? 8 : 1) void learn_tables_kernel(const RowInfo* __restrict__ rows,
                                                                    const float* __restrict__ W,
                                                                    const float* __restrict__ init_thresholds,
                                                                    const float* __restrict__ init_mappings,
                                                                    int iters, float* __restrict__ thr_out,
                                                                    float* __restrict__ map_out,
                                                                    float* __restrict__ mse_out, int K, int nlmax) {
    extern __shared__ __align__(16) uint8_t lsm[];
    // LDS: reduced sums (fp64) [2][16] + 2 | tables T[16], M[16] | flag (4 words) | column sums [2][nlmax][256]
    double* red = reinterpret_cast<double*>(lsm);
    float* T_l = reinterpret_cast<float*>(red + 2 * 16 + 2);
    float* M_l = T_l + 16;
    int* flag = reinterpret_cast<int*>(M_l + 16);
    float* col = reinterpret_cast<float*>(flag + 4);

    const int n = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const RowInfo ri = rows[n];
    const int bits = ri.bits(), nl = 1 << bits, nt = nl - 1;
    const float4* w4 = reinterpret_cast<const float4*>(W + (size_t)n * K);
    const int units = K >> 3;

    // ---- the row: every pass requested before the first is used; normalised weights and block scales stay in
    // registers; sum a and sum a u^2 on the way
    float uu[NP][8], aa[NP], us[NP];
    {
        float4 q0[NP], q1[NP];
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const int un = min(p * kLearnThreads + tid, units - 1);             // past the row: clamped, unused
            q0[p] = w4[2 * un]; q1[p] = w4[2 * un + 1];
        }
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const bool ok = p * kLearnThreads + tid < units;      // units is a multiple of 8: the 8 lanes of a block agree
            const float v[8] = {q0[p].x, q0[p].y, q0[p].z, q0[p].w, q1[p].x, q1[p].y, q1[p].z, q1[p].w};
            float a = 0.0f;
#pragma unroll
            for (int i = 0; i < 8; ++i) a = fmaxf(a, fabsf(v[i]));
            a = dpp_max_f32<0xB1>(a);                             // lanes l ^ 1
            a = dpp_max_f32<0x4E>(a);                             // l ^ 2
            a = fmaxf(a, __shfl_xor(a, 4));
            a = ok ? a : 0.0f;
            const float inv = (a == 0.0f) ? 0.0f : 1.0f / a;      // IEEE division, once per block
            float s = 0.0f;
#pragma unroll
            for (int i = 0; i < 8; ++i) { uu[p][i] = v[i] * inv; s += uu[p][i]; }
            aa[p] = a; us[p] = s;
        }
    }
    double sa = 0.0, sauu = 0.0;
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        float q = 0.0f;                                            // 8 squares of values in [-1, 1]: fp32 is plenty, fp64 from there on
#pragma unroll
        for (int i = 0; i < 8; ++i) q += uu[p][i] * uu[p][i];
        sa += 8.0 * (double)aa[p]; sauu += (double)aa[p] * (double)q;
    }
    if (tid < 16) {
        T_l[tid] = tid < nt ? init_thresholds[(size_t)ri.cb() * kTableStride + tid] : __builtin_inff();
        M_l[tid] = tid < nl ? init_mappings[(size_t)ri.cb() * kTableStride + tid] : 0.0f;
    }
    sa = wave_sum(sa); sauu = wave_sum(sauu);
    // totals over the four wavefronts, through the reduced-sums area
    if (lane == 0) { red[2 * wave] = sa; red[2 * wave + 1] = sauu; }
    __syncthreads();
    const double wsum = red[0] + red[2] + red[4] + red[6];
    const double s2 = red[1] + red[3] + red[5] + red[7];
    __syncthreads();

    float* mse_row = mse_out + (size_t)n * (iters + 1);
    double mse_prev = 0.0;
    int done = 0;
    if (wsum > 0.0) {
        for (int t = 1; t <= iters; ++t) {
            // E-step: my column of the [bin][thread] sums
            if (bits == 4) estep_wide<NP>(T_l, uu, aa, col, tid, nlmax);
            else if (bits == 2) estep_narrow<2, NP>(T_l, uu, aa, us, col, tid, nlmax);
            else estep_narrow<1, NP>(T_l, uu, aa, us, col, tid, nlmax);
            __syncthreads();
            // column sums in fp64: the 2 x nl (table, bin) pairs are dealt over the four wavefronts
            for (int pi = wave; pi < 2 * nl; pi += kLearnThreads / 64) {          // uniform over the wavefront
                const int tab = pi >= nl ? 1 : 0, bin = pi - tab * nl;
                double s = 0.0;
#pragma unroll
                for (int i = 0; i < kLearnThreads / 64; ++i) s += (double)col[(tab * nlmax + bin) * kLearnThreads + lane + 64 * i];
                s = wave_sum(s);
                if (lane == 0) red[tab * 16 + bin] = s;
            }
            __syncthreads();
            // M-step and error terms, one lane per level (wavefront 0); thresholds and the stop
            // decision by lane 0
            if (wave == 0) {
                double e_old = 0.0, e_new = 0.0;
                float mn = 0.0f;
                if (lane < nl) {
                    const double S0 = red[lane], S1 = red[16 + lane], m0 = (double)M_l[lane];
                    e_old = -2.0 * m0 * S1 + m0 * m0 * S0;
                    mn = S0 > 0.0 ? (float)(S1 / S0) : M_l[lane];
                    const double m1 = (double)mn;
                    e_new = -2.0 * m1 * S1 + m1 * m1 * S0;
                }
                e_old = wave_sum(e_old) + s2; e_new = wave_sum(e_new) + s2;
                const float mnext = __shfl_down(mn, 1);
                if (lane < nl) M_l[lane] = mn;
                if (lane < nt) T_l[lane] = (float)(((double)mn + (double)mnext) * 0.5);
                if (lane == 0) {
                    if (t == 1) { mse_prev = e_old / wsum; mse_row[0] = (float)mse_prev; }
                    const double mse_t = fmax(e_new, 0.0) / wsum;
                    mse_row[t] = (float)mse_t;
                    flag[0] = !(mse_t < mse_prev);                 // the MSE stopped going down
                    mse_prev = mse_t;
                }
            }
            __syncthreads();
            done = t;
            if (flag[0]) break;                                     // uniform: read after the barrier
            __syncthreads();                                        // flag is rewritten in the next iteration
        }
    }
    // ---- results
    if (iters == 0 && wsum > 0.0) {          // only the error of the initial tables: one binning pass with the decoded level
        double e = 0.0;
#pragma unroll
        for (int p = 0; p < NP; ++p)
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                int c = 0;
                for (int j = 0; j < nt; ++j) c += (T_l[j] < uu[p][i]) ? 1 : 0;
                const double d = (double)uu[p][i] - (double)M_l[c];
                e += (double)aa[p] * d * d;
            }
        e = wave_sum(e);
        __syncthreads();
        if (lane == 0) red[wave] = e;
        __syncthreads();
        if (tid == 0) mse_row[0] = (float)((red[0] + red[1] + red[2] + red[3]) / wsum);
    }
    if (tid == 0) {
        if (wsum > 0.0) {
            for (int t = done + 1; t <= iters; ++t) mse_row[t] = mse_row[done];
        } else {
            for (int t = 0; t <= iters; ++t) mse_row[t] = 0.0f;
        }
    }
    if (tid < 16) {
        thr_out[(size_t)n * kTableStride + tid] = T_l[tid];
        map_out[(size_t)n * kTableStride + tid] = M_l[tid];
    }
}

size_t learn_lds_bytes(int nlmax) { return (size_t)2 * nlmax * kLearnThreads * 4 + (2 * 16 + 2) * 8 + 2 * 16 * 4 + 16; }

bool learn_supported(int K) { return K <= kLearnMaxK; }

hipError_t launch_learn_tables(const lowra_layout& L, const float* W, const float* init_thresholds,
                               const float* init_mappings, int iters, float* thr_out, float* map_out,
                               float* mse_out, hipStream_t st) {
    if (L.N == 0) return hipSuccess;
    const int nlmax = L.n_by_bits[4] > 0 ? 16 : (L.n_by_bits[2] > 0 ? 4 : 2);      // levels of the widest row
    const int np = (L.K / 8 + kLearnThreads - 1) / kLearnThreads;                  // eighths of blocks per thread
    const dim3 grid(L.N), block(kLearnThreads);
    const size_t lds = learn_lds_bytes(nlmax);
    KernelTimer timer(st);
#define LOWRA_LEARN(NP) learn_tables_kernel<NP><<<grid, block, lds, st>>>(L.d_rows, W, init_thresholds, init_mappings, iters, thr_out, map_out, mse_out, L.K, nlmax)
    if (np <= 1) LOWRA_LEARN(1);
    else if (np <= 2) LOWRA_LEARN(2);
    else if (np <= 4) LOWRA_LEARN(4);
    else LOWRA_LEARN(8);
#undef LOWRA_LEARN
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Threshold averaging (Sec. 5): entry j of every b-bit channel becomes the mean of entry j over
// the matrix's b-bit channels.  One workgroup per (width, entry): fixed-order fp64 sum, then the
// write-back.  In place on thr [N][16].
__global__ __launch_bounds__(256) void average_thresholds_kernel(const RowInfo* __restrict__ rows, int N, float* __restrict__ thr) {
    __shared__ double part[4];
    __shared__ long long cnt_part[4];
    const int widx = blockIdx.x / 15, j = blockIdx.x % 15;      // widths 1, 2, 4
    const int b = 1 << widx;
    if (j >= (1 << b) - 1) return;                               // uniform
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    double s = 0.0, c = 0.0;
    for (int n = tid; n < N; n += 256)
        if (rows[n].bits() == b) { s += (double)thr[(size_t)n * kTableStride + j]; c += 1.0; }
    s = wave_sum(s); c = wave_sum(c);
    if (lane == 0) { part[wave] = s; cnt_part[wave] = (long long)c; }
    __syncthreads();
    const double tot = part[0] + part[1] + part[2] + part[3];
    const long long cnt = cnt_part[0] + cnt_part[1] + cnt_part[2] + cnt_part[3];
    if (cnt == 0) return;
    const float m = (float)(tot / (double)cnt);
    for (int n = tid; n < N; n += 256)
        if (rows[n].bits() == b) thr[(size_t)n * kTableStride + j] = m;
}

hipError_t launch_average_thresholds(const lowra_layout& L, float* thr, hipStream_t st) {
    if (L.N == 0) return hipSuccess;
    average_thresholds_kernel<<<dim3(45), dim3(256), 0, st>>>(L.d_rows, L.N, thr);
    return hipGetLastError();
}

}  // namespace lowra
