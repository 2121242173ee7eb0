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
// algorithmic traffic): it is normalised exactly as in the quantize kernel and kept in LDS as
// fp32 together with the block scales.  Every iteration is then LDS-only: a thread walks its
// elements (consecutive threads, consecutive elements), bins them against the thresholds in
// registers, and adds a and a u into ITS OWN column of a [bin][thread] table in LDS -- plain
// read-modify-write without atomics or bank conflicts, and a fixed summation order.  The 16 x 2
// column sums are then reduced by the four wavefronts, and one thread updates the tables.  The
// squared error never needs a second pass: sum a (u - m)^2 over a bin is
// sum a u^2 - 2 m sum a u + m^2 sum a.
#include "lowra_host.h"

namespace lowra {

constexpr int kLearnThreads = 256;
constexpr int kLearnMaxK = 16384;          // the row lives in LDS: 4 B per weight + 4 B per block

// E-step of one thread: its elements k = tid, tid + 256, ... binned against the row's thresholds;
// sums of a and a u per bin into column `tid` of col [2][nlmax][256] (nlmax = levels of the matrix's widest row).  Narrow rows (<= 4 bins) keep the
// sums in registers and store them once; 4-bit rows add into LDS (a thread touches only its column).
template <int BITS>
__device__ __forceinline__ void estep(const float* T_l, const float* u_l, const float* a_l, float* col, int K, int tid, int nlmax) {
    constexpr int NL = 1 << BITS, NT = NL - 1;
    float T[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) T[j] = T_l[j];
    if (BITS <= 2) {
        float s0[NL], s1[NL];
#pragma unroll
        for (int j = 0; j < NL; ++j) { s0[j] = 0.0f; s1[j] = 0.0f; }
        for (int k = tid; k < K; k += kLearnThreads) {
            const float uk = u_l[k], ak = a_l[k >> 6];
            int c = 0;
#pragma unroll
            for (int j = 0; j < NT; ++j) c += (T[j] < uk) ? 1 : 0;
            const float au = ak * uk;
#pragma unroll
            for (int j = 0; j < NL; ++j) { s0[j] += (c == j) ? ak : 0.0f; s1[j] += (c == j) ? au : 0.0f; }
        }
#pragma unroll
        for (int j = 0; j < NL; ++j) { col[j * kLearnThreads + tid] = s0[j]; col[(nlmax + j) * kLearnThreads + tid] = s1[j]; }
    } else {
#pragma unroll
        for (int j = 0; j < NL; ++j) { col[j * kLearnThreads + tid] = 0.0f; col[(nlmax + j) * kLearnThreads + tid] = 0.0f; }
        for (int k = tid; k < K; k += kLearnThreads) {
            const float uk = u_l[k], ak = a_l[k >> 6];
            int c = 0;
#pragma unroll
            for (int j = 0; j < NT; ++j) c += (T[j] < uk) ? 1 : 0;
            col[c * kLearnThreads + tid] += ak;
            col[(nlmax + c) * kLearnThreads + tid] += ak * uk;
        }
    }
}

__global__ __launch_bounds__(kLearnThreads) void learn_tables_kernel(const RowInfo* __restrict__ rows,
                                                                    const float* __restrict__ W,
                                                                    const float* __restrict__ init_thresholds,
                                                                    const float* __restrict__ init_mappings,
                                                                    int iters, float* __restrict__ thr_out,
                                                                    float* __restrict__ map_out,
                                                                    float* __restrict__ mse_out, int K, int nlmax) {
    extern __shared__ __align__(16) uint8_t lsm[];
    // LDS: reduced sums (fp64) [2][16] + 2 | tables T[16], M[16] | flag (4 words) | u [K] | column sums [2][nlmax][256] | a [K/64]
    double* red = reinterpret_cast<double*>(lsm);
    float* T_l = reinterpret_cast<float*>(red + 2 * 16 + 2);
    float* M_l = T_l + 16;
    int* flag = reinterpret_cast<int*>(M_l + 16);
    float* u_l = reinterpret_cast<float*>(flag + 4);               // 16-byte aligned: 272 + 128 + 16 bytes in front
    float* col = u_l + K;
    float* a_l = col + 2 * nlmax * kLearnThreads;

    const int n = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const RowInfo ri = rows[n];
    const int bits = ri.bits(), nl = 1 << bits, nt = nl - 1;
    const float4* w4 = reinterpret_cast<const float4*>(W + (size_t)n * K);
    const int units = K >> 3;

    // ---- the row: normalised weights and block scales into LDS; sum a and sum a u^2 on the way
    double sa = 0.0, sauu = 0.0;
    for (int base = 0; base < units; base += 2 * kLearnThreads) {   // two passes requested together: a K = 4096 row is in flight at once
        float4 q0[2], q1[2];
#pragma unroll
        for (int ps = 0; ps < 2; ++ps) {
            const int un = min(base + ps * kLearnThreads + tid, units - 1);     // past the row: clamped, unused
            q0[ps] = w4[2 * un]; q1[ps] = w4[2 * un + 1];
        }
#pragma unroll
        for (int ps = 0; ps < 2; ++ps) {
            const int un = base + ps * kLearnThreads + tid;      // a lane owns 8 consecutive weights, a block is 8 adjacent lanes
            if (un < units) {                                     // units is a multiple of 8: the 8 lanes of a block agree
                const float v[8] = {q0[ps].x, q0[ps].y, q0[ps].z, q0[ps].w, q1[ps].x, q1[ps].y, q1[ps].z, q1[ps].w};
                float a = 0.0f;
#pragma unroll
                for (int i = 0; i < 8; ++i) a = fmaxf(a, fabsf(v[i]));
                a = dpp_max_f32<0xB1>(a);                         // lanes l ^ 1
                a = dpp_max_f32<0x4E>(a);                         // l ^ 2
                a = fmaxf(a, __shfl_xor(a, 4));
                const float inv = (a == 0.0f) ? 0.0f : 1.0f / a;  // IEEE division, once per block
                float un8[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) un8[i] = v[i] * inv;
                *reinterpret_cast<float4*>(u_l + 8 * un) = make_float4(un8[0], un8[1], un8[2], un8[3]);
                *reinterpret_cast<float4*>(u_l + 8 * un + 4) = make_float4(un8[4], un8[5], un8[6], un8[7]);
                if ((un & 7) == 0) a_l[un >> 3] = a;
                float uu = 0.0f;                                   // 8 squares of values in [-1, 1]: fp32 is plenty, fp64 from there on
#pragma unroll
                for (int i = 0; i < 8; ++i) uu += un8[i] * un8[i];
                sa += 8.0 * (double)a; sauu += (double)a * (double)uu;
            }
        }
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
            if (bits == 4) estep<4>(T_l, u_l, a_l, col, K, tid, nlmax);
            else if (bits == 2) estep<2>(T_l, u_l, a_l, col, K, tid, nlmax);
            else estep<1>(T_l, u_l, a_l, col, K, tid, nlmax);
            __syncthreads();
            // column sums: wavefront w reduces bins 4w .. 4w+3 of both tables, in fp64
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int bin = 4 * wave + (q & 3), tab = q >> 2;
                if (bin < nl) {                                    // uniform over the wavefront: bins past the row's width are not used
                    double s = 0.0;
#pragma unroll
                    for (int i = 0; i < kLearnThreads / 64; ++i) s += (double)col[(tab * nlmax + bin) * kLearnThreads + lane + 64 * i];
                    s = wave_sum(s);
                    if (lane == 0) red[tab * 16 + bin] = s;
                }
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
    if (tid == 0) {
        if (wsum > 0.0) {
            if (iters == 0) {       // only the error of the initial tables: needs one binning pass; done by this thread alone
                double e = 0.0;
                for (int k = 0; k < K; ++k) {
                    int c = 0;
                    for (int j = 0; j < nt; ++j) c += (T_l[j] < u_l[k]) ? 1 : 0;
                    const double d = (double)u_l[k] - (double)M_l[c];
                    e += (double)a_l[k >> 6] * d * d;
                }
                mse_row[0] = (float)(e / wsum);
            }
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

size_t learn_lds_bytes(int K, int nlmax) {
    return (size_t)K * 4 + (size_t)(K >> 6) * 4 + (size_t)2 * nlmax * kLearnThreads * 4 + (2 * 16 + 2) * 8 + 2 * 16 * 4 + 16;
}

bool learn_supported(int K) { return K <= kLearnMaxK; }

hipError_t launch_learn_tables(const lowra_layout& L, const float* W, const float* init_thresholds,
                               const float* init_mappings, int iters, float* thr_out, float* map_out,
                               float* mse_out, hipStream_t st) {
    if (L.N == 0) return hipSuccess;
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(learn_tables_kernel),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)learn_lds_bytes(kLearnMaxK, 16));
    if (attr != hipSuccess) return attr;
    const int nlmax = L.n_by_bits[4] > 0 ? 16 : (L.n_by_bits[2] > 0 ? 4 : 2);      // levels of the widest row
    KernelTimer timer(st);
    learn_tables_kernel<<<dim3(L.N), dim3(kLearnThreads), learn_lds_bytes(L.K, nlmax), st>>>(L.d_rows, W, init_thresholds, init_mappings,
                                                                                            iters, thr_out, map_out, mse_out, L.K, nlmax);
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
