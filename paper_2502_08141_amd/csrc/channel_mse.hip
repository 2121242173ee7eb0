// Per-channel error table (paper Sec. 6.1: every channel's MSE under 1-, 2- and 4-bit
// quantization, the input of the precision assignment), and a greedy budgeted assignment that
// stands in for the paper's two-level ILP (Sec. 6).
//
//   mse[n][p] = (1/K) sum_k ( W[n,k] - mappings[p][code_p] * absmax )^2      p = 0, 1, 2: 1, 2, 4 bits
// with absmax, normalisation and binning exactly as in the quantize kernel (App. A.1) and the fp32
// decode of App. A.2: quantize -> decode -> squared error fused in one pass over W, nothing packed.
//
// Mapping: one workgroup per channel, a lane owns 8 consecutive weights (a block is 8 adjacent
// lanes), all three widths from the same registers.  The 4-bit code -- the number of thresholds
// strictly below u, App. A.1 -- is found by bisection over the sorted thresholds instead of 15
// compares: the first two steps choose among register constants, the last two read the threshold
// from LDS (16 consecutive banks: any mix of indices is conflict-free), and so does the level;
// the narrower widths are selected in registers.  HBM-read bound: 4 B/weight once.
#include <algorithm>
#include <queue>
#include <tuple>
#include <vector>

#include "lowra_host.h"

namespace lowra {

__global__ __launch_bounds__(256) void channel_mse_kernel(const float* __restrict__ W, const float* __restrict__ thr3,
                                                          const float* __restrict__ map3, float* __restrict__ mse, int K) {
    __shared__ float lev4[16];
    __shared__ float thr4[16];                                    // sorted, entry 15 unused
    __shared__ double part[4][3];
    const int n = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float4* w4 = reinterpret_cast<const float4*>(W + (size_t)n * K);
    const int units = K >> 3;
    if (tid < 16) { lev4[tid] = map3[2 * kTableStride + tid]; thr4[tid] = thr3[2 * kTableStride + tid]; }
    const float t1 = thr3[0];
    const float t2a = thr3[kTableStride], t2b = thr3[kTableStride + 1], t2c = thr3[kTableStride + 2];
    const float t4_3 = thr3[2 * kTableStride + 3], t4_7 = thr3[2 * kTableStride + 7], t4_11 = thr3[2 * kTableStride + 11];
    const float m1a = map3[0], m1b = map3[1];
    const float m2a = map3[kTableStride], m2b = map3[kTableStride + 1], m2c = map3[kTableStride + 2], m2d = map3[kTableStride + 3];
    __syncthreads();
    float e1 = 0.0f, e2 = 0.0f, e4 = 0.0f;
    for (int base = 0; base < units; base += 2 * 256) {          // two passes requested together: a K = 4096 row is in flight at once
        float4 q0[2], q1[2];
#pragma unroll
        for (int ps = 0; ps < 2; ++ps) {
            const int un = min(base + ps * 256 + tid, units - 1);                // past the row: clamped, unused
            q0[ps] = w4[2 * un]; q1[ps] = w4[2 * un + 1];
        }
#pragma unroll
        for (int ps = 0; ps < 2; ++ps) {
            const int un = base + ps * 256 + tid;
            if (un < units) {                                     // units is a multiple of 8: the 8 lanes of a block agree
                const float v[8] = {q0[ps].x, q0[ps].y, q0[ps].z, q0[ps].w, q1[ps].x, q1[ps].y, q1[ps].z, q1[ps].w};
                float a = 0.0f;
#pragma unroll
                for (int i = 0; i < 8; ++i) a = fmaxf(a, fabsf(v[i]));
                a = dpp_max_f32<0xB1>(a);
                a = dpp_max_f32<0x4E>(a);
                a = fmaxf(a, __shfl_xor(a, 4));
                const float inv = (a == 0.0f) ? 0.0f : 1.0f / a;  // IEEE division, once per block
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const float u = v[i] * inv;
                    const float l1 = (t1 < u) ? m1b : m1a;
                    const float l2 = (t2c < u) ? m2d : ((t2b < u) ? m2c : ((t2a < u) ? m2b : m2a));
                    // thresholds ascending: #{j : T[j] < u} by bisection, the code's bits from the top
                    const int b3 = (t4_7 < u) ? 1 : 0;
                    int c4 = 2 * b3 + (((b3 ? t4_11 : t4_3) < u) ? 1 : 0);
                    c4 = 2 * c4 + ((thr4[4 * c4 + 1] < u) ? 1 : 0);
                    c4 = 2 * c4 + ((thr4[2 * c4] < u) ? 1 : 0);
                    const float l4 = lev4[c4];
                    const float d1 = v[i] - l1 * a, d2 = v[i] - l2 * a, d4 = v[i] - l4 * a;
                    e1 = fmaf(d1, d1, e1); e2 = fmaf(d2, d2, e2); e4 = fmaf(d4, d4, e4);   // (the build does not contract on its own)
                }
            }
        }
    }
    const double s1 = wave_sum((double)e1), s2 = wave_sum((double)e2), s4 = wave_sum((double)e4);
    if (lane == 0) { part[wave][0] = s1; part[wave][1] = s2; part[wave][2] = s4; }
    __syncthreads();
    if (tid < 3) mse[(size_t)n * 3 + tid] = (float)((part[0][tid] + part[1][tid] + part[2][tid] + part[3][tid]) / (double)K);
}

hipError_t launch_channel_mse(int N, int K, const float* W, const float* thr3, const float* map3, float* mse, hipStream_t st) {
    if (N == 0) return hipSuccess;
    KernelTimer timer(st);
    channel_mse_kernel<<<dim3(N), dim3(256), 0, st>>>(W, thr3, map3, mse, K);
    return hipGetLastError();
}

// Greedy assignment on the host.  Every channel starts at 1 bit; an upgrade is 1 -> 2 bits (cost
// params bits) or, once a channel is at 2 bits, 2 -> 4 (cost 2 params); the upgrade with the
// largest error reduction per bit that still fits the budget and reduces the error is applied
// until none is left; ties go to the lower channel.  An upgrade that does not fit never fits
// later (the remaining budget only shrinks), so a heap of the currently available upgrades is
// enough.  fp64 throughout, the same expressions as the reference statement of the rule.
bool assign_greedy_host(int N, const int64_t* params, const float* mse, double budget_bpp, uint8_t* bits) {
    if (N < 0 || !(budget_bpp >= 1.0)) return false;
    double total = 0.0;
    for (int n = 0; n < N; ++n) {
        if (params[n] <= 0) return false;
        total += (double)params[n];
        bits[n] = 1;
    }
    double remaining = budget_bpp * total - total;
    struct Up { double eff; int n; };
    auto worse = [](const Up& x, const Up& y) { return x.eff < y.eff || (x.eff == y.eff && x.n > y.n); };
    std::priority_queue<Up, std::vector<Up>, decltype(worse)> heap(worse);
    auto offer = [&](int n) {
        if (bits[n] == 4) return;
        const double pn = (double)params[n];
        const double cost = bits[n] == 1 ? pn : 2.0 * pn;
        const double gain = bits[n] == 1 ? pn * ((double)mse[n * 3] - (double)mse[n * 3 + 1])
                                         : pn * ((double)mse[n * 3 + 1] - (double)mse[n * 3 + 2]);
        if (!(gain > 0.0)) return;
        heap.push(Up{gain / cost, n});
    };
    for (int n = 0; n < N; ++n) offer(n);
    while (!heap.empty()) {
        const Up u = heap.top();
        heap.pop();
        const double cost = bits[u.n] == 1 ? (double)params[u.n] : 2.0 * (double)params[u.n];
        if (cost > remaining) continue;                      // never fits again
        remaining -= cost;
        bits[u.n] = bits[u.n] == 1 ? 2 : 4;
        offer(u.n);
    }
    return true;
}

}  // namespace lowra
