/*
 * LowRA hot-path ORACLE -- test infrastructure, not product code.
 *
 * A plain, slow, obviously-correct CPU statement of what the quantizer, the
 * dequantizer and the dequant-fused LoRA linear compute.  Only the tests, the
 * smoke check and the benchmark's cpu_baseline leg may call it.  It shares no
 * code, header, table or helper with the HIP library.
 *
 * Notation (paper Sec. 4.1, App. A):
 *   W [N,K] fp32 row-major, N = output channels, K = input features.
 *   Group g of channel n = elements k in [64g, 64g+64); G = K/64   (Sec. 4.1,
 *   "Groupwise Normalization": 64-element blocks scaled by their absmax).
 *   bits[n] in {1,2,4}                       ("Precs", App. A; P = {1,2,4}, Sec. 6.2)
 *   thresholds[c][0 .. 2^b-2] ascending      (bin edges, Sec. 4.1)
 *   mappings[c][0 .. 2^b-1]                  (representative values, Sec. 4.1)
 *   cb[n] = table index of channel n (per-channel tables when C == N).
 *
 * Steps, in the paper's order (App. A.1 quantize, App. A.2 dequantize):
 *   Q1  a[n,g] = max_k |W[n,64g+k]|                                (fp32, exact)
 *   Q2  inv    = a == 0 ? 0 : 1.0f / a                            (one IEEE fp32 division per group)
 *   Q3  u      = W[n,64g+k] * inv                                 (one fp32 multiply, round-to-nearest)
 *   Q4  code   = #{ j < 2^b-1 : T[cb(n)][j] < u }                 (strict <; a tie falls in the lower bin)
 *   Q5  row n occupies bytes [off[n], off[n] + K*b/8), off = exclusive prefix sum
 *       in channel order; code k sits at stream bits [k*b, (k+1)*b), stream bit i =
 *       bit (i mod 8) of byte (i div 8)  (LSB first)
 *   D1  w32    = Mtab[cb(n)][code] * a[n,g]                       (one fp32 multiply)
 *   D2  What   = bf16 round-to-nearest-even of w32                (fp32 variant: w32)
 *   L1  y[m,n]  = sum_k x[m,k] What[n,k] + s sum_j (sum_k x[m,k] A[j,k]) B[n,j]      (fp64)
 *   L2  dX[m,k] = sum_n dY[m,n] What[n,k] + s sum_j (sum_n dY[m,n] B[n,j]) A[j,k]    (fp64)
 * The LoRA equation is the standard one the paper builds on (Sec. 2.1).
 * The mapping/threshold learner (Sec. 5, App. G: weighted Lloyd-Max), threshold averaging, the
 * per-channel error table (Sec. 6.1) and a greedy budgeted precision assignment (stand-in for
 * the ILP of Sec. 6) and the adapter gradients are stated step by step at the end of this file.
 *
 * Parity pins (tests/test_oracle_*.py): brute-force nearest level, numpy
 * searchsorted, bit-by-bit unpacker round trip, hand-worked byte patterns, 1-bit
 * sign closed form, quantization error bound, the init tables printed in the
 * paper's App. F listing, numpy fp64 matmul, adjoint identity, torch's bf16 cast.
 * Learner pins (tests/test_oracle_learner.py): numpy's weighted average (1-bit closed form),
 * scipy's kmeans2 when all blocks weigh the same, brute-force fixed-point condition,
 * non-increasing MSE, scale invariance, a hand-worked block, the printed init tables.
 * Error table and assignment pins (tests/test_oracle_assign.py): quantize + decode + numpy mean,
 * the 1-bit closed form, the quantizer's error bound, exhaustive search on tiny instances.
 * Adapter gradient pins (tests/test_oracle_grads.py): numpy fp64 matmul, difference quotients of L1.
 * The alternating low-rank initialiser (Sec. 4.1, App. D) is composed in lowra_oracle.py from Q1-Q5,
 * D1-D2 and numpy's SVD; its pins (tests/test_oracle_loftq.py): exact recovery of a rank-r matrix, the
 * Eckart-Young value through the Gram matrix's eigenvalues, no competitor subspace doing better, the
 * first step being the quantization of W, outputs consistent with the reported objective, and an
 * objective below plain quantization that does not increase (learned tables).
 *
 * Build: gcc -O2 -fopenmp -ffp-contract=off -fno-fast-math -shared -fPIC
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define GROUP 64
#define TSTRIDE 16 /* table row stride: room for the 16 levels of 4 bits */

enum { OK = 0, ERR_ARG = 1, ERR_BITS = 2, ERR_TABLE = 3, ERR_NONFINITE = 4, ERR_ALLOC = 5 };

int lowra_oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static int valid_bits(int b) { return b == 1 || b == 2 || b == 4; }

static float bits_to_float(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
static uint32_t float_to_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }

/* D2: fp32 -> bf16, round to nearest, ties to even (training runs in bf16, App. I). */
uint16_t lowra_oracle_bf16_rne(float f) {
    uint32_t u = float_to_bits(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u); /* quiet NaN */
    uint32_t keep = u >> 16, drop = u & 0xffffu;
    if (drop > 0x8000u || (drop == 0x8000u && (keep & 1u))) keep += 1u;
    return (uint16_t)keep;
}
void lowra_oracle_bf16_rne_array(size_t n, const float* in, uint16_t* out) {
    for (size_t i = 0; i < n; ++i) out[i] = lowra_oracle_bf16_rne(in[i]);
}
static float bf16_to_float(uint16_t h) { return bits_to_float((uint32_t)h << 16); }

/* Q5 offsets: the paper's bit accounting, bits(channel) = precision * parameters (Sec. 6.2). */
int lowra_oracle_row_offsets(int N, int K, const uint8_t* bits, int64_t* off) {
    if (N < 0 || K <= 0 || K % GROUP) return ERR_ARG;
    off[0] = 0;
    for (int n = 0; n < N; ++n) {
        if (!valid_bits(bits[n])) return ERR_BITS;
        off[n + 1] = off[n] + (int64_t)K * bits[n] / 8;
    }
    return OK;
}

static int check_tables(int N, const uint8_t* bits, const int32_t* cb, int C) {
    for (int n = 0; n < N; ++n) {
        if (!valid_bits(bits[n])) return ERR_BITS;
        if (cb[n] < 0 || cb[n] >= C) return ERR_TABLE;
    }
    return OK;
}

/* The group scale as a 16-bit value (Sec. 4.1 "Groupwise Normalization" does not fix the scale's type; the variant
 * stores it as bf16): round to nearest even; a maximum so close to the largest float that it would round to
 * infinity keeps the largest finite bf16 instead.  Returned as the float it stands for. */
static float scale_to_bf16_value(float a) {
    uint16_t h = lowra_oracle_bf16_rne(a);
    if ((h & 0x7fffu) == 0x7f80u) h = (uint16_t)((h & 0x8000u) | 0x7f7fu);
    return bf16_to_float(h);
}

/* Q1-Q4: absmax and one code per weight (unpacked, one byte each).  scale_bf16 != 0: the scale is rounded to bf16
 * right after Q1, and that value normalises (Q2-Q3) and is returned (as a float; the decoder multiplies by it). */
int lowra_oracle_quantize_codes_s(int N, int K, const float* W, const uint8_t* bits,
                                  const int32_t* cb, int C, const float* thresholds, int scale_bf16,
                                  uint8_t* codes, float* absmax) {
    if (N < 0 || K <= 0 || K % GROUP) return ERR_ARG;
    int rc = check_tables(N, bits, cb, C);
    if (rc) return rc;
    const int G = K / GROUP;
    for (int n = 0; n < N; ++n) { /* thresholds must ascend (they partition the domain, Sec. 4.1) */
        const float* T = thresholds + (size_t)cb[n] * TSTRIDE;
        const int nt = (1 << bits[n]) - 1;
        for (int j = 0; j < nt; ++j) {
            if (isnan(T[j])) return ERR_TABLE;
            if (j && T[j] < T[j - 1]) return ERR_TABLE;
        }
    }
    int bad = 0;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        const float* T = thresholds + (size_t)cb[n] * TSTRIDE;
        const int nt = (1 << bits[n]) - 1;
        for (int g = 0; g < G; ++g) {
            const float* w = W + (size_t)n * K + (size_t)g * GROUP;
            float a = 0.0f;                                   /* Q1 */
            for (int k = 0; k < GROUP; ++k) {
                if (!isfinite(w[k])) bad = 1;
                float m = fabsf(w[k]);
                if (m > a) a = m;
            }
            if (scale_bf16) a = scale_to_bf16_value(a);
            absmax[(size_t)n * G + g] = a;
            const float inv = (a == 0.0f) ? 0.0f : 1.0f / a;  /* Q2 */
            for (int k = 0; k < GROUP; ++k) {
                const float u = w[k] * inv;                   /* Q3 */
                int code = 0;                                 /* Q4 */
                for (int j = 0; j < nt; ++j)
                    if (T[j] < u) ++code;
                codes[(size_t)n * K + (size_t)g * GROUP + k] = (uint8_t)code;
            }
        }
    }
    return bad ? ERR_NONFINITE : OK;
}
int lowra_oracle_quantize_codes(int N, int K, const float* W, const uint8_t* bits,
                                const int32_t* cb, int C, const float* thresholds,
                                uint8_t* codes, float* absmax) {
    return lowra_oracle_quantize_codes_s(N, K, W, bits, cb, C, thresholds, 0, codes, absmax);
}

/* Q5: bit-pack the codes of every row at its own width. */
int lowra_oracle_pack(int N, int K, const uint8_t* bits, const uint8_t* codes, uint8_t* packed) {
    if (N < 0 || K <= 0 || K % GROUP) return ERR_ARG;
    int64_t* off = (int64_t*)malloc(sizeof(int64_t) * ((size_t)N + 1));
    if (!off) return ERR_ALLOC;
    int rc = lowra_oracle_row_offsets(N, K, bits, off);
    if (rc) { free(off); return rc; }
    memset(packed, 0, (size_t)off[N]);
    for (int n = 0; n < N; ++n) {
        const int b = bits[n];
        uint8_t* row = packed + off[n];
        for (int k = 0; k < K; ++k) {
            const unsigned code = codes[(size_t)n * K + k];
            if (code >> b) { free(off); return ERR_ARG; }
            for (int i = 0; i < b; ++i) {
                const int64_t sbit = (int64_t)k * b + i;      /* position in the row's bit stream */
                if ((code >> i) & 1u) row[sbit / 8] |= (uint8_t)(1u << (sbit % 8));
            }
        }
    }
    free(off);
    return OK;
}

/* Inverse of Q5. */
int lowra_oracle_unpack(int N, int K, const uint8_t* bits, const uint8_t* packed, uint8_t* codes) {
    if (N < 0 || K <= 0 || K % GROUP) return ERR_ARG;
    int64_t* off = (int64_t*)malloc(sizeof(int64_t) * ((size_t)N + 1));
    if (!off) return ERR_ALLOC;
    int rc = lowra_oracle_row_offsets(N, K, bits, off);
    if (rc) { free(off); return rc; }
    for (int n = 0; n < N; ++n) {
        const int b = bits[n];
        const uint8_t* row = packed + off[n];
        for (int k = 0; k < K; ++k) {
            unsigned code = 0;
            for (int i = 0; i < b; ++i) {
                const int64_t sbit = (int64_t)k * b + i;
                code |= (unsigned)((row[sbit / 8] >> (sbit % 8)) & 1u) << i;
            }
            codes[(size_t)n * K + k] = (uint8_t)code;
        }
    }
    free(off);
    return OK;
}

/* Q1-Q5 (App. A.1). */
int lowra_oracle_quantize_s(int N, int K, const float* W, const uint8_t* bits, const int32_t* cb,
                            int C, const float* thresholds, int scale_bf16, uint8_t* packed, float* absmax) {
    uint8_t* codes = (uint8_t*)malloc((size_t)N * K + 1);
    if (!codes) return ERR_ALLOC;
    int rc = lowra_oracle_quantize_codes_s(N, K, W, bits, cb, C, thresholds, scale_bf16, codes, absmax);
    if (rc == OK) rc = lowra_oracle_pack(N, K, bits, codes, packed);
    free(codes);
    return rc;
}
int lowra_oracle_quantize(int N, int K, const float* W, const uint8_t* bits, const int32_t* cb,
                          int C, const float* thresholds, uint8_t* packed, float* absmax) {
    return lowra_oracle_quantize_s(N, K, W, bits, cb, C, thresholds, 0, packed, absmax);
}

/* D1-D2 (App. A.2).  out_dtype 0: bf16 bit patterns (uint16), 1: fp32. */
int lowra_oracle_dequantize(int N, int K, const uint8_t* packed, const float* absmax,
                            const uint8_t* bits, const int32_t* cb, int C, const float* mappings,
                            int out_dtype, void* out) {
    if (N < 0 || K <= 0 || K % GROUP || (out_dtype != 0 && out_dtype != 1)) return ERR_ARG;
    int rc = check_tables(N, bits, cb, C);
    if (rc) return rc;
    uint8_t* codes = (uint8_t*)malloc((size_t)N * K + 1);
    if (!codes) return ERR_ALLOC;
    rc = lowra_oracle_unpack(N, K, bits, packed, codes);
    if (rc) { free(codes); return rc; }
    const int G = K / GROUP;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        const float* Mt = mappings + (size_t)cb[n] * TSTRIDE;
        for (int k = 0; k < K; ++k) {
            const float a = absmax[(size_t)n * G + k / GROUP];
            const float w32 = Mt[codes[(size_t)n * K + k]] * a;            /* D1 */
            if (out_dtype == 0) ((uint16_t*)out)[(size_t)n * K + k] = lowra_oracle_bf16_rne(w32); /* D2 */
            else ((float*)out)[(size_t)n * K + k] = w32;
        }
    }
    free(codes);
    return OK;
}

/* What as doubles (every bf16 is exactly representable). */
static double* decode_to_double(int N, int K, const uint8_t* packed, const float* absmax,
                                const uint8_t* bits, const int32_t* cb, int C,
                                const float* mappings, int* rc) {
    uint16_t* h = (uint16_t*)malloc(sizeof(uint16_t) * ((size_t)N * K + 1));
    double* d = (double*)malloc(sizeof(double) * ((size_t)N * K + 1));
    if (!h || !d) { free(h); free(d); *rc = ERR_ALLOC; return NULL; }
    *rc = lowra_oracle_dequantize(N, K, packed, absmax, bits, cb, C, mappings, 0, h);
    if (*rc) { free(h); free(d); return NULL; }
    for (size_t i = 0; i < (size_t)N * K; ++i) d[i] = (double)bf16_to_float(h[i]);
    free(h);
    return d;
}

/* L1.  x [M,K], A [r,K], B [N,r] are bf16 bit patterns; y [M,N] fp64. */
int lowra_oracle_linear_fwd(int N, int K, const uint8_t* packed, const float* absmax,
                            const uint8_t* bits, const int32_t* cb, int C, const float* mappings,
                            int M, const uint16_t* x, int r, const uint16_t* A, const uint16_t* B,
                            float s, double* y) {
    if (M < 0 || r < 0) return ERR_ARG;
    int rc = OK;
    double* Wd = decode_to_double(N, K, packed, absmax, bits, cb, C, mappings, &rc);
    if (rc) return rc;
    double* t = (double*)malloc(sizeof(double) * ((size_t)M * r + 1)); /* t = x A^T */
    if (!t) { free(Wd); return ERR_ALLOC; }
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m)
        for (int j = 0; j < r; ++j) {
            double acc = 0.0;
            for (int k = 0; k < K; ++k)
                acc += (double)bf16_to_float(x[(size_t)m * K + k]) * (double)bf16_to_float(A[(size_t)j * K + k]);
            t[(size_t)m * r + j] = acc;
        }
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m)
        for (int n = 0; n < N; ++n) {
            double base = 0.0;
            for (int k = 0; k < K; ++k)
                base += (double)bf16_to_float(x[(size_t)m * K + k]) * Wd[(size_t)n * K + k];
            double lora = 0.0;
            for (int j = 0; j < r; ++j)
                lora += t[(size_t)m * r + j] * (double)bf16_to_float(B[(size_t)n * r + j]);
            y[(size_t)m * N + n] = base + (double)s * lora;
        }
    free(t);
    free(Wd);
    return OK;
}

/* L2.  dY [M,N] bf16 bit patterns; dX [M,K] fp64.  The base stays frozen, so no dW (Sec. 3). */
int lowra_oracle_linear_bwd_input(int N, int K, const uint8_t* packed, const float* absmax,
                                  const uint8_t* bits, const int32_t* cb, int C,
                                  const float* mappings, int M, const uint16_t* dY, int r,
                                  const uint16_t* A, const uint16_t* B, float s, double* dX) {
    if (M < 0 || r < 0) return ERR_ARG;
    int rc = OK;
    double* Wd = decode_to_double(N, K, packed, absmax, bits, cb, C, mappings, &rc);
    if (rc) return rc;
    int fail = 0;
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m) {
        double* u = (double*)malloc(sizeof(double) * ((size_t)r + 1)); /* u = dY B */
        if (!u) { fail = 1; continue; }
        for (int j = 0; j < r; ++j) {
            double acc = 0.0;
            for (int n = 0; n < N; ++n)
                acc += (double)bf16_to_float(dY[(size_t)m * N + n]) * (double)bf16_to_float(B[(size_t)n * r + j]);
            u[j] = acc;
        }
        double* row = dX + (size_t)m * K;                /* sum over n, n ascending, for all k at once */
        for (int k = 0; k < K; ++k) row[k] = 0.0;
        for (int n = 0; n < N; ++n) {
            const double g = (double)bf16_to_float(dY[(size_t)m * N + n]);
            for (int k = 0; k < K; ++k) row[k] += g * Wd[(size_t)n * K + k];
        }
        for (int k = 0; k < K; ++k) {
            double lora = 0.0;
            for (int j = 0; j < r; ++j)
                lora += u[j] * (double)bf16_to_float(A[(size_t)j * K + k]);
            row[k] += (double)s * lora;
        }
        free(u);
    }
    free(Wd);
    return fail ? ERR_ALLOC : OK;
}

/* ------------------------------------------------------------------------------------------
 * Mapping/threshold learner (Sec. 5 "Weighted Lloyd's for LoRA Quantization", App. G).
 * Per output channel n at its width b: weighted Lloyd-Max on the normalised weights u_i
 * (Q1-Q3), every element weighted by the absmax a_i of its 64-element block.
 *
 *   E-step   c(i) = #{ j < 2^b-1 : T[j] < u_i }      the quantizer's own binning (Q4).  With T the
 *                                                    midpoints of M this is App. G's nearest level,
 *                                                    a tie going to the lower level
 *   M-step   M[j] = sum_{c(i)=j} a_i u_i / sum_{c(i)=j} a_i     (App. G); an empty bin keeps its level
 *            T[j] = (M[j] + M[j+1]) / 2                         (Sec. 5: midpoints of consecutive levels)
 *   mse[0]   = sum a_i (u_i - M0[c0(i)])^2 / sum a_i            initial tables, their own binning
 *   mse[t]   = sum a_i (u_i - Mt[c(i)])^2 / sum a_i, t >= 1     the binning of iteration t (by T of
 *                                                               iteration t-1) with the levels it produced
 *   Stop after `iters` iterations, or after the first iteration whose mse is not below the one
 *   before (Sec. 5: no further decrease of the MSE ends the search); the tables computed last are the result.
 *   A channel whose weights are all zero (sum a_i = 0) keeps the initial tables, mse = 0.
 *
 * Sums in fp64 in element order; after every iteration the tables are rounded to fp32 (they are
 * fp32 at the library boundary, and the next E-step compares fp32 values like Q4).  Unused table
 * entries: thresholds +inf, mappings 0.  mse_out [N][iters+1] (entries past the stop repeat the
 * last value), iters_done [N].
 */
int lowra_oracle_learn_tables(int N, int K, const float* W, const uint8_t* bits, const int32_t* cb, int C,
                              const float* init_thresholds, const float* init_mappings, int iters,
                              float* thr_out, float* map_out, double* mse_out, int32_t* iters_done) {
    if (N < 0 || K <= 0 || K % GROUP || iters < 0) return ERR_ARG;
    int rc = check_tables(N, bits, cb, C);
    if (rc) return rc;
    const int G = K / GROUP;
    int fail = 0;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        const int nl = 1 << bits[n], nt = nl - 1;
        float T[TSTRIDE], Mp[TSTRIDE];
        for (int j = 0; j < TSTRIDE; ++j) {
            T[j] = j < nt ? init_thresholds[(size_t)cb[n] * TSTRIDE + j] : INFINITY;
            Mp[j] = j < nl ? init_mappings[(size_t)cb[n] * TSTRIDE + j] : 0.0f;
        }
        float* u = (float*)malloc(sizeof(float) * (size_t)K);
        float* a = (float*)malloc(sizeof(float) * (size_t)G);
        if (!u || !a) { fail = 1; free(u); free(a); continue; }
        double wsum = 0.0;
        for (int g = 0; g < G; ++g) {                       /* Q1-Q3 */
            const float* w = W + (size_t)n * K + (size_t)g * GROUP;
            float am = 0.0f;
            for (int k = 0; k < GROUP; ++k) { float m = fabsf(w[k]); if (m > am) am = m; }
            a[g] = am;
            const float inv = (am == 0.0f) ? 0.0f : 1.0f / am;
            for (int k = 0; k < GROUP; ++k) u[g * GROUP + k] = w[k] * inv;
            wsum += (double)am * GROUP;
        }
        double* mse = mse_out + (size_t)n * (iters + 1);
        int done = 0;
        if (wsum == 0.0) {
            for (int t = 0; t <= iters; ++t) mse[t] = 0.0;
        } else {
            for (int t = 1; t <= iters; ++t) {
                double S0[TSTRIDE] = {0}, S1[TSTRIDE] = {0}, err0 = 0.0;
                for (int k = 0; k < K; ++k) {               /* E-step */
                    int c = 0;
                    for (int j = 0; j < nt; ++j) if (T[j] < u[k]) ++c;
                    const double ak = a[k / GROUP];
                    S0[c] += ak; S1[c] += ak * (double)u[k];
                    if (t == 1) { const double d = (double)u[k] - (double)Mp[c]; err0 += ak * d * d; }
                }
                if (t == 1) mse[0] = err0 / wsum;
                for (int j = 0; j < nl; ++j)                /* M-step */
                    if (S0[j] > 0.0) Mp[j] = (float)(S1[j] / S0[j]);
                double err = 0.0;                           /* error of this binning with the new levels */
                for (int k = 0; k < K; ++k) {
                    int c = 0;
                    for (int j = 0; j < nt; ++j) if (T[j] < u[k]) ++c;
                    const double d = (double)u[k] - (double)Mp[c];
                    err += (double)a[k / GROUP] * d * d;
                }
                mse[t] = err / wsum;
                for (int j = 0; j < nt; ++j) T[j] = (float)(((double)Mp[j] + (double)Mp[j + 1]) * 0.5);
                done = t;
                if (!(mse[t] < mse[t - 1])) break;          /* the MSE stopped going down */
            }
            if (iters == 0) {                               /* only the error of the initial tables */
                double err0 = 0.0;
                for (int k = 0; k < K; ++k) {
                    int c = 0;
                    for (int j = 0; j < nt; ++j) if (T[j] < u[k]) ++c;
                    const double d = (double)u[k] - (double)Mp[c];
                    err0 += (double)a[k / GROUP] * d * d;
                }
                mse[0] = err0 / wsum;
            }
            for (int t = done + 1; t <= iters; ++t) mse[t] = mse[done];
        }
        iters_done[n] = done;
        for (int j = 0; j < TSTRIDE; ++j) {
            thr_out[(size_t)n * TSTRIDE + j] = T[j];
            map_out[(size_t)n * TSTRIDE + j] = Mp[j];
        }
        free(u); free(a);
    }
    return fail ? ERR_ALLOC : OK;
}

/* Threshold averaging (Sec. 5, last paragraph: the thresholds are averaged, read as: over the
 * channels of the matrix that share a width).  In place on thr [N][16]: entry j < 2^b-1 of every
 * b-bit channel becomes the mean (fp64 sum in channel order, rounded to fp32) of entry j over all
 * b-bit channels. */
int lowra_oracle_average_thresholds(int N, const uint8_t* bits, float* thr) {
    if (N < 0) return ERR_ARG;
    for (int n = 0; n < N; ++n) if (!valid_bits(bits[n])) return ERR_BITS;
    for (int b = 1; b <= 4; b <<= 1) {
        const int nt = (1 << b) - 1;
        for (int j = 0; j < nt; ++j) {
            double s = 0.0; long cnt = 0;
            for (int n = 0; n < N; ++n) if (bits[n] == b) { s += (double)thr[(size_t)n * TSTRIDE + j]; ++cnt; }
            if (!cnt) continue;
            const float m = (float)(s / (double)cnt);
            for (int n = 0; n < N; ++n) if (bits[n] == b) thr[(size_t)n * TSTRIDE + j] = m;
        }
    }
    return OK;
}

/* ------------------------------------------------------------------------------------------
 * Per-channel error table (Sec. 6.1: every channel's MSE under 1-, 2- and 4-bit quantization).
 * For width index p (0, 1, 2 = 1, 2, 4 bits) with tables thresholds[p], mappings[p]:
 *   mse[n][p] = (1/K) sum_k ( W[n,k] - w32(n,k;p) )^2,   w32 = mappings[p][code] * a   (Q1-Q4, D1)
 * i.e. the error of quantizing and decoding the channel at that width, decoded in fp32 (the
 * bf16 rounding of D2 belongs to the training path, not to the quantizer's error); the difference
 * is taken in fp32, squared and summed in fp64.
 */
int lowra_oracle_channel_mse(int N, int K, const float* W, const float* thresholds, const float* mappings,
                             double* mse) {
    if (N < 0 || K <= 0 || K % GROUP) return ERR_ARG;
    const int G = K / GROUP;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        double acc[3] = {0.0, 0.0, 0.0};
        for (int g = 0; g < G; ++g) {
            const float* w = W + (size_t)n * K + (size_t)g * GROUP;
            float a = 0.0f;
            for (int k = 0; k < GROUP; ++k) { float m = fabsf(w[k]); if (m > a) a = m; }
            const float inv = (a == 0.0f) ? 0.0f : 1.0f / a;
            for (int k = 0; k < GROUP; ++k) {
                const float u = w[k] * inv;
                for (int p = 0; p < 3; ++p) {
                    const int nt = (1 << (1 << p)) - 1;
                    const float* T = thresholds + (size_t)p * TSTRIDE;
                    int code = 0;
                    for (int j = 0; j < nt; ++j) if (T[j] < u) ++code;
                    const float w32 = mappings[(size_t)p * TSTRIDE + code] * a;
                    const float d = w[k] - w32;
                    acc[p] += (double)d * (double)d;
                }
            }
        }
        for (int p = 0; p < 3; ++p) mse[(size_t)n * 3 + p] = acc[p] / (double)K;
    }
    return OK;
}

/* Budgeted precision assignment, a greedy stand-in for the paper's two-level ILP (Sec. 6: minimise
 * the total quantization error sum_n params[n] * mse[n][p_n] under sum_n params[n] * bits_n <=
 * budget * sum_n params[n]).  Every channel starts at 1 bit.  An upgrade is 1 -> 2 bits (cost
 * params[n] bits, gain params[n] (mse[n][0] - mse[n][1])) or, for a channel already at 2 bits,
 * 2 -> 4 (cost 2 params[n], gain params[n] (mse[n][1] - mse[n][2])).  Repeatedly apply the upgrade
 * with the largest gain per bit among those that fit the remaining budget and have a positive
 * gain; ties go to the lower channel index.  All arithmetic in fp64.  Returns ERR_ARG when the
 * budget is below 1 bit per parameter. */
int lowra_oracle_assign_greedy(int N, const int64_t* params, const float* mse, double budget_bpp, uint8_t* bits) {
    if (N < 0 || !(budget_bpp >= 1.0)) return ERR_ARG;
    double total = 0.0;
    for (int n = 0; n < N; ++n) { if (params[n] <= 0) return ERR_ARG; total += (double)params[n]; bits[n] = 1; }
    double remaining = budget_bpp * total - total;
    for (;;) {
        int best = -1; double best_eff = 0.0;
        for (int n = 0; n < N; ++n) {
            if (bits[n] == 4) continue;
            const double pn = (double)params[n];
            const double cost = bits[n] == 1 ? pn : 2.0 * pn;
            const double gain = bits[n] == 1 ? pn * ((double)mse[n * 3] - (double)mse[n * 3 + 1])
                                             : pn * ((double)mse[n * 3 + 1] - (double)mse[n * 3 + 2]);
            if (cost > remaining || !(gain > 0.0)) continue;
            const double eff = gain / cost;
            if (best < 0 || eff > best_eff) { best = n; best_eff = eff; }
        }
        if (best < 0) break;
        remaining -= bits[best] == 1 ? (double)params[best] : 2.0 * (double)params[best];
        bits[best] = bits[best] == 1 ? 2 : 4;
    }
    return OK;
}

/* ------------------------------------------------------------------------------------------
 * Adapter gradients of the layer y = x What^T + s (x A^T) B^T (Sec. 2.1; only the low-rank
 * tensors are trained, Sec. 3).  With dY the gradient of the loss with respect to y:
 *   G1  dB[n,j] = s sum_m dY[m,n] t[m,j],   t = x A^T   [M,r]
 *   G2  dA[j,k] = s sum_m u[m,j] x[m,k],    u = dY B    [M,r]
 * fp64 on the bf16 inputs.  The quantized base does not enter.
 */
int lowra_oracle_adapter_grads(int N, int K, int M, int r, const uint16_t* x, const uint16_t* dY,
                               const uint16_t* A, const uint16_t* B, float s, double* dA, double* dB) {
    if (N < 0 || K <= 0 || M < 0 || r <= 0) return ERR_ARG;
    double* t = (double*)malloc(sizeof(double) * ((size_t)M * r + 1));
    double* u = (double*)malloc(sizeof(double) * ((size_t)M * r + 1));
    if (!t || !u) { free(t); free(u); return ERR_ALLOC; }
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m)
        for (int j = 0; j < r; ++j) {
            double acc = 0.0;
            for (int k = 0; k < K; ++k)
                acc += (double)bf16_to_float(x[(size_t)m * K + k]) * (double)bf16_to_float(A[(size_t)j * K + k]);
            t[(size_t)m * r + j] = acc;
            acc = 0.0;
            for (int n = 0; n < N; ++n)
                acc += (double)bf16_to_float(dY[(size_t)m * N + n]) * (double)bf16_to_float(B[(size_t)n * r + j]);
            u[(size_t)m * r + j] = acc;
        }
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)                              /* G1 */
        for (int j = 0; j < r; ++j) {
            double acc = 0.0;
            for (int m = 0; m < M; ++m) acc += (double)bf16_to_float(dY[(size_t)m * N + n]) * t[(size_t)m * r + j];
            dB[(size_t)n * r + j] = (double)s * acc;
        }
#pragma omp parallel for schedule(static)
    for (int j = 0; j < r; ++j)                              /* G2 */
        for (int k = 0; k < K; ++k) {
            double acc = 0.0;
            for (int m = 0; m < M; ++m) acc += u[(size_t)m * r + j] * (double)bf16_to_float(x[(size_t)m * K + k]);
            dA[(size_t)j * K + k] = (double)s * acc;
        }
    free(t); free(u);
    return OK;
}
