// Host side of the two linear entry points: workspace layout and launch sequence.
//
//   forward        y  = x  What^T + s (x A^T) B^T        (Sec. 2.1 LoRA form, Sec. 3 step P5)
//   input gradient dX = dY What   + s (dY B) A           (the base is frozen: no dW, Sec. 3)
//
// The LoRA term rides inside the fused GEMM as an extension of the contraction: the forward runs
// over [x | t] against [What | B] with t = s x A^T, the backward over [dY | u] against [What ; A]
// with u = s dY B.  t and u ([M, RP], RP = r rounded up to 64) come from a small MFMA kernel.
#include <algorithm>
#include <atomic>
#include <new>

#include "gemm_common.h"

namespace lowra {

hipError_t launch_gemm_fwd(const GemmParams& p, int tiling, hipStream_t st);
hipError_t launch_gemm_bwd(const GemmParams& p, hipStream_t st);
BwdSplitPlan gemm_bwd_split_plan(int N, int K, int M);
hipError_t launch_gemv_fwd(const GemvParams& p, hipStream_t st);
hipError_t launch_skinny_ws(const uint16_t* P, int ldp, int M, const uint16_t* Q, int ldq, int r, int Kc,
                            float s, uint16_t* out, int RP, float* scratch, hipStream_t st);
size_t skinny_scratch_bytes(int M, int Kc, int RP);
hipError_t launch_skinny_qt(const uint16_t* P, int ldp, int M, const uint16_t* Qt, int Kc, float s, uint16_t* out,
                            float* scratch, hipStream_t st);
hipError_t launch_pad_cols(const uint16_t* src, int R, int c, uint16_t* dst, int CP, hipStream_t st);
hipError_t launch_transpose(const uint16_t* src, int R, int c, uint16_t* dst, hipStream_t st);

// measurement hook (lowra_set_kernel_timer): events recorded around the dominant kernel of a call only.
// The pair is published as one atomic pointer to an immutable record, so a call running on another
// thread sees either the old pair or the new one, never a mix; records are kept until the process ends
// (a call may still hold one), which costs 16 bytes per lowra_set_kernel_timer call.
struct TimerPair { hipEvent_t start, stop; };
static std::atomic<const TimerPair*> g_timer{nullptr};
void set_kernel_timer(hipEvent_t start, hipEvent_t stop) {
    const TimerPair* p = start ? new (std::nothrow) TimerPair{start, stop} : nullptr;
    g_timer.store(p, std::memory_order_release);
}
KernelTimer::KernelTimer(hipStream_t s) : st(s), pair(g_timer.load(std::memory_order_acquire)) {
    if (pair) (void)hipEventRecord(static_cast<const TimerPair*>(pair)->start, st);
}
KernelTimer::~KernelTimer() { if (pair) (void)hipEventRecord(static_cast<const TimerPair*>(pair)->stop, st); }

// dst[0 .. count) = +0 in bf16, by a kernel (a memset node in a captured graph is avoided on purpose)
__global__ __launch_bounds__(256) void zero_bf16_kernel(uint16_t* __restrict__ dst, size_t count) {
    const size_t stride = (size_t)gridDim.x * 256 * 8;
    for (size_t o = ((size_t)blockIdx.x * 256 + threadIdx.x) * 8; o < count; o += stride) {
        if (o + 8 <= count) *reinterpret_cast<uint4*>(dst + o) = make_uint4(0u, 0u, 0u, 0u);   // dst is 16-byte aligned
        else for (size_t e = o; e < count; ++e) dst[e] = 0;
    }
}
hipError_t launch_zero_bf16(uint16_t* dst, size_t count, hipStream_t st) {
    if (count == 0) return hipSuccess;
    const unsigned grid = (unsigned)std::min<size_t>((count + 2047) / 2048, 2048);
    zero_bf16_kernel<<<dim3(grid), dim3(256), 0, st>>>(dst, count);
    return hipGetLastError();
}

static inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }
static inline int round_up(int v, int m) { return (v + m - 1) / m * m; }

// bf16 group scales widened to fp32 (exact) for the kernels that read fp32 scales; the copy sits at the end of
// the call's workspace.
__global__ __launch_bounds__(256) void expand_scales_kernel(const uint16_t* __restrict__ src, size_t count, float* __restrict__ dst) {
    for (size_t o = (size_t)blockIdx.x * 256 + threadIdx.x; o < count; o += (size_t)gridDim.x * 256)
        dst[o] = bf16_bits_to_float(src[o]);
}
hipError_t launch_expand_scales(const uint16_t* src, size_t count, float* dst, hipStream_t st) {
    if (count == 0) return hipSuccess;
    const unsigned grid = (unsigned)std::min<size_t>((count + 255) / 256, 4096);
    expand_scales_kernel<<<dim3(grid), dim3(256), 0, st>>>(src, count, dst);
    return hipGetLastError();
}
size_t expanded_scale_bytes(const lowra_layout& L) {
    return L.scale_bf16 ? align256((size_t)L.N * L.G * sizeof(float)) : 0;
}

// forward:  [ t : M x RP ][ B padded : N x RP, only when r % 64 != 0 ][ partial sums of t, tall inputs only ]
// backward: [ u : M x RP ][ B^T : r x N, used unless r == 64 ][ partial sums of u, tall inputs only ]
static size_t gemv_workspace_bytes(const lowra_layout& L, int r);
static size_t linear_workspace_bytes_fp32(const lowra_layout& L, int op, int M, int r);
static size_t bwd_split_bytes(const lowra_layout& L, int M);
size_t linear_workspace_bytes(const lowra_layout& L, int op, int M, int r) {
    return align256(linear_workspace_bytes_fp32(L, op, M, r)) + expanded_scale_bytes(L);
}
// With bf16 scales: widen them behind the call's own scratch and run the call on the copy.
static hipError_t with_fp32_scales(const lowra_layout& L, int op, const LinearArgs& a, LinearArgs& b, bool native, hipStream_t st) {
    b = a;
    if (!L.scale_bf16 || native) return hipSuccess;                // the streaming small-token kernels read bf16 scales themselves
    float* dst = reinterpret_cast<float*>(static_cast<uint8_t*>(a.workspace) + align256(linear_workspace_bytes_fp32(L, op, a.M, a.r)));
    b.absmax = dst;
    return launch_expand_scales(reinterpret_cast<const uint16_t*>(a.absmax), (size_t)L.N * L.G, dst, st);
}
static size_t linear_workspace_bytes_fp32(const lowra_layout& L, int op, int M, int r) {
    if (r <= 0) {    // no rank-r term: only the streaming small-token kernels need scratch (descriptors, partial results)
        if (op == 0) return M >= 1 && M <= 16 && gemv_stream_supported(L, M, 0) ? gemv_stream_workspace_bytes(L, M, 0) : 0;
        const size_t small = M >= 1 && M <= 16 && gemv_stream_bwd_supported(L, M, 0) ? gemv_stream_bwd_workspace_bytes(L, M, 0) : 0;
        return std::max(small, bwd_split_bytes(L, M));
    }
    const size_t RP = (size_t)round_up(r, BK);
    const size_t t = align256((size_t)M * RP * 2);
    if (op == 0) {
        const size_t gemm = t + ((size_t)r == RP ? 0 : align256((size_t)L.N * RP * 2)) + skinny_scratch_bytes(M, L.K, (int)RP);
        size_t small = 0;                                                           // either path may be chosen
        if (M <= 16) small = std::max(gemv_workspace_bytes(L, r), gemv_stream_supported(L, M, r) ? gemv_stream_workspace_bytes(L, M, r) : 0);
        return std::max(gemm, small);
    }
    const size_t gemm = t + align256((size_t)r * L.N * 2) + align256(skinny_scratch_bytes(M, L.N, (int)RP)) + bwd_split_bytes(L, M);
    return M <= 16 && gemv_stream_bwd_supported(L, M, r) ? std::max(gemm, gemv_stream_bwd_workspace_bytes(L, M, r)) : gemm;
}

static void fill_params(GemmParams& p, const lowra_layout& L, const LinearArgs& a, int RP) {
    p.rows = L.d_rows; p.gemm_rows = L.d_gemm_rows; p.tile_order = L.d_tile_order; p.packed = a.packed; p.absmax = a.absmax;
    p.mappings = a.mappings; p.act = a.act; p.ext_act = nullptr; p.ext_w = nullptr; p.lora_A = a.A;
    p.lora_r = a.r; p.out = a.out; p.M = a.M; p.N = L.N; p.K = L.K; p.G = L.G; p.RP = RP;
    p.any4 = L.n_by_bits[4] > 0; p.C = L.C;
    p.ld_act = 0; p.splits = 1; p.rows_per_split = 0; p.split_first = 0; p.split_out = nullptr;
}
// fp32 partial tiles of an input gradient whose contraction is split between workgroups
static size_t bwd_split_bytes(const lowra_layout& L, int M) {
    const BwdSplitPlan pl = gemm_bwd_split_plan(L.N, L.K, M);
    return pl.splits > 1 ? align256((size_t)pl.splits * pl.tail * BM * BN * sizeof(float)) : 0;
}

// The small-token path pads the tokens to one 16-row MFMA tile.
bool gemv_fwd_fits(int K);
bool gemv_fwd_supported(const lowra_layout& L, int M) { return M <= 16 && gemv_fwd_fits(L.K); }
static size_t gemv_workspace_bytes(const lowra_layout& L, int r) {
    return r > 0 ? (size_t)((L.K + 255) / 256) * 16 * round_up(r, 16) * sizeof(float) : 0;
}

hipError_t launch_linear_fwd(const lowra_layout& L, const LinearArgs& a_in, int path, int tiling, hipStream_t st) {
    if (a_in.M == 0 || L.N == 0) return hipSuccess;
    LinearArgs a;
    hipError_t e_scales = with_fp32_scales(L, 0, a_in, a, path == 1 && gemv_stream_supported(L, a_in.M, a_in.r), st);
    if (e_scales != hipSuccess) return e_scales;
    const int RP = a.r > 0 ? round_up(a.r, BK) : 0;
    // A single matrix is too little work for the streaming kernel's set-up (descriptor kernel, tables, pipeline fill):
    // measured 20-50 us per call against 15-25 us for the general kernel.  It runs here only when asked for
    // (LOWRA_PATH_GEMV); the batched entry point is where it pays.
    if (path == 1 && gemv_stream_supported(L, a.M, a.r)) {
        KernelTimer timer(st);
        return launch_gemv_stream(L, a, st);
    }
    if (path != 2 && gemv_fwd_supported(L, a.M)) {     // LOWRA_PATH_AUTO, LOWRA_PATH_GEMV_GENERAL, or a shape the streaming kernel does not take
        GemvParams g;
        g.sorted_rows = L.d_sorted_rows; g.packed = a.packed; g.packed_bytes = L.packed_bytes; g.absmax = a.absmax;
        g.mappings = a.mappings; g.x = a.act; g.A = a.A; g.B = a.B; g.tp = static_cast<float*>(a.workspace);
        g.y = a.out; g.s = a.s;
        g.M = a.M; g.N = L.N; g.K = L.K; g.G = L.G; g.r = a.r; g.RT = a.r > 0 ? round_up(a.r, 16) : 0;
        KernelTimer timer(st);
        return launch_gemv_fwd(g, st);
    }
    GemmParams p;
    fill_params(p, L, a, RP);
    if (RP) {
        uint16_t* ws_t = static_cast<uint16_t*>(a.workspace);
        float* scratch = reinterpret_cast<float*>(static_cast<uint8_t*>(a.workspace) + align256((size_t)a.M * RP * 2) +
                                                  (a.r == RP ? 0 : align256((size_t)L.N * RP * 2)));
        hipError_t e = launch_skinny_ws(a.act, L.K, a.M, a.A, L.K, a.r, L.K, a.s, ws_t, RP, scratch, st);
        if (e != hipSuccess) return e;
        p.ext_act = ws_t;
        p.ext_w = a.B;
        if (a.r != RP) {
            uint16_t* ws_b = reinterpret_cast<uint16_t*>(static_cast<uint8_t*>(a.workspace) + align256((size_t)a.M * RP * 2));
            if ((e = launch_pad_cols(a.B, L.N, a.r, ws_b, RP, st)) != hipSuccess) return e;
            p.ext_w = ws_b;
        }
    }
    KernelTimer timer(st);
    return launch_gemm_fwd(p, tiling, st);
}

hipError_t launch_linear_bwd_input(const lowra_layout& L, const LinearArgs& a_in, int path, hipStream_t st) {
    if (a_in.M == 0) return hipSuccess;
    LinearArgs a;
    hipError_t e_scales = with_fp32_scales(L, 1, a_in, a, path != 2 && gemv_stream_bwd_supported(L, a_in.M, a_in.r), st);
    if (e_scales != hipSuccess) return e_scales;
    // Few tokens: the streaming kernel reads the codes once at the memory's pace (the GEMM below would pad the tokens
    // to a 256-row tile).  LOWRA_PATH_GEMM keeps the GEMM.
    if (path != 2 && gemv_stream_bwd_supported(L, a.M, a.r)) {
        KernelTimer timer(st);
        return launch_gemv_stream_bwd(L, a, st);
    }
    const int RP = a.r > 0 ? round_up(a.r, BK) : 0;
    GemmParams p;
    fill_params(p, L, a, RP);
    p.ld_act = L.N;
    const BwdSplitPlan split_plan = gemm_bwd_split_plan(L.N, L.K, a.M);
    p.splits = split_plan.splits;
    if (p.splits > 1) {           // the partial tiles sit behind the rank-r term's scratch
        p.rows_per_split = split_plan.rows_per_split;
        p.split_first = split_plan.first;
        const size_t before = RP ? align256((size_t)a.M * RP * 2) + align256((size_t)a.r * L.N * 2) + align256(skinny_scratch_bytes(a.M, L.N, RP)) : 0;
        p.split_out = reinterpret_cast<float*>(static_cast<uint8_t*>(a.workspace) + before);
    }
    if (RP) {
        uint8_t* ws = static_cast<uint8_t*>(a.workspace);
        uint16_t* ws_u = reinterpret_cast<uint16_t*>(ws);
        uint16_t* ws_bt = reinterpret_cast<uint16_t*>(ws + align256((size_t)a.M * RP * 2));
        float* scratch = reinterpret_cast<float*>(ws + align256((size_t)a.M * RP * 2) + align256((size_t)a.r * L.N * 2));
        hipError_t e;
        if (a.r == 64) {                                                     // B [N, 64] is read in place
            if ((e = launch_skinny_qt(a.act, L.N, a.M, a.B, L.N, a.s, ws_u, scratch, st)) != hipSuccess) return e;
        } else {
            if ((e = launch_transpose(a.B, L.N, a.r, ws_bt, st)) != hipSuccess) return e;          // B^T [r, N]
            if ((e = launch_skinny_ws(a.act, L.N, a.M, ws_bt, L.N, a.r, L.N, a.s, ws_u, RP, scratch, st)) != hipSuccess) return e;
        }
        p.ext_act = ws_u;
    }
    KernelTimer timer(st);
    return launch_gemm_bwd(p, st);
}

}  // namespace lowra
