// C ABI of the LowRA HIP library: host-side validation, layout planning, dispatch.
#include <algorithm>
#include <atomic>
#include <mutex>
#include <new>
#include <numeric>

#include "../../include/lowra.h"
#include "gemm_common.h"

namespace {

std::atomic<int> g_linear_path{LOWRA_PATH_AUTO};
std::atomic<int> g_fwd_tiling{-1};        // lowra_set_fwd_tiling: -1 = the planner chooses
constexpr int kMaxRank = 128;
constexpr int kFwdTileRows = 256;

bool valid_bits(int b) { return b == 1 || b == 2 || b == 4; }
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

lowra_status plan_rows(int N, int K, int group, const uint8_t* bits, int64_t* off) {
    if (!bits && N > 0) return LOWRA_INVALID_ARG;
    if (!off || N < 0 || K <= 0) return LOWRA_INVALID_ARG;
    if (group != lowra::kGroup || K % lowra::kGroup != 0) return LOWRA_UNSUPPORTED;
    off[0] = 0;
    for (int n = 0; n < N; ++n) {
        if (!valid_bits(bits[n])) return LOWRA_UNSUPPORTED;
        off[n + 1] = off[n] + (int64_t)K * bits[n] / 8;
    }
    if (off[N] >= ((int64_t)1 << 32)) return LOWRA_UNSUPPORTED;   // rows are addressed with 32-bit byte offsets
    return LOWRA_OK;
}

}  // namespace

// ---- scratch of lowra_linear_fwd_static: device memory that exists without any allocation call.
// Every GPU the library runs on holds its own copy of this array, at its own address, until the
// process ends.  In host code the array's NAME is only a handle for hipGetSymbolAddress: the device
// address is looked up once per device (with that device current) and kept; kernels and copies only
// ever get that looked-up pointer.
static __device__ __align__(256) unsigned char scratch[LOWRA_STATIC_SCRATCH_BYTES];
namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (null on failure).  The first call on a device does
// the lookup (which may load the library's code object there); later calls only read the table.
void* static_scratch_of_current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}
}  // namespace

extern "C" {

const char* lowra_status_string(lowra_status st) {
    switch (st) {
        case LOWRA_OK: return "ok";
        case LOWRA_INVALID_ARG: return "invalid argument";
        case LOWRA_UNSUPPORTED: return "unsupported configuration";
        case LOWRA_MISALIGNED: return "pointer not 16-byte aligned";
        case LOWRA_WORKSPACE_TOO_SMALL: return "workspace too small";
        case LOWRA_HIP_ERROR: return "HIP runtime error";
        case LOWRA_OUT_OF_MEMORY: return "host allocation failed";
        default: return "unknown status";
    }
}

lowra_status lowra_plan_rows(int N, int K, int group, const uint8_t* bits_host, int64_t* row_offset_host) {
    return plan_rows(N, K, group, bits_host, row_offset_host);
}

// The body of lowra_layout_create.  `L` is owned by the caller (the wrapper below destroys it on any
// failure, including an exception from a host container).
static lowra_status layout_create_impl(int N, int K, int group, const uint8_t* bits_host,
                                       const int32_t* codebook_id_host, int C,
                                       const uint8_t* codebook_bits_host, lowra_layout*& L) {
    L = new (std::nothrow) lowra_layout();
    if (!L) return LOWRA_OUT_OF_MEMORY;
    L->row_offset.resize((size_t)N + 1);
    lowra_status st = plan_rows(N, K, group, bits_host, L->row_offset.data());
    if (st != LOWRA_OK) return st;
    for (int c = 0; c < C; ++c)
        if (!valid_bits(codebook_bits_host[c])) return LOWRA_UNSUPPORTED;
    for (int n = 0; n < N; ++n) {
        const int c = codebook_id_host[n];
        if (c < 0 || c >= C || codebook_bits_host[c] != bits_host[n]) return LOWRA_INVALID_ARG;
    }
    L->N = N; L->K = K; L->G = K / lowra::kGroup; L->C = C;
    L->packed_bytes = (size_t)L->row_offset[N];
    L->bits.assign(bits_host, bits_host + N);
    L->cb.assign(codebook_id_host, codebook_id_host + N);
    for (int n = 0; n < N; ++n) L->n_by_bits[bits_host[n]]++;

    // per-channel records and the width-sorted order inside every 256-row forward tile
    std::vector<lowra::RowInfo> rows((size_t)N);
    for (int n = 0; n < N; ++n) {
        rows[n].offset = (uint32_t)L->row_offset[n];
        rows[n].bits_cb = (uint32_t)bits_host[n] | ((uint32_t)codebook_id_host[n] << 8);
    }
    const int tiles = (N + kFwdTileRows - 1) / kFwdTileRows;
    // order: rows of every tile stably sorted by width (the small-token kernel walks it);
    // gemm_order: natural order, except that a tile holding 4-bit rows moves them behind the others
    // (the forward GEMM's wavefronts own runs of 64 positions and decode 1- and 2-bit rows alike)
    std::vector<uint16_t> order((size_t)tiles * kFwdTileRows), gemm_order((size_t)tiles * kFwdTileRows);
    for (int t = 0; t < tiles; ++t) {
        uint16_t* o = order.data() + (size_t)t * kFwdTileRows;
        uint16_t* go = gemm_order.data() + (size_t)t * kFwdTileRows;
        auto width = [&](uint16_t a) { const int n = t * kFwdTileRows + a; return n < N ? (int)bits_host[n] : 8; };
        std::iota(o, o + kFwdTileRows, (uint16_t)0);
        std::stable_sort(o, o + kFwdTileRows, [&](uint16_t a, uint16_t b) { return width(a) < width(b); });
        std::iota(go, go + kFwdTileRows, (uint16_t)0);
        std::stable_partition(go, go + kFwdTileRows, [&](uint16_t a) { return width(a) != 4; });
    }

    std::vector<lowra::SortedRow> sorted(order.size());
    for (size_t idx = 0; idx < order.size(); ++idx) {
        const int n = (int)(idx / kFwdTileRows) * kFwdTileRows + order[idx];
        if (n < N) sorted[idx] = lowra::SortedRow{rows[n].offset, rows[n].bits_cb, n, 0};
        else sorted[idx] = lowra::SortedRow{0u, 1u, -1, 0};
    }

    // the forward GEMM's row order as records too: one load gives a lane everything about its row
    std::vector<lowra::SortedRow> gemm_rows(gemm_order.size());
    for (size_t idx = 0; idx < gemm_order.size(); ++idx) {
        const int n = (int)(idx / kFwdTileRows) * kFwdTileRows + gemm_order[idx];
        if (n < N) gemm_rows[idx] = lowra::SortedRow{rows[n].offset, rows[n].bits_cb, n, 0};
        else gemm_rows[idx] = lowra::SortedRow{0u, 1u, -1, (int32_t)gemm_order[idx]};
    }

    // the streaming small-token kernel's order: classes (width, table) in ascending order, rows of a class in
    // channel order, every class padded to whole 16-row strips
    L->cb_bits.assign(codebook_bits_host, codebook_bits_host + C);
    std::vector<lowra::GvRow> gv;
    {
        std::vector<uint32_t> keys;                                   // distinct width | table << 8, ascending
        for (int n = 0; n < N && keys.size() <= (size_t)lowra::kGvMaxClasses; ++n)
            if (std::find(keys.begin(), keys.end(), rows[n].bits_cb) == keys.end()) keys.push_back(rows[n].bits_cb);
        if (N > 0 && keys.size() <= (size_t)lowra::kGvMaxClasses) {
            std::sort(keys.begin(), keys.end(), [](uint32_t a, uint32_t b) {
                return (a & 0xffu) != (b & 0xffu) ? (a & 0xffu) < (b & 0xffu) : a < b; });
            L->gv_nclasses = (int)keys.size();
            for (size_t c = 0; c < keys.size(); ++c) {
                uint32_t first_off = 0; bool have = false;
                for (int n = 0; n < N; ++n)
                    if (rows[n].bits_cb == keys[c]) {
                        if (!have) { first_off = rows[n].offset; have = true; }
                        gv.push_back(lowra::GvRow{rows[n].offset, n});
                    }
                while (gv.size() % 16) gv.push_back(lowra::GvRow{first_off, -1});
                L->gv_cls_end[c] = (int)(gv.size() / 16);
                L->gv_cls_bits_cb[c] = (int)keys[c];
            }
            for (size_t c = keys.size(); c < (size_t)lowra::kGvMaxClasses; ++c) {
                L->gv_cls_end[c] = (int)(gv.size() / 16);
                L->gv_cls_bits_cb[c] = L->gv_cls_bits_cb[keys.size() - 1];
            }
            L->gv_nstrips = (int)(gv.size() / 16);
        }
    }

    if (hipGetDevice(&L->device) != hipSuccess) return LOWRA_HIP_ERROR;
    // every use of the library on a device starts here: look up this device's static scratch now, so that
    // lowra_linear_fwd_static finds it ready (e.g. under graph capture)
    if (!static_scratch_of_current_device()) return LOWRA_HIP_ERROR;
    if (N > 0) {
        if (hipMalloc(reinterpret_cast<void**>(&L->d_rows), rows.size() * sizeof(lowra::RowInfo)) != hipSuccess ||
            hipMalloc(reinterpret_cast<void**>(&L->d_tile_order), order.size() * sizeof(uint16_t)) != hipSuccess ||
            hipMalloc(reinterpret_cast<void**>(&L->d_sorted_rows), sorted.size() * sizeof(lowra::SortedRow)) != hipSuccess ||
            hipMalloc(reinterpret_cast<void**>(&L->d_gemm_rows), gemm_rows.size() * sizeof(lowra::SortedRow)) != hipSuccess ||
            hipMemcpy(L->d_gemm_rows, gemm_rows.data(), gemm_rows.size() * sizeof(lowra::SortedRow), hipMemcpyHostToDevice) != hipSuccess ||
            hipMemcpy(L->d_sorted_rows, sorted.data(), sorted.size() * sizeof(lowra::SortedRow), hipMemcpyHostToDevice) != hipSuccess ||
            hipMemcpy(L->d_rows, rows.data(), rows.size() * sizeof(lowra::RowInfo), hipMemcpyHostToDevice) != hipSuccess ||
            hipMemcpy(L->d_tile_order, gemm_order.data(), gemm_order.size() * sizeof(uint16_t), hipMemcpyHostToDevice) != hipSuccess) {
            (void)hipGetLastError();
            return LOWRA_HIP_ERROR;
        }
        if (!gv.empty() &&
            (hipMalloc(reinterpret_cast<void**>(&L->d_gv_rows), gv.size() * sizeof(lowra::GvRow)) != hipSuccess ||
             hipMemcpy(L->d_gv_rows, gv.data(), gv.size() * sizeof(lowra::GvRow), hipMemcpyHostToDevice) != hipSuccess)) {
            (void)hipGetLastError();
            return LOWRA_HIP_ERROR;
        }
    }
    return LOWRA_OK;
}

lowra_status lowra_layout_create(int N, int K, int group, const uint8_t* bits_host,
                                 const int32_t* codebook_id_host, int C,
                                 const uint8_t* codebook_bits_host, lowra_layout** out) {
    if (!out) return LOWRA_INVALID_ARG;
    *out = nullptr;
    if (N < 0 || K <= 0 || C <= 0 || !codebook_bits_host) return LOWRA_INVALID_ARG;
    if (N > 0 && (!bits_host || !codebook_id_host)) return LOWRA_INVALID_ARG;
    if (C >= (1 << 24)) return LOWRA_UNSUPPORTED;
    lowra_layout* L = nullptr;
    lowra_status st;
    try {
        st = layout_create_impl(N, K, group, bits_host, codebook_id_host, C, codebook_bits_host, L);
    } catch (const std::bad_alloc&) {
        st = LOWRA_OUT_OF_MEMORY;
    } catch (...) {
        st = LOWRA_INVALID_ARG;
    }
    if (st != LOWRA_OK) { lowra_layout_destroy(L); return st; }
    *out = L;
    return LOWRA_OK;
}


void lowra_layout_destroy(lowra_layout* L) {
    if (!L) return;
    if (L->d_rows) (void)hipFree(L->d_rows);
    if (L->d_tile_order) (void)hipFree(L->d_tile_order);
    if (L->d_sorted_rows) (void)hipFree(L->d_sorted_rows);
    if (L->d_gemm_rows) (void)hipFree(L->d_gemm_rows);
    if (L->d_gv_rows) (void)hipFree(L->d_gv_rows);
    delete L;
}

size_t lowra_packed_bytes(const lowra_layout* L) { return L ? L->packed_bytes : 0; }

lowra_status lowra_layout_set_scale_dtype(lowra_layout* L, int scale_dtype) {
    if (!L || (scale_dtype != LOWRA_SCALE_FP32 && scale_dtype != LOWRA_SCALE_BF16)) return LOWRA_INVALID_ARG;
    L->scale_bf16 = scale_dtype == LOWRA_SCALE_BF16;
    return LOWRA_OK;
}

size_t lowra_workspace_bytes(const lowra_layout* L, int op, int M, int r) {
    if (!L || r < 0) return 0;
    if ((op == LOWRA_OP_LINEAR_FWD || op == LOWRA_OP_LINEAR_BWD_INPUT) && M > 0) return lowra::linear_workspace_bytes(*L, op, M, r);   // may need scratch at rank 0 too
    if (r == 0) return 0;
    if (op == LOWRA_OP_LOFTQ_INIT) return r <= 64 ? lowra::loftq_workspace_bytes(*L, r) : 0;      // no token count
    if (M <= 0) return 0;
    if (op == LOWRA_OP_ADAPTER_GRADS) return lowra::adapter_grads_workspace_bytes(*L, M, r);
    if (op != LOWRA_OP_LINEAR_FWD && op != LOWRA_OP_LINEAR_BWD_INPUT) return 0;
    return lowra::linear_workspace_bytes(*L, op, M, r);
}

lowra_status lowra_quantize(const lowra_layout* L, const float* W, const float* thresholds,
                            uint8_t* packed, float* absmax, void* stream) {
    if (!L || !thresholds) return LOWRA_INVALID_ARG;
    if (L->N == 0) return LOWRA_OK;
    if (!W || !packed || !absmax) return LOWRA_INVALID_ARG;
    if (!aligned16(W) || !aligned16(thresholds) || !aligned16(packed) || !aligned16(absmax)) return LOWRA_MISALIGNED;
    return lowra::launch_quantize(*L, W, thresholds, packed, absmax, static_cast<hipStream_t>(stream)) == hipSuccess
               ? LOWRA_OK : LOWRA_HIP_ERROR;
}

lowra_status lowra_quantize_batch(int count, const lowra_layout* const* layouts, const float* const* W,
                                  const float* const* thresholds, uint8_t* const* packed, float* const* absmax,
                                  void* stream) {
    if (count < 0) return LOWRA_INVALID_ARG;
    if (count == 0) return LOWRA_OK;
    if (!layouts || !W || !thresholds || !packed || !absmax) return LOWRA_INVALID_ARG;
    for (int i = 0; i < count; ++i) {                      // everything is checked before anything is launched
        const lowra_layout* L = layouts[i];
        if (!L || !thresholds[i]) return LOWRA_INVALID_ARG;
        if (L->N == 0) continue;
        if (!W[i] || !packed[i] || !absmax[i]) return LOWRA_INVALID_ARG;
        if (!aligned16(W[i]) || !aligned16(thresholds[i]) || !aligned16(packed[i]) || !aligned16(absmax[i])) return LOWRA_MISALIGNED;
    }
    return lowra::launch_quantize_batch(count, layouts, W, thresholds, packed, reinterpret_cast<void* const*>(absmax),
                                        static_cast<hipStream_t>(stream)) == hipSuccess
               ? LOWRA_OK : LOWRA_HIP_ERROR;
}

lowra_status lowra_dequantize(const lowra_layout* L, const uint8_t* packed, const float* absmax,
                              const float* mappings, int out_dtype, void* out, void* stream) {
    if (!L || !mappings) return LOWRA_INVALID_ARG;
    if (out_dtype != LOWRA_OUT_BF16 && out_dtype != LOWRA_OUT_FP32) return LOWRA_INVALID_ARG;
    if (L->N == 0) return LOWRA_OK;
    if (!packed || !absmax || !out) return LOWRA_INVALID_ARG;
    if (!aligned16(packed) || !aligned16(absmax) || !aligned16(mappings) || !aligned16(out)) return LOWRA_MISALIGNED;
    return lowra::launch_dequantize(*L, packed, absmax, mappings, out_dtype, out, static_cast<hipStream_t>(stream)) == hipSuccess
               ? LOWRA_OK : LOWRA_HIP_ERROR;
}

lowra_status lowra_learn_tables(const lowra_layout* L, const float* W, const float* init_thresholds,
                                const float* init_mappings, int iterations, float* thresholds_out,
                                float* mappings_out, float* mse_out, void* stream) {
    if (!L || !init_thresholds || !init_mappings || iterations < 0) return LOWRA_INVALID_ARG;
    if (iterations > 64 || !lowra::learn_supported(L->K)) return LOWRA_UNSUPPORTED;
    if (L->N == 0) return LOWRA_OK;
    if (!W || !thresholds_out || !mappings_out || !mse_out) return LOWRA_INVALID_ARG;
    if (!aligned16(W) || !aligned16(init_thresholds) || !aligned16(init_mappings) || !aligned16(thresholds_out) ||
        !aligned16(mappings_out) || !aligned16(mse_out))
        return LOWRA_MISALIGNED;
    return lowra::launch_learn_tables(*L, W, init_thresholds, init_mappings, iterations, thresholds_out, mappings_out,
                                      mse_out, static_cast<hipStream_t>(stream)) == hipSuccess ? LOWRA_OK : LOWRA_HIP_ERROR;
}

lowra_status lowra_average_thresholds(const lowra_layout* L, float* thresholds, void* stream) {
    if (!L) return LOWRA_INVALID_ARG;
    if (L->N == 0) return LOWRA_OK;
    if (!thresholds) return LOWRA_INVALID_ARG;
    if (!aligned16(thresholds)) return LOWRA_MISALIGNED;
    return lowra::launch_average_thresholds(*L, thresholds, static_cast<hipStream_t>(stream)) == hipSuccess ? LOWRA_OK : LOWRA_HIP_ERROR;
}

lowra_status lowra_adapter_grads(const lowra_layout* L, const uint16_t* x, const uint16_t* dY, int M,
                                 const uint16_t* A, const uint16_t* B, int r, float s, float* dA, float* dB,
                                 void* workspace, size_t workspace_bytes, void* stream) {
    if (!L || M < 0 || r <= 0) return LOWRA_INVALID_ARG;
    if (L->N % 8 != 0 || r > 64) return LOWRA_UNSUPPORTED;
    if (!A || !B || !dA || !dB) return LOWRA_INVALID_ARG;
    if (!aligned16(A) || !aligned16(B) || !aligned16(dA) || !aligned16(dB)) return LOWRA_MISALIGNED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (M == 0 || L->N == 0) {       // no tokens or no channels: both gradients are zero
        return lowra::launch_zero_grads(L->N, L->K, r, dA, dB, st) == hipSuccess ? LOWRA_OK : LOWRA_HIP_ERROR;
    }
    if (!x || !dY || !workspace) return LOWRA_INVALID_ARG;
    if (!aligned16(x) || !aligned16(dY) || !aligned16(workspace)) return LOWRA_MISALIGNED;
    if (workspace_bytes < lowra::adapter_grads_workspace_bytes(*L, M, r)) return LOWRA_WORKSPACE_TOO_SMALL;
    return lowra::launch_adapter_grads(*L, x, dY, M, A, B, r, s, dA, dB, workspace, st) == hipSuccess ? LOWRA_OK : LOWRA_HIP_ERROR;
}

const uint16_t* lowra_linear_side_product(const lowra_layout* L, int op, int M, int r, const void* workspace) {
    if (!L || !workspace || (op != LOWRA_OP_LINEAR_FWD && op != LOWRA_OP_LINEAR_BWD_INPUT)) return nullptr;
    if (r <= 0 || r > 64 || M <= 0 || L->N == 0) return nullptr;
    if (M <= 16 && g_linear_path.load() != LOWRA_PATH_GEMM) return nullptr;       // a small-token kernel ran: no [M][64] intermediate
    return static_cast<const uint16_t*>(workspace);
}

lowra_status lowra_adapter_grads_from_side(const lowra_layout* L, const uint16_t* x, const uint16_t* dY, int M, int r,
                                           const uint16_t* st_side, const uint16_t* su_side, float* dA, float* dB,
                                           void* workspace, size_t workspace_bytes, void* stream) {
    if (!L || M < 0 || r <= 0) return LOWRA_INVALID_ARG;
    if (L->N % 8 != 0 || r > 64) return LOWRA_UNSUPPORTED;
    if (!dA || !dB) return LOWRA_INVALID_ARG;
    if (!aligned16(dA) || !aligned16(dB)) return LOWRA_MISALIGNED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (M == 0 || L->N == 0) {       // no tokens or no channels: both gradients are zero
        return lowra::launch_zero_grads(L->N, L->K, r, dA, dB, st) == hipSuccess ? LOWRA_OK : LOWRA_HIP_ERROR;
    }
    if (!x || !dY || !st_side || !su_side || !workspace) return LOWRA_INVALID_ARG;
    if (!aligned16(x) || !aligned16(dY) || !aligned16(st_side) || !aligned16(su_side) || !aligned16(workspace)) return LOWRA_MISALIGNED;
    if (workspace_bytes < lowra::adapter_grads_workspace_bytes(*L, M, r)) return LOWRA_WORKSPACE_TOO_SMALL;
    return lowra::launch_adapter_grads_from_side(*L, x, dY, M, r, st_side, su_side, dA, dB, workspace, st) == hipSuccess ? LOWRA_OK
                                                                                                                        : LOWRA_HIP_ERROR;
}

lowra_status lowra_loftq_init(const lowra_layout* L, const float* W, const float* thresholds, const float* mappings,
                              int r, int steps, int power_iterations, const uint16_t* omega, uint8_t* packed,
                              float* absmax, uint16_t* A, uint16_t* B, void* workspace, size_t workspace_bytes,
                              void* stream) {
    if (!L || !thresholds || !mappings || r < 0 || steps < 1 || power_iterations < 1) return LOWRA_INVALID_ARG;
    if (r > 64 || steps > 64 || power_iterations > 64 || L->scale_bf16) return LOWRA_UNSUPPORTED;
    if (L->N == 0) return LOWRA_OK;
    if (!W || !packed || !absmax) return LOWRA_INVALID_ARG;
    if (!aligned16(W) || !aligned16(thresholds) || !aligned16(mappings) || !aligned16(packed) || !aligned16(absmax)) return LOWRA_MISALIGNED;
    if (r > 0) {
        if (!omega || !A || !B || !workspace) return LOWRA_INVALID_ARG;
        if (!aligned16(omega) || !aligned16(A) || !aligned16(B) || !aligned16(workspace)) return LOWRA_MISALIGNED;
        if (workspace_bytes < lowra::loftq_workspace_bytes(*L, r)) return LOWRA_WORKSPACE_TOO_SMALL;
    }
    return lowra::launch_loftq(*L, W, thresholds, mappings, r, steps, power_iterations, omega, packed, absmax, A, B, workspace,
                               static_cast<hipStream_t>(stream)) == hipSuccess ? LOWRA_OK : LOWRA_HIP_ERROR;
}

lowra_status lowra_channel_mse(int N, int K, const float* W, const float* thresholds3, const float* mappings3,
                               float* mse_out, void* stream) {
    if (N < 0 || K <= 0 || !thresholds3 || !mappings3) return LOWRA_INVALID_ARG;
    if (K % 64 != 0) return LOWRA_UNSUPPORTED;
    if (N == 0) return LOWRA_OK;
    if (!W || !mse_out) return LOWRA_INVALID_ARG;
    if (!aligned16(W) || !aligned16(thresholds3) || !aligned16(mappings3)) return LOWRA_MISALIGNED;
    return lowra::launch_channel_mse(N, K, W, thresholds3, mappings3, mse_out, static_cast<hipStream_t>(stream)) == hipSuccess
               ? LOWRA_OK : LOWRA_HIP_ERROR;
}

lowra_status lowra_assign_precisions(int N, const int64_t* channel_params_host, const float* mse_host,
                                     double budget_bits_per_param, uint8_t* bits_out_host) {
    if (N < 0 || (N > 0 && (!channel_params_host || !mse_host || !bits_out_host))) return LOWRA_INVALID_ARG;
    return lowra::assign_greedy_host(N, channel_params_host, mse_host, budget_bits_per_param, bits_out_host)
               ? LOWRA_OK : LOWRA_INVALID_ARG;
}

static lowra_status check_linear(const lowra_layout* L, int op, const uint8_t* packed, const float* absmax,
                                 const float* mappings, const uint16_t* act, int M, const uint16_t* A,
                                 const uint16_t* B, int r, const uint16_t* out, const void* workspace,
                                 size_t workspace_bytes) {
    if (!L || M < 0 || r < 0) return LOWRA_INVALID_ARG;
    if (L->N % 8 != 0 || r > kMaxRank) return LOWRA_UNSUPPORTED;
    if (M == 0 || L->N == 0) return LOWRA_OK;
    if (!packed || !absmax || !mappings || !act || !out) return LOWRA_INVALID_ARG;
    if (r > 0 && (!A || !B)) return LOWRA_INVALID_ARG;
    if (!aligned16(packed) || !aligned16(absmax) || !aligned16(mappings) || !aligned16(act) || !aligned16(out) ||
        (r > 0 && (!aligned16(A) || !aligned16(B))))
        return LOWRA_MISALIGNED;
    const size_t need = lowra::linear_workspace_bytes(*L, op, M, r);
    if (need > 0) {
        if (!workspace) return LOWRA_INVALID_ARG;
        if (!aligned16(workspace)) return LOWRA_MISALIGNED;
        if (workspace_bytes < need) return LOWRA_WORKSPACE_TOO_SMALL;
    }
    return LOWRA_OK;
}

lowra_status lowra_linear_fwd(const lowra_layout* L, const uint8_t* packed, const float* absmax,
                              const float* mappings, const uint16_t* x, int M, const uint16_t* A,
                              const uint16_t* B, int r, float s, uint16_t* y, void* workspace,
                              size_t workspace_bytes, void* stream) {
    lowra_status st = check_linear(L, LOWRA_OP_LINEAR_FWD, packed, absmax, mappings, x, M, A, B, r, y, workspace, workspace_bytes);
    if (st != LOWRA_OK || M == 0 || L->N == 0) return st;
    lowra::LinearArgs a{packed, absmax, mappings, x, M, A, B, r, s, y, workspace};
    return lowra::launch_linear_fwd(*L, a, g_linear_path.load(), g_fwd_tiling.load(), static_cast<hipStream_t>(stream)) == hipSuccess
               ? LOWRA_OK : LOWRA_HIP_ERROR;
}

lowra_status lowra_linear_fwd_static(const lowra_layout* L, const uint8_t* packed, const float* absmax,
                                     const float* mappings, const uint16_t* x, int M, const uint16_t* A,
                                     const uint16_t* B, int r, float s, uint16_t* y, void* stream) {
    if (!L) return LOWRA_INVALID_ARG;
    const size_t need = M > 0 ? lowra::linear_workspace_bytes(*L, LOWRA_OP_LINEAR_FWD, M, r) : 0;
    if (need > (size_t)LOWRA_STATIC_SCRATCH_BYTES) return LOWRA_WORKSPACE_TOO_SMALL;   // beyond the static scratch: use lowra_linear_fwd
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return LOWRA_HIP_ERROR;
    if (dev != L->device) return LOWRA_INVALID_ARG;               // the layout's index arrays live on another device
    void* ws = static_scratch_of_current_device();
    if (!ws) return LOWRA_HIP_ERROR;
    return lowra_linear_fwd(L, packed, absmax, mappings, x, M, A, B, r, s, y, ws, (size_t)LOWRA_STATIC_SCRATCH_BYTES, stream);
}

lowra_status lowra_linear_bwd_input(const lowra_layout* L, const uint8_t* packed, const float* absmax,
                                    const float* mappings, const uint16_t* dY, int M, const uint16_t* A,
                                    const uint16_t* B, int r, float s, uint16_t* dX, void* workspace,
                                    size_t workspace_bytes, void* stream) {
    lowra_status st = check_linear(L, LOWRA_OP_LINEAR_BWD_INPUT, packed, absmax, mappings, dY, M, A, B, r, dX, workspace, workspace_bytes);
    if (st != LOWRA_OK || M == 0) return st;
    if (L->N == 0) {   // empty contraction: dX = 0, written by a fill kernel (no memset node, so the call can be captured)
        return lowra::launch_zero_bf16(dX, (size_t)M * L->K, static_cast<hipStream_t>(stream)) == hipSuccess ? LOWRA_OK : LOWRA_HIP_ERROR;
    }
    lowra::LinearArgs a{packed, absmax, mappings, dY, M, A, B, r, s, dX, workspace};
    return lowra::launch_linear_bwd_input(*L, a, g_linear_path.load(), static_cast<hipStream_t>(stream)) == hipSuccess
               ? LOWRA_OK : LOWRA_HIP_ERROR;
}

// ---- several small-token forwards in one run
static lowra_status check_batch_item(const lowra_fwd_item& it, int M, int r) {
    if (!it.layout) return LOWRA_INVALID_ARG;
    if (it.layout->N % 8 != 0 || it.layout->N == 0 || !lowra::gemv_fwd_supported(*it.layout, M)) return LOWRA_UNSUPPORTED;
    if (!it.packed || !it.absmax || !it.x || !it.y || (r > 0 && (!it.A || !it.B))) return LOWRA_INVALID_ARG;
    if (!aligned16(it.packed) || !aligned16(it.absmax) || !aligned16(it.x) || !aligned16(it.y) ||
        (r > 0 && (!aligned16(it.A) || !aligned16(it.B))))
        return LOWRA_MISALIGNED;
    return LOWRA_OK;
}
static size_t batch_item_ws(const lowra_layout& L, int r) {
    // the general kernel's partial sums of x A^T, or the streaming kernel's (same size) plus its per-chunk partial outputs
    const size_t b = r > 0 ? (size_t)((L.K + 255) / 256) * 16 * (size_t)((r + 15) / 16 * 16) * sizeof(float) : 0;
    const size_t general = (b + 255) & ~(size_t)255;
    return lowra::gemv_stream_supported(L, 16, r) ? std::max(general, lowra::gemv_stream_batch_item_ws(L, r)) : general;
}

size_t lowra_fwd_batch_workspace_bytes(int n, const lowra_fwd_item* items, int r) {
    if (n <= 0 || !items || r < 0) return 0;
    size_t tot = 0;
    for (int i = 0; i < n; ++i) if (items[i].layout) tot += batch_item_ws(*items[i].layout, r);
    return tot;
}

static lowra_status fwd_batch_create_impl(int n, const lowra_fwd_item* items, const float* mappings, int M, int r, float s,
                                          void* workspace, lowra_fwd_batch*& b) {
    std::vector<lowra::GemvParams> ps;
    std::vector<lowra::GsBatchItem> fast;
    uint8_t* ws = static_cast<uint8_t*>(workspace);
    const int path = g_linear_path.load();
    for (int i = 0; i < n; ++i) {
        const lowra_layout& L = *items[i].layout;
        // the streaming kernel builds one set of tables per launch: its matrices must agree on the codebooks' widths
        const bool stream = path != LOWRA_PATH_GEMV_GENERAL && lowra::gemv_stream_supported(L, M, r) &&
                            (fast.empty() || (fast[0].L->cb_bits == L.cb_bits && fast[0].L->scale_bf16 == L.scale_bf16));
        if (!stream && L.scale_bf16) return LOWRA_UNSUPPORTED;      // the general kernel reads fp32 scales
        if (stream) {
            fast.push_back(lowra::GsBatchItem{&L, items[i].packed, items[i].absmax, items[i].x, items[i].A, items[i].B, items[i].y, ws});
        } else {
            lowra::GemvParams g;
            g.sorted_rows = L.d_sorted_rows; g.packed = items[i].packed; g.packed_bytes = L.packed_bytes; g.absmax = items[i].absmax;
            g.mappings = mappings; g.x = items[i].x; g.A = items[i].A; g.B = items[i].B; g.tp = reinterpret_cast<float*>(ws);
            g.y = items[i].y; g.s = s;
            g.M = M; g.N = L.N; g.K = L.K; g.G = L.G; g.r = r; g.RT = r > 0 ? (r + 15) / 16 * 16 : 0; g.xbufs = 0;
            ps.push_back(g);
        }
        ws += batch_item_ws(L, r);
    }
    b = new (std::nothrow) lowra_fwd_batch;
    if (!b) return LOWRA_OUT_OF_MEMORY;
    (void)hipGetDevice(&b->device);
    if (!ps.empty() && lowra::gemv_batch_build(ps, *b) != hipSuccess) return LOWRA_HIP_ERROR;
    if (!fast.empty() && lowra::gemv_stream_batch_build(fast, mappings, M, r, s, b->gs) != hipSuccess) return LOWRA_HIP_ERROR;
    return LOWRA_OK;
}

lowra_status lowra_fwd_batch_create(int n, const lowra_fwd_item* items, const float* mappings, int M, int r, float s,
                                    void* workspace, size_t workspace_bytes, lowra_fwd_batch** out) {
    if (!out) return LOWRA_INVALID_ARG;
    *out = nullptr;
    if (n <= 0 || !items || !mappings || M < 1 || r < 0) return LOWRA_INVALID_ARG;
    if (M > 16 || r > kMaxRank) return LOWRA_UNSUPPORTED;
    if (!aligned16(mappings)) return LOWRA_MISALIGNED;
    for (int i = 0; i < n; ++i) {
        const lowra_status st = check_batch_item(items[i], M, r);
        if (st != LOWRA_OK) return st;
    }
    const size_t need = lowra_fwd_batch_workspace_bytes(n, items, r);
    if (need > 0) {
        if (!workspace) return LOWRA_INVALID_ARG;
        if (!aligned16(workspace)) return LOWRA_MISALIGNED;
        if (workspace_bytes < need) return LOWRA_WORKSPACE_TOO_SMALL;
    }
    lowra_fwd_batch* b = nullptr;
    lowra_status st;
    try {
        st = fwd_batch_create_impl(n, items, mappings, M, r, s, workspace, b);
    } catch (const std::bad_alloc&) {
        st = LOWRA_OUT_OF_MEMORY;
    } catch (...) {
        st = LOWRA_INVALID_ARG;
    }
    if (st != LOWRA_OK) { (void)hipGetLastError(); lowra_fwd_batch_destroy(b); return st; }
    *out = b;
    return LOWRA_OK;
}

lowra_status lowra_fwd_batch_run(const lowra_fwd_batch* b, void* stream) {
    if (!b) return LOWRA_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (lowra::gemv_stream_batch_run(b->gs, st) != hipSuccess) return LOWRA_HIP_ERROR;
    return lowra::gemv_batch_run(*b, st) == hipSuccess ? LOWRA_OK : LOWRA_HIP_ERROR;
}

void lowra_fwd_batch_destroy(lowra_fwd_batch* b) {
    if (!b) return;
    lowra::gemv_batch_free(*b);
    lowra::gemv_stream_batch_free(b->gs);
    delete b;
}

// ---- several small-token input gradients in one run
static lowra_status check_bwd_item(const lowra_bwd_item& it, int M, int r) {
    if (!it.layout) return LOWRA_INVALID_ARG;
    if (!lowra::gemv_stream_bwd_supported(*it.layout, M, r)) return LOWRA_UNSUPPORTED;
    if (!it.packed || !it.absmax || !it.dY || !it.dX || (r > 0 && (!it.A || !it.B))) return LOWRA_INVALID_ARG;
    if (!aligned16(it.packed) || !aligned16(it.absmax) || !aligned16(it.dY) || !aligned16(it.dX) ||
        (r > 0 && (!aligned16(it.A) || !aligned16(it.B))))
        return LOWRA_MISALIGNED;
    return LOWRA_OK;
}

size_t lowra_bwd_batch_workspace_bytes(int n, const lowra_bwd_item* items, int M, int r) {
    if (n <= 0 || !items || r < 0 || M < 1 || M > 16) return 0;
    size_t tot = 0;
    int chunks = 0;
    for (int i = 0; i < n; ++i)
        if (items[i].layout) { tot += lowra::gemv_stream_bwd_batch_item_ws(*items[i].layout, r); chunks += lowra::gemv_stream_bwd_nchunks(*items[i].layout); }
    return tot + lowra::gemv_stream_bwd_batch_slots_ws(chunks, M);
}

lowra_status lowra_bwd_batch_create(int n, const lowra_bwd_item* items, const float* mappings, int M, int r, float s,
                                    void* workspace, size_t workspace_bytes, lowra_bwd_batch** out) {
    if (!out) return LOWRA_INVALID_ARG;
    *out = nullptr;
    if (n <= 0 || !items || !mappings || M < 1 || r < 0) return LOWRA_INVALID_ARG;
    if (M > 16 || r > kMaxRank) return LOWRA_UNSUPPORTED;
    if (!aligned16(mappings)) return LOWRA_MISALIGNED;
    for (int i = 0; i < n; ++i) {
        const lowra_status st = check_bwd_item(items[i], M, r);
        if (st != LOWRA_OK) return st;
        if (items[i].layout->cb_bits != items[0].layout->cb_bits || items[i].layout->scale_bf16 != items[0].layout->scale_bf16)
            return LOWRA_UNSUPPORTED;                                // one set of decode tables and one scale type per launch
    }
    if (!workspace) return LOWRA_INVALID_ARG;
    if (!aligned16(workspace)) return LOWRA_MISALIGNED;
    if (workspace_bytes < lowra_bwd_batch_workspace_bytes(n, items, M, r)) return LOWRA_WORKSPACE_TOO_SMALL;
    lowra_bwd_batch* b = nullptr;
    lowra_status st = LOWRA_OK;
    try {
        std::vector<lowra::GbBatchItem> v;
        uint8_t* ws = static_cast<uint8_t*>(workspace);
        for (int i = 0; i < n; ++i) {
            v.push_back(lowra::GbBatchItem{items[i].layout, items[i].packed, items[i].absmax, items[i].dY, items[i].A, items[i].B, items[i].dX, ws});
            ws += lowra::gemv_stream_bwd_batch_item_ws(*items[i].layout, r);
        }
        b = new lowra_bwd_batch;
        (void)hipGetDevice(&b->device);
        if (lowra::gemv_stream_bwd_batch_build(v, mappings, M, r, s, reinterpret_cast<float*>(ws), b->gb) != hipSuccess) st = LOWRA_HIP_ERROR;
    } catch (const std::bad_alloc&) {
        st = LOWRA_OUT_OF_MEMORY;
    } catch (...) {
        st = LOWRA_INVALID_ARG;
    }
    if (st != LOWRA_OK) { (void)hipGetLastError(); lowra_bwd_batch_destroy(b); return st; }
    *out = b;
    return LOWRA_OK;
}

lowra_status lowra_bwd_batch_run(const lowra_bwd_batch* b, void* stream) {
    if (!b) return LOWRA_INVALID_ARG;
    return lowra::gemv_stream_bwd_batch_run(b->gb, static_cast<hipStream_t>(stream)) == hipSuccess ? LOWRA_OK : LOWRA_HIP_ERROR;
}

void lowra_bwd_batch_destroy(lowra_bwd_batch* b) {
    if (!b) return;
    lowra::gemv_stream_bwd_batch_free(b->gb);
    delete b;
}

lowra_status lowra_set_kernel_timer(void* start_event, void* stop_event) {
    if ((start_event == nullptr) != (stop_event == nullptr)) return LOWRA_INVALID_ARG;
    lowra::set_kernel_timer(static_cast<hipEvent_t>(start_event), static_cast<hipEvent_t>(stop_event));
    return LOWRA_OK;
}

lowra_status lowra_set_linear_path(int path) {
    if (path != LOWRA_PATH_AUTO && path != LOWRA_PATH_GEMV && path != LOWRA_PATH_GEMM && path != LOWRA_PATH_GEMV_GENERAL) return LOWRA_INVALID_ARG;
    g_linear_path.store(path);
    return LOWRA_OK;
}

lowra_status lowra_plan_fwd_tiling(int N, int M, int compute_units, int* rows_a, int* rows_b, int* cols_a) {
    if (N <= 0 || M <= 0 || compute_units <= 0 || !rows_a || !rows_b || !cols_a) return LOWRA_INVALID_ARG;
    lowra::plan_fwd_tiling(N, M, compute_units, rows_a, rows_b, cols_a);
    return LOWRA_OK;
}

lowra_status lowra_set_fwd_tiling(int rows_a, int rows_b, int cols_a) {
    if (rows_a == 0 && rows_b == 0) { g_fwd_tiling.store(-1); return LOWRA_OK; }
    const auto ok = [](int r) { return r == 256 || r == 192 || r == 128; };
    if (!ok(rows_a) || !ok(rows_b) || rows_b > rows_a || cols_a < 0 || cols_a > 0x7ffff) return LOWRA_INVALID_ARG;
    if (rows_a != rows_b && rows_a == 192 && rows_b != 128) return LOWRA_INVALID_ARG;
    g_fwd_tiling.store((rows_a / 32) << 8 | (rows_b / 32) << 4 | cols_a << 12);
    return LOWRA_OK;
}

}  // extern "C"
