// Internal host-side declarations: the layout object and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "lowra_dev.h"

struct lowra_layout {
    int N = 0, K = 0, G = 0, C = 0;
    int device = -1;
    bool scale_bf16 = false;                // the group scales are stored as bf16 (2 bytes per group) instead of fp32
    size_t packed_bytes = 0;
    int n_by_bits[5] = {0, 0, 0, 0, 0};     // channel count per width
    std::vector<uint8_t> bits;              // host copies
    std::vector<int32_t> cb;
    std::vector<int64_t> row_offset;
    lowra::RowInfo* d_rows = nullptr;       // [N] device
    lowra::SortedRow* d_sorted_rows = nullptr;  // [ceil(N/256)*256] device: rows in per-tile width-sorted order
    lowra::SortedRow* d_gemm_rows = nullptr;    // [ceil(N/256)*256] device: rows in the forward GEMM's per-tile order (pad = local row of a padding entry)
    uint16_t* d_tile_order = nullptr;       // [ceil(N/256)*256] device: per 256-row tile, the forward GEMM's row order (natural, 4-bit rows last)
    // Streaming small-token kernel: all rows of the matrix stably sorted by (width, table) class, every class
    // padded to a multiple of 16 rows, so that a 16-row strip has one width and one table.  Built only when the
    // matrix has at most kGvMaxClasses classes (else gv_nstrips == 0 and that kernel is not used).
    std::vector<uint8_t> cb_bits;           // host copy of codebook_bits [C]
    lowra::GvRow* d_gv_rows = nullptr;      // [gv_nstrips * 16] device
    int gv_nstrips = 0;
    int gv_nclasses = 0;
    int gv_cls_end[4] = {0, 0, 0, 0};       // strips [gv_cls_end[c-1], gv_cls_end[c]) belong to class c
    int gv_cls_bits_cb[4] = {0, 0, 0, 0};   // width | table << 8 of class c
};

namespace lowra {
struct GemvParams;
// one launch of the small-token kernel: the matrices of a batch that take the same instantiation
struct GemvBatchGroup {
    int W, PER;
    size_t sh;                  // dynamic LDS bytes
    int nmat, nstrips;
    GemvParams* d_descs;        // [nmat] device
    int* d_strip0;              // [nmat + 1] device: first 16-channel strip of each matrix
    int* d_owner;               // [nstrips] device: the matrix of each strip
};
}  // namespace lowra

namespace lowra {
// the matrices of a batch that take the streaming small-token kernel: one persistent launch for all of them
struct GsBatchItem {
    const lowra_layout* L;
    const uint8_t* packed; const float* absmax; const uint16_t* x; const uint16_t* A; const uint16_t* B; uint16_t* y;
    uint8_t* ws;                // this matrix's piece of the workspace
};
struct GsBatch {
    void* d_segs = nullptr; int* d_wg_first = nullptr; void* d_units = nullptr; void* d_sums = nullptr;
    void* d_titems = nullptr;
    int nwg = 0, nsums = 0, nt = 0, max_count = 0, M = 0;
    const float* mappings = nullptr;
    std::vector<uint8_t> cb_bits;
    bool scale_bf16 = false;
};
// the same for the streaming small-token input gradient
struct GbBatchItem {
    const lowra_layout* L;
    const uint8_t* packed; const float* absmax; const uint16_t* dY; const uint16_t* A; const uint16_t* B; uint16_t* dX;
    uint8_t* ws;                // this matrix's piece of the workspace
};
struct GbBatch {
    void* d_segs = nullptr; int* d_wg_first = nullptr; int* d_wg_slot0 = nullptr; void* d_units = nullptr;
    void* d_pre = nullptr; void* d_items = nullptr;
    int nwg = 0, nitems = 0, P = 0, M = 0, nslots = 0, max_quads = 0, max_nslots = 0;
    const float* mappings = nullptr;
    float* part = nullptr;      // the batch's partial slots
    std::vector<uint8_t> cb_bits;
    bool scale_bf16 = false;
};
}  // namespace lowra

struct lowra_bwd_batch {
    int device = -1;
    lowra::GbBatch gb;
};

struct lowra_fwd_batch {
    int device = -1;
    lowra::GsBatch gs;
    std::vector<lowra::GemvBatchGroup> groups;
    lowra::GemvParams* d_tdescs = nullptr;   // matrices with a LoRA term, for the partial-sum kernel
    int* d_blk0 = nullptr;                   // [nt + 1] first 256-column block of each
    int* d_towner = nullptr;                 // [nblk_total] the matrix of each block
    int nt = 0, nblk_total = 0;
};

namespace lowra {

// Each launcher validates nothing (the C ABI did) and returns the launch status.
hipError_t launch_quantize(const lowra_layout& L, const float* W, const float* thresholds,
                           uint8_t* packed, void* absmax, hipStream_t st);
constexpr int kQuantizeBatchMax = 8;       // matrices per launch of the batched quantizer
hipError_t launch_quantize_batch(int count, const lowra_layout* const* layouts, const float* const* W,
                                 const float* const* thresholds, uint8_t* const* packed, void* const* absmax, hipStream_t st);
hipError_t launch_dequantize(const lowra_layout& L, const uint8_t* packed, const void* absmax,
                             const float* mappings, int out_dtype, void* out, hipStream_t st);

bool learn_supported(int K);
hipError_t launch_learn_tables(const lowra_layout& L, const float* W, const float* init_thresholds,
                               const float* init_mappings, int iters, float* thr_out, float* map_out,
                               float* mse_out, hipStream_t st);
hipError_t launch_average_thresholds(const lowra_layout& L, float* thr, hipStream_t st);

hipError_t launch_channel_mse(int N, int K, const float* W, const float* thr3, const float* map3, float* mse, hipStream_t st);
bool assign_greedy_host(int N, const int64_t* params, const float* mse, double budget_bpp, uint8_t* bits);

hipError_t launch_zero_grads(int N, int K, int r, float* dA, float* dB, hipStream_t st);
size_t adapter_grads_workspace_bytes(const lowra_layout& L, int M, int r);
hipError_t launch_adapter_grads(const lowra_layout& L, const uint16_t* x, const uint16_t* dY, int M, const uint16_t* A,
                                const uint16_t* B, int r, float s, float* dA, float* dB, void* workspace, hipStream_t st);
hipError_t launch_adapter_grads_from_side(const lowra_layout& L, const uint16_t* x, const uint16_t* dY, int M, int r,
                                          const uint16_t* ts, const uint16_t* us, float* dA, float* dB, void* workspace, hipStream_t st);

size_t loftq_workspace_bytes(const lowra_layout& L, int r);
hipError_t launch_loftq(const lowra_layout& L, const float* W, const float* thresholds, const float* mappings, int r, int steps,
                        int iters, const uint16_t* omega, uint8_t* packed, float* absmax, uint16_t* A_out, uint16_t* B_out,
                        void* workspace, hipStream_t st);

bool gemv_fwd_supported(const lowra_layout& L, int M);
bool gemv_stream_supported(const lowra_layout& L, int M, int r);
size_t gemv_stream_workspace_bytes(const lowra_layout& L, int M, int r);
size_t gemv_stream_batch_item_ws(const lowra_layout& L, int r);
hipError_t gemv_stream_batch_build(const std::vector<GsBatchItem>& items, const float* mappings, int M, int r, float s, GsBatch& b);
hipError_t gemv_stream_batch_run(const GsBatch& b, hipStream_t st);
void gemv_stream_batch_free(GsBatch& b);
bool gemv_stream_bwd_supported(const lowra_layout& L, int M, int r);
size_t gemv_stream_bwd_workspace_bytes(const lowra_layout& L, int M, int r);
size_t gemv_stream_bwd_batch_item_ws(const lowra_layout& L, int r);
size_t gemv_stream_bwd_batch_slots_ws(int nchunks_total, int M);
int gemv_stream_bwd_nchunks(const lowra_layout& L);
hipError_t gemv_stream_bwd_batch_build(const std::vector<GbBatchItem>& items, const float* mappings, int M, int r, float s,
                                       float* part, GbBatch& b);
hipError_t gemv_stream_bwd_batch_run(const GbBatch& b, hipStream_t st);
void gemv_stream_bwd_batch_free(GbBatch& b);
hipError_t gemv_batch_build(std::vector<GemvParams>& items, lowra_fwd_batch& b);
hipError_t gemv_batch_run(const lowra_fwd_batch& b, hipStream_t st);
void gemv_batch_free(lowra_fwd_batch& b);

struct LinearArgs {
    const uint8_t* packed;
    const float* absmax;
    const float* mappings;
    const uint16_t* act;   // x [M,K] (fwd) or dY [M,N] (bwd)
    int M;
    const uint16_t* A;     // [r,K]
    const uint16_t* B;     // [N,r]
    int r;
    float s;
    uint16_t* out;         // y [M,N] (fwd) or dX [M,K] (bwd)
    void* workspace;
};
// bf16 group scales -> fp32 (exact), for the kernels that read fp32 scales
hipError_t launch_expand_scales(const uint16_t* src, size_t count, float* dst, hipStream_t st);
size_t expanded_scale_bytes(const lowra_layout& L);
void set_kernel_timer(hipEvent_t start, hipEvent_t stop);
hipError_t launch_zero_bf16(uint16_t* dst, size_t count, hipStream_t st);
// Records the measurement hook's events (if set) on `st` around the launches made during its lifetime.
struct KernelTimer {
    hipStream_t st;
    const void* pair;      // the event pair that was set when the call started (null: none)
    explicit KernelTimer(hipStream_t s);
    ~KernelTimer();
};
size_t linear_workspace_bytes(const lowra_layout& L, int op, int M, int r);
void plan_fwd_tiling(int N, int M, int units, int* rows_a, int* rows_b, int* cols_a);
// tiling: -1, or the forward GEMM's tile plan forced by lowra_set_fwd_tiling
hipError_t launch_linear_fwd(const lowra_layout& L, const LinearArgs& a, int path, int tiling, hipStream_t st);
hipError_t launch_gemv_stream(const lowra_layout& L, const LinearArgs& a, hipStream_t st);
hipError_t launch_gemv_stream_bwd(const lowra_layout& L, const LinearArgs& a, hipStream_t st);
hipError_t launch_linear_bwd_input(const lowra_layout& L, const LinearArgs& a, int path, hipStream_t st);

}  // namespace lowra
