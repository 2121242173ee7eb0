// Internal host-side declarations: the layout object and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "lowra_dev.h"

struct lowra_layout {
    int N = 0, K = 0, G = 0, C = 0;
    int device = -1;
    size_t packed_bytes = 0;
    int n_by_bits[5] = {0, 0, 0, 0, 0};     // channel count per width
    std::vector<uint8_t> bits;              // host copies
    std::vector<int32_t> cb;
    std::vector<int64_t> row_offset;
    lowra::RowInfo* d_rows = nullptr;       // [N] device
    lowra::SortedRow* d_sorted_rows = nullptr;  // [ceil(N/256)*256] device: rows in per-tile width-sorted order
    lowra::SortedRow* d_gemm_rows = nullptr;    // [ceil(N/256)*256] device: rows in the forward GEMM's per-tile order (pad = local row of a padding entry)
    uint16_t* d_tile_order = nullptr;       // [ceil(N/256)*256] device: per 256-row tile, the forward GEMM's row order (natural, 4-bit rows last)
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

struct lowra_fwd_batch {
    int device = -1;
    std::vector<lowra::GemvBatchGroup> groups;
    lowra::GemvParams* d_tdescs = nullptr;   // matrices with a LoRA term, for the partial-sum kernel
    int* d_blk0 = nullptr;                   // [nt + 1] first 256-column block of each
    int* d_towner = nullptr;                 // [nblk_total] the matrix of each block
    int nt = 0, nblk_total = 0;
};

namespace lowra {

// Each launcher validates nothing (the C ABI did) and returns the launch status.
hipError_t launch_quantize(const lowra_layout& L, const float* W, const float* thresholds,
                           uint8_t* packed, float* absmax, hipStream_t st);
hipError_t launch_dequantize(const lowra_layout& L, const uint8_t* packed, const float* absmax,
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

size_t loftq_workspace_bytes(const lowra_layout& L, int r);
hipError_t launch_loftq(const lowra_layout& L, const float* W, const float* thresholds, const float* mappings, int r, int steps,
                        int iters, const uint16_t* omega, uint8_t* packed, float* absmax, uint16_t* A_out, uint16_t* B_out,
                        void* workspace, hipStream_t st);

bool gemv_fwd_supported(const lowra_layout& L, int M);
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
hipError_t launch_linear_fwd(const lowra_layout& L, const LinearArgs& a, int path, hipStream_t st);
hipError_t launch_linear_bwd_input(const lowra_layout& L, const LinearArgs& a, int path, hipStream_t st);

}  // namespace lowra
