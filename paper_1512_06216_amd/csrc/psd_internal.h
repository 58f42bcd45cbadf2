// Internal declarations shared by the translation units of libpsd (not installed).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "psd.h"

namespace psd {

// Records a failing HIP call for psd_last_hip_error() and maps it to PSD_E_HIP.
psd_status hip_failed(hipError_t e);

#define PSD_HIP_TRY(expr)                                        \
    do {                                                         \
        hipError_t e__ = (expr);                                 \
        if (e__ != hipSuccess) return ::psd::hip_failed(e__);    \
    } while (0)

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Value of a psd_tune_set() knob; -1 = let the library choose.
int tune_value(int knob);
// Compute units of the current device (queried once per device, then cached).
int device_cu_count();

// ---- launchers (one per kernel family); arguments are already validated ----------------
struct DenseSeg {
    const float* G[PSD_MAX_MULTI_WORKERS];
    float* W;
    float* Mom;
    int64_t n;
    int64_t q, r;          // n = q * S + r, 0 <= r < S
    int32_t P;
    int32_t S;
    int32_t block_begin;   // first workgroup of this segment
    int32_t chunks;        // workgroups per shard
};
struct DenseTable {
    DenseSeg seg[PSD_MAX_MULTI_SEGMENTS];
    int32_t L;
};
struct DenseWide {          // single layer, up to PSD_MAX_WORKERS copies
    const float* G[PSD_MAX_WORKERS];
    float* W;
    float* Mom;
    int64_t n;
    int64_t q, r;          // n = q * S + r, 0 <= r < S
    int32_t P;
    int32_t S;
    int32_t chunks;
};
psd_status launch_dense_table(const DenseTable& t, int32_t total_blocks, float lr, float mu, float wd, hipStream_t st);
psd_status launch_dense_wide(const DenseWide& a, float lr, float mu, float wd, hipStream_t st);
int32_t dense_chunks_for(int64_t n, int32_t S);   // workgroups per shard

struct PackSide {            // one of the two stacked matrices of a layer
    const float* src[PSD_MAX_WORKERS];
    void* dst;
    int64_t cols, ld;
};
struct PackArgs {
    PackSide u, v;           // errors (B x N blocks -> K x ldu), activations (B x M blocks -> K x ldv)
    int64_t B;
    int32_t P;
    int32_t bx_u;            // workgroup columns serving u (filled in by launch_pack)
};
psd_status launch_pack(PackArgs& a, int32_t out_dtype, hipStream_t st);

// ---- reconstruction.  part / splits: with splits > 1 the contraction is split over `splits`
// workgroups per tile, each storing a partial dW (N x M, sfb_part_stride apart) to `part`, and the
// partials are summed in split order and the update applied by launch_sfb_reduce.
psd_status launch_sfb_f32(const float* U, int64_t ldu, const float* V, int64_t ldv, float* W, float* Mom,
                          int64_t N, int64_t M, int64_t K, float lr, float mu, float wd, float* part, int splits,
                          hipStream_t st);
psd_status launch_sfb_bf16(const uint16_t* U, int64_t ldu, const uint16_t* V, int64_t ldv, float* W, float* Mom,
                           int64_t N, int64_t M, int64_t K, float lr, float mu, float wd, float* part, int splits,
                           hipStream_t st);
// reconstruction straight from the P per-worker blocks (B x ld each, no stacked copy); served when a block
// holds whole k-stages of the kernel (16 rows fp32, 32 rows bf16)
bool sfb_f32_blocks_supported(int64_t B);
bool sfb_bf16_blocks_supported(int64_t B);
psd_status launch_sfb_f32_blocks(const float* const* U_p, int64_t ldu, const float* const* V_p, int64_t ldv, int64_t P,
                                 int64_t B, float* W, float* Mom, int64_t N, int64_t M, float lr, float mu, float wd,
                                 hipStream_t st);
psd_status launch_sfb_bf16_blocks(const uint16_t* const* U_p, int64_t ldu, const uint16_t* const* V_p, int64_t ldv,
                                  int64_t P, int64_t B, float* W, float* Mom, int64_t N, int64_t M, float lr, float mu,
                                  float wd, hipStream_t st);
// how many ways each kernel would split K for this layer when it is given a workspace (1 = not at all)
int sfb_f32_splits(int64_t N, int64_t M, int64_t K);
int sfb_bf16_splits(int64_t N, int64_t M, int64_t K);
psd_status launch_sfb_reduce(const float* part, int splits, int64_t N, int64_t M, float* W, float* Mom, float lr,
                             float mu, float wd, hipStream_t st);

constexpr int kMaxSplits = 4;
// Split only for layers that leave most of the chip idle: while the split workgroups still number at
// most one per CU (half the slots) and every split keeps at least kMinSplitRows k rows.  A split
// costs 8 extra bytes of HBM traffic per weight and split (partial written, then read) plus a second
// launch.  Measured: 64 tiles (1024 -> 1000, K = 8192) 64 -> 32 us, 16 tiles (512 -> 512, K = 16384)
// 115 -> 37 us; but 256 tiles (4096 -> 1000, one workgroup per CU already) lose at every K tried
// (K = 2048: 39 -> 49 us, K = 8192: 103 -> 107 us), so such layers are not split.
constexpr int64_t kMinSplitRows = 512;
inline int sfb_splits_for(int64_t tiles, int64_t slots, int64_t K)
{
    int s = 1;
    while (s < kMaxSplits && tiles * (s + 1) <= slots / 2 && K / (s + 1) >= kMinSplitRows) ++s;
    return s;
}
// elements between two partials: N*M rounded up so that every partial starts 16-byte aligned
inline int64_t sfb_part_stride(int64_t N, int64_t M) { return (N * M + 3) / 4 * 4; }

psd_status launch_bias(const void* U, int64_t ldu, int32_t dtype, int64_t N, int64_t K, float* bias, float* mom,
                       float lr, float mu, float wd, hipStream_t st);

}  // namespace psd
