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

struct PackArgs {
    const float* src[PSD_MAX_WORKERS];
    void* dst;
    int64_t cols, ld, B;
    int32_t P;
};
psd_status launch_pack(const PackArgs& a, int32_t out_dtype, hipStream_t st);

psd_status launch_sfb_f32(const float* U, int64_t ldu, const float* V, int64_t ldv, float* W, float* Mom,
                          int64_t N, int64_t M, int64_t K, float lr, float mu, float wd, hipStream_t st);
psd_status launch_sfb_bf16(const uint16_t* U, int64_t ldu, const uint16_t* V, int64_t ldv, float* W, float* Mom,
                           int64_t N, int64_t M, int64_t K, float lr, float mu, float wd, hipStream_t st);

psd_status launch_bias(const void* U, int64_t ldu, int32_t dtype, int64_t N, int64_t K, float* bias, float* mom,
                       float lr, float mu, float wd, hipStream_t st);

}  // namespace psd
