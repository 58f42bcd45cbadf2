// Bias gradient of an FC layer under sufficient-factor broadcasting, with the momentum-SGD
// update fused: for z = W a + b the per-sample gradient w.r.t. b is the error vector itself
// (the same chain rule that gives Eq. 5 for W), so with the stacked errors U (K x N) that a
// worker holds after SFB step 2
//     db[n] = sum_k U[k][n] ;  mom_b = mu*mom_b + lr*(db + wd*b) ;  b = b - mom_b.
// The paper's volume analysis counts weights only (Table 3); the bias needs no extra
// communication because U is already there.
//
// HBM-bound column sum (K*N factor elements read once, N outputs).  A workgroup of 16
// wavefronts owns 128 adjacent columns: lane l of every wavefront reads columns 2l, 2l+1 of
// one row with a single 4-byte (bf16) or 8-byte (fp32) load, wavefront w takes rows
// k = w, w+16, ..., and the 16 partial sums meet in LDS, added in wavefront order.
#include "psd_device.h"
#include "psd_internal.h"

namespace psd {
namespace {

constexpr int kWaves = 16, kThreads = 64 * kWaves, kCols = 128;

template <bool BF16>
__global__ void __launch_bounds__(kThreads)
bias_kernel(const void* __restrict__ Uv, int64_t ldu, int N, int K, float* __restrict__ bias,
            float* __restrict__ mom, float lr, float mu, float wd)
{
    __shared__ float part[kWaves][kCols];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t c0 = int64_t(blockIdx.x) * kCols + 2 * lane;      // first of this lane's two columns
    float s0 = 0.f, s1 = 0.f;
    if (c0 < ldu) {                                                  // ldu is even: c0 + 1 < ldu as well
        if constexpr (BF16) {
            const uint16_t* U = static_cast<const uint16_t*>(Uv);
            int k = wave;
            for (; k + 7 * kWaves < K; k += 8 * kWaves) {            // 8 independent loads in flight per lane
                uint32_t v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    v[u] = *reinterpret_cast<const uint32_t*>(U + int64_t(k + u * kWaves) * ldu + c0);
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    s0 += __uint_as_float(v[u] << 16);               // bf16 -> fp32 is a shift
                    s1 += __uint_as_float(v[u] & 0xffff0000u);
                }
            }
            for (; k < K; k += kWaves) {
                const uint32_t v = *reinterpret_cast<const uint32_t*>(U + int64_t(k) * ldu + c0);
                s0 += __uint_as_float(v << 16);
                s1 += __uint_as_float(v & 0xffff0000u);
            }
        } else {
            const float* U = static_cast<const float*>(Uv);
            int k = wave;
            for (; k + 7 * kWaves < K; k += 8 * kWaves) {
                float2 v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    v[u] = *reinterpret_cast<const float2*>(U + int64_t(k + u * kWaves) * ldu + c0);
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    s0 += v[u].x;
                    s1 += v[u].y;
                }
            }
            for (; k < K; k += kWaves) {
                const float2 v = *reinterpret_cast<const float2*>(U + int64_t(k) * ldu + c0);
                s0 += v.x;
                s1 += v.y;
            }
        }
    }
    part[wave][2 * lane] = s0;
    part[wave][2 * lane + 1] = s1;
    __syncthreads();
    if (threadIdx.x < kCols) {
        const int64_t n = int64_t(blockIdx.x) * kCols + threadIdx.x;
        if (n < N) {
            float d = part[0][threadIdx.x];
#pragma unroll
            for (int w = 1; w < kWaves; ++w) d += part[w][threadIdx.x];
            float b = bias[n], m = mom[n];
            upd(d, b, m, lr, mu, wd);
            mom[n] = m;
            bias[n] = b;
        }
    }
}

}  // namespace

psd_status launch_bias(const void* U, int64_t ldu, int32_t dtype, int64_t N, int64_t K, float* bias, float* mom,
                       float lr, float mu, float wd, hipStream_t st)
{
    const int64_t blocks = (N + kCols - 1) / kCols;
    if (blocks < 1 || blocks > 0x7fffffff) return PSD_E_INVALID;
    if (dtype == PSD_BF16)
        hipLaunchKernelGGL(bias_kernel<true>, dim3(static_cast<uint32_t>(blocks)), dim3(kThreads), 0, st, U, ldu,
                           static_cast<int>(N), static_cast<int>(K), bias, mom, lr, mu, wd);
    else
        hipLaunchKernelGGL(bias_kernel<false>, dim3(static_cast<uint32_t>(blocks)), dim3(kThreads), 0, st, U, ldu,
                           static_cast<int>(N), static_cast<int>(K), bias, mom, lr, mu, wd);
    PSD_HIP_TRY(hipGetLastError());
    return PSD_OK;
}

}  // namespace psd
