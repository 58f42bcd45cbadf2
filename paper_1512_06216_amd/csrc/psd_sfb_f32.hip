// SFB reconstruction with fused momentum-SGD update, fp32 factors (Section 4.3.1 step 3,
// Eq. 5; Algorithm 3's update line):
//     dW[n][m] = sum_k U[k][n] * V[k][m] ;  Mom = mu*Mom + lr*dW ;  W = W - Mom
//
// A dense contraction over K = P*B, so it runs on the fp32 MFMA pipe
// (v_mfma_f32_32x32x2_f32: one k per lane, which is exactly how the K-outer stacked
// factors sit in memory -- no transpose is needed for fp32).
//
// Tiling: a 256-lane workgroup (4 wavefronts, 2 x 2) owns a 128 x 128 tile of W; each
// wavefront a 64 x 64 sub-tile as 2 x 2 MFMA blocks of 32 x 32.  MFMA row i of block t
// stands for n = n0 + 2*i + t (columns likewise), so one lane's LDS operand read is one
// 8-byte load and one lane owns 2 adjacent m in the epilogue (8-byte W/Mom accesses,
// 256 contiguous bytes per half wavefront).  dW lives only in accumulator registers.
#include "psd_internal.h"

namespace psd {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int TN = 128, TM = 128;   // workgroup tile (n, m)
constexpr int KT = 16;              // k rows per LDS stage
constexpr int THREADS = 256;

// Loads one 16-byte chunk of a K-outer operand row, or zeros outside the matrix.
__device__ __forceinline__ float4 ld_chunk(const float* __restrict__ X, int64_t ld, int64_t k, int64_t K, int64_t col)
{
    if (k < K && col < ld) return *reinterpret_cast<const float4*>(X + k * ld + col);   // ld % 4 == 0
    return make_float4(0.f, 0.f, 0.f, 0.f);
}

__global__ void __launch_bounds__(THREADS)
sfb_f32_kernel(const float* __restrict__ U, int64_t ldu, const float* __restrict__ V, int64_t ldv,
               float* __restrict__ W, float* __restrict__ Mom, int N, int M, int K, float lr, float mu,
               int tiles_m)
{
    __shared__ __attribute__((aligned(16))) float As[2][KT][TN];
    __shared__ __attribute__((aligned(16))) float Bs[2][KT][TM];

    const int tile_n = blockIdx.x / tiles_m, tile_m = blockIdx.x % tiles_m;
    const int64_t n0 = int64_t(tile_n) * TN, m0 = int64_t(tile_m) * TM;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wn0 = (wave >> 1) * 64, wm0 = (wave & 1) * 64;     // wavefront sub-tile origin
    const int l32 = lane & 31, lhi = lane >> 5;

    // global -> LDS assignment: a stage is KT rows x 32 chunks per operand = 512 chunks, 2 per lane
    const int ld_row = tid >> 5;          // 0..7 (and +8)
    const int ld_col = (tid & 31) * 4;    // float offset inside the tile row

    f32x16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    float4 ra[2], rb[2];
    auto fetch = [&](int64_t k0) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            ra[h] = ld_chunk(U, ldu, k0 + ld_row + 8 * h, K, n0 + ld_col);
            rb[h] = ld_chunk(V, ldv, k0 + ld_row + 8 * h, K, m0 + ld_col);
        }
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            *reinterpret_cast<float4*>(&As[buf][ld_row + 8 * h][ld_col]) = ra[h];
            *reinterpret_cast<float4*>(&Bs[buf][ld_row + 8 * h][ld_col]) = rb[h];
        }
    };

    const int steps = (K + KT - 1) / KT;
    fetch(0);
    stash(0);
    __syncthreads();
    for (int s = 0; s < steps; ++s) {
        const int buf = s & 1;
        if (s + 1 < steps) fetch(int64_t(s + 1) * KT);
#pragma unroll
        for (int kk = 0; kk < KT; kk += 2) {
            // lanes 0..31 feed k = kk, lanes 32..63 feed k = kk + 1
            const float2 a = *reinterpret_cast<const float2*>(&As[buf][kk + lhi][wn0 + 2 * l32]);
            const float2 b = *reinterpret_cast<const float2*>(&Bs[buf][kk + lhi][wm0 + 2 * l32]);
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, b.x, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, b.y, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b.x, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b.y, acc[1][1], 0, 0, 0);
        }
        if (s + 1 < steps) {
            stash(buf ^ 1);          // the other buffer was last read before the previous barrier
            __syncthreads();
        }
    }

    // Epilogue.  Accumulator register r of a 32x32 block holds MFMA row 8*(r/4) + 4*(lane/32) + r%4,
    // column lane%32.  Block (ta, tb): n = n0 + wn0 + 2*row + ta, m = m0 + wm0 + 2*col + tb.
    const int64_t mcol = m0 + wm0 + 2 * l32;
    const bool pair_ok = (M % 2 == 0);   // 8-byte accesses need an even row length
#pragma unroll
    for (int ta = 0; ta < 2; ++ta) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = 8 * (r >> 2) + 4 * lhi + (r & 3);
            const int64_t n = n0 + wn0 + 2 * row + ta;
            if (n >= N) continue;
            const float d0 = acc[ta][0][r], d1 = acc[ta][1][r];
            float* wp = W + n * int64_t(M) + mcol;
            float* mp = Mom + n * int64_t(M) + mcol;
            if (pair_ok && mcol + 1 < M) {
                float2 w = *reinterpret_cast<float2*>(wp), mo = *reinterpret_cast<float2*>(mp);
                mo.x = __fmaf_rn(mu, mo.x, lr * d0);
                mo.y = __fmaf_rn(mu, mo.y, lr * d1);
                w.x -= mo.x;
                w.y -= mo.y;
                *reinterpret_cast<float2*>(mp) = mo;
                *reinterpret_cast<float2*>(wp) = w;
            } else {
                if (mcol < M) {
                    const float mo = __fmaf_rn(mu, mp[0], lr * d0);
                    mp[0] = mo;
                    wp[0] -= mo;
                }
                if (mcol + 1 < M) {
                    const float mo = __fmaf_rn(mu, mp[1], lr * d1);
                    mp[1] = mo;
                    wp[1] -= mo;
                }
            }
        }
    }
}

}  // namespace

psd_status launch_sfb_f32(const float* U, int64_t ldu, const float* V, int64_t ldv, float* W, float* Mom,
                          int64_t N, int64_t M, int64_t K, float lr, float mu, hipStream_t st)
{
    const int64_t tiles_n = (N + TN - 1) / TN, tiles_m = (M + TM - 1) / TM;
    const int64_t tiles = tiles_n * tiles_m;
    if (tiles < 1 || tiles > 0x7fffffff) return PSD_E_INVALID;
    hipLaunchKernelGGL(sfb_f32_kernel, dim3(static_cast<uint32_t>(tiles)), dim3(THREADS), 0, st, U, ldu, V, ldv, W, Mom,
                       static_cast<int>(N), static_cast<int>(M), static_cast<int>(K), lr, mu,
                       static_cast<int>(tiles_m));
    PSD_HIP_TRY(hipGetLastError());
    return PSD_OK;
}

}  // namespace psd
