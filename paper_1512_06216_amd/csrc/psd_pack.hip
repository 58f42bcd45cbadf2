// Factor stacking (SFB steps 1-2 of Section 4.3.1, receiver side): P per-worker blocks of
// B samples become one K x ld matrix, row k = p*B + b, optionally rounded to bf16.
//
// Memcpy-class, HBM-bound.  One lane produces one 16-byte output chunk (4 fp32 or 8 bf16),
// so every store is a full aligned 16 bytes and a wavefront writes 1 KiB contiguous.
// Source rows start at b*cols floats, which is only 4-byte aligned when cols is odd
// (e.g. 21841 classes); loads therefore use a 4-byte-aligned vector type and leave the
// choice of instruction to the compiler.  U (errors) and V (activations) of a layer are
// stacked by ONE launch: the first bx_u workgroup columns serve U, the rest V.
#include "psd_internal.h"

namespace psd {
namespace {

constexpr int kPackThreads = 256;
constexpr int64_t kPackMaxRows = 65535;            // grid.y limit; longer stacks loop over rows

struct __attribute__((packed, aligned(4))) f32x4_a4 { float x, y, z, w; };

// fp32 -> bf16 bits, round to nearest even; NaN keeps sign and top payload bits, made quiet.
__device__ __forceinline__ uint32_t bf16_rne(float f)
{
    const uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

template <bool BF16>
__global__ void __launch_bounds__(kPackThreads) pack_kernel(const PackArgs a)
{
    constexpr int E = BF16 ? 8 : 4;                     // elements per 16-byte output chunk
    const bool is_v = static_cast<int>(blockIdx.x) >= a.bx_u;
    const PackSide& s = is_v ? a.v : a.u;
    const int64_t chunk = int64_t(is_v ? blockIdx.x - a.bx_u : blockIdx.x) * kPackThreads + threadIdx.x;
    const int64_t j0 = chunk * E;
    if (j0 >= s.ld) return;
    const int64_t K = a.B * a.P;
    for (int64_t k = blockIdx.y; k < K; k += gridDim.y) {           // stacked row
        const int p = static_cast<int>(k / a.B);
        const int64_t b = k - int64_t(p) * a.B;
        const float* __restrict__ src = s.src[p] + b * s.cols + j0;
        float v[E];
        if (j0 + E <= s.cols) {
#pragma unroll
            for (int q = 0; q < E / 4; ++q) {
                const f32x4_a4 t = *reinterpret_cast<const f32x4_a4*>(src + 4 * q);
                v[4 * q + 0] = t.x; v[4 * q + 1] = t.y; v[4 * q + 2] = t.z; v[4 * q + 3] = t.w;
            }
        } else {
#pragma unroll
            for (int e = 0; e < E; ++e) v[e] = (j0 + e < s.cols) ? src[e] : 0.0f;   // zero the padding columns
        }
        if constexpr (BF16) {
            uint4 o;
            o.x = bf16_rne(v[0]) | (bf16_rne(v[1]) << 16);
            o.y = bf16_rne(v[2]) | (bf16_rne(v[3]) << 16);
            o.z = bf16_rne(v[4]) | (bf16_rne(v[5]) << 16);
            o.w = bf16_rne(v[6]) | (bf16_rne(v[7]) << 16);
            *reinterpret_cast<uint4*>(static_cast<uint16_t*>(s.dst) + k * s.ld + j0) = o;
        } else {
            *reinterpret_cast<float4*>(static_cast<float*>(s.dst) + k * s.ld + j0) = make_float4(v[0], v[1], v[2], v[3]);
        }
    }
}

}  // namespace

psd_status launch_pack(PackArgs& a, int32_t out_dtype, hipStream_t st)
{
    const int E = out_dtype == PSD_BF16 ? 8 : 4;
    const int64_t K = a.B * a.P;
    // ld is a multiple of E (validated)
    const int64_t bx_u = (a.u.ld / E + kPackThreads - 1) / kPackThreads, bx_v = (a.v.ld / E + kPackThreads - 1) / kPackThreads;
    if (bx_u < 1 || bx_v < 1 || bx_u + bx_v > 0x7fffffff || K < 1) return PSD_E_INVALID;
    a.bx_u = static_cast<int32_t>(bx_u);
    dim3 grid(static_cast<uint32_t>(bx_u + bx_v), static_cast<uint32_t>(K < kPackMaxRows ? K : kPackMaxRows));
    if (out_dtype == PSD_BF16)
        hipLaunchKernelGGL(pack_kernel<true>, grid, dim3(kPackThreads), 0, st, a);
    else
        hipLaunchKernelGGL(pack_kernel<false>, grid, dim3(kPackThreads), 0, st, a);
    PSD_HIP_TRY(hipGetLastError());
    return PSD_OK;
}

}  // namespace psd
