// SFB reconstruction with fused momentum-SGD update, bf16 factors, fp32 accumulation and
// fp32 W / Mom (Section 4.3.1 step 3, Eq. 5; Algorithm 3's update line):
//     dW[n][m] = sum_k U[k][n] * V[k][m] ;  Mom = mu*Mom + lr*dW ;  W = W - Mom
//
// The contraction index k is the OUTER dimension of both stacked factor matrices, while
// v_mfma_f32_32x32x16_bf16 wants 8 consecutive k in one lane.  The tiles are copied to LDS
// as they are (K-outer, 16-byte chunks) and read back with gfx950's transposing LDS load
// (ds_read_b64_tr_b16): a 16-lane group reads four k rows x 16 columns and each lane ends
// up with the 4 k values of its own column.
#include "psd_internal.h"

namespace psd {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int THREADS = 256;   // 4 wavefronts as 2 (n) x 2 (m)
constexpr int KT = 32;         // k rows per LDS stage (two MFMA k-steps of 16)
constexpr int PAD = 16;        // bf16 elements of row padding: row stride = 32 bytes mod 128,
                               // so the 4 rows one 16-lane group reads fall in distinct banks

template <int BN, int BM>
struct Tile {
    static constexpr int TN = 64 * BN, TM = 64 * BM;          // workgroup tile
    static constexpr int LDA = TN + PAD, LDB = TM + PAD;      // LDS row strides (elements)
    static constexpr int A_ELEMS = KT * LDA, B_ELEMS = KT * LDB;
    static constexpr int CH_A = KT * TN / 8 / THREADS;        // 16-byte chunks per lane per stage
    static constexpr int CH_B = KT * TM / 8 / THREADS;
    static constexpr size_t LDS_BYTES = size_t(2) * (A_ELEMS + B_ELEMS) * 2;
};

__device__ __forceinline__ uint4 ld_chunk(const uint16_t* __restrict__ X, int64_t ld, int64_t k, int64_t K, int64_t col)
{
    if (k < K && col < ld) return *reinterpret_cast<const uint4*>(X + k * ld + col);   // ld % 8 == 0
    return make_uint4(0u, 0u, 0u, 0u);
}

// Transposing read of a (4 k) x (16 columns) patch whose top-left element is `patch`.
// Lane L of a 16-lane group supplies the address of 4 adjacent columns in row (L%16)/4,
// starting at column 4*(L%4); afterwards lane i of the group holds rows 0..3 of column i.
__device__ __forceinline__ bf16x4 read_tr(const uint16_t* patch, int ld_elems, int lane)
{
    const int l16 = lane & 15;
    const uint16_t* p = patch + (l16 >> 2) * ld_elems + 4 * (l16 & 3);
    return __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
        (__attribute__((address_space(3))) bf16x4*)(p));
}

template <int BN, int BM>
__global__ void __launch_bounds__(THREADS)
sfb_bf16_kernel(const uint16_t* __restrict__ U, int64_t ldu, const uint16_t* __restrict__ V, int64_t ldv,
                float* __restrict__ W, float* __restrict__ Mom, int N, int M, int K, float lr, float mu,
                int tiles_m)
{
    using T = Tile<BN, BM>;
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
    uint16_t* As = lds;                        // [2][KT][LDA]
    uint16_t* Bs = lds + 2 * T::A_ELEMS;       // [2][KT][LDB]

    const int tile_n = blockIdx.x / tiles_m, tile_m = blockIdx.x % tiles_m;
    const int64_t n0 = int64_t(tile_n) * T::TN, m0 = int64_t(tile_m) * T::TM;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wn0 = (wave >> 1) * 32 * BN, wm0 = (wave & 1) * 32 * BM;
    const int grp = lane >> 4;                 // 16-lane group: columns +16*(grp%2), k rows +8*(grp/2)

    f32x16 acc[BN][BM];
#pragma unroll
    for (int a = 0; a < BN; ++a)
#pragma unroll
        for (int b = 0; b < BM; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    uint4 ra[T::CH_A], rb[T::CH_B];
    constexpr int CPR_A = T::TN / 8, CPR_B = T::TM / 8;       // chunks per tile row
    auto fetch = [&](int64_t k0) {
#pragma unroll
        for (int h = 0; h < T::CH_A; ++h) {
            const int c = tid + h * THREADS;
            ra[h] = ld_chunk(U, ldu, k0 + c / CPR_A, K, n0 + (c % CPR_A) * 8);
        }
#pragma unroll
        for (int h = 0; h < T::CH_B; ++h) {
            const int c = tid + h * THREADS;
            rb[h] = ld_chunk(V, ldv, k0 + c / CPR_B, K, m0 + (c % CPR_B) * 8);
        }
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int h = 0; h < T::CH_A; ++h) {
            const int c = tid + h * THREADS;
            *reinterpret_cast<uint4*>(As + buf * T::A_ELEMS + (c / CPR_A) * T::LDA + (c % CPR_A) * 8) = ra[h];
        }
#pragma unroll
        for (int h = 0; h < T::CH_B; ++h) {
            const int c = tid + h * THREADS;
            *reinterpret_cast<uint4*>(Bs + buf * T::B_ELEMS + (c / CPR_B) * T::LDB + (c % CPR_B) * 8) = rb[h];
        }
    };

    const int steps = (K + KT - 1) / KT;
    fetch(0);
    stash(0);
    __syncthreads();
    for (int s = 0; s < steps; ++s) {
        const int buf = s & 1;
        if (s + 1 < steps) fetch(int64_t(s + 1) * KT);
        const uint16_t* Ab = As + buf * T::A_ELEMS;
        const uint16_t* Bb = Bs + buf * T::B_ELEMS;
#pragma unroll
        for (int ks = 0; ks < KT; ks += 16) {
            // this lane's 8 k values: ks + 8*(grp/2) + 0..7 (the same for both operands)
            const int krow = ks + 8 * (grp >> 1);
            bf16x8 a[BN], b[BM];
#pragma unroll
            for (int bn = 0; bn < BN; ++bn) {
                const uint16_t* patch = Ab + krow * T::LDA + wn0 + 32 * bn + 16 * (grp & 1);
                const bf16x4 lo = read_tr(patch, T::LDA, lane);
                const bf16x4 hi = read_tr(patch + 4 * T::LDA, T::LDA, lane);
                a[bn] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            }
#pragma unroll
            for (int bm = 0; bm < BM; ++bm) {
                const uint16_t* patch = Bb + krow * T::LDB + wm0 + 32 * bm + 16 * (grp & 1);
                const bf16x4 lo = read_tr(patch, T::LDB, lane);
                const bf16x4 hi = read_tr(patch + 4 * T::LDB, T::LDB, lane);
                b[bm] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            }
#pragma unroll
            for (int bn = 0; bn < BN; ++bn)
#pragma unroll
                for (int bm = 0; bm < BM; ++bm)
                    acc[bn][bm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[bn], b[bm], acc[bn][bm], 0, 0, 0);
        }
        if (s + 1 < steps) {
            stash(buf ^ 1);
            __syncthreads();
        }
    }

    // Epilogue: register r of a block holds row 8*(r/4) + 4*(lane/32) + r%4, column lane%32.
    const int l32 = lane & 31, lhi = lane >> 5;
#pragma unroll
    for (int bn = 0; bn < BN; ++bn) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t n = n0 + wn0 + 32 * bn + 8 * (r >> 2) + 4 * lhi + (r & 3);
            if (n >= N) continue;
#pragma unroll
            for (int bm = 0; bm < BM; ++bm) {
                const int64_t m = m0 + wm0 + 32 * bm + l32;
                if (m >= M) continue;
                const int64_t off = n * int64_t(M) + m;
                const float mo = __fmaf_rn(mu, Mom[off], lr * acc[bn][bm][r]);
                Mom[off] = mo;
                W[off] = W[off] - mo;
            }
        }
    }
}

template <int BN, int BM>
psd_status launch_tile(const uint16_t* U, int64_t ldu, const uint16_t* V, int64_t ldv, float* W, float* Mom,
                       int64_t N, int64_t M, int64_t K, float lr, float mu, hipStream_t st)
{
    using T = Tile<BN, BM>;
    const int64_t tiles_n = (N + T::TN - 1) / T::TN, tiles_m = (M + T::TM - 1) / T::TM;
    const int64_t tiles = tiles_n * tiles_m;
    if (tiles < 1 || tiles > 0x7fffffff) return PSD_E_INVALID;
    auto kern = sfb_bf16_kernel<BN, BM>;
    static bool attr_done = false;    // raising the dynamic LDS limit is idempotent
    if (!attr_done) {
        PSD_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, int(T::LDS_BYTES)));
        attr_done = true;
    }
    hipLaunchKernelGGL(kern, dim3(static_cast<uint32_t>(tiles)), dim3(THREADS), T::LDS_BYTES, st, U, ldu, V, ldv, W,
                       Mom, static_cast<int>(N), static_cast<int>(M), static_cast<int>(K), lr, mu,
                       static_cast<int>(tiles_m));
    PSD_HIP_TRY(hipGetLastError());
    return PSD_OK;
}

}  // namespace

psd_status launch_sfb_bf16(const uint16_t* U, int64_t ldu, const uint16_t* V, int64_t ldv, float* W, float* Mom,
                           int64_t N, int64_t M, int64_t K, float lr, float mu, hipStream_t st)
{
    // small layers: 128 x 128 tiles so more workgroups exist; large layers: 256 x 256 tiles
    // (each wavefront 128 x 128) to cut LDS operand traffic per MFMA
    const int64_t big_tiles = ((N + 255) / 256) * ((M + 255) / 256);
    if (big_tiles >= 256) return launch_tile<4, 4>(U, ldu, V, ldv, W, Mom, N, M, K, lr, mu, st);
    return launch_tile<2, 2>(U, ldu, V, ldv, W, Mom, N, M, K, lr, mu, st);
}

}  // namespace psd
