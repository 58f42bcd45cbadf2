// SFB reconstruction with fused momentum-SGD update, bf16 factors, fp32 accumulation and
// fp32 W / Mom (Section 4.3.1 step 3, Eq. 5; Algorithm 3's update line):
//     dW[n][m] = sum_k U[k][n] * V[k][m] ;  Mom = mu*Mom + lr*dW ;  W = W - Mom
//
// The contraction index k is the OUTER dimension of both stacked factor matrices, while
// v_mfma_f32_32x32x16_bf16 wants 8 consecutive k in one lane.  The tiles are copied to LDS
// as they are (K-outer, 16-byte chunks) and read back with gfx950's transposing LDS load
// (ds_read_b64_tr_b16): a 16-lane group reads four k rows x 16 columns and each lane ends
// up with the 4 k values of its own column.
//
// Pipeline: global loads run two k-stages ahead of the MFMAs (two register stages, two
// LDS buffers, one barrier per stage), because one stage of MFMA work (~0.4 us) is shorter
// than a loaded HBM/L2 round trip.
//
// MFMA operand roles are swapped (rows = m, columns = n) so that the four consecutive
// accumulator rows a lane owns are four adjacent m of one W row; the epilogue turns each
// block through LDS so that W and Mom move in 16-byte accesses, 128 contiguous bytes per row.
#include <cstdlib>
#include "psd_internal.h"

namespace psd {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int KT = 32;         // k rows per LDS stage (two MFMA k-steps of 16)
constexpr int PAD = 16;        // bf16 elements of row padding: row stride = 32 bytes mod 128,
                               // so the 4 rows one 16-lane group reads fall in distinct banks
constexpr int GROUP_N = 8;     // tile rows per raster group (L2 reuse of the V panels)

// WN x WM wavefronts, each owning BN x BM MFMA blocks of 32 x 32; OCC = wavefronts per SIMD
template <int WN_, int WM_, int BN_, int BM_, int OCC_>
struct Cfg {
    static constexpr int WN = WN_, WM = WM_, BN = BN_, BM = BM_, OCC = OCC_;
    static constexpr int THREADS = 64 * WN * WM;
    static constexpr int TN = 32 * BN * WN, TM = 32 * BM * WM;   // workgroup tile
    static constexpr int LDA = TN + PAD, LDB = TM + PAD;         // LDS row strides (elements)
    static constexpr int A_ELEMS = KT * LDA, B_ELEMS = KT * LDB;
    static constexpr int CPR_A = TN / 8, CPR_B = TM / 8;         // 16-byte chunks per tile row
    static constexpr int CH_A = KT * CPR_A / THREADS, CH_B = KT * CPR_B / THREADS;
    static constexpr size_t LDS_BYTES = size_t(2) * (A_ELEMS + B_ELEMS) * 2;
    static_assert(KT * CPR_A % THREADS == 0 && KT * CPR_B % THREADS == 0, "tile rows must split evenly");
};

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// Buffer descriptor over a whole stacked factor matrix (K * ld bf16).  Loads through it are
// range-checked by the hardware: a 16-byte chunk at or beyond `bytes` returns zeros, which
// is what the k tail of the last stage needs, with no branch in the loop.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t factor_rsrc(const uint16_t* X, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(X), 0, static_cast<int>(bytes), 0x00020000);
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

__device__ __forceinline__ void upd(float d, float& w, float& mo, float lr, float mu)
{
    mo = __fmaf_rn(mu, mo, lr * d);
    w = w - mo;
}

template <class C>
__global__ void __launch_bounds__(C::THREADS, C::OCC)
sfb_bf16_kernel(const uint16_t* __restrict__ U, int64_t ldu, const uint16_t* __restrict__ V, int64_t ldv,
                float* __restrict__ W, float* __restrict__ Mom, int N, int M, int K, float lr, float mu,
                int tiles_n, int tiles_m, uint32_t u_bytes, uint32_t v_bytes)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
    uint16_t* As = lds;                        // [2][KT][LDA]   U tile (n columns)
    uint16_t* Bs = lds + 2 * C::A_ELEMS;       // [2][KT][LDB]   V tile (m columns)

    // Workgroup -> tile.  Consecutive workgroup ids go round-robin over the 8 XCDs; give each
    // XCD a contiguous run of the tile sequence, and order that sequence in groups of GROUP_N
    // tile rows so that the workgroups sharing an L2 re-use the same few U and V panels.
    const int T = tiles_n * tiles_m;
    const int b = blockIdx.x, xcd = b & 7;
    const int lin = xcd * (T >> 3) + (xcd < (T & 7) ? xcd : (T & 7)) + (b >> 3);
    const int per_group = GROUP_N * tiles_m;
    const int g = lin / per_group, in_g = lin - g * per_group;
    const int rows_g = tiles_n - g * GROUP_N < GROUP_N ? tiles_n - g * GROUP_N : GROUP_N;
    const int tile_n = g * GROUP_N + in_g % rows_g, tile_m = in_g / rows_g;

    const int64_t n0 = int64_t(tile_n) * C::TN, m0 = int64_t(tile_m) * C::TM;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wn0 = (wave / C::WM) * 32 * C::BN, wm0 = (wave % C::WM) * 32 * C::BM;
    const int grp = lane >> 4;                 // 16-lane group: columns +16*(grp%2), k rows +8*(grp/2)

    f32x16 acc[C::BN][C::BM];
#pragma unroll
    for (int a = 0; a < C::BN; ++a)
#pragma unroll
        for (int c = 0; c < C::BM; ++c)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][c][r] = 0.f;

    uint4 ra[2][C::CH_A], rb[2][C::CH_B];      // two register stages of prefetched chunks
    // byte offset of this lane's chunk h inside a stage that starts at row 0; a column past
    // ld wraps into the next row, which only feeds outputs n >= N (m >= M) that are never stored
    const __amdgpu_buffer_rsrc_t rsrc_u = factor_rsrc(U, u_bytes), rsrc_v = factor_rsrc(V, v_bytes);
    uint32_t off_a[C::CH_A], off_b[C::CH_B];
#pragma unroll
    for (int h = 0; h < C::CH_A; ++h) {
        const int c = tid + h * C::THREADS;
        off_a[h] = static_cast<uint32_t>(((c / C::CPR_A) * ldu + n0 + (c % C::CPR_A) * 8) * 2);
    }
#pragma unroll
    for (int h = 0; h < C::CH_B; ++h) {
        const int c = tid + h * C::THREADS;
        off_b[h] = static_cast<uint32_t>(((c / C::CPR_B) * ldv + m0 + (c % C::CPR_B) * 8) * 2);
    }
    const uint32_t stage_a = static_cast<uint32_t>(KT * ldu * 2), stage_b = static_cast<uint32_t>(KT * ldv * 2);
    auto fetch = [&](int st, uint32_t stage) {
#pragma unroll
        for (int h = 0; h < C::CH_A; ++h) {
            const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrc_u, off_a[h] + stage * stage_a, 0, 0);
            ra[st][h] = make_uint4(v.x, v.y, v.z, v.w);
        }
#pragma unroll
        for (int h = 0; h < C::CH_B; ++h) {
            const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrc_v, off_b[h] + stage * stage_b, 0, 0);
            rb[st][h] = make_uint4(v.x, v.y, v.z, v.w);
        }
    };
    auto stash = [&](int st, int buf) {
#pragma unroll
        for (int h = 0; h < C::CH_A; ++h) {
            const int c = tid + h * C::THREADS;
            *reinterpret_cast<uint4*>(As + buf * C::A_ELEMS + (c / C::CPR_A) * C::LDA + (c % C::CPR_A) * 8) = ra[st][h];
        }
#pragma unroll
        for (int h = 0; h < C::CH_B; ++h) {
            const int c = tid + h * C::THREADS;
            *reinterpret_cast<uint4*>(Bs + buf * C::B_ELEMS + (c / C::CPR_B) * C::LDB + (c % C::CPR_B) * 8) = rb[st][h];
        }
    };
    const int steps = (K + KT - 1) / KT;
    // this lane's 8 k values of a 16-row MFMA step: ks + 8*(grp/2) + 0..7 (the same for both operands)
    auto load_frags = [&](int buf, int ks, bf16x8 (&a)[C::BN], bf16x8 (&bb)[C::BM]) {
        const uint16_t* Ab = As + buf * C::A_ELEMS;
        const uint16_t* Bb = Bs + buf * C::B_ELEMS;
        const int krow = ks + 8 * (grp >> 1);
#pragma unroll
        for (int bn = 0; bn < C::BN; ++bn) {
            const uint16_t* patch = Ab + krow * C::LDA + wn0 + 32 * bn + 16 * (grp & 1);
            const bf16x4 lo = read_tr(patch, C::LDA, lane);
            const bf16x4 hi = read_tr(patch + 4 * C::LDA, C::LDA, lane);
            a[bn] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        }
#pragma unroll
        for (int bm = 0; bm < C::BM; ++bm) {
            const uint16_t* patch = Bb + krow * C::LDB + wm0 + 32 * bm + 16 * (grp & 1);
            const bf16x4 lo = read_tr(patch, C::LDB, lane);
            const bf16x4 hi = read_tr(patch + 4 * C::LDB, C::LDB, lane);
            bb[bm] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        }
    };
    // rows of the MFMA block = m (V operand), columns = n (U operand)
    auto mma = [&](const bf16x8 (&a)[C::BN], const bf16x8 (&bb)[C::BM]) {
#pragma unroll
        for (int bn = 0; bn < C::BN; ++bn)
#pragma unroll
            for (int bm = 0; bm < C::BM; ++bm)
                acc[bn][bm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bb[bm], a[bn], acc[bn][bm], 0, 0, 0);
    };
    // One k-stage: LDS buffer `buf` holds stage t, register set `st` holds stage t+1 (st = (t+1)&1).
    // Both MFMA steps' operand reads are issued up front so the second hides behind the first
    // step's MFMAs; the next stage is written to the other LDS buffer between the two steps.
    // The body is branch-free on purpose: stages past the end of K are fetched as zeros by the
    // range check and stashed into a buffer nobody reads, which keeps the two register sets'
    // loads distinguishable for the wait-count logic (the older set is waited for, the newer
    // one stays in flight).
    auto stage = [&](int buf, int st, int t) {
        bf16x8 a0[C::BN], b0[C::BM], a1[C::BN], b1[C::BM];
load_frags(buf, 0, a0, b0);
        load_frags(buf, 16, a1, b1);
        __builtin_amdgcn_sched_barrier(0);     // keep every operand read ahead of the first MFMA
        mma(a0, b0);
        stash(st, buf ^ 1);
        fetch(st, t + 3);
        mma(a1, b1);
        __syncthreads();
    };

    fetch(0, 0);
    fetch(1, 1);                               // stages beyond K read as zeros (range check)
    stash(0, 0);
    fetch(0, 2);
    __syncthreads();
    const int steps2 = (steps + 1) & ~1;       // an odd count runs one extra all-zero stage
    for (int t = 0; t < steps2; t += 2) {
        stage(0, 1, t);
        stage(1, 0, t + 1);
    }

    // Epilogue.  Accumulator register r of block (bn, bm) holds MFMA row 8*(r/4) + 4*(lane/32) + r%4
    // (= m offset) and column lane%32 (= n offset): four adjacent m per register quad.
    const int l32 = lane & 31, lhi = lane >> 5;
    if (M % 4 == 0) {
        // Fast path.  Held as they are, the quads of one W row sit in 2 lanes x 4 registers, and a
        // wavefront access would touch 32 rows x 32 bytes: measured at ~3.1 TB/s for the W/Mom
        // read-modify-write, against ~4.9 TB/s once every row gets >= 128 contiguous bytes per
        // instruction.  So each 32 x 32 block is turned through a private LDS patch: written as
        // held, read back with 8 lanes per row, then 8 rows x 128 bytes per global access.
        constexpr int PLD = 36;                            // patch row stride in floats (144 B: conflict-free)
        float* patch = reinterpret_cast<float*>(lds) + wave * (32 * PLD);
        const int prow = lane >> 3, pcol = 4 * (lane & 7);
#pragma unroll
        for (int bn = 0; bn < C::BN; ++bn) {
#pragma unroll
            for (int bm = 0; bm < C::BM; ++bm) {
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    *reinterpret_cast<float4*>(patch + l32 * PLD + 8 * q + 4 * lhi) =
                        make_float4(acc[bn][bm][4 * q], acc[bn][bm][4 * q + 1], acc[bn][bm][4 * q + 2],
                                    acc[bn][bm][4 * q + 3]);
                float4 d[4], w[4], mo[4];
                const int64_t m = m0 + wm0 + 32 * bm + pcol;
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    const int64_t n = n0 + wn0 + 32 * bn + prow + 8 * jj;
                    d[jj] = *reinterpret_cast<const float4*>(patch + (prow + 8 * jj) * PLD + pcol);
                    if (n < N && m < M) {                  // m % 4 == 0 and M % 4 == 0: whole quad inside
                        w[jj] = *reinterpret_cast<const float4*>(W + n * int64_t(M) + m);
                        mo[jj] = *reinterpret_cast<const float4*>(Mom + n * int64_t(M) + m);
                    }
                }
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    const int64_t n = n0 + wn0 + 32 * bn + prow + 8 * jj;
                    if (n < N && m < M) {
                        upd(d[jj].x, w[jj].x, mo[jj].x, lr, mu);
                        upd(d[jj].y, w[jj].y, mo[jj].y, lr, mu);
                        upd(d[jj].z, w[jj].z, mo[jj].z, lr, mu);
                        upd(d[jj].w, w[jj].w, mo[jj].w, lr, mu);
                        *reinterpret_cast<float4*>(Mom + n * int64_t(M) + m) = mo[jj];
                        *reinterpret_cast<float4*>(W + n * int64_t(M) + m) = w[jj];
                    }
                }
            }
        }
    } else {
        // rows of W are not 16-byte aligned: plain 4-byte accesses straight from the accumulators
#pragma unroll
        for (int bn = 0; bn < C::BN; ++bn) {
            const int64_t n = n0 + wn0 + 32 * bn + l32;
            if (n >= N) continue;
            float* wrow = W + n * int64_t(M);
            float* mrow = Mom + n * int64_t(M);
#pragma unroll
            for (int bm = 0; bm < C::BM; ++bm)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int64_t m = m0 + wm0 + 32 * bm + 8 * (r >> 2) + 4 * lhi + (r & 3);
                    if (m < M) {
                        float wv = wrow[m], mv = mrow[m];
                        upd(acc[bn][bm][r], wv, mv, lr, mu);
                        mrow[m] = mv;
                        wrow[m] = wv;
                    }
                }
        }
    }
}

template <class C>
psd_status launch_cfg(const uint16_t* U, int64_t ldu, const uint16_t* V, int64_t ldv, float* W, float* Mom,
                      int64_t N, int64_t M, int64_t K, float lr, float mu, hipStream_t st)
{
    const int64_t tiles_n = (N + C::TN - 1) / C::TN, tiles_m = (M + C::TM - 1) / C::TM;
    const int64_t tiles = tiles_n * tiles_m;
    if (tiles < 1 || tiles > 0x3fffffff) return PSD_E_INVALID;
    // 32-bit byte offsets into each factor matrix, with room for the two stages of read-ahead
    const int64_t u_bytes = K * ldu * 2, v_bytes = K * ldv * 2;
    const int64_t reach = (int64_t(1) << 32) - 8 * KT * (ldu > ldv ? ldu : ldv) * 2 - 4096;
    if (u_bytes > reach || v_bytes > reach) return PSD_E_UNSUPPORTED;
    auto kern = sfb_bf16_kernel<C>;
    static bool attr_done = false;    // raising the dynamic LDS limit is idempotent
    if (!attr_done) {
        PSD_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, int(C::LDS_BYTES)));
        attr_done = true;
    }
    hipLaunchKernelGGL(kern, dim3(static_cast<uint32_t>(tiles)), dim3(C::THREADS), C::LDS_BYTES, st, U, ldu, V, ldv, W,
                       Mom, static_cast<int>(N), static_cast<int>(M), static_cast<int>(K), lr, mu,
                       static_cast<int>(tiles_n), static_cast<int>(tiles_m), static_cast<uint32_t>(u_bytes),
                       static_cast<uint32_t>(v_bytes));
    PSD_HIP_TRY(hipGetLastError());
    return PSD_OK;
}

using Cfg256x256w4 = Cfg<2, 2, 4, 4, 1>;   // 4 wavefronts of 128 x 128, one workgroup per CU
using Cfg256x128w4 = Cfg<2, 2, 4, 2, 2>;   // 4 wavefronts of 128 x 64, two workgroups per CU
using Cfg128x256w4 = Cfg<2, 2, 2, 4, 2>;   // 4 wavefronts of 64 x 128, two workgroups per CU
using Cfg256x256w8 = Cfg<2, 4, 4, 2, 2>;   // 8 wavefronts of 128 x 64, one workgroup per CU
using Cfg128x128w4 = Cfg<2, 2, 2, 2, 2>;   // small layers: more workgroups

}  // namespace

psd_status launch_sfb_bf16(const uint16_t* U, int64_t ldu, const uint16_t* V, int64_t ldv, float* W, float* Mom,
                           int64_t N, int64_t M, int64_t K, float lr, float mu, hipStream_t st)
{
    // PSD_SFB_BF16_TILE overrides the tile choice (tuning aid): 0..4 in the order above
    const char* e = std::getenv("PSD_SFB_BF16_TILE");
    int pick = e ? std::atoi(e) : -1;
    if (pick < 0) {
        const int64_t big_tiles = ((N + 255) / 256) * ((M + 255) / 256);
        pick = big_tiles >= 256 ? 2 : 4;
    }
    switch (pick) {
        case 0: return launch_cfg<Cfg256x256w4>(U, ldu, V, ldv, W, Mom, N, M, K, lr, mu, st);
        case 1: return launch_cfg<Cfg256x128w4>(U, ldu, V, ldv, W, Mom, N, M, K, lr, mu, st);
        case 2: return launch_cfg<Cfg128x256w4>(U, ldu, V, ldv, W, Mom, N, M, K, lr, mu, st);
        case 3: return launch_cfg<Cfg256x256w8>(U, ldu, V, ldv, W, Mom, N, M, K, lr, mu, st);
        case 4: return launch_cfg<Cfg128x128w4>(U, ldu, V, ldv, W, Mom, N, M, K, lr, mu, st);
        default: return PSD_E_INVALID;
    }
}

}  // namespace psd
