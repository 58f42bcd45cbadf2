// SFB reconstruction with fused momentum-SGD update, fp32 factors (Section 4.3.1 step 3,
// Eq. 5; Algorithm 3's update line):
//     dW[n][m] = sum_k U[k][n] * V[k][m] ;  Mom = mu*Mom + lr*dW ;  W = W - Mom
//
// A dense contraction over K = P*B, so it runs on the fp32 MFMA pipe
// (v_mfma_f32_32x32x2_f32: one k per lane, which is exactly how the K-outer stacked
// factors sit in memory -- no transpose is needed for fp32).
//
// Tiling: a 256-lane workgroup (4 wavefronts, 2 x 2) owns a 128 x 128 (or 64 x 128) tile of W;
// each wavefront a 64 x 64 (32 x 64) sub-tile of 32 x 32 MFMA blocks.  MFMA row i of block t
// stands for n = n0 + 2*i + t (columns likewise), so one lane's LDS operand read is one
// 8-byte load and one lane owns 2 adjacent m in the epilogue (8-byte W/Mom accesses,
// 256 contiguous bytes per half wavefront).  dW lives only in accumulator registers.
//
// Feeding: the same scheme as the bf16 kernel.  Tiles go global -> LDS without registers
// (buffer_load_dwordx4 ... lds) into a ring of NSTAGE buffers with NSTAGE-1 stages in flight;
// the buffer range check zero-fills the K tail.  A stage is 16 k rows = two half-stages of
// 4 MFMA k-pairs; the operand reads of one half are issued before the MFMAs of the half before
// and interleaved with them, and the workgroup barrier sits between the two halves.
#include "psd_device.h"
#include "psd_internal.h"

namespace psd {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int TM = 128;             // workgroup tile width (m)
constexpr int KT = 16;              // k rows per LDS stage
constexpr int THREADS = 256;
constexpr int NSTAGE = 4;           // ring depth

// BN = MFMA blocks per wavefront along n: workgroup tile (64*BN) x 128, wavefront tile (32*BN) x 64.
// BN = 2 is the default; BN = 1 doubles the number of workgroups for layers with few tiles.
// PART = true (layers with too few tiles to fill the chip): `splits` workgroups per tile, workgroup
// (tile, s) contracts over k-stages [s * stages_per_split, (s+1) * stages_per_split) and stores its
// partial dW tile to part + s * part_stride (N x M row-major); the partials are summed in split order
// and the update applied by the parameter-server sum kernel afterwards.
// BLK = true: the factors are not stacked.  Row k = p*B + b of U is row b of the p-th worker's B x N block
// (V likewise, B x M), read where it lies: a stage of KT rows never straddles two blocks because KT divides
// B, so the only difference is that the buffer descriptor is re-aimed whenever the stages move on to the
// next block (and aimed at nothing past the last one, which reads as zeros like the K tail does).
struct BlockPtrs { const float* u[PSD_MAX_WORKERS]; const float* v[PSD_MAX_WORKERS]; };

template <int BN, bool PART, bool BLK>
__device__ __forceinline__ void
sfb_f32_body(const float* __restrict__ U, int64_t ldu, const float* __restrict__ V, int64_t ldv,
             float* __restrict__ W, float* __restrict__ Mom, int N, int M, int K, float lr, float mu, float wd,
             int tiles_m, int tiles, uint32_t u_bytes, uint32_t v_bytes, float* __restrict__ part,
             int64_t part_stride, int stages_per_split, const BlockPtrs* blocks, int n_blocks, int stages_per_block)
{
    static_assert(!(PART && BLK), "blocks read in place are not combined with a split of K");
    constexpr int TN = 64 * BN;
    constexpr int RA = TN * 4, RB = TM * 4;                       // LDS row bytes
    constexpr int A_BYTES = KT * RA, B_BYTES = KT * RB, STAGE_BYTES = A_BYTES + B_BYTES;
    constexpr int NI_A = A_BYTES / 1024 / 4, NI_B = B_BYTES / 1024 / 4;   // 1 KiB DMA runs per wavefront
    constexpr int LPS = NI_A + NI_B;
    __shared__ __attribute__((aligned(1024))) char lds[NSTAGE * STAGE_BYTES];
    const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(
        (__attribute__((address_space(3))) void*)lds));

    const int split = PART ? __builtin_amdgcn_readfirstlane(blockIdx.x / tiles) : 0;   // (the division runs on the vector ALU)
    const int tile = PART ? blockIdx.x - split * tiles : blockIdx.x;
    const int tile_n = tile / tiles_m, tile_m = tile % tiles_m;
    // this workgroup's k range: rows at or past k_end read as zeros (descriptor size), rows before
    // k_begin are skipped (offsets)
    const int k_begin = PART ? split * stages_per_split * KT : 0;
    const int k_end = PART ? (k_begin + stages_per_split * KT < K ? k_begin + stages_per_split * KT : K) : K;
    if constexpr (PART) {
        u_bytes = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(int64_t(k_end) * ldu * 4));
        v_bytes = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(int64_t(k_end) * ldv * 4));
    }
    const int64_t n0 = int64_t(tile_n) * TN, m0 = int64_t(tile_m) * TM;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wn0 = (wave >> 1) * 32 * BN, wm0 = (wave & 1) * 64;     // wavefront sub-tile origin
    const int l32 = lane & 31, lhi = lane >> 5;

    // DMA plan: run j of this wavefront covers chunks f = (wave*NI + j)*64 + lane of the stage
    i32x4 rsrc_u = raw_rsrc(U, u_bytes), rsrc_v = raw_rsrc(V, v_bytes);
    int blk = 0, stage_in_blk = 0;               // BLK: where the next stage to be requested lies
    auto aim_block = [&]() {                     // BLK: descriptors over block `blk` (u_bytes, v_bytes = one block)
        const bool live = blk < n_blocks;
        const int i = live ? blk : 0;            // the table is never indexed past its end
        rsrc_u = raw_rsrc(uniform_ptr(blocks->u[i]), live ? u_bytes : 0u);
        rsrc_v = raw_rsrc(uniform_ptr(blocks->v[i]), live ? v_bytes : 0u);
    };
    if constexpr (BLK) aim_block();
    uint32_t voff_a[NI_A], voff_b[NI_B];
#pragma unroll
    for (int j = 0; j < NI_A; ++j) {
        const int f = (wave * NI_A + j) * 64 + lane;
        voff_a[j] = static_cast<uint32_t>(((k_begin + f / (TN / 4)) * ldu + n0 + (f % (TN / 4)) * 4) * 4);
    }
#pragma unroll
    for (int j = 0; j < NI_B; ++j) {
        const int f = (wave * NI_B + j) * 64 + lane;
        voff_b[j] = static_cast<uint32_t>(((k_begin + f / (TM / 4)) * ldv + m0 + (f % (TM / 4)) * 4) * 4);
    }
    const uint32_t step_a = static_cast<uint32_t>(KT * ldu * 4), step_b = static_cast<uint32_t>(KT * ldv * 4);
    auto issue = [&](int t) {                    // stage t -> ring buffer t % NSTAGE; past K: zeros
        const uint32_t base = lds0 + static_cast<uint32_t>(t % NSTAGE) * STAGE_BYTES;
        const uint32_t s = static_cast<uint32_t>(BLK ? stage_in_blk : t);     // stages are requested in order
#pragma unroll
        for (int j = 0; j < NI_A; ++j)
            dma_b128(base + (wave * NI_A + j) * 1024, voff_a[j] + s * step_a, rsrc_u);
#pragma unroll
        for (int j = 0; j < NI_B; ++j)
            dma_b128(base + A_BYTES + (wave * NI_B + j) * 1024, voff_b[j] + s * step_b, rsrc_v);
        if constexpr (BLK) {
            if (++stage_in_blk == stages_per_block) {
                stage_in_blk = 0;
                ++blk;
                aim_block();
            }
        }
    };

    f32x16 acc[BN][2];
#pragma unroll
    for (int a = 0; a < BN; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    // One half-stage = 4 MFMA k-pairs.  Lanes 0..31 feed k = 2*kk, lanes 32..63 feed k = 2*kk + 1.
    // MFMA row i of block t stands for n = 2*i + t (BN = 2) or n = i (BN = 1); columns m = 2*j + t.
    struct Half { f32x2 a[4]; f32x2 b[4]; };
    const uint32_t rd_a = static_cast<uint32_t>(lhi * RA + (wn0 + BN * l32) * 4);
    const uint32_t rd_b = static_cast<uint32_t>(A_BYTES + lhi * RB + (wm0 + 2 * l32) * 4);
    auto load_half = [&](int t, int h, Half& f) {
        const uint32_t base = lds0 + static_cast<uint32_t>(t % NSTAGE) * STAGE_BYTES;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const int krow = 2 * (4 * h + kk);
            const auto pa = reinterpret_cast<__attribute__((address_space(3))) const char*>(base + rd_a + krow * RA);
            const auto pb = reinterpret_cast<__attribute__((address_space(3))) const char*>(base + rd_b + krow * RB);
            if constexpr (BN == 2) f.a[kk] = *reinterpret_cast<__attribute__((address_space(3))) const f32x2*>(pa);
            else f.a[kk].x = *reinterpret_cast<__attribute__((address_space(3))) const float*>(pa);
            f.b[kk] = *reinterpret_cast<__attribute__((address_space(3))) const f32x2*>(pb);
        }
    };
    auto mma_half = [&](const Half& f) {
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a[kk].x, f.b[kk].x, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a[kk].x, f.b[kk].y, acc[0][1], 0, 0, 0);
            if constexpr (BN == 2) {
                acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a[kk].y, f.b[kk].x, acc[1][0], 0, 0, 0);
                acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a[kk].y, f.b[kk].y, acc[1][1], 0, 0, 0);
            }
        }
    };
    auto interleave = [&]() { interleave_groups<8, 8 * BN>(); };

    const int steps = k_end > k_begin ? (k_end - k_begin + KT - 1) / KT : 0;
#pragma unroll
    for (int t = 0; t < NSTAGE - 1; ++t) issue(t);
    wait_vmcnt<(NSTAGE - 2) * LPS>();
    __syncthreads();
    Half h0, h1;
    load_half(0, 0, h0);
    for (int t = 0; t < steps; ++t) {
        load_half(t, 1, h1);
        mma_half(h0);
        interleave();
        __builtin_amdgcn_sched_barrier(0);
        wait_vmcnt<(NSTAGE - 3) * LPS>();         // stage t+1 has landed
        __syncthreads();                          // ... for every wavefront, and stage t-1 is free
        issue(t + NSTAGE - 1);
        load_half(t + 1, 0, h0);
        mma_half(h1);
        interleave();
        __builtin_amdgcn_sched_barrier(0);
    }
    wait_vmcnt<0>();                              // nothing may still be landing in LDS at exit

    // Epilogue.  Accumulator register r of a 32x32 block holds MFMA row 8*(r/4) + 4*(lane/32) + r%4,
    // column lane%32.  Block (ta, tb): n = n0 + wn0 + BN*row + ta, m = m0 + wm0 + 2*col + tb.
    const int64_t mcol = m0 + wm0 + 2 * l32;
    const bool pair_ok = (M % 2 == 0);   // 8-byte accesses need an even row length
#pragma unroll
    for (int ta = 0; ta < BN; ++ta) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = 8 * (r >> 2) + 4 * lhi + (r & 3);
            const int64_t n = n0 + wn0 + BN * row + ta;
            if (n >= N) continue;
            const float d0 = acc[ta][0][r], d1 = acc[ta][1][r];
            if constexpr (PART) {
                float* dp = part + split * part_stride + n * int64_t(M) + mcol;
                if (pair_ok && mcol + 1 < M) {
                    *reinterpret_cast<float2*>(dp) = make_float2(d0, d1);
                } else {
                    if (mcol < M) dp[0] = d0;
                    if (mcol + 1 < M) dp[1] = d1;
                }
                continue;
            }
            float* wp = W + n * int64_t(M) + mcol;
            float* mp = Mom + n * int64_t(M) + mcol;
            if (pair_ok && mcol + 1 < M) {
                float2 w = *reinterpret_cast<float2*>(wp), mo = *reinterpret_cast<float2*>(mp);
                upd(d0, w.x, mo.x, lr, mu, wd);
                upd(d1, w.y, mo.y, lr, mu, wd);
                *reinterpret_cast<float2*>(mp) = mo;
                *reinterpret_cast<float2*>(wp) = w;
            } else {
                if (mcol < M) {
                    float w = wp[0], mo = mp[0];
                    upd(d0, w, mo, lr, mu, wd);
                    mp[0] = mo;
                    wp[0] = w;
                }
                if (mcol + 1 < M) {
                    float w = wp[1], mo = mp[1];
                    upd(d1, w, mo, lr, mu, wd);
                    mp[1] = mo;
                    wp[1] = w;
                }
            }
        }
    }
}

template <int BN, bool PART>
__global__ void __launch_bounds__(THREADS)
sfb_f32_kernel(const float* __restrict__ U, int64_t ldu, const float* __restrict__ V, int64_t ldv,
               float* __restrict__ W, float* __restrict__ Mom, int N, int M, int K, float lr, float mu, float wd,
               int tiles_m, int tiles, uint32_t u_bytes, uint32_t v_bytes, float* __restrict__ part,
               int64_t part_stride, int stages_per_split)
{
    sfb_f32_body<BN, PART, false>(U, ldu, V, ldv, W, Mom, N, M, K, lr, mu, wd, tiles_m, tiles, u_bytes, v_bytes, part,
                                  part_stride, stages_per_split, nullptr, 0, 0);
}

// the P per-worker blocks read in place (u_bytes, v_bytes: the size of ONE block)
template <int BN>
__global__ void __launch_bounds__(THREADS)
sfb_f32_blocks_kernel(BlockPtrs blocks, int n_blocks, int stages_per_block, int64_t ldu, int64_t ldv,
                      float* __restrict__ W, float* __restrict__ Mom, int N, int M, int K, float lr, float mu, float wd,
                      int tiles_m, int tiles, uint32_t u_bytes, uint32_t v_bytes)
{
    sfb_f32_body<BN, false, true>(nullptr, ldu, nullptr, ldv, W, Mom, N, M, K, lr, mu, wd, tiles_m, tiles, u_bytes, v_bytes,
                                  nullptr, 0, 0, &blocks, n_blocks, stages_per_block);
}

template <int BN>
psd_status launch_f32(const float* U, int64_t ldu, const float* V, int64_t ldv, float* W, float* Mom,
                      int64_t N, int64_t M, int64_t K, float lr, float mu, float wd, float* part, int splits,
                      hipStream_t st)
{
    constexpr int TN = 64 * BN;
    const int64_t tiles_n = (N + TN - 1) / TN, tiles_m = (M + TM - 1) / TM;
    const int64_t tiles = tiles_n * tiles_m;
    if (tiles < 1 || tiles * splits > 0x7fffffff) return PSD_E_INVALID;
    // 32-bit byte offsets into each factor matrix, with room for the stages of read-ahead
    const int64_t u_bytes = K * ldu * 4, v_bytes = K * ldv * 4;
    const int64_t reach = (int64_t(1) << 32) - (NSTAGE + 2) * KT * (ldu > ldv ? ldu : ldv) * 4 - 4096;
    if (u_bytes > reach || v_bytes > reach) return PSD_E_UNSUPPORTED;
    const int64_t stages = (K + KT - 1) / KT;
    const int sps = static_cast<int>((stages + splits - 1) / splits);
    auto kern = splits > 1 ? sfb_f32_kernel<BN, true> : sfb_f32_kernel<BN, false>;
    hipLaunchKernelGGL(kern, dim3(static_cast<uint32_t>(tiles * splits)), dim3(THREADS), 0, st, U, ldu, V, ldv, W, Mom,
                       static_cast<int>(N), static_cast<int>(M), static_cast<int>(K), lr, mu, wd,
                       static_cast<int>(tiles_m), static_cast<int>(tiles), static_cast<uint32_t>(u_bytes),
                       static_cast<uint32_t>(v_bytes), part, sfb_part_stride(N, M), sps);
    PSD_HIP_TRY(hipGetLastError());
    if (splits > 1) return launch_sfb_reduce(part, splits, N, M, W, Mom, lr, mu, wd, st);
    return PSD_OK;
}

template <int BN>
psd_status launch_f32_blocks(const BlockPtrs& blocks, int64_t P, int64_t B, int64_t ldu, int64_t ldv, float* W,
                             float* Mom, int64_t N, int64_t M, float lr, float mu, float wd, hipStream_t st)
{
    constexpr int TN = 64 * BN;
    const int64_t tiles_n = (N + TN - 1) / TN, tiles_m = (M + TM - 1) / TM;
    const int64_t tiles = tiles_n * tiles_m;
    if (tiles < 1 || tiles > 0x7fffffff) return PSD_E_INVALID;
    const int64_t u_bytes = B * ldu * 4, v_bytes = B * ldv * 4;        // one block
    if (u_bytes >= (int64_t(1) << 32) || v_bytes >= (int64_t(1) << 32)) return PSD_E_UNSUPPORTED;
    hipLaunchKernelGGL(sfb_f32_blocks_kernel<BN>, dim3(static_cast<uint32_t>(tiles)), dim3(THREADS), 0, st, blocks,
                       static_cast<int>(P), static_cast<int>(B / KT), ldu, ldv, W, Mom, static_cast<int>(N),
                       static_cast<int>(M), static_cast<int>(P * B), lr, mu, wd, static_cast<int>(tiles_m), static_cast<int>(tiles),
                       static_cast<uint32_t>(u_bytes), static_cast<uint32_t>(v_bytes));
    PSD_HIP_TRY(hipGetLastError());
    return PSD_OK;
}

// tile choice (and, with a workspace, the split of K) for one layer
void choose_f32(int64_t N, int64_t M, int64_t K, bool may_split, int* bn, int* splits)
{
    // 128 x 128 tiles unless that leaves fewer than two workgroups per compute unit (one workgroup's
    // four wavefronts cannot hide LDS and barrier latency on their own); with a workspace, few tiles
    // are made up for by splitting K instead of by halving the tile
    const int64_t slots = 2 * int64_t(device_cu_count());
    const int64_t tiles128 = ((N + 127) / 128) * ((M + TM - 1) / TM);
    const int forced = tune_value(PSD_TUNE_SFB_F32_TILE);
    const int s128 = may_split ? sfb_splits_for(tiles128, slots, K) : 1;
    if (forced == 1 || forced == 2) *bn = forced;
    else *bn = (tiles128 < slots && s128 == 1) ? 1 : 2;
    const int64_t tiles = ((N + 64 * *bn - 1) / (64 * *bn)) * ((M + TM - 1) / TM);
    *splits = may_split ? sfb_splits_for(tiles, slots, K) : 1;
}

}  // namespace

int sfb_f32_splits(int64_t N, int64_t M, int64_t K)
{
    int bn, s;
    choose_f32(N, M, K, true, &bn, &s);
    return s;
}

psd_status launch_sfb_f32(const float* U, int64_t ldu, const float* V, int64_t ldv, float* W, float* Mom,
                          int64_t N, int64_t M, int64_t K, float lr, float mu, float wd, float* part, int splits,
                          hipStream_t st)
{
    int bn, s;
    choose_f32(N, M, K, splits > 1, &bn, &s);
    if (bn == 1) return launch_f32<1>(U, ldu, V, ldv, W, Mom, N, M, K, lr, mu, wd, part, splits, st);
    return launch_f32<2>(U, ldu, V, ldv, W, Mom, N, M, K, lr, mu, wd, part, splits, st);
}

bool sfb_f32_blocks_supported(int64_t B) { return B % KT == 0; }     // whole k-stages per block

psd_status launch_sfb_f32_blocks(const float* const* U_p, int64_t ldu, const float* const* V_p, int64_t ldv, int64_t P,
                                 int64_t B, float* W, float* Mom, int64_t N, int64_t M, float lr, float mu, float wd,
                                 hipStream_t st)
{
    if (P < 1 || P > PSD_MAX_WORKERS || !sfb_f32_blocks_supported(B)) return PSD_E_UNSUPPORTED;
    BlockPtrs blocks;
    for (int64_t p = 0; p < PSD_MAX_WORKERS; ++p) {
        blocks.u[p] = p < P ? U_p[p] : nullptr;
        blocks.v[p] = p < P ? V_p[p] : nullptr;
    }
    int bn, s;
    choose_f32(N, M, P * B, false, &bn, &s);
    if (bn == 1) return launch_f32_blocks<1>(blocks, P, B, ldu, ldv, W, Mom, N, M, lr, mu, wd, st);
    return launch_f32_blocks<2>(blocks, P, B, ldu, ldv, W, Mom, N, M, lr, mu, wd, st);
}

}  // namespace psd
