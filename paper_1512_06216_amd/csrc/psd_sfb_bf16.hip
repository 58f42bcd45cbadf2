// SFB reconstruction with fused momentum-SGD update, bf16 factors, fp32 accumulation and
// fp32 W / Mom (Section 4.3.1 step 3, Eq. 5; Algorithm 3's update line):
//     dW[n][m] = sum_k U[k][n] * V[k][m] ;  Mom = mu*Mom + lr*dW ;  W = W - Mom
//
// Layout problem.  The contraction index k is the OUTER dimension of both stacked factor
// matrices, while v_mfma_f32_32x32x16_bf16 wants 8 consecutive k in one lane.  Tiles are
// copied to LDS as they are (K-outer, 16-byte chunks) and read back with gfx950's
// transposing LDS load (ds_read_b64_tr_b16): a 16-lane group reads four k rows x 16 columns
// and each lane ends up with the 4 k values of its own column.
//
// Feeding the MFMA pipe.  One k-stage of MFMA work (~0.4 us) is much shorter than a loaded
// L2/HBM round trip (>1 us at the tail), so the tiles travel global -> LDS without passing
// through registers (buffer_load_dwordx4 ... lds) and NSTAGE-1 stages are kept in flight in
// an NSTAGE-deep ring of LDS buffers.  The DMA writes whole 1 KiB runs, so rows cannot be
// padded; bank conflicts of the transposing reads are avoided by XOR-swizzling the 16-byte
// chunk index of a row with its row number instead.  Rows past the end of K are zero-filled
// by the buffer range check, so there is no tail code.
//
// MFMA operand roles are swapped (rows = m, columns = n) so that the four consecutive
// accumulator rows a lane owns are four adjacent m of one W row; the epilogue turns each
// block through LDS so that W and Mom move in 16-byte accesses, 128 contiguous bytes per row.
#include <atomic>
#include "psd_device.h"
#include "psd_internal.h"

namespace psd {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;

constexpr int KT = 32;         // k rows per LDS stage (two MFMA k-steps of 16)
constexpr int GROUP_N = 8;     // tile rows per raster group (L2 reuse of the V panels)
constexpr int PLD = 36;        // epilogue patch row stride in floats (144 B: conflict-free)

// WN x WM wavefronts, each owning BN x BM MFMA blocks of 32 x 32; NSTAGE LDS buffers;
// OCC = wavefronts per SIMD the register budget is sized for
template <int WN_, int WM_, int BN_, int BM_, int NSTAGE_, int OCC_>
struct Cfg {
    static constexpr int WN = WN_, WM = WM_, BN = BN_, BM = BM_, NSTAGE = NSTAGE_, OCC = OCC_;
    static constexpr int WAVES = WN * WM, THREADS = 64 * WAVES;
    static constexpr int TN = 32 * BN * WN, TM = 32 * BM * WM;   // workgroup tile
    static constexpr int RA = TN * 2, RB = TM * 2;               // LDS row bytes (U tile, V tile)
    static constexpr int A_BYTES = KT * RA, B_BYTES = KT * RB, STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int NI_A = A_BYTES / 1024 / WAVES;          // 1 KiB DMA instructions per wavefront
    static constexpr int NI_B = B_BYTES / 1024 / WAVES;
    static constexpr int PATCH_BYTES = WAVES * 32 * PLD * 4;
    static constexpr size_t LDS_BYTES =
        size_t(NSTAGE) * STAGE_BYTES > size_t(PATCH_BYTES) ? size_t(NSTAGE) * STAGE_BYTES : size_t(PATCH_BYTES);
    static_assert(A_BYTES % (1024 * WAVES) == 0 && B_BYTES % (1024 * WAVES) == 0, "stage must split into 1 KiB runs");
    static_assert(RA % 128 == 0 && RB % 128 == 0, "the swizzle permutes chunks inside 128-byte groups");
    static_assert(NSTAGE >= 3, "the pipeline keeps at least one stage in flight beyond the one being awaited");
};

__device__ __forceinline__ bf16x4 read_tr(uint32_t lds_addr)
{
    return __builtin_amdgcn_ds_read_tr16_b64_v4bf16(reinterpret_cast<lds_bf16x4*>(lds_addr));
}

// PART = false: one workgroup per tile contracts over all of K and applies the update.
// PART = true (layers with too few tiles to fill the chip): the grid holds `splits` workgroups per
// tile, workgroup (tile, s) contracts over k-stages [s * stages_per_split, (s+1) * stages_per_split)
// and stores its partial dW tile to part + s * part_stride (N x M row-major); the partials are summed
// in split order and the update applied by the parameter-server sum kernel afterwards.
// BLK = true: the factors are not stacked.  Row k = p*B + b of U is row b of the p-th worker's B x ldu block
// (V likewise), read where it lies: a stage of KT rows never straddles two blocks because KT divides B, so
// the only difference is that the buffer descriptors are re-aimed whenever the stages move on to the next
// block (and aimed at nothing past the last one, which reads as zeros like the K tail does).
struct BlockPtrs { const uint16_t* u[PSD_MAX_WORKERS]; const uint16_t* v[PSD_MAX_WORKERS]; };

template <class C, bool PART, bool BLK, bool STREAM>
__device__ __forceinline__ void
sfb_bf16_body(const uint16_t* __restrict__ U, int64_t ldu, const uint16_t* __restrict__ V, int64_t ldv,
              float* __restrict__ W, float* __restrict__ Mom, int N, int M, int K, float lr, float mu, float wd,
              int tiles_n, int tiles_m, uint32_t u_bytes, uint32_t v_bytes, float* __restrict__ part,
              int64_t part_stride, int stages_per_split, int skew_blocks, int skew_ticks,
              const BlockPtrs* blocks, int n_blocks, int stages_per_block)
{
    static_assert(!(PART && BLK), "blocks read in place are not combined with a split of K");
    // Measurement aid (off unless asked for): the workgroups that start first on the odd-numbered
    // XCDs wait skew_ticks of the 100 MHz wall clock, which puts the two halves of the chip out of
    // phase (MFMA loop on one, W / Mom update on the other).  The wait ends by the clock; the
    // iteration cap only bounds it should the clock not advance.
    if (skew_ticks > 0 && (blockIdx.x & 1) && static_cast<int>(blockIdx.x) < skew_blocks) {
        const long long t0 = wall_clock64();
        for (int i = 0; i < 200000 && wall_clock64() - t0 < skew_ticks; ++i) __builtin_amdgcn_s_sleep(8);
    }
    extern __shared__ __attribute__((aligned(1024))) uint16_t lds[];
    const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(
        (__attribute__((address_space(3))) void*)lds));

    // Workgroup -> tile.  Consecutive workgroup ids go round-robin over the 8 XCDs; give each
    // XCD a contiguous run of the tile sequence, and order that sequence in groups of GROUP_N
    // tile rows so that the workgroups sharing an L2 re-use the same few U and V panels.
    const int T = tiles_n * tiles_m;
    const int split = PART ? __builtin_amdgcn_readfirstlane(blockIdx.x / T) : 0;   // (the division runs on the vector ALU)
    const int b = PART ? blockIdx.x - split * T : blockIdx.x, xcd = b & 7;
    const int lin = xcd * (T >> 3) + (xcd < (T & 7) ? xcd : (T & 7)) + (b >> 3);
    const int per_group = GROUP_N * tiles_m;
    const int g = lin / per_group, in_g = lin - g * per_group;
    const int rows_g = tiles_n - g * GROUP_N < GROUP_N ? tiles_n - g * GROUP_N : GROUP_N;
    const int tile_n = g * GROUP_N + in_g % rows_g, tile_m = in_g / rows_g;

    const int64_t n0 = int64_t(tile_n) * C::TN, m0 = int64_t(tile_m) * C::TM;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wn0 = (wave / C::WM) * 32 * C::BN, wm0 = (wave % C::WM) * 32 * C::BM;
    const int grp = lane >> 4, l16 = lane & 15;

    // ---- DMA plan: instruction j of this wavefront moves one 1 KiB run of a stage (a whole number
    // of rows, or row fragments for 384-byte rows), lane i carrying the chunk that belongs at
    // physical position i of that run.
    // physical chunk pc of row r holds logical chunk pc ^ ((r & 3) << 1)
    // this workgroup's k range: rows at or past k_end read as zeros (descriptor size), rows before
    // k_begin are skipped (offsets)
    const int k_begin = PART ? split * stages_per_split * KT : 0;
    const int k_end = PART ? (k_begin + stages_per_split * KT < K ? k_begin + stages_per_split * KT : K) : K;
    if constexpr (PART) {
        u_bytes = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(int64_t(k_end) * ldu * 2));
        v_bytes = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(int64_t(k_end) * ldv * 2));
    }
    i32x4 rsrc_u = raw_rsrc(U, u_bytes), rsrc_v = raw_rsrc(V, v_bytes);
    int blk = 0, stage_in_blk = 0;               // BLK: where the next stage to be requested lies
    auto aim_block = [&]() {                     // BLK: descriptors over block `blk` (u_bytes, v_bytes = one block)
        const bool live = blk < n_blocks;
        const int i = live ? blk : 0;            // the table is never indexed past its end
        rsrc_u = raw_rsrc(uniform_ptr(blocks->u[i]), live ? u_bytes : 0u);
        rsrc_v = raw_rsrc(uniform_ptr(blocks->v[i]), live ? v_bytes : 0u);
    };
    if constexpr (BLK) aim_block();
    uint32_t voff_a[C::NI_A], voff_b[C::NI_B];
    {
        constexpr int LPR = C::RA / 16;              // 16-byte chunks per row
#pragma unroll
        for (int j = 0; j < C::NI_A; ++j) {
            const int f = (wave * C::NI_A + j) * 64 + lane;   // chunk index inside the stage
            const int r = f / LPR;
            const int lc = (f % LPR) ^ ((r & 3) << 1);
            voff_a[j] = static_cast<uint32_t>(((k_begin + r) * ldu + n0 + lc * 8) * 2);
        }
    }
    {
        constexpr int LPR = C::RB / 16;
#pragma unroll
        for (int j = 0; j < C::NI_B; ++j) {
            const int f = (wave * C::NI_B + j) * 64 + lane;
            const int r = f / LPR;
            const int lc = (f % LPR) ^ ((r & 3) << 1);
            voff_b[j] = static_cast<uint32_t>(((k_begin + r) * ldv + m0 + lc * 8) * 2);
        }
    }
    const uint32_t step_a = static_cast<uint32_t>(KT * ldu * 2), step_b = static_cast<uint32_t>(KT * ldv * 2);
    auto issue = [&](int t) {                    // stage t -> ring buffer t % NSTAGE (stages are requested in order)
        const uint32_t base = lds0 + static_cast<uint32_t>(t % C::NSTAGE) * C::STAGE_BYTES;
        const uint32_t s = static_cast<uint32_t>(BLK ? stage_in_blk : t);
#pragma unroll
        for (int j = 0; j < C::NI_A; ++j)
            dma_b128(base + (wave * C::NI_A + j) * 1024, voff_a[j] + s * step_a, rsrc_u);
#pragma unroll
        for (int j = 0; j < C::NI_B; ++j)
            dma_b128(base + C::A_BYTES + (wave * C::NI_B + j) * 1024, voff_b[j] + s * step_b, rsrc_v);
        if constexpr (BLK) {
            if (++stage_in_blk == stages_per_block) {
                stage_in_blk = 0;
                ++blk;
                aim_block();
            }
        }
    };

    // ---- transposing-read plan.  A 16-lane group reads a (4 k) x (16 column) patch: lane L
    // supplies the address of 4 adjacent columns of row (L%16)/4 starting at column 4*(L%4), and
    // ends up with rows 0..3 of column L%16.  Lane groups: columns +16*(grp%2), k rows +8*(grp/2).
    // The byte address of this lane's piece inside a stage buffer, for k-step 0, low half:
    uint32_t rd_a[C::BN], rd_b[C::BM];
    {
        const int row = 8 * (grp >> 1) + (l16 >> 2);           // row & 3 == l16 >> 2
        const int sw = (l16 >> 2) << 1;
#pragma unroll
        for (int bn = 0; bn < C::BN; ++bn) {
            const int chunk = (((wn0 + 32 * bn + 16 * (grp & 1)) >> 3) ^ sw) + ((l16 & 3) >> 1);
            rd_a[bn] = static_cast<uint32_t>(row * C::RA + chunk * 16 + (l16 & 1) * 8);
        }
#pragma unroll
        for (int bm = 0; bm < C::BM; ++bm) {
            const int chunk = (((wm0 + 32 * bm + 16 * (grp & 1)) >> 3) ^ sw) + ((l16 & 3) >> 1);
            rd_b[bm] = static_cast<uint32_t>(C::A_BYTES + row * C::RB + chunk * 16 + (l16 & 1) * 8);
        }
    }

    f32x16 acc[C::BN][C::BM];
#pragma unroll
    for (int a = 0; a < C::BN; ++a)
#pragma unroll
        for (int c = 0; c < C::BM; ++c)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][c][r] = 0.f;

    // this lane's 8 k values of a 16-row MFMA step: ks + 8*(grp/2) + 0..7 (the same for both operands)
    auto load_frags = [&](uint32_t base, int ks, bf16x8 (&a)[C::BN], bf16x8 (&bb)[C::BM]) {
#pragma unroll
        for (int bn = 0; bn < C::BN; ++bn) {
            const bf16x4 lo = read_tr(base + rd_a[bn] + ks * C::RA);
            const bf16x4 hi = read_tr(base + rd_a[bn] + (ks + 4) * C::RA);
            a[bn] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        }
#pragma unroll
        for (int bm = 0; bm < C::BM; ++bm) {
            const bf16x4 lo = read_tr(base + rd_b[bm] + ks * C::RB);
            const bf16x4 hi = read_tr(base + rd_b[bm] + (ks + 4) * C::RB);
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

    const int steps = k_end > k_begin ? (k_end - k_begin + KT - 1) / KT : 0;
    constexpr int LPS = C::NI_A + C::NI_B;       // DMA instructions per wavefront per stage
    auto stage_base = [&](int t) { return lds0 + static_cast<uint32_t>(t % C::NSTAGE) * C::STAGE_BYTES; };

    // Software pipeline (one wavefront may be alone on its SIMD, so it has to overlap with itself):
    // the operand reads of one MFMA step are always issued before the MFMAs of the step before,
    // also across the stage boundary, and the barrier sits between the two steps of a stage.
    //   F0 = step 0 of stage t (read during the previous iteration)
    //   read F1 = step 1 of stage t | MFMA(F0) | stage t+1 landed? barrier | DMA stage t+NSTAGE-1 |
    //   read F0 = step 0 of stage t+1 | MFMA(F1)
    // The barrier tells both that every wavefront's share of stage t+1 is visible and that nobody
    // still reads stage t-1, whose buffer the new DMA overwrites.  Stages past K are zeros.
    bf16x8 a0[C::BN], b0[C::BM], a1[C::BN], b1[C::BM];
#pragma unroll
    for (int t = 0; t < C::NSTAGE - 1; ++t) issue(t);
    wait_vmcnt<(C::NSTAGE - 2) * LPS>();
    __syncthreads();
    load_frags(stage_base(0), 0, a0, b0);
    // A wavefront issues at most one LDS instruction per ~16 cycles and one MFMA per 32, in program
    // order; operand reads are therefore spread between the MFMAs they do not feed (1 MFMA, then
    // its share of reads, ...) so that their issue time hides under MFMA execution.
    auto interleave = [&]() { interleave_groups<2 * (C::BN + C::BM), C::BN * C::BM>(); };
    for (int t = 0; t < steps; ++t) {
        load_frags(stage_base(t), 16, a1, b1);
        mma(a0, b0);
        interleave();
        __builtin_amdgcn_sched_barrier(0);
        wait_vmcnt<(C::NSTAGE - 3) * LPS>();
        __syncthreads();
        issue(t + C::NSTAGE - 1);
        load_frags(stage_base(t + 1), 0, a0, b0);
        mma(a1, b1);
        interleave();
        __builtin_amdgcn_sched_barrier(0);
    }
    wait_vmcnt<0>();                             // trailing zero stages must not land on the epilogue patch
    __syncthreads();

    // Epilogue.  Accumulator register r of block (bn, bm) holds MFMA row 8*(r/4) + 4*(lane/32) + r%4
    // (= m offset) and column lane%32 (= n offset): four adjacent m per register quad.
    const int l32 = lane & 31, lhi = lane >> 5;
    if (M % 4 == 0) {
        // Fast path.  Held as they are, the quads of one W row sit in 2 lanes x 4 registers, and a
        // wavefront access would touch 32 rows x 32 bytes: measured at ~3.1 TB/s for the W/Mom
        // read-modify-write, against ~4.9 TB/s once every row gets >= 128 contiguous bytes per
        // instruction.  So each 32 x 32 block is turned through a private LDS patch: written as
        // held, read back with 8 lanes per row, then 8 rows x 128 bytes per global access.
        float* patch = reinterpret_cast<float*>(lds) + wave * (32 * PLD);
        const int prow = lane >> 3, pcol = 4 * (lane & 7);
        // STREAM: W / Mom with the streaming hint.  The host asks for it when their rows start on cache-line
        // boundaries (every 128-byte access is then a whole line); with rows that start mid-line (M = 3000)
        // the hint makes the partial-line stores expensive (measured 3000 -> 21841: 468 -> 534 us).
        constexpr bool stream = STREAM;
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
                if constexpr (PART) {
                    float* dst = part + split * part_stride;
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj) {
                        const int64_t n = n0 + wn0 + 32 * bn + prow + 8 * jj;
                        d[jj] = *reinterpret_cast<const float4*>(patch + (prow + 8 * jj) * PLD + pcol);
                        if (n < N && m < M) *reinterpret_cast<float4*>(dst + n * int64_t(M) + m) = d[jj];
                    }
                    continue;
                }
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    const int64_t n = n0 + wn0 + 32 * bn + prow + 8 * jj;
                    d[jj] = *reinterpret_cast<const float4*>(patch + (prow + 8 * jj) * PLD + pcol);
                    if (n < N && m < M) {                  // m % 4 == 0 and M % 4 == 0: whole quad inside
                        const float* wp = W + n * int64_t(M) + m;
                        const float* mp = Mom + n * int64_t(M) + m;
                        w[jj] = stream ? load_stream4(wp) : *reinterpret_cast<const float4*>(wp);
                        mo[jj] = stream ? load_stream4(mp) : *reinterpret_cast<const float4*>(mp);
                    }
                }
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    const int64_t n = n0 + wn0 + 32 * bn + prow + 8 * jj;
                    if (n < N && m < M) {
                        upd(d[jj].x, w[jj].x, mo[jj].x, lr, mu, wd);
                        upd(d[jj].y, w[jj].y, mo[jj].y, lr, mu, wd);
                        upd(d[jj].z, w[jj].z, mo[jj].z, lr, mu, wd);
                        upd(d[jj].w, w[jj].w, mo[jj].w, lr, mu, wd);
                        if (stream) {
                            store_stream4(Mom + n * int64_t(M) + m, mo[jj]);
                            store_stream4(W + n * int64_t(M) + m, w[jj]);
                        } else {
                            *reinterpret_cast<float4*>(Mom + n * int64_t(M) + m) = mo[jj];
                            *reinterpret_cast<float4*>(W + n * int64_t(M) + m) = w[jj];
                        }
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
                    if constexpr (PART) {
                        if (m < M) part[split * part_stride + n * int64_t(M) + m] = acc[bn][bm][r];
                        continue;
                    }
                    if (m < M) {
                        float wv = wrow[m], mv = mrow[m];
                        upd(acc[bn][bm][r], wv, mv, lr, mu, wd);
                        mrow[m] = mv;
                        wrow[m] = wv;
                    }
                }
        }
    }
}

template <class C, bool PART, bool STREAM>
__global__ void __launch_bounds__(C::THREADS, C::OCC)
sfb_bf16_kernel(const uint16_t* __restrict__ U, int64_t ldu, const uint16_t* __restrict__ V, int64_t ldv,
                float* __restrict__ W, float* __restrict__ Mom, int N, int M, int K, float lr, float mu, float wd,
                int tiles_n, int tiles_m, uint32_t u_bytes, uint32_t v_bytes, float* __restrict__ part,
                int64_t part_stride, int stages_per_split, int skew_blocks, int skew_ticks)
{
    sfb_bf16_body<C, PART, false, STREAM>(U, ldu, V, ldv, W, Mom, N, M, K, lr, mu, wd, tiles_n, tiles_m, u_bytes, v_bytes, part,
                                  part_stride, stages_per_split, skew_blocks, skew_ticks, nullptr, 0, 0);
}

// the P per-worker blocks read in place (u_bytes, v_bytes: the size of ONE block)
template <class C, bool STREAM>
__global__ void __launch_bounds__(C::THREADS, C::OCC)
sfb_bf16_blocks_kernel(BlockPtrs blocks, int n_blocks, int stages_per_block, int64_t ldu, int64_t ldv,
                       float* __restrict__ W, float* __restrict__ Mom, int N, int M, int K, float lr, float mu, float wd,
                       int tiles_n, int tiles_m, uint32_t u_bytes, uint32_t v_bytes)
{
    sfb_bf16_body<C, false, true, STREAM>(nullptr, ldu, nullptr, ldv, W, Mom, N, M, K, lr, mu, wd, tiles_n, tiles_m, u_bytes,
                                  v_bytes, nullptr, 0, 0, 0, 0, &blocks, n_blocks, stages_per_block);
}

template <class C>
psd_status launch_cfg_blocks(const BlockPtrs& blocks, int64_t P, int64_t B, int64_t ldu, int64_t ldv, float* W, float* Mom,
                             int64_t N, int64_t M, float lr, float mu, float wd, hipStream_t st)
{
    const int64_t tiles_n = (N + C::TN - 1) / C::TN, tiles_m = (M + C::TM - 1) / C::TM;
    const int64_t tiles = tiles_n * tiles_m;
    if (tiles < 1 || tiles > 0x3fffffff) return PSD_E_INVALID;
    const int64_t u_bytes = B * ldu * 2, v_bytes = B * ldv * 2;          // one block
    if (u_bytes >= (int64_t(1) << 32) || v_bytes >= (int64_t(1) << 32)) return PSD_E_UNSUPPORTED;
    auto kern = M % 32 == 0 ? sfb_bf16_blocks_kernel<C, true> : sfb_bf16_blocks_kernel<C, false>;
    static std::atomic<bool> attr_done{false};
    if (!attr_done.load(std::memory_order_acquire)) {
        PSD_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(sfb_bf16_blocks_kernel<C, true>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, int(C::LDS_BYTES)));
        PSD_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(sfb_bf16_blocks_kernel<C, false>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, int(C::LDS_BYTES)));
        attr_done.store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL(kern, dim3(static_cast<uint32_t>(tiles)), dim3(C::THREADS), C::LDS_BYTES, st,
                       blocks, static_cast<int>(P), static_cast<int>(B / KT), ldu, ldv, W, Mom, static_cast<int>(N),
                       static_cast<int>(M), static_cast<int>(P * B), lr, mu, wd, static_cast<int>(tiles_n),
                       static_cast<int>(tiles_m), static_cast<uint32_t>(u_bytes), static_cast<uint32_t>(v_bytes));
    PSD_HIP_TRY(hipGetLastError());
    return PSD_OK;
}

template <class C>
psd_status launch_cfg(const uint16_t* U, int64_t ldu, const uint16_t* V, int64_t ldv, float* W, float* Mom,
                      int64_t N, int64_t M, int64_t K, float lr, float mu, float wd, float* part, int splits,
                      hipStream_t st)
{
    const int64_t tiles_n = (N + C::TN - 1) / C::TN, tiles_m = (M + C::TM - 1) / C::TM;
    const int64_t tiles = tiles_n * tiles_m;
    if (tiles < 1 || tiles * splits > 0x3fffffff) return PSD_E_INVALID;
    // 32-bit byte offsets into each factor matrix, with room for the stages of read-ahead
    const int64_t u_bytes = K * ldu * 2, v_bytes = K * ldv * 2;
    const int64_t reach = (int64_t(1) << 32) - (C::NSTAGE + 2) * KT * (ldu > ldv ? ldu : ldv) * 2 - 4096;
    if (u_bytes > reach || v_bytes > reach) return PSD_E_UNSUPPORTED;
    // W / Mom are streamed when their rows start on cache-line boundaries (see the epilogue)
    auto kern = splits > 1 ? sfb_bf16_kernel<C, true, false>
                           : (M % 32 == 0 ? sfb_bf16_kernel<C, false, true> : sfb_bf16_kernel<C, false, false>);
    // raise the dynamic LDS limit once per process (idempotent, so a race between two first
    // callers is harmless; the flag only saves the call on later launches)
    static std::atomic<bool> attr_done{false};
    if (!attr_done.load(std::memory_order_acquire)) {
        PSD_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(sfb_bf16_kernel<C, true, false>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, int(C::LDS_BYTES)));
        PSD_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(sfb_bf16_kernel<C, false, true>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, int(C::LDS_BYTES)));
        PSD_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(sfb_bf16_kernel<C, false, false>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, int(C::LDS_BYTES)));
        attr_done.store(true, std::memory_order_release);
    }
    const int skew = tune_value(PSD_TUNE_SFB_BF16_SKEW_US);
    const int64_t stages = (K + KT - 1) / KT;
    const int sps = static_cast<int>((stages + splits - 1) / splits);
    hipLaunchKernelGGL(kern, dim3(static_cast<uint32_t>(tiles * splits)), dim3(C::THREADS), C::LDS_BYTES, st, U, ldu, V,
                       ldv, W, Mom, static_cast<int>(N), static_cast<int>(M), static_cast<int>(K), lr, mu, wd,
                       static_cast<int>(tiles_n), static_cast<int>(tiles_m), static_cast<uint32_t>(u_bytes),
                       static_cast<uint32_t>(v_bytes), part, sfb_part_stride(N, M), sps,
                       device_cu_count() * C::OCC, skew > 0 ? skew * 100 : 0);
    PSD_HIP_TRY(hipGetLastError());
    if (splits > 1) return launch_sfb_reduce(part, splits, N, M, W, Mom, lr, mu, wd, st);
    return PSD_OK;
}

using Cfg128x256w4 = Cfg<2, 2, 2, 4, 3, 2>;   // 4 wavefronts of 64 x 128, 3 stages (72 KiB), two workgroups per CU
using Cfg128x192w4 = Cfg<2, 2, 2, 3, 4, 2>;   // 4 wavefronts of 64 x 96, 4 stages (80 KiB), two workgroups per CU
using Cfg128x128w4 = Cfg<2, 2, 2, 2, 4, 2>;   // small layers: more workgroups (64 KiB, two per CU)

}  // namespace

namespace {
struct Bf16Tile { int id, tn, tm; };
// tile choice (and, with a workspace, the split of K) for one layer
void choose_bf16(int64_t N, int64_t M, int64_t K, bool may_split, Bf16Tile* tile, int* splits)
{
    static const Bf16Tile tiles_by_id[] = {{0, 128, 256}, {1, 128, 192}, {2, 128, 128}};
    const int64_t slots = int64_t(device_cu_count()) * 2;
    int pick = tune_value(PSD_TUNE_SFB_BF16_TILE);
    if (pick < 0 || pick > 2) {
        // Workgroups of one launch run in rounds of (CUs x workgroups per CU); a partly filled last
        // round costs as much as a full one.  Pick the tile whose rounds x tile area is smallest
        // (ties go to the larger tile; the 128 x 128 tile pays ~10% for its lower MFMA duty).
        const int weight[] = {100, 100, 110};
        int64_t best = -1;
        for (const Bf16Tile& c : tiles_by_id) {
            const int64_t tiles = ((N + c.tn - 1) / c.tn) * ((M + c.tm - 1) / c.tm);
            const int64_t cost = ((tiles + slots - 1) / slots) * c.tn * c.tm * weight[c.id];
            if (best < 0 || cost < best) { best = cost; pick = c.id; }
        }
    }
    *tile = tiles_by_id[pick];
    const int64_t tiles = ((N + tile->tn - 1) / tile->tn) * ((M + tile->tm - 1) / tile->tm);
    *splits = may_split ? sfb_splits_for(tiles, slots, K) : 1;
}
}  // namespace

int sfb_bf16_splits(int64_t N, int64_t M, int64_t K)
{
    Bf16Tile t;
    int s;
    choose_bf16(N, M, K, true, &t, &s);
    return s;
}

psd_status launch_sfb_bf16(const uint16_t* U, int64_t ldu, const uint16_t* V, int64_t ldv, float* W, float* Mom,
                           int64_t N, int64_t M, int64_t K, float lr, float mu, float wd, float* part, int splits,
                           hipStream_t st)
{
    Bf16Tile t;
    int unused;
    choose_bf16(N, M, K, false, &t, &unused);
    switch (t.id) {
        case 0: return launch_cfg<Cfg128x256w4>(U, ldu, V, ldv, W, Mom, N, M, K, lr, mu, wd, part, splits, st);
        case 1: return launch_cfg<Cfg128x192w4>(U, ldu, V, ldv, W, Mom, N, M, K, lr, mu, wd, part, splits, st);
        default: return launch_cfg<Cfg128x128w4>(U, ldu, V, ldv, W, Mom, N, M, K, lr, mu, wd, part, splits, st);
    }
}

bool sfb_bf16_blocks_supported(int64_t B) { return B % KT == 0; }

psd_status launch_sfb_bf16_blocks(const uint16_t* const* U_p, int64_t ldu, const uint16_t* const* V_p, int64_t ldv,
                                  int64_t P, int64_t B, float* W, float* Mom, int64_t N, int64_t M, float lr, float mu,
                                  float wd, hipStream_t st)
{
    if (P < 1 || P > PSD_MAX_WORKERS || !sfb_bf16_blocks_supported(B)) return PSD_E_UNSUPPORTED;
    BlockPtrs blocks;
    for (int64_t p = 0; p < PSD_MAX_WORKERS; ++p) {
        blocks.u[p] = p < P ? U_p[p] : nullptr;
        blocks.v[p] = p < P ? V_p[p] : nullptr;
    }
    Bf16Tile t;
    int unused;
    choose_bf16(N, M, P * B, false, &t, &unused);
    switch (t.id) {
        case 0: return launch_cfg_blocks<Cfg128x256w4>(blocks, P, B, ldu, ldv, W, Mom, N, M, lr, mu, wd, st);
        case 1: return launch_cfg_blocks<Cfg128x192w4>(blocks, P, B, ldu, ldv, W, Mom, N, M, lr, mu, wd, st);
        default: return launch_cfg_blocks<Cfg128x128w4>(blocks, P, B, ldu, ldv, W, Mom, N, M, lr, mu, wd, st);
    }
}

}  // namespace psd
