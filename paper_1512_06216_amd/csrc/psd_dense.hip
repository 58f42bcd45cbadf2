// Parameter-server route on one GPU: per key, sum the P dense gradient copies and apply
// the momentum-SGD update (Algorithm 1 master node; Algorithm 3 non-FC branch).
//
// HBM-bound streaming kernel: (4P + 16) bytes per key, P + 3 flops.  The reduction runs
// over the P copies, which all sit in one lane's registers, so there is nothing to reduce
// across lanes and nothing to stage in LDS: the design is all about keeping many 16-byte
// loads in flight per lane and every wavefront access a full 1 KiB contiguous segment.
//
// Grid: shard-major.  Workgroup g serves chunk g % chunks of shard g / chunks, so consecutive
// workgroups (which the hardware deals round-robin over the 8 XCDs) stream consecutive
// memory and the whole launch walks the key space once, shard after shard.  Giving each
// XCD its own shard instead (workgroup g -> shard g % S) was measured 6% slower at S = 8 and
// 10% slower at S = 64: eight far-apart streams per array collide on HBM channels.
#include "psd_device.h"
#include "psd_internal.h"

namespace psd {

constexpr int kDenseThreads = 256;
constexpr int kDenseUnroll = 2;                                   // float4 per lane per chunk
constexpr int64_t kDenseChunk = int64_t(kDenseThreads) * 4 * kDenseUnroll;  // keys per workgroup

int32_t dense_chunks_for(int64_t n, int32_t S)
{
    const int64_t longest = (n + S - 1) / S;   // floor((s+1)n/S) - floor(sn/S) <= ceil(n/S)
    return static_cast<int32_t>((longest + kDenseChunk - 1) / kDenseChunk);
}

namespace {

// 16-byte streaming load: the gradient copies are read exactly once
__device__ __forceinline__ float4 ld_stream(const float* p) { return load_stream4(p); }

// W and Mom of a layer of at least this many keys are read and written with the streaming hint as well.
// Below it, leaving them to the caches is faster (W + Mom of such a layer, 8 bytes per key, fit the 256 MB
// last-level cache beside the gradient copies streaming past); above it the hint is: measured at P = 8,
// 16.8 M keys 83.8 % of 8 TB/s cached against 75.2 % streamed, 20 M 73.2 / 75.1, 37.7 M 70.0 / 73.8,
// 89.5 M 67.8 / 70.5.
constexpr int64_t kDenseStreamKeys = 19000000;

// keys [lo, hi) of one layer; PC > 0: number of copies known at compile time; stream: W / Mom streamed
// (the same for every lane of the launch's layer: a uniform branch around each access)
template <int PC>
__device__ __forceinline__ void dense_span(const float* const* __restrict__ G, int P, float* __restrict__ W,
                                           float* __restrict__ Mom, int64_t lo, int64_t hi, float lr, float mu, float wd, bool stream)
{
    const int nP = PC > 0 ? PC : P;
    // W, Mom and every G[p] are 16-byte aligned, so key i is float4-aligned iff i % 4 == 0
    int64_t lo4 = (lo + 3) & ~int64_t(3);
    if (lo4 > hi) lo4 = hi;
    const int64_t hi4 = lo4 + ((hi - lo4) & ~int64_t(3));

    int64_t idx[kDenseUnroll];
    float4 acc[kDenseUnroll], w[kDenseUnroll], m[kDenseUnroll];
#pragma unroll
    for (int u = 0; u < kDenseUnroll; ++u) {
        idx[u] = lo4 + (int64_t(u) * kDenseThreads + threadIdx.x) * 4;
        if (idx[u] < hi4) {
            if constexpr (PC > 0) {
                float4 g[PC];
#pragma unroll
                for (int p = 0; p < PC; ++p) g[p] = ld_stream(G[p] + idx[u]);
                w[u] = stream ? load_stream4(W + idx[u]) : *reinterpret_cast<const float4*>(W + idx[u]);
                m[u] = stream ? load_stream4(Mom + idx[u]) : *reinterpret_cast<const float4*>(Mom + idx[u]);
                acc[u] = g[0];
#pragma unroll
                for (int p = 1; p < PC; ++p) {
                    acc[u].x += g[p].x; acc[u].y += g[p].y; acc[u].z += g[p].z; acc[u].w += g[p].w;
                }
            } else {
                w[u] = stream ? load_stream4(W + idx[u]) : *reinterpret_cast<const float4*>(W + idx[u]);
                m[u] = stream ? load_stream4(Mom + idx[u]) : *reinterpret_cast<const float4*>(Mom + idx[u]);
                acc[u] = ld_stream(G[0] + idx[u]);
                for (int p = 1; p < nP; ++p) {
                    const float4 g = ld_stream(G[p] + idx[u]);
                    acc[u].x += g.x; acc[u].y += g.y; acc[u].z += g.z; acc[u].w += g.w;
                }
            }
        }
    }
#pragma unroll
    for (int u = 0; u < kDenseUnroll; ++u) {
        if (idx[u] < hi4) {
            upd(acc[u].x, w[u].x, m[u].x, lr, mu, wd);
            upd(acc[u].y, w[u].y, m[u].y, lr, mu, wd);
            upd(acc[u].z, w[u].z, m[u].z, lr, mu, wd);
            upd(acc[u].w, w[u].w, m[u].w, lr, mu, wd);
            if (stream) {
                store_stream4(Mom + idx[u], m[u]);
                store_stream4(W + idx[u], w[u]);
            } else {
                *reinterpret_cast<float4*>(Mom + idx[u]) = m[u];
                *reinterpret_cast<float4*>(W + idx[u]) = w[u];
            }
        }
    }
    // at most 3 unaligned keys at each end of the span
    const int nh = static_cast<int>(lo4 - lo), nt = static_cast<int>(hi - hi4);
    const int t = threadIdx.x;
    if (t < nh + nt) {
        const int64_t i = t < nh ? lo + t : hi4 + (t - nh);
        float g = G[0][i];
        for (int p = 1; p < nP; ++p) g += G[p][i];
        float wv = W[i], mv = Mom[i];
        upd(g, wv, mv, lr, mu, wd);
        Mom[i] = mv;
        W[i] = wv;
    }
}

__device__ __forceinline__ void dense_block(const float* const* G, int P, float* W, float* Mom, int64_t q, int64_t r, int S,
                                            int chunks, int local_block, float lr, float mu, float wd)
{
    const int s = local_block / chunks;
    const int64_t c = local_block % chunks;
    // shard s owns [floor(s n / S), floor((s+1) n / S)).  With n = q S + r this is s q + floor(s r / S):
    // exact, and for S < 2^16 the division is a cheap 32-bit one (a 64-bit division per workgroup
    // costs a measurable share of a workgroup that only lives for about a microsecond); q and r come
    // from the host
    int64_t begin, end;
    if (S < (1 << 16)) {
        const uint32_t rr = static_cast<uint32_t>(r), su = static_cast<uint32_t>(s), Su = static_cast<uint32_t>(S);
        begin = int64_t(s) * q + (su * rr) / Su;
        end = int64_t(s + 1) * q + ((su + 1u) * rr) / Su;
    } else {
        begin = int64_t(s) * q + (int64_t(s) * r) / S;
        end = int64_t(s + 1) * q + (int64_t(s + 1) * r) / S;
    }
    const int64_t lo = begin + c * kDenseChunk;
    if (lo >= end) return;
    const int64_t hi = lo + kDenseChunk < end ? lo + kDenseChunk : end;
    const bool stream = q * S + r >= kDenseStreamKeys;       // n = q S + r
    switch (P) {
        case 8: dense_span<8>(G, P, W, Mom, lo, hi, lr, mu, wd, stream); break;
        case 4: dense_span<4>(G, P, W, Mom, lo, hi, lr, mu, wd, stream); break;
        case 2: dense_span<2>(G, P, W, Mom, lo, hi, lr, mu, wd, stream); break;
        case 16: dense_span<16>(G, P, W, Mom, lo, hi, lr, mu, wd, stream); break;
        default: dense_span<0>(G, P, W, Mom, lo, hi, lr, mu, wd, stream); break;
    }
}

__global__ void __launch_bounds__(kDenseThreads) dense_ps_table_kernel(const DenseTable t, float lr, float mu, float wd)
{
    // which layer does this workgroup belong to (at most 16 segments: linear scan)
    int l = 0;
    const int b = blockIdx.x;
    for (int j = 1; j < t.L; ++j)
        if (b >= t.seg[j].block_begin) l = j;
    const DenseSeg& sg = t.seg[l];
    dense_block(sg.G, sg.P, sg.W, sg.Mom, sg.q, sg.r, sg.S, sg.chunks, b - sg.block_begin, lr, mu, wd);
}

__global__ void __launch_bounds__(kDenseThreads) dense_ps_wide_kernel(const DenseWide a, float lr, float mu, float wd)
{
    dense_block(a.G, a.P, a.W, a.Mom, a.q, a.r, a.S, a.chunks, blockIdx.x, lr, mu, wd);
}

}  // namespace

psd_status launch_dense_table(const DenseTable& t, int32_t total_blocks, float lr, float mu, float wd, hipStream_t st)
{
    hipLaunchKernelGGL(dense_ps_table_kernel, dim3(total_blocks), dim3(kDenseThreads), 0, st, t, lr, mu, wd);
    PSD_HIP_TRY(hipGetLastError());
    return PSD_OK;
}

psd_status launch_dense_wide(const DenseWide& a, float lr, float mu, float wd, hipStream_t st)
{
    const int64_t blocks = int64_t(a.chunks) * a.S;
    if (blocks < 1 || blocks > (int64_t(1) << 30)) return PSD_E_INVALID;
    hipLaunchKernelGGL(dense_ps_wide_kernel, dim3(static_cast<uint32_t>(blocks)), dim3(kDenseThreads), 0, st, a, lr, mu, wd);
    PSD_HIP_TRY(hipGetLastError());
    return PSD_OK;
}

// Second stage of a split reconstruction: the `splits` partial dW matrices are exactly "several dense
// copies of one gradient", so the parameter-server kernel sums them (in split order) and updates.
psd_status launch_sfb_reduce(const float* part, int splits, int64_t N, int64_t M, float* W, float* Mom, float lr,
                             float mu, float wd, hipStream_t st)
{
    DenseWide a;
    for (int p = 0; p < PSD_MAX_WORKERS; ++p) a.G[p] = p < splits ? part + p * sfb_part_stride(N, M) : nullptr;
    a.W = W; a.Mom = Mom; a.n = N * M; a.P = splits; a.S = 1;
    a.q = a.n; a.r = 0;
    a.chunks = dense_chunks_for(a.n, 1);
    return launch_dense_wide(a, lr, mu, wd, st);
}

}  // namespace psd
