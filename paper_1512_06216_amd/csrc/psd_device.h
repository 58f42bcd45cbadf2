// Device-side helpers shared by the kernels of libpsd (not installed).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace psd {

typedef int i32x4 __attribute__((ext_vector_type(4)));

// The update of Algorithm 3's update line with the momentum / weight-decay reading of Lambda
// (Section 3.3, Eq. 3-4):  Mom <- mu*Mom + lr*(d + wd*w) ;  w <- w - Mom.
// The ONE place this arithmetic lives: every kernel (fp32 / bf16 reconstruction, dense
// parameter-server sum, bias) calls it, so the routes cannot drift apart.
__device__ __forceinline__ void upd(float d, float& w, float& mo, float lr, float mu, float wd)
{
    mo = __fmaf_rn(mu, mo, lr * __fmaf_rn(wd, w, d));   // wd = 0 leaves d unchanged
    w = w - mo;
}

// Streaming ("non-temporal") accesses for data that is touched exactly once per launch -- W and Mom in
// every update, the gradient copies of the parameter-server sum.  Without the hint every W / Mom line is
// allocated in the XCD's 4 MB L2 on its way through and the update leaves the L2 full of dirty lines; the
// factor fetches of the workgroups that are in their MFMA loop then have those write-backs on their miss
// path.  Measured on the bf16 reconstruction: the hint on both the loads and the stores takes fc6 from
// 220 to 198 us and the 4096 -> 1000 layer from 38 to 31 us while the bytes that cross the L2 / fabric
// boundary stay the same (636 against 630 MB) and the mean L1 -> L2 read latency falls from 477 to 404
// cycles (either hint alone: no gain; the scope bits sc0 / sc1 on top: slower).  Only for accesses that
// cover whole cache lines: streamed stores to parts of a line are expensive.
typedef float f32x4_nt __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 load_stream4(const float* p)
{
    const f32x4_nt v = __builtin_nontemporal_load(reinterpret_cast<const f32x4_nt*>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store_stream4(float* p, float4 x)
{
    const f32x4_nt v = {x.x, x.y, x.z, x.w};
    __builtin_nontemporal_store(v, reinterpret_cast<f32x4_nt*>(p));
}

// global -> LDS without registers, 16 bytes per lane: lane i's chunk lands at
// lds_addr_uniform + 16*i.  A lane whose offset is at or past the descriptor's size writes zeros.
// The statement overwrites m0.  m0 cannot be named as a clobber (the compiler reserves it, ignores it
// in clobber lists and warns); that is safe here because the compiler sets m0 itself right before
// each of its own uses and the kernels that call this contain no such use (no LDS-DMA builtin, no
// indexed register moves, no message sends).
__device__ __forceinline__ void dma_b128(uint32_t lds_addr_uniform, uint32_t voff, i32x4 rsrc)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :
                 : "s"(lds_addr_uniform), "v"(voff), "s"(rsrc)
                 : "memory");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N <= 63, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

// A pointer every lane holds alike, moved to scalar registers (buffer descriptors live there).
template <class T>
__device__ __forceinline__ const T* uniform_ptr(const T* p)
{
    const uint64_t a = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(a));
    const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(a >> 32));
    return reinterpret_cast<const T*>((static_cast<uint64_t>(hi) << 32) | lo);
}

// Raw buffer descriptor over `bytes` bytes at X (stride 0: byte-granular range check).
__device__ __forceinline__ i32x4 raw_rsrc(const void* X, uint32_t bytes)
{
    const uint64_t a = reinterpret_cast<uint64_t>(X);
    i32x4 r;
    r.x = static_cast<int>(a & 0xffffffffu);
    r.y = static_cast<int>((a >> 32) & 0xffffu);
    r.z = static_cast<int>(bytes);
    r.w = 0x00020000;
    return r;
}

// Scheduling pattern for one pipeline phase holding MF MFMAs and R LDS reads that do not depend
// on each other: 1 MFMA, then its share of the reads, and so on.
template <int R, int MF, int I = 0>
__device__ __forceinline__ void interleave_groups()
{
    if constexpr (I < MF) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                    // one MFMA
        constexpr int n = R * (I + 1) / MF - R * I / MF;
        if constexpr (n > 0) __builtin_amdgcn_sched_group_barrier(0x100, n, 0);  // n DS reads
        interleave_groups<R, MF, I + 1>();
    }
}

// The same with V vector-memory loads spread over the phase as well.
template <int R, int V, int MF, int I = 0>
__device__ __forceinline__ void interleave_groups_vmem()
{
    if constexpr (I < MF) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        constexpr int n = R * (I + 1) / MF - R * I / MF;
        if constexpr (n > 0) __builtin_amdgcn_sched_group_barrier(0x100, n, 0);
        constexpr int v = V * (I + 1) / MF - V * I / MF;
        if constexpr (v > 0) __builtin_amdgcn_sched_group_barrier(0x020, v, 0);  // v VMEM reads
        interleave_groups_vmem<R, V, MF, I + 1>();
    }
}

}  // namespace psd
