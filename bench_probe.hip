// Hardware probes behind the design notes (measurement harness, not part of the library; nothing of the
// method is computed here).  Build and run on an MI355X:
//     hipcc --offload-arch=gfx950 -O3 -Xclang -target-feature -Xclang -packed-fp32-ops bench_probe.hip -o bench_probe
//     ./bench_probe stream          # bare streams: what HBM gives a "P reads + read-modify-write of two arrays" pattern
//     ./bench_probe coresident      # MFMA-only workgroups and streaming workgroups sharing the compute units
//     ./bench_probe xcd             # the same read-modify-write stream from the CUs of 1, 2, 4 or all 8 XCDs only
// Every access is bounds-checked by construction (fixed sizes below); every loop has a fixed trip count.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <vector>

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e), __LINE__); exit(1); } } while (0)

// ---------------------------------------------------------------------------------------------------
// stream: out[i] (two arrays, read-modify-write) from P read-only arrays, no shard logic, 2 x 16 bytes per lane
// ---------------------------------------------------------------------------------------------------
struct Ptrs { const float* g[8]; };

// NT: W and Mom are read and written with the streaming (non-temporal) hint as well, like the P read-only arrays
template <int P, bool NT>
__global__ void __launch_bounds__(256) stream_kernel(Ptrs in, float* __restrict__ W, float* __restrict__ Mom, size_t n4)
{
    const size_t base = size_t(blockIdx.x) * 512 + threadIdx.x;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const size_t i = base + u * 256;
        if (i >= n4) continue;
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int p = 0; p < P; ++p) acc += __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(in.g[p]) + i);
        f32x4 w, m;
        if constexpr (NT) {
            w = __builtin_nontemporal_load(reinterpret_cast<f32x4*>(W) + i);
            m = __builtin_nontemporal_load(reinterpret_cast<f32x4*>(Mom) + i);
        } else {
            w = reinterpret_cast<f32x4*>(W)[i];
            m = reinterpret_cast<f32x4*>(Mom)[i];
        }
        m = 0.9f * m + 0.01f * acc;
        w = w - m;
        if constexpr (NT) {
            __builtin_nontemporal_store(m, reinterpret_cast<f32x4*>(Mom) + i);
            __builtin_nontemporal_store(w, reinterpret_cast<f32x4*>(W) + i);
        } else {
            reinterpret_cast<f32x4*>(Mom)[i] = m;
            reinterpret_cast<f32x4*>(W)[i] = w;
        }
    }
}

template <int P, bool NT>
static void run_stream(size_t n, hipEvent_t e0, hipEvent_t e1)
{
    const int sets = 2;
    std::vector<Ptrs> in(sets);
    std::vector<float*> W(sets), Mom(sets);
    for (int s = 0; s < sets; ++s) {
        for (int p = 0; p < 8; ++p) { float* x = nullptr; if (p < P) { CK(hipMalloc(&x, n * 4)); CK(hipMemset(x, 0, n * 4)); } in[s].g[p] = x; }
        CK(hipMalloc(&W[s], n * 4)); CK(hipMalloc(&Mom[s], n * 4)); CK(hipMemset(W[s], 0, n * 4)); CK(hipMemset(Mom[s], 0, n * 4));
    }
    const size_t n4 = n / 4;
    const unsigned grid = static_cast<unsigned>((n4 + 511) / 512);
    for (int i = 0; i < 60; ++i) stream_kernel<P, NT><<<grid, 256>>>(in[i % sets], W[i % sets], Mom[i % sets], n4);
    CK(hipDeviceSynchronize());
    float best = 1e30f, sum = 0;
    for (int rep = 0; rep < 5; ++rep) {
        CK(hipEventRecord(e0));
        for (int i = 0; i < 20; ++i) stream_kernel<P, NT><<<grid, 256>>>(in[i % sets], W[i % sets], Mom[i % sets], n4);
        CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
        float ms; CK(hipEventElapsedTime(&ms, e0, e1)); ms /= 20; sum += ms; if (ms < best) best = ms;
    }
    const double bytes = double(n) * (4.0 * P + 16.0);
    printf("  P = %d reads + W/Mom read-modify-write (%s), %10zu keys: mean %8.1f us = %6.0f GB/s (%.1f %% of 8 TB/s), best %8.1f us\n",
           P, NT ? "W/Mom streamed" : "W/Mom cached  ", n, sum / 5 * 1e3, bytes / (sum / 5) / 1e6, bytes / (sum / 5) / 1e6 / 80.0, best * 1e3);
    for (int s = 0; s < sets; ++s) { for (int p = 0; p < P; ++p) CK(hipFree(const_cast<float*>(in[s].g[p]))); CK(hipFree(W[s])); CK(hipFree(Mom[s])); }
}

// ---------------------------------------------------------------------------------------------------
// coresident: workgroups [0, n_mfma) issue MFMAs from registers (no memory access at all), the others stream
// ---------------------------------------------------------------------------------------------------
struct Rec { unsigned hwid, xcc; long long t0, t1, cyc; };
constexpr size_t N4 = 147456;     // float4 per array per streaming workgroup (576 steps of 256 lanes)

__global__ void __launch_bounds__(256, 2) mixed(const uint4* in, float* out, float* __restrict__ W, float* __restrict__ Mom,
                                                int iters, int n_mfma, int kind, Rec* rec)
{
    extern __shared__ float dummy[];     // 70000 bytes asked for at launch: at most two workgroups per CU
    const long long w0 = wall_clock64(), c0 = clock64();
    if (static_cast<int>(blockIdx.x) < n_mfma) {
        bf16x8 a[4], b[2];
        for (int i = 0; i < 4; ++i) a[i] = __builtin_bit_cast(bf16x8, in[(threadIdx.x * 8 + i) % 4096]);
        for (int i = 0; i < 2; ++i) b[i] = __builtin_bit_cast(bf16x8, in[(threadIdx.x * 8 + 4 + i) % 4096]);
        f32x16 acc[8];
        for (int i = 0; i < 8; ++i) for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
        for (int it = 0; it < iters; ++it)
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i % 4], b[i / 4], acc[i], 0, 0, 0);
        float s = 0;
        for (int i = 0; i < 8; ++i) for (int r = 0; r < 16; ++r) s += acc[i][r];
        out[blockIdx.x * 256 + threadIdx.x] = s;
    } else {
        const size_t wg = blockIdx.x - n_mfma;                          // < 256: its own slice of W and Mom
        float4* w4 = reinterpret_cast<float4*>(W) + wg * N4;
        float4* m4 = reinterpret_cast<float4*>(Mom) + wg * N4;
        float4 sum = make_float4(0, 0, 0, 0);
        for (size_t i = threadIdx.x; i < N4; i += 256 * 4) {            // N4 = 144 * 1024: i + 768 < N4
            float4 w[4], m[4];
            if (kind != 2) {
#pragma unroll
                for (int u = 0; u < 4; ++u) { w[u] = w4[i + u * 256]; m[u] = m4[i + u * 256]; }
            } else {
#pragma unroll
                for (int u = 0; u < 4; ++u) { w[u] = make_float4(i, u, 1, 2); m[u] = make_float4(u, i, 3, 4); }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                m[u].x = 0.9f * m[u].x + 0.01f; m[u].y = 0.9f * m[u].y + 0.01f; m[u].z = 0.9f * m[u].z + 0.01f; m[u].w = 0.9f * m[u].w + 0.01f;
                w[u].x -= m[u].x; w[u].y -= m[u].y; w[u].z -= m[u].z; w[u].w -= m[u].w;
                if (kind != 1) { m4[i + u * 256] = m[u]; w4[i + u * 256] = w[u]; }
                else { sum.x += w[u].x; sum.y += w[u].y; sum.z += m[u].z; sum.w += m[u].w; }
            }
        }
        if (kind == 1 && sum.x == 12345.678f) out[threadIdx.x] = sum.y + sum.z + sum.w;
    }
    if (iters < 0) dummy[threadIdx.x] = 0;
    __syncthreads();
    if (threadIdx.x == 0) {
        Rec r;
        r.hwid = __builtin_amdgcn_s_getreg((31 << 11) | (0 << 6) | 4);      // HW_ID: wave, SIMD, CU, SH, SE
        r.xcc = __builtin_amdgcn_s_getreg((31 << 11) | (0 << 6) | 20);      // XCC_ID
        r.t0 = w0; r.t1 = wall_clock64(); r.cyc = clock64() - c0;
        rec[blockIdx.x] = r;
    }
}

static void run_coresident(hipEvent_t e0, hipEvent_t e1)
{
    std::vector<unsigned> hr(4096 * 4), hz(4096 * 4, 0); srand(1);
    for (auto& x : hr) { unsigned lo = 0x3c00 + (rand() & 0x3ff), hi = 0xbc00 + (rand() & 0x3ff); x = lo | (hi << 16); }
    uint4 *dr, *dz; CK(hipMalloc(&dr, 4096 * 16)); CK(hipMemcpy(dr, hr.data(), 4096 * 16, hipMemcpyHostToDevice));
    CK(hipMalloc(&dz, 4096 * 16)); CK(hipMemcpy(dz, hz.data(), 4096 * 16, hipMemcpyHostToDevice));
    float* o; CK(hipMalloc(&o, 2048 * 256 * 4));
    const size_t n = 256 * N4 * 4;
    float *W, *Mom; CK(hipMalloc(&W, n * 4)); CK(hipMalloc(&Mom, n * 4)); CK(hipMemset(W, 0, n * 4)); CK(hipMemset(Mom, 0, n * 4));
    CK(hipFuncSetAttribute((const void*)mixed, hipFuncAttributeMaxDynamicSharedMemorySize, 140000));
    Rec* rec; CK(hipMalloc(&rec, 1024 * sizeof(Rec)));
    const int iters = 3000;
    const char* kn[3] = {"read+write", "read only", "write only"};
    struct Run { int n_mfma, n_str, kind, zero; };
    const Run runs[] = {{256, 0, 0, 0}, {256, 0, 0, 1}, {0, 256, 0, 0}, {0, 256, 1, 0}, {0, 256, 2, 0},
                        {256, 256, 0, 0}, {256, 256, 1, 0}, {256, 256, 2, 0}, {256, 256, 0, 1}};
    for (int rep = 0; rep < 3; ++rep)
        for (const Run& r : runs) {
            const int grid = r.n_mfma + r.n_str;
            float ms;
            CK(hipDeviceSynchronize()); CK(hipEventRecord(e0));
            mixed<<<grid, 256, 70000>>>(r.zero ? dz : dr, o, W, Mom, iters, r.n_mfma, r.kind, rec);
            CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1)); CK(hipEventElapsedTime(&ms, e0, e1));
            if (rep == 0) continue;                                     // first round: clocks settling
            std::vector<Rec> h(grid); CK(hipMemcpy(h.data(), rec, grid * sizeof(Rec), hipMemcpyDeviceToHost));
            long long tmin = h[0].t0; for (auto& x : h) if (x.t0 < tmin) tmin = x.t0;
            double md = 0, mc = 0, me = 0, sd = 0, se = 0;
            std::map<unsigned, int> cum, cus;
            for (int i = 0; i < grid; ++i) {
                const unsigned key = ((h[i].xcc & 15) << 16) | (h[i].hwid & 0xff00);
                if (i < r.n_mfma) { md += (h[i].t1 - h[i].t0) / 100.0; mc += h[i].cyc; me += (h[i].t1 - tmin) / 100.0; cum[key]++; }
                else { sd += (h[i].t1 - h[i].t0) / 100.0; se += (h[i].t1 - tmin) / 100.0; cus[key]++; }
            }
            int both = 0; for (auto& kv : cum) if (cus.count(kv.first)) ++both;
            printf("  mfma wgs %3d (%s data), stream wgs %3d (%-10s): %6.3f ms |", r.n_mfma, r.zero ? "zero  " : "random", r.n_str, r.n_str ? kn[r.kind] : "-", ms);
            if (r.n_mfma) printf(" MFMA wg: %6.1f us, ends at %6.1f, %4.0f MHz, %5.2f cycles per MFMA |", md / r.n_mfma, me / r.n_mfma, mc / md, mc / r.n_mfma / (iters * 8.0));
            if (r.n_str) printf(" stream wg: %6.1f us, ends at %6.1f |", sd / r.n_str, se / r.n_str);
            if (r.n_mfma && r.n_str) printf(" CUs holding one of each: %d", both);
            printf("\n");
        }
}

// ---------------------------------------------------------------------------------------------------
// xcd: every workgroup owns a slice of W and Mom; only those that find themselves on an XCD of the
// given set stream it (read-modify-write), the others leave at once.  What can ONE accelerator die
// pull from memory when the other seven are idle?
// ---------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256, 2) xcd_stream(float* __restrict__ W, float* __restrict__ Mom, unsigned xcd_set, Rec* rec)
{
    extern __shared__ float dummy[];     // 70000 bytes asked for at launch: at most two workgroups per CU
    const long long w0 = wall_clock64();
    const unsigned xcc = __builtin_amdgcn_s_getreg((31 << 11) | (0 << 6) | 20) & 15;
    const bool active = (xcd_set >> xcc) & 1;
    if (active) {
        float4* w4 = reinterpret_cast<float4*>(W) + size_t(blockIdx.x) * N4;       // blockIdx.x < 512: inside the arrays
        float4* m4 = reinterpret_cast<float4*>(Mom) + size_t(blockIdx.x) * N4;
        for (size_t i = threadIdx.x; i < N4; i += 256 * 4) {                       // N4 = 144 * 1024: i + 768 < N4
            float4 w[4], m[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) { w[u] = w4[i + u * 256]; m[u] = m4[i + u * 256]; }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                m[u].x = 0.9f * m[u].x + 0.01f; m[u].y = 0.9f * m[u].y + 0.01f; m[u].z = 0.9f * m[u].z + 0.01f; m[u].w = 0.9f * m[u].w + 0.01f;
                w[u].x -= m[u].x; w[u].y -= m[u].y; w[u].z -= m[u].z; w[u].w -= m[u].w;
                m4[i + u * 256] = m[u]; w4[i + u * 256] = w[u];
            }
        }
    }
    if (xcd_set == 0xffffffffu) dummy[threadIdx.x] = 0;
    __syncthreads();
    if (threadIdx.x == 0) {
        Rec r;
        r.hwid = __builtin_amdgcn_s_getreg((31 << 11) | (0 << 6) | 4);
        r.xcc = xcc | (active ? 0x100 : 0);
        r.t0 = w0; r.t1 = wall_clock64(); r.cyc = 0;
        rec[blockIdx.x] = r;
    }
}

static void run_xcd(hipEvent_t e0, hipEvent_t e1)
{
    const int max_grid = 512;
    const size_t n = size_t(max_grid) * N4 * 4;
    float *W, *Mom; CK(hipMalloc(&W, n * 4)); CK(hipMalloc(&Mom, n * 4)); CK(hipMemset(W, 0, n * 4)); CK(hipMemset(Mom, 0, n * 4));
    CK(hipFuncSetAttribute((const void*)xcd_stream, hipFuncAttributeMaxDynamicSharedMemorySize, 140000));
    Rec* rec; CK(hipMalloc(&rec, max_grid * sizeof(Rec)));
    const unsigned sets[] = {0xff, 0x01, 0x10, 0x03, 0x0f, 0x55, 0xff};
    for (int grid : {256, 512})
        for (int rep = 0; rep < 2; ++rep)
            for (unsigned set : sets) {
                float ms;
                CK(hipDeviceSynchronize()); CK(hipEventRecord(e0));
                xcd_stream<<<grid, 256, 70000>>>(W, Mom, set, rec);
                CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1)); CK(hipEventElapsedTime(&ms, e0, e1));
                if (rep == 0) continue;                                  // first round: clocks settling
                std::vector<Rec> h(grid); CK(hipMemcpy(h.data(), rec, grid * sizeof(Rec), hipMemcpyDeviceToHost));
                int active = 0; long long t0 = 0, t1 = 0; std::map<unsigned, int> cus;
                for (auto& x : h) if (x.xcc & 0x100) {
                    if (!active || x.t0 < t0) t0 = x.t0;
                    if (!active || x.t1 > t1) t1 = x.t1;
                    ++active; cus[((x.xcc & 15) << 16) | (x.hwid & 0xff00)]++;
                }
                const double us = (t1 - t0) / 100.0, bytes = double(active) * N4 * 16 * 4;      // two arrays, read and written
                int nx = 0; for (int b = 0; b < 8; ++b) nx += (set >> b) & 1;
                printf("  XCD set 0x%02x (%d XCDs), %3d workgroups launched: %3d stream on %3d CUs, %7.1f us from first start to last end = %6.0f GB/s, %5.0f GB/s per XCD (event time %7.1f us)\n",
                       set, nx, grid, active, (int)cus.size(), us, bytes / us / 1e3, bytes / us / 1e3 / nx, ms * 1e3);
            }
}

int main(int argc, char** argv)
{
    hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    const char* what = argc > 1 ? argv[1] : "stream";
    if (!strcmp(what, "stream")) {
        printf("bare streams (two rotating buffer sets, 20 launches per timing, mean of 5):\n");
        for (size_t n : {size_t(2332704), size_t(16777216), size_t(37748736), size_t(89460736)}) {
            run_stream<8, false>(n, e0, e1);
            run_stream<8, true>(n, e0, e1);
        }
        run_stream<0, false>(37748736, e0, e1);
        run_stream<0, true>(37748736, e0, e1);
        run_stream<1, false>(37748736, e0, e1);
        run_stream<4, false>(37748736, e0, e1);
        run_stream<4, true>(37748736, e0, e1);
    } else if (!strcmp(what, "coresident")) {
        printf("one launch, two kinds of workgroups (each 256 lanes, at most two per CU); times per workgroup from the 100 MHz clock:\n");
        run_coresident(e0, e1);
    } else if (!strcmp(what, "xcd")) {
        printf("read-modify-write stream of two arrays (2.36 MB per array and workgroup) from the CUs of a subset of the XCDs:\n");
        run_xcd(e0, e1);
    } else {
        printf("usage: bench_probe stream|coresident|xcd\n");
        return 2;
    }
    return 0;
}
