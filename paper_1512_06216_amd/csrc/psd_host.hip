// Host side of libpsd: route selection, shard ranges, argument validation and the
// per-iteration issue order.  No device code here.
#include <atomic>
#include "psd_internal.h"

namespace psd {
static thread_local int32_t g_last_hip_error = 0;
psd_status hip_failed(hipError_t e)
{
    g_last_hip_error = static_cast<int32_t>(e);
    return PSD_E_HIP;
}

static std::atomic<int> g_tune[PSD_TUNE_COUNT_] = {{-1}, {-1}, {-1}};
int tune_value(int knob) { return knob >= 0 && knob < PSD_TUNE_COUNT_ ? g_tune[knob].load(std::memory_order_relaxed) : -1; }

int device_cu_count()
{
    constexpr int kMaxDev = 64;
    static std::atomic<int> cached[kMaxDev];          // 0 = not queried yet
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDev) return 256;
    int cus = cached[dev].load(std::memory_order_relaxed);
    if (cus == 0) {
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
        cached[dev].store(cus, std::memory_order_relaxed);
    }
    return cus;
}
}  // namespace psd

using namespace psd;

namespace {

// a*b, reporting overflow of 64-bit unsigned arithmetic
inline bool mul_u64(uint64_t a, uint64_t b, uint64_t* out) { return __builtin_mul_overflow(a, b, out); }
inline bool add_u64(uint64_t a, uint64_t b, uint64_t* out) { return __builtin_add_overflow(a, b, out); }

inline size_t elem_size(int32_t dtype) { return dtype == PSD_BF16 ? 2 : 4; }

bool valid_plan_sizes(const psd_plan* p)
{
    return p->M >= 1 && p->N >= 1 && p->B >= 1 && p->P >= 1 && p->P <= PSD_MAX_WORKERS &&
           p->M < (int64_t(1) << 31) && p->N < (int64_t(1) << 31) &&
           p->B * p->P < (int64_t(1) << 31);
}

bool valid_ld(int64_t ld, int64_t cols, int32_t dtype)
{
    return ld >= cols && ld < (int64_t(1) << 31) && (static_cast<uint64_t>(ld) * elem_size(dtype)) % 16 == 0;
}

}  // namespace

extern "C" {

int32_t psd_version(void) { return 2; }

psd_status psd_tune_set(int32_t knob, int32_t value)
{
    if (knob < 0 || knob >= PSD_TUNE_COUNT_) return PSD_E_INVALID;
    const int32_t limit = knob == PSD_TUNE_SFB_BF16_SKEW_US ? 200 : 2;
    const int32_t low = knob == PSD_TUNE_SFB_F32_TILE ? 1 : 0;
    if (value != -1 && (value < low || value > limit)) return PSD_E_INVALID;
    g_tune[knob].store(value, std::memory_order_relaxed);
    return PSD_OK;
}

int32_t psd_last_hip_error(void) { return g_last_hip_error; }

const char* psd_status_string(psd_status s)
{
    switch (s) {
        case PSD_OK: return "ok";
        case PSD_E_INVALID: return "invalid argument (size, enum, alignment or leading dimension)";
        case PSD_E_NULL: return "null pointer";
        case PSD_E_UNSUPPORTED: return "unsupported request";
        case PSD_E_OVERFLOW: return "communication volume overflows 64 bits";
        case PSD_E_HIP: return "HIP call failed (see psd_last_hip_error)";
        case PSD_E_WORKSPACE: return "workspace smaller than psd_sfb_workspace_bytes asks for";
        default: return "unknown status";
    }
}

// Algorithm 3 with the three volumes of Section 4.3.1.
psd_status psd_plan_layer(int32_t kind, int64_t M, int64_t N, int64_t B, int64_t P, psd_plan* out)
{
    if (!out) return PSD_E_NULL;
    if (kind != PSD_LAYER_CONV && kind != PSD_LAYER_FC) return PSD_E_INVALID;
    if (M < 1 || N < 1 || B < 1 || P < 1 || P > PSD_MAX_WORKERS) return PSD_E_INVALID;
    const uint64_t m = M, n = N, b = B, p = P;
    uint64_t mn_sum, mn_prod, t, sfb, dense, sfps, pb_sum;
    if (add_u64(m, n, &mn_sum) || mul_u64(m, n, &mn_prod)) return PSD_E_OVERFLOW;
    // (P-1)^2 * B * (M+N)
    if (mul_u64((p - 1) * (p - 1), b, &t) || mul_u64(t, mn_sum, &sfb)) return PSD_E_OVERFLOW;
    // 2 * P * M * N
    if (mul_u64(2 * p, mn_prod, &dense)) return PSD_E_OVERFLOW;
    // P*B*(M+N) + P*M*N
    if (mul_u64(p, b, &t) || mul_u64(t, mn_sum, &pb_sum) || mul_u64(p, mn_prod, &t) ||
        add_u64(pb_sum, t, &sfps))
        return PSD_E_OVERFLOW;
    out->M = M; out->N = N; out->B = B; out->P = P;
    out->kind = kind;
    out->reserved = 0;
    out->cost_sfb = sfb; out->cost_ps_dense = dense; out->cost_sf_ps = sfps;
    if (kind == PSD_LAYER_CONV) {
        out->route_alg3 = PSD_ROUTE_PS_DENSE;
        out->route_vs_dense = PSD_ROUTE_PS_DENSE;
    } else {
        out->route_alg3 = (sfb <= sfps) ? PSD_ROUTE_SFB : PSD_ROUTE_SF_PS;       // tie -> SFB
        out->route_vs_dense = (sfb <= dense) ? PSD_ROUTE_SFB : PSD_ROUTE_PS_DENSE;
    }
    return PSD_OK;
}

psd_status psd_shard_range(int64_t n, int32_t S, int32_t s, int64_t* begin, int64_t* end)
{
    if (!begin || !end) return PSD_E_NULL;
    if (n < 1 || S < 1 || S > n || s < 0 || s >= S) return PSD_E_INVALID;
    *begin = static_cast<int64_t>((static_cast<__int128>(s) * n) / S);
    *end = static_cast<int64_t>((static_cast<__int128>(s + 1) * n) / S);
    return PSD_OK;
}

int64_t psd_factor_ld(int64_t cols, int32_t dtype)
{
    if (cols < 1 || (dtype != PSD_F32 && dtype != PSD_BF16)) return 0;
    const int64_t q = dtype == PSD_BF16 ? 64 : 32;      // 128 bytes
    return (cols + q - 1) / q * q;
}

psd_status psd_pack_factors(const psd_plan* plan, const float* const* delta_p, const float* const* act_p,
                            int32_t out_dtype, void* U, int64_t ldu, void* V, int64_t ldv, void* stream)
{
    if (!plan || !delta_p || !act_p || !U || !V) return PSD_E_NULL;
    if (out_dtype != PSD_F32 && out_dtype != PSD_BF16) return PSD_E_INVALID;
    if (!valid_plan_sizes(plan)) return PSD_E_INVALID;
    if (!valid_ld(ldu, plan->N, out_dtype) || !valid_ld(ldv, plan->M, out_dtype)) return PSD_E_INVALID;
    if (!aligned16(U) || !aligned16(V)) return PSD_E_INVALID;
    for (int64_t p = 0; p < plan->P; ++p) {
        if (!delta_p[p] || !act_p[p]) return PSD_E_NULL;
        if (!aligned16(delta_p[p]) || !aligned16(act_p[p])) return PSD_E_INVALID;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    PackArgs a;
    a.P = static_cast<int32_t>(plan->P);
    a.B = plan->B;
    for (int p = 0; p < PSD_MAX_WORKERS; ++p) {
        a.u.src[p] = p < a.P ? delta_p[p] : nullptr;
        a.v.src[p] = p < a.P ? act_p[p] : nullptr;
    }
    a.u.dst = U; a.u.cols = plan->N; a.u.ld = ldu;
    a.v.dst = V; a.v.cols = plan->M; a.v.ld = ldv;
    return launch_pack(a, out_dtype, st);          // one launch stacks both matrices
}

size_t psd_sfb_workspace_bytes(const psd_plan* plan, int32_t factor_dtype)
{
    if (!plan || !valid_plan_sizes(plan) || (factor_dtype != PSD_F32 && factor_dtype != PSD_BF16)) return 0;
    const int64_t K = plan->P * plan->B;
    const int splits = factor_dtype == PSD_F32 ? sfb_f32_splits(plan->N, plan->M, K) : sfb_bf16_splits(plan->N, plan->M, K);
    if (splits <= 1) return 0;
    return static_cast<size_t>(splits) * static_cast<size_t>(sfb_part_stride(plan->N, plan->M)) * sizeof(float);
}

psd_status psd_sync_fc_sfb(const psd_plan* plan, int32_t factor_dtype, const void* U, int64_t ldu,
                           const void* V, int64_t ldv, float* W, float* Mom, float lr, float mu, float wd,
                           void* workspace, size_t workspace_bytes, void* stream)
{
    if (!plan || !U || !V || !W || !Mom) return PSD_E_NULL;
    if (factor_dtype != PSD_F32 && factor_dtype != PSD_BF16) return PSD_E_INVALID;
    if (!(wd >= 0.0f)) return PSD_E_INVALID;          // also rejects NaN
    if (!valid_plan_sizes(plan)) return PSD_E_INVALID;
    if (!valid_ld(ldu, plan->N, factor_dtype) || !valid_ld(ldv, plan->M, factor_dtype)) return PSD_E_INVALID;
    if (!aligned16(U) || !aligned16(V) || !aligned16(W) || !aligned16(Mom)) return PSD_E_INVALID;
    if (W == Mom) return PSD_E_INVALID;
    // no workspace: one workgroup per tile over all of K.  A workspace: the split the query sized it for.
    int splits = 1;
    if (workspace_bytes != 0) {
        if (!workspace) return PSD_E_NULL;
        if (!aligned16(workspace)) return PSD_E_INVALID;
        const size_t need = psd_sfb_workspace_bytes(plan, factor_dtype);
        if (workspace_bytes < need) return PSD_E_WORKSPACE;
        if (need != 0) splits = static_cast<int>(need / (static_cast<size_t>(sfb_part_stride(plan->N, plan->M)) * sizeof(float)));
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int64_t K = plan->P * plan->B;
    float* part = splits > 1 ? static_cast<float*>(workspace) : nullptr;
    if (factor_dtype == PSD_F32)
        return launch_sfb_f32(static_cast<const float*>(U), ldu, static_cast<const float*>(V), ldv, W, Mom,
                              plan->N, plan->M, K, lr, mu, wd, part, splits, st);
    return launch_sfb_bf16(static_cast<const uint16_t*>(U), ldu, static_cast<const uint16_t*>(V), ldv, W, Mom,
                           plan->N, plan->M, K, lr, mu, wd, part, splits, st);
}

int32_t psd_sfb_blocks_supported(const psd_plan* plan, int32_t factor_dtype, int64_t ldu, int64_t ldv)
{
    if (!plan || !valid_plan_sizes(plan) || (factor_dtype != PSD_F32 && factor_dtype != PSD_BF16)) return 0;
    if (!valid_ld(ldu, plan->N, factor_dtype) || !valid_ld(ldv, plan->M, factor_dtype)) return 0;
    return (factor_dtype == PSD_F32 ? sfb_f32_blocks_supported(plan->B) : sfb_bf16_blocks_supported(plan->B)) ? 1 : 0;
}

psd_status psd_sync_fc_sfb_blocks(const psd_plan* plan, int32_t factor_dtype, const void* const* U_p, int64_t ldu,
                                  const void* const* V_p, int64_t ldv, float* W, float* Mom, float lr, float mu,
                                  float wd, void* stream)
{
    if (!plan || !U_p || !V_p || !W || !Mom) return PSD_E_NULL;
    if (factor_dtype != PSD_F32 && factor_dtype != PSD_BF16) return PSD_E_INVALID;
    if (!(wd >= 0.0f)) return PSD_E_INVALID;          // also rejects NaN
    if (!valid_plan_sizes(plan)) return PSD_E_INVALID;
    if (!aligned16(W) || !aligned16(Mom) || W == Mom) return PSD_E_INVALID;
    for (int64_t p = 0; p < plan->P; ++p) {
        if (!U_p[p] || !V_p[p]) return PSD_E_NULL;
        if (!aligned16(U_p[p]) || !aligned16(V_p[p])) return PSD_E_INVALID;
    }
    // rows that are not a multiple of 16 bytes (or shorter than the layer is wide), or blocks that do not hold
    // whole k-stages: this layer has to be stacked
    if (!psd_sfb_blocks_supported(plan, factor_dtype, ldu, ldv)) return PSD_E_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (factor_dtype == PSD_F32)
        return launch_sfb_f32_blocks(reinterpret_cast<const float* const*>(U_p), ldu,
                                     reinterpret_cast<const float* const*>(V_p), ldv, plan->P, plan->B, W, Mom, plan->N,
                                     plan->M, lr, mu, wd, st);
    return launch_sfb_bf16_blocks(reinterpret_cast<const uint16_t* const*>(U_p), ldu,
                                  reinterpret_cast<const uint16_t* const*>(V_p), ldv, plan->P, plan->B, W, Mom, plan->N,
                                  plan->M, lr, mu, wd, st);
}

psd_status psd_sync_fc_bias(const psd_plan* plan, int32_t factor_dtype, const void* U, int64_t ldu, float* bias,
                            float* mom_bias, float lr, float mu, float wd, void* stream)
{
    if (!plan || !U || !bias || !mom_bias) return PSD_E_NULL;
    if (factor_dtype != PSD_F32 && factor_dtype != PSD_BF16) return PSD_E_INVALID;
    if (!(wd >= 0.0f)) return PSD_E_INVALID;
    if (!valid_plan_sizes(plan) || !valid_ld(ldu, plan->N, factor_dtype)) return PSD_E_INVALID;
    if (!aligned16(U) || !aligned16(bias) || !aligned16(mom_bias) || bias == mom_bias) return PSD_E_INVALID;
    return launch_bias(U, ldu, factor_dtype, plan->N, plan->P * plan->B, bias, mom_bias, lr, mu, wd,
                       static_cast<hipStream_t>(stream));
}

static psd_status check_dense(int64_t n, int32_t P, int32_t maxP, const float* const* G, const float* W,
                              const float* Mom, int32_t S)
{
    if (n < 0 || P < 1 || P > maxP || S < 1) return PSD_E_INVALID;
    if (n == 0) return PSD_OK;                       // empty layer: nothing is dereferenced
    if (!G || !W || !Mom) return PSD_E_NULL;
    if (S > n) return PSD_E_INVALID;
    if (!aligned16(W) || !aligned16(Mom) || W == Mom) return PSD_E_INVALID;
    for (int32_t p = 0; p < P; ++p) {
        if (!G[p]) return PSD_E_NULL;
        if (!aligned16(G[p])) return PSD_E_INVALID;
    }
    return PSD_OK;
}

psd_status psd_sync_dense_ps(int64_t n, int32_t P, const float* const* G, float* W, float* Mom,
                             float lr, float mu, float wd, int32_t S, void* stream)
{
    if (!(wd >= 0.0f)) return PSD_E_INVALID;
    psd_status r = check_dense(n, P, PSD_MAX_WORKERS, G, W, Mom, S);
    if (r != PSD_OK) return r;
    if (n == 0) return PSD_OK;
    DenseWide a;
    for (int p = 0; p < PSD_MAX_WORKERS; ++p) a.G[p] = p < P ? G[p] : nullptr;
    a.W = W; a.Mom = Mom; a.n = n; a.P = P; a.S = S;
    a.q = n / S; a.r = n % S;
    a.chunks = dense_chunks_for(n, S);
    return launch_dense_wide(a, lr, mu, wd, static_cast<hipStream_t>(stream));
}

psd_status psd_sync_dense_ps_multi(int32_t L, const psd_dense_segment* segs, float lr, float mu, float wd, void* stream)
{
    if (!segs) return PSD_E_NULL;
    if (L < 1 || L > PSD_MAX_MULTI_SEGMENTS || !(wd >= 0.0f)) return PSD_E_INVALID;
    DenseTable t;
    int64_t blocks = 0;
    int32_t used = 0;
    for (int32_t l = 0; l < L; ++l) {
        const psd_dense_segment& s = segs[l];
        psd_status r = check_dense(s.n, s.P, PSD_MAX_MULTI_WORKERS, s.G, s.W, s.Mom, s.S);
        if (r != PSD_OK) return r;
        if (s.n == 0) continue;
        DenseSeg& d = t.seg[used++];
        for (int p = 0; p < PSD_MAX_MULTI_WORKERS; ++p) d.G[p] = p < s.P ? s.G[p] : nullptr;
        d.W = s.W; d.Mom = s.Mom; d.n = s.n; d.P = s.P; d.S = s.S;
        d.q = s.n / s.S; d.r = s.n % s.S;
        d.chunks = dense_chunks_for(s.n, s.S);
        d.block_begin = static_cast<int32_t>(blocks);
        blocks += static_cast<int64_t>(d.chunks) * s.S;
        if (blocks > (int64_t(1) << 30)) return PSD_E_INVALID;
    }
    if (used == 0) return PSD_OK;
    t.L = used;
    return launch_dense_table(t, static_cast<int32_t>(blocks), lr, mu, wd, static_cast<hipStream_t>(stream));
}

namespace {

// One event per host thread that orders the other streams of a fused parameter-server group after the
// group's single launch (created on first use, never destroyed; holds no device memory).
psd_status fuse_event(hipEvent_t* out)
{
    static thread_local hipEvent_t ev = nullptr;
    if (!ev) PSD_HIP_TRY(hipEventCreateWithFlags(&ev, hipEventDisableTiming));
    *out = ev;
    return PSD_OK;
}

// may this layer's parameter-server sum share a launch with others that wait for the same event `ready`?
// may this layer's parameter-server sum share a launch with others that wait for the same event `ready`?
// Events that order the reconstruction kernels of one iteration one after the other (one per host thread
// and position, created on first use, never destroyed).
psd_status chain_event(int i, hipEvent_t* out)
{
    static thread_local hipEvent_t ev[2] = {nullptr, nullptr};
    if (!ev[i & 1]) PSD_HIP_TRY(hipEventCreateWithFlags(&ev[i & 1], hipEventDisableTiming));
    *out = ev[i & 1];
    return PSD_OK;
}

bool fusable_ps_layer(const psd_layer_task& t, int32_t rule, const void* ready)
{
    const int32_t route = rule == PSD_RULE_ALG3 ? t.plan.route_alg3 : t.plan.route_vs_dense;
    return route == PSD_ROUTE_PS_DENSE && t.ev_ready == ready && t.G && t.plan.P <= PSD_MAX_MULTI_WORKERS;
}

}  // namespace

// Algorithm 2's order: the top layer's gradient exists first, so its synchronisation is
// issued first; every layer goes to its own stream.
psd_status psd_sync_iteration(int32_t L, const psd_layer_task* layers, float lr, float mu, float wd, int32_t rule)
{
    if (!layers) return PSD_E_NULL;
    if (L < 1 || (rule != PSD_RULE_ALG3 && rule != PSD_RULE_SFB_VS_DENSE)) return PSD_E_INVALID;
    for (int32_t l = L - 1; l >= 0; --l) {
        const psd_layer_task& t = layers[l];
        const int32_t route = rule == PSD_RULE_ALG3 ? t.plan.route_alg3 : t.plan.route_vs_dense;
        hipStream_t st = static_cast<hipStream_t>(t.stream);

        // A run of parameter-server layers whose gradients become available together (no ev_ready, or one
        // and the same event) gains nothing from being issued one by one: their sums go into ONE launch on
        // the top layer's stream, and the other layers' streams are ordered after it.
        int32_t lo = l;
        if (fusable_ps_layer(t, rule, t.ev_ready))
            while (lo > 0 && l - lo + 1 < PSD_MAX_MULTI_SEGMENTS && fusable_ps_layer(layers[lo - 1], rule, t.ev_ready)) --lo;
        if (lo < l) {
            if (t.ev_ready) PSD_HIP_TRY(hipStreamWaitEvent(st, static_cast<hipEvent_t>(t.ev_ready), 0));
            psd_dense_segment segs[PSD_MAX_MULTI_SEGMENTS];
            for (int32_t j = l; j >= lo; --j) {
                const psd_layer_task& u = layers[j];
                uint64_t n;
                if (mul_u64(static_cast<uint64_t>(u.plan.M), static_cast<uint64_t>(u.plan.N), &n) || n > (uint64_t(1) << 40))
                    return PSD_E_INVALID;
                psd_dense_segment& sg = segs[l - j];
                sg.n = static_cast<int64_t>(n); sg.P = static_cast<int32_t>(u.plan.P); sg.S = u.S;
                sg.G = u.G; sg.W = u.W; sg.Mom = u.Mom;
                if (u.ev_begin) PSD_HIP_TRY(hipEventRecord(static_cast<hipEvent_t>(u.ev_begin), st));
            }
            const psd_status r = psd_sync_dense_ps_multi(l - lo + 1, segs, lr, mu, wd, t.stream);
            if (r != PSD_OK) return r;
            hipEvent_t done = nullptr;
            bool other_streams = false;
            for (int32_t j = l; j >= lo; --j) {
                const psd_layer_task& u = layers[j];
                if (u.ev_end) PSD_HIP_TRY(hipEventRecord(static_cast<hipEvent_t>(u.ev_end), st));
                other_streams = other_streams || u.stream != t.stream;
            }
            if (other_streams) {
                const psd_status e = fuse_event(&done);
                if (e != PSD_OK) return e;
                PSD_HIP_TRY(hipEventRecord(done, st));
                for (int32_t j = l - 1; j >= lo; --j)
                    if (layers[j].stream != t.stream)
                        PSD_HIP_TRY(hipStreamWaitEvent(static_cast<hipStream_t>(layers[j].stream), done, 0));
            }
            l = lo;               // the loop's --l moves below the group
            continue;
        }

        if (t.ev_ready) PSD_HIP_TRY(hipStreamWaitEvent(st, static_cast<hipEvent_t>(t.ev_ready), 0));
        psd_status r;
        if (route == PSD_ROUTE_PS_DENSE) {
            if (!t.G) return PSD_E_UNSUPPORTED;   // route needs dense gradient copies
            uint64_t n;
            if (mul_u64(static_cast<uint64_t>(t.plan.M), static_cast<uint64_t>(t.plan.N), &n) ||
                n > (uint64_t(1) << 40))
                return PSD_E_INVALID;
            if (t.ev_begin) PSD_HIP_TRY(hipEventRecord(static_cast<hipEvent_t>(t.ev_begin), st));
            r = psd_sync_dense_ps(static_cast<int64_t>(n), static_cast<int32_t>(t.plan.P), t.G, t.W, t.Mom,
                                  lr, mu, wd, t.S, t.stream);
        } else if (route == PSD_ROUTE_SFB || route == PSD_ROUTE_SF_PS) {
            if (t.plan.kind != PSD_LAYER_FC) return PSD_E_INVALID;
            if (!t.U && !t.V) {
                // no stacked buffers given: delta_p / act_p hold blocks of factor_dtype, read where they lie
                if (t.ev_begin) PSD_HIP_TRY(hipEventRecord(static_cast<hipEvent_t>(t.ev_begin), st));
                r = psd_sync_fc_sfb_blocks(&t.plan, t.factor_dtype, t.delta_p, t.ldu ? t.ldu : t.plan.N, t.act_p,
                                           t.ldv ? t.ldv : t.plan.M, t.W, t.Mom, lr, mu, wd, t.stream);
            } else {
                r = psd_pack_factors(&t.plan, static_cast<const float* const*>(static_cast<const void*>(t.delta_p)),
                                     static_cast<const float* const*>(static_cast<const void*>(t.act_p)), t.factor_dtype,
                                     t.U, t.ldu, t.V, t.ldv, t.stream);
                if (r == PSD_OK && t.ev_begin) PSD_HIP_TRY(hipEventRecord(static_cast<hipEvent_t>(t.ev_begin), st));
                if (r == PSD_OK)
                    r = psd_sync_fc_sfb(&t.plan, t.factor_dtype, t.U, t.ldu, t.V, t.ldv, t.W, t.Mom, lr, mu, wd,
                                        t.workspace, t.workspace_bytes, t.stream);
            }
        } else {
            return PSD_E_INVALID;
        }
        if (r != PSD_OK) return r;
        if (t.ev_end) PSD_HIP_TRY(hipEventRecord(static_cast<hipEvent_t>(t.ev_end), st));
    }
    return PSD_OK;
}

}  // extern "C"
