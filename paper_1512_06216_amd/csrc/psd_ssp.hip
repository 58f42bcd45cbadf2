// Bounded staleness (stale synchronous parallel consistency, Section 3.2) on one worker GPU: the update
// produced at clock c is applied s clocks later, so that the parameters read at clock t hold exactly
// the updates of clocks 0 .. t-s-1, the view the consistency model guarantees.  Host logic only: the
// pending updates wait in a ring of s+1 caller-owned buffers (stacked factors of an FC layer, dense
// gradient copies of a parameter-server layer) and are applied by the same kernels as without staleness.
#include "psd_internal.h"

extern "C" {

psd_status psd_ssp_init(psd_ssp_state* st, int32_t s)
{
    if (!st) return PSD_E_NULL;
    if (s < 0 || s > PSD_MAX_STALENESS) return PSD_E_INVALID;
    st->s = s;
    st->reserved = 0;
    st->clock = 0;
    return PSD_OK;
}

psd_status psd_ssp_slots(const psd_ssp_state* st, int32_t* push_slot, int32_t* due_slot)
{
    if (!st || !push_slot || !due_slot) return PSD_E_NULL;
    if (st->s < 0 || st->s > PSD_MAX_STALENESS || st->clock < 0) return PSD_E_INVALID;
    const int64_t ring = int64_t(st->s) + 1;
    *push_slot = static_cast<int32_t>(st->clock % ring);
    // the update of clock c falls due at clock c + s: the reader at clock c + s + 1 must see it
    *due_slot = st->clock >= st->s ? static_cast<int32_t>((st->clock - st->s) % ring) : -1;
    return PSD_OK;
}

psd_status psd_ssp_clock_fc(psd_ssp_state* st, const psd_plan* plan, int32_t factor_dtype,
                            const float* const* delta_p, const float* const* act_p, void* const* U_ring, int64_t ldu,
                            void* const* V_ring, int64_t ldv, float* W, float* Mom, float lr, float mu, float wd,
                            void* workspace, size_t workspace_bytes, void* stream)
{
    if (!st || !plan || !U_ring || !V_ring) return PSD_E_NULL;
    if ((delta_p == nullptr) != (act_p == nullptr)) return PSD_E_NULL;     // both (a new clock's factors) or neither (drain)
    int32_t push, due;
    psd_status r = psd_ssp_slots(st, &push, &due);
    if (r != PSD_OK) return r;
    for (int32_t i = 0; i <= st->s; ++i)
        if (!U_ring[i] || !V_ring[i]) return PSD_E_NULL;
    if (delta_p) {
        r = psd_pack_factors(plan, delta_p, act_p, factor_dtype, U_ring[push], ldu, V_ring[push], ldv, stream);
        if (r != PSD_OK) return r;
    } else if (st->s == 0) {
        return PSD_E_INVALID;        // nothing is ever pending without staleness: there is nothing to drain
    }
    if (due >= 0) {
        r = psd_sync_fc_sfb(plan, factor_dtype, U_ring[due], ldu, V_ring[due], ldv, W, Mom, lr, mu, wd, workspace,
                            workspace_bytes, stream);
        if (r != PSD_OK) return r;
    }
    st->clock += 1;
    return PSD_OK;
}

psd_status psd_ssp_clock_dense(psd_ssp_state* st, int64_t n, int32_t P, const float* const* const* G_ring, float* W,
                               float* Mom, float lr, float mu, float wd, int32_t S, void* stream)
{
    if (!st || !G_ring) return PSD_E_NULL;
    int32_t push, due;
    psd_status r = psd_ssp_slots(st, &push, &due);
    if (r != PSD_OK) return r;
    (void)push;                      // the caller has written this clock's copies into G_ring[push] already
    if (due >= 0) {
        if (!G_ring[due]) return PSD_E_NULL;
        r = psd_sync_dense_ps(n, P, G_ring[due], W, Mom, lr, mu, wd, S, stream);
        if (r != PSD_OK) return r;
    }
    st->clock += 1;
    return PSD_OK;
}

}  // extern "C"
