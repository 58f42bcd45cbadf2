/*
 * psd.h -- C ABI of the MI355X (gfx950) implementation of the per-layer gradient
 * synchronisation compute of Poseidon's structure-aware communication protocol
 * (arXiv 1512.06216, Section 4.3, Algorithm 3; issue order of Section 4.2, Algorithm 2).
 *
 * Symbols.  A fully-connected layer has M inputs and N outputs; W and Mom are N x M,
 * row-major fp32 (one row per output neuron, Section 3.3).  B is the batch per worker
 * (the paper's "batch size K"), P the number of workers, K = P*B the number of stacked
 * samples.  U (K x N, errors) and V (K x M, activations) are the stacked sufficient
 * factors of Section 4.3.1; row k = p*B + b holds sample b of worker p.
 *
 * Conventions for every entry point:
 *   - returns a psd_status (0 = ok, negative = error); never throws, aborts or prints;
 *   - pointers marked [dev] are device memory owned by the caller, never retained or
 *     freed; pointers marked [host] are host memory read before the call returns;
 *   - device work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and the call returns without synchronising;
 *   - [dev] base pointers must be 16-byte aligned, buffers must not overlap;
 *   - sizes are validated on the host before anything is launched; no entry point
 *     allocates device memory.
 */
#ifndef PSD_H
#define PSD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t psd_status;
enum {
    PSD_OK = 0,
    PSD_E_INVALID = -1,     /* a size, enum value, alignment or leading dimension is out of range */
    PSD_E_NULL = -2,        /* a required pointer is NULL */
    PSD_E_UNSUPPORTED = -3, /* valid request this build cannot serve (e.g. route needs data not given) */
    PSD_E_OVERFLOW = -4,    /* a communication volume does not fit in 64 bits */
    PSD_E_HIP = -5,         /* a HIP call failed; see psd_last_hip_error() */
    PSD_E_WORKSPACE = -6    /* a workspace was passed that is smaller than psd_sfb_workspace_bytes() asks for */
};

enum { PSD_LAYER_CONV = 0, PSD_LAYER_FC = 1 };                      /* layer kind       */
enum { PSD_ROUTE_PS_DENSE = 0, PSD_ROUTE_SFB = 1, PSD_ROUTE_SF_PS = 2 }; /* route        */
enum { PSD_RULE_ALG3 = 0, PSD_RULE_SFB_VS_DENSE = 1 };              /* which comparison */
enum { PSD_F32 = 0, PSD_BF16 = 1 };                                 /* factor dtype     */

#define PSD_MAX_WORKERS 64  /* P, single-layer entry points */
#define PSD_MAX_MULTI_SEGMENTS 16
#define PSD_MAX_MULTI_WORKERS 16

/* Result of the route selection of Algorithm 3. */
typedef struct psd_plan {
    int64_t M, N, B, P;
    int32_t kind;            /* PSD_LAYER_* */
    int32_t route_alg3;      /* Algorithm 3 as printed: conv -> PS_DENSE; FC -> SFB if
                                cost_sfb <= cost_sf_ps, else SF_PS */
    int32_t route_vs_dense;  /* the prose comparison of Section 4.3.1: FC -> SFB if
                                cost_sfb <= cost_ps_dense, else PS_DENSE */
    int32_t reserved;
    uint64_t cost_sfb;       /* (P-1)^2 * B * (M+N) floats: factors to and from P-1 peers   */
    uint64_t cost_ps_dense;  /* 2 * P * M * N floats: full matrices pushed and pulled       */
    uint64_t cost_sf_ps;     /* P*B*(M+N) + P*M*N floats: factors up, full matrix back down */
} psd_plan;

/* Algorithm 3's route choice and the three communication volumes of Section 4.3.1.
 * Host only, integer only.  M, N, B, P >= 1, P <= PSD_MAX_WORKERS.  For a conv layer M and
 * N are any factorisation of its parameter count (only M*N matters).  `out` [host]. */
psd_status psd_plan_layer(int32_t kind, int64_t M, int64_t N, int64_t B, int64_t P, psd_plan* out);

/* Key range [*begin, *end) of shard s when keys 0..n-1 (the row-major flattened
 * parameters of one layer) are split into S contiguous balanced ranges:
 * begin = floor(s*n/S), end = floor((s+1)*n/S).  Needs 1 <= S <= n, 0 <= s < S.
 * The paper's parameter server (Section 3.2) is sharded but does not define the ranges;
 * this is the definition used throughout.  Host only. */
psd_status psd_shard_range(int64_t n, int32_t S, int32_t s, int64_t* begin, int64_t* end);

/* Recommended leading dimension (in elements) of a stacked factor matrix with `cols` columns:
 * cols rounded up to a multiple of 128 bytes (32 f32 or 64 bf16 elements), so that every row starts
 * on a cache-line boundary.  The entry points accept any leading dimension >= cols whose rows are a
 * multiple of 16 bytes (4 f32 / 8 bf16 elements); rows that start mid-line cost the bf16
 * reconstruction of odd-width layers 3-7 % (a 256-byte tile row then spans three lines, not two).
 * Returns 0 for bad arguments. */
int64_t psd_factor_ld(int64_t cols, int32_t dtype);

/* SFB steps 1-2 of Section 4.3.1 seen from the receiving worker: stack the P per-worker
 * factor blocks into U and V, optionally rounding fp32 -> bf16 (nearest even; NaN stays a
 * quiet NaN with its sign, +-Inf kept, overflow -> Inf).
 *   delta_p [host] array of P [dev] pointers, each B x N fp32 row-major (errors)
 *   act_p   [host] array of P [dev] pointers, each B x M fp32 row-major (activations)
 *   U [dev] K x ldu, V [dev] K x ldv elements of `out_dtype`; U[p*B+b][j] = delta_p[p][b][j].
 *   ldu >= N, ldv >= M, and ld * element size must be a multiple of 16 bytes; columns
 *   N..ldu-1 (M..ldv-1) are written as zero.
 * plan->M,N,B,P give the sizes. */
psd_status psd_pack_factors(const psd_plan* plan, const float* const* delta_p,
                            const float* const* act_p, int32_t out_dtype,
                            void* U, int64_t ldu, void* V, int64_t ldv, void* stream);

/* SFB step 3 and Algorithm 3's update line on one worker, fused:
 *     dW[n][m] = sum_{k<K} U[k][n] * V[k][m]          (Eq. 5 summed over all P*B samples)
 *     Mom <- mu*Mom + lr*(dW + wd*W) ;  W <- W - Mom  (momentum SGD with L2 weight decay wd, the
 *                                                      "regularisation and momentum" term Lambda of
 *                                                      Section 3.3; sum over workers, no 1/P; wd = 0
 *                                                      gives plain momentum SGD)
 * U, V [dev] as written by psd_pack_factors (same dtype and leading dimensions);
 * W, Mom [dev] N x M fp32 row-major, updated in place; dW is never stored.
 * fp32 factors: fp32 MFMA, fp32 accumulation.  bf16 factors: bf16 MFMA with fp32
 * accumulation; W and Mom stay fp32.  The same call serves the SF_PS route (the server
 * runs the identical reconstruction over the same P*B factors).
 * Size limit: the kernels address each stacked factor matrix with 32-bit byte offsets, so K * ldu and
 * K * ldv times the element size must stay below 4 GiB less a few k-stages of read-ahead (the largest
 * layer named in the paper, a VGG-16-sized 25088 -> 4096 one at K = 2048, needs 0.2 GiB); a larger
 * layer is refused with PSD_E_UNSUPPORTED before anything is launched.
 *
 * workspace [dev] (optional): scratch for layers with so few output tiles (128 x 128 weights each)
 * that most compute units would get none (e.g. a 1024 -> 1000 classifier).  With workspace_bytes == 0 (workspace may be NULL) every tile is contracted
 * over all of K by one workgroup.  With a workspace of at least psd_sfb_workspace_bytes() bytes,
 * 16-byte aligned, the sum over k is split over up to 4 workgroups per tile: each stores a partial dW
 * (N x M fp32) to the workspace, then the partials are added in split order and the update is applied
 * (same arithmetic; only the order of the fp32 additions over k changes).  A non-zero workspace_bytes
 * below the queried size is refused with PSD_E_WORKSPACE.  The workspace is not retained; its contents
 * after the call are unspecified; calls that share one workspace must not overlap in time. */
psd_status psd_sync_fc_sfb(const psd_plan* plan, int32_t factor_dtype,
                           const void* U, int64_t ldu, const void* V, int64_t ldv,
                           float* W, float* Mom, float lr, float mu, float wd,
                           void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of workspace with which psd_sync_fc_sfb would split this layer's sum over k (a multiple of
 * 16), or 0 if it would not split it (enough tiles already, K too short, bad arguments).  Host only;
 * depends on the layer shape, the factor dtype, the current device's CU count and the pinned tile. */
size_t psd_sfb_workspace_bytes(const psd_plan* plan, int32_t factor_dtype);

/* psd_sync_fc_sfb for callers that cannot allocate and have no workspace to pass: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and arithmetic as
 * psd_sync_fc_sfb called with a workspace of exactly psd_sfb_workspace_bytes() bytes, but the partial
 * tiles of a split layer go to a fixed PSD_STATIC_SCRATCH_BYTES array that lives in the library's device
 * code (each GPU the library runs on holds its own copy until the process ends).  Calls no allocating
 * routine.  A layer whose split needs more than PSD_STATIC_SCRATCH_BYTES is refused with
 * PSD_E_WORKSPACE (use psd_sync_fc_sfb with your own workspace, or none); a layer that is not split
 * needs no scratch and runs as psd_sync_fc_sfb without a workspace.  All calls on one GPU share that
 * GPU's array: calls that overlap in time on one GPU (different streams, different threads) race on it
 * and must be serialised by the caller.  The array keeps the last call's partials; nothing has to be
 * cleared between calls. */
#define PSD_STATIC_SCRATCH_BYTES (16u << 20)
psd_status psd_sync_fc_sfb_static(const psd_plan* plan, int32_t factor_dtype,
                                  const void* U, int64_t ldu, const void* V, int64_t ldv,
                                  float* W, float* Mom, float lr, float mu, float wd, void* stream);

/* psd_sync_fc_sfb WITHOUT the stacking pass: the reconstruction reads the P per-worker factor blocks where
 * they lie (row k = p*B + b of U is row b of U_p[p], of V row b of V_p[p]) -- the stacked matrices of SFB
 * steps 1-2 need not exist when the factors can be used as they were received: fp32 factors straight from
 * backpropagation and from the peers (ldu = N, ldv = M), or bf16 factors that every sender rounded before
 * sending (a block is then what psd_pack_factors writes for a one-worker plan).
 * Same arithmetic in the same order as psd_sync_fc_sfb (no workspace) on the stacked matrices: results are
 * identical bit for bit.
 *   U_p, V_p [host] arrays of P [dev] pointers to B x ldu and B x ldv elements of factor_dtype, row-major,
 *   16-byte aligned, read only.  ldu >= N, ldv >= M, rows a multiple of 16 bytes.
 * Served when B is a multiple of the kernel's k-stage (16 rows for fp32, 32 for bf16: a stage never
 * straddles two blocks); psd_sfb_blocks_supported tells (1 = yes).  Any other layer is refused with
 * PSD_E_UNSUPPORTED before anything is launched: stack it. */
int32_t psd_sfb_blocks_supported(const psd_plan* plan, int32_t factor_dtype, int64_t ldu, int64_t ldv);
psd_status psd_sync_fc_sfb_blocks(const psd_plan* plan, int32_t factor_dtype, const void* const* U_p, int64_t ldu,
                                  const void* const* V_p, int64_t ldv, float* W, float* Mom, float lr, float mu,
                                  float wd, void* stream);

/* Bias of an FC layer under SFB.  For z = W a + b the per-sample gradient w.r.t. b is the error
 * vector itself (the chain rule behind Eq. 5), so with the stacked errors U of the layer
 *     db[n] = sum_{k<K} U[k][n] ;  mom_bias <- mu*mom_bias + lr*(db + wd*bias) ;  bias <- bias - mom_bias.
 * No extra communication: U is what SFB already delivered (the paper's volumes count weights
 * only, Table 3).  U [dev] K x ldu as written by psd_pack_factors; bias, mom_bias [dev] N fp32,
 * in place, 16-byte aligned.  fp32 accumulation, 16 interleaved partial sums per column. */
psd_status psd_sync_fc_bias(const psd_plan* plan, int32_t factor_dtype, const void* U, int64_t ldu,
                            float* bias, float* mom_bias, float lr, float mu, float wd, void* stream);

/* Parameter-server route (Algorithm 1 master node; Algorithm 3 non-FC branch): for every
 * key i of every shard, g = sum_{p<P} G[p][i] (summed in p order, fp32), then the same
 * update (momentum mu, step lr, weight decay wd) on W[i], Mom[i].
 *   G [host] array of P [dev] pointers to n fp32 each (read only); W, Mom [dev] n fp32,
 *   in place.  1 <= P <= PSD_MAX_WORKERS; n >= 0 (n == 0 is a no-op); 1 <= S <= n.
 * The shards (psd_shard_range) are processed one after the other in key order inside one
 * launch; S changes which workgroup touches which key, never a value. */
psd_status psd_sync_dense_ps(int64_t n, int32_t P, const float* const* G,
                             float* W, float* Mom, float lr, float mu, float wd, int32_t S, void* stream);

/* One segment (layer) of a batched parameter-server launch. */
typedef struct psd_dense_segment {
    int64_t n;                 /* keys in this layer */
    int32_t P;                 /* copies, 1..PSD_MAX_MULTI_WORKERS */
    int32_t S;                 /* shards, 1..n */
    const float* const* G;     /* [host] array of P [dev] pointers */
    float* W;                  /* [dev] n fp32 */
    float* Mom;                /* [dev] n fp32 */
} psd_dense_segment;

/* Several layers' parameter-server updates in ONE kernel launch (the five small conv
 * layers of an AlexNet-sized net would otherwise be launch-latency bound).
 * 1 <= L <= PSD_MAX_MULTI_SEGMENTS; segs [host].  Same arithmetic as psd_sync_dense_ps. */
psd_status psd_sync_dense_ps_multi(int32_t L, const psd_dense_segment* segs,
                                   float lr, float mu, float wd, void* stream);

/* One layer of an iteration for psd_sync_iteration. */
typedef struct psd_layer_task {
    psd_plan plan;             /* from psd_plan_layer */
    int32_t factor_dtype;      /* FC: PSD_F32 or PSD_BF16 */
    int32_t S;                 /* PS route: shards */
    const void* const* delta_p; /* FC: [host] P [dev] pointers to the workers' error blocks: B x N fp32 each */
    const void* const* act_p;   /* FC: [host] P [dev] pointers to the workers' activation blocks: B x M fp32 each
                                   (for both: B x ldu / B x ldv elements of factor_dtype when read in place, see V) */
    void* U; int64_t ldu;      /* FC: [dev] K x ldu stacked errors (written, then read) */
    void* V; int64_t ldv;      /* FC: [dev] K x ldv stacked activations.  U == V == NULL: no stacked copy;
                                  delta_p / act_p then hold blocks of factor_dtype with leading dimensions
                                  ldu / ldv (0 = N / M) that are read in place (psd_sync_fc_sfb_blocks) */
    const float* const* G;     /* PS route: [host] P [dev] pointers, M*N fp32 each (may be
                                  NULL for an FC layer that is routed to SFB / SF_PS) */
    float* W; float* Mom;      /* [dev] N x M fp32 */
    void* workspace;           /* FC: optional [dev] scratch of workspace_bytes bytes (see psd_sync_fc_sfb) */
    size_t workspace_bytes;    /* 0 = none */
    void* stream;              /* the stream this layer's work is enqueued on */
    void* ev_ready;            /* optional hipEvent_t (or NULL): the layer's stream waits for it before any
                                  of the layer's work starts -- "the gradient of this layer exists"
                                  (Algorithm 2: a layer is synchronised as soon as backpropagation has
                                  produced its gradient, while lower layers are still computing) */
    void* ev_begin;            /* optional hipEvent_t (or NULL) recorded on `stream` right before */
    void* ev_end;              /* ... and right after the layer's reconstruct+update or
                                  sum+update kernel (factor packing lies outside the pair) */
} psd_layer_task;

/* One iteration's synchronisation in the order of Algorithm 2: layers are given bottom-up
 * (layers[0] is the lowest layer) and issued top-down, layer L-1 first, each on its own
 * stream as if its gradient had just been produced by backpropagation.  Each layer follows
 * the route its plan holds under `rule`: PS_DENSE -> psd_sync_dense_ps; SFB or SF_PS ->
 * psd_pack_factors then psd_sync_fc_sfb (with the layer's workspace, if any), or psd_sync_fc_sfb_blocks
 * alone for a layer given without stacked buffers.  Layers own disjoint
 * parameters (Section 4.2), so no ordering between streams is needed; the caller synchronises the
 * streams.
 * Consecutive PS_DENSE layers whose gradients become available together (none has an ev_ready, or all
 * name the same event), so that nothing is gained by issuing them one by one, with at most
 * PSD_MAX_MULTI_WORKERS copies, are summed by ONE
 * psd_sync_dense_ps_multi launch on the stream of the topmost of them (up to PSD_MAX_MULTI_SEGMENTS
 * per launch); the streams of the other layers of the group are made to wait for that launch, and
 * every group member's ev_begin / ev_end are recorded around it.
 * Stops at and returns the first error. */
psd_status psd_sync_iteration(int32_t L, const psd_layer_task* layers, float lr, float mu, float wd,
                              int32_t rule);

/* ---- Bounded staleness (stale synchronous parallel consistency, Section 3.2) -------------------
 * With staleness s, a worker that reads the parameters at clock t is guaranteed the updates of all
 * workers from clocks 0 .. t-s-1; s = 0 is bulk synchronous.  On one worker this means: the update
 * produced at clock c (the stacked factors of an FC layer, the dense copies of a parameter-server layer)
 * is applied at the end of clock c+s.  The pending updates wait in a ring of s+1 caller-owned buffers;
 * psd_ssp_state (host memory, caller-owned, one per layer) counts the clocks.  The arithmetic of an
 * update is that of psd_sync_fc_sfb / psd_sync_dense_ps; only WHEN it is applied changes, so after
 * T clocks the parameters equal those of T-s bulk-synchronous clocks and s updates are still pending. */
#define PSD_MAX_STALENESS 15
typedef struct psd_ssp_state {
    int32_t s;         /* staleness bound, 0..PSD_MAX_STALENESS */
    int32_t reserved;
    int64_t clock;     /* the clock the next psd_ssp_clock_* call stands for; starts at 0 */
} psd_ssp_state;

/* Sets st to clock 0 with staleness s. */
psd_status psd_ssp_init(psd_ssp_state* st, int32_t s);

/* Ring slots of the current clock: *push_slot = clock mod (s+1) is where this clock's factors /
 * gradient copies go; *due_slot is the slot whose update falls due now (that of clock - s), or -1
 * during the first s clocks when nothing is due yet.  Host only. */
psd_status psd_ssp_slots(const psd_ssp_state* st, int32_t* push_slot, int32_t* due_slot);

/* One clock of an FC layer under SFB: stacks this clock's per-worker factor blocks (as
 * psd_pack_factors) into U_ring[push_slot], V_ring[push_slot], then, if an update is due, rebuilds
 * and applies it from U_ring[due_slot], V_ring[due_slot] (as psd_sync_fc_sfb, same workspace rules), then
 * advances the clock.  U_ring, V_ring [host]: s+1 [dev] buffers each, K x ldu / K x ldv elements of
 * factor_dtype.  delta_p == act_p == NULL drains: nothing is stacked, the due update is applied (call it
 * s times after the last clock to apply what is still pending; invalid for s = 0). */
psd_status psd_ssp_clock_fc(psd_ssp_state* st, const psd_plan* plan, int32_t factor_dtype,
                            const float* const* delta_p, const float* const* act_p,
                            void* const* U_ring, int64_t ldu, void* const* V_ring, int64_t ldv,
                            float* W, float* Mom, float lr, float mu, float wd,
                            void* workspace, size_t workspace_bytes, void* stream);

/* One clock of a parameter-server layer: G_ring [host] holds s+1 [host] arrays of P [dev] pointers;
 * the caller has put this clock's copies into G_ring[push_slot] (entries of slots that are not due
 * are not looked at); if an update is due it is summed and applied from G_ring[due_slot] (as
 * psd_sync_dense_ps), then the clock advances. */
psd_status psd_ssp_clock_dense(psd_ssp_state* st, int64_t n, int32_t P, const float* const* const* G_ring,
                               float* W, float* Mom, float lr, float mu, float wd, int32_t S, void* stream);

/* Tuning / test hook (not part of the method): pins a choice the library otherwise makes itself.
 * Process-wide, takes effect on the next call; value -1 restores the automatic choice; any other value
 * outside the listed range is refused with PSD_E_INVALID and changes nothing.  Results never depend on
 * these choices (only speed does).
 *   PSD_TUNE_SFB_BF16_TILE: workgroup tile of the bf16 reconstruction, rows n x columns m of W:
 *                           0 = 128 x 256, 1 = 128 x 192, 2 = 128 x 128
 *   PSD_TUNE_SFB_F32_TILE:  ... of the fp32 reconstruction: 1 = 64 x 128, 2 = 128 x 128
 *   PSD_TUNE_SFB_BF16_SKEW_US: 0..200 (default and -1: 0).  The workgroups of the bf16 reconstruction that
 *                           start first on the odd-numbered accelerator dies (XCDs) wait this many
 *                           microseconds before they begin, so that one half of the chip is in its MFMA
 *                           loop while the other half streams its W / Mom update.  A measurement aid
 *                           for studying how the two phases share the chip. */
enum { PSD_TUNE_SFB_BF16_TILE = 0, PSD_TUNE_SFB_F32_TILE = 1, PSD_TUNE_SFB_BF16_SKEW_US = 2, PSD_TUNE_COUNT_ = 3 };
psd_status psd_tune_set(int32_t knob, int32_t value);

const char* psd_status_string(psd_status s);
/* hipError_t value of the most recent failing HIP call on this thread (0 if none). */
int32_t psd_last_hip_error(void);
/* Library version, for the binding's load check. */
int32_t psd_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PSD_H */
