/*
 * CPU oracle for the SACP gradient-synchronisation path (Poseidon, arXiv 1512.06216).
 *
 * TEST INFRASTRUCTURE ONLY.  Plain loops, float64 arithmetic, no blocking, no tricks.
 * It shares no code with the HIP library and must never be called from the product
 * path; only the tests, the smoke check and the benchmark's cpu_baseline leg use it.
 *
 * Naming (see oracle/psd_oracle.py for the full statement of the readings taken):
 *   M = layer inputs  (length of an activation vector a),
 *   N = layer outputs (length of an error vector delta),
 *   B = batch per worker (the paper's K), P = workers, K = P*B stacked rows,
 *   U is K x N (errors), V is K x M (activations), W and Mom are N x M, all row-major.
 *
 * Every function here has at least one pin in tests/test_oracle_*.py that does not
 * come from this file (paper's printed numbers, finite differences, numpy/torch
 * library routines, closed forms).
 */
#include <stdint.h>
#include <string.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---- fp32 -> bf16, round to nearest, ties to even ------------------------------------
 * Not in the paper (fp32 throughout); the bf16-factor variant is this build's extension.
 * Written from the definition of rounding, not as a bit trick: the two bf16 neighbours
 * of x are found by truncation, the nearer one wins, a tie goes to the even mantissa.
 * The neighbour above the largest finite bf16 is taken as 2^128 (IEEE overflow rule:
 * round as if the exponent range were unbounded, then deliver infinity).
 */
static double bf16_bits_value(uint32_t hi16)
{
    /* value of the bf16 pattern hi16 (sign ignored, finite or the "next after max") */
    uint32_t e = (hi16 >> 7) & 0xffu, m = hi16 & 0x7fu;
    if (e == 0) return ldexp((double)m, -126 - 7);
    return ldexp((double)(128u + m), (int)e - 127 - 7); /* e==255,m==0 -> 2^128 */
}

uint16_t orc_bf16_from_f32(float x)
{
    uint32_t u;
    memcpy(&u, &x, 4);
    uint32_t sign = u >> 31, mag = u & 0x7fffffffu;
    if (mag > 0x7f800000u) return (uint16_t)((sign << 15) | 0x7fc0u | ((mag >> 16) & 0x3fu)); /* NaN stays NaN, made quiet */
    if (mag == 0x7f800000u) return (uint16_t)((sign << 15) | 0x7f80u);
    uint32_t lo = mag >> 16, hi = lo + 1u;
    double ax = fabs((double)x);
    double dlo = ax - bf16_bits_value(lo);
    double dhi = bf16_bits_value(hi) - ax;
    uint32_t r;
    if (dlo < dhi) r = lo;
    else if (dhi < dlo) r = hi;
    else r = (lo & 1u) ? hi : lo;
    return (uint16_t)((sign << 15) | r);
}

void orc_bf16_round_array(const float* in, uint16_t* out, int64_t count)
{
    for (int64_t i = 0; i < count; ++i) out[i] = orc_bf16_from_f32(in[i]);
}

float orc_f32_from_bf16(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

void orc_bf16_widen_array(const uint16_t* in, float* out, int64_t count)
{
    for (int64_t i = 0; i < count; ++i) out[i] = orc_f32_from_bf16(in[i]);
}

/* ---- reconstruction: dW = sum over all K stacked samples of delta_k a_k^T -------------
 * Section 4.3.1, Eq. 5 (per-sample gradient is the outer product of the error and the
 * activation) and SFB step 3 / Alg. 3's SFB branch (sum over every worker's factors).
 * dW[n][m] = sum_{k=0..K-1} U[k][n] * V[k][m], accumulated in k order in float64.
 */
void orc_rebuild(const float* U, const float* V, int64_t K, int64_t N, int64_t M, double* dW)
{
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        double* row = dW + n * M;
        for (int64_t m = 0; m < M; ++m) row[m] = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            double u = (double)U[k * N + n];
            const float* v = V + k * M;
            for (int64_t m = 0; m < M; ++m) row[m] += u * (double)v[m];
        }
    }
}

/* the same definition, evaluated only at `count` sampled (n,m) positions */
void orc_rebuild_samples(const float* U, const float* V, int64_t K, int64_t N, int64_t M,
                         const int64_t* idx_n, const int64_t* idx_m, int64_t count, double* out)
{
#pragma omp parallel for schedule(static)
    for (int64_t s = 0; s < count; ++s) {
        int64_t n = idx_n[s], m = idx_m[s];
        double acc = 0.0;
        for (int64_t k = 0; k < K; ++k) acc += (double)U[k * N + n] * (double)V[k * M + m];
        out[s] = acc;
    }
}

/* ---- momentum-SGD update ---------------------------------------------------------------
 * Section 3.3, Eq. 3-4 (additive update with step size and a momentum term) and Alg. 3's
 * update line.  Reading taken (the paper gives no explicit momentum formula):
 *   mom' = mu*mom + lr*(dW + wd*w) ;  w' = w - mom'
 * (wd = L2 weight decay, the regularisation part of Lambda; wd = 0: plain momentum SGD),
 * evaluated in float64 from the fp32 inputs, each result rounded to fp32 once.
 */
void orc_update(const double* dW, float* W, float* Mom, float lr, float mu, float wd, int64_t count)
{
    double dlr = (double)lr, dmu = (double)mu, dwd = (double)wd;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) {
        double mom = dmu * (double)Mom[i] + dlr * (dW[i] + dwd * (double)W[i]);
        double w = (double)W[i] - mom;
        Mom[i] = (float)mom;
        W[i] = (float)w;
    }
}

/* ---- key-range shards -------------------------------------------------------------------
 * The paper's server is a sharded key-value store (Section 3.2) but the ranges are not
 * defined there.  Reading taken: keys 0..n-1 are the row-major flattened parameters;
 * shard s of S owns [floor(s*n/S), floor((s+1)*n/S)).
 */
void orc_shard_range(int64_t n, int64_t S, int64_t s, int64_t* begin, int64_t* end)
{
    /* n < 2^40 and S <= 2^20 in every use, so the products fit in int64 */
    *begin = (s * n) / S;
    *end = ((s + 1) * n) / S;
}

/* ---- parameter-server path: sum the P dense copies per key, shard by shard, then update --
 * Alg. 1 master node (collect gradients, update the part of the parameters for which a
 * gradient was received) and Alg. 3's non-FC branch.  Sum over workers, not mean
 * (Eq. 2 and Eq. 4 sum over p).
 */
void orc_dense_ps(const float* const* G, int64_t P, int64_t n, int64_t S,
                  float* W, float* Mom, float lr, float mu, float wd)
{
    double dlr = (double)lr, dmu = (double)mu, dwd = (double)wd;
    for (int64_t s = 0; s < S; ++s) {
        int64_t b, e;
        orc_shard_range(n, S, s, &b, &e);
#pragma omp parallel for schedule(static)
        for (int64_t i = b; i < e; ++i) {
            double g = 0.0;
            for (int64_t p = 0; p < P; ++p) g += (double)G[p][i];
            double mom = dmu * (double)Mom[i] + dlr * (g + dwd * (double)W[i]);
            double w = (double)W[i] - mom;
            Mom[i] = (float)mom;
            W[i] = (float)w;
        }
    }
}

/* ---- bias gradient ---------------------------------------------------------------------
 * For z = W a + b the per-sample gradient w.r.t. b is the error vector (the chain rule that
 * gives Eq. 5 for W), so db[n] = sum over all K stacked samples of U[k][n], in float64.
 */
void orc_bias_grad(const float* U, int64_t K, int64_t N, double* db)
{
    for (int64_t n = 0; n < N; ++n) {
        double acc = 0.0;
        for (int64_t k = 0; k < K; ++k) acc += (double)U[k * N + n];
        db[n] = acc;
    }
}

/* thread count used by the timed cpu_baseline runs (no arithmetic) */
void orc_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}
