"""CPU oracle for the SACP gradient-synchronisation path (Poseidon, arXiv 1512.06216).

TEST INFRASTRUCTURE ONLY: used by tests/, the smoke check and the benchmark's
cpu_baseline leg.  It shares no code with the HIP library; the product path never
imports it.  Integer logic is written with Python's unbounded ints, heavy loops live
in psd_oracle.c (plain loops, float64), glue is numpy.

Readings of the paper used here (each is also listed in the design notes):
  * Symbols.  The paper's W is M x N with an M-dimensional error; this build names
    M = inputs (length of a), N = outputs (length of delta); the cost formulas only
    contain M+N and M*N, so they are unaffected.  The paper's "batch size K" is the
    per-worker batch, called B here; K = P*B is the number of stacked samples.
  * The update sums over all P workers' samples, own worker included, with no 1/P
    (Eq. 2, Eq. 4, Alg. 3 SFB branch).
  * Lambda ("regularisation and momentum", Section 3.3) is applied once per update:
    mom' = mu*mom + lr*(dW + wd*w), w' = w - mom'  (L2 weight decay wd added to the gradient
    before the momentum, as in the Caffe solver the paper builds on; wd = 0 by default).
  * Bounded staleness (Section 3.2): a worker that reads at clock t is guaranteed the updates of clocks
    0 .. t-s-1 from all workers; this oracle evaluates exactly that guaranteed view (updates that a real
    server might deliver early are not included), applied in clock order.
  * Costs: SFB (P-1)^2 B (M+N); full matrices 2 P M N; factors-to-server
    P B (M+N) + P M N (Section 4.3.1).  Alg. 3 compares the first with the third and
    takes SFB on equality.

Pins (tests/test_oracle_*.py): the three communication volumes and two ratios printed in
Section 4.3.1; finite-difference gradients of a tiny FC layer; K=1 outer product; rank
bound; linearity; row-permutation invariance; numpy float64 matmul; closed forms of the
update; torch's CPU bf16 cast; brute-force shard cover; SFB path == PS path; bias gradient
against finite differences and numpy's column sum; the staleness window against a literal clock-by-clock
simulation of a server that withholds each update for s clocks and against the closed form with plain SGD.
Parity unpinned: none.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from fractions import Fraction

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libpsd_oracle.so")
_SRC = os.path.join(_HERE, "psd_oracle.c")

ROUTE_PS_DENSE, ROUTE_SFB, ROUTE_SF_PS = 0, 1, 2
KIND_CONV, KIND_FC = 0, 1
U64_MAX = (1 << 64) - 1


def build(force=False):
    """Compile psd_oracle.c with gcc (baseline x86-64 code so it runs on any host)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-ffp-contract=off", "-o", _SO, _SRC, "-lm"])
    return _SO


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        i64, f32p = ctypes.c_int64, ctypes.POINTER(ctypes.c_float)
        f64p, u16p = ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_uint16)
        i64p = ctypes.POINTER(ctypes.c_int64)
        L.orc_num_threads.restype = ctypes.c_int
        L.orc_bf16_round_array.argtypes = [f32p, u16p, i64]
        L.orc_bf16_widen_array.argtypes = [u16p, f32p, i64]
        L.orc_rebuild.argtypes = [f32p, f32p, i64, i64, i64, f64p]
        L.orc_rebuild_samples.argtypes = [f32p, f32p, i64, i64, i64, i64p, i64p, i64, f64p]
        L.orc_update.argtypes = [f64p, f32p, f32p, ctypes.c_float, ctypes.c_float, ctypes.c_float, i64]
        L.orc_shard_range.argtypes = [i64, i64, i64, i64p, i64p]
        L.orc_bias_grad.argtypes = [f32p, i64, i64, f64p]
        L.orc_bias_grad.restype = None
        L.orc_dense_ps.argtypes = [ctypes.POINTER(f32p), i64, i64, i64, f32p, f32p,
                                   ctypes.c_float, ctypes.c_float, ctypes.c_float]
        for fn in (L.orc_bf16_round_array, L.orc_bf16_widen_array, L.orc_rebuild,
                   L.orc_rebuild_samples, L.orc_update, L.orc_shard_range, L.orc_dense_ps):
            fn.restype = None
        _lib = L
    return _lib


def num_threads():
    return int(lib().orc_num_threads())


def set_num_threads(n):
    """OpenMP threads used by the C loops from now on (for the timed baseline runs)."""
    lib().orc_set_num_threads(ctypes.c_int(int(n)))


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


# --------------------------------------------------------------------------------------
# Route selection (Alg. 3; communication volumes of Section 4.3.1)
# --------------------------------------------------------------------------------------
def plan_layer(kind, M, N, B, P):
    """Communication volumes in floats and the route each rule picks.

    cost_sfb       every worker sends and receives B factor pairs to/from P-1 peers
    cost_ps_dense  every worker pushes and pulls the full M x N matrix
    cost_sf_ps     factors up to the server, full matrix back down
    route_alg3     Alg. 3 as printed: conv -> PS; FC -> SFB iff cost_sfb <= cost_sf_ps
    route_vs_dense the comparison made in the prose: FC -> SFB iff cost_sfb <= cost_ps_dense
    """
    for v in (M, N, B, P):
        if int(v) != v or v < 1:
            raise ValueError("M, N, B, P must be positive integers")
    M, N, B, P = int(M), int(N), int(B), int(P)
    cost_sfb = (P - 1) ** 2 * B * (M + N)
    cost_ps_dense = 2 * P * M * N
    cost_sf_ps = P * B * (M + N) + P * M * N
    if max(cost_sfb, cost_ps_dense, cost_sf_ps) > U64_MAX:
        raise OverflowError("cost does not fit in 64 bits")
    if kind == KIND_CONV:
        route_alg3 = route_vs_dense = ROUTE_PS_DENSE
    elif kind == KIND_FC:
        route_alg3 = ROUTE_SFB if cost_sfb <= cost_sf_ps else ROUTE_SF_PS
        route_vs_dense = ROUTE_SFB if cost_sfb <= cost_ps_dense else ROUTE_PS_DENSE
    else:
        raise ValueError("unknown layer kind")
    return dict(M=M, N=N, B=B, P=P, kind=kind, cost_sfb=cost_sfb, cost_ps_dense=cost_ps_dense,
                cost_sf_ps=cost_sf_ps, route_alg3=route_alg3, route_vs_dense=route_vs_dense)


def sfb_breakeven_batch(M, N, P):
    """Largest per-worker batch for which Alg. 3 still picks SFB, from solving its
    inequality for B exactly: ((P-1)^2 - P) B (M+N) <= P M N.  None = SFB for every B."""
    c = (P - 1) ** 2 - P
    if c <= 0:
        return None
    return int(Fraction(P * M * N, c * (M + N)))  # floor of a positive rational


# --------------------------------------------------------------------------------------
# Key-range shards
# --------------------------------------------------------------------------------------
def shard_range(n, S, s):
    if not (1 <= S <= n) or not (0 <= s < S):
        raise ValueError("need 1 <= S <= n and 0 <= s < S")
    return (s * n) // S, ((s + 1) * n) // S


# --------------------------------------------------------------------------------------
# bf16 (this build's extension; the paper is fp32 throughout)
# --------------------------------------------------------------------------------------
def bf16_round_bits(x):
    """fp32 array -> uint16 bf16 bit patterns, round to nearest even."""
    a, pa = _f32(x)
    out = np.empty(a.shape, dtype=np.uint16)
    lib().orc_bf16_round_array(pa, out.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)), a.size)
    return out


def bf16_widen(bits):
    """uint16 bf16 bit patterns -> the fp32 values they denote (exact)."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32)


# --------------------------------------------------------------------------------------
# Pack / stack (SFB steps 1-2 seen from the receiver: P blocks of B samples -> K rows)
# --------------------------------------------------------------------------------------
def pack_factors(delta, act, out_dtype="f32"):
    """Stack per-worker blocks: U[p*B+b] = delta[p][b], V[p*B+b] = act[p][b].

    out_dtype "f32": float32 arrays; "bf16": uint16 bit patterns (RNE)."""
    P = len(delta)
    B, N = delta[0].shape
    M = act[0].shape[1]
    U = np.empty((P * B, N), dtype=np.float32)
    V = np.empty((P * B, M), dtype=np.float32)
    for p in range(P):
        for b in range(B):
            U[p * B + b, :] = delta[p][b, :]
            V[p * B + b, :] = act[p][b, :]
    if out_dtype == "f32":
        return U, V
    if out_dtype == "bf16":
        return bf16_round_bits(U), bf16_round_bits(V)
    raise ValueError(out_dtype)


def _factor_values(X):
    """Stacked factors as the fp32 values the arithmetic sees."""
    X = np.asarray(X)
    if X.dtype == np.uint16:
        return np.ascontiguousarray(bf16_widen(X))
    return np.ascontiguousarray(X, dtype=np.float32)


# --------------------------------------------------------------------------------------
# Reconstruction and update
# --------------------------------------------------------------------------------------
def rebuild(U, V):
    """dW (N x M, float64) = sum_k U[k]^T V[k]  (Eq. 5 summed over all stacked samples)."""
    U, V = _factor_values(U), _factor_values(V)
    K, N = U.shape
    K2, M = V.shape
    if K != K2:
        raise ValueError("U and V must stack the same number of samples")
    dW = np.empty((N, M), dtype=np.float64)
    lib().orc_rebuild(U.ctypes.data_as(ctypes.POINTER(ctypes.c_float)),
                      V.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), K, N, M,
                      dW.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    return dW


def rebuild_samples(U, V, idx_n, idx_m):
    U, V = _factor_values(U), _factor_values(V)
    K, N = U.shape
    M = V.shape[1]
    idx_n = np.ascontiguousarray(idx_n, dtype=np.int64)
    idx_m = np.ascontiguousarray(idx_m, dtype=np.int64)
    assert idx_n.shape == idx_m.shape and idx_n.min() >= 0 and idx_n.max() < N
    assert idx_m.min() >= 0 and idx_m.max() < M
    out = np.empty(idx_n.shape, dtype=np.float64)
    i64p = ctypes.POINTER(ctypes.c_int64)
    lib().orc_rebuild_samples(U.ctypes.data_as(ctypes.POINTER(ctypes.c_float)),
                              V.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), K, N, M,
                              idx_n.ctypes.data_as(i64p), idx_m.ctypes.data_as(i64p),
                              idx_n.size, out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    return out


def momentum_update(dW, W, Mom, lr, mu, wd=0.0):
    """Returns (W', Mom') as new float32 arrays; mom' = mu*mom + lr*(dW + wd*w), w' = w - mom'."""
    dW = np.ascontiguousarray(dW, dtype=np.float64)
    W2 = np.array(W, dtype=np.float32, copy=True, order="C")
    Mom2 = np.array(Mom, dtype=np.float32, copy=True, order="C")
    assert dW.shape == W2.shape == Mom2.shape
    lib().orc_update(dW.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
                     W2.ctypes.data_as(ctypes.POINTER(ctypes.c_float)),
                     Mom2.ctypes.data_as(ctypes.POINTER(ctypes.c_float)),
                     np.float32(lr), np.float32(mu), np.float32(wd), W2.size)
    return W2, Mom2


def sync_fc_sfb(U, V, W, Mom, lr, mu, wd=0.0):
    """Alg. 3 SFB branch on one worker: rebuild from all stacked factors, then update."""
    return momentum_update(rebuild(U, V), W, Mom, lr, mu, wd)


def bias_grad(U):
    """db (N, float64) = sum_k U[k]: gradient of the loss w.r.t. the bias of z = W a + b."""
    U = _factor_values(U)
    K, N = U.shape
    db = np.empty(N, dtype=np.float64)
    lib().orc_bias_grad(U.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), K, N,
                        db.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    return db


def sync_fc_bias(U, bias, mom_bias, lr, mu, wd=0.0):
    """Bias of an FC layer under SFB: column sums of the stacked errors, then the same update."""
    return momentum_update(bias_grad(U), bias, mom_bias, lr, mu, wd)


def sync_dense_ps(G, W, Mom, lr, mu, S=1, wd=0.0):
    """Server side of the PS route: per key-range shard, sum the P copies and update."""
    P = len(G)
    Gc = [np.ascontiguousarray(g, dtype=np.float32).ravel() for g in G]
    n = Gc[0].size
    assert all(g.size == n for g in Gc)
    if not (1 <= S <= max(n, 1)):
        raise ValueError("need 1 <= S <= n")
    W2 = np.array(W, dtype=np.float32, copy=True, order="C")
    Mom2 = np.array(Mom, dtype=np.float32, copy=True, order="C")
    f32p = ctypes.POINTER(ctypes.c_float)
    ptrs = (f32p * P)(*[g.ctypes.data_as(f32p) for g in Gc])
    lib().orc_dense_ps(ptrs, P, n, S, W2.ctypes.data_as(f32p), Mom2.ctypes.data_as(f32p),
                       np.float32(lr), np.float32(mu), np.float32(wd))
    return W2, Mom2


# --------------------------------------------------------------------------------------
# Bounded staleness (stale synchronous parallel consistency, Section 3.2)
# --------------------------------------------------------------------------------------
def ssp_updates_visible(t, s):
    """How many clocks' updates a worker that reads the parameters at clock t is guaranteed to see under
    staleness s: those of clocks 0 .. t-s-1 (Section 3.2), i.e. max(0, t - s).  s = 0 is bulk
    synchronous: every earlier clock."""
    t, s = int(t), int(s)
    if t < 0 or s < 0:
        raise ValueError("clock and staleness are non-negative")
    return max(0, t - s)


def ssp_visible_state(updates, W0, Mom0, s, t):
    """Parameters (W, Mom) as guaranteed visible to a reader at clock t under staleness s.

    updates[c] is a function (W, Mom) -> (W', Mom') applying the summed update of clock c (for example
    lambda W, M: sync_fc_sfb(U_c, V_c, W, M, lr, mu)).  The updates of clocks 0 .. t-s-1 are applied in
    clock order; later clocks' updates are still pending and not part of the guaranteed view."""
    W = np.array(W0, dtype=np.float32, copy=True)
    Mom = np.array(Mom0, dtype=np.float32, copy=True)
    for c in range(ssp_updates_visible(t, s)):
        W, Mom = updates[c](W, Mom)
    return W, Mom


def rel_frob(x, ref):
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    d = np.linalg.norm((x - ref).ravel())
    r = np.linalg.norm(ref.ravel())
    return d / r if r > 0 else d
