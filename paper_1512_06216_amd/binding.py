"""ctypes binding of libpsd.so (declared in include/psd.h): argument marshalling only.

Every step of the path runs inside the library's HIP kernels; torch is used for device
memory and streams.  There is no CPU fallback: if the library has not been built, the
first call raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libpsd.so")

OK, E_INVALID, E_NULL, E_UNSUPPORTED, E_OVERFLOW, E_HIP, E_WORKSPACE = 0, -1, -2, -3, -4, -5, -6
LAYER_CONV, LAYER_FC = 0, 1
ROUTE_PS_DENSE, ROUTE_SFB, ROUTE_SF_PS = 0, 1, 2
RULE_ALG3, RULE_SFB_VS_DENSE = 0, 1
F32, BF16 = 0, 1
TUNE_SFB_BF16_TILE, TUNE_SFB_F32_TILE, TUNE_SFB_BF16_SKEW_US = 0, 1, 2
ROUTE_NAMES = {ROUTE_PS_DENSE: "PS_DENSE", ROUTE_SFB: "SFB", ROUTE_SF_PS: "SF_PS"}
MAX_WORKERS, MAX_MULTI_SEGMENTS, MAX_MULTI_WORKERS = 64, 16, 16
STATIC_SCRATCH_BYTES = 16 << 20

_f32p = ctypes.POINTER(ctypes.c_float)
_f32pp = ctypes.POINTER(_f32p)


class Plan(ctypes.Structure):
    _fields_ = [("M", ctypes.c_int64), ("N", ctypes.c_int64), ("B", ctypes.c_int64), ("P", ctypes.c_int64),
                ("kind", ctypes.c_int32), ("route_alg3", ctypes.c_int32), ("route_vs_dense", ctypes.c_int32),
                ("reserved", ctypes.c_int32), ("cost_sfb", ctypes.c_uint64), ("cost_ps_dense", ctypes.c_uint64),
                ("cost_sf_ps", ctypes.c_uint64)]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_ if k != "reserved"}

    @property
    def K(self):
        return self.P * self.B


class DenseSegment(ctypes.Structure):
    _fields_ = [("n", ctypes.c_int64), ("P", ctypes.c_int32), ("S", ctypes.c_int32), ("G", _f32pp),
                ("W", _f32p), ("Mom", _f32p)]


class SspState(ctypes.Structure):
    _fields_ = [("s", ctypes.c_int32), ("reserved", ctypes.c_int32), ("clock", ctypes.c_int64)]


class LayerTask(ctypes.Structure):
    _fields_ = [("plan", Plan), ("factor_dtype", ctypes.c_int32), ("S", ctypes.c_int32),
                ("delta_p", _f32pp), ("act_p", _f32pp),
                ("U", ctypes.c_void_p), ("ldu", ctypes.c_int64), ("V", ctypes.c_void_p), ("ldv", ctypes.c_int64),
                ("G", _f32pp), ("W", _f32p), ("Mom", _f32p), ("workspace", ctypes.c_void_p),
                ("workspace_bytes", ctypes.c_size_t), ("stream", ctypes.c_void_p),
                ("ev_ready", ctypes.c_void_p), ("ev_begin", ctypes.c_void_p), ("ev_end", ctypes.c_void_p)]


class PsdError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = lib().psd_status_string(status).decode()
        if status == E_HIP:
            msg += " [hipError %d]" % lib().psd_last_hip_error()
        super().__init__("%s: %s (status %d)" % (where, msg, status))


# name -> (restype, argtypes); also the list of symbols the header declares
SIGNATURES = {
    "psd_plan_layer": (ctypes.c_int32, [ctypes.c_int32, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                        ctypes.c_int64, ctypes.POINTER(Plan)]),
    "psd_shard_range": (ctypes.c_int32, [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32,
                                         ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int64)]),
    "psd_factor_ld": (ctypes.c_int64, [ctypes.c_int64, ctypes.c_int32]),
    "psd_pack_factors": (ctypes.c_int32, [ctypes.POINTER(Plan), _f32pp, _f32pp, ctypes.c_int32, ctypes.c_void_p,
                                          ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]),
    "psd_sync_fc_sfb": (ctypes.c_int32, [ctypes.POINTER(Plan), ctypes.c_int32, ctypes.c_void_p, ctypes.c_int64,
                                         ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p,
                                         ctypes.c_float, ctypes.c_float, ctypes.c_float, ctypes.c_void_p,
                                         ctypes.c_size_t, ctypes.c_void_p]),
    "psd_sfb_workspace_bytes": (ctypes.c_size_t, [ctypes.POINTER(Plan), ctypes.c_int32]),
    "psd_sync_fc_sfb_static": (ctypes.c_int32, [ctypes.POINTER(Plan), ctypes.c_int32, ctypes.c_void_p, ctypes.c_int64,
                                                ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p,
                                                ctypes.c_float, ctypes.c_float, ctypes.c_float, ctypes.c_void_p]),
    "psd_sfb_blocks_supported": (ctypes.c_int32, [ctypes.POINTER(Plan), ctypes.c_int32, ctypes.c_int64, ctypes.c_int64]),
    "psd_sync_fc_sfb_blocks": (ctypes.c_int32, [ctypes.POINTER(Plan), ctypes.c_int32, _f32pp, ctypes.c_int64, _f32pp,
                                                ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_float,
                                                ctypes.c_float, ctypes.c_float, ctypes.c_void_p]),
    "psd_sync_fc_bias": (ctypes.c_int32, [ctypes.POINTER(Plan), ctypes.c_int32, ctypes.c_void_p, ctypes.c_int64,
                                          ctypes.c_void_p, ctypes.c_void_p, ctypes.c_float, ctypes.c_float,
                                          ctypes.c_float, ctypes.c_void_p]),
    "psd_sync_dense_ps": (ctypes.c_int32, [ctypes.c_int64, ctypes.c_int32, _f32pp, ctypes.c_void_p, ctypes.c_void_p,
                                           ctypes.c_float, ctypes.c_float, ctypes.c_float, ctypes.c_int32,
                                           ctypes.c_void_p]),
    "psd_sync_dense_ps_multi": (ctypes.c_int32, [ctypes.c_int32, ctypes.POINTER(DenseSegment), ctypes.c_float,
                                                 ctypes.c_float, ctypes.c_float, ctypes.c_void_p]),
    "psd_sync_iteration": (ctypes.c_int32, [ctypes.c_int32, ctypes.POINTER(LayerTask), ctypes.c_float,
                                            ctypes.c_float, ctypes.c_float, ctypes.c_int32]),
    "psd_ssp_init": (ctypes.c_int32, [ctypes.POINTER(SspState), ctypes.c_int32]),
    "psd_ssp_slots": (ctypes.c_int32, [ctypes.POINTER(SspState), ctypes.POINTER(ctypes.c_int32),
                                       ctypes.POINTER(ctypes.c_int32)]),
    "psd_ssp_clock_fc": (ctypes.c_int32, [ctypes.POINTER(SspState), ctypes.POINTER(Plan), ctypes.c_int32, _f32pp, _f32pp,
                                          ctypes.POINTER(ctypes.c_void_p), ctypes.c_int64,
                                          ctypes.POINTER(ctypes.c_void_p), ctypes.c_int64, ctypes.c_void_p,
                                          ctypes.c_void_p, ctypes.c_float, ctypes.c_float, ctypes.c_float,
                                          ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]),
    "psd_ssp_clock_dense": (ctypes.c_int32, [ctypes.POINTER(SspState), ctypes.c_int64, ctypes.c_int32,
                                             ctypes.POINTER(_f32pp), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_float,
                                             ctypes.c_float, ctypes.c_float, ctypes.c_int32, ctypes.c_void_p]),
    "psd_tune_set": (ctypes.c_int32, [ctypes.c_int32, ctypes.c_int32]),
    "psd_status_string": (ctypes.c_char_p, [ctypes.c_int32]),
    "psd_last_hip_error": (ctypes.c_int32, []),
    "psd_version": (ctypes.c_int32, []),
}

_lib = None


def lib():
    """Loads libpsd.so; raises if it is missing (build it with __graft_entry__.build())."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libpsd.so is not built (%s): run `python -c 'import __graft_entry__ as g; "
                               "g.build()'`; there is no fallback path" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


def _check(status, where):
    if status != OK:
        raise PsdError(status, where)


def _stream_handle(stream):
    if stream is None:
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)


def _dev_ptr(t, dtype, min_elems, what):
    """Device pointer of a tensor after checking it can hold what the kernel will touch."""
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous()):
        raise ValueError("%s must be a contiguous CUDA tensor" % what)
    if t.dtype not in (dtype if isinstance(dtype, tuple) else (dtype,)):
        raise ValueError("%s has dtype %s" % (what, t.dtype))
    if t.numel() < min_elems:
        raise ValueError("%s holds %d elements, needs %d" % (what, t.numel(), min_elems))
    return t.data_ptr()


def _ptr_array(tensors, min_elems, what, dtype=torch.float32):
    arr = (_f32p * len(tensors))()
    for i, t in enumerate(tensors):
        arr[i] = ctypes.cast(_dev_ptr(t, dtype, min_elems, "%s[%d]" % (what, i)), _f32p)
    return arr


_FACTOR_TORCH = {F32: (torch.float32,), BF16: (torch.bfloat16, torch.int16, torch.uint16)}


# ---------------------------------------------------------------------------------------
def plan_layer(kind, M, N, B, P):
    p = Plan()
    _check(lib().psd_plan_layer(kind, M, N, B, P, ctypes.byref(p)), "psd_plan_layer")
    return p


def tune_set(knob, value):
    """Pins (or with -1 releases) a kernel tile choice; tuning / test hook."""
    _check(lib().psd_tune_set(knob, value), "psd_tune_set")


def shard_range(n, S, s):
    b, e = ctypes.c_int64(), ctypes.c_int64()
    _check(lib().psd_shard_range(n, S, s, ctypes.byref(b), ctypes.byref(e)), "psd_shard_range")
    return b.value, e.value


def factor_ld(cols, dtype):
    ld = lib().psd_factor_ld(cols, dtype)
    if ld <= 0:
        raise PsdError(E_INVALID, "psd_factor_ld")
    return ld


def alloc_factors(plan, dtype, device="cuda"):
    """Device buffers for the stacked factors: (U, ldu, V, ldv).  Memory only."""
    ldu, ldv = factor_ld(plan.N, dtype), factor_ld(plan.M, dtype)
    td = torch.float32 if dtype == F32 else torch.bfloat16
    U = torch.empty((plan.K, ldu), dtype=td, device=device)
    V = torch.empty((plan.K, ldv), dtype=td, device=device)
    return U, ldu, V, ldv


def pack_factors(plan, delta, act, out_dtype, U, ldu, V, ldv, stream=None):
    if len(delta) != plan.P or len(act) != plan.P:
        raise ValueError("need P per-worker blocks")
    d = _ptr_array(delta, plan.B * plan.N, "delta")
    a = _ptr_array(act, plan.B * plan.M, "act")
    up = _dev_ptr(U, _FACTOR_TORCH.get(out_dtype, ()), plan.K * ldu, "U")
    vp = _dev_ptr(V, _FACTOR_TORCH.get(out_dtype, ()), plan.K * ldv, "V")
    _check(lib().psd_pack_factors(ctypes.byref(plan), d, a, out_dtype, up, ldu, vp, ldv, _stream_handle(stream)),
           "psd_pack_factors")


def sfb_workspace_bytes(plan, factor_dtype):
    return int(lib().psd_sfb_workspace_bytes(ctypes.byref(plan), factor_dtype))


def alloc_workspace(plan, factor_dtype, device="cuda"):
    """Device scratch of the queried size, or None if the layer would not use one.  Memory only."""
    n = sfb_workspace_bytes(plan, factor_dtype)
    return torch.empty(n // 4, dtype=torch.float32, device=device) if n else None


def _workspace_args(workspace):
    if workspace is None:
        return None, 0
    if not (isinstance(workspace, torch.Tensor) and workspace.is_cuda and workspace.is_contiguous()):
        raise ValueError("workspace must be a contiguous CUDA tensor")
    return workspace.data_ptr(), workspace.numel() * workspace.element_size()


def sync_fc_sfb(plan, factor_dtype, U, ldu, V, ldv, W, Mom, lr, mu, stream=None, wd=0.0, workspace=None):
    up = _dev_ptr(U, _FACTOR_TORCH.get(factor_dtype, ()), plan.K * ldu, "U")
    vp = _dev_ptr(V, _FACTOR_TORCH.get(factor_dtype, ()), plan.K * ldv, "V")
    wp = _dev_ptr(W, torch.float32, plan.N * plan.M, "W")
    mp = _dev_ptr(Mom, torch.float32, plan.N * plan.M, "Mom")
    ws, ws_bytes = _workspace_args(workspace)
    _check(lib().psd_sync_fc_sfb(ctypes.byref(plan), factor_dtype, up, ldu, vp, ldv, wp, mp, lr, mu, wd,
                                 ws, ws_bytes, _stream_handle(stream)), "psd_sync_fc_sfb")


def sync_fc_sfb_static(plan, factor_dtype, U, ldu, V, ldv, W, Mom, lr, mu, stream=None, wd=0.0):
    """sync_fc_sfb on the library's own fixed scratch array (allocates nothing)."""
    up = _dev_ptr(U, _FACTOR_TORCH.get(factor_dtype, ()), plan.K * ldu, "U")
    vp = _dev_ptr(V, _FACTOR_TORCH.get(factor_dtype, ()), plan.K * ldv, "V")
    wp = _dev_ptr(W, torch.float32, plan.N * plan.M, "W")
    mp = _dev_ptr(Mom, torch.float32, plan.N * plan.M, "Mom")
    _check(lib().psd_sync_fc_sfb_static(ctypes.byref(plan), factor_dtype, up, ldu, vp, ldv, wp, mp, lr, mu, wd,
                                        _stream_handle(stream)), "psd_sync_fc_sfb_static")


def sfb_blocks_supported(plan, factor_dtype=F32, ldu=0, ldv=0):
    """ldu / ldv = 0: dense blocks (rows of N and M elements)."""
    return bool(lib().psd_sfb_blocks_supported(ctypes.byref(plan), factor_dtype, ldu or plan.N, ldv or plan.M))


def sync_fc_sfb_blocks(plan, factor_dtype, U_blocks, ldu, V_blocks, ldv, W, Mom, lr, mu, stream=None, wd=0.0):
    """Reconstruction + update straight from the P per-worker blocks (B x ldu and B x ldv elements of
    factor_dtype each), no stacked copy.  ldu / ldv = 0: dense blocks."""
    if len(U_blocks) != plan.P or len(V_blocks) != plan.P:
        raise ValueError("need P per-worker blocks")
    ldu, ldv = ldu or plan.N, ldv or plan.M
    fd = _FACTOR_TORCH.get(factor_dtype, ())
    d = _ptr_array(U_blocks, plan.B * ldu, "U_blocks", fd)
    a = _ptr_array(V_blocks, plan.B * ldv, "V_blocks", fd)
    wp = _dev_ptr(W, torch.float32, plan.N * plan.M, "W")
    mp = _dev_ptr(Mom, torch.float32, plan.N * plan.M, "Mom")
    _check(lib().psd_sync_fc_sfb_blocks(ctypes.byref(plan), factor_dtype, d, ldu, a, ldv, wp, mp, lr, mu, wd,
                                        _stream_handle(stream)), "psd_sync_fc_sfb_blocks")


def sync_fc_bias(plan, factor_dtype, U, ldu, bias, mom_bias, lr, mu, stream=None, wd=0.0):
    up = _dev_ptr(U, _FACTOR_TORCH.get(factor_dtype, ()), plan.K * ldu, "U")
    bp = _dev_ptr(bias, torch.float32, plan.N, "bias")
    mp = _dev_ptr(mom_bias, torch.float32, plan.N, "mom_bias")
    _check(lib().psd_sync_fc_bias(ctypes.byref(plan), factor_dtype, up, ldu, bp, mp, lr, mu, wd,
                                  _stream_handle(stream)), "psd_sync_fc_bias")


def sync_dense_ps(G, W, Mom, lr, mu, S, stream=None, wd=0.0):
    n = W.numel()
    g = _ptr_array(G, n, "G")
    wp = _dev_ptr(W, torch.float32, n, "W")
    mp = _dev_ptr(Mom, torch.float32, n, "Mom")
    _check(lib().psd_sync_dense_ps(n, len(G), g, wp, mp, lr, mu, wd, S, _stream_handle(stream)),
           "psd_sync_dense_ps")


class DenseMulti:
    """Marshalled, reusable argument block for psd_sync_dense_ps_multi.  layers: list of (G_list, W, Mom, S)."""

    def __init__(self, layers):
        self.segs = (DenseSegment * len(layers))()
        self._keep = []
        for i, (G, W, Mom, S) in enumerate(layers):
            n = W.numel()
            g = _ptr_array(G, n, "G")
            self._keep.append(g)
            self.segs[i].n, self.segs[i].P, self.segs[i].S = n, len(G), S
            self.segs[i].G = ctypes.cast(g, _f32pp)
            self.segs[i].W = ctypes.cast(_dev_ptr(W, torch.float32, n, "W"), _f32p)
            self.segs[i].Mom = ctypes.cast(_dev_ptr(Mom, torch.float32, n, "Mom"), _f32p)
        self.L = len(layers)

    def run(self, lr, mu, stream=None, wd=0.0):
        _check(lib().psd_sync_dense_ps_multi(self.L, self.segs, lr, mu, wd, _stream_handle(stream)),
               "psd_sync_dense_ps_multi")


def sync_dense_ps_multi(layers, lr, mu, stream=None, wd=0.0):
    """layers: list of (G_list, W, Mom, S)."""
    DenseMulti(layers).run(lr, mu, stream, wd)


MAX_STALENESS = 15


class SspFc:
    """An FC layer under staleness s: the clock state and the ring of s+1 stacked-factor buffers
    (memory only; every clock is one library call)."""

    def __init__(self, plan, factor_dtype, s, device="cuda"):
        self.plan, self.dtype, self.state = plan, factor_dtype, SspState()
        _check(lib().psd_ssp_init(ctypes.byref(self.state), s), "psd_ssp_init")
        self.bufs = [alloc_factors(plan, factor_dtype, device) for _ in range(s + 1)]
        self.ldu, self.ldv = self.bufs[0][1], self.bufs[0][3]
        self.U_ring = (ctypes.c_void_p * (s + 1))(*[b[0].data_ptr() for b in self.bufs])
        self.V_ring = (ctypes.c_void_p * (s + 1))(*[b[2].data_ptr() for b in self.bufs])

    def slots(self):
        a, b = ctypes.c_int32(), ctypes.c_int32()
        _check(lib().psd_ssp_slots(ctypes.byref(self.state), ctypes.byref(a), ctypes.byref(b)), "psd_ssp_slots")
        return a.value, b.value

    def clock(self, delta, act, W, Mom, lr, mu, wd=0.0, workspace=None, stream=None):
        """delta / act: this clock's per-worker blocks, or None, None to drain."""
        plan = self.plan
        d = _ptr_array(delta, plan.B * plan.N, "delta") if delta is not None else None
        a = _ptr_array(act, plan.B * plan.M, "act") if act is not None else None
        ws, ws_bytes = _workspace_args(workspace)
        _check(lib().psd_ssp_clock_fc(ctypes.byref(self.state), ctypes.byref(plan), self.dtype, d, a, self.U_ring, self.ldu,
                                      self.V_ring, self.ldv, _dev_ptr(W, torch.float32, plan.N * plan.M, "W"),
                                      _dev_ptr(Mom, torch.float32, plan.N * plan.M, "Mom"), lr, mu, wd, ws, ws_bytes,
                                      _stream_handle(stream)), "psd_ssp_clock_fc")


class SspDense:
    """A parameter-server layer under staleness s: the clock state and the ring of s+1 sets of P
    gradient copies (the caller's tensors; this object only keeps the pointer table)."""

    def __init__(self, s):
        self.state = SspState()
        _check(lib().psd_ssp_init(ctypes.byref(self.state), s), "psd_ssp_init")
        self.ring = (_f32pp * (s + 1))()
        self._keep = [None] * (s + 1)

    def clock(self, G, W, Mom, lr, mu, S, wd=0.0, stream=None):
        """G: this clock's P copies (kept alive by this object until their slot is reused), or None to drain."""
        n = W.numel()
        push = self.state.clock % (self.state.s + 1)
        P = None
        if G is not None:
            arr = _ptr_array(G, n, "G")
            self._keep[push] = (arr, list(G))
            self.ring[push] = ctypes.cast(arr, _f32pp)
        for k in self._keep:
            if k is not None:
                P = len(k[1])
        if P is None:
            raise ValueError("no gradient copies have been pushed yet")
        _check(lib().psd_ssp_clock_dense(ctypes.byref(self.state), n, P, self.ring, _dev_ptr(W, torch.float32, n, "W"),
                                         _dev_ptr(Mom, torch.float32, n, "Mom"), lr, mu, wd, S, _stream_handle(stream)),
               "psd_ssp_clock_dense")


class Iteration:
    """Marshalled, reusable argument block for psd_sync_iteration (layers bottom-up).

    Each layer is a dict: FC  -> plan, factor_dtype, delta, act, U, ldu, V, ldv, W, Mom, stream[, workspace]
                                 (U = V = None: delta / act are blocks of factor_dtype with leading dimensions
                                 ldu / ldv (0 or absent = dense) that are read in place, nothing is stacked)
                         conv -> plan, G, S, W, Mom, stream
    plus optional ev_ready (the layer's stream waits for it first) and ev_begin / ev_end (recorded
    around the layer's sync kernel); all raw hipEvent_t handles as ints.
    Building it does no device work; run() makes the single library call.
    """

    def __init__(self, layers):
        self.tasks = (LayerTask * len(layers))()
        self._keep = []
        for i, L in enumerate(layers):
            t = self.tasks[i]
            plan = L["plan"]
            t.plan = plan
            n = plan.M * plan.N
            t.W = ctypes.cast(_dev_ptr(L["W"], torch.float32, n, "W"), _f32p)
            t.Mom = ctypes.cast(_dev_ptr(L["Mom"], torch.float32, n, "Mom"), _f32p)
            t.stream = _stream_handle(L.get("stream"))
            t.workspace, t.workspace_bytes = _workspace_args(L.get("workspace"))
            self._keep.append(L.get("workspace"))
            t.ev_ready = L.get("ev_ready")
            t.ev_begin, t.ev_end = L.get("ev_begin"), L.get("ev_end")   # raw hipEvent_t handles or None
            t.S = L.get("S", 1)
            t.factor_dtype = L.get("factor_dtype", F32)
            if L.get("G") is not None:
                g = _ptr_array(L["G"], n, "G")
                self._keep.append(g)
                t.G = ctypes.cast(g, _f32pp)
            if L.get("delta") is not None:
                fd = _FACTOR_TORCH.get(t.factor_dtype, ())
                if L.get("U") is not None or L.get("V") is not None:
                    d = _ptr_array(L["delta"], plan.B * plan.N, "delta")
                    a = _ptr_array(L["act"], plan.B * plan.M, "act")
                    t.U, t.ldu = _dev_ptr(L["U"], fd, plan.K * L["ldu"], "U"), L["ldu"]
                    t.V, t.ldv = _dev_ptr(L["V"], fd, plan.K * L["ldv"], "V"), L["ldv"]
                else:
                    # no stacked buffers: delta / act are blocks of factor_dtype, read in place
                    t.ldu, t.ldv = L.get("ldu") or plan.N, L.get("ldv") or plan.M
                    d = _ptr_array(L["delta"], plan.B * t.ldu, "delta", fd)
                    a = _ptr_array(L["act"], plan.B * t.ldv, "act", fd)
                self._keep += [d, a]
                t.delta_p, t.act_p = ctypes.cast(d, _f32pp), ctypes.cast(a, _f32pp)
        self.L = len(layers)

    def run(self, lr, mu, rule=RULE_ALG3, wd=0.0):
        _check(lib().psd_sync_iteration(self.L, self.tasks, lr, mu, wd, rule), "psd_sync_iteration")
