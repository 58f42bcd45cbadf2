"""Parity of the HIP path (through the C ABI) with the CPU oracle, element by element.

Bars: bit-exact for packing, shard indexing, route decisions and for integer-valued
inputs (every partial sum below 2^24, so fp32 results do not depend on summation order);
relative Frobenius error <= 1e-5 for fp32 factors and for bf16 factors against the oracle
fed the same rounded factors; <= 2e-2 for bf16 factors against the oracle fed the
unrounded fp32 factors.  Errors are taken on three tensors: Mom', W' - W, and W'.
"""
import numpy as np
import pytest
import torch

from oracle import psd_oracle as orc
from paper_1512_06216_amd import binding as psd
from paper_1512_06216_amd import inputs

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-5
TOL_BF16_VS_F32 = 2e-2
DEV = "cuda:0"


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def bits16(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def three_errors(W0, W_gpu, Mom_gpu, W_ref, Mom_ref):
    W0 = W0.astype(np.float64)
    return (orc.rel_frob(Mom_gpu, Mom_ref),
            orc.rel_frob(W_gpu.astype(np.float64) - W0, W_ref.astype(np.float64) - W0),
            orc.rel_frob(W_gpu, W_ref))


def run_pack(d, dtype):
    plan = psd.plan_layer(psd.LAYER_FC, d["M"], d["N"], d["B"], d["P"])
    U, ldu, V, ldv = psd.alloc_factors(plan, dtype, DEV)
    # poison so that unwritten elements show
    U.view(torch.int16).fill_(0x7fc1)
    V.view(torch.int16).fill_(0x7fc1)
    delta = [dev(x) for x in d["delta"]]
    act = [dev(x) for x in d["act"]]
    psd.pack_factors(plan, delta, act, dtype, U, ldu, V, ldv)
    torch.cuda.synchronize()
    return plan, U, ldu, V, ldv


def run_sfb(d, dtype, lr, mu):
    plan, U, ldu, V, ldv = run_pack(d, dtype)
    W, Mom = dev(d["W"]), dev(d["Mom"])
    psd.sync_fc_sfb(plan, dtype, U, ldu, V, ldv, W, Mom, lr, mu)
    torch.cuda.synchronize()
    return W.cpu().numpy(), Mom.cpu().numpy(), (U, V)


# ---------------------------------------------------------------------------------------
# pack / stack: bit-exact
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("M,N,B,P", [(256, 128, 32, 4), (37, 29, 3, 5), (1, 1, 1, 1), (1001, 2185, 7, 3),
                                     (8, 21841, 2, 2), (4096, 1000, 16, 8)])
@pytest.mark.parametrize("dtype", [psd.F32, psd.BF16])
def test_pack_bit_exact(M, N, B, P, dtype):
    d = inputs.fc_layer(M, N, B, P, seed=100 + M % 7)
    # make a few values special so that rounding corner cases travel through the kernel
    d["delta"][0].flat[0] = np.float32(1.0 + 2.0 ** -8)       # bf16 tie
    d["act"][P - 1].flat[-1] = np.float32(np.inf)
    d["act"][0].flat[0] = np.float32(1e-40)                    # subnormal
    plan, U, ldu, V, ldv = run_pack(d, dtype)
    name = "f32" if dtype == psd.F32 else "bf16"
    Uo, Vo = orc.pack_factors(d["delta"], d["act"], name)
    if dtype == psd.F32:
        Ug, Vg = U.cpu().numpy().view(np.uint32), V.cpu().numpy().view(np.uint32)
        Uo, Vo = Uo.view(np.uint32), Vo.view(np.uint32)
    else:
        Ug, Vg = bits16(U), bits16(V)
    assert np.array_equal(Ug[:, :N], Uo) and np.array_equal(Vg[:, :M], Vo)
    assert not Ug[:, N:].any() and not Vg[:, M:].any()          # padding columns are zero


def test_pack_maximum_worker_count():
    d = inputs.fc_layer(40, 24, 1, 64, seed=64)                  # P = 64 workers, one sample each
    for dtype, name in ((psd.F32, "f32"), (psd.BF16, "bf16")):
        plan, U, ldu, V, ldv = run_pack(d, dtype)
        Uo, Vo = orc.pack_factors(d["delta"], d["act"], name)
        Ug = U.cpu().numpy().view(np.uint32) if dtype == psd.F32 else bits16(U)
        Vg = V.cpu().numpy().view(np.uint32) if dtype == psd.F32 else bits16(V)
        Uo = Uo.view(np.uint32) if dtype == psd.F32 else Uo
        Vo = Vo.view(np.uint32) if dtype == psd.F32 else Vo
        assert np.array_equal(Ug[:, :24], Uo) and np.array_equal(Vg[:, :40], Vo)


def test_pack_nan_stays_nan():
    d = inputs.fc_layer(16, 8, 2, 2, seed=3)
    d["delta"][1][1, 3] = np.float32(np.nan)
    plan, U, ldu, V, ldv = run_pack(d, psd.BF16)
    Uo, _ = orc.pack_factors(d["delta"], d["act"], "bf16")
    assert np.array_equal(bits16(U)[:, :8], Uo)


# ---------------------------------------------------------------------------------------
# dense parameter-server route
# ---------------------------------------------------------------------------------------
DENSE_CASES = [(1, 1, 1), (3, 2, 3), (5, 8, 1), (1000, 8, 8), (1003, 3, 7), (2051, 8, 8), (34848, 8, 8),
               (4099, 5, 4099), (70001, 17, 8), (307200, 8, 8), (9, 64, 2), (65536 + 13, 4, 1), (8197, 16, 3)]


@pytest.mark.parametrize("n,P,S", DENSE_CASES)
def test_dense_integer_inputs_bit_exact(n, P, S):
    d = inputs.dense_layer_integer(n, P, seed=n % 101)
    W, Mom = dev(d["W"]), dev(d["Mom"])
    psd.sync_dense_ps([dev(g) for g in d["G"]], W, Mom, 0.125, 0.5, S)
    torch.cuda.synchronize()
    Wr, Mr = orc.sync_dense_ps(d["G"], d["W"], d["Mom"], 0.125, 0.5, S)
    assert np.array_equal(W.cpu().numpy(), Wr) and np.array_equal(Mom.cpu().numpy(), Mr)


@pytest.mark.parametrize("n,P,S", [(34848, 8, 8), (884736, 8, 8), (100003, 3, 5)])
def test_dense_gaussian(n, P, S):
    d = inputs.dense_layer(n, P, seed=n % 103, mom_std=1e-3)
    W, Mom = dev(d["W"]), dev(d["Mom"])
    psd.sync_dense_ps([dev(g) for g in d["G"]], W, Mom, inputs.LR, inputs.MU, S)
    torch.cuda.synchronize()
    Wr, Mr = orc.sync_dense_ps(d["G"], d["W"], d["Mom"], inputs.LR, inputs.MU, S)
    e = three_errors(d["W"], W.cpu().numpy(), Mom.cpu().numpy(), Wr, Mr)
    assert max(e) <= TOL_F32, e


def test_dense_sharding_does_not_change_bits():
    d = inputs.dense_layer(50021, 8, seed=77, mom_std=1e-3)
    G = [dev(g) for g in d["G"]]
    outs = []
    for S in (1, 2, 8, 13, 50021):
        W, Mom = dev(d["W"]), dev(d["Mom"])
        psd.sync_dense_ps(G, W, Mom, inputs.LR, inputs.MU, S)
        torch.cuda.synchronize()
        outs.append((W.cpu().numpy(), Mom.cpu().numpy()))
    for w, m in outs[1:]:
        assert np.array_equal(w, outs[0][0]) and np.array_equal(m, outs[0][1])


def test_dense_multi_equals_single_calls():
    sizes = inputs.conv_sizes() + [0, 5]
    layers, refs = [], []
    for i, n in enumerate(sizes):
        d = inputs.dense_layer_integer(n, 8 if i % 2 == 0 else 3, seed=200 + i)
        W, Mom = dev(d["W"]), dev(d["Mom"])
        S = 8 if n >= 8 else 1
        layers.append(([dev(g) for g in d["G"]], W, Mom, S))
        refs.append(orc.sync_dense_ps(d["G"], d["W"], d["Mom"], 0.25, 0.5, S))
    psd.sync_dense_ps_multi(layers, 0.25, 0.5)
    torch.cuda.synchronize()
    for (G, W, Mom, S), (Wr, Mr) in zip(layers, refs):
        assert np.array_equal(W.cpu().numpy(), Wr) and np.array_equal(Mom.cpu().numpy(), Mr)


# ---------------------------------------------------------------------------------------
# SFB reconstruct + update
# ---------------------------------------------------------------------------------------
SFB_INT_SHAPES = [  # M, N, B, P  (K = P*B): ragged tiles, K tails, K = 1, odd widths
    (256, 128, 32, 4), (1, 1, 1, 1), (7, 5, 1, 1), (130, 129, 3, 5), (384, 1000, 16, 8), (257, 300, 5, 3),
    (512, 21841 // 16, 8, 2), (640, 520, 33, 1), (96, 64, 1, 17),
]


@pytest.mark.parametrize("M,N,B,P", SFB_INT_SHAPES)
@pytest.mark.parametrize("dtype", [psd.F32, psd.BF16])
def test_sfb_integer_factors_bit_exact(M, N, B, P, dtype):
    d = inputs.fc_layer_integer(M, N, B, P, seed=M + N)
    Wg, Mg, _ = run_sfb(d, dtype, 0.25, 0.5)
    U, V = orc.pack_factors(d["delta"], d["act"])
    Wr, Mr = orc.sync_fc_sfb(U, V, d["W"], d["Mom"], 0.25, 0.5)
    assert np.array_equal(Mg, Mr), np.argwhere(Mg != Mr)[:8]
    assert np.array_equal(Wg, Wr)


@pytest.mark.parametrize("dtype", [psd.F32, psd.BF16])
def test_sfb_smallest_leading_dimensions_bit_exact(dtype):
    """Stacked factors whose rows are padded to 16 bytes only (the least the entry points accept, rows then
    start in the middle of cache lines) instead of the 128 bytes psd_factor_ld recommends."""
    M, N, B, P = 1001, 333, 9, 5
    d = inputs.fc_layer_integer(M, N, B, P, seed=77)
    plan = psd.plan_layer(psd.LAYER_FC, M, N, B, P)
    q = 4 if dtype == psd.F32 else 8
    ldu, ldv = (N + q - 1) // q * q, (M + q - 1) // q * q
    assert (ldu, ldv) != (psd.factor_ld(N, dtype), psd.factor_ld(M, dtype))
    td = torch.float32 if dtype == psd.F32 else torch.bfloat16
    U, V = torch.empty(plan.K, ldu, dtype=td, device=DEV), torch.empty(plan.K, ldv, dtype=td, device=DEV)
    psd.pack_factors(plan, [dev(x) for x in d["delta"]], [dev(x) for x in d["act"]], dtype, U, ldu, V, ldv)
    W, Mom = dev(d["W"]), dev(d["Mom"])
    psd.sync_fc_sfb(plan, dtype, U, ldu, V, ldv, W, Mom, 0.25, 0.5)
    torch.cuda.synchronize()
    Uo, Vo = orc.pack_factors(d["delta"], d["act"])
    Wr, Mr = orc.sync_fc_sfb(Uo, Vo, d["W"], d["Mom"], 0.25, 0.5)
    assert np.array_equal(Mom.cpu().numpy(), Mr) and np.array_equal(W.cpu().numpy(), Wr)


@pytest.fixture
def pinned_tile():
    """Pins a kernel tile through the library's tuning hook and releases it afterwards."""
    pinned = []

    def pin(knob, value):
        psd.tune_set(knob, value)
        pinned.append(knob)
    yield pin
    for knob in pinned:
        psd.tune_set(knob, -1)


@pytest.mark.parametrize("tile", [0, 1, 2])
@pytest.mark.parametrize("M,N,B,P", [(520, 300, 11, 5),       # ragged tiles both ways, K tail, K shorter than the row prefetch
                                     (700, 260, 160, 9)])     # K = 1440: past the unrolled prefetch stages, ragged stage tail
def test_sfb_bf16_every_tile_shape_bit_exact(tile, M, N, B, P, pinned_tile):
    # every kernel instantiation the tile heuristic can pick (and the tuning-only one)
    pinned_tile(psd.TUNE_SFB_BF16_TILE, tile)
    d = inputs.fc_layer_integer(M=M, N=N, B=B, P=P, seed=tile + 50, amax=2 if B * P > 1000 else 3)
    Wg, Mg, _ = run_sfb(d, psd.BF16, 0.25, 0.5)
    U, V = orc.pack_factors(d["delta"], d["act"])
    Wr, Mr = orc.sync_fc_sfb(U, V, d["W"], d["Mom"], 0.25, 0.5)
    assert np.array_equal(Mg, Mr) and np.array_equal(Wg, Wr)


def test_sfb_bf16_phase_skew_changes_no_bit(pinned_tile):
    """The measurement aid that starts half of the chip's first workgroups late only shifts work in time."""
    pinned_tile(psd.TUNE_SFB_BF16_SKEW_US, 15)
    d = inputs.fc_layer_integer(M=1500, N=2100, B=40, P=5, seed=58)        # 17 x 8 tiles of 128 x 192
    Wg, Mg, _ = run_sfb(d, psd.BF16, 0.25, 0.5)
    U, V = orc.pack_factors(d["delta"], d["act"])
    Wr, Mr = orc.sync_fc_sfb(U, V, d["W"], d["Mom"], 0.25, 0.5)
    assert np.array_equal(Mg, Mr) and np.array_equal(Wg, Wr)


@pytest.mark.parametrize("tile", [1, 2])
def test_sfb_f32_both_tile_shapes_bit_exact(tile, pinned_tile):
    pinned_tile(psd.TUNE_SFB_F32_TILE, tile)
    d = inputs.fc_layer_integer(M=391, N=203, B=7, P=3, seed=tile + 60)
    Wg, Mg, _ = run_sfb(d, psd.F32, 0.25, 0.5)
    U, V = orc.pack_factors(d["delta"], d["act"])
    Wr, Mr = orc.sync_fc_sfb(U, V, d["W"], d["Mom"], 0.25, 0.5)
    assert np.array_equal(Mg, Mr) and np.array_equal(Wg, Wr)


@pytest.mark.parametrize("dtype", [psd.F32, psd.BF16])
def test_weight_decay_bit_exact_on_both_routes(dtype):
    # wd, lr, mu powers of two and integer data: every intermediate is exact in fp32
    d = inputs.fc_layer_integer(M=260, N=141, B=6, P=4, seed=71)
    plan, U, ldu, V, ldv = run_pack(d, dtype)
    W, Mom = dev(d["W"]), dev(d["Mom"])
    psd.sync_fc_sfb(plan, dtype, U, ldu, V, ldv, W, Mom, 0.25, 0.5, wd=0.5)
    torch.cuda.synchronize()
    Uo, Vo = orc.pack_factors(d["delta"], d["act"])
    Wr, Mr = orc.sync_fc_sfb(Uo, Vo, d["W"], d["Mom"], 0.25, 0.5, wd=0.5)
    assert np.array_equal(Mom.cpu().numpy(), Mr) and np.array_equal(W.cpu().numpy(), Wr)
    if dtype == psd.F32:
        g = inputs.dense_layer_integer(70001, 5, seed=72)
        W, Mom = dev(g["W"]), dev(g["Mom"])
        psd.sync_dense_ps([dev(x) for x in g["G"]], W, Mom, 0.25, 0.5, 7, wd=0.5)
        torch.cuda.synchronize()
        Wr, Mr = orc.sync_dense_ps(g["G"], g["W"], g["Mom"], 0.25, 0.5, 7, wd=0.5)
        assert np.array_equal(Mom.cpu().numpy(), Mr) and np.array_equal(W.cpu().numpy(), Wr)


def test_weight_decay_gaussian_within_tolerance():
    d = inputs.fc_layer(M=1000, N=500, B=32, P=4, seed=73, mom_std=1e-4)
    for dtype, name in ((psd.F32, "f32"), (psd.BF16, "bf16")):
        plan, U, ldu, V, ldv = run_pack(d, dtype)
        W, Mom = dev(d["W"]), dev(d["Mom"])
        psd.sync_fc_sfb(plan, dtype, U, ldu, V, ldv, W, Mom, inputs.LR, inputs.MU, wd=5e-4)
        torch.cuda.synchronize()
        Uo, Vo = orc.pack_factors(d["delta"], d["act"], name)
        Wr, Mr = orc.sync_fc_sfb(Uo, Vo, d["W"], d["Mom"], inputs.LR, inputs.MU, wd=5e-4)
        e = three_errors(d["W"], W.cpu().numpy(), Mom.cpu().numpy(), Wr, Mr)
        assert max(e) <= TOL_F32, (name, e)


SPLIT_SHAPES = [  # M, N, B, P: few output tiles and K >= 1024, so that a workspace makes the kernels split K
    (1024, 1000, 256, 8),      # GoogLeNet-sized classifier at batch 256 per worker: 64 tiles, split in four
    (520, 300, 220, 5),        # ragged tiles both ways, K = 1100: ragged last stage and uneven splits
    (521, 130, 128, 9),        # rows of W not 16-byte aligned (element-wise epilogue), K = 1152
    (128, 128, 512, 4),        # a single tile, K = 2048: the deepest split
]


@pytest.mark.parametrize("M,N,B,P", SPLIT_SHAPES)
@pytest.mark.parametrize("dtype", [psd.F32, psd.BF16])
def test_sfb_split_k_with_workspace_bit_exact_and_equal_to_unsplit(M, N, B, P, dtype):
    """With a workspace the sum over k is split over several workgroups per tile and finished by the
    parameter-server sum kernel.  Integer-valued factors: bit-exact against the oracle; Gaussian factors:
    within tolerance of the oracle and of the unsplit kernel."""
    d = inputs.fc_layer_integer(M, N, B, P, seed=M + 3 * N)
    plan, U, ldu, V, ldv = run_pack(d, dtype)
    ws = psd.alloc_workspace(plan, dtype, DEV)
    assert ws is not None and 2 <= ws.numel() * 4 // ((N * M + 3) // 4 * 16) <= 4
    ws.fill_(float("nan"))                                 # stale contents must not matter
    W, Mom = dev(d["W"]), dev(d["Mom"])
    psd.sync_fc_sfb(plan, dtype, U, ldu, V, ldv, W, Mom, 0.25, 0.5, wd=0.25, workspace=ws)
    torch.cuda.synchronize()
    Uo, Vo = orc.pack_factors(d["delta"], d["act"])
    Wr, Mr = orc.sync_fc_sfb(Uo, Vo, d["W"], d["Mom"], 0.25, 0.5, wd=0.25)
    assert np.array_equal(Mom.cpu().numpy(), Mr), np.argwhere(Mom.cpu().numpy() != Mr)[:8]
    assert np.array_equal(W.cpu().numpy(), Wr)

    g = inputs.fc_layer(M, N, B, P, seed=M + N, mom_std=1e-4)
    plan, U, ldu, V, ldv = run_pack(g, dtype)
    name = "f32" if dtype == psd.F32 else "bf16"
    Uo, Vo = orc.pack_factors(g["delta"], g["act"], name)
    Wr, Mr = orc.sync_fc_sfb(Uo, Vo, g["W"], g["Mom"], inputs.LR, inputs.MU)
    outs = []
    for workspace in (ws, None):
        W, Mom = dev(g["W"]), dev(g["Mom"])
        psd.sync_fc_sfb(plan, dtype, U, ldu, V, ldv, W, Mom, inputs.LR, inputs.MU, workspace=workspace)
        torch.cuda.synchronize()
        e = three_errors(g["W"], W.cpu().numpy(), Mom.cpu().numpy(), Wr, Mr)
        assert max(e) <= TOL_F32, (workspace is not None, e)
        outs.append(Mom.cpu().numpy())
    assert orc.rel_frob(outs[0], outs[1]) <= TOL_F32


def test_sfb_workspace_is_ignored_by_layers_that_fill_the_gpu():
    d = inputs.fc_layer_integer(2048, 2048, 8, 4, seed=12)      # 256 tiles of 128 x 128 ... K = 32: no split either way
    plan, U, ldu, V, ldv = run_pack(d, psd.BF16)
    assert psd.sfb_workspace_bytes(plan, psd.BF16) == 0
    spare = torch.full((1024,), float("nan"), device=DEV)
    W, Mom = dev(d["W"]), dev(d["Mom"])
    psd.sync_fc_sfb(plan, psd.BF16, U, ldu, V, ldv, W, Mom, 0.25, 0.5, workspace=spare)
    torch.cuda.synchronize()
    Uo, Vo = orc.pack_factors(d["delta"], d["act"])
    Wr, Mr = orc.sync_fc_sfb(Uo, Vo, d["W"], d["Mom"], 0.25, 0.5)
    assert np.array_equal(Mom.cpu().numpy(), Mr) and np.array_equal(W.cpu().numpy(), Wr)
    assert torch.isnan(spare).all()                              # untouched


def _random_shapes(count, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        P = int(rng.integers(1, 10))
        B = int(rng.integers(1, 40))
        out.append((int(rng.integers(1, 700)), int(rng.integers(1, 700)), B, P))
    return out


@pytest.mark.parametrize("dtype", [psd.F32, psd.BF16])
def test_sfb_random_shapes_bit_exact(dtype):
    # 24 seeded random layer shapes (any width, any K tail) with integer data: pack, reconstruct,
    # update and the bias path must all equal the oracle bit for bit
    for (M, N, B, P) in _random_shapes(24, seed=2024):
        d = inputs.fc_layer_integer(M, N, B, P, seed=M * 1000 + N)
        plan, U, ldu, V, ldv = run_pack(d, dtype)
        W, Mom = dev(d["W"]), dev(d["Mom"])
        psd.sync_fc_sfb(plan, dtype, U, ldu, V, ldv, W, Mom, 0.25, 0.5, wd=0.25)
        b0 = np.arange(N, dtype=np.float32) - N // 2
        bias, mb = dev(b0), dev(np.zeros(N, np.float32))
        psd.sync_fc_bias(plan, dtype, U, ldu, bias, mb, 0.25, 0.5)
        torch.cuda.synchronize()
        Uo, Vo = orc.pack_factors(d["delta"], d["act"])
        Wr, Mr = orc.sync_fc_sfb(Uo, Vo, d["W"], d["Mom"], 0.25, 0.5, wd=0.25)
        assert np.array_equal(Mom.cpu().numpy(), Mr) and np.array_equal(W.cpu().numpy(), Wr), (M, N, B, P)
        br, mr = orc.sync_fc_bias(Uo, b0, np.zeros(N, np.float32), 0.25, 0.5)
        assert np.array_equal(bias.cpu().numpy(), br) and np.array_equal(mb.cpu().numpy(), mr), (M, N, B, P)


def test_dense_random_sizes_bit_exact():
    rng = np.random.default_rng(77)
    for _ in range(24):
        n = int(rng.integers(1, 300000))
        P = int(rng.integers(1, 20))
        S = int(rng.integers(1, min(n, 40) + 1))
        d = inputs.dense_layer_integer(n, P, seed=n)
        W, Mom = dev(d["W"]), dev(d["Mom"])
        psd.sync_dense_ps([dev(g) for g in d["G"]], W, Mom, 0.125, 0.5, S, wd=0.5)
        torch.cuda.synchronize()
        Wr, Mr = orc.sync_dense_ps(d["G"], d["W"], d["Mom"], 0.125, 0.5, S, wd=0.5)
        assert np.array_equal(W.cpu().numpy(), Wr) and np.array_equal(Mom.cpu().numpy(), Mr), (n, P, S)


def test_sfb_single_sample_is_exact_outer_product():
    d = inputs.fc_layer(M=200, N=150, B=1, P=1, seed=5)
    d["Mom"][:] = 0
    Wg, Mg, _ = run_sfb(d, psd.F32, 1.0, 0.0)
    want = d["delta"][0].T.astype(np.float32) * d["act"][0].astype(np.float32)   # one product per element
    assert np.array_equal(Mg, want.astype(np.float32))


@pytest.mark.parametrize("cfg", [1, 2])
def test_sfb_fp32_configs(cfg):
    d = inputs.fc_config(cfg)
    Wg, Mg, _ = run_sfb(d, psd.F32, inputs.LR, inputs.MU)
    U, V = orc.pack_factors(d["delta"], d["act"])
    Wr, Mr = orc.sync_fc_sfb(U, V, d["W"], d["Mom"], inputs.LR, inputs.MU)
    e = three_errors(d["W"], Wg, Mg, Wr, Mr)
    assert max(e) <= TOL_F32, e
    # second step on top of the first: momentum buffer is now non-zero
    d2 = dict(d, W=Wg, Mom=Mg)
    Wg2, Mg2, _ = run_sfb(d2, psd.F32, inputs.LR, inputs.MU)
    Wr2, Mr2 = orc.sync_fc_sfb(U, V, Wg, Mg, inputs.LR, inputs.MU)
    e = three_errors(Wg, Wg2, Mg2, Wr2, Mr2)
    assert max(e) <= TOL_F32, e


def test_sfb_bf16_small_gaussian_both_bars():
    d = inputs.fc_layer(M=700, N=333, B=24, P=5, seed=21, mom_std=1e-4)
    Wg, Mg, _ = run_sfb(d, psd.BF16, inputs.LR, inputs.MU)
    Ub, Vb = orc.pack_factors(d["delta"], d["act"], "bf16")
    Wr, Mr = orc.sync_fc_sfb(Ub, Vb, d["W"], d["Mom"], inputs.LR, inputs.MU)
    e = three_errors(d["W"], Wg, Mg, Wr, Mr)
    assert max(e) <= TOL_F32, e
    U, V = orc.pack_factors(d["delta"], d["act"])
    Wr, Mr = orc.sync_fc_sfb(U, V, d["W"], d["Mom"], inputs.LR, inputs.MU)
    e = three_errors(d["W"], Wg, Mg, Wr, Mr)
    assert max(e) <= TOL_BF16_VS_F32, e


def _whole_matrix_checks(d, Wg, Mg, factor_name, lr, mu, tol_vs_unrounded=None):
    """Whole-matrix comparison with the float64 oracle fed the very factor bits the kernel saw: the three
    relative Frobenius errors, and every single element against the worst-case bound of an fp32 sum of
    K products in any order (unit roundoff 2^-24, K + 4 roundings) plus the fp32 roundings of the update."""
    U, V = orc.pack_factors(d["delta"], d["act"], factor_name)
    Wr, Mr = orc.sync_fc_sfb(U, V, d["W"], d["Mom"], lr, mu)
    e = three_errors(d["W"], Wg, Mg, Wr, Mr)
    assert max(e) <= TOL_F32, e
    K = U.shape[0]
    Uv = orc.bf16_widen(U) if U.dtype == np.uint16 else U
    Vv = orc.bf16_widen(V) if V.dtype == np.uint16 else V
    mass = orc.rebuild(np.abs(Uv), np.abs(Vv))                       # sum_k |u||v| per element (float64)
    u = 2.0 ** -24
    bound_m = (K + 4) * u * np.float64(np.float32(lr)) * mass + 4 * u * np.abs(Mr.astype(np.float64)) + 1e-30
    err_m = np.abs(Mg.astype(np.float64) - Mr.astype(np.float64))
    bad = np.argwhere(err_m > bound_m)
    assert bad.size == 0, (bad[:5], err_m[tuple(bad[0])], bound_m[tuple(bad[0])])
    bound_w = bound_m + 4 * u * np.abs(Wr.astype(np.float64))
    err_w = np.abs(Wg.astype(np.float64) - Wr.astype(np.float64))
    bad = np.argwhere(err_w > bound_w)
    assert bad.size == 0, (bad[:5], err_w[tuple(bad[0])], bound_w[tuple(bad[0])])
    if tol_vs_unrounded is not None:
        U32, V32 = orc.pack_factors(d["delta"], d["act"])
        Wr, Mr = orc.sync_fc_sfb(U32, V32, d["W"], d["Mom"], lr, mu)
        e = three_errors(d["W"], Wg, Mg, Wr, Mr)
        assert max(e) <= tol_vs_unrounded, e


@pytest.mark.parametrize("cfg", [3, 4])
def test_sfb_bf16_full_size_whole_matrix(cfg):
    """Configs 3 and 4 at full size, in the launch shape the benchmark times, compared with the
    oracle over the WHOLE matrix: against the oracle fed the bf16-rounded factors (1e-5 and the
    per-element bound) and against the oracle fed the unrounded fp32 factors (2e-2)."""
    d = inputs.fc_config(cfg)
    Wg, Mg, _ = run_sfb(d, psd.BF16, inputs.LR, inputs.MU)
    _whole_matrix_checks(d, Wg, Mg, "bf16", inputs.LR, inputs.MU, tol_vs_unrounded=TOL_BF16_VS_F32)
    if cfg == 4:
        # rows of (softmax - onehot) sum to zero, so each column of dW sums to ~0
        col = Mg.astype(np.float64).sum(axis=0)
        assert np.abs(col).max() <= 2e-2 * np.abs(Mg.astype(np.float64)).sum(axis=0).max()


@pytest.mark.parametrize("M,N,dtype", [(9216, 4096, psd.BF16), (4096, 21841, psd.BF16), (4096, 1000, psd.F32),
                                       (9216, 4096, psd.F32)])
def test_sfb_full_size_integer_factors_bit_exact(M, N, dtype):
    """The production tile choice, the multi-round XCD raster, every ragged tile of N = 21841 and the
    LDS ring in steady state (K = 2048), compared bit for bit: integer-valued factors keep every partial
    sum below 2^24 (|u v| <= 9, K = 2048), so the fp32 result does not depend on the summation order."""
    d = inputs.fc_layer_integer(M, N, 256, 8, seed=M + N + 7)
    Wg, Mg, _ = run_sfb(d, dtype, 0.25, 0.5)
    U, V = orc.pack_factors(d["delta"], d["act"])
    Wr, Mr = orc.sync_fc_sfb(U, V, d["W"], d["Mom"], 0.25, 0.5)
    assert np.array_equal(Mg, Mr), np.argwhere(Mg != Mr)[:8]
    assert np.array_equal(Wg, Wr)


SECOND_WORKLOAD = [
    (3000, 3000, 256, 8, psd.BF16),      # FC stack of the ImageNet-22K network (Section 5.1.3)
    (3000, 3000, 256, 8, psd.F32),
    (3000, 21841, 256, 8, psd.BF16),     # its 21 841-way classifier
    (1024, 1000, 32, 8, psd.BF16),       # GoogLeNet's single FC layer at batch 32 per node (Section 5.1.2)
    (1024, 1000, 32, 8, psd.F32),
    (25088, 4096, 8, 8, psd.BF16),       # VGG-16-sized FC stack (Table 3) at its batch of 64 (Table 2) over 8 workers
    (25088, 4096, 8, 8, psd.F32),
    (4096, 4096, 8, 8, psd.BF16),
    (4096, 1000, 8, 8, psd.F32),
]


@pytest.mark.parametrize("M,N,B,P,dtype", SECOND_WORKLOAD)
def test_sfb_second_workload_shapes_whole_matrix(M, N, B, P, dtype):
    d = inputs.fc_layer(M, N, B, P, seed=M + N + B, delta_kind="softmax" if N == 21841 else "gauss")
    Wg, Mg, _ = run_sfb(d, dtype, inputs.LR, inputs.MU)
    _whole_matrix_checks(d, Wg, Mg, "f32" if dtype == psd.F32 else "bf16", inputs.LR, inputs.MU)


def test_sfb_vgg16_first_fc_layer_at_full_batch_integer_bit_exact():
    # the widest factor matrix of any workload here (25088 inputs, K = 2048: 103 MB of bf16 activations)
    d = inputs.fc_layer_integer(25088, 4096, 256, 8, seed=16)
    Wg, Mg, _ = run_sfb(d, psd.BF16, 0.25, 0.5)
    U, V = orc.pack_factors(d["delta"], d["act"])
    Wr, Mr = orc.sync_fc_sfb(U, V, d["W"], d["Mom"], 0.25, 0.5)
    assert np.array_equal(Mg, Mr) and np.array_equal(Wg, Wr)


@pytest.mark.parametrize("M,N,B,P", [(16, 1, 1, 1), (40, 127, 3, 5), (64, 1000, 16, 8), (8, 21841, 4, 2), (32, 300, 1, 37)])
@pytest.mark.parametrize("dtype", [psd.F32, psd.BF16])
def test_bias_integer_errors_bit_exact(M, N, B, P, dtype):
    d = inputs.fc_layer_integer(M, N, B, P, seed=N + B)
    plan, U, ldu, V, ldv = run_pack(d, dtype)
    rng = np.random.default_rng(N)
    b0 = rng.integers(-64, 65, size=N).astype(np.float32)
    m0 = rng.integers(-8, 9, size=N).astype(np.float32)
    bias, mom = dev(b0), dev(m0)
    psd.sync_fc_bias(plan, dtype, U, ldu, bias, mom, 0.25, 0.5, wd=0.5)
    torch.cuda.synchronize()
    Uo, _ = orc.pack_factors(d["delta"], d["act"])
    br, mr = orc.sync_fc_bias(Uo, b0, m0, 0.25, 0.5, wd=0.5)
    assert np.array_equal(mom.cpu().numpy(), mr) and np.array_equal(bias.cpu().numpy(), br)


@pytest.mark.parametrize("cfg,dtype", [(2, psd.F32), (3, psd.BF16), (4, psd.BF16)])
def test_bias_full_size_configs(cfg, dtype):
    d = inputs.fc_config(cfg)
    plan, U, ldu, V, ldv = run_pack(d, dtype)
    N = d["N"]
    b0 = (np.random.default_rng(cfg).standard_normal(N) * 0.1).astype(np.float32)
    bias, mom = dev(b0), dev(np.zeros(N, np.float32))
    psd.sync_fc_bias(plan, dtype, U, ldu, bias, mom, inputs.LR, inputs.MU)
    torch.cuda.synchronize()
    Uo, _ = orc.pack_factors(d["delta"], d["act"], "f32" if dtype == psd.F32 else "bf16")
    br, mr = orc.sync_fc_bias(Uo, b0, np.zeros(N, np.float32), inputs.LR, inputs.MU)
    if cfg == 4:
        # softmax errors: every column sum is a difference of nearly equal numbers (the classes'
        # probabilities against the rare one-hot hits), so compare absolutely, scaled by sum |U|
        scale = np.float64(np.float32(inputs.LR)) * np.abs(orc.bf16_widen(Uo).astype(np.float64)).sum(axis=0)
        assert np.all(np.abs(mom.cpu().numpy().astype(np.float64) - mr) <= 1e-6 * scale + 1e-12)
    else:
        assert orc.rel_frob(mom.cpu().numpy(), mr) <= TOL_F32
    assert orc.rel_frob(bias.cpu().numpy(), br) <= TOL_F32


BLOCK_SHAPES = [  # M, N, B, P with B a multiple of 16 and N, M multiples of 4
    (256, 128, 32, 4),        # config 1
    (520, 300, 16, 5),        # ragged tiles both ways, one k-stage per block
    (132, 64, 48, 3),         # three stages per block, blocks exhausted mid ring: the trailing stages must read as zeros
    (260, 204, 16, 64),       # the largest worker count: every entry of the pointer table in use
]


@pytest.mark.parametrize("M,N,B,P", BLOCK_SHAPES)
def test_sfb_blocks_in_place_bit_exact_and_identical_to_the_stacked_path(M, N, B, P):
    """fp32 reconstruction straight from the P per-worker blocks: bit-exact against the oracle on integer
    data, and on Gaussian data the very bits of pack + reconstruct (same arithmetic, same order)."""
    d = inputs.fc_layer_integer(M=M, N=N, B=B, P=P, seed=M + P, amax=2 if B * P > 500 else 3)
    plan = psd.plan_layer(psd.LAYER_FC, M, N, B, P)
    assert psd.sfb_blocks_supported(plan)
    W, Mom = dev(d["W"]), dev(d["Mom"])
    psd.sync_fc_sfb_blocks(plan, psd.F32, [dev(x) for x in d["delta"]], 0, [dev(x) for x in d["act"]], 0, W, Mom, 0.25, 0.5,
                           wd=0.5)
    torch.cuda.synchronize()
    U, V = orc.pack_factors(d["delta"], d["act"])
    Wr, Mr = orc.sync_fc_sfb(U, V, d["W"], d["Mom"], 0.25, 0.5, wd=0.5)
    assert np.array_equal(Mom.cpu().numpy(), Mr) and np.array_equal(W.cpu().numpy(), Wr)

    g = inputs.fc_layer(M=M, N=N, B=B, P=P, seed=M + 2 * P, mom_std=1e-4)
    Ws, Ms, _ = run_sfb(g, psd.F32, inputs.LR, inputs.MU)
    W, Mom = dev(g["W"]), dev(g["Mom"])
    psd.sync_fc_sfb_blocks(plan, psd.F32, [dev(x) for x in g["delta"]], 0, [dev(x) for x in g["act"]], 0, W, Mom,
                           inputs.LR, inputs.MU)
    torch.cuda.synchronize()
    assert np.array_equal(Mom.cpu().numpy(), Ms) and np.array_equal(W.cpu().numpy(), Ws)


@pytest.mark.parametrize("seed", range(6))
def test_sfb_blocks_in_place_random_shapes_identical_to_the_stacked_path(seed):
    """Random layer shapes, worker counts and block paddings, both factor dtypes: the blocks read in place give
    the very bits of the stacked path (which the other tests tie to the oracle)."""
    rng = np.random.default_rng(4200 + seed)
    for dtype, stage, q in ((psd.F32, 16, 4), (psd.BF16, 32, 8)):
        M, N = int(rng.integers(1, 700)), int(rng.integers(1, 500))
        P, B = int(rng.integers(1, 10)), stage * int(rng.integers(1, 4))
        # block rows: the narrowest the entry point accepts, or padded further
        ldu = (N + q - 1) // q * q + q * int(rng.integers(0, 3))
        ldv = (M + q - 1) // q * q + q * int(rng.integers(0, 3))
        td = torch.float32 if dtype == psd.F32 else torch.bfloat16
        plan = psd.plan_layer(psd.LAYER_FC, M, N, B, P)
        assert psd.sfb_blocks_supported(plan, dtype, ldu, ldv), (M, N, B, P, ldu, ldv)
        d = inputs.fc_layer(M=M, N=N, B=B, P=P, seed=900 + seed, mom_std=1e-4)
        Ub, Vb = [], []
        for p in range(P):
            u = torch.zeros(B, ldu, dtype=td, device=DEV)
            v = torch.zeros(B, ldv, dtype=td, device=DEV)
            u[:, :N] = dev(d["delta"][p]).to(td)         # torch rounds to nearest even, as the pack kernel does
            v[:, :M] = dev(d["act"][p]).to(td)
            Ub.append(u)
            Vb.append(v)
        U, V = torch.cat(Ub).contiguous(), torch.cat(Vb).contiguous()      # the stacked matrices, same leading dimensions
        Ws, Ms = dev(d["W"]), dev(d["Mom"])
        psd.sync_fc_sfb(plan, dtype, U, ldu, V, ldv, Ws, Ms, inputs.LR, inputs.MU, wd=1e-3)
        Wb, Mb = dev(d["W"]), dev(d["Mom"])
        psd.sync_fc_sfb_blocks(plan, dtype, Ub, ldu, Vb, ldv, Wb, Mb, inputs.LR, inputs.MU, wd=1e-3)
        torch.cuda.synchronize()
        assert torch.equal(Ws, Wb) and torch.equal(Ms, Mb), (M, N, B, P, ldu, ldv, dtype)


def test_sfb_blocks_in_place_at_the_classifier_size():
    """Config 2 (4096 -> 1000, K = 2048, fp32) without the stacking pass: whole matrix against the oracle."""
    d = inputs.fc_config(2)
    plan = psd.plan_layer(psd.LAYER_FC, d["M"], d["N"], d["B"], d["P"])
    W, Mom = dev(d["W"]), dev(d["Mom"])
    psd.sync_fc_sfb_blocks(plan, psd.F32, [dev(x) for x in d["delta"]], 0, [dev(x) for x in d["act"]], 0, W, Mom,
                           inputs.LR, inputs.MU)
    torch.cuda.synchronize()
    _whole_matrix_checks(d, W.cpu().numpy(), Mom.cpu().numpy(), "f32", inputs.LR, inputs.MU)


@pytest.mark.parametrize("M,N,B,P,dtype", [(256, 128, 11, 4, psd.F32), (256, 130, 16, 4, psd.F32), (21841, 64, 16, 2, psd.F32),
                                           (256, 128, 16, 4, psd.BF16)])
def test_sfb_blocks_in_place_refuses_layers_it_cannot_read(M, N, B, P, dtype):
    # a k-stage would straddle two blocks (B), or rows of a dense block would not be 16-byte aligned (N, M)
    plan = psd.plan_layer(psd.LAYER_FC, M, N, B, P)
    assert not psd.sfb_blocks_supported(plan, dtype)
    td = torch.float32 if dtype == psd.F32 else torch.bfloat16
    W, Mom = torch.zeros(N, M, device=DEV), torch.zeros(N, M, device=DEV)
    U_blocks = [torch.zeros(B, N, device=DEV, dtype=td) for _ in range(P)]
    V_blocks = [torch.zeros(B, M, device=DEV, dtype=td) for _ in range(P)]
    with pytest.raises(psd.PsdError) as e:
        psd.sync_fc_sfb_blocks(plan, dtype, U_blocks, 0, V_blocks, 0, W, Mom, 0.01, 0.9)
    assert e.value.status == psd.E_UNSUPPORTED


BF16_BLOCK_SHAPES = [  # M, N, B, P with B a multiple of 32; odd widths get padded rows
    (256, 128, 32, 4),
    (700, 260, 64, 9),        # K = 576: ragged tiles both ways, two stages per block
    (1001, 333, 32, 5),       # odd widths: blocks with padded rows (ld from psd_factor_ld), element-wise epilogue
    (260, 204, 32, 64),       # every entry of the pointer table in use
]


@pytest.mark.parametrize("M,N,B,P", BF16_BLOCK_SHAPES)
def test_sfb_bf16_blocks_in_place_bit_exact_and_identical_to_the_stacked_path(M, N, B, P):
    """bf16 factors that arrive already rounded, one block per worker (what psd_pack_factors writes for a
    one-worker plan), read in place: bit-exact against the oracle on integer data, and the very bits of the
    stacked path on Gaussian data."""
    plan = psd.plan_layer(psd.LAYER_FC, M, N, B, P)
    one = psd.plan_layer(psd.LAYER_FC, M, N, B, 1)
    ldu, ldv = psd.factor_ld(N, psd.BF16), psd.factor_ld(M, psd.BF16)
    assert psd.sfb_blocks_supported(plan, psd.BF16, ldu, ldv)

    def sender_side(d):            # every worker rounds its own block
        Ub, Vb = [], []
        for p in range(P):
            U, _, V, _ = psd.alloc_factors(one, psd.BF16, DEV)
            psd.pack_factors(one, [dev(d["delta"][p])], [dev(d["act"][p])], psd.BF16, U, ldu, V, ldv)
            Ub.append(U)
            Vb.append(V)
        return Ub, Vb

    d = inputs.fc_layer_integer(M=M, N=N, B=B, P=P, seed=M + P, amax=2 if B * P > 500 else 3)
    Ub, Vb = sender_side(d)
    W, Mom = dev(d["W"]), dev(d["Mom"])
    psd.sync_fc_sfb_blocks(plan, psd.BF16, Ub, ldu, Vb, ldv, W, Mom, 0.25, 0.5, wd=0.5)
    torch.cuda.synchronize()
    U, V = orc.pack_factors(d["delta"], d["act"])
    Wr, Mr = orc.sync_fc_sfb(U, V, d["W"], d["Mom"], 0.25, 0.5, wd=0.5)
    assert np.array_equal(Mom.cpu().numpy(), Mr) and np.array_equal(W.cpu().numpy(), Wr)

    g = inputs.fc_layer(M=M, N=N, B=B, P=P, seed=M + 2 * P, mom_std=1e-4)
    Ws, Ms, _ = run_sfb(g, psd.BF16, inputs.LR, inputs.MU)
    Ub, Vb = sender_side(g)
    W, Mom = dev(g["W"]), dev(g["Mom"])
    psd.sync_fc_sfb_blocks(plan, psd.BF16, Ub, ldu, Vb, ldv, W, Mom, inputs.LR, inputs.MU)
    torch.cuda.synchronize()
    assert np.array_equal(Mom.cpu().numpy(), Ms) and np.array_equal(W.cpu().numpy(), Ws)


def test_sfb_bf16_blocks_in_place_at_the_fc6_size():
    """Config 3 (9216 -> 4096, K = 2048, bf16) from eight ready-made bf16 blocks: whole matrix against the oracle."""
    d = inputs.fc_config(3)
    plan = psd.plan_layer(psd.LAYER_FC, d["M"], d["N"], d["B"], d["P"])
    one = psd.plan_layer(psd.LAYER_FC, d["M"], d["N"], d["B"], 1)
    ldu, ldv = psd.factor_ld(d["N"], psd.BF16), psd.factor_ld(d["M"], psd.BF16)
    Ub, Vb = [], []
    for p in range(d["P"]):
        U, _, V, _ = psd.alloc_factors(one, psd.BF16, DEV)
        psd.pack_factors(one, [dev(d["delta"][p])], [dev(d["act"][p])], psd.BF16, U, ldu, V, ldv)
        Ub.append(U)
        Vb.append(V)
    W, Mom = dev(d["W"]), dev(d["Mom"])
    psd.sync_fc_sfb_blocks(plan, psd.BF16, Ub, ldu, Vb, ldv, W, Mom, inputs.LR, inputs.MU)
    torch.cuda.synchronize()
    _whole_matrix_checks(d, W.cpu().numpy(), Mom.cpu().numpy(), "bf16", inputs.LR, inputs.MU)


def test_iteration_reads_fp32_blocks_in_place_when_no_stacked_buffers_are_given():
    layers = inputs.cnn_iteration(scale=8, B=16, P=4)
    out = []
    for in_place in (False, True):
        tasks, state = _build_iteration(layers, psd.F32, [None] * len(layers))
        if in_place:
            switched = 0
            for t in tasks:
                if "delta" in t and psd.sfb_blocks_supported(t["plan"]):     # the 512 -> 125 layer keeps its stacked buffers
                    t.update(U=None, V=None, ldu=0, ldv=0)
                    switched += 1
            assert switched == 2
        psd.Iteration(tasks).run(inputs.LR, inputs.MU, psd.RULE_ALG3)
        torch.cuda.synchronize()
        out.append([(W.cpu().numpy(), Mom.cpu().numpy()) for W, Mom in state])
    for (w0, m0), (w1, m1) in zip(*out):
        assert np.array_equal(w0, w1) and np.array_equal(m0, m1)


def test_iteration_reads_bf16_blocks_in_place():
    """Layers handed to psd_sync_iteration as ready-made bf16 blocks (no stacked buffers): same bits as the
    iteration that stacks and rounds the fp32 blocks itself."""
    layers = inputs.cnn_iteration(scale=8, B=32, P=4)
    out = []
    for in_place in (False, True):
        tasks, state = _build_iteration(layers, psd.BF16, [None] * len(layers))
        if in_place:
            switched = 0
            for t in tasks:
                if "delta" not in t:
                    continue
                plan = t["plan"]
                one = psd.plan_layer(psd.LAYER_FC, plan.M, plan.N, plan.B, 1)
                Ub, Vb = [], []
                for p in range(plan.P):
                    U, ldu, V, ldv = psd.alloc_factors(one, psd.BF16, DEV)
                    psd.pack_factors(one, [t["delta"][p]], [t["act"][p]], psd.BF16, U, ldu, V, ldv)
                    Ub.append(U)
                    Vb.append(V)
                assert psd.sfb_blocks_supported(plan, psd.BF16, ldu, ldv)
                t.update(U=None, V=None, delta=Ub, act=Vb, ldu=ldu, ldv=ldv)
                switched += 1
            assert switched == 3
        psd.Iteration(tasks).run(inputs.LR, inputs.MU, psd.RULE_ALG3)
        torch.cuda.synchronize()
        out.append([(W.cpu().numpy(), Mom.cpu().numpy()) for W, Mom in state])
    for (w0, m0), (w1, m1) in zip(*out):
        assert np.array_equal(w0, w1) and np.array_equal(m0, m1)


def test_sfb_equals_ps_route_on_the_same_gradients():
    # Section 4.3.1: factors reconstruct the gradient exactly, so both routes agree
    d = inputs.fc_layer_integer(M=300, N=200, B=4, P=3, seed=31)
    Wg, Mg, _ = run_sfb(d, psd.F32, 0.25, 0.5)
    G = [dev((d["delta"][p].astype(np.float64).T @ d["act"][p].astype(np.float64)).astype(np.float32).ravel())
         for p in range(3)]
    W, Mom = dev(d["W"].ravel()), dev(d["Mom"].ravel())
    psd.sync_dense_ps(G, W, Mom, 0.25, 0.5, 8)
    torch.cuda.synchronize()
    assert np.array_equal(W.cpu().numpy(), Wg.ravel()) and np.array_equal(Mom.cpu().numpy(), Mg.ravel())


# ---------------------------------------------------------------------------------------
# whole iteration (config 5): routes, issue order, per-layer parity
# ---------------------------------------------------------------------------------------
def _build_iteration(layers, factor_dtype, streams):
    tasks, state = [], []
    for L, st in zip(layers, streams):
        if L["kind"] == "conv":
            plan = psd.plan_layer(psd.LAYER_CONV, L["n"], 1, inputs.CNN_B, L["P"])
            W, Mom = dev(L["W"]), dev(L["Mom"])
            tasks.append(dict(plan=plan, G=[dev(g) for g in L["G"]], S=min(inputs.CNN_S, L["n"]), W=W, Mom=Mom,
                              stream=st))
        else:
            plan = psd.plan_layer(psd.LAYER_FC, L["M"], L["N"], L["B"], L["P"])
            U, ldu, V, ldv = psd.alloc_factors(plan, factor_dtype, DEV)
            W, Mom = dev(L["W"]), dev(L["Mom"])
            tasks.append(dict(plan=plan, factor_dtype=factor_dtype, delta=[dev(x) for x in L["delta"]],
                              act=[dev(x) for x in L["act"]], U=U, ldu=ldu, V=V, ldv=ldv, W=W, Mom=Mom, stream=st))
        state.append((W, Mom))
    return tasks, state


@pytest.mark.parametrize("factor_dtype", [psd.F32, psd.BF16])
def test_iteration_scaled_down_matches_oracle_and_ignores_issue_order(factor_dtype):
    layers = inputs.cnn_iteration(scale=8, B=16, P=4)
    results = []
    for order in ("own_streams", "one_stream", "reversed_list"):
        streams = [torch.cuda.Stream(device=DEV) for _ in layers] if order != "one_stream" else [None] * len(layers)
        tasks, state = _build_iteration(layers, factor_dtype, streams)
        torch.cuda.synchronize()
        if order == "reversed_list":
            # give the library the layers in the opposite order: a different issue sequence,
            # which must not matter because layers own disjoint parameters (Section 4.2)
            psd.Iteration(tasks[::-1]).run(inputs.LR, inputs.MU, psd.RULE_ALG3)
        else:
            psd.Iteration(tasks).run(inputs.LR, inputs.MU, psd.RULE_ALG3)
        torch.cuda.synchronize()
        results.append([(W.cpu().numpy(), Mom.cpu().numpy()) for W, Mom in state])
    for other in results[1:]:
        for (w0, m0), (w1, m1) in zip(results[0], other):
            assert np.array_equal(w0, w1) and np.array_equal(m0, m1)
    name = "f32" if factor_dtype == psd.F32 else "bf16"
    for L, (Wg, Mg) in zip(layers, results[0]):
        if L["kind"] == "conv":
            Wr, Mr = orc.sync_dense_ps(L["G"], L["W"], L["Mom"], inputs.LR, inputs.MU, min(inputs.CNN_S, L["n"]))
        else:
            U, V = orc.pack_factors(L["delta"], L["act"], name)
            Wr, Mr = orc.sync_fc_sfb(U, V, L["W"], L["Mom"], inputs.LR, inputs.MU)
        e = three_errors(L["W"], Wg, Mg, Wr, Mr)
        assert max(e) <= TOL_F32, (L["name"], e)


def test_iteration_full_size_in_the_benchmark_configuration():
    """Config 5 at full size, issued exactly as bench.py does (one stream per layer, Algorithm 3
    routes, bf16 factors): every layer, conv and FC, compared whole with the oracle."""
    layers = inputs.cnn_iteration()
    streams = [torch.cuda.Stream(device=DEV) for _ in layers]
    tasks, state = _build_iteration(layers, psd.BF16, streams)
    torch.cuda.synchronize()
    psd.Iteration(tasks).run(inputs.LR, inputs.MU, psd.RULE_ALG3)
    torch.cuda.synchronize()
    for L, (W, Mom) in zip(layers, state):
        Wg, Mg = W.cpu().numpy(), Mom.cpu().numpy()
        if L["kind"] == "conv":
            Wr, Mr = orc.sync_dense_ps(L["G"], L["W"], L["Mom"], inputs.LR, inputs.MU, inputs.CNN_S)
            e = three_errors(L["W"], Wg, Mg, Wr, Mr)
            assert max(e) <= TOL_F32, (L["name"], e)
        else:
            _whole_matrix_checks(L, Wg, Mg, "bf16", inputs.LR, inputs.MU)


def test_iteration_waits_for_the_layers_gradient_event():
    """Algorithm 2: a layer is synchronised as soon as its gradient exists.  The factors are written by
    a 'backward' stream only after a long stretch of other work; the layer's stream must wait for the
    event that marks them ready (without the wait it would read the zeros the buffers start with)."""
    import ctypes
    hip = ctypes.CDLL("libamdhip64.so")
    hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
    hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
    hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
    d = inputs.fc_layer(M=512, N=384, B=16, P=4, seed=41)
    g = inputs.dense_layer(50000, 4, seed=42)
    plan = psd.plan_layer(psd.LAYER_FC, d["M"], d["N"], d["B"], d["P"])
    pconv = psd.plan_layer(psd.LAYER_CONV, g["n"], 1, d["B"], g["P"])
    U, ldu, V, ldv = psd.alloc_factors(plan, psd.BF16, DEV)
    delta = [torch.zeros_like(dev(x)) for x in d["delta"]]
    act = [torch.zeros_like(dev(x)) for x in d["act"]]
    G = [torch.zeros_like(dev(x)) for x in g["G"]]
    src_delta, src_act, src_G = [dev(x) for x in d["delta"]], [dev(x) for x in d["act"]], [dev(x) for x in g["G"]]
    W, Mom, Wc, Mc = dev(d["W"]), dev(d["Mom"]), dev(g["W"]), dev(g["Mom"])
    backward = torch.cuda.Stream(device=DEV)
    s_fc, s_conv = torch.cuda.Stream(device=DEV), torch.cuda.Stream(device=DEV)
    ev_fc, ev_conv = ctypes.c_void_p(), ctypes.c_void_p()
    assert hip.hipEventCreate(ctypes.byref(ev_fc)) == 0 and hip.hipEventCreate(ctypes.byref(ev_conv)) == 0
    big = torch.randn(4096, 4096, device=DEV)
    torch.cuda.synchronize()
    with torch.cuda.stream(backward):
        for _ in range(20):                       # stand-in for the rest of backpropagation (tens of ms)
            big = (big @ big) * 1e-3
        for dst, src in zip(delta + act, src_delta + src_act):
            dst.copy_(src)
        assert hip.hipEventRecord(ev_fc, ctypes.c_void_p(backward.cuda_stream)) == 0      # top layer ready first
        for _ in range(5):
            big = (big @ big) * 1e-3
        for dst, src in zip(G, src_G):
            dst.copy_(src)
        assert hip.hipEventRecord(ev_conv, ctypes.c_void_p(backward.cuda_stream)) == 0
    tasks = [dict(plan=pconv, G=G, S=8, W=Wc, Mom=Mc, stream=s_conv, ev_ready=ev_conv.value),
             dict(plan=plan, factor_dtype=psd.BF16, delta=delta, act=act, U=U, ldu=ldu, V=V, ldv=ldv, W=W, Mom=Mom,
                  stream=s_fc, ev_ready=ev_fc.value)]
    psd.Iteration(tasks).run(inputs.LR, inputs.MU, psd.RULE_ALG3)      # issued while 'backward' is still busy
    torch.cuda.synchronize()
    Uo, Vo = orc.pack_factors(d["delta"], d["act"], "bf16")
    Wr, Mr = orc.sync_fc_sfb(Uo, Vo, d["W"], d["Mom"], inputs.LR, inputs.MU)
    assert max(three_errors(d["W"], W.cpu().numpy(), Mom.cpu().numpy(), Wr, Mr)) <= TOL_F32
    Wr, Mr = orc.sync_dense_ps(g["G"], g["W"], g["Mom"], inputs.LR, inputs.MU, 8)
    assert max(three_errors(g["W"], Wc.cpu().numpy(), Mc.cpu().numpy(), Wr, Mr)) <= TOL_F32
    hip.hipEventDestroy(ev_fc)
    hip.hipEventDestroy(ev_conv)


def test_iteration_fused_parameter_server_launch_orders_every_layers_stream():
    """Conv layers without a readiness event are summed by one launch on the top conv layer's stream; work
    a caller then enqueues on ANY of those layers' own streams must see that layer updated."""
    sizes = [70001, 300000, 1234567, 5]
    layers = [inputs.dense_layer_integer(n, 8, seed=300 + i) for i, n in enumerate(sizes)]
    streams = [torch.cuda.Stream(device=DEV) for _ in layers]
    tasks, state = [], []
    for d, st in zip(layers, streams):
        plan = psd.plan_layer(psd.LAYER_CONV, d["n"], 1, 16, d["P"])
        W, Mom = dev(d["W"]), dev(d["Mom"])
        tasks.append(dict(plan=plan, G=[dev(g) for g in d["G"]], S=min(8, d["n"]), W=W, Mom=Mom, stream=st))
        state.append((W, Mom))
    torch.cuda.synchronize()
    psd.Iteration(tasks).run(0.25, 0.5, psd.RULE_ALG3, wd=0.5)
    seen = []
    for (W, Mom), st in zip(state, streams):
        with torch.cuda.stream(st):                    # no device-wide synchronisation in between
            seen.append((W.clone(), Mom.clone()))
    for st in streams:
        st.synchronize()
    for d, (Wc, Mc) in zip(layers, seen):
        Wr, Mr = orc.sync_dense_ps(d["G"], d["W"], d["Mom"], 0.25, 0.5, min(8, d["n"]), wd=0.5)
        assert np.array_equal(Wc.cpu().numpy(), Wr) and np.array_equal(Mc.cpu().numpy(), Mr), d["n"]


def test_pack_more_rows_than_one_grid_dimension_holds():
    # K = P*B = 70 000 stacked samples: the pack kernel's row index wraps around its grid
    d = inputs.fc_layer_integer(8, 4, 1094, 64, seed=70)
    plan, U, ldu, V, ldv = run_pack(d, psd.BF16)
    Uo, Vo = orc.pack_factors(d["delta"], d["act"], "bf16")
    assert np.array_equal(bits16(U)[:, :4], Uo) and np.array_equal(bits16(V)[:, :8], Vo)


def test_iteration_routes_follow_the_plan():
    # fc8-shaped layer at P=8, B=256: Algorithm 3 says SF_PS, the prose rule says SFB; both
    # run the reconstruction.  A layer whose route is PS_DENSE but has no dense copies is refused.
    plan = psd.plan_layer(psd.LAYER_FC, 4096, 1000, 256, 8)
    assert psd.ROUTE_NAMES[plan.route_alg3] == "SF_PS" and psd.ROUTE_NAMES[plan.route_vs_dense] == "SFB"
    d = inputs.fc_layer(64, 32, 256, 16, seed=9)        # tiny layer, huge batch: vs-dense rule -> PS_DENSE
    plan = psd.plan_layer(psd.LAYER_FC, 64, 32, 256, 16)
    assert plan.route_vs_dense == psd.ROUTE_PS_DENSE and plan.route_alg3 == psd.ROUTE_SF_PS
    U, ldu, V, ldv = psd.alloc_factors(plan, psd.F32, DEV)
    task = dict(plan=plan, factor_dtype=psd.F32, delta=[dev(x) for x in d["delta"]], act=[dev(x) for x in d["act"]],
                U=U, ldu=ldu, V=V, ldv=ldv, W=dev(d["W"]), Mom=dev(d["Mom"]), stream=None)
    with pytest.raises(psd.PsdError) as ei:
        psd.Iteration([task]).run(inputs.LR, inputs.MU, psd.RULE_SFB_VS_DENSE)
    assert ei.value.status == psd.E_UNSUPPORTED
    # with the dense copies present the PS route runs and equals the SFB result
    G = [dev((d["delta"][p].astype(np.float64).T @ d["act"][p].astype(np.float64)).astype(np.float32).ravel())
         for p in range(16)]
    W2, Mom2 = dev(d["W"]), dev(d["Mom"])
    psd.Iteration([dict(task, G=G, S=4, W=W2, Mom=Mom2)]).run(inputs.LR, inputs.MU, psd.RULE_SFB_VS_DENSE)
    psd.Iteration([task]).run(inputs.LR, inputs.MU, psd.RULE_ALG3)
    torch.cuda.synchronize()
    assert orc.rel_frob(Mom2.cpu().numpy(), task["Mom"].cpu().numpy()) <= TOL_F32


# ---------------------------------------------------------------------------------------
# bounded staleness (Section 3.2): the update of clock c is applied at clock c + s
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("s", [0, 1, 3])
@pytest.mark.parametrize("dtype", [psd.F32, psd.BF16])
def test_ssp_fc_layer_over_several_clocks_matches_the_guaranteed_view(s, dtype):
    """After every clock t the weights on the GPU must be exactly what a reader at clock t+1 is guaranteed
    under staleness s: the updates of clocks 0 .. t-s, applied in clock order (integer data, lr and mu
    powers of two, no weight decay: six clocks add six fractional bits, everything stays exact in fp32).
    Then the ring is drained and the result equals T bulk-synchronous clocks."""
    T, M, N, B, P = 6, 200, 150, 5, 3
    sets = [inputs.fc_layer_integer(M, N, B, P, seed=900 + c) for c in range(T)]
    plan = psd.plan_layer(psd.LAYER_FC, M, N, B, P)
    layer = psd.SspFc(plan, dtype, s, DEV)
    W, Mom = dev(sets[0]["W"]), dev(sets[0]["Mom"])
    packed = [orc.pack_factors(d["delta"], d["act"]) for d in sets]
    updates = [(lambda w, m, UV=UV: orc.sync_fc_sfb(UV[0], UV[1], w, m, 0.25, 0.5)) for UV in packed]
    for t in range(T):
        push, due = layer.slots()
        assert push == t % (s + 1) and due == (-1 if t < s else (t - s) % (s + 1))
        layer.clock([dev(x) for x in sets[t]["delta"]], [dev(x) for x in sets[t]["act"]], W, Mom, 0.25, 0.5)
        torch.cuda.synchronize()
        Wr, Mr = orc.ssp_visible_state(updates, sets[0]["W"], sets[0]["Mom"], s, t + 1)
        assert np.array_equal(W.cpu().numpy(), Wr) and np.array_equal(Mom.cpu().numpy(), Mr), (s, t)
    for k in range(s):                                   # drain what is still pending
        layer.clock(None, None, W, Mom, 0.25, 0.5)
    torch.cuda.synchronize()
    Wr, Mr = orc.ssp_visible_state(updates, sets[0]["W"], sets[0]["Mom"], 0, T)
    assert np.array_equal(W.cpu().numpy(), Wr) and np.array_equal(Mom.cpu().numpy(), Mr)
    if s == 0:
        with pytest.raises(psd.PsdError):
            layer.clock(None, None, W, Mom, 0.25, 0.5)   # nothing can be pending without staleness


@pytest.mark.parametrize("s", [0, 2])
def test_ssp_parameter_server_layer_over_several_clocks(s):
    T, n, P = 5, 70001, 4
    sets = [inputs.dense_layer(n, P, seed=950 + c, mom_std=1e-3) for c in range(T)]
    layer = psd.SspDense(s)
    W, Mom = dev(sets[0]["W"]), dev(sets[0]["Mom"])
    updates = [(lambda w, m, G=d["G"]: orc.sync_dense_ps(G, w, m, inputs.LR, inputs.MU, 7)) for d in sets]
    for t in range(T):
        layer.clock([dev(g) for g in sets[t]["G"]], W, Mom, inputs.LR, inputs.MU, 7)
        torch.cuda.synchronize()
        Wr, Mr = orc.ssp_visible_state(updates, sets[0]["W"], sets[0]["Mom"], s, t + 1)
        e = three_errors(sets[0]["W"], W.cpu().numpy(), Mom.cpu().numpy(), Wr, Mr) if t >= s else (0.0,)
        assert max(e) <= TOL_F32, (s, t, e)
        if t < s:                                        # nothing applied yet: the state is untouched
            assert np.array_equal(W.cpu().numpy(), sets[0]["W"]) and np.array_equal(Mom.cpu().numpy(), sets[0]["Mom"])
    for k in range(s):
        layer.clock(None, W, Mom, inputs.LR, inputs.MU, 7)
    torch.cuda.synchronize()
    Wr, Mr = orc.ssp_visible_state(updates, sets[0]["W"], sets[0]["Mom"], 0, T)
    assert max(three_errors(sets[0]["W"], W.cpu().numpy(), Mom.cpu().numpy(), Wr, Mr)) <= TOL_F32
