"""Pins for the oracle's factor stacking and its fp32 -> bf16 rounding."""
import struct
from fractions import Fraction

import numpy as np
import torch

from oracle import psd_oracle as orc


def test_row_map_with_index_encoding_inputs():
    # every element carries its own (p, b, column, which-factor) so a wrong row, block or
    # swapped factor is visible; values are small integers, exact in fp32
    P, B, N, M = 3, 4, 5, 7
    delta = [np.array([[1000 * p + 100 * b + j for j in range(N)] for b in range(B)], np.float32)
             for p in range(P)]
    act = [np.array([[-(1000 * p + 100 * b + i) - 0.5 for i in range(M)] for b in range(B)], np.float32)
           for p in range(P)]
    U, V = orc.pack_factors(delta, act)
    assert U.shape == (P * B, N) and V.shape == (P * B, M)
    for k in range(P * B):
        p, b = divmod(k, B)
        assert U[k].tolist() == [1000 * p + 100 * b + j for j in range(N)]
        assert V[k].tolist() == [-(1000 * p + 100 * b + i) - 0.5 for i in range(M)]
    # library routine that does the same thing
    assert np.array_equal(U, np.concatenate(delta, axis=0))
    assert np.array_equal(V, np.vstack(act))


def _bf16_exact(x):
    """Nearest-even bf16 of a finite float by exact rational arithmetic over candidates."""
    if x == 0:
        return 0x8000 if struct.pack("<f", x)[3] & 0x80 else 0
    sign = 0x8000 if x < 0 else 0
    ax = Fraction(abs(x))
    best = None
    bits = struct.unpack("<I", struct.pack("<f", abs(x)))[0] >> 16
    for cand in (bits - 1, bits, bits + 1):
        if cand < 0 or cand > 0x7f80:
            continue
        e, m = cand >> 7, cand & 0x7f
        val = Fraction(m, 1 << 133) if e == 0 else Fraction(128 + m) * Fraction(2) ** (e - 134)
        key = (abs(val - ax), cand & 1)  # distance, then even mantissa
        if best is None or key < best[0]:
            best = (key, cand)
    return sign | best[1]


def test_bf16_hand_cases():
    cases = {
        1.0: 0x3f80,
        1.0 + 2.0 ** -8: 0x3f80,               # tie -> even (down)
        1.0 + 2.0 ** -8 + 2.0 ** -23: 0x3f81,  # just above the tie
        1.0 + 3 * 2.0 ** -8: 0x3f82,           # tie -> even (up)
        -2.5: 0xc020,
        0.0: 0x0000,
        (2 - 2.0 ** -7) * 2.0 ** 127: 0x7f7f,  # largest finite bf16
        (2 - 2.0 ** -8) * 2.0 ** 127: 0x7f80,  # it plus half an ulp: tie -> even -> +inf
        (2 - 2.0 ** -8 - 2.0 ** -23) * 2.0 ** 127: 0x7f7f,  # one fp32 ulp below that tie
        float("inf"): 0x7f80,
        float("-inf"): 0xff80,
        2.0 ** -133: 0x0001,                   # smallest bf16 subnormal
        2.0 ** -134: 0x0000,                   # tie between 0 and it -> even (0)
    }
    x = np.array(list(cases), dtype=np.float32)
    assert orc.bf16_round_bits(x).tolist() == list(cases.values())
    assert orc.bf16_round_bits(np.array([-0.0], np.float32)).tolist() == [0x8000]
    nan = orc.bf16_round_bits(np.array([np.nan], np.float32))[0]
    assert (nan & 0x7f80) == 0x7f80 and (nan & 0x7f) != 0 and (nan & 0x40)


def test_bf16_against_exact_rationals():
    rng = np.random.default_rng(7)
    bits = rng.integers(0, 0x7f800000, size=4000, dtype=np.uint32)
    bits[:1000] &= np.uint32(0xffff8000)   # many exact ties / representables
    bits[:500] |= np.uint32(0x8000)
    x = bits.view(np.float32) * np.where(rng.random(4000) < 0.5, -1, 1).astype(np.float32)
    got = orc.bf16_round_bits(x)
    for xi, gi in zip(x.tolist(), got.tolist()):
        assert gi == _bf16_exact(xi), (xi, hex(gi))


def test_bf16_against_torch_cpu_cast_all_upper_halves():
    # all 2^16 upper halves x {below, exactly at, above the tie, zero, all ones} lower halves
    hi = np.arange(1 << 16, dtype=np.uint32) << 16
    for low in (0x0000, 0x7fff, 0x8000, 0x8001, 0xffff, 0x0001):
        u = hi | np.uint32(low)
        x = u.view(np.float32)
        finite_or_inf = ~np.isnan(x)
        got = orc.bf16_round_bits(x)
        want = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        assert np.array_equal(got[finite_or_inf], want[finite_or_inf])
        nan_out = got[~finite_or_inf]
        assert np.all((nan_out & 0x7f80) == 0x7f80) and np.all((nan_out & 0x7f) != 0)


def test_bf16_widen_is_exact_inverse_on_representables():
    b = np.arange(1 << 16, dtype=np.uint16)
    x = orc.bf16_widen(b)
    ok = ~np.isnan(x)
    assert np.array_equal(orc.bf16_round_bits(x)[ok], b[ok])
    assert np.array_equal(x[ok], torch.from_numpy(b.view(np.int16).copy()).view(torch.bfloat16).float().numpy()[ok])


def test_pack_bf16_rounds_after_stacking():
    rng = np.random.default_rng(3)
    delta = [rng.standard_normal((2, 3), dtype=np.float32) for _ in range(2)]
    act = [rng.standard_normal((2, 4), dtype=np.float32) for _ in range(2)]
    Ub, Vb = orc.pack_factors(delta, act, "bf16")
    want_u = torch.from_numpy(np.concatenate(delta)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    want_v = torch.from_numpy(np.concatenate(act)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert Ub.dtype == np.uint16 and np.array_equal(Ub, want_u) and np.array_equal(Vb, want_v)
