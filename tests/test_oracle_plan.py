"""Pins for the oracle's route selection (Alg. 3, Section 4.3.1) and key-range shards.

None of the expected values here comes from the oracle itself: they are the paper's
printed numbers (tests/golden/), independently re-derived closed forms, or brute force.
"""
import itertools
from fractions import Fraction

import pytest

from oracle import psd_oracle as orc
from paper_1512_06216_amd import inputs

FC, CONV = orc.KIND_FC, orc.KIND_CONV


def test_paper_worked_example(golden):
    g = golden("sec431_comm_volumes.txt")
    P, B, M, N = int(g["P"]), int(g["K"]), int(g["M"]), int(g["N"])
    p = orc.plan_layer(FC, M, N, B, P)
    # the paper prints one decimal in millions; ratios to one decimal / an integer
    assert round(p["cost_sfb"] / 1e6, 1) == g["sfb_millions"]
    assert round(p["cost_ps_dense"] / 1e6, 1) == g["full_matrix_millions"]
    assert round(p["cost_sf_ps"] / 1e6, 1) == g["sf_to_server_millions"]
    assert round(p["cost_ps_dense"] / p["cost_sfb"], 1) == g["full_over_sfb_ratio"]
    assert round(p["cost_sf_ps"] / p["cost_sfb"]) == g["sf_to_server_over_sfb_ratio"]
    assert p["route_alg3"] == orc.ROUTE_SFB and p["route_vs_dense"] == orc.ROUTE_SFB


def test_table3_shapes(golden):
    g = golden("table3_param_split.txt")
    conv = sum(inputs.conv_sizes())
    fc = sum(m * n for m, n in inputs.FC_SHAPES)
    assert round(conv / 1e6, 1) == g["conv_millions"]
    assert round(fc / 1e6) == g["fc_millions"]
    # Table 3 prints 3.75 / 96.25 %; the weight-only counts give 3.83 / 96.17 % (the
    # paper's percentages follow its rounded 2.3M / 61.3M totals) -- agree to half a point
    assert abs(100 * conv / (conv + fc) - g["conv_percent"]) < 0.5
    assert abs(100 * fc / (conv + fc) - g["fc_percent"]) < 0.5


def test_single_worker_sends_nothing():
    for M, N, B in [(7, 5, 3), (4096, 1000, 256)]:
        assert orc.plan_layer(FC, M, N, B, 1)["cost_sfb"] == 0


def test_sfb_cost_counts_messages_by_brute_force():
    # Section 4.3.1: every worker exchanges B pairs of (M + N)-vectors with P-1 peers; the
    # paper's total is (P-1)^2 B (M+N).  Count it by enumeration for tiny cases.
    for P, B, M, N in itertools.product([1, 2, 3, 5], [1, 4], [3, 6], [2, 7]):
        total = 0
        for _a in range(P - 1):
            for _b in range(P - 1):
                for _s in range(B):
                    total += M + N
        assert orc.plan_layer(FC, M, N, B, P)["cost_sfb"] == total
        # full matrices: P workers, one push and one pull of M*N floats each
        assert orc.plan_layer(FC, M, N, B, P)["cost_ps_dense"] == sum(2 * M * N for _ in range(P))
        assert orc.plan_layer(FC, M, N, B, P)["cost_sf_ps"] == sum(B * (M + N) + M * N for _ in range(P))


def test_quadratic_growth_in_workers():
    # Section 4.3.1 (last paragraph): SFB's volume grows quadratically with the node count
    M, N, B = 4096, 4096, 256
    c = [orc.plan_layer(FC, M, N, B, P)["cost_sfb"] for P in range(1, 40)]
    second = [c[i + 2] - 2 * c[i + 1] + c[i] for i in range(len(c) - 2)]
    assert len(set(second)) == 1 and second[0] == 2 * B * (M + N)
    d = [orc.plan_layer(FC, M, N, B, P)["cost_ps_dense"] for P in range(1, 40)]
    assert len({d[i + 1] - d[i] for i in range(len(d) - 1)}) == 1  # linear


def test_symmetry_in_M_and_N():
    for M, N, B, P in [(4096, 1000, 256, 8), (9216, 4096, 32, 16), (3, 5, 1, 2)]:
        a, b = orc.plan_layer(FC, M, N, B, P), orc.plan_layer(FC, N, M, B, P)
        for k in ("cost_sfb", "cost_ps_dense", "cost_sf_ps", "route_alg3", "route_vs_dense"):
            assert a[k] == b[k]


def test_alg3_decision_matches_rational_breakeven():
    # Solve Alg. 3's inequality for B by hand with exact rationals and compare decisions.
    for M, N, P in itertools.product([8, 100, 4096], [8, 1000, 21841], [1, 2, 3, 4, 8, 16, 33]):
        c = (P - 1) ** 2 - P
        for B in [1, 2, 31, 32, 64, 128, 256, 1000, 5000]:
            if c <= 0:
                want = orc.ROUTE_SFB
            else:
                want = orc.ROUTE_SFB if Fraction(B) <= Fraction(P * M * N, c * (M + N)) else orc.ROUTE_SF_PS
            assert orc.plan_layer(FC, M, N, B, P)["route_alg3"] == want
        be = orc.sfb_breakeven_batch(M, N, P)
        if be is None:
            assert c <= 0
        else:
            assert be < 1 or orc.plan_layer(FC, M, N, max(be, 1), P)["route_alg3"] == orc.ROUTE_SFB
            assert orc.plan_layer(FC, M, N, be + 1, P)["route_alg3"] == orc.ROUTE_SF_PS


def test_tie_goes_to_sfb():
    # P=3: (P-1)^2 - P = 1, so equality holds when B (M+N) = 3 M N, e.g. M=N=2, B=3
    p = orc.plan_layer(FC, 2, 2, 3, 3)
    assert p["cost_sfb"] == p["cost_sf_ps"] and p["route_alg3"] == orc.ROUTE_SFB
    # vs-dense tie: (P-1)^2 B (M+N) = 2 P M N with P=2: B (M+N) = 4 M N, M=N=1, B=2
    p = orc.plan_layer(FC, 1, 1, 2, 2)
    assert p["cost_sfb"] == p["cost_ps_dense"] and p["route_vs_dense"] == orc.ROUTE_SFB


def test_conv_always_goes_to_the_server():
    for M, N, B, P in [(363, 96, 256, 8), (2, 2, 1, 1)]:
        p = orc.plan_layer(CONV, M, N, B, P)
        assert p["route_alg3"] == orc.ROUTE_PS_DENSE == p["route_vs_dense"]


# Routes for the workloads of this build, worked out by hand from the three formulas
# (costs written out so a slip in any formula shows).
HAND = [
    # M, N, B, P, sfb, sf_ps, dense, alg3, vs_dense
    (256, 128, 32, 4, 9 * 32 * 384, 4 * 32 * 384 + 4 * 256 * 128, 2 * 4 * 256 * 128, "SFB", "SFB"),
    (4096, 1000, 256, 8, 49 * 256 * 5096, 8 * 256 * 5096 + 8 * 4096000, 16 * 4096000, "SF_PS", "SFB"),
    (9216, 4096, 256, 8, 49 * 256 * 13312, 2048 * 13312 + 8 * 9216 * 4096, 16 * 9216 * 4096, "SFB", "SFB"),
    (4096, 4096, 256, 8, 49 * 256 * 8192, 2048 * 8192 + 8 * 4096 * 4096, 16 * 4096 * 4096, "SFB", "SFB"),
    (4096, 21841, 256, 8, 49 * 256 * 25937, 2048 * 25937 + 8 * 4096 * 21841, 16 * 4096 * 21841, "SFB", "SFB"),
    (4096, 4096, 256, 16, 225 * 256 * 8192, 4096 * 8192 + 16 * 4096 * 4096, 32 * 4096 * 4096, "SF_PS", "SFB"),
]
NAMES = {"SFB": orc.ROUTE_SFB, "SF_PS": orc.ROUTE_SF_PS, "PS": orc.ROUTE_PS_DENSE}


@pytest.mark.parametrize("row", HAND)
def test_workload_routes(row):
    M, N, B, P, sfb, sf_ps, dense, a3, vd = row
    p = orc.plan_layer(FC, M, N, B, P)
    assert (p["cost_sfb"], p["cost_sf_ps"], p["cost_ps_dense"]) == (sfb, sf_ps, dense)
    assert p["route_alg3"] == NAMES[a3] and p["route_vs_dense"] == NAMES[vd]
    assert (sfb <= sf_ps) == (a3 == "SFB") and (sfb <= dense) == (vd == "SFB")


def test_22k_grid_is_all_sfb():
    for B in (32, 64, 128, 256):
        for P in (2, 4, 8, 16):
            p = orc.plan_layer(FC, 4096, 21841, B, P)
            assert (P - 1) ** 2 * B * (4096 + 21841) <= P * B * (4096 + 21841) + P * 4096 * 21841
            assert p["route_alg3"] == orc.ROUTE_SFB and p["route_vs_dense"] == orc.ROUTE_SFB


def test_costs_need_64_bits_and_overflow_is_reported():
    assert orc.plan_layer(FC, 4096, 21841, 256, 16)["cost_ps_dense"] > 2 ** 31
    with pytest.raises(OverflowError):
        orc.plan_layer(FC, 2 ** 31, 2 ** 31, 1, 4)
    with pytest.raises(ValueError):
        orc.plan_layer(FC, 0, 4, 1, 1)


# ---------------------------------------------------------------------------------------
# shards
# ---------------------------------------------------------------------------------------
def test_shards_cover_disjoint_balanced():
    for n in list(range(1, 40)) + [97, 1000, 34848, 21841 * 4096]:
        for S in [1, 2, 3, 7, 8, 16, 37]:
            if S > n:
                continue
            r = [orc.shard_range(n, S, s) for s in range(S)]
            assert r[0][0] == 0 and r[-1][1] == n
            assert all(r[i][1] == r[i + 1][0] for i in range(S - 1))
            sizes = [e - b for b, e in r]
            assert max(sizes) - min(sizes) <= 1 and min(sizes) >= 1


def test_shards_brute_force_owner():
    # key i belongs to the shard s with s*n <= i*S + (something) ... check by enumeration:
    # the ranges assign each key exactly once and in order
    for n, S in [(10, 3), (11, 11), (13, 5), (64, 8)]:
        owner = [-1] * n
        for s in range(S):
            b, e = orc.shard_range(n, S, s)
            for i in range(b, e):
                assert owner[i] == -1
                owner[i] = s
        assert owner == sorted(owner) and -1 not in owner and set(owner) == set(range(S))


def test_config5_shard_sizes():
    # 8 shards of each conv layer: all five counts divide by 8 (hand arithmetic)
    want = [34848 // 8, 307200 // 8, 884736 // 8, 663552 // 8, 442368 // 8]
    assert want == [4356, 38400, 110592, 82944, 55296]
    for n, w in zip(inputs.conv_sizes(), want):
        for s in range(8):
            b, e = orc.shard_range(n, 8, s)
            assert (b, e) == (s * w, (s + 1) * w)


def test_shard_range_rejects_bad_arguments():
    for n, S, s in [(4, 5, 0), (4, 0, 0), (4, 2, 2), (4, 2, -1)]:
        with pytest.raises(ValueError):
            orc.shard_range(n, S, s)


# ---------------------------------------------------------------------------------------
# Fig. 4 (missing from the paper text): the three strategies between fc6 and fc7
# (M = N = 4096) as the node count P and the per-node batch K vary.  The figure itself is
# gone, but its caption and the paragraph after it fix what it must show.
# ---------------------------------------------------------------------------------------
def test_fig4_regenerated_from_the_closed_forms():
    M = N = 4096
    # (1) varying P at K = 256: SFB grows quadratically and eventually loses to both others
    sfb = [orc.plan_layer(FC, M, N, 256, P)["cost_sfb"] for P in range(1, 65)]
    dense = [orc.plan_layer(FC, M, N, 256, P)["cost_ps_dense"] for P in range(1, 65)]
    sfps = [orc.plan_layer(FC, M, N, 256, P)["cost_sf_ps"] for P in range(1, 65)]
    assert all(a < b for a, b in zip(sfb[:8], dense[:8]))            # small clusters: SFB wins clearly
    first_loss_vs_sfps = next(P for P in range(1, 65) if sfb[P - 1] > sfps[P - 1])
    first_loss_vs_dense = next(P for P in range(1, 65) if sfb[P - 1] > dense[P - 1])
    assert first_loss_vs_sfps == 11 and first_loss_vs_dense == 18    # hand-solved from the inequalities
    assert all(sfps[i] < dense[i] for i in range(64))                # factors-to-server always beats full matrices here
    # (2) varying K at P = 8: "SFB usually outperforms the other two with a smaller batch size"
    for K in (1, 16, 64, 256):
        p = orc.plan_layer(FC, M, N, K, 8)
        assert p["cost_sfb"] < p["cost_sf_ps"] < p["cost_ps_dense"]
    big = orc.plan_layer(FC, M, N, 1024, 8)
    assert big["cost_sfb"] > big["cost_sf_ps"]                        # large batches flip the choice
    assert big["route_alg3"] == orc.ROUTE_SF_PS
    # SFB and factors-to-server grow linearly in K, full matrices do not depend on K
    c = [orc.plan_layer(FC, M, N, K, 8) for K in (100, 200, 300)]
    assert c[1]["cost_sfb"] - c[0]["cost_sfb"] == c[2]["cost_sfb"] - c[1]["cost_sfb"]
    assert c[0]["cost_ps_dense"] == c[2]["cost_ps_dense"]
