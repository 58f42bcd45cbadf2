"""Pins of the oracle's bounded-staleness view (Section 3.2): what a reader at clock t is guaranteed
to see under staleness s.  None of the expected values below comes from the oracle itself."""
from collections import deque

import numpy as np
import pytest

from oracle import psd_oracle as orc
from paper_1512_06216_amd import inputs


def test_window_is_all_clocks_up_to_t_minus_s_minus_1():
    # the statement of Section 3.2, written out clock by clock
    for s in range(0, 5):
        for t in range(0, 12):
            guaranteed = [c for c in range(0, t) if c <= t - s - 1]
            assert orc.ssp_updates_visible(t, s) == len(guaranteed)
            assert guaranteed == list(range(len(guaranteed)))          # a prefix: clocks 0 .. t-s-1
    # s = 0 is bulk synchronous: the reader at clock t has every earlier clock
    assert [orc.ssp_updates_visible(t, 0) for t in range(5)] == [0, 1, 2, 3, 4]
    with pytest.raises(ValueError):
        orc.ssp_updates_visible(-1, 0)


def test_window_equals_a_server_that_withholds_each_update_for_s_clocks():
    """Literal simulation: at the end of clock c the workers hand the server the update of clock c; the
    server holds the s most recent ones back.  What it has released before clock t starts is the view."""
    for s in range(0, 4):
        pending, released = deque(), []
        for t in range(0, 10):
            assert orc.ssp_updates_visible(t, s) == len(released)
            pending.append(t)                      # clock t's update is produced during clock t
            while len(pending) > s:
                released.append(pending.popleft())
        assert released == list(range(10 - s))


def test_plain_sgd_view_is_initial_weights_minus_the_sum_of_released_gradients():
    # mu = 0, wd = 0: W_visible(t) = W0 - lr * sum_{c <= t-s-1} dW_c, with dW_c from numpy's float64 matmul
    lr, T = 0.125, 6
    rng = np.random.default_rng(5)
    sets = [inputs.fc_layer_integer(M=24, N=10, B=3, P=2, seed=50 + c) for c in range(T)]
    W0 = sets[0]["W"]
    packed = [orc.pack_factors(d["delta"], d["act"]) for d in sets]
    updates = [(lambda W, M, UV=UV: orc.sync_fc_sfb(UV[0], UV[1], W, M, lr, 0.0)) for UV in packed]
    dW = [UV[0].astype(np.float64).T @ UV[1].astype(np.float64) for UV in packed]
    for s in (0, 1, 3):
        for t in range(0, T + 1):
            W, Mom = orc.ssp_visible_state(updates, W0, np.zeros_like(W0), s, t)
            n = max(0, t - s)
            want = W0.astype(np.float64) - lr * sum(dW[:n], np.zeros_like(dW[0]))
            assert np.array_equal(W, want.astype(np.float32)), (s, t)      # small integers: exact


def test_staleness_zero_is_the_bulk_synchronous_sequence_bit_for_bit():
    lr, mu, T = inputs.LR, inputs.MU, 4
    sets = [inputs.fc_layer(M=40, N=12, B=4, P=3, seed=70 + c, mom_std=1e-3) for c in range(T)]
    packed = [orc.pack_factors(d["delta"], d["act"]) for d in sets]
    updates = [(lambda W, M, UV=UV: orc.sync_fc_sfb(UV[0], UV[1], W, M, lr, mu)) for UV in packed]
    W, Mom = sets[0]["W"], sets[0]["Mom"]
    for t in range(T + 1):
        Wv, Mv = orc.ssp_visible_state(updates, sets[0]["W"], sets[0]["Mom"], 0, t)
        assert np.array_equal(Wv, W) and np.array_equal(Mv, Mom)
        if t < T:
            W, Mom = orc.sync_fc_sfb(packed[t][0], packed[t][1], W, Mom, lr, mu)
    # and a stale view is an earlier bulk-synchronous state: view(t, s) == view(t - s, 0)
    for s in (1, 2):
        for t in range(T + 1):
            a = orc.ssp_visible_state(updates, sets[0]["W"], sets[0]["Mom"], s, t)
            b = orc.ssp_visible_state(updates, sets[0]["W"], sets[0]["Mom"], 0, max(0, t - s))
            assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
