"""Pins for the EMA + priority oracle (section 3.4 importance scores, head weights,
times the posterior mean of Eq. 5): closed forms of the recurrence and special cases."""
import numpy as np
import pytest

RES, HOST, PROT, SCORED = 1, 2, 4, 8


def one_row(n_blocks, n_tok=None):
    n_tok = n_blocks * 16 if n_tok is None else n_tok
    return np.array([n_tok], np.int32), np.array([0], np.int64)


def test_constant_input_closed_form_and_fixed_point(oracle):
    ntok, off = one_row(4)
    m = np.array([0.4, 0.1, 0.3, 0.2], np.float32)
    s0 = np.array([1.0, 0.0, 0.3, 0.5], np.float32)
    S, state = s0.copy(), np.full(4, RES | SCORED, np.uint8)
    prio = np.zeros(4, np.float32)
    w, pair, p_hat = np.ones(1, np.float32), np.zeros(4, np.uint8), np.ones(16, np.float32)
    d = 0.9
    for t in range(1, 41):
        oracle.ema_update(ntok, off, m, d, w, pair, p_hat, state, S, prio)
        want = d ** t * s0.astype(np.float64) + (1 - d ** t) * m.astype(np.float64)
        np.testing.assert_allclose(S, want, rtol=2e-6)
    assert S[2] == np.float32(0.3)                      # S == m is a fixed point
    np.testing.assert_array_equal(prio, S)              # w = 1, p_hat = 1


def test_first_observation_initialises_and_sets_scored(oracle):
    ntok, off = one_row(3)
    m = np.array([0.5, 0.25, 0.25], np.float32)
    S = np.array([9.0, 9.0, 9.0], np.float32)
    state = np.array([RES, RES | SCORED, 0], np.uint8)        # unit 2 is not resident
    prio = np.zeros(3, np.float32)
    oracle.ema_update(ntok, off, m, 0.5, np.ones(1, np.float32), np.zeros(3, np.uint8),
                      np.ones(16, np.float32), state, S, prio)
    np.testing.assert_array_equal(S, np.array([0.5, 0.5 * 9 + 0.5 * 0.25, 9.0], np.float32))
    np.testing.assert_array_equal(state, np.array([RES | SCORED, RES | SCORED, 0], np.uint8))
    assert prio[0] == 0.5 and np.isinf(prio[2]) and prio[2] > 0


@pytest.mark.parametrize("decay,want", [(0.0, "x"), (1.0, "s")])
def test_decay_extremes(oracle, decay, want):
    ntok, off = one_row(2)
    m, S = np.array([0.7, 0.3], np.float32), np.array([0.2, 0.8], np.float32)
    s_before = S.copy()
    state, prio = np.full(2, RES | SCORED, np.uint8), np.zeros(2, np.float32)
    oracle.ema_update(ntok, off, m, decay, np.ones(1, np.float32), np.zeros(2, np.uint8),
                      np.ones(16, np.float32), state, S, prio)
    np.testing.assert_array_equal(S, m if want == "x" else s_before)


def test_priority_is_weight_times_ema_times_posterior(oracle):
    rng = np.random.default_rng(0)
    ntok = np.array([40, 64, 7], np.int32)           # 3, 4, 1 blocks
    off = np.array([0, 5, 12], np.int64)             # gaps after each row
    n = 14
    mass = rng.random(n).astype(np.float32)
    S = rng.random(n).astype(np.float32)
    state = np.zeros(n, np.uint8)
    for o, k in zip(off, (3, 4, 1)):
        state[o:o + k] = RES | SCORED
    pair = rng.integers(0, 16, n).astype(np.uint8)
    p_hat = rng.random(16).astype(np.float32)
    w = np.array([4.0, 1.0, 0.5], np.float32)
    prio = np.full(n, -1.0, np.float32)
    S_in = S.copy()
    oracle.ema_update(ntok, off, mass, 0.95, w, pair, p_hat, state, S, prio)
    for r, (o, k) in enumerate(zip(off, (3, 4, 1))):
        for u in range(o, o + k):
            s = 0.95 * float(S_in[u]) + (1 - 0.95) * float(mass[u])
            assert abs(S[u] - s) <= 1e-6 * s
            assert abs(prio[u] - float(w[r]) * float(S[u]) * float(p_hat[pair[u]])) <= 1e-6 * abs(prio[u])
    untouched = np.ones(n, bool)
    for o, k in zip(off, (3, 4, 1)):
        untouched[o:o + k] = False
    assert np.all(prio[untouched] == -1.0) and np.all(S[untouched] == S_in[untouched])


def test_inactive_row_keeps_ema_but_refreshes_priority(oracle):
    ntok = np.array([32, 32], np.int32)
    off = np.array([0, 2], np.int64)
    mass = np.array([0.9, 0.1, 0.6, 0.4], np.float32)
    S = np.array([0.5, 0.5, 0.5, 0.5], np.float32)
    state = np.full(4, RES | SCORED, np.uint8)
    prio = np.zeros(4, np.float32)
    p_hat = np.full(16, 0.25, np.float32)
    active = np.array([1, 0], np.uint8)
    oracle.ema_update(ntok, off, mass, 0.5, np.ones(2, np.float32), np.zeros(4, np.uint8), p_hat,
                      state, S, prio, row_active=active)
    np.testing.assert_array_equal(S, np.array([0.7, 0.3, 0.5, 0.5], np.float32))
    np.testing.assert_array_equal(prio, S * np.float32(0.25))


def test_on_host_unit_keeps_its_ema(oracle):
    ntok, off = one_row(2)
    S = np.array([0.4, 0.6], np.float32)
    state = np.array([HOST | SCORED, RES | SCORED], np.uint8)
    prio = np.zeros(2, np.float32)
    oracle.ema_update(ntok, off, np.array([0.0, 1.0], np.float32), 0.5, np.full(1, 2.0, np.float32),
                      np.zeros(2, np.uint8), np.ones(16, np.float32), state, S, prio)
    np.testing.assert_array_equal(S, np.array([0.4, 0.8], np.float32))
    np.testing.assert_array_equal(prio, np.array([0.8, 1.6], np.float32))
