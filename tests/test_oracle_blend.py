"""Pins for the blended reuse estimate (section 3.3, the two paragraphs after Eq. 5):
brute force with a bounded deque per pair, closed forms while the window still holds every
observation, the limits the text states (confidence saturates towards 1; fresh pairs follow the
empirical frequency, well-observed pairs the posterior; a distribution shift is tracked faster by the
blend than by the posterior), and agreement with the plain posterior update."""
from collections import deque

import numpy as np
import pytest

from paper_2604_26968_amd import synth


def fresh(window):
    return (np.zeros(16, np.uint32), np.zeros(16, np.uint32),
            np.full((16, window), 255, np.uint8), np.zeros(16, np.uint32))


def brute(ev_p, ev_o, window, kappa, a0=1.0, b0=1.0, state=None):
    """Independent restatement: one deque(maxlen=window) per pair."""
    st = state or {"h": [0] * 16, "m": [0] * 16, "dq": [deque(maxlen=window) for _ in range(16)]}
    for p, o in zip(ev_p.tolist(), ev_o.tolist()):
        if p >= 16 or o > 1:
            continue
        st["h" if o else "m"][p] += 1
        st["dq"][p].append(o)
    post, conf, blend = [], [], []
    for i in range(16):
        h, m = st["h"][i], st["m"][i]
        po = (a0 + h) / (a0 + b0 + h + m)
        n = h + m
        c = n / (n + kappa) if n + kappa > 0 else 0.0
        f = sum(st["dq"][i]) / len(st["dq"][i]) if st["dq"][i] else po
        post.append(po), conf.append(c), blend.append(c * po + (1 - c) * f)
    return np.array(post), np.array(conf), np.array(blend), st


@pytest.mark.parametrize("window,kappa,n_events", [(8, 4.0, 300), (64, 16.0, 5000), (5, 0.5, 37), (1, 10.0, 50)])
def test_against_deque_brute_force_over_several_calls(oracle, window, kappa, n_events):
    hits, misses, win, head = fresh(window)
    st = None
    for call in range(4):
        ev_p, ev_o = synth.make_events(n_events, 100 + call, reuse_prob=np.linspace(0.1, 0.9, 16))
        if call == 2:   # malformed events are skipped by both
            ev_p = ev_p.copy(); ev_o = ev_o.copy()
            ev_p[::7] = 16 + (np.arange(len(ev_p[::7])) % 200)
            ev_o[3::11] = 2
        p_hat, conf, p_blend = oracle.beta_blend_update(ev_p, ev_o, hits, misses, win, head, kappa)
        bp, bc, bb, st = brute(ev_p, ev_o, window, kappa, state=st)
        np.testing.assert_allclose(p_hat, bp, rtol=1e-7)
        np.testing.assert_allclose(conf, bc, rtol=1e-7)
        np.testing.assert_allclose(p_blend, bb, rtol=1e-7)
        assert list(hits) == st["h"] and list(misses) == st["m"]


def test_posterior_and_counters_equal_plain_update(oracle):
    ev_p, ev_o = synth.make_events(3000, 5)
    hits, misses, win, head = fresh(32)
    p_hat, _, _ = oracle.beta_blend_update(ev_p, ev_o, hits, misses, win, head, 8.0, alpha0=0.5, beta0=2.0)
    h2, m2 = np.zeros(16, np.uint32), np.zeros(16, np.uint32)
    p2 = oracle.beta_update(ev_p, ev_o, h2, m2, alpha0=0.5, beta0=2.0)
    np.testing.assert_array_equal(p_hat, p2)
    np.testing.assert_array_equal(hits, h2)
    np.testing.assert_array_equal(misses, m2)


def test_closed_form_while_window_holds_everything(oracle):
    """n <= window: f = h / n, so blend = c (1 + h) / (2 + n) + (1 - c) h / n with c = n / (n + kappa)."""
    kappa = 10.0
    for h, m in ((3, 1), (0, 5), (7, 0), (20, 20)):
        hits, misses, win, head = fresh(64)
        ev_o = np.r_[np.ones(h, np.uint8), np.zeros(m, np.uint8)]
        _, conf, blend = oracle.beta_blend_update(np.full(h + m, 9, np.uint8), ev_o, hits, misses, win, head, kappa)
        n = h + m
        c = n / (n + kappa)
        assert conf[9] == np.float32(c)
        assert abs(float(blend[9]) - (c * (1 + h) / (2 + n) + (1 - c) * h / n)) < 1e-7
        # untouched pairs: no observation -> confidence 0, empty window -> the prior mean
        assert conf[0] == 0 and blend[0] == np.float32(0.5)


def test_confidence_is_monotone_and_saturates_towards_one(oracle):
    hits, misses, win, head = fresh(16)
    last = -1.0
    for step in range(12):
        n_new = 2 ** step
        _, conf, _ = oracle.beta_blend_update(np.full(n_new, 2, np.uint8), np.ones(n_new, np.uint8),
                                              hits, misses, win, head, 25.0)
        assert conf[2] > last
        last = float(conf[2])
    assert 0.99 < last < 1.0
    # n == kappa is the half-way point
    hits, misses, win, head = fresh(16)
    _, conf, _ = oracle.beta_blend_update(np.full(25, 2, np.uint8), np.ones(25, np.uint8), hits, misses, win, head, 25.0)
    assert conf[2] == np.float32(0.5)


def test_kappa_zero_is_the_posterior_and_huge_kappa_the_window_frequency(oracle):
    ev_p, ev_o = synth.make_events(4000, 11, reuse_prob=np.linspace(0.2, 0.8, 16))
    hits, misses, win, head = fresh(50)
    p_hat, conf, blend = oracle.beta_blend_update(ev_p, ev_o, hits, misses, win, head, 0.0)
    np.testing.assert_array_equal(blend, p_hat)
    assert np.all(conf == 1)
    hits, misses, win, head = fresh(50)
    _, conf, blend = oracle.beta_blend_update(ev_p, ev_o, hits, misses, win, head, 1e12)
    for i in range(16):
        last = ev_o[ev_p == i][-50:]
        assert abs(float(blend[i]) - last.mean()) < 1e-6


def test_only_the_last_window_observations_count(oracle):
    """1000 misses then exactly `window` reuses: the window frequency is 1 whatever came before."""
    hits, misses, win, head = fresh(20)
    ev_o = np.r_[np.zeros(1000, np.uint8), np.ones(20, np.uint8)]
    _, conf, blend = oracle.beta_blend_update(np.full(1020, 4, np.uint8), ev_o, hits, misses, win, head, 1e12)
    assert abs(float(blend[4]) - 1.0) < 1e-6
    # one more miss pushes one reuse out: 19 / 20
    _, _, blend = oracle.beta_blend_update(np.array([4], np.uint8), np.array([0], np.uint8), hits, misses, win, head, 1e12)
    assert abs(float(blend[4]) - 19 / 20) < 1e-6
    assert head[4] == (1021 % 20)


def test_blend_tracks_a_distribution_shift_faster_than_the_posterior(oracle):
    """Section 3.3: the blend adapts quickly to a shift.  400 observations at reuse rate 0.9, then the
    rate drops to 0.1: after 60 more observations the blend is closer to 0.1 than the posterior mean."""
    rng = np.random.default_rng(3)
    hits, misses, win, head = fresh(32)
    o1 = (rng.random(400) < 0.9).astype(np.uint8)
    o2 = (rng.random(60) < 0.1).astype(np.uint8)
    oracle.beta_blend_update(np.full(400, 1, np.uint8), o1, hits, misses, win, head, 400.0)
    p_hat, conf, blend = oracle.beta_blend_update(np.full(60, 1, np.uint8), o2, hits, misses, win, head, 400.0)
    assert abs(float(blend[1]) - 0.1) < abs(float(p_hat[1]) - 0.1) - 0.2
    assert p_hat[1] > blend[1]


def test_rejects_bad_arguments(oracle):
    hits, misses, win, head = fresh(8)
    e = np.zeros(1, np.uint8)
    with pytest.raises(oracle.OracleError):
        oracle.beta_blend_update(e, e, hits, misses, win, head, -1.0)
    head[3] = 8
    with pytest.raises(oracle.OracleError):
        oracle.beta_blend_update(e, e, hits, misses, win, head, 1.0)
