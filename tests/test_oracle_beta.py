"""Pins for the Beta-posterior oracle (section 3.3, Eq. 5): closed forms, the
convergence figures the paper states, and counting identities."""
import numpy as np
import pytest

from paper_2604_26968_amd import synth


def fresh():
    return np.zeros(16, np.uint32), np.zeros(16, np.uint32)


def test_prior_mean_and_single_updates(oracle):
    hits, misses = fresh()
    p = oracle.beta_update(np.zeros(0, np.uint8), np.zeros(0, np.uint8), hits, misses)
    np.testing.assert_array_equal(p, np.full(16, 0.5, np.float32))     # Beta(1,1) mean
    p = oracle.beta_update(np.array([5], np.uint8), np.array([1], np.uint8), hits, misses)
    assert p[5] == np.float32(2 / 3) and hits[5] == 1 and misses[5] == 0
    p = oracle.beta_update(np.array([5, 9], np.uint8), np.array([0, 0], np.uint8), hits, misses)
    assert p[5] == np.float32(2 / 4) and p[9] == np.float32(1 / 3)
    assert np.all(np.delete(p, [5, 9]) == 0.5)


@pytest.mark.parametrize("n", [1, 10, 100, 499])
def test_n_hits_closed_form(oracle, n):
    hits, misses = fresh()
    p = oracle.beta_update(np.full(n, 3, np.uint8), np.ones(n, np.uint8), hits, misses)
    assert p[3] == np.float32((1 + n) / (2 + n))
    hits, misses = fresh()
    p = oracle.beta_update(np.full(n, 3, np.uint8), np.zeros(n, np.uint8), hits, misses)
    assert p[3] == np.float32(1 / (2 + n))


def test_pair_index_is_four_times_block_type_plus_transition(oracle):
    # (system_prompt = 0, same_tool_repeat = 0) is pair 0; (intermediate_reasoning = 3, agent_handoff = 3) is 15
    hits, misses = fresh()
    ev = np.array([4 * 0 + 0, 4 * 3 + 3, 4 * 1 + 2], np.uint8)
    oracle.beta_update(ev, np.array([1, 0, 1], np.uint8), hits, misses)
    assert hits[0] == 1 and misses[15] == 1 and hits[6] == 1 and hits.sum() + misses.sum() == 3


def test_paper_convergence_above_097_within_500(oracle):
    """Section 5.5: the (system_prompt, same_tool_repeat) posterior mean exceeds 0.97 within 500
    observations.  With 486 reuses in 500 lookups the mean is 487/502 > 0.97; with 485 it is not."""
    for n_hit, above in ((486, True), (485, False)):
        hits, misses = fresh()
        out = np.r_[np.ones(n_hit, np.uint8), np.zeros(500 - n_hit, np.uint8)]
        p = oracle.beta_update(np.zeros(500, np.uint8), out, hits, misses)
        assert (p[0] > 0.97) == above
        assert abs(float(p[0]) - (1 + n_hit) / 502) < 1e-7


def test_symmetric_priors_wash_out_within_100(oracle):
    """Table 9 footnote: three symmetric priors agree after 100 observations."""
    ev_p, ev_o = synth.make_events(1600, 7, reuse_prob=np.linspace(0.05, 0.95, 16))
    ps = []
    for a0 in (0.5, 1.0, 2.0):
        hits, misses = fresh()
        ps.append(oracle.beta_update(ev_p, ev_o, hits, misses, alpha0=a0, beta0=a0).astype(np.float64))
        n_obs = hits + misses
    assert n_obs.min() >= 60
    spread = np.max(ps, 0) - np.min(ps, 0)
    assert spread.max() < 0.02
    # closed form of the spread for a symmetric prior a: |h + a|/(n + 2a)
    for a0, p in zip((0.5, 1.0, 2.0), ps):
        np.testing.assert_allclose(p, (hits + a0) / (n_obs + 2 * a0), rtol=1e-6)


def test_counts_are_histograms_and_bad_events_are_skipped(oracle):
    ev_p, ev_o = synth.make_events(5000, 3, pair_weights=synth.categorical_weights(4))
    ev_p[17], ev_o[40], ev_p[99] = 16, 2, 255
    hits, misses = fresh()
    hits[2], misses[7] = 10, 20           # counters accumulate across calls
    bad = np.zeros(1, np.uint32)
    oracle.beta_update(ev_p, ev_o, hits, misses, n_bad=bad)
    ok = (ev_p < 16) & (ev_o <= 1)
    want_h = np.bincount(ev_p[ok & (ev_o == 1)], minlength=16)
    want_m = np.bincount(ev_p[ok & (ev_o == 0)], minlength=16)
    want_h[2] += 10
    want_m[7] += 20
    np.testing.assert_array_equal(hits, want_h)
    np.testing.assert_array_equal(misses, want_m)
    assert bad[0] == 3 and hits.sum() + misses.sum() == 5000 - 3 + 30


def test_rejects_nonpositive_prior(oracle):
    hits, misses = fresh()
    with pytest.raises(oracle.OracleError):
        oracle.beta_update(np.zeros(1, np.uint8), np.zeros(1, np.uint8), hits, misses, alpha0=0.0)
