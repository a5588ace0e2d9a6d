"""Pins for the refined EMA (section 3.4: positional distance decay; sections 3.4 / 3.7: per-head
multipliers chosen by the transition type): reduction to the plain update, closed forms, a
vectorised numpy restatement, and the ordering the decay is meant to produce."""
import numpy as np
import pytest

RES, HOST, PROT, SCORED = 1, 2, 4, 8


def random_rows(rng, n_rows, max_blocks=40, gap=3):
    ntok = rng.integers(1, max_blocks * 16, n_rows).astype(np.int32)
    nb = (ntok + 15) // 16
    off = np.zeros(n_rows, np.int64)
    pos = 0
    for r in range(n_rows):
        off[r] = pos
        pos += nb[r] + rng.integers(0, gap)
    return ntok, off, int(pos) + 1


def random_state(rng, n):
    st = rng.choice(np.array([0, RES, RES | SCORED, HOST | SCORED, RES | SCORED | PROT, HOST], np.uint8), n)
    return st.astype(np.uint8)


def test_no_decay_no_multipliers_is_the_plain_update_bit_for_bit(oracle):
    rng = np.random.default_rng(1)
    ntok, off, n = random_rows(rng, 12)
    mass, S0 = rng.random(n).astype(np.float32), rng.random(n).astype(np.float32)
    st0 = random_state(rng, n)
    w = rng.random(12).astype(np.float32) * 4
    pair, p_hat = rng.integers(0, 16, n).astype(np.uint8), rng.random(16).astype(np.float32)
    act = (rng.random(12) < 0.7).astype(np.uint8)
    out = []
    for ex in (False, True):
        S, st, prio = S0.copy(), st0.copy(), np.full(n, -1, np.float32)
        if ex:
            oracle.ema_update_ex(ntok, off, mass, 0.9, 1.0, w, pair, p_hat, st, S, prio, row_active=act)
        else:
            oracle.ema_update(ntok, off, mass, 0.9, w, pair, p_hat, st, S, prio, row_active=act)
        out.append((S, st, prio))
    for a, b in zip(*out):
        np.testing.assert_array_equal(a, b)


def test_numpy_restatement(oracle):
    """Same recurrence written with whole-array numpy operations in fp64."""
    rng = np.random.default_rng(2)
    n_rows, n_seq, n_heads = 24, 5, 6
    ntok, off, n = random_rows(rng, n_rows)
    mass, S0 = rng.random(n).astype(np.float32), rng.random(n).astype(np.float32)
    st0 = random_state(rng, n)
    w = (1 + rng.integers(0, 8, n_rows)).astype(np.float32)
    pair, p_hat = rng.integers(0, 16, n).astype(np.uint8), rng.random(16).astype(np.float32)
    row_seq = rng.integers(0, n_seq, n_rows).astype(np.int32)
    row_head = rng.integers(0, n_heads, n_rows).astype(np.int32)
    trans = np.array([0, 3, 255, 1, 2], np.uint8)
    mult = (0.25 + rng.random((4, n_heads)) * 2).astype(np.float32)
    decay, delta = 0.8, 0.93
    S, st, prio = S0.copy(), st0.copy(), np.zeros(n, np.float32)
    oracle.ema_update_ex(ntok, off, mass, decay, delta, w, pair, p_hat, st, S, prio,
                         row_seq=row_seq, row_head=row_head, seq_transition=trans, head_mult=mult)
    # restatement
    row_of = np.full(n, -1)
    dist = np.zeros(n)
    for r in range(n_rows):
        nb = (ntok[r] + 15) // 16
        row_of[off[r]:off[r] + nb] = r
        dist[off[r]:off[r] + nb] = np.arange(nb)[::-1]
    used = row_of >= 0
    x = np.power(delta, dist) * mass.astype(np.float64)
    res = used & ((st0 & RES) != 0)
    first = res & ((st0 & SCORED) == 0)
    later = res & ((st0 & SCORED) != 0)
    S_want = S0.astype(np.float64)
    S_want[first] = x[first]
    S_want[later] = decay * S0[later].astype(np.float64) + (1 - decay) * x[later]
    np.testing.assert_allclose(S, S_want.astype(np.float32), rtol=1e-7)
    st_want = st0.copy()
    st_want[first] |= SCORED
    np.testing.assert_array_equal(st, st_want)
    t = trans[row_seq]
    m_row = np.where(t <= 3, mult[np.minimum(t, 3), row_head], 1.0)
    scored = used & ((st_want & SCORED) != 0)
    r_idx = row_of[scored]
    want = w[r_idx].astype(np.float64) * m_row[r_idx] * S[scored].astype(np.float64) * p_hat[pair[scored]]
    np.testing.assert_allclose(prio[scored], want, rtol=2e-7)
    assert np.all(np.isposinf(prio[used & ~scored]))
    assert np.all(prio[~used] == 0)            # entries outside every row are not written


@pytest.mark.parametrize("nb,n_tok", [(6, 96), (6, 81), (1, 3)])
def test_distance_counts_blocks_back_from_the_last_block(oracle, nb, n_tok):
    ntok, off = np.array([n_tok], np.int32), np.array([0], np.int64)
    mass = np.ones(nb, np.float32)
    S, st, prio = np.zeros(nb, np.float32), np.full(nb, RES, np.uint8), np.zeros(nb, np.float32)
    oracle.ema_update_ex(ntok, off, mass, 0.5, 0.5, np.ones(1, np.float32), np.zeros(nb, np.uint8),
                         np.ones(16, np.float32), st, S, prio)
    np.testing.assert_array_equal(S, (0.5 ** np.arange(nb)[::-1]).astype(np.float32))   # exact powers of two
    np.testing.assert_array_equal(prio, S)


def test_constant_input_closed_form_with_decay(oracle):
    """Constant mass m at distance d: S_t = decay^t S_0 + (1 - decay^t) delta^d m."""
    nb = 5
    ntok, off = np.array([nb * 16], np.int32), np.array([0], np.int64)
    m = np.array([0.4, 0.1, 0.3, 0.15, 0.05], np.float32)
    s0 = np.array([1.0, 0.0, 0.3, 0.5, 0.2], np.float32)
    S, st, prio = s0.copy(), np.full(nb, RES | SCORED, np.uint8), np.zeros(nb, np.float32)
    decay, delta = 0.9, 0.8
    d = np.arange(nb)[::-1]
    for t in range(1, 31):
        oracle.ema_update_ex(ntok, off, m, decay, delta, np.ones(1, np.float32), np.zeros(nb, np.uint8),
                             np.ones(16, np.float32), st, S, prio)
        want = decay ** t * s0.astype(np.float64) + (1 - decay ** t) * delta ** d * m.astype(np.float64)
        np.testing.assert_allclose(S, want, rtol=3e-6)


def test_equal_masses_make_the_farthest_blocks_the_first_victims(oracle):
    nb = 32
    ntok, off = np.array([nb * 16], np.int32), np.array([0], np.int64)
    S, st, prio = np.zeros(nb, np.float32), np.full(nb, RES, np.uint8), np.zeros(nb, np.float32)
    oracle.ema_update_ex(ntok, off, np.full(nb, 1 / nb, np.float32), 0.9, 0.97, np.ones(1, np.float32),
                         np.zeros(nb, np.uint8), np.ones(16, np.float32), st, S, prio)
    assert np.all(np.diff(prio) > 0)
    np.testing.assert_array_equal(oracle.select_victims(prio, st, k=5), np.arange(5))


def test_multiplier_only_scales_priority_and_only_during_a_transition(oracle):
    nb, n_heads = 3, 4
    ntok = np.full(n_heads * 2, nb * 16, np.int32)
    off = (np.arange(n_heads * 2) * nb).astype(np.int64)
    n = n_heads * 2 * nb
    rng = np.random.default_rng(4)
    mass = rng.random(n).astype(np.float32)
    row_seq = np.repeat(np.array([0, 1], np.int32), n_heads)
    row_head = np.tile(np.arange(n_heads, dtype=np.int32), 2)
    mult = np.array([[1, 1, 1, 1], [2, 0.5, 1, 4], [1, 1, 1, 1], [1, 1, 1, 1]], np.float32)
    base = {}
    for name, trans in (("none", [255, 255]), ("switch0", [1, 255])):
        S, st, prio = np.zeros(n, np.float32), np.full(n, RES, np.uint8), np.zeros(n, np.float32)
        oracle.ema_update_ex(ntok, off, mass, 0.9, 1.0, np.ones(len(ntok), np.float32), np.zeros(n, np.uint8),
                             np.ones(16, np.float32), st, S, prio, row_seq=row_seq, row_head=row_head,
                             seq_transition=np.array(trans, np.uint8), head_mult=mult)
        base[name] = (S, prio)
    np.testing.assert_array_equal(base["none"][0], base["switch0"][0])      # S unaffected
    ratio = base["switch0"][1] / base["none"][1]
    want = np.r_[np.repeat(mult[1], nb), np.ones(n_heads * nb)]
    np.testing.assert_array_equal(ratio.astype(np.float32), want.astype(np.float32))  # powers of two: exact


def test_rejects_bad_arguments(oracle):
    ntok, off = np.array([16], np.int32), np.array([0], np.int64)
    a = dict(mass=np.ones(1, np.float32), row_weight=np.ones(1, np.float32), pair=np.zeros(1, np.uint8),
             p_hat=np.ones(16, np.float32), state=np.full(1, RES, np.uint8), S=np.zeros(1, np.float32),
             prio=np.zeros(1, np.float32))
    for delta in (0.0, 1.5, -0.1):
        with pytest.raises(oracle.OracleError):
            oracle.ema_update_ex(ntok, off, a["mass"], 0.9, delta, a["row_weight"], a["pair"], a["p_hat"],
                                 a["state"], a["S"], a["prio"])
    with pytest.raises(oracle.OracleError):     # head index outside the table
        oracle.ema_update_ex(ntok, off, a["mass"], 0.9, 1.0, a["row_weight"], a["pair"], a["p_hat"], a["state"],
                             a["S"], a["prio"], row_seq=np.zeros(1, np.int32), row_head=np.array([7], np.int32),
                             seq_transition=np.zeros(1, np.uint8), head_mult=np.ones((4, 2), np.float32))
