"""Pins for position-aware prefetching (section 3.5): the per-layer window from the observed
attention span (exact integer arithmetic, checked with Fractions and closed forms) and the
candidate keys inside the window around the decode position (numpy restatement, window edges,
ordering)."""
from fractions import Fraction

import numpy as np
import pytest

RES, HOST, PROT, SCORED = 1, 2, 4, 8


def span_brute(masses, resident, theta):
    """Exact: smallest s >= 1 with sum of the last s fixed-point masses >= theta * total."""
    q = []
    for m, r in zip(masses, resident):
        m = float(np.float32(m))
        q.append(int(Fraction(min(m, 1.0)) * 2 ** 32) if (r and m > 0) else 0)   # floor of an exact product
    total = sum(q)
    if total == 0:
        return None
    acc = 0
    for s in range(1, len(q) + 1):
        acc += q[-s]
        if Fraction(acc) >= theta * total:
            return s
    return len(q)


def run_span(oracle, ntok, off, layer, mass, state, theta=(9, 10), n_layers=None, w_min=0, w_max=1 << 30,
             active=None, window0=None, sums=None):
    n_layers = n_layers or int(layer.max()) + 1
    s, c = sums if sums else (np.zeros(n_layers, np.uint64), np.zeros(n_layers, np.uint32))
    win = np.full(n_layers, -7, np.int32) if window0 is None else window0
    oracle.span_update(ntok, off, layer, mass, state, theta[0], theta[1], s, c, w_min, w_max, win, row_active=active)
    return s, c, win


def test_uniform_masses_give_ceil_theta_nb(oracle):
    for nb in (1, 2, 10, 37, 500):
        ntok, off = np.array([nb * 16], np.int32), np.array([0], np.int64)
        mass, st = np.full(nb, 0.125, np.float32), np.full(nb, RES, np.uint8)
        s, c, win = run_span(oracle, ntok, off, np.zeros(1, np.int32), mass, st, theta=(9, 10))
        want = -(-9 * nb // 10)
        assert s[0] == want and c[0] == 1 and win[0] == 16 * want


def test_geometric_masses_closed_form(oracle):
    """mass 2^-d at distance d (exact in fixed point): trailing s blocks hold (1 - 2^-s) / (1 - 2^-nb)."""
    nb = 20
    ntok, off = np.array([nb * 16 - 5], np.int32), np.array([0], np.int64)
    mass = (0.5 ** np.arange(nb)[::-1]).astype(np.float32)
    st = np.full(nb, RES, np.uint8)
    for num, den, want in ((1, 2, 1), (3, 4, 2), (7, 8, 3), (9, 10, 4), (999, 1000, 10), (1, 1, 20), (0, 1, 1)):
        s, _, _ = run_span(oracle, ntok, off, np.zeros(1, np.int32), mass, st, theta=(num, den))
        assert s[0] == want, (num, den, s[0])


def test_random_rows_against_fraction_brute_force_and_layer_mean(oracle):
    rng = np.random.default_rng(5)
    n_rows, n_layers = 60, 4
    nb = rng.integers(1, 50, n_rows)
    ntok = (nb * 16 - rng.integers(0, 16, n_rows)).astype(np.int32)
    off = np.r_[0, np.cumsum(nb + 2)[:-1]].astype(np.int64)
    n = int(off[-1] + nb[-1] + 2)
    mass = (rng.random(n) ** 4).astype(np.float32)
    mass[rng.random(n) < 0.05] = np.nan
    mass[rng.random(n) < 0.05] = -1.0
    mass[rng.random(n) < 0.02] = 1000.0                     # clamps to 1
    st = np.where(rng.random(n) < 0.7, RES, HOST).astype(np.uint8)
    layer = rng.integers(0, n_layers, n_rows).astype(np.int32)
    active = (rng.random(n_rows) < 0.8).astype(np.uint8)
    theta = Fraction(17, 20)
    s, c, win = run_span(oracle, ntok, off, layer, mass, st, theta=(17, 20), n_layers=n_layers + 1, active=active,
                         w_min=32, w_max=400)
    want_s, want_c = [0] * (n_layers + 1), [0] * (n_layers + 1)
    for r in range(n_rows):
        if not active[r]:
            continue
        sl = slice(off[r], off[r] + nb[r])
        sp = span_brute(mass[sl], (st[sl] & RES) != 0, theta)
        if sp is not None:
            want_s[layer[r]] += sp
            want_c[layer[r]] += 1
    assert list(s) == want_s and list(c) == want_c
    for l in range(n_layers):
        assert win[l] == min(max(16 * -(-want_s[l] // want_c[l]), 32), 400)
    assert win[n_layers] == -7                              # a layer without observations keeps its window


def test_local_layers_get_narrow_windows_and_global_layers_wide_ones(oracle):
    """Section 3.5: narrow for layers that attend locally, wide for layers that attend globally."""
    nb = 64
    ntok, off = np.full(2, nb * 16, np.int32), np.array([0, nb], np.int64)
    local = (0.3 ** np.arange(nb)[::-1]).astype(np.float32)           # mass piled on the newest blocks
    glob = np.full(nb, 1 / nb, np.float32)
    s, c, win = run_span(oracle, ntok, off, np.array([0, 1], np.int32), np.r_[local, glob],
                         np.full(2 * nb, RES, np.uint8))
    assert win[0] == 16 * 2 and win[1] == 16 * 58          # 1 - 0.3^2 = 0.91 >= 0.9;  ceil(0.9 * 64) = 58


def test_sums_accumulate_over_calls(oracle):
    ntok, off = np.array([160], np.int32), np.array([0], np.int64)
    st = np.full(10, RES, np.uint8)
    sums = (np.zeros(1, np.uint64), np.zeros(1, np.uint32))
    run_span(oracle, ntok, off, np.zeros(1, np.int32), np.full(10, 0.1, np.float32), st, sums=sums)     # span 9
    m = np.zeros(10, np.float32); m[-1] = 1
    _, _, win = run_span(oracle, ntok, off, np.zeros(1, np.int32), m, st, sums=sums)                  # span 1
    assert sums[0][0] == 10 and sums[1][0] == 2 and win[0] == 16 * 5


# ---- candidate keys -------------------------------------------------------------------------
def keys_numpy(ntok, off, layer, pos, window, state, pair, p_est, delta, n):
    key = np.full(n, -5.0, np.float32)
    cand = np.full(n, 77, np.uint8)
    for r in range(len(ntok)):
        nb = (ntok[r] + 15) // 16
        b = np.arange(nb)
        uid = off[r] + b
        npos, w = int(pos[r]), int(window[layer[r]])
        on_host = ((state[uid] & HOST) != 0) & ((state[uid] & RES) == 0)
        ok = on_host & (16 * b + 15 >= npos - w) & (16 * b <= npos) & (npos >= 0)
        k = 1.0 - p_est[pair[uid]].astype(np.float64) * np.power(delta, (npos // 16 - b).astype(np.float64))
        key[uid] = np.where(ok, k, np.inf).astype(np.float32)
        cand[uid] = np.where(ok, RES | SCORED, 0)
    return key, cand


def test_keys_against_numpy_restatement_and_select_brute_force(oracle):
    rng = np.random.default_rng(6)
    n_rows, n_layers = 40, 5
    nb = rng.integers(1, 70, n_rows)
    ntok = (nb * 16 - rng.integers(0, 16, n_rows)).astype(np.int32)
    off = np.r_[0, np.cumsum(nb + 1)[:-1]].astype(np.int64)
    n = int(off[-1] + nb[-1] + 1)
    layer = rng.integers(0, n_layers, n_rows).astype(np.int32)
    pos = np.where(rng.random(n_rows) < 0.15, -1, ntok - rng.integers(0, 3, n_rows)).astype(np.int32)
    window = np.array([0, 16, 100, 333, 5000], np.int32)
    state = rng.choice(np.array([RES | SCORED, HOST | SCORED, HOST, HOST | RES, 0], np.uint8), n).astype(np.uint8)
    pair = rng.integers(0, 16, n).astype(np.uint8)
    p_est = rng.random(16).astype(np.float32)
    key, cand = np.full(n, -5.0, np.float32), np.full(n, 77, np.uint8)
    oracle.prefetch_keys(ntok, off, layer, pos, window, state, pair, p_est, 0.98, key, cand)
    k2, c2 = keys_numpy(ntok, off, layer, pos, window, state, pair, p_est, 0.98, n)
    np.testing.assert_array_equal(cand, c2)
    np.testing.assert_allclose(key, k2, rtol=1e-6)
    # the list = k lowest (key, uid) among the candidates
    k = 25
    got = oracle.select_victims(key, cand, k=k)
    ids = np.flatnonzero(cand == (RES | SCORED))
    order = ids[np.lexsort((ids, key[ids]))][:k]
    np.testing.assert_array_equal(got, np.sort(order))


@pytest.mark.parametrize("npos,w,want", [
    (100, 0, [6]),                 # only the block that holds position 100
    (100, 4, [6]),                 # 96 .. 100 still inside block 6
    (100, 5, [5, 6]),              # position 95 is the last token of block 5
    (95, 0, [5]),
    (96, 16, [5, 6]),
    (100, 1000, [0, 1, 2, 3, 4, 5, 6]),
    (200, 30, []),                 # decode position beyond the stored blocks by more than the window
    (127, 20, [6, 7]),             # block 7 starts at 112 <= 127
])
def test_window_edges(oracle, npos, w, want):
    nb = 8
    ntok, off = np.array([nb * 16], np.int32), np.array([0], np.int64)
    state = np.full(nb, HOST, np.uint8)
    key, cand = np.zeros(nb, np.float32), np.zeros(nb, np.uint8)
    oracle.prefetch_keys(ntok, off, np.zeros(1, np.int32), np.array([npos], np.int32), np.array([w], np.int32),
                         state, np.zeros(nb, np.uint8), np.ones(16, np.float32), 1.0, key, cand)
    assert list(np.flatnonzero(cand)) == want
    assert np.all(key[cand != 0] == 0) and np.all(np.isposinf(key[cand == 0]))


def test_nearer_blocks_and_likelier_pairs_come_first(oracle):
    nb = 12
    ntok, off = np.array([nb * 16], np.int32), np.array([0], np.int64)
    state = np.full(nb, HOST | SCORED, np.uint8)
    key, cand = np.zeros(nb, np.float32), np.zeros(nb, np.uint8)
    p_est = np.full(16, 0.5, np.float32)
    oracle.prefetch_keys(ntok, off, np.zeros(1, np.int32), np.array([nb * 16 - 1], np.int32),
                         np.array([10000], np.int32), state, np.zeros(nb, np.uint8), p_est, 0.5, key, cand)
    np.testing.assert_array_equal(key, (1 - 0.5 * 0.5 ** np.arange(nb)[::-1]).astype(np.float32))
    np.testing.assert_array_equal(oracle.select_victims(key, cand, k=3), [9, 10, 11])
    # a likelier pair on a farther block overtakes a nearer block of an unlikely pair
    pair = np.zeros(nb, np.uint8); pair[5] = 1
    p_est[1] = 1.0; p_est[0] = 0.01
    oracle.prefetch_keys(ntok, off, np.zeros(1, np.int32), np.array([nb * 16 - 1], np.int32),
                         np.array([10000], np.int32), state, pair, p_est, 0.9, key, cand)
    assert oracle.select_victims(key, cand, k=1)[0] == 5


def test_distance_is_counted_from_the_block_of_the_decode_position(oracle):
    """Decode position inside block 6 of a 12-block row: block b <= 6 is 6 - b blocks away (not
    counted from the end of the stored row); blocks after the position are no candidates."""
    nb = 12
    ntok, off = np.array([nb * 16], np.int32), np.array([0], np.int64)
    state = np.full(nb, HOST, np.uint8)
    key, cand = np.zeros(nb, np.float32), np.zeros(nb, np.uint8)
    oracle.prefetch_keys(ntok, off, np.zeros(1, np.int32), np.array([100], np.int32), np.array([10000], np.int32),
                         state, np.zeros(nb, np.uint8), np.ones(16, np.float32), 0.5, key, cand)
    assert list(np.flatnonzero(cand)) == [0, 1, 2, 3, 4, 5, 6]
    np.testing.assert_array_equal(key[:7], (1 - 0.5 ** np.arange(7)[::-1]).astype(np.float32))
    assert np.all(np.isposinf(key[7:]))
