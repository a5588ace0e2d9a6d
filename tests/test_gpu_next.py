"""GPU parity for the refinements beyond the base pass: blended reuse estimate (section 3.3),
EMA with positional decay and transition multipliers (sections 3.4, 3.7), attention-span windows
and position-window prefetch lists (section 3.5).  Every call goes through the C ABI; expected
values come from the oracle only."""
import numpy as np
import pytest
import torch

from paper_2604_26968_amd import synth
from tests.harness import DeviceCase, host_pools, ref_row_weight

pytestmark = pytest.mark.gpu

RES, HOST, PROT, SCORED = 1, 2, 4, 8


def dev_of(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


# ------------------------------------------------------------------ blended estimate
@pytest.mark.parametrize("window,kappa", [(1, 3.0), (7, 0.0), (64, 16.0), (1000, 250.0), (65536, 1e6)])
def test_blend_counters_ring_and_estimates(oracle, window, kappa):
    """Counters, ring contents and ring heads bit-exact; estimates within 1e-6 relative (a handful
    of fp32 roundings against fp64).  Several calls so that the ring wraps and chunks of 1024 events
    are crossed; one call is longer than the ring for every pair, one holds malformed events."""
    from paper_2604_26968_amd import kvm
    hits, misses = np.zeros(16, np.uint32), np.zeros(16, np.uint32)
    win, head = np.full((16, window), 255, np.uint8), np.zeros(16, np.uint32)
    d_hits, d_misses = torch.zeros(16, dtype=torch.int32, device="cuda"), torch.zeros(16, dtype=torch.int32, device="cuda")
    d_win = torch.full((16, window), 255, dtype=torch.uint8, device="cuda")
    d_head = torch.zeros(16, dtype=torch.int32, device="cuda")
    d_out = [torch.zeros(16, dtype=torch.float32, device="cuda") for _ in range(3)]
    d_bad = torch.zeros(1, dtype=torch.int32, device="cuda")
    bad = np.zeros(1, np.uint32)
    w = synth.categorical_weights(9)
    for call, n in enumerate([0, 1, 63, 1024, 1025, 5000, 40000, 3]):
        ev_p, ev_o = synth.make_events(n, 70 + call, pair_weights=w, reuse_prob=np.linspace(0.05, 0.95, 16))
        if n >= 1024:
            ev_p, ev_o = ev_p.copy(), ev_o.copy()
            ev_p[5::97] = 16 + (np.arange(len(ev_p[5::97])) % 100)
            ev_o[11::131] = 2 + (np.arange(len(ev_o[11::131])) % 50)
        want = oracle.beta_blend_update(ev_p, ev_o, hits, misses, win, head, kappa, alpha0=1.0, beta0=1.0, n_bad=bad)
        kvm.kvm_beta_blend_update(dev_of(ev_p) if n else None, dev_of(ev_o) if n else None, d_hits, d_misses, d_win,
                                  d_head, kappa, *d_out, n_bad=d_bad)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(d_hits.cpu().numpy().view(np.uint32), hits)
        np.testing.assert_array_equal(d_misses.cpu().numpy().view(np.uint32), misses)
        np.testing.assert_array_equal(d_win.cpu().numpy(), win)
        np.testing.assert_array_equal(d_head.cpu().numpy().view(np.uint32), head)
        assert int(d_bad.item()) == int(bad[0])
        for got, ref in zip(d_out, want):
            np.testing.assert_allclose(got.cpu().numpy(), ref, rtol=1e-6, atol=1e-12)


def test_blend_single_pair_burst_longer_than_the_ring(oracle):
    """All events on one pair: only the last `window` survive, wherever the head stood."""
    from paper_2604_26968_amd import kvm
    window = 100
    rng = np.random.default_rng(1)
    hits, misses = np.zeros(16, np.uint32), np.zeros(16, np.uint32)
    win, head = np.full((16, window), 255, np.uint8), np.zeros(16, np.uint32)
    d_hits, d_misses = torch.zeros(16, dtype=torch.int32, device="cuda"), torch.zeros(16, dtype=torch.int32, device="cuda")
    d_win = torch.full((16, window), 255, dtype=torch.uint8, device="cuda")
    d_head = torch.zeros(16, dtype=torch.int32, device="cuda")
    d_out = [torch.zeros(16, dtype=torch.float32, device="cuda") for _ in range(3)]
    for n in (37, 4099, 100, 2048):
        ev_p = np.full(n, 13, np.uint8)
        ev_o = (rng.random(n) < 0.3).astype(np.uint8)
        want = oracle.beta_blend_update(ev_p, ev_o, hits, misses, win, head, 50.0)
        kvm.kvm_beta_blend_update(dev_of(ev_p), dev_of(ev_o), d_hits, d_misses, d_win, d_head, 50.0, *d_out)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(d_win.cpu().numpy(), win)
        np.testing.assert_array_equal(d_head.cpu().numpy().view(np.uint32), head)
        np.testing.assert_allclose(d_out[2].cpu().numpy(), want[2], rtol=1e-6)


# ------------------------------------------------------------------ EMA refinements
def ema_case():
    case = synth.make_case(synth.Shape(3, 8, 2, 64, synth.BF16, True, [100, 3300, 33, 700]), seed=16, uid_gap=2,
                           pair_weights=synth.categorical_weights(1))
    rng = np.random.default_rng(3)
    res = np.flatnonzero(case.state & RES)
    gone = rng.choice(res, size=len(res) // 5, replace=False)
    case.state[gone] = (case.state[gone] & ~np.uint8(RES)) | HOST
    return case


@pytest.mark.parametrize("pos_decay,with_mult", [(1.0, False), (0.97, False), (1.0, True), (0.999, True), (0.5, True)])
def test_ema_ex_multi_step(oracle, pos_decay, with_mult):
    """S within 2e-6 relative per step (the positional factor is one fp32 exp2 of an exactly reduced
    argument plus one product; the rest as in the plain update), abs floor for values that underflow;
    state bits exact."""
    from paper_2604_26968_amd import kvm
    pos_decay = float(np.float32(pos_decay))       # the value the C ABI's float argument carries
    case = ema_case()
    dev = DeviceCase(case)
    rng = np.random.default_rng(0)
    n_seq = len(case.shape.seq_lens)
    n_heads = case.shape.n_layers * case.shape.n_kv_heads
    row_head = synth.row_head_index(case)
    mult = (0.25 + 2 * rng.random((4, n_heads))).astype(np.float32) if with_mult else None
    S, prio = np.zeros(case.n_uids, np.float32), np.full(case.n_uids, -3.0, np.float32)
    dev.prio.fill_(-3.0)
    state = case.state.copy()
    d_seq, d_head = dev_of(case.row_seq), dev_of(row_head)
    d_mult = dev_of(mult) if with_mult else None
    for step in range(5):
        mass = rng.random(case.n_uids).astype(np.float32)
        p_hat = rng.random(16).astype(np.float32)
        trans = rng.choice(np.array([0, 1, 2, 3, 255, 4], np.uint8), n_seq).astype(np.uint8)
        active = (rng.random(case.n_rows) < 0.8).astype(np.uint8) if step else None
        dev.mass.copy_(torch.from_numpy(mass))
        dev.p_hat.copy_(torch.from_numpy(p_hat))
        ex = kvm.make_ema_ex(pos_decay, d_seq if with_mult else None, d_head if with_mult else None,
                             dev_of(trans) if with_mult else None, d_mult)
        kvm.kvm_ema_update_ex(dev.rows(active), dev.mass, 0.9, ex, dev.row_weight, dev.pair, dev.p_hat, dev.state,
                              dev.S, dev.prio)
        torch.cuda.synchronize()
        oracle.ema_update_ex(case.row_ntok, case.row_off, mass, 0.9, pos_decay, ref_row_weight(oracle, case), case.pair, p_hat,
                             state, S, prio, row_seq=case.row_seq if with_mult else None,
                             row_head=row_head if with_mult else None, seq_transition=trans if with_mult else None,
                             head_mult=mult, row_active=active)
        gS, gprio = dev.S.cpu().numpy(), dev.prio.cpu().numpy()
        np.testing.assert_array_equal(dev.state.cpu().numpy(), state)
        np.testing.assert_allclose(gS, S, rtol=2e-6, atol=1e-37)
        fin = np.isfinite(prio)
        np.testing.assert_array_equal(np.isposinf(gprio), np.isposinf(prio))
        np.testing.assert_allclose(gprio[fin], prio[fin], rtol=2e-6, atol=1e-37)
        dev.S.copy_(torch.from_numpy(S))        # identical inputs for the next step


def test_ema_ex_without_refinements_equals_plain_kernel_bit_for_bit():
    from paper_2604_26968_amd import kvm
    case = ema_case()
    rng = np.random.default_rng(5)
    mass = dev_of(rng.random(case.n_uids).astype(np.float32))
    S0 = rng.random(case.n_uids).astype(np.float32)
    out = []
    for ex in (False, True):
        dev = DeviceCase(case)
        dev.mass.copy_(mass)
        dev.S.copy_(torch.from_numpy(S0))
        dev.p_hat.copy_(torch.linspace(0.1, 0.9, 16))
        if ex:
            kvm.kvm_ema_update_ex(dev.rows(), dev.mass, 0.95, kvm.make_ema_ex(1.0), dev.row_weight, dev.pair,
                                  dev.p_hat, dev.state, dev.S, dev.prio)
        else:
            kvm.kvm_ema_update(dev.rows(), dev.mass, 0.95, dev.row_weight, dev.pair, dev.p_hat, dev.state, dev.S,
                               dev.prio)
        torch.cuda.synchronize()
        out.append((dev.S.cpu().numpy(), dev.prio.cpu().numpy(), dev.state.cpu().numpy()))
    for a, b in zip(*out):
        np.testing.assert_array_equal(a, b)


def test_ema_ex_long_row_positional_factor(oracle):
    """8,192-block rows: the factor spans 0.9995^8191 = 0.017 .. 1 and, for 0.9, underflows to 0."""
    from paper_2604_26968_amd import kvm
    case = synth.make_case(synth.Shape(1, 8, 1, 64, synth.BF16, True, [131072]), seed=2)
    for pos_decay in (float(np.float32(0.9995)), float(np.float32(0.9))):
        dev = DeviceCase(case)
        dev.mass.fill_(1.0)
        dev.p_hat.fill_(1.0)
        kvm.kvm_ema_update_ex(dev.rows(), dev.mass, 0.9, kvm.make_ema_ex(pos_decay), dev.row_weight, dev.pair,
                              dev.p_hat, dev.state, dev.S, dev.prio)
        torch.cuda.synchronize()
        S, prio, state = (np.zeros(case.n_uids, np.float32), np.zeros(case.n_uids, np.float32), case.state.copy())
        oracle.ema_update_ex(case.row_ntok, case.row_off, np.ones(case.n_uids, np.float32), 0.9, pos_decay,
                             ref_row_weight(oracle, case), case.pair, np.ones(16, np.float32), state, S, prio)
        np.testing.assert_allclose(dev.S.cpu().numpy(), S, rtol=1e-6, atol=1e-37)


# ------------------------------------------------------------------ prefetching
def prefetch_case(seed=4):
    case = synth.make_case(synth.Shape(4, 8, 2, 64, synth.BF16, True, [100, 2500, 33, 900, 16]), seed=seed, uid_gap=1,
                           pair_weights=synth.categorical_weights(2))
    rng = np.random.default_rng(seed)
    res = np.flatnonzero(case.state & RES)
    gone = rng.choice(res, size=len(res) // 2, replace=False)
    case.state[gone] = (case.state[gone] & ~np.uint8(RES)) | HOST
    return case


def span_ws(n_rows):
    """Scratch for kvm_span_update, handed over with garbage in it."""
    from paper_2604_26968_amd import kvm
    return torch.full((max(kvm.kvm_workspace_bytes(kvm.OP_SPAN, 0, n_rows), 4),), 0x7F, dtype=torch.uint8, device="cuda")


@pytest.mark.parametrize("theta", [(9, 10), (1, 2), (1, 1), (0, 1), (65535, 65536)])
def test_span_update_exact(oracle, theta):
    """Integer results: span sums, counts and windows are bit-exact."""
    from paper_2604_26968_amd import kvm
    case = prefetch_case()
    dev = DeviceCase(case)
    L = case.shape.n_layers
    rng = np.random.default_rng(8)
    row_layer = synth.row_layer_index(case)
    s_sum, s_cnt, win = np.zeros(L + 1, np.uint64), np.zeros(L + 1, np.uint32), np.full(L + 1, -7, np.int32)
    d_sum = torch.zeros(L + 1, dtype=torch.int64, device="cuda")
    d_cnt = torch.zeros(L + 1, dtype=torch.int32, device="cuda")
    d_win = torch.full((L + 1,), -7, dtype=torch.int32, device="cuda")
    d_layer = dev_of(row_layer)
    for step in range(3):
        # masses concentrated near the end, more sharply in the early layers; a few odd values
        mass = np.zeros(case.n_uids, np.float32)
        for r in range(case.n_rows):
            nb = (case.row_ntok[r] + 15) // 16
            sharp = 0.5 + 0.1 * row_layer[r] + 0.3 * rng.random()
            m = (sharp ** np.arange(nb)[::-1]) * rng.random(nb)
            mass[case.row_off[r]:case.row_off[r] + nb] = m / max(m.sum(), 1e-30)
        mass[rng.random(case.n_uids) < 0.01] = np.nan
        mass[rng.random(case.n_uids) < 0.01] = -0.5
        mass[rng.random(case.n_uids) < 0.005] = 3.0
        active = (rng.random(case.n_rows) < 0.8).astype(np.uint8) if step else None
        oracle.span_update(case.row_ntok, case.row_off, row_layer, mass, case.state, theta[0], theta[1], s_sum, s_cnt,
                           32, 2000, win, row_active=active)
        dev.mass.copy_(torch.from_numpy(mass))
        kvm.kvm_span_update(dev.rows(active), d_layer, dev.mass, dev.state, theta[0], theta[1], d_sum, d_cnt, 32, 2000,
                            d_win, span_ws(case.n_rows))
        torch.cuda.synchronize()
        np.testing.assert_array_equal(d_sum.cpu().numpy().view(np.uint64), s_sum)
        np.testing.assert_array_equal(d_cnt.cpu().numpy().view(np.uint32), s_cnt)
        np.testing.assert_array_equal(d_win.cpu().numpy(), win)
    assert win[L] == -7 and s_cnt[:L].min() > 0


def test_span_long_rows(oracle):
    """8,192-block rows cross many 64-block chunks; uniform masses give ceil(theta nb) exactly."""
    from paper_2604_26968_amd import kvm
    case = synth.make_case(synth.Shape(2, 8, 1, 64, synth.BF16, True, [131072, 70000]), seed=2)
    dev = DeviceCase(case)
    row_layer = synth.row_layer_index(case)
    rng = np.random.default_rng(1)
    for kind in ("uniform", "random"):
        mass = np.full(case.n_uids, 2.0 ** -13, np.float32) if kind == "uniform" else \
            (rng.random(case.n_uids) ** 8).astype(np.float32)
        s_sum, s_cnt, win = np.zeros(2, np.uint64), np.zeros(2, np.uint32), np.zeros(2, np.int32)
        oracle.span_update(case.row_ntok, case.row_off, row_layer, mass, case.state, 9, 10, s_sum, s_cnt, 0, 1 << 30, win)
        d_sum = torch.zeros(2, dtype=torch.int64, device="cuda")
        d_cnt = torch.zeros(2, dtype=torch.int32, device="cuda")
        d_win = torch.zeros(2, dtype=torch.int32, device="cuda")
        dev.mass.copy_(torch.from_numpy(mass))
        kvm.kvm_span_update(dev.rows(), dev_of(row_layer), dev.mass, dev.state, 9, 10, d_sum, d_cnt, 0, 1 << 30, d_win,
                            span_ws(case.n_rows))
        torch.cuda.synchronize()
        np.testing.assert_array_equal(d_sum.cpu().numpy().view(np.uint64), s_sum)
        np.testing.assert_array_equal(d_win.cpu().numpy(), win)
        if kind == "uniform":
            assert s_sum[0] == -(-9 * 8192 // 10) + -(-9 * 4375 // 10)


@pytest.mark.parametrize("n_layers", [7, 2048, 2500])
def test_span_many_rows_and_layers(oracle, n_layers):
    """10,000 short rows (several workgroups of the per-layer fold, a ragged last one) dealt over few,
    many and more layers than the fold has cells; rows given in an order unrelated to their layers;
    some rows with a layer out of range.  Accumulators start non-zero."""
    from paper_2604_26968_amd import kvm
    rng = np.random.default_rng(n_layers)
    n_rows = 10000
    row_ntok = rng.integers(0, 400, n_rows).astype(np.int32)
    nb = (row_ntok.astype(np.int64) + 15) // 16
    row_off = np.zeros(n_rows, np.int64)
    row_off[1:] = np.cumsum(nb[:-1])
    n = int(nb.sum())
    row_layer = rng.integers(0, n_layers, n_rows).astype(np.int32)
    row_layer[rng.random(n_rows) < 0.01] = n_layers
    row_layer[rng.random(n_rows) < 0.01] = -1
    mass = (rng.random(n) ** 6).astype(np.float32)
    state = np.where(rng.random(n) < 0.7, 9, 2).astype(np.uint8)
    s_sum = rng.integers(0, 1000, n_layers).astype(np.uint64)
    s_cnt = rng.integers(1, 5, n_layers).astype(np.uint32)
    win = np.full(n_layers, -3, np.int32)
    d_sum, d_cnt, d_win = dev_of(s_sum.view(np.int64)), dev_of(s_cnt.view(np.int32)), dev_of(win)
    # the library skips rows whose layer is out of range; the oracle refuses them, so it gets them as inactive rows
    in_range = (row_layer >= 0) & (row_layer < n_layers)
    oracle.span_update(row_ntok, row_off, np.where(in_range, row_layer, 0).astype(np.int32), mass, state, 4, 5, s_sum,
                       s_cnt, 16, 4096, win, row_active=in_range.astype(np.uint8))
    rows = kvm.make_rows(dev_of(row_ntok), dev_of(row_off), torch.zeros(n_rows, dtype=torch.int64, device="cuda"),
                         torch.zeros(n, dtype=torch.int32, device="cuda"), 1, n_rows)
    kvm.kvm_span_update(rows, dev_of(row_layer), dev_of(mass), dev_of(state), 4, 5, d_sum, d_cnt, 16, 4096, d_win,
                        span_ws(n_rows))
    torch.cuda.synchronize()
    np.testing.assert_array_equal(d_sum.cpu().numpy().view(np.uint64), s_sum)
    np.testing.assert_array_equal(d_cnt.cpu().numpy().view(np.uint32), s_cnt)
    np.testing.assert_array_equal(d_win.cpu().numpy(), win)


def test_span_workspace_too_small():
    from paper_2604_26968_amd import kvm
    case = synth.tiny_gqa()
    dev = DeviceCase(case)
    L = case.shape.n_layers
    z64, z32 = torch.zeros(L, dtype=torch.int64, device="cuda"), torch.zeros(L, dtype=torch.int32, device="cuda")
    with pytest.raises(kvm.KvmError) as e:
        kvm.kvm_span_update(dev.rows(), dev_of(synth.row_layer_index(case)), dev.mass, dev.state, 9, 10, z64, z32, 0, 100,
                            z32.clone(), torch.zeros(4 * case.n_rows - 4, dtype=torch.uint8, device="cuda"))
    assert e.value.code == kvm.ENOSPC


@pytest.mark.parametrize("pos_decay", [1.0, 0.98, 0.5])
def test_prefetch_keys_and_list(oracle, pos_decay):
    """Candidate flags exact; keys within 2e-7 absolute (keys are 1 - y with y in [0, 1] known to
    ~1e-7 relative); the list built by the selector from the library's own keys equals the oracle's
    selection on those same keys, and differs from the oracle's end-to-end list only at the cutoff."""
    from paper_2604_26968_amd import kvm
    pos_decay = float(np.float32(pos_decay))
    case = prefetch_case(seed=9)
    dev = DeviceCase(case)
    rng = np.random.default_rng(2)
    L = case.shape.n_layers
    row_layer = synth.row_layer_index(case)
    row_pos = np.where(rng.random(case.n_rows) < 0.1, -1, case.row_ntok - rng.integers(0, 20, case.n_rows)).astype(np.int32)
    window = np.array([0, 48, 400, 100000], np.int32)[:L]
    p_est = rng.random(16).astype(np.float32)
    key, cand = np.full(case.n_uids, -2.0, np.float32), np.full(case.n_uids, 99, np.uint8)
    oracle.prefetch_keys(case.row_ntok, case.row_off, row_layer, row_pos, window, case.state, case.pair, p_est,
                         pos_decay, key, cand)
    d_key = torch.full((case.n_uids,), -2.0, dtype=torch.float32, device="cuda")
    d_cand = torch.full((case.n_uids,), 99, dtype=torch.uint8, device="cuda")
    kvm.kvm_prefetch_keys(dev.rows(), dev_of(row_layer), dev_of(row_pos), dev_of(window), dev.state, dev.pair,
                          dev_of(p_est), pos_decay, d_key, d_cand)
    torch.cuda.synchronize()
    gkey, gcand = d_key.cpu().numpy(), d_cand.cpu().numpy()
    np.testing.assert_array_equal(gcand, cand)
    isc = cand == (RES | SCORED)
    assert isc.sum() > 100
    np.testing.assert_array_equal(np.isposinf(gkey), np.isposinf(key))
    np.testing.assert_allclose(gkey[isc], key[isc], rtol=0, atol=2e-7)
    assert np.all(gkey[~isc & (cand == 99)] == -2.0)          # gaps between rows are not written
    k = int(isc.sum()) // 3
    kvm.kvm_select_victims(d_key, d_cand, dev.victims, dev.n_victims, dev.ws, k=k)
    torch.cuda.synchronize()
    got = dev.victims[: int(dev.n_victims.item())].cpu().numpy()
    np.testing.assert_array_equal(got, oracle.select_victims(gkey, gcand, k=k))       # identical keys: exact
    want = oracle.select_victims(key, cand, k=k)
    assert len(got) == len(want) == k
    diff = np.setxor1d(got, want)
    cutoff = np.max(key[want])
    assert np.all(np.abs(key[diff] - cutoff) <= 4e-7)


def test_prefetch_list_feeds_unpack(oracle):
    """The whole chain on the device: keys -> select -> unpack with the device-side count; the pool,
    table and state afterwards equal the oracle's chain."""
    from paper_2604_26968_amd import kvm

    case = synth.make_case(synth.Shape(2, 4, 2, 64, synth.BF16, True, [600, 200]), seed=12, spare_slots=0)
    dev = DeviceCase(case)
    k8, v8 = host_pools(case)
    rng = np.random.default_rng(3)
    sh = case.shape
    rec = sh.unit_k_bytes + sh.unit_v_bytes
    # evict a third of the units to the host through the library's own pack (oracle mirrors it)
    res = np.flatnonzero((case.state & RES) & ~((case.state & PROT) >> 2))
    out = np.sort(rng.choice(res, size=len(res) // 3, replace=False)).astype(np.int64)
    hs = np.arange(len(out), dtype=np.int32)
    tbl, st = case.slot_tbl.copy(), case.state.copy()
    staging, freed = oracle.pack(k8, v8, sh.unit_k_bytes, sh.unit_v_bytes, tbl, st, out, hs)
    g_staging, g_freed = dev.pack(out, hs)
    np.testing.assert_array_equal(g_staging, staging)
    # prefetch list: the blocks near the decode positions
    row_layer = synth.row_layer_index(case)
    row_pos = case.row_ntok.copy()
    window = np.array([64, 256], np.int32)
    p_est = np.linspace(0.2, 0.9, 16).astype(np.float32)
    key, cand = np.zeros(case.n_uids, np.float32), np.zeros(case.n_uids, np.uint8)
    oracle.prefetch_keys(case.row_ntok, case.row_off, row_layer, row_pos, window, st, case.pair, p_est, 1.0, key, cand)
    k = 10
    want = oracle.select_victims(key, cand, k=k)
    assert len(want) == k
    d_key = torch.zeros(case.n_uids, dtype=torch.float32, device="cuda")
    d_cand = torch.zeros(case.n_uids, dtype=torch.uint8, device="cuda")
    kvm.kvm_prefetch_keys(dev.rows(), dev_of(row_layer), dev_of(row_pos), dev_of(window), dev.state, dev.pair,
                          dev_of(p_est), 1.0, d_key, d_cand)
    kvm.kvm_select_victims(d_key, d_cand, dev.victims, dev.n_victims, dev.ws, k=k)
    torch.cuda.synchronize()
    got = dev.victims[:k].cpu().numpy()
    np.testing.assert_array_equal(got, want)         # pos_decay 1: keys are 1 - p_est exactly on both sides
    # records of the chosen units, in list order, as they sit on the host; frames = the first k freed
    host_slot = -1 - tbl[want]
    recs = np.ascontiguousarray(staging.reshape(-1, rec)[host_slot])
    dst = freed[:k].astype(np.int32)
    oracle.unpack(k8, v8, sh.unit_k_bytes, sh.unit_v_bytes, tbl, st, want, dst, recs)
    h_in = torch.from_numpy(recs.reshape(-1)).pin_memory()
    kvm.kvm_unpack(dev.pool, dev.slot_tbl, dev.state, dev.victims, k, dev_of(dst), None, h_in, n_dev=dev.n_victims,
                   n_bad=dev.n_bad)
    torch.cuda.synchronize()
    gk, gv = dev.pools_host()
    np.testing.assert_array_equal(gk, k8)
    np.testing.assert_array_equal(gv, v8)
    np.testing.assert_array_equal(dev.slot_tbl.cpu().numpy(), tbl)
    np.testing.assert_array_equal(dev.state.cpu().numpy(), st)
    assert int(dev.n_bad.item()) == 0


# ------------------------------------------------------------------ in-place exchange
@pytest.mark.parametrize("shape", [
    synth.Shape(2, 8, 2, 128, synth.BF16, True, [300, 77]),
    synth.Shape(4, 16, 1, 576, synth.BF16, False, [400]),
])
def test_exchange_in_place_with_slot_addressed_tier(oracle, shape):
    """Pools, tier, tables and state after the call equal the oracle's, byte for byte, including
    skipped pairs and lists cut short by the device-side counts."""
    from paper_2604_26968_amd import kvm
    case = synth.make_case(shape, seed=31)
    k8, v8 = host_pools(case)
    rng = np.random.default_rng(8)
    uk, uv = shape.unit_k_bytes, shape.unit_v_bytes
    rec = uk + uv
    res = np.flatnonzero(case.state & RES)
    first_out = np.sort(rng.choice(res, size=len(res) // 3, replace=False)).astype(np.int64)
    n_tier = len(first_out) + 7
    hs = rng.permutation(n_tier)[:len(first_out)].astype(np.int32)
    tbl, st = case.slot_tbl.copy(), case.state.copy()
    staging, _ = oracle.pack(k8, v8, uk, uv, tbl, st, first_out, hs)
    tier = rng.integers(0, 256, size=(n_tier, rec), dtype=np.uint8)
    tier[hs] = staging
    # device side starts from the same situation
    case.slot_tbl[:], case.state[:] = tbl, st
    dev = DeviceCase(case)
    d_tier = torch.from_numpy(tier.reshape(-1).copy()).pin_memory()
    n = 24
    res_now = np.flatnonzero(st & RES)
    outs = rng.choice(res_now, size=n, replace=False).astype(np.int64)
    ins = rng.choice(first_out, size=n, replace=False).astype(np.int64)
    outs[3] = -1
    ins[9] = np.setdiff1d(res_now, outs)[0]                              # already resident
    outs[12] = np.setdiff1d(first_out, ins)[0]                          # not resident (and in neither list otherwise)
    bad = np.zeros(1, np.uint32)
    for n_out_dev, n_in_dev in ((None, None), (15, 22)):
        lim = n if n_out_dev is None else min(n_out_dev, n_in_dev)
        oracle.exchange(k8, v8, uk, uv, tbl, st, outs[:lim], ins[:lim], tier, n_bad=bad)
        kvm.kvm_exchange(dev.pool, dev.slot_tbl, dev.state, dev_of(outs), dev_of(ins), n, d_tier,
                         n_out_dev=None if n_out_dev is None else torch.tensor([n_out_dev], device="cuda"),
                         n_in_dev=None if n_in_dev is None else torch.tensor([n_in_dev], device="cuda"),
                         n_bad=dev.n_bad)
        torch.cuda.synchronize()
        gk, gv = dev.pools_host()
        np.testing.assert_array_equal(gk, k8)
        if v8 is not None:
            np.testing.assert_array_equal(gv, v8)
        np.testing.assert_array_equal(d_tier.numpy().reshape(n_tier, rec), tier)
        np.testing.assert_array_equal(dev.slot_tbl.cpu().numpy(), tbl)
        np.testing.assert_array_equal(dev.state.cpu().numpy(), st)
        assert int(dev.n_bad.item()) == int(bad[0])
        # second round: the same lists reversed bring everything back except the skipped pairs
        outs, ins = ins.copy(), outs.copy()
    assert bad[0] >= 3


# ------------------------------------------------------------------ content addressing
def duplicate_some_frames(case, rng, n_groups, group_size):
    """Copy the K and V frames of a few units over others: groups of identical content."""
    res = np.flatnonzero(case.state & RES)
    pick = rng.choice(res, size=n_groups * group_size, replace=False).reshape(n_groups, group_size)
    for grp in pick:
        src = case.slot_tbl[grp[0]]
        for u in grp[1:]:
            case.k_pool[case.slot_tbl[u]] = case.k_pool[src]
            if case.v_pool is not None:
                case.v_pool[case.slot_tbl[u]] = case.v_pool[src]
    return pick


@pytest.mark.parametrize("shape", [
    synth.Shape(2, 8, 2, 128, synth.BF16, True, [300, 77]),
    synth.Shape(1, 4, 2, 64, synth.FP16, True, [512]),
    synth.Shape(3, 16, 1, 576, synth.BF16, False, [400]),
])
def test_unit_digests_bit_exact(oracle, shape):
    """Digests are bytes: exact.  Units that are not in HBM and malformed uids give zero digests."""
    from paper_2604_26968_amd import kvm
    case = synth.make_case(shape, seed=41)
    rng = np.random.default_rng(4)
    duplicate_some_frames(case, rng, 3, 4)
    res = np.flatnonzero(case.state & RES)
    gone = rng.choice(res, size=5, replace=False)
    case.state[gone] = (case.state[gone] & ~np.uint8(RES)) | HOST
    dev = DeviceCase(case)
    k8, v8 = host_pools(case)
    uids = np.r_[np.arange(case.n_uids), [-1, case.n_uids, 2 ** 40]].astype(np.int64)
    rng.shuffle(uids)
    bad = np.zeros(1, np.uint32)
    want = oracle.hash_units(k8, v8, shape.unit_k_bytes, shape.unit_v_bytes, case.slot_tbl, case.state, uids, n_bad=bad)
    d = torch.full((len(uids), 32), 7, dtype=torch.uint8, device="cuda")
    kvm.kvm_hash_units(dev.pool, dev.slot_tbl, dev.state, dev_of(uids), len(uids), d, n_bad=dev.n_bad)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(d.cpu().numpy(), want)
    assert int(dev.n_bad.item()) == int(bad[0]) > 5


def test_dedup_store_matches_the_sequential_definition(oracle):
    """Several calls with repeated digests inside a call and across calls, releases in between;
    canonical uids and the store's contents (digest -> canonical uid, count) are exact."""
    from paper_2604_26968_amd import kvm
    rng = np.random.default_rng(5)
    catalogue = rng.integers(0, 256, size=(300, 32), dtype=np.uint8)
    catalogue[0, :8] = 0                          # a digest whose first 8 bytes are zero is still a valid key
    ref = oracle.DedupStore(1024)
    store = kvm.make_store(1024)
    n_full = torch.zeros(1, dtype=torch.int32, device="cuda")
    n_col = torch.zeros(1, dtype=torch.int32, device="cuda")
    d_bad = torch.zeros(1, dtype=torch.int32, device="cuda")
    bad = np.zeros(1, np.uint32)
    next_uid = 1000

    def store_dict():
        t = {k: v.cpu().numpy() for k, v in store.tensors.items()}
        out = {}
        for e in np.flatnonzero(t["canon"] >= 0):
            out[t["digest"][e].tobytes()] = (int(t["canon"][e]), int(t["refs"][e]))
        assert np.all(t["pending"] == -1)
        return out

    for call, n in enumerate([1, 50, 700, 3, 2000]):
        zipf = np.minimum(rng.zipf(1.3, n) - 1, 299)
        digests = catalogue[zipf].copy()
        if n >= 50:
            digests[7] = 0                         # a failed hash: skipped
        uids = (next_uid + rng.permutation(n)).astype(np.int64)
        next_uid += n
        keep = digests.any(axis=1)
        want = uids.copy()
        want[keep] = ref.insert(digests[keep], uids[keep])
        canon = torch.zeros(n, dtype=torch.int64, device="cuda")
        ws = torch.full((n,), 0x7F7F7F7F7F7F7F7F, dtype=torch.int64, device="cuda")
        kvm.kvm_dedup_insert(store, dev_of(digests), dev_of(uids), n, canon, ws, n_full=n_full, n_collide=n_col)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(canon.cpu().numpy(), want)
        assert int(n_full.item()) == 0 and int(n_col.item()) == 0
        assert store_dict() == ref.as_dict()
        rel = catalogue[rng.integers(0, 300, 40)]
        ref.release(rel, n_bad=bad)
        kvm.kvm_dedup_release(store, dev_of(rel), len(rel), n_bad=d_bad)
        torch.cuda.synchronize()
        assert int(d_bad.item()) == int(bad[0])
        assert store_dict() == ref.as_dict()


def test_hash_then_dedup_finds_the_planted_duplicates(oracle):
    from paper_2604_26968_amd import kvm
    case = synth.make_case(synth.Shape(2, 8, 2, 128, synth.BF16, True, [1000, 400]), seed=43)
    rng = np.random.default_rng(6)
    groups = duplicate_some_frames(case, rng, 20, 5)
    dev = DeviceCase(case)
    uids = np.flatnonzero(case.state & RES).astype(np.int64)
    n = len(uids)
    d = torch.zeros((n, 32), dtype=torch.uint8, device="cuda")
    kvm.kvm_hash_units(dev.pool, dev.slot_tbl, dev.state, dev_of(uids), n, d)
    store = kvm.make_store(1 << 12)
    canon = torch.zeros(n, dtype=torch.int64, device="cuda")
    ws = torch.full((n,), 0x7F7F7F7F7F7F7F7F, dtype=torch.int64, device="cuda")
    kvm.kvm_dedup_insert(store, d, dev_of(uids), n, canon, ws)
    torch.cuda.synchronize()
    canon = canon.cpu().numpy()
    k8, v8 = host_pools(case)
    ref = oracle.DedupStore(n)
    want = ref.insert(oracle.hash_units(k8, v8, case.shape.unit_k_bytes, case.shape.unit_v_bytes, case.slot_tbl,
                                        case.state, uids), uids)
    np.testing.assert_array_equal(canon, want)
    dup = uids[canon != uids]
    assert len(dup) == 20 * 4
    for grp in groups:
        assert len(set(canon[np.searchsorted(uids, grp)])) == 1 and canon[np.searchsorted(uids, grp)][0] == grp.min()


@pytest.mark.parametrize("shape", [
    synth.Shape(2, 8, 2, 128, synth.BF16, True, [1000, 400]),
    synth.Shape(2, 128, 1, 576, synth.BF16, False, [700]),          # latent units, no V
])
def test_duplicates_share_frames_and_get_their_own_back(oracle, shape):
    """hash -> insert -> kvm_dedup_share: the duplicates read their canonical unit's frame, their own frames
    come back free, tables / state / reader counts equal the oracle's; scoring gives the same masses as before
    (same bytes); the selection never names a unit that shares a frame and pack refuses one; kvm_dedup_unshare
    gives every such unit a frame of its own with the same bytes, tables equal the oracle's."""
    from paper_2604_26968_amd import kvm
    from tests.harness import oracle_score
    SHARED = kvm.ST_SHARED
    case = synth.make_case(shape, seed=45, spare_slots=20)
    rng = np.random.default_rng(8)
    groups = duplicate_some_frames(case, rng, 12, 4)
    # (the canonical copy of a group is its first unit in list order, i.e. its smallest uid)
    case.state[np.sort(groups[0])[1]] |= PROT            # a duplicate whose block is still being written
    case.state[np.sort(groups[1])[0]] |= PROT            # a canonical copy that is
    dev = DeviceCase(case)
    k8, v8 = host_pools(case)
    uk, uv = shape.unit_k_bytes, shape.unit_v_bytes
    n_slots = case.n_slots
    uids = np.flatnonzero(case.state & RES).astype(np.int64)
    n = len(uids)
    q = synth.make_queries(case, 3)
    scale = 1.0 / np.sqrt(shape.dim)
    dev.mass.fill_(-1.0)
    kvm.kvm_score_step(dev.pool, dev.rows(), dev_of(q.view(np.int16)), scale, dev.mass, dev.ws)
    torch.cuda.synchronize()
    mass_before = dev.mass.cpu().numpy()
    # digests and canonical uids on both sides
    d = torch.zeros((n, 32), dtype=torch.uint8, device="cuda")
    kvm.kvm_hash_units(dev.pool, dev.slot_tbl, dev.state, dev_of(uids), n, d)
    store = kvm.make_store(1 << 12)
    canon = torch.zeros(n, dtype=torch.int64, device="cuda")
    ws = torch.full((n,), 0x7F7F7F7F7F7F7F7F, dtype=torch.int64, device="cuda")
    kvm.kvm_dedup_insert(store, d, dev_of(uids), n, canon, ws)
    ref_store = oracle.DedupStore(n)
    tbl, st = case.slot_tbl.copy(), case.state.copy()
    want_canon = ref_store.insert(oracle.hash_units(k8, v8, uk, uv, tbl, st, uids), uids)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(canon.cpu().numpy(), want_canon)
    # share: the whole list plus two malformed entries
    lst = np.r_[uids, [-2, case.n_uids + 3]].astype(np.int64)
    cn = np.r_[want_canon, [0, 1]].astype(np.int64)
    refs = torch.zeros(n_slots, dtype=torch.int32, device="cuda")
    freed = torch.full((len(lst),), -7, dtype=torch.int32, device="cuda")
    kvm.kvm_dedup_share(dev.slot_tbl, dev.state, n_slots, dev_of(lst), dev_of(cn), len(lst), refs, freed,
                        n_bad=dev.n_bad)
    o_refs = np.zeros(n_slots, np.uint32)
    bad = np.zeros(1, np.uint32)
    o_freed = oracle.dedup_share(tbl, st, n_slots, lst, cn, o_refs, n_bad=bad)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(freed.cpu().numpy(), o_freed)
    np.testing.assert_array_equal(dev.slot_tbl.cpu().numpy(), tbl)
    np.testing.assert_array_equal(dev.state.cpu().numpy(), st)
    np.testing.assert_array_equal(refs.cpu().numpy().view(np.uint32), o_refs)
    assert int(dev.n_bad.item()) == int(bad[0]) == 2
    n_shared = int((o_freed >= 0).sum())
    is_dup = want_canon != uids
    want_shared = is_dup & ((case.state[uids] & PROT) == 0) & ((case.state[want_canon] & PROT) == 0)
    assert n_shared == int(want_shared.sum()) and 20 <= n_shared < int(is_dup.sum()) == 12 * 3
    assert int(o_refs.sum()) == n_shared + len(np.unique(want_canon[want_shared]))
    # same bytes behind every unit: same masses, bit for bit
    dev.mass.fill_(-1.0)
    kvm.kvm_score_step(dev.pool, dev.rows(), dev_of(q.view(np.int16)), scale, dev.mass, dev.ws)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(dev.mass.cpu().numpy(), mass_before)
    want_mass = oracle_score(oracle, case, q, scale, fill=-1.0, slot_tbl=tbl)
    w = want_mass != -1.0
    np.testing.assert_allclose(mass_before[w], want_mass[w], rtol=1e-3, atol=1e-9)
    # units that share a frame are never victims, whatever their priority, and pack refuses them
    shared = np.flatnonzero(st & SHARED)
    assert len(shared) == n_shared + len(np.unique(want_canon[want_shared]))
    st_sel = st.copy()
    st_sel[(st_sel & RES) != 0] |= SCORED
    prio = rng.random(case.n_uids).astype(np.float32) + 1.0
    prio[shared] = 0.0
    from tests.test_gpu_parity import select_both
    dcase = DeviceCase(synth.tiny_gqa(1))
    got = select_both(oracle, dcase, prio, st_sel, k=len(uids))
    assert not np.intersect1d(got, shared).size and len(got) == int(((st_sel & (RES | PROT | SCORED | SHARED)) == (RES | SCORED)).sum())
    some = np.r_[shared[:5], got[:5]].astype(np.int64)
    hs = np.arange(len(some), dtype=np.int32)
    want_staging, want_freed = oracle.pack(k8, v8, uk, uv, tbl, st, some, hs, n_bad=bad)
    got_staging, got_freed = dev.pack(some, hs, direct=True)
    np.testing.assert_array_equal(got_freed, want_freed)
    np.testing.assert_array_equal(got_freed[:5], -1)
    np.testing.assert_array_equal(got_staging[5:], want_staging[5:])
    np.testing.assert_array_equal(dev.slot_tbl.cpu().numpy(), tbl)
    np.testing.assert_array_equal(dev.state.cpu().numpy(), st)
    # ---- every sharing unit gets a frame of its own again (the frames given up, then the spare ones) ---------
    free = np.r_[o_freed[o_freed >= 0], want_freed[want_freed >= 0], np.setdiff1d(np.arange(n_slots), case.slot_tbl[case.slot_tbl >= 0])]
    order = rng.permutation(len(shared))
    ul = np.r_[shared[order], got[5:7], [case.n_uids + 9]].astype(np.int64)       # two units that share nothing, one bad
    assert len(free) >= len(ul)
    nf = free[:len(ul)].astype(np.int32)
    back = torch.full((len(ul),), -7, dtype=torch.int32, device="cuda")
    dev.n_bad.zero_()
    kvm.kvm_dedup_unshare(dev.pool, dev.slot_tbl, dev.state, dev_of(ul), dev_of(nf), len(ul), refs, back,
                          n_bad=dev.n_bad)
    bad[:] = 0
    o_back = oracle.dedup_unshare(k8, v8, uk, uv, tbl, st, ul, nf, o_refs, n_bad=bad)
    torch.cuda.synchronize()
    g_back = back.cpu().numpy()
    # which item of the last readers of a frame reports it free is not defined: compare per frame
    np.testing.assert_array_equal(np.sort(g_back), np.sort(o_back))
    moved = np.arange(len(shared))
    assert np.all((g_back[moved] == -1) | (g_back[moved] >= 0)) and np.array_equal(g_back[len(shared):], o_back[len(shared):])
    np.testing.assert_array_equal(dev.slot_tbl.cpu().numpy(), tbl)
    np.testing.assert_array_equal(dev.state.cpu().numpy(), st)
    assert not refs.any().item() and not o_refs.any() and not (st & SHARED).any()
    assert int(dev.n_bad.item()) == int(bad[0]) == 1
    gk, gv = dev.pools_host()
    res = np.flatnonzero(st & RES)
    np.testing.assert_array_equal(gk[tbl[res]], k8[tbl[res]])
    if v8 is not None:
        np.testing.assert_array_equal(gv[tbl[res]], v8[tbl[res]])
    assert len(np.unique(tbl[res])) == len(res)
    dev.mass.fill_(-1.0)
    kvm.kvm_score_step(dev.pool, dev.rows(), dev_of(q.view(np.int16)), scale, dev.mass, dev.ws)
    torch.cuda.synchronize()
    m_after = dev.mass.cpu().numpy()
    # rows that lost a unit to the pack above are renormalised; every other unit reads the same bytes as at the start
    case.k_pool[:] = k8.view(np.uint16).reshape(case.k_pool.shape)         # the pool as the oracle's unshare left it
    want_after = oracle_score(oracle, case, q, scale, fill=-1.0, slot_tbl=tbl)
    w = want_after != -1.0
    np.testing.assert_array_equal(m_after != -1.0, w)
    np.testing.assert_allclose(m_after[w], want_after[w], rtol=1e-3, atol=1e-9)


def test_dedup_table_too_small_reports_it():
    from paper_2604_26968_amd import kvm
    rng = np.random.default_rng(7)
    digests = rng.integers(1, 256, size=(100, 32), dtype=np.uint8)
    store = kvm.make_store(16)
    n_full = torch.zeros(1, dtype=torch.int32, device="cuda")
    canon = torch.zeros(100, dtype=torch.int64, device="cuda")
    ws = torch.full((100,), 0x7F7F7F7F7F7F7F7F, dtype=torch.int64, device="cuda")
    uids = np.arange(100, dtype=np.int64)
    kvm.kvm_dedup_insert(store, dev_of(digests), dev_of(uids), 100, canon, ws, n_full=n_full)
    torch.cuda.synchronize()
    assert int(n_full.item()) == 100 - 16
    np.testing.assert_array_equal(canon.cpu().numpy(), uids)       # all distinct: every item is its own canonical copy
    assert int((store.tensors["canon"] >= 0).sum().item()) == 16


# ------------------------------------------------------------------ exchange overlapped with scoring
@pytest.mark.parametrize("shape,n_pairs", [
    (synth.Shape(2, 8, 2, 128, synth.BF16, True, [700, 77, 1300]), 60),       # dot2 kernel, g = 4
    (synth.Shape(2, 32, 1, 128, synth.FP16, True, [900]), 20),                # matrix-core kernel, g = 32
    (synth.Shape(3, 128, 1, 576, synth.BF16, False, [9000, 300]), 30),        # wide kernel, rows of several tiles
])
def test_exchange_in_three_parts_rides_along_with_scoring(oracle, shape, n_pairs):
    """begin -> score with the transfer in the same launch -> end.  Masses equal the oracle's scoring of
    the table with the out-units taken out (neither unit of a pair is in HBM meanwhile); pools, tier,
    tables and state afterwards equal the oracle's plain exchange, byte for byte."""
    from paper_2604_26968_amd import kvm
    from tests.harness import oracle_score
    case = synth.make_case(shape, seed=51)
    k8, v8 = host_pools(case)
    rng = np.random.default_rng(9)
    uk, uv = shape.unit_k_bytes, shape.unit_v_bytes
    rec = uk + uv
    res = np.flatnonzero(case.state & RES)
    first_out = np.sort(rng.choice(res, size=len(res) // 3, replace=False)).astype(np.int64)
    n_tier = len(first_out) + 3
    hs = rng.permutation(n_tier)[:len(first_out)].astype(np.int32)
    tbl, st = case.slot_tbl.copy(), case.state.copy()
    staging, _ = oracle.pack(k8, v8, uk, uv, tbl, st, first_out, hs)
    tier = rng.integers(0, 256, size=(n_tier, rec), dtype=np.uint8)
    tier[hs] = staging
    case.slot_tbl[:], case.state[:] = tbl, st
    dev = DeviceCase(case)
    d_tier = torch.from_numpy(tier.reshape(-1).copy()).pin_memory()
    n = n_pairs
    res_now = np.flatnonzero(st & RES)
    outs = rng.choice(res_now, size=n, replace=False).astype(np.int64)
    ins = rng.choice(first_out, size=n, replace=False).astype(np.int64)
    outs[1] = -1
    ins[4] = np.setdiff1d(res_now, outs)[0]
    outs[6] = np.setdiff1d(first_out, ins)[0]
    # oracle: the plain exchange gives the final state and tells which pairs were valid
    tbl_f, st_f, k_f, tier_f = tbl.copy(), st.copy(), k8.copy(), tier.copy()
    v_f = v8.copy() if v8 is not None else None
    bad = np.zeros(1, np.uint32)
    oracle.exchange(k_f, v_f, uk, uv, tbl_f, st_f, outs, ins, tier_f, n_bad=bad)
    ok_out = np.array([0 <= u < case.n_uids and bool(st[u] & RES) and not bool(st_f[u] & RES) for u in outs])
    assert ok_out.sum() == n - 3 and bad[0] == 3
    tbl_mid = tbl.copy()
    tbl_mid[outs[ok_out]] = -1                       # out of HBM for this scoring pass
    q = synth.make_queries(case, 5)
    scale = 1.0 / np.sqrt(shape.dim)
    want_mass = oracle_score(oracle, case, q, scale, fill=-1.0, slot_tbl=tbl_mid)
    # device
    frame = torch.full((n,), -5, dtype=torch.int32, device="cuda")
    host = torch.full((n,), -5, dtype=torch.int64, device="cuda")
    d_outs, d_ins = dev_of(outs), dev_of(ins)
    kvm.kvm_exchange_begin(dev.pool, dev.slot_tbl, dev.state, d_outs, d_ins, n, n_tier, frame, host, n_bad=dev.n_bad)
    dev.mass.fill_(-1.0)
    kvm.kvm_score_step_xfer(dev.pool, dev.rows(), dev_of(q.view(np.int16)), scale, dev.mass, dev.ws, frame, host, n,
                            d_tier)
    torch.cuda.synchronize()
    got_mass = dev.mass.cpu().numpy()
    mid_state = dev.state.cpu().numpy()
    assert not np.any(mid_state[outs[ok_out]] & RES) and not np.any(mid_state[ins[ok_out]] & RES)
    kvm.kvm_exchange_end(dev.slot_tbl, dev.state, d_ins, frame, n)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(frame.cpu().numpy() >= 0, ok_out)
    np.testing.assert_array_equal(frame.cpu().numpy()[ok_out], tbl[outs[ok_out]])
    np.testing.assert_array_equal(host.cpu().numpy()[ok_out], -1 - tbl[ins[ok_out]])
    assert int(dev.n_bad.item()) == 3
    written = want_mass != -1.0
    np.testing.assert_array_equal(got_mass != -1.0, written)
    np.testing.assert_allclose(got_mass[written], want_mass[written], rtol=1e-3, atol=1e-9)
    gk, gv = dev.pools_host()
    np.testing.assert_array_equal(gk, k_f)
    if v8 is not None:
        np.testing.assert_array_equal(gv, v_f)
    np.testing.assert_array_equal(d_tier.numpy().reshape(n_tier, rec), tier_f)
    np.testing.assert_array_equal(dev.slot_tbl.cpu().numpy(), tbl_f)
    np.testing.assert_array_equal(dev.state.cpu().numpy(), st_f)


@pytest.mark.parametrize("shape,n_pairs,n_out", [
    (synth.Shape(2, 8, 2, 128, synth.BF16, True, [700, 77, 1300]), 40, 70),   # dot2 kernel, g = 4
    (synth.Shape(2, 16, 2, 128, synth.BF16, True, [900, 200]), 0, 50),        # matrix-core kernel, g = 8, no swaps
    (synth.Shape(2, 32, 1, 128, synth.FP16, True, [900]), 20, 33),            # matrix-core kernel, g = 32
    (synth.Shape(3, 128, 1, 576, synth.BF16, False, [9000, 300]), 30, 25),    # wide kernel, rows of several tiles
])
def test_pack_in_two_parts_rides_along_with_scoring(oracle, shape, n_pairs, n_out):
    """kvm_pack_begin -> the scoring launch copies the frames out (one-way pairs, in one list with the
    swap pairs of a deferred exchange) -> tables, state and tier equal the oracle's pack (records at their
    host slots) and exchange; masses equal the oracle's scoring of the table without the units that left."""
    from paper_2604_26968_amd import kvm
    from tests.harness import oracle_score
    case = synth.make_case(shape, seed=77)
    k8, v8 = host_pools(case)
    rng = np.random.default_rng(21)
    uk, uv = shape.unit_k_bytes, shape.unit_v_bytes
    rec = uk + uv
    res = np.flatnonzero(case.state & RES)
    first_out = np.sort(rng.choice(res, size=len(res) // 3, replace=False)).astype(np.int64)
    n_tier = len(first_out) + n_out + 5
    hs = rng.permutation(len(first_out) + 2)[:len(first_out)].astype(np.int32)      # slots below len(first_out) + 2
    tbl, st = case.slot_tbl.copy(), case.state.copy()
    staging, _ = oracle.pack(k8, v8, uk, uv, tbl, st, first_out, hs)
    tier = rng.integers(0, 256, size=(n_tier, rec), dtype=np.uint8)
    tier[hs] = staging
    case.slot_tbl[:], case.state[:] = tbl, st
    dev = DeviceCase(case)
    d_tier = torch.from_numpy(tier.reshape(-1).copy()).pin_memory()
    res_now = np.flatnonzero(st & RES)
    pick = rng.choice(res_now, size=n_pairs + n_out, replace=False).astype(np.int64)
    outs, packs = pick[:n_pairs].copy(), pick[n_pairs:].copy()
    ins = rng.choice(first_out, size=n_pairs, replace=False).astype(np.int64)
    pack_slots = (len(first_out) + 2 + np.arange(n_out)).astype(np.int32)             # free slots of the tier
    packs[2] = -7                                     # malformed uid
    packs[5] = first_out[0]                           # not in HBM
    pack_slots[9] = n_tier + 4                        # slot outside the tier
    # oracle: exchange of the pairs, pack of the list; records of accepted entries go to their slots
    tbl_f, st_f, k_f, tier_f = tbl.copy(), st.copy(), k8.copy(), tier.copy()
    v_f = v8.copy() if v8 is not None else None
    bad = np.zeros(1, np.uint32)
    if n_pairs:
        oracle.exchange(k_f, v_f, uk, uv, tbl_f, st_f, outs, ins, tier_f, n_bad=bad)
    ok_pack = np.array([0 <= u < case.n_uids and bool(st[u] & RES) and 0 <= h < n_tier
                        for u, h in zip(packs, pack_slots)])
    assert ok_pack.sum() == n_out - 3
    # the oracle's pack takes any host slot number; entries the device refuses for their slot are left out here
    want_staging, want_freed = oracle.pack(k_f, v_f, uk, uv, tbl_f, st_f, packs[ok_pack], pack_slots[ok_pack])
    tier_f[pack_slots[ok_pack]] = want_staging
    tbl_mid = tbl.copy()
    tbl_mid[outs] = -1
    tbl_mid[packs[ok_pack]] = -1
    q = synth.make_queries(case, 5)
    scale = 1.0 / np.sqrt(shape.dim)
    want_mass = oracle_score(oracle, case, q, scale, fill=-1.0, slot_tbl=tbl_mid)
    # device: one list, swap pairs first
    n = n_pairs + n_out
    frame = torch.full((n,), -5, dtype=torch.int32, device="cuda")
    host = torch.full((n,), -5, dtype=torch.int64, device="cuda")
    if n_pairs:
        kvm.kvm_exchange_begin(dev.pool, dev.slot_tbl, dev.state, dev_of(outs), dev_of(ins), n_pairs, n_tier,
                               frame[:n_pairs], host[:n_pairs], n_bad=dev.n_bad)
    kvm.kvm_pack_begin(dev.pool, dev.slot_tbl, dev.state, dev_of(packs), n_out, dev_of(pack_slots), n_tier,
                       frame[n_pairs:], host[n_pairs:], n_bad=dev.n_bad)
    torch.cuda.synchronize()
    # after begin: tables and state are final for the packed units, their frames still hold their bytes
    np.testing.assert_array_equal(dev.slot_tbl.cpu().numpy()[packs[ok_pack]], tbl_f[packs[ok_pack]])
    np.testing.assert_array_equal(dev.state.cpu().numpy()[packs[ok_pack]], st_f[packs[ok_pack]])
    got_frame = frame.cpu().numpy()[n_pairs:]
    np.testing.assert_array_equal(got_frame[ok_pack], want_freed)
    np.testing.assert_array_equal(got_frame[~ok_pack], -1)
    got_host = host.cpu().numpy()[n_pairs:]
    np.testing.assert_array_equal(got_host[ok_pack], pack_slots[ok_pack].astype(np.int64) | kvm.XFER_OUT_ONLY)
    np.testing.assert_array_equal(got_host[~ok_pack], -1)
    assert int(dev.n_bad.item()) == 3
    dev.mass.fill_(-1.0)
    kvm.kvm_score_step_xfer(dev.pool, dev.rows(), dev_of(q.view(np.int16)), scale, dev.mass, dev.ws, frame, host, n,
                            d_tier)
    if n_pairs:
        kvm.kvm_exchange_end(dev.slot_tbl, dev.state, dev_of(ins), frame[:n_pairs], n_pairs)
    torch.cuda.synchronize()
    got_mass = dev.mass.cpu().numpy()
    written = want_mass != -1.0
    np.testing.assert_array_equal(got_mass != -1.0, written)
    np.testing.assert_allclose(got_mass[written], want_mass[written], rtol=1e-3, atol=1e-9)
    gk, gv = dev.pools_host()
    np.testing.assert_array_equal(gk, k_f)              # one-way: the frames keep their bytes
    if v8 is not None:
        np.testing.assert_array_equal(gv, v_f)
    np.testing.assert_array_equal(d_tier.numpy().reshape(n_tier, rec), tier_f)
    np.testing.assert_array_equal(dev.slot_tbl.cpu().numpy(), tbl_f)
    np.testing.assert_array_equal(dev.state.cpu().numpy(), st_f)


def test_pack_begin_takes_its_count_from_the_device_and_moves_without_rows(oracle):
    """kvm_pack_begin with a device-side list length shorter than the list (entries beyond it are left alone and
    get -1), then the transfer in a launch that scores nothing (no rows): the records still arrive."""
    from paper_2604_26968_amd import kvm
    shape = synth.Shape(1, 4, 2, 64, synth.FP16, True, [512, 100])
    case = synth.make_case(shape, seed=12)
    k8, v8 = host_pools(case)
    dev = DeviceCase(case)
    uk, uv = shape.unit_k_bytes, shape.unit_v_bytes
    rec = uk + uv
    rng = np.random.default_rng(2)
    res = np.flatnonzero(case.state & RES)
    uids = rng.choice(res, size=20, replace=False).astype(np.int64)
    n_dev = torch.tensor([13], dtype=torch.int64, device="cuda")
    slots = np.arange(5, 25, dtype=np.int32)
    n_tier = 30
    d_tier = torch.zeros(n_tier * rec, dtype=torch.uint8).pin_memory()
    frame = torch.full((20,), -5, dtype=torch.int32, device="cuda")
    host = torch.full((20,), -5, dtype=torch.int64, device="cuda")
    kvm.kvm_pack_begin(dev.pool, dev.slot_tbl, dev.state, dev_of(uids), 20, dev_of(slots), n_tier, frame, host,
                       n_dev=n_dev, n_bad=dev.n_bad)
    tbl, st = case.slot_tbl.copy(), case.state.copy()
    want_staging, want_freed = oracle.pack(k8, v8, uk, uv, tbl, st, uids[:13], slots[:13])
    torch.cuda.synchronize()
    np.testing.assert_array_equal(frame.cpu().numpy(), np.r_[want_freed, np.full(7, -1)])
    np.testing.assert_array_equal(host.cpu().numpy(), np.r_[slots[:13].astype(np.int64) | kvm.XFER_OUT_ONLY, np.full(7, -1)])
    np.testing.assert_array_equal(dev.slot_tbl.cpu().numpy(), tbl)
    np.testing.assert_array_equal(dev.state.cpu().numpy(), st)
    assert int(dev.n_bad.item()) == 0
    none = kvm.make_rows(dev.row_ntok[:0], dev.row_off[:0], dev.row_q_off[:0], dev.slot_tbl, shape.g, 0)
    q = torch.zeros(8, dtype=torch.int16, device="cuda")
    dev.mass.fill_(-1.0)
    kvm.kvm_score_step_xfer(dev.pool, none, q, 1.0, dev.mass, dev.ws, frame, host, 20, d_tier)
    torch.cuda.synchronize()
    got = d_tier.numpy().reshape(n_tier, rec)
    np.testing.assert_array_equal(got[slots[:13]], want_staging)
    assert not got[np.setdiff1d(np.arange(n_tier), slots[:13])].any() and bool((dev.mass == -1.0).all())
    gk, gv = dev.pools_host()
    np.testing.assert_array_equal(gk, k8)
    np.testing.assert_array_equal(gv, v8)


def test_end_to_end_overlapped_exchange_dynamics(oracle):
    """The pass as the bench runs it by default, five steps on a twin of the Llama-3-8B-shaped workload:
    beta -> score (with the previous step's exchange bytes in the same launch) -> ema -> exchange_end ->
    select to budget -> exchange_begin.  Masses, EMA state, victim sets, tables, pools and the host tier
    follow the oracle step by step; each exchange as a whole equals the oracle's plain exchange."""
    from paper_2604_26968_amd import kvm
    from tests.harness import oracle_score
    from tests.test_gpu_parity import victims_agree, MASS_RTOL, MASS_ATOL
    shape = synth.Shape(2, 8, 2, 128, synth.BF16, True, [700, 2100, 333])
    case = synth.make_case(shape, seed=61, pair_weights=synth.categorical_weights(3))
    sh = case.shape
    uk, uv = sh.unit_k_bytes, sh.unit_v_bytes
    rec = uk + uv
    rng = np.random.default_rng(2)
    k8, v8 = host_pools(case)
    # start: 40 % of the units on the host tier (slot-addressed), the rest in HBM
    res = np.flatnonzero((case.state & RES) != 0)
    res = res[(case.state[res] & PROT) == 0]
    first_out = np.sort(rng.choice(res, size=int(0.4 * len(res)), replace=False)).astype(np.int64)
    n_tier = len(first_out)
    hs = rng.permutation(n_tier).astype(np.int32)
    staging, _ = oracle.pack(k8, v8, uk, uv, case.slot_tbl, case.state, first_out, hs)
    tier = np.zeros((n_tier, rec), np.uint8)
    tier[hs] = staging
    dev = DeviceCase(case)
    d_tier = torch.from_numpy(tier.reshape(-1).copy()).pin_memory()
    budget = int(np.sum((case.state & RES) != 0)) - 30           # 30 victims and 30 prefetches per step
    n = 30
    S, prio = np.zeros(case.n_uids, np.float32), np.zeros(case.n_uids, np.float32)
    hits, misses = np.zeros(16, np.uint32), np.zeros(16, np.uint32)
    frame = torch.full((n,), -1, dtype=torch.int32, device="cuda")
    host = torch.full((n,), -1, dtype=torch.int64, device="cuda")
    d_ins = torch.full((n,), -1, dtype=torch.int64, device="cuda")
    pending = None                                               # (ins, frames, hosts, expected final state)
    w = synth.categorical_weights(8)
    scale = 1 / np.sqrt(128)
    for step in range(5):
        q = synth.make_queries(case, 80 + step)
        ev = synth.make_events(512, 500 + step, pair_weights=w, reuse_prob=np.linspace(0.2, 0.95, 16))
        gh, gm, gp = dev.beta(*ev)
        p_hat = oracle.beta_update(ev[0], ev[1], hits, misses)
        np.testing.assert_array_equal(gh, hits)
        # score: the tables are as exchange_begin left them; the transfer of the previous step rides along
        dev.mass.fill_(-1.0)
        kvm.kvm_score_step_xfer(dev.pool, dev.rows(), torch.from_numpy(q.view(np.int16)).cuda(), scale, dev.mass,
                                dev.ws, frame, host, n, d_tier)
        torch.cuda.synchronize()
        gmass = dev.mass.cpu().numpy()
        omass = oracle_score(oracle, case, q, scale, fill=-1.0)
        np.testing.assert_array_equal(gmass != -1.0, omass != -1.0)
        wr = omass != -1.0
        np.testing.assert_allclose(gmass[wr], omass[wr], rtol=MASS_RTOL, atol=MASS_ATOL)
        gS, gprio, gstate = dev.ema(0.95)
        oracle.ema_update(case.row_ntok, case.row_off, omass, 0.95, ref_row_weight(oracle, case), case.pair, p_hat, case.state,
                          S, prio)
        np.testing.assert_array_equal(gstate, case.state)
        resm = (case.state & RES) != 0
        np.testing.assert_allclose(gS[resm], S[resm], rtol=MASS_RTOL)
        # the previous exchange completes: incoming units get their frames
        kvm.kvm_exchange_end(dev.slot_tbl, dev.state, d_ins, frame, n)
        if pending is not None:
            ins, frames, hosts, want = pending
            k8[frames], tier[hosts, :uk] = tier[hosts, :uk].copy(), k8[frames].copy()
            v8[frames], tier[hosts, uk:] = tier[hosts, uk:].copy(), v8[frames].copy()
            case.slot_tbl[ins] = frames
            case.state[ins] = (case.state[ins] & ~np.uint8(HOST)) | RES
            case.k_pool[:] = k8.view(np.uint16).reshape(case.k_pool.shape)
            # ... and the whole exchange equals the oracle's plain one (SCORED bits set meanwhile aside)
            tbl_w, st_w, k_w, v_w, tier_w = want
            np.testing.assert_array_equal(case.slot_tbl, tbl_w)
            np.testing.assert_array_equal(case.state & ~np.uint8(SCORED), st_w & ~np.uint8(SCORED))
            np.testing.assert_array_equal(k8, k_w)
            np.testing.assert_array_equal(v8, v_w)
            np.testing.assert_array_equal(tier, tier_w)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(dev.slot_tbl.cpu().numpy(), case.slot_tbl)
        np.testing.assert_array_equal(dev.state.cpu().numpy(), case.state)
        gk, gvv = dev.pools_host()
        np.testing.assert_array_equal(gk, k8)
        np.testing.assert_array_equal(gvv, v8)
        np.testing.assert_array_equal(d_tier.numpy().reshape(n_tier, rec), tier)
        # victims down to the budget; both sides continue with the oracle's list
        n_over = int(np.sum((case.state & RES) != 0)) - budget
        gv = dev.select(k=-1, budget=budget)
        ov = oracle.select_victims(prio, case.state, k=-1, budget_units=budget)
        victims_agree(gv, ov, prio, case.state)
        assert len(ov) == n_over == n
        on_host = np.flatnonzero(((case.state & HOST) != 0) & ((case.state & RES) == 0))
        ins = rng.choice(on_host, size=n, replace=False).astype(np.int64)
        outs = ov.astype(np.int64)
        # what the oracle's plain exchange makes of it (on copies)
        want = (case.slot_tbl.copy(), case.state.copy(), k8.copy(), v8.copy(), tier.copy())
        oracle.exchange(want[2], want[3], uk, uv, want[0], want[1], outs, ins, want[4])
        # begin: the victims leave the table now
        frames, hosts = case.slot_tbl[outs].copy(), (-1 - case.slot_tbl[ins]).astype(np.int64)
        case.slot_tbl[outs] = (-1 - hosts).astype(np.int32)
        case.state[outs] = (case.state[outs] & ~np.uint8(RES)) | HOST
        d_ins = dev_of(ins)
        kvm.kvm_exchange_begin(dev.pool, dev.slot_tbl, dev.state, dev_of(outs), d_ins, n, n_tier, frame, host,
                               n_bad=dev.n_bad)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(frame.cpu().numpy(), frames)
        np.testing.assert_array_equal(host.cpu().numpy(), hosts)
        np.testing.assert_array_equal(dev.slot_tbl.cpu().numpy(), case.slot_tbl)
        np.testing.assert_array_equal(dev.state.cpu().numpy(), case.state)
        pending = (ins, frames, hosts, want)
    assert int(dev.n_bad.item()) == 0


def test_end_to_end_pipelined_selection_dynamics(oracle):
    """The pass as the bench runs it by default: the victims are chosen from the priorities the previous
    step left, on a second stream, while the scoring launch (with the previous exchange's bytes riding
    along) runs on the first; then ema -> exchange_end -> exchange_begin with those victims.  Nothing is
    synchronised inside a step on the GPU side; at the end of every step masses, EMA state, victims,
    tables, pools and the host tier are compared with the oracle, which takes the same stages in order."""
    from paper_2604_26968_amd import kvm
    from tests.harness import oracle_score
    from tests.test_gpu_parity import victims_agree, MASS_RTOL, MASS_ATOL
    shape = synth.Shape(2, 8, 2, 128, synth.BF16, True, [700, 2100, 333])
    case = synth.make_case(shape, seed=62, pair_weights=synth.categorical_weights(3))
    sh = case.shape
    uk, uv = sh.unit_k_bytes, sh.unit_v_bytes
    rec = uk + uv
    rng = np.random.default_rng(3)
    k8, v8 = host_pools(case)
    res = np.flatnonzero((case.state & RES) != 0)
    res = res[(case.state[res] & PROT) == 0]
    first_out = np.sort(rng.choice(res, size=int(0.4 * len(res)), replace=False)).astype(np.int64)
    n_tier = len(first_out)
    hs = rng.permutation(n_tier).astype(np.int32)
    staging, _ = oracle.pack(k8, v8, uk, uv, case.slot_tbl, case.state, first_out, hs)
    tier = np.zeros((n_tier, rec), np.uint8)
    tier[hs] = staging
    dev = DeviceCase(case)
    d_tier = torch.from_numpy(tier.reshape(-1).copy()).pin_memory()
    n = 24
    S, prio = np.zeros(case.n_uids, np.float32), np.zeros(case.n_uids, np.float32)
    hits, misses = np.zeros(16, np.uint32), np.zeros(16, np.uint32)
    frame = torch.full((n,), -1, dtype=torch.int32, device="cuda")
    host = torch.full((n,), -1, dtype=torch.int64, device="cuda")
    d_ins = torch.full((n,), -1, dtype=torch.int64, device="cuda")
    d_outs = torch.zeros(n, dtype=torch.int64, device="cuda")
    ws_select = torch.full((max(kvm.kvm_workspace_bytes(kvm.OP_SELECT, case.n_uids), 256),), 0x7F, dtype=torch.uint8,
                           device="cuda")
    main, side = torch.cuda.current_stream(), torch.cuda.Stream()
    pending = None
    w = synth.categorical_weights(8)
    scale = 1 / np.sqrt(128)
    # one plain step first, so that there are scored units to choose from
    q = synth.make_queries(case, 70)
    omass = oracle_score(oracle, case, q, scale, fill=-1.0)
    dev.score(q, scale, fill=-1.0)
    p_hat = oracle.beta_update(np.zeros(0, np.uint8), np.zeros(0, np.uint8), hits, misses)
    dev.beta(np.zeros(0, np.uint8), np.zeros(0, np.uint8))
    oracle.ema_update(case.row_ntok, case.row_off, omass, 0.95, ref_row_weight(oracle, case), case.pair, p_hat, case.state, S, prio)
    dev.ema(0.95)
    for step in range(5):
        q = synth.make_queries(case, 80 + step)
        ev = synth.make_events(512, 600 + step, pair_weights=w, reuse_prob=np.linspace(0.2, 0.95, 16))
        d_q = torch.from_numpy(q.view(np.int16)).cuda()
        d_ev = (torch.from_numpy(ev[0]).cuda(), torch.from_numpy(ev[1]).cuda())
        dev.mass.fill_(-1.0)
        # ---- GPU: the whole step without a synchronisation
        side.wait_stream(main)
        kvm.kvm_beta_update(d_ev[0], d_ev[1], dev.hits, dev.misses, dev.p_hat, n_bad=dev.n_bad, stream=side)
        kvm.kvm_select_victims(dev.prio, dev.state, d_outs, dev.n_victims, ws_select, k=n, stream=side)
        kvm.kvm_score_step_xfer(dev.pool, dev.rows(), d_q, scale, dev.mass, dev.ws, frame, host, n, d_tier)
        main.wait_stream(side)
        kvm.kvm_ema_update(dev.rows(), dev.mass, 0.95, dev.row_weight, dev.pair, dev.p_hat, dev.state, dev.S, dev.prio)
        kvm.kvm_exchange_end(dev.slot_tbl, dev.state, d_ins, frame, n)
        torch.cuda.synchronize()
        # ---- oracle: the same stages in order
        p_hat = oracle.beta_update(ev[0], ev[1], hits, misses)
        ov = oracle.select_victims(prio, case.state, k=n)
        gv = d_outs[: int(dev.n_victims.item())].cpu().numpy()
        victims_agree(gv, ov, prio, case.state)
        assert len(ov) == n
        omass = oracle_score(oracle, case, q, scale, fill=-1.0)
        gmass = dev.mass.cpu().numpy()
        np.testing.assert_array_equal(gmass != -1.0, omass != -1.0)
        wr = omass != -1.0
        np.testing.assert_allclose(gmass[wr], omass[wr], rtol=MASS_RTOL, atol=MASS_ATOL)
        oracle.ema_update(case.row_ntok, case.row_off, omass, 0.95, ref_row_weight(oracle, case), case.pair, p_hat, case.state,
                          S, prio)
        resm = (case.state & RES) != 0
        np.testing.assert_allclose(dev.S.cpu().numpy()[resm], S[resm], rtol=MASS_RTOL)
        np.testing.assert_array_equal(dev.hits.cpu().numpy().view(np.uint32), hits)
        if pending is not None:
            ins, frames, hosts = pending
            k8[frames], tier[hosts, :uk] = tier[hosts, :uk].copy(), k8[frames].copy()
            v8[frames], tier[hosts, uk:] = tier[hosts, uk:].copy(), v8[frames].copy()
            case.slot_tbl[ins] = frames
            case.state[ins] = (case.state[ins] & ~np.uint8(HOST)) | RES
            case.k_pool[:] = k8.view(np.uint16).reshape(case.k_pool.shape)
        np.testing.assert_array_equal(dev.slot_tbl.cpu().numpy(), case.slot_tbl)
        np.testing.assert_array_equal(dev.state.cpu().numpy(), case.state)
        gk, gvv = dev.pools_host()
        np.testing.assert_array_equal(gk, k8)
        np.testing.assert_array_equal(gvv, v8)
        np.testing.assert_array_equal(d_tier.numpy().reshape(n_tier, rec), tier)
        # ---- both sides continue with the oracle's victims
        on_host = np.flatnonzero(((case.state & HOST) != 0) & ((case.state & RES) == 0))
        ins = rng.choice(on_host, size=n, replace=False).astype(np.int64)
        outs = ov.astype(np.int64)
        frames, hosts = case.slot_tbl[outs].copy(), (-1 - case.slot_tbl[ins]).astype(np.int64)
        case.slot_tbl[outs] = (-1 - hosts).astype(np.int32)
        case.state[outs] = (case.state[outs] & ~np.uint8(RES)) | HOST
        d_outs.copy_(torch.from_numpy(outs))
        d_ins.copy_(torch.from_numpy(ins))
        kvm.kvm_exchange_begin(dev.pool, dev.slot_tbl, dev.state, d_outs, d_ins, n, n_tier, frame, host,
                               n_bad=dev.n_bad)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(frame.cpu().numpy(), frames)
        np.testing.assert_array_equal(host.cpu().numpy(), hosts)
        np.testing.assert_array_equal(dev.slot_tbl.cpu().numpy(), case.slot_tbl)
        pending = (ins, frames, hosts)
    assert int(dev.n_bad.item()) == 0


def test_transfer_pairs_with_frame_numbers_outside_the_pool_are_skipped(oracle):
    """kvm_score_step_xfer takes the pair lists as they are: a frame number that is negative or not below
    n_slots, or a tier slot outside the tier (a caller's mistake; kvm_exchange_begin never writes one), moves nothing, the other pairs trade
    contents with their tier records, and scoring is unaffected."""
    from paper_2604_26968_amd import kvm
    from tests.harness import oracle_score
    shape = synth.Shape(1, 8, 2, 128, synth.BF16, True, [700, 1200])
    case = synth.make_case(shape, seed=61, spare_slots=8)
    dev = DeviceCase(case)
    rec = shape.unit_k_bytes + shape.unit_v_bytes
    rng = np.random.default_rng(3)
    spare = np.setdiff1d(np.arange(case.n_slots), case.slot_tbl[case.slot_tbl >= 0])[:8].astype(np.int32)
    frames = spare.copy()                     # frames no unit uses: scoring cannot see them
    frames[1], frames[4], frames[6] = -1, case.n_slots, 2**31 - 1
    hosts = np.arange(8, dtype=np.int64)
    hosts[0], hosts[3] = 8, -2                # tier records that do not exist
    valid = (frames >= 0) & (frames < case.n_slots) & (hosts >= 0) & (hosts < 8)
    tier = rng.integers(0, 256, size=(8, rec), dtype=np.uint8)
    d_tier = torch.from_numpy(tier.reshape(-1).copy()).pin_memory()
    k_before, v_before = dev.pools_host()
    k_before, v_before = k_before.copy(), v_before.copy()
    q = synth.make_queries(case, 8)
    scale = 1.0 / np.sqrt(shape.dim)
    kvm.kvm_score_step_xfer(dev.pool, dev.rows(), dev_of(q.view(np.int16)), scale, dev.mass, dev.ws, dev_of(frames),
                            dev_of(hosts), 8, d_tier)
    torch.cuda.synchronize()
    np.testing.assert_allclose(dev.mass.cpu().numpy(), oracle_score(oracle, case, q, scale), rtol=1e-3, atol=1e-9)
    k_after, v_after = dev.pools_host()
    tier_after = d_tier.numpy().reshape(8, rec)
    want_k, want_v, want_tier = k_before.copy(), v_before.copy(), tier.copy()
    for i in np.flatnonzero(valid):
        f = frames[i]
        want_tier[i] = np.concatenate([k_before[f], v_before[f]])
        want_k[f], want_v[f] = tier[i, :shape.unit_k_bytes], tier[i, shape.unit_k_bytes:]
    np.testing.assert_array_equal(k_after, want_k)
    np.testing.assert_array_equal(v_after, want_v)
    np.testing.assert_array_equal(tier_after, want_tier)
