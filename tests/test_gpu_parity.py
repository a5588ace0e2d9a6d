"""GPU parity: every stage of the HIP path against the CPU oracle on the same
seeded inputs, through the C ABI.

Tolerances
  masses      rel 1e-3 (bf16/fp16 inputs, fp32 accumulation), abs floor 1e-9
  S, prio     rel 2e-6 per step when fed identical masses (fp32 vs fp64 arithmetic)
  counters, victims (on identical keys), tables, staging bytes: bit-exact
"""
import numpy as np
import pytest
import torch

from paper_2604_26968_amd import synth
from tests.harness import DeviceCase, host_pools, oracle_score, ref_row_weight, run_step_gpu, run_step_oracle

pytestmark = pytest.mark.gpu

RES, HOST, PROT, SCORED = 1, 2, 4, 8
MASS_RTOL, MASS_ATOL = 1e-3, 1e-9


def evict_some(case, frac, seed):
    """Mark a random fraction of units as living on the host (table < 0, state ON_HOST)."""
    rng = np.random.default_rng(seed)
    res = np.nonzero(case.state & RES)[0]
    gone = rng.choice(res, size=int(len(res) * frac), replace=False)
    case.slot_tbl[gone] = -1 - np.arange(len(gone), dtype=np.int32)
    case.state[gone] = (case.state[gone] & ~np.uint8(RES)) | HOST
    return gone


def check_mass(o, case, q, scale, agg=0, row_active=None, need_written=True):
    dev = DeviceCase(case)
    got = dev.score(q, scale, agg=agg, row_active=row_active, fill=-7.0)
    want = oracle_score(o, case, q, scale, agg=agg, row_active=row_active, fill=-7.0)
    written = want != -7.0
    np.testing.assert_array_equal(got[~written], -7.0)          # untouched entries stay untouched
    np.testing.assert_allclose(got[written], want[written], rtol=MASS_RTOL, atol=MASS_ATOL)
    assert written.any() or not need_written
    return got, want


# ------------------------------------------------------------------- scoring
def test_score_tiny_gqa_fp16(oracle):
    case = synth.tiny_gqa(1)
    for step in range(3):
        check_mass(oracle, case, synth.make_queries(case, 2 + step), 1 / 8)


@pytest.mark.parametrize("hq,hkv,dim,dtype", [
    (1, 1, 128, synth.BF16),     # MHA, g = 1
    (4, 2, 64, synth.FP16),      # g = 2
    (32, 8, 128, synth.BF16),    # g = 4 (Llama-3-8B shape)
    (64, 8, 128, synth.BF16),    # g = 8 (Llama-3-70B shape)
    (8, 1, 128, synth.FP16),     # MQA, g = 8
    (6, 2, 128, synth.BF16),     # g = 3: queries staged in LDS
    (32, 1, 128, synth.BF16),    # MQA, g = 32
    (16, 1, 64, synth.BF16),     # g = 16
    (5, 1, 96, synth.FP16),      # odd g, dim 96
    (2, 1, 256, synth.BF16),     # dim 256
    (12, 1, 128, synth.FP16),    # g = 12: one 16-query column tile on the matrix cores
    (24, 1, 256, synth.BF16),    # g = 24, dim 256: two column tiles
    (40, 1, 64, synth.BF16),     # g = 40: three column tiles (padded to four)
    (128, 1, 128, synth.FP16),   # g = 128, dim 128: eight column tiles
    (4, 1, 32, synth.BF16),      # the smallest head the library takes: one 16-byte load per lane and unit
    (16, 4, 192, synth.FP16),    # g = 4, dim 192: beyond the dot-product kernel's 128 channels
    (3, 1, 192, synth.BF16),     # odd g, dim 192
])
def test_score_shapes_ragged_rows(oracle, hq, hkv, dim, dtype):
    """Rows of 1 .. 200 blocks with ragged tails, gaps in uid space, spare pool frames,
    NaN patterns behind the last token, 30 % of the units not resident."""
    lens = [16 * 64 + 5, 1, 16, 17, 3000, 16 * 128, 777]
    case = synth.make_case(synth.Shape(2, hq, hkv, dim, dtype, True, lens), seed=hq * 131 + dim,
                           spare_slots=9, uid_gap=3, poison_tail=True)
    evict_some(case, 0.3, 5)
    q = synth.make_queries(case, 17)
    check_mass(oracle, case, q, 1.0 / np.sqrt(dim))
    check_mass(oracle, case, q, 1.0 / np.sqrt(dim), agg=1)


def test_score_inactive_empty_and_fully_evicted_rows(oracle):
    case = synth.make_case(synth.Shape(1, 8, 2, 128, synth.BF16, True, [100, 0, 50, 300]), seed=3)
    # every unit of row 0 (sequence 0, head 0) evicted
    nb0 = 7
    case.slot_tbl[case.row_off[0]: case.row_off[0] + nb0] = -5
    case.state[case.row_off[0]: case.row_off[0] + nb0] = HOST
    active = np.ones(case.n_rows, np.uint8)
    active[-1] = 0
    q = synth.make_queries(case, 4)
    got, want = check_mass(oracle, case, q, 0.09, row_active=active)
    assert np.all(got[case.row_off[0]: case.row_off[0] + nb0] == -7.0)
    assert np.all(got[case.row_off[-1]:] == -7.0)


def test_score_sharp_softmax_large_logits(oracle):
    """Queries scaled so logits reach several hundred: the two-level max / sum must not overflow."""
    case = synth.make_case(synth.Shape(1, 4, 1, 128, synth.BF16, True, [2000]), seed=8)
    q = synth.make_queries(case, 5, scale=6.0)
    got, want = check_mass(oracle, case, q, 1.0)
    assert got.max() > 0.5 and np.isfinite(got).all()


def test_score_tile_boundaries(oracle):
    """Rows of exactly one tile (512 blocks), one block more, and several tiles, g = 4 and g = 2."""
    for hq, hkv, dtype in ((4, 1, synth.BF16), (4, 2, synth.FP16)):
        lens = [16 * 512, 16 * 512 + 1, 16 * 1024 + 3, 16 * 511 + 15, 16 * 1537]
        case = synth.make_case(synth.Shape(1, hq, hkv, 64, dtype, True, lens), seed=77, uid_gap=1)
        evict_some(case, 0.35, 3)
        # a whole tile of the last row not resident
        o = case.row_off[-1] + 512
        case.slot_tbl[o:o + 512] = -9
        case.state[o:o + 512] = HOST
        q = synth.make_queries(case, 31)
        check_mass(oracle, case, q, 0.125)
        check_mass(oracle, case, q, 0.125, agg=1)


@pytest.mark.parametrize("hq,hkv,dim", [(1, 1, 128), (4, 1, 128), (32, 1, 128), (128, 1, 576)])
def test_score_rows_with_wholly_evicted_tiles(oracle, hq, hkv, dim):
    """Rows of several tiles in which the first, a middle or the last tile holds no resident block
    (after heavy eviction only a handful of blocks of a long row remain): the empty tile must count
    as nothing in the row's normaliser, whatever the workspace held before."""
    has_v = dim != 576
    lens = [16 * 780 - 2, 16 * 1537, 16 * 2048, 16 * 600 + 7]
    case = synth.make_case(synth.Shape(1, hq, hkv, dim, synth.BF16, has_v, lens), seed=5 + hq)
    keep = {0: [779, 521], 1: [600, 1536], 2: [3, 2047], 3: [599]}
    for r in range(case.n_rows):
        o, nb = int(case.row_off[r]), (int(case.row_ntok[r]) + 15) // 16
        gone = np.setdiff1d(np.arange(nb), keep[r])
        case.slot_tbl[o + gone] = -3
        case.state[o + gone] = HOST
    q = synth.make_queries(case, 23)
    got, want = check_mass(oracle, case, q, 1.0 / np.sqrt(dim))
    for r in range(case.n_rows):
        o = int(case.row_off[r])
        if hq == 1:
            assert abs(sum(got[o + b] for b in keep[r]) - 1.0) < 1e-5
    check_mass(oracle, case, q, 1.0 / np.sqrt(dim), agg=1)


@pytest.mark.parametrize("seed", range(16))
def test_score_random_configurations(oracle, seed):
    """Seeded random shapes: group size, head dim, dtype, lognormal row lengths up to ~20k tokens,
    uid gaps, spare frames, inactive rows, and eviction that mixes scattered single blocks with
    contiguous spans (whole tiles of a long row, prefixes, everything but the tail)."""
    rng = np.random.default_rng(1000 + seed)
    hq, hkv, dim = [(1, 1, 128), (8, 8, 64), (4, 1, 128), (8, 2, 128), (8, 1, 128), (32, 1, 128), (16, 1, 256),
                    (20, 1, 64), (64, 1, 128), (128, 1, 576), (7, 1, 96), (48, 1, 128), (128, 1, 128),
                    (16, 1, 576), (2, 1, 64), (64, 8, 128)][seed]
    dtype = synth.BF16 if rng.random() < 0.6 else synth.FP16
    n_seq = int(rng.integers(2, 7))
    lens = [int(x) for x in np.clip(np.exp(rng.normal(7.5, 1.3, n_seq)), 1, 20000)]
    lens[int(rng.integers(n_seq))] = int(rng.integers(9000, 20000))        # always one row of many tiles
    case = synth.make_case(synth.Shape(1, hq, hkv, dim, dtype, dim != 576, lens), seed=2000 + seed,
                           spare_slots=int(rng.integers(0, 20)), uid_gap=int(rng.integers(0, 4)), poison_tail=True)
    evict_some(case, float(rng.choice([0.0, 0.2, 0.6, 0.95])), seed)
    for r in range(case.n_rows):
        o, nb = int(case.row_off[r]), (int(case.row_ntok[r]) + 15) // 16
        kind = rng.integers(5)
        if kind == 0 or nb < 2:
            continue
        if kind == 1:       # a prefix
            a, b = 0, int(rng.integers(1, nb))
        elif kind == 2:     # everything but the last block
            a, b = 0, nb - 1
        elif kind == 3:     # a span in the middle
            a = int(rng.integers(0, nb - 1))
            b = int(rng.integers(a + 1, nb))
        else:               # the tail
            a, b = int(rng.integers(0, nb)), nb
        case.slot_tbl[o + a:o + b] = -2
        case.state[o + a:o + b] = HOST
    active = (rng.random(case.n_rows) < 0.85).astype(np.uint8)
    q = synth.make_queries(case, 3000 + seed)
    scale = float(rng.choice([1.0, 0.5, 2.0])) / np.sqrt(dim)
    active[int(np.argmax(case.row_ntok))] = 1
    check_mass(oracle, case, q, scale, agg=int(rng.integers(2)), row_active=active, need_written=False)


@pytest.mark.parametrize("hq,hkv,dim", [(8, 2, 128), (32, 1, 128), (128, 1, 576)])
def test_score_rows_listed_in_arbitrary_order(oracle, hq, hkv, dim):
    """Nothing ties a row's place in the row arrays to the place of its units or of its queries:
    rows listed in a shuffled order (short and long ones mixed, one of several tiles) give the same
    masses, bit for bit, as the same rows listed in order."""
    lens = [16 * 700 + 3, 40, 16 * 90, 16 * 1300 + 9, 500, 16]
    case = synth.make_case(synth.Shape(2, hq, hkv, dim, synth.BF16, dim != 576, lens), seed=77 + hq, uid_gap=2,
                           poison_tail=True)
    evict_some(case, 0.4, 11)
    q = synth.make_queries(case, 41)
    scale = 1.0 / np.sqrt(dim)
    got_in_order, _ = check_mass(oracle, case, q, scale)
    perm = np.random.default_rng(5).permutation(case.n_rows)
    case.row_ntok, case.row_off, case.row_q_off = case.row_ntok[perm].copy(), case.row_off[perm].copy(), \
        case.row_q_off[perm].copy()
    case.row_seq = case.row_seq[perm].copy()
    got_shuffled, _ = check_mass(oracle, case, q, scale)
    np.testing.assert_array_equal(got_shuffled, got_in_order)


@pytest.mark.parametrize("hq,dim,n_blocks", [(64, 128, 2200), (128, 128, 4500), (8, 128, 9000)])
def test_score_rows_of_more_tiles_than_one_fold_batch(oracle, hq, dim, n_blocks):
    """The row merge folds a row's tile values sixteen (or, with two threads per query, thirty-two) at
    a time: rows of 18, 71 and 18 tiles take it through more than one batch on each of its kernels."""
    case = synth.make_case(synth.Shape(1, hq, 1, dim, synth.BF16, True, [16 * n_blocks - 5, 300]), seed=hq + 3)
    evict_some(case, 0.5, 2)
    check_mass(oracle, case, synth.make_queries(case, 9), 1.0 / np.sqrt(dim))


def test_score_tens_of_thousands_of_short_rows(oracle):
    """40,000 rows of one to three blocks: the plan's scan runs over hundreds of workgroup totals and
    carries across its own chunks; a few rows are inactive or empty."""
    rng = np.random.default_rng(8)
    lens = [int(x) for x in rng.integers(0, 41, size=1000)]
    case = synth.make_case(synth.Shape(1, 40, 40, 64, synth.FP16, True, lens), seed=4, poison_tail=True)
    assert case.n_rows == 40000
    evict_some(case, 0.25, 3)
    active = (rng.random(case.n_rows) < 0.97).astype(np.uint8)
    check_mass(oracle, case, synth.make_queries(case, 10), 0.125, row_active=active)


def test_score_llama8b_twin(oracle):
    case = synth.llama8b_twin(n_seq=2, n_layers=1)
    evict_some(case, 0.4, 9)
    check_mass(oracle, case, synth.make_queries(case, 21), 1 / np.sqrt(128))


def test_score_long_rows_8192_blocks(oracle):
    case = synth.llama70b_twin(n_tok=131072 - 5)      # 8192 blocks, ragged tail, g = 8
    evict_some(case, 0.5, 2)
    check_mass(oracle, case, synth.make_queries(case, 22), 1 / np.sqrt(128))


def test_score_mla_latent_576_g128(oracle):
    case = synth.mla_twin(n_seq=2, n_tok=1500)
    evict_some(case, 0.25, 4)
    check_mass(oracle, case, synth.make_queries(case, 23), 1 / 24)


def test_score_mla_large_and_uneven_logits(oracle):
    """The wide kernel takes exponentials against a running reference per query.  Small-integer keys
    and queries make every logit exact in fp32, so logits of hundreds of nats can be used: heads of very
    different scale, keys that grow along the row (the maximum keeps rising, the reference is refreshed
    mid-tile) and blocks that vanish against it must all come out right, over several tiles."""
    shape = synth.Shape(1, 128, 1, 576, synth.BF16, False, [10000, 300])
    case = synth.make_case(shape, seed=19)
    rng = np.random.default_rng(19)
    for r in range(case.n_rows):
        nb = (case.row_ntok[r] + 15) // 16
        for b in range(nb):
            slot = case.slot_tbl[case.row_off[r] + b]
            k = rng.integers(-1, 2, 16 * 576).astype(np.float32) * (1 + (3 * b) // nb)      # growth 1, 2, 3
            case.k_pool[slot] = synth.to_bits(k, shape.dtype)
    evict_some(case, 0.3, 6)
    q = rng.integers(-1, 2, (case.n_rows, 128, 576)).astype(np.float32)
    q *= np.array([1, 2, 4, 8], np.float32)[np.arange(128) % 4][None, :, None]                 # per-head scales
    qb = synth.to_bits(q.reshape(-1), shape.dtype)
    got, want = check_mass(oracle, case, qb, 0.25)                # logits up to several hundred nats
    assert np.isfinite(got).all() and got.max() > 0.3


def test_score_properties(oracle):
    """Properties that hold at any size: per-query masses sum to 1 (mean aggregation),
    zero queries give token fractions exactly."""
    case = synth.make_case(synth.Shape(1, 4, 1, 128, synth.BF16, True, [5000, 333]), seed=12)
    dev = DeviceCase(case)
    mean = dev.score(synth.make_queries(case, 1), 0.1, agg=1, fill=0.0)
    for r in range(case.n_rows):
        nb = (case.row_ntok[r] + 15) // 16
        assert abs(mean[case.row_off[r]: case.row_off[r] + nb].sum() - 1.0) < 1e-4
    zero = dev.score(np.zeros(dev.q_elems, np.uint16), 1.0, fill=0.0)
    for r in range(case.n_rows):
        n = int(case.row_ntok[r])
        nb = (n + 15) // 16
        want = np.array([min(16, n - 16 * b) / n for b in range(nb)], np.float32)
        np.testing.assert_allclose(zero[case.row_off[r]: case.row_off[r] + nb], want, rtol=1e-6)


# ---------------------------------------------------------------------- beta
def test_beta_counts_bit_exact(oracle):
    case = synth.tiny_gqa(1)
    dev = DeviceCase(case)
    hits, misses = np.zeros(16, np.uint32), np.zeros(16, np.uint32)
    bad = np.zeros(1, np.uint32)
    w = synth.categorical_weights(5)
    for step, n in enumerate([0, 1, 25, 4096, 200000]):
        ev = synth.make_events(n, 30 + step, pair_weights=w, reuse_prob=np.linspace(0.1, 0.9, 16))
        if n >= 25:
            ev[0][3], ev[1][7] = 200, 9                     # two malformed events
        want_p = oracle.beta_update(ev[0], ev[1], hits, misses, n_bad=bad)
        h, m, p = dev.beta(*ev)
        np.testing.assert_array_equal(h, hits)
        np.testing.assert_array_equal(m, misses)
        np.testing.assert_allclose(p, want_p, rtol=1e-6)
        assert int(dev.n_bad.item()) == int(bad[0])
    for a0, b0 in ((0.5, 0.5), (2.0, 3.0)):
        want_p = oracle.beta_update(np.zeros(0, np.uint8), np.zeros(0, np.uint8), hits, misses, a0, b0)
        _, _, p = dev.beta(np.zeros(0, np.uint8), np.zeros(0, np.uint8), a0, b0)
        np.testing.assert_allclose(p, want_p, rtol=1e-6)


# ----------------------------------------------------------------------- ema
def test_ema_priority_multi_step(oracle):
    case = synth.make_case(synth.Shape(2, 8, 2, 64, synth.BF16, True, [100, 700, 33]), seed=6, uid_gap=2,
                           pair_weights=synth.categorical_weights(1))
    evict_some(case, 0.2, 1)
    dev = DeviceCase(case)
    rng = np.random.default_rng(0)
    S, prio = np.zeros(case.n_uids, np.float32), np.full(case.n_uids, -3.0, np.float32)
    dev.prio.fill_(-3.0)
    state = case.state.copy()
    for step in range(6):
        mass = rng.random(case.n_uids).astype(np.float32)
        p_hat = rng.random(16).astype(np.float32)
        active = (rng.random(case.n_rows) < 0.8).astype(np.uint8) if step else None
        dev.mass.copy_(torch.from_numpy(mass))
        dev.p_hat.copy_(torch.from_numpy(p_hat))
        gS, gprio, gstate = dev.ema(0.95, row_active=active)
        oracle.ema_update(case.row_ntok, case.row_off, mass, 0.95, ref_row_weight(oracle, case), case.pair, p_hat, state,
                          S, prio, row_active=active)
        np.testing.assert_array_equal(gstate, state)
        np.testing.assert_allclose(gS, S, rtol=2e-6)
        fin = np.isfinite(prio)
        np.testing.assert_array_equal(np.isposinf(gprio), np.isposinf(prio))
        np.testing.assert_allclose(gprio[fin], prio[fin], rtol=2e-6)
        # keep both sides on identical inputs for the next step
        dev.S.copy_(torch.from_numpy(S))


# -------------------------------------------------------------------- select
def select_both(oracle, dev, prio, state, k=-1, budget=0, cap=None, shift=0):
    from paper_2604_26968_amd import kvm
    # shift > 0: the arrays start `shift` elements into their allocations (no 16-byte alignment)
    dev.prio = torch.cat([torch.zeros(shift), torch.from_numpy(prio)]).cuda()[shift:]
    dev.state = torch.cat([torch.zeros(shift, dtype=torch.uint8), torch.from_numpy(state)]).cuda()[shift:]
    assert shift == 0 or dev.prio.data_ptr() % 16 != 0 or dev.state.data_ptr() % 16 != 0
    dev.victims = torch.full((max(len(prio), 1),), -1, dtype=torch.int64, device="cuda")
    dev.ws = torch.full((max(kvm.kvm_workspace_bytes(kvm.OP_SELECT, len(prio)), 256),), 0x7F, dtype=torch.uint8,
                         device="cuda")
    got = dev.select(k=k, budget=budget, cap=cap)
    want = oracle.select_victims(prio, state, k=k, budget_units=budget, victims_cap=cap)
    np.testing.assert_array_equal(got, want)
    return got


@pytest.mark.parametrize("n", [1, 63, 4096, 4097, 100_000, 1_500_000])
@pytest.mark.parametrize("levels", [None, 7])
def test_select_matches_oracle_on_identical_keys(oracle, n, levels):
    rng = np.random.default_rng(n + (levels or 0))
    prio = (rng.random(n) ** 4).astype(np.float32)          # skewed, many small values
    if levels:
        prio = (np.floor(prio * levels) / levels).astype(np.float32)
    state = rng.choice(np.array([0, RES, RES | SCORED, RES | SCORED | PROT, HOST | SCORED, RES | SCORED,
                                 RES | SCORED], np.uint8), size=n)
    dev = DeviceCase(synth.tiny_gqa(1))
    n_el = int(np.sum((state & (RES | PROT | SCORED)) == (RES | SCORED)))
    n_res = int(np.sum((state & RES) != 0))
    for k in sorted({0, 1, n_el // 3, max(n_el - 1, 0), n_el, n_el + 5}):
        select_both(oracle, dev, prio, state, k=k)
    select_both(oracle, dev, prio, state, k=-1, budget=int(0.6 * n_res))
    select_both(oracle, dev, prio, state, k=-1, budget=n_res + 3)
    select_both(oracle, dev, prio, state, k=n_el, cap=min(5, n))


@pytest.mark.parametrize("n", [4097, 300_000])
@pytest.mark.parametrize("shift", [1, 3, 4])
def test_select_arrays_without_vector_alignment(oracle, n, shift):
    # the emit kernel fetches 16-byte vectors only from aligned arrays; these take its element-wise path
    rng = np.random.default_rng(n + shift)
    prio = (np.floor(rng.random(n) ** 4 * 50) / 50).astype(np.float32)
    state = rng.choice(np.array([RES | SCORED, RES | SCORED, HOST | SCORED, RES | SCORED | PROT], np.uint8), size=n)
    dev = DeviceCase(synth.tiny_gqa(1))
    for k in (1, 37, n // 5):
        select_both(oracle, dev, prio, state, k=k, shift=shift)


def test_select_few_victims_among_many_units(oracle):
    # k far below the number of chunks: most chunks of the emit pass hold nothing to write, and the ties of
    # the threshold value (a seventh of the units) that are still wanted end in the first chunks
    n = 1_200_000
    rng = np.random.default_rng(12)
    prio = (np.floor(rng.random(n) * 7) / 7 + 0.5).astype(np.float32)
    lows = rng.choice(n, size=150, replace=False)
    prio[lows] = rng.random(150).astype(np.float32) * 0.4
    state = np.full(n, RES | SCORED, np.uint8)
    state[rng.choice(n, size=n // 10, replace=False)] = HOST | SCORED
    dev = DeviceCase(synth.tiny_gqa(1))
    for k in (3, 150, 151, 190, 4000):
        got = select_both(oracle, dev, prio, state, k=k)
        assert len(got) == k


def test_select_special_values(oracle):
    prio = np.array([np.nan, 0.5, np.inf, -0.0, 0.0, 0.1, 1e-45, 3e38, 0.1], np.float32)
    state = np.full(len(prio), RES | SCORED, np.uint8)
    dev = DeviceCase(synth.tiny_gqa(1))
    for k in range(len(prio) + 1):
        select_both(oracle, dev, prio, state, k=k)
    select_both(oracle, dev, np.zeros(0, np.float32), np.zeros(0, np.uint8), k=3)
    same = np.full(10000, 0.25, np.float32)
    got = select_both(oracle, dev, same, np.full(10000, RES | SCORED, np.uint8), k=4500)
    np.testing.assert_array_equal(got, np.arange(4500))


# --------------------------------------------------------------- pack / unpack
@pytest.mark.parametrize("direct", [False, True])
@pytest.mark.parametrize("shape", [
    synth.Shape(2, 8, 2, 128, synth.BF16, True, [300, 77]),
    synth.Shape(1, 4, 2, 64, synth.FP16, True, [512]),
    synth.Shape(2, 16, 1, 576, synth.BF16, False, [200]),      # latent units, no V
])
def test_pack_unpack_bytes_and_tables(oracle, shape, direct):
    case = synth.make_case(shape, seed=7, spare_slots=11)
    dev = DeviceCase(case, staging_records=5)            # forces several staging chunks
    k8, v8 = host_pools(case)
    rng = np.random.default_rng(3)
    res = np.nonzero(case.state & RES)[0]
    uids = rng.choice(res, size=min(37, len(res)), replace=False).astype(np.int64)
    uids = np.r_[uids, [-4, case.n_uids + 2]].astype(np.int64)       # two malformed entries
    host = (500 + np.arange(len(uids))).astype(np.int32)
    tbl, st = case.slot_tbl.copy(), case.state.copy()
    bad = np.zeros(1, np.uint32)
    want_staging, want_freed = oracle.pack(k8, v8, shape.unit_k_bytes, shape.unit_v_bytes, tbl, st, uids, host,
                                           n_bad=bad)
    got_staging, got_freed = dev.pack(uids, host, direct=direct)
    np.testing.assert_array_equal(got_freed, want_freed)
    ok = want_freed >= 0
    np.testing.assert_array_equal(got_staging[ok], want_staging[ok])
    np.testing.assert_array_equal(dev.slot_tbl.cpu().numpy(), tbl)
    np.testing.assert_array_equal(dev.state.cpu().numpy(), st)
    assert int(dev.n_bad.item()) == int(bad[0]) == 2

    # bring them back into rotated frames, after the frames were overwritten
    good = uids[ok]
    dst = np.roll(want_freed[ok], 5).astype(np.int32)
    junk = torch.full_like(dev.k_pool[0], 0x5A5A)
    for s in want_freed[ok]:
        dev.k_pool[int(s)] = junk
        k8[s] = 0x5A
    oracle.unpack(k8, v8, shape.unit_k_bytes, shape.unit_v_bytes, tbl, st, good, dst, want_staging[ok])
    dev.unpack(good, dst, got_staging[ok], direct=direct)
    gk, gv = dev.pools_host()
    np.testing.assert_array_equal(gk, k8)
    if v8 is not None:
        np.testing.assert_array_equal(gv, v8)
    np.testing.assert_array_equal(dev.slot_tbl.cpu().numpy(), tbl)
    np.testing.assert_array_equal(dev.state.cpu().numpy(), st)


def test_pack_unpack_split_phases_with_caller_copies(oracle):
    """Gather-only pack (records stay in device staging) + the caller's own copy on a side stream,
    then the caller's copy back + scatter-only unpack: same bytes and tables as the oracle."""
    from paper_2604_26968_amd import kvm
    shape = synth.Shape(2, 8, 2, 128, synth.BF16, True, [400, 90])
    case = synth.make_case(shape, seed=17, spare_slots=3)
    dev = DeviceCase(case)
    k8, v8 = host_pools(case)
    rng = np.random.default_rng(5)
    uids = rng.choice(np.nonzero(case.state & RES)[0], size=50, replace=False).astype(np.int64)
    hs = np.arange(50, dtype=np.int32)
    tbl, st = case.slot_tbl.copy(), case.state.copy()
    want, want_freed = oracle.pack(k8, v8, shape.unit_k_bytes, shape.unit_v_bytes, tbl, st, uids, hs)
    rec = dev.rec
    d_uids, d_hs = torch.from_numpy(uids).cuda(), torch.from_numpy(hs).cuda()
    freed = torch.full((50,), -1, dtype=torch.int32, device="cuda")
    sdev = torch.zeros(50 * rec, dtype=torch.uint8, device="cuda")
    host = torch.zeros(50 * rec, dtype=torch.uint8, pin_memory=True)
    side = torch.cuda.Stream()
    done = torch.cuda.Event()
    kvm.kvm_pack(dev.pool, dev.slot_tbl, dev.state, d_uids, 50, d_hs, freed, sdev, None, n_bad=dev.n_bad)
    done.record()
    with torch.cuda.stream(side):
        side.wait_event(done)
        host.copy_(sdev, non_blocking=True)
    side.synchronize()
    np.testing.assert_array_equal(host.numpy().reshape(50, rec), want)
    np.testing.assert_array_equal(freed.cpu().numpy(), want_freed)
    np.testing.assert_array_equal(dev.state.cpu().numpy(), st)
    # too small a device staging buffer is refused when there is no host buffer
    with pytest.raises(kvm.KvmError) as e:
        kvm.kvm_pack(dev.pool, dev.slot_tbl, dev.state, d_uids, 50, d_hs, freed, sdev[:10 * rec], None)
    assert e.value.code == kvm.ENOSPC
    # back: caller copies host -> device staging, library scatters
    dst = np.roll(want_freed, 7).astype(np.int32)
    sdev.zero_()
    with torch.cuda.stream(side):
        sdev.copy_(host, non_blocking=True)
        done.record(side)
    torch.cuda.current_stream().wait_event(done)
    kvm.kvm_unpack(dev.pool, dev.slot_tbl, dev.state, d_uids, 50, torch.from_numpy(dst).cuda(), sdev, None,
                   n_bad=dev.n_bad)
    torch.cuda.synchronize()
    oracle.unpack(k8, v8, shape.unit_k_bytes, shape.unit_v_bytes, tbl, st, uids, dst, want)
    gk, gv = dev.pools_host()
    np.testing.assert_array_equal(gk, k8)
    np.testing.assert_array_equal(gv, v8)
    np.testing.assert_array_equal(dev.slot_tbl.cpu().numpy(), tbl)
    assert int(dev.n_bad.item()) == 0


@pytest.mark.parametrize("shape", [
    synth.Shape(2, 8, 2, 128, synth.BF16, True, [300, 77]),
    synth.Shape(4, 16, 1, 576, synth.BF16, False, [400]),
])
def test_swap_equals_pack_then_unpack(oracle, shape):
    """The fused call leaves tables, pools and host records exactly as the oracle's pack followed
    by unpack into the freed frames, including skipped entries."""
    from paper_2604_26968_amd import kvm
    case = synth.make_case(shape, seed=23)
    out_first = evict_some(case, 0.3, 4)                        # these live on the host already
    dev = DeviceCase(case)
    k8, v8 = host_pools(case)
    rng = np.random.default_rng(6)
    n = 20
    res = np.nonzero(case.state & RES)[0]
    out_uids = rng.choice(res, size=n, replace=False).astype(np.int64)
    in_uids = rng.choice(out_first, size=n, replace=False).astype(np.int64)
    out_uids[3] = -1                     # malformed victim: its partner cannot come in either
    in_uids[7] = res[0] if res[0] not in out_uids else res[1]   # already resident: frame 7 stays free
    hs = (900 + np.arange(n)).astype(np.int32)
    rec = dev.rec
    host_in = rng.integers(0, 256, size=(n, rec), dtype=np.uint8)
    tbl, st = case.slot_tbl.copy(), case.state.copy()
    bad = np.zeros(1, np.uint32)
    want_out, want_freed = oracle.pack(k8, v8, shape.unit_k_bytes, shape.unit_v_bytes, tbl, st, out_uids, hs, n_bad=bad)
    oracle.unpack(k8, v8, shape.unit_k_bytes, shape.unit_v_bytes, tbl, st, in_uids, want_freed, host_in, n_bad=bad)
    h_out = torch.zeros(n * rec, dtype=torch.uint8, pin_memory=True)
    h_in = torch.from_numpy(host_in.reshape(-1).copy()).pin_memory()
    freed = torch.full((n,), -7, dtype=torch.int32, device="cuda")
    kvm.kvm_swap(dev.pool, dev.slot_tbl, dev.state, torch.from_numpy(out_uids).cuda(), torch.from_numpy(in_uids).cuda(),
                 n, torch.from_numpy(hs).cuda(), freed, h_out, h_in, n_bad=dev.n_bad)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(freed.cpu().numpy(), want_freed)
    ok = want_freed >= 0
    np.testing.assert_array_equal(h_out.numpy().reshape(n, rec)[ok], want_out[ok])
    gk, gv = dev.pools_host()
    np.testing.assert_array_equal(gk, k8)
    if v8 is not None:
        np.testing.assert_array_equal(gv, v8)
    np.testing.assert_array_equal(dev.slot_tbl.cpu().numpy(), tbl)
    np.testing.assert_array_equal(dev.state.cpu().numpy(), st)
    assert int(dev.n_bad.item()) == int(bad[0]) == 3


def test_pack_unpack_round_trip_is_identity():
    case = synth.make_case(synth.Shape(2, 8, 2, 128, synth.BF16, True, [1000]), seed=2)
    dev = DeviceCase(case)
    k0, v0 = dev.pools_host()
    uids = np.nonzero(case.state & RES)[0][::3].astype(np.int64)
    staging, freed = dev.pack(uids, np.arange(len(uids), dtype=np.int32))
    assert np.all(dev.slot_tbl.cpu().numpy()[uids] == -1 - np.arange(len(uids)))
    dev.unpack(uids, freed, staging)
    k1, v1 = dev.pools_host()
    np.testing.assert_array_equal(k0, k1)
    np.testing.assert_array_equal(v0, v1)
    np.testing.assert_array_equal(dev.slot_tbl.cpu().numpy(), case.slot_tbl)
    np.testing.assert_array_equal(dev.state.cpu().numpy(), case.state)


# ----------------------------------------------------------------- end to end
def victims_agree(got, want, prio_ref, state_ref, rtol=2e-3):
    """Same size; any unit in one set only must have an oracle priority within rtol of the cutoff."""
    assert len(got) == len(want)
    diff = np.setxor1d(got, want)
    if len(diff) == 0 or len(want) == 0:
        return
    cutoff = np.max(prio_ref[want])
    assert np.all(np.abs(prio_ref[diff] - cutoff) <= rtol * cutoff), (diff, prio_ref[diff], cutoff)


def test_end_to_end_tiny_config(oracle):
    """Config 1: 8 decode steps of beta -> score -> ema, then evict 8 units, pack, unpack, compare pools."""
    case = synth.tiny_gqa(1)
    dev = DeviceCase(case)
    k0, v0 = dev.pools_host()
    S, prio = np.zeros(case.n_uids, np.float32), np.zeros(case.n_uids, np.float32)
    hits, misses = np.zeros(16, np.uint32), np.zeros(16, np.uint32)
    for step in range(8):
        q = synth.make_queries(case, 2 + step)
        ev = synth.make_events(25, 300 + step)
        o = run_step_oracle(oracle, case, q, ev, S, prio, hits, misses, scale=1 / 8, decay=0.9,
                            k=8 if step == 7 else 0)
        # both sides move the oracle's victim list, so the staging bytes are compared whatever the GPU selected
        g = run_step_gpu(dev, q, ev, scale=1 / 8, decay=0.9, k=8 if step == 7 else 0, pack_uids=o["victims"])
        np.testing.assert_array_equal(g["hits"], o["hits"])
        np.testing.assert_array_equal(g["misses"], o["misses"])
        np.testing.assert_allclose(g["p_hat"], o["p_hat"], rtol=1e-6)
        np.testing.assert_allclose(g["mass"], o["mass"], rtol=MASS_RTOL, atol=MASS_ATOL)
        np.testing.assert_allclose(g["S"], o["S"], rtol=MASS_RTOL)
        np.testing.assert_allclose(g["prio"], o["prio"], rtol=MASS_RTOL)
        victims_agree(g["victims"], o["victims"], o["prio"], case.state)
    assert len(g["victims"]) == 8 and len(o["victims"]) == 8
    np.testing.assert_array_equal(g["staging"], o["staging"])
    np.testing.assert_array_equal(g["freed"], o["freed"])
    k1, v1 = dev.pools_host()
    np.testing.assert_array_equal(k0, k1)
    np.testing.assert_array_equal(v0, v1)


def test_end_to_end_eviction_dynamics(oracle):
    """Twin of the Llama-3-8B-shaped workload: budget eviction every step, victims leave the pool,
    an equal number of host units comes back into the freed frames."""
    case = synth.make_case(synth.Shape(2, 8, 2, 128, synth.BF16, True, [700, 2100, 333]), seed=14,
                           pair_weights=synth.categorical_weights(3), spare_slots=0)
    dev = DeviceCase(case)
    sh = case.shape
    k8, v8 = host_pools(case)
    S, prio = np.zeros(case.n_uids, np.float32), np.zeros(case.n_uids, np.float32)
    hits, misses = np.zeros(16, np.uint32), np.zeros(16, np.uint32)
    n_res0 = int(np.sum(case.state & RES != 0))
    budget = int(0.6 * n_res0)
    host_store = {}                                   # uid -> record bytes (the host tier)
    rng = np.random.default_rng(0)
    w = synth.categorical_weights(8)
    for step in range(5):
        q = synth.make_queries(case, 50 + step)
        ev = synth.make_events(512, 400 + step, pair_weights=w, reuse_prob=np.linspace(0.2, 0.95, 16))
        gh, gm, gp = dev.beta(*ev)
        p_hat = oracle.beta_update(ev[0], ev[1], hits, misses)
        np.testing.assert_array_equal(gh, hits)
        gmass = dev.score(q, 1 / np.sqrt(128))
        omass = oracle_score(oracle, case, q, 1 / np.sqrt(128))
        res = (case.state & RES) != 0
        np.testing.assert_allclose(gmass[res], omass[res], rtol=MASS_RTOL, atol=MASS_ATOL)
        gS, gprio, gstate = dev.ema(0.95)
        oracle.ema_update(case.row_ntok, case.row_off, omass, 0.95, ref_row_weight(oracle, case), case.pair, p_hat,
                          case.state, S, prio)
        np.testing.assert_array_equal(gstate, case.state)
        np.testing.assert_allclose(gS[res], S[res], rtol=MASS_RTOL)
        gv = dev.select(k=-1, budget=budget)
        ov = oracle.select_victims(prio, case.state, k=-1, budget_units=budget)
        victims_agree(gv, ov, prio, case.state)
        assert len(ov) == (n_res0 - budget if step == 0 else n_back)
        # both sides evict the oracle's victim list so that the states stay comparable
        hs = np.arange(len(ov), dtype=np.int32) + 1000 * step
        ostag, ofreed = oracle.pack(k8, v8, sh.unit_k_bytes, sh.unit_v_bytes, case.slot_tbl, case.state, ov, hs)
        gstag, gfreed = dev.pack(ov, hs)
        np.testing.assert_array_equal(gstag, ostag)
        np.testing.assert_array_equal(gfreed, ofreed)
        for u, rec in zip(ov, ostag):
            host_store[int(u)] = rec.copy()
        # prefetch: a random sample of host units returns into the freed frames
        n_back = min(len(ofreed), 40)
        back = rng.choice(np.array(sorted(host_store)), size=n_back, replace=False).astype(np.int64)
        recs = np.stack([host_store.pop(int(u)) for u in back])
        dst = ofreed[:n_back].astype(np.int32)
        oracle.unpack(k8, v8, sh.unit_k_bytes, sh.unit_v_bytes, case.slot_tbl, case.state, back, dst, recs)
        dev.unpack(back, dst, recs)
        np.testing.assert_array_equal(dev.slot_tbl.cpu().numpy(), case.slot_tbl)
        np.testing.assert_array_equal(dev.state.cpu().numpy(), case.state)
        # the oracle scores from case.k_pool: keep it in step with the pool bytes after unpack
        case.k_pool[:] = k8.view(np.uint16).reshape(case.k_pool.shape)
    gk, gvv = dev.pools_host()
    resident_slots = case.slot_tbl[(case.state & RES) != 0]
    np.testing.assert_array_equal(gk[resident_slots], k8[resident_slots])
    np.testing.assert_array_equal(gvv[resident_slots], v8[resident_slots])


# ------------------------------------------------------------------- timing
def test_kernel_timing_counts_and_filter():
    """kvm_timing_* brackets launches with events while enabled; kvm_timing_only restricts it to one name."""
    from paper_2604_26968_amd import kvm
    buf = torch.zeros(1 << 22, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    kvm.kvm_timing_only(None)
    kvm.kvm_timing_reset()
    kvm.kvm_probe_read(buf, sink)                   # not enabled: not recorded
    kvm.kvm_timing_enable(True)
    try:
        kvm.kvm_probe_read(buf, sink)
        kvm.kvm_probe_read(buf, sink)
        kvm.kvm_timing_only("score_partial")
        kvm.kvm_probe_read(buf, sink)               # filtered out
        kvm.kvm_timing_only("probe_read")
        kvm.kvm_probe_read(buf, sink)
    finally:
        kvm.kvm_timing_enable(False)
        kvm.kvm_timing_only(None)
    torch.cuda.synchronize()
    cnt, ms = kvm.kvm_timing_read("probe_read")
    assert cnt == 3 and 0.0 < ms < 1000.0
    assert kvm.kvm_timing_read("score_partial")[0] == 0
    assert kvm.kvm_timing_read("no such kernel")[0] == 0
    kvm.kvm_timing_reset()
    assert kvm.kvm_timing_read("probe_read")[0] == 0


def test_overlapping_rows_beyond_the_tile_bound_score_nothing():
    """Rows must not overlap in uid space.  If a caller's rows do, and so much that their tiles exceed
    the bound the workspace is sized for (n_uids / tile + n_rows), the plan is refused on the device:
    no record is written past its array, nothing is scored, masses keep their old values."""
    from paper_2604_26968_amd import kvm
    case = synth.make_case(synth.Shape(1, 4, 1, 128, synth.BF16, True, [32768]), seed=77)
    dev = DeviceCase(case)
    copies = 50                                    # 50 rows over the same 2,048 units: 200 tiles > 2048 / 512 + 50
    ntok = torch.full((copies,), 32768, dtype=torch.int32, device="cuda")
    off = torch.zeros(copies, dtype=torch.int64, device="cuda")
    q_off = torch.zeros(copies, dtype=torch.int64, device="cuda")
    rows = kvm.make_rows(ntok, off, q_off, dev.slot_tbl, 4, 4 * 128)
    ws = torch.full((kvm.kvm_workspace_bytes(kvm.OP_SCORE, case.n_uids, copies, 4, 128),), 0x7F, dtype=torch.uint8,
                    device="cuda")
    q = torch.from_numpy(synth.make_queries(case, 3).view(np.int16)).cuda()
    dev.mass.fill_(-5.0)
    kvm.kvm_score_step(dev.pool, rows, q, 0.1, dev.mass, ws)
    torch.cuda.synchronize()
    assert bool((dev.mass == -5.0).all())
    # the same rows, few enough to stay inside the bound, are scored (each writes the same values)
    rows2 = kvm.make_rows(ntok[:1], off[:1], q_off[:1], dev.slot_tbl, 4, 4 * 128)
    kvm.kvm_score_step(dev.pool, rows2, q, 0.1, dev.mass, ws)
    torch.cuda.synchronize()
    assert bool((dev.mass >= 0).all())
