"""Pins for the scoring oracle (Eq. 1 summed per 16-token block, group max of
section 3.4): a torch CPU softmax over token-major K, closed forms, invariants."""
import numpy as np
import pytest
import torch

from paper_2604_26968_amd import synth

B = synth.BLOCK


def small_case(seed=5, lens=(70, 16, 33), L=2, hq=4, hkv=2, dim=32, dtype=synth.BF16, **kw):
    return synth.make_case(synth.Shape(L, hq, hkv, dim, dtype, True, list(lens)), seed, **kw)


def run(o, case, q, scale, agg=0, mass=None, want_q=True, row_active=None):
    if mass is None:
        mass = np.full(case.n_uids, -7.0, np.float32)
    mq = np.full(case.n_uids * case.shape.g, -7.0, np.float64) if want_q else None
    o.score_step(case.k_pool, case.shape.dim, case.shape.dtype, case.row_ntok, case.row_off,
                 case.row_q_off, case.slot_tbl, q, case.shape.g, scale, mass, agg=agg,
                 row_active=row_active, mass_q=mq)
    return mass, (mq.reshape(case.n_uids, case.shape.g) if want_q else None)


def torch_bits(bits, dtype):
    """Decode 16-bit patterns with torch (a library decoder independent of the oracle's)."""
    t = torch.from_numpy(bits.astype(np.uint16).view(np.int16).copy())
    return t.view(torch.bfloat16 if dtype == synth.BF16 else torch.float16).double()


def torch_reference(case, q, scale, agg=0):
    """softmax(K q * scale) with torch on token-major K, summed per block, group max/mean."""
    sh = case.shape
    out = np.full(case.n_uids, -7.0, np.float32)
    per_q = np.full((case.n_uids, sh.g), -7.0)
    for r in range(case.n_rows):
        n = int(case.row_ntok[r])
        nb = (n + B - 1) // B
        if n == 0:
            continue
        uids = case.row_off[r] + np.arange(nb)
        res = case.slot_tbl[uids] >= 0
        if not res.any():
            continue
        toks = []
        for b in np.nonzero(res)[0]:
            unit = case.k_pool[case.slot_tbl[uids[b]]]
            tm = synth.tokens_from_unit(unit, sh.dim)            # [16, dim] token-major
            toks.append(tm[: min(B, n - b * B)])
        K = torch_bits(np.concatenate(toks), sh.dtype)           # [n_res_tokens, dim]
        Q = torch_bits(q[case.row_q_off[r]: case.row_q_off[r] + sh.g * sh.dim], sh.dtype).reshape(sh.g, sh.dim)
        P = torch.softmax((K @ Q.T) * scale, dim=0)              # [tokens, g]
        pos = 0
        for b in np.nonzero(res)[0]:
            k = min(B, n - b * B)
            per_q[uids[b]] = P[pos:pos + k].sum(0).numpy()
            pos += k
        m = per_q[uids[res]]
        out[uids[res]] = (m.max(1) if agg == 0 else m.mean(1)).astype(np.float32)
    return out, per_q


def test_decoders_match_library_exhaustively(oracle):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    for dtype in (synth.BF16, synth.FP16):
        want = torch_bits(bits, dtype).numpy()
        got = np.array([oracle.decode(int(b), dtype) for b in bits])
        both_nan = np.isnan(want) & np.isnan(got)
        assert np.all((want == got) | both_nan)
        assert np.all(np.signbit(want) == np.signbit(got))


@pytest.mark.parametrize("dtype", [synth.BF16, synth.FP16])
@pytest.mark.parametrize("agg", [0, 1])
def test_matches_torch_softmax(oracle, dtype, agg):
    case = small_case(dtype=dtype, spare_slots=5, uid_gap=2)
    q = synth.make_queries(case, 9)
    scale = 1.0 / np.sqrt(case.shape.dim)
    got, got_q = run(oracle, case, q, scale, agg)
    want, want_q = torch_reference(case, q, scale, agg)
    np.testing.assert_allclose(got_q, want_q, rtol=1e-12, atol=1e-300)
    np.testing.assert_allclose(got, want, rtol=1e-7)
    assert np.all(got[case.state == 0] == -7.0)       # gaps between rows are never written


def test_g1_is_plain_softmax(oracle):
    case = small_case(hq=2, hkv=2, lens=(100,), L=1)
    q = synth.make_queries(case, 3)
    got, got_q = run(oracle, case, q, 0.3)
    want, _ = torch_reference(case, q, 0.3)
    np.testing.assert_allclose(got, want, rtol=1e-7)
    np.testing.assert_allclose(got, got_q[:, 0].astype(np.float32), rtol=0)


def test_per_query_masses_sum_to_one(oracle):
    case = small_case(lens=(257, 40))
    q = synth.make_queries(case, 4, scale=3.0)
    mass, mq = run(oracle, case, q, 0.5)
    for r in range(case.n_rows):
        nb = (case.row_ntok[r] + B - 1) // B
        sl = slice(case.row_off[r], case.row_off[r] + nb)
        np.testing.assert_allclose(mq[sl].sum(0), 1.0, rtol=1e-12)
        # the group maximum sums to something in [1, g]
        assert 1.0 - 1e-6 <= mass[sl].sum() <= case.shape.g + 1e-6
    mean, _ = run(oracle, case, q, 0.5, agg=1)
    for r in range(case.n_rows):
        nb = (case.row_ntok[r] + B - 1) // B
        assert abs(mean[case.row_off[r]: case.row_off[r] + nb].sum() - 1.0) < 1e-5


def test_zero_query_gives_token_fractions(oracle):
    case = small_case(lens=(70, 16, 33, 5))
    q = np.zeros(case.n_rows * case.shape.g * case.shape.dim, np.uint16)
    mass, _ = run(oracle, case, q, 1.0)
    for r in range(case.n_rows):
        n = int(case.row_ntok[r])
        nb = (n + B - 1) // B
        want = np.array([min(B, n - b * B) / n for b in range(nb)], np.float32)
        np.testing.assert_array_equal(mass[case.row_off[r]: case.row_off[r] + nb], want)


def test_identical_keys_give_token_fractions(oracle):
    case = small_case(lens=(45,), L=1)
    tok = synth.to_bits(np.random.default_rng(0).standard_normal(case.shape.dim).astype(np.float32),
                        case.shape.dtype)
    unit = synth.unit_from_tokens(np.tile(tok, (B, 1)))
    case.k_pool[:] = unit
    q = synth.make_queries(case, 8)
    mass, _ = run(oracle, case, q, 0.7)
    want = np.array([16 / 45, 16 / 45, 13 / 45], np.float32)
    for r in range(case.n_rows):
        np.testing.assert_allclose(mass[case.row_off[r]: case.row_off[r] + 3], want, rtol=1e-7)


def test_slot_permutation_leaves_masses_bit_identical(oracle):
    case = small_case(lens=(90, 31), spare_slots=7)
    q = synth.make_queries(case, 6)
    base, base_q = run(oracle, case, q, 0.2)
    rng = np.random.default_rng(1)
    perm = rng.permutation(case.n_slots)
    moved = np.empty_like(case.k_pool)
    moved[perm] = case.k_pool                      # old slot s now lives in perm[s]
    tbl = case.slot_tbl.copy()
    tbl[tbl >= 0] = perm[tbl[tbl >= 0]]
    case.k_pool, case.slot_tbl = moved, tbl.astype(np.int32)
    again, again_q = run(oracle, case, q, 0.2)
    np.testing.assert_array_equal(base, again)
    np.testing.assert_array_equal(base_q, again_q)


def test_block_order_permutation_permutes_masses(oracle):
    case = small_case(lens=(64,), L=1, hq=2, hkv=1)       # 4 full blocks, one row
    q = synth.make_queries(case, 2)
    base, _ = run(oracle, case, q, 0.4)
    order = np.array([2, 0, 3, 1])
    case.slot_tbl[:4] = case.slot_tbl[:4][order]
    again, _ = run(oracle, case, q, 0.4)
    np.testing.assert_allclose(again[:4], base[:4][order], rtol=1e-6)


def test_dominant_token_takes_all_mass(oracle):
    case = small_case(lens=(80,), L=1, hq=1, hkv=1)
    dim = case.shape.dim
    qf = np.random.default_rng(3).standard_normal(dim).astype(np.float32)
    q = synth.to_bits(qf, case.shape.dtype)
    # token 37 (block 2, position 5) is 40 * q: its logit exceeds all others by far
    slot = case.slot_tbl[case.row_off[0] + 2]
    toks = synth.tokens_from_unit(case.k_pool[slot], dim)
    toks[5] = synth.to_bits(40.0 * qf, case.shape.dtype)
    case.k_pool[slot] = synth.unit_from_tokens(toks)
    mass, _ = run(oracle, case, q, 1.0)
    assert mass[2] > 1.0 - 1e-6 and np.all(mass[[0, 1, 3, 4]] < 1e-6)


def test_nonresident_block_equals_deleted_block(oracle):
    case = small_case(lens=(64,), L=1, hq=2, hkv=1)
    q = synth.make_queries(case, 12)
    full, _ = run(oracle, case, q, 0.3)
    # evict block 1: masses of the rest must equal those of the 3-block row without it
    case.slot_tbl[1] = -1 - 99
    part, _ = run(oracle, case, q, 0.3)
    assert part[1] == -7.0
    short = small_case(lens=(48,), L=1, hq=2, hkv=1)
    short.k_pool, short.n_slots = case.k_pool, case.n_slots
    short.slot_tbl[:3] = np.array([case.slot_tbl[0], case.slot_tbl[2], case.slot_tbl[3]])
    ref, _ = run(oracle, short, q, 0.3)
    np.testing.assert_array_equal(part[[0, 2, 3]], ref[:3])
    assert not np.allclose(part[[0, 2, 3]], full[[0, 2, 3]])


def test_tail_tokens_are_never_read(oracle):
    clean = small_case(lens=(37, 50))
    dirty = small_case(lens=(37, 50), poison_tail=True)
    assert not np.array_equal(clean.k_pool, dirty.k_pool)
    q = synth.make_queries(clean, 1)
    a, _ = run(oracle, clean, q, 0.25)
    b, _ = run(oracle, dirty, q, 0.25)
    np.testing.assert_array_equal(a, b)
    assert np.all(np.isfinite(b[dirty.state != 0]))


def test_inactive_and_empty_rows_untouched(oracle):
    case = small_case(lens=(40, 0, 20))
    q = synth.make_queries(case, 1)
    active = np.ones(case.n_rows, np.uint8)
    active[0] = 0
    mass, _ = run(oracle, case, q, 0.25, row_active=active)
    nb0 = 3
    assert np.all(mass[case.row_off[0]: case.row_off[0] + nb0] == -7.0)
    assert np.all(mass[case.row_off[1]: case.row_off[1] + nb0] != -7.0)
