"""Pins for the pack / unpack oracle (tier 0 <-> tier 1 moves of section 3.2):
numpy fancy indexing as the gather, round-trip identities, table transitions."""
import numpy as np

from paper_2604_26968_amd import synth

RES, HOST, PROT, SCORED = 1, 2, 4, 8


def pools(case):
    k8 = case.k_pool.view(np.uint8).reshape(case.n_slots, -1).copy()
    v8 = case.v_pool.view(np.uint8).reshape(case.n_slots, -1).copy() if case.v_pool is not None else None
    return k8, v8


def test_pack_is_a_gather_and_updates_tables(oracle):
    case = synth.make_case(synth.Shape(2, 4, 2, 32, synth.BF16, True, [70, 33]), 3, spare_slots=4)
    k8, v8 = pools(case)
    rng = np.random.default_rng(0)
    uids = rng.choice(np.nonzero(case.state & RES)[0], size=11, replace=False).astype(np.int64)
    host = (1000 + np.arange(11)).astype(np.int32)
    tbl, st = case.slot_tbl.copy(), case.state.copy()
    staging, freed = oracle.pack(k8, v8, 1024, 1024, tbl, st, uids, host)
    slots = case.slot_tbl[uids]
    np.testing.assert_array_equal(freed, slots)
    np.testing.assert_array_equal(staging[:, :1024], k8[slots])
    np.testing.assert_array_equal(staging[:, 1024:], v8[slots])
    np.testing.assert_array_equal(tbl[uids], -1 - host)
    assert np.all((st[uids] & RES) == 0) and np.all((st[uids] & HOST) != 0)
    assert np.all((st[uids] & PROT) == (case.state[uids] & PROT))
    rest = np.setdiff1d(np.arange(case.n_uids), uids)
    np.testing.assert_array_equal(tbl[rest], case.slot_tbl[rest])
    np.testing.assert_array_equal(st[rest], case.state[rest])


def test_round_trip_same_slots_is_identity_and_permuted_slots_permute(oracle):
    case = synth.make_case(synth.Shape(1, 2, 2, 64, synth.FP16, True, [200]), 5)
    k8, v8 = pools(case)
    k0, v0 = k8.copy(), v8.copy()
    uids = np.nonzero(case.state & RES)[0][::2].astype(np.int64)
    host = np.arange(len(uids), dtype=np.int32)
    tbl, st = case.slot_tbl.copy(), case.state.copy()
    staging, freed = oracle.pack(k8, v8, 2048, 2048, tbl, st, uids, host)
    k8[freed] = 0xAB                                   # the frames are reused by someone else meanwhile
    v8[freed] = 0xCD
    oracle.unpack(k8, v8, 2048, 2048, tbl, st, uids, freed, staging)
    np.testing.assert_array_equal(k8, k0)
    np.testing.assert_array_equal(v8, v0)
    np.testing.assert_array_equal(tbl, case.slot_tbl)
    np.testing.assert_array_equal(st, case.state)
    # second trip into rotated frames: contents follow the table
    staging, freed = oracle.pack(k8, v8, 2048, 2048, tbl, st, uids, host)
    dst = np.roll(freed, 3)
    oracle.unpack(k8, v8, 2048, 2048, tbl, st, uids, dst, staging)
    np.testing.assert_array_equal(tbl[uids], dst)
    np.testing.assert_array_equal(k8[tbl[uids]], k0[case.slot_tbl[uids]])
    np.testing.assert_array_equal(v8[tbl[uids]], v0[case.slot_tbl[uids]])


def test_latent_units_have_no_v(oracle):
    case = synth.make_case(synth.Shape(1, 4, 1, 64, synth.BF16, False, [48]), 2)
    k8, _ = pools(case)
    uids = np.array([2, 0], np.int64)
    tbl, st = case.slot_tbl.copy(), case.state.copy()
    staging, freed = oracle.pack(k8, None, 2048, 0, tbl, st, uids, np.array([7, 8], np.int32))
    assert staging.shape == (2, 2048)
    np.testing.assert_array_equal(staging, k8[case.slot_tbl[uids]])


def test_bad_entries_are_skipped_and_counted(oracle):
    case = synth.make_case(synth.Shape(1, 2, 2, 32, synth.BF16, True, [64]), 9)
    k8, v8 = pools(case)
    tbl, st = case.slot_tbl.copy(), case.state.copy()
    st[1] = HOST | SCORED
    tbl[1] = -5
    uids = np.array([0, 1, -3, case.n_uids, 2], np.int64)
    bad = np.zeros(1, np.uint32)
    staging, freed = oracle.pack(k8, v8, 1024, 1024, tbl, st, uids, np.arange(5, dtype=np.int32), n_bad=bad)
    assert bad[0] == 3
    np.testing.assert_array_equal(freed, [case.slot_tbl[0], -1, -1, -1, case.slot_tbl[2]])
    assert np.all(staging[1:4] == 0)
    np.testing.assert_array_equal(staging[4, :1024], k8[case.slot_tbl[2]])
    # unpack refuses resident uids and frames outside the pool
    bad[:] = 0
    k_before = k8.copy()
    oracle.unpack(k8, v8, 1024, 1024, tbl, st, np.array([3, 0], np.int64),
                  np.array([0, case.n_slots], np.int32), staging[:2], n_bad=bad)
    assert bad[0] == 2
    np.testing.assert_array_equal(k8, k_before)
