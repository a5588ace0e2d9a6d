"""Pins for content addressing (section 3.6): SHA-256 against the digests published with the
standard and against hashlib around every padding boundary; unit hashing against hashlib over
numpy-gathered records; the store against a Python dictionary."""
import hashlib
import os

import numpy as np
import pytest

from paper_2604_26968_amd import synth

RES, HOST, PROT, SCORED = 1, 2, 4, 8
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "sha256_vectors.txt")


def golden_vectors():
    out = []
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        spec, digest = line.rstrip("\n").split("\t")
        if spec == "empty":
            msg = b""
        elif spec.startswith("ascii:"):
            msg = spec[6:].encode()
        else:
            _, ch, cnt = spec.split(":")
            msg = ch.encode() * int(cnt)
        out.append((msg, digest))
    return out


def test_published_digests(oracle):
    vec = golden_vectors()
    assert len(vec) == 4
    for msg, digest in vec:
        assert oracle.sha256(msg).hex() == digest


def test_every_length_around_the_padding_boundaries_against_hashlib(oracle):
    rng = np.random.default_rng(0)
    for n in list(range(0, 200)) + [255, 256, 257, 4095, 4096, 8191, 8192, 8193, 18432]:
        msg = rng.integers(0, 256, n, dtype=np.uint8).tobytes()
        assert oracle.sha256(msg) == hashlib.sha256(msg).digest(), n


def pools(case):
    k8 = case.k_pool.view(np.uint8).reshape(case.n_slots, -1).copy()
    v8 = case.v_pool.view(np.uint8).reshape(case.n_slots, -1).copy() if case.v_pool is not None else None
    return k8, v8


@pytest.mark.parametrize("latent", [False, True])
def test_unit_digest_is_sha256_of_k_frame_then_v_frame(oracle, latent):
    shape = synth.Shape(2, 4, 1, 576, synth.BF16, False, [100]) if latent else \
        synth.Shape(2, 4, 2, 64, synth.FP16, True, [70, 33])
    case = synth.make_case(shape, 3)
    k8, v8 = pools(case)
    st = case.state.copy()
    st[5] = HOST                                   # not in HBM: zero digest
    uids = np.array([0, 5, 7, case.n_uids, -1, 2], np.int64)
    bad = np.zeros(1, np.uint32)
    d = oracle.hash_units(k8, v8, shape.unit_k_bytes, shape.unit_v_bytes, case.slot_tbl, st, uids, n_bad=bad)
    assert bad[0] == 3
    for i, u in enumerate(uids):
        if u in (0, 7, 2):
            slot = case.slot_tbl[u]
            rec = k8[slot].tobytes() + (v8[slot].tobytes() if v8 is not None else b"")
            assert d[i].tobytes() == hashlib.sha256(rec).digest()
        else:
            assert not d[i].any()


def test_store_against_a_dictionary(oracle):
    rng = np.random.default_rng(1)
    contents = [rng.integers(0, 256, 32, dtype=np.uint8) for _ in range(40)]      # 40 distinct digests
    store = oracle.DedupStore(64)
    ref = {}
    next_uid = 100
    for call in range(5):
        n = int(rng.integers(1, 60))
        pick = rng.integers(0, 40, n)
        digests = np.stack([contents[p] for p in pick])
        uids = np.arange(next_uid, next_uid + n, dtype=np.int64)
        next_uid += n
        canon = store.insert(digests, uids)
        for i in range(n):
            key = digests[i].tobytes()
            if key not in ref or ref[key][1] == 0:
                ref[key] = [int(uids[i]), 1]
            else:
                ref[key][1] += 1
            assert canon[i] == ref[key][0]
        assert store.as_dict() == {k: tuple(v) for k, v in ref.items()}
        # release a few references, some of them unknown or already at zero
        rel = rng.integers(0, 40, 15)
        rd = np.stack([contents[p] for p in rel] + [np.full(32, 255, np.uint8)])
        bad = np.zeros(1, np.uint32)
        store.release(rd, n_bad=bad)
        want_bad = 1
        for p in rel:
            key = contents[p].tobytes()
            if key in ref and ref[key][1] > 0:
                ref[key][1] -= 1
            else:
                want_bad += 1
        assert bad[0] == want_bad
        assert store.as_dict() == {k: tuple(v) for k, v in ref.items()}


def test_first_occurrence_is_canonical_and_duplicates_point_to_it(oracle):
    store = oracle.DedupStore(8)
    a, b = np.full(32, 1, np.uint8), np.full(32, 2, np.uint8)
    canon = store.insert(np.stack([a, b, a, a, b]), np.array([10, 11, 12, 13, 14], np.int64))
    np.testing.assert_array_equal(canon, [10, 11, 10, 10, 11])
    assert store.as_dict() == {a.tobytes(): (10, 3), b.tobytes(): (11, 2)}
    store.release(np.stack([a, a, a]))
    canon = store.insert(np.stack([a]), np.array([99], np.int64))          # revived: new canonical copy
    assert canon[0] == 99 and store.as_dict()[a.tobytes()] == (99, 1)
    with pytest.raises(oracle.OracleError):                                 # list full
        store.insert(np.arange(32 * 8, dtype=np.uint8).reshape(8, 32), np.arange(8, dtype=np.int64))
