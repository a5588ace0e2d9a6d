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


# ------------------------------------------------------------------ frames shared by duplicates
RES, HOST, PROT, SCORED, SHARED = 1, 2, 4, 8, 16


class SharingModel:
    """Frame sharing written out with Python containers: who reads which frame, by content.  The frame of a
    unit is looked up in a dictionary, the readers of a frame are a set; nothing else."""

    def __init__(self, frame_of, flags):
        self.frame_of = dict(frame_of)                 # uid -> frame, units in HBM only
        self.flags = dict(flags)                       # uid -> set of flag names
        self.readers = {}
        for u, f in self.frame_of.items():
            self.readers.setdefault(f, set()).add(u)

    def share(self, u, c, n_uids):
        if not (0 <= u < n_uids and 0 <= c < n_uids):
            return "bad"
        if u == c or u not in self.frame_of or c not in self.frame_of:
            return None
        if "prot" in self.flags[u] or "shared" in self.flags[u] or "prot" in self.flags[c]:
            return None
        fu, fc = self.frame_of[u], self.frame_of[c]
        if fu == fc:
            return None
        self.readers[fu].discard(u)
        self.readers[fc].add(u)
        self.frame_of[u] = fc
        self.flags[u].add("shared")
        self.flags[c].add("shared")
        return fu

    def unshare(self, u, nf, n_uids, n_slots):
        if not (0 <= u < n_uids and 0 <= nf < n_slots):
            return "bad", nf
        if u not in self.frame_of or "shared" not in self.flags[u]:
            return None, nf
        f = self.frame_of[u]
        self.readers[f].discard(u)
        self.readers.setdefault(nf, set()).add(u)
        self.frame_of[u] = nf
        self.flags[u].discard("shared")
        return "moved", (f if not self.readers[f] else -1)


def sharing_case(seed, n_uids=60, n_slots=80, n_contents=9):
    rng = np.random.default_rng(seed)
    content = rng.integers(0, n_contents, size=n_uids)             # which content a unit holds
    in_hbm = rng.random(n_uids) < 0.8
    frames = rng.permutation(n_slots)[:n_uids].astype(np.int32)
    tbl = np.where(in_hbm, frames, -1 - np.arange(n_uids)).astype(np.int32)
    state = np.where(in_hbm, RES | SCORED, HOST).astype(np.uint8)
    state[rng.random(n_uids) < 0.1] |= PROT
    uk, uv = 64, 64
    k = np.zeros((n_slots, uk), np.uint8)
    v = np.zeros((n_slots, uv), np.uint8)
    for u in range(n_uids):
        if in_hbm[u]:
            k[tbl[u]] = content[u] * 3 + 1
            v[tbl[u]] = content[u] * 3 + 2
    # canonical copy of a content = its first unit (what the store reports in list order)
    first = {}
    canon = np.array([first.setdefault(int(c), u) for u, c in enumerate(content)], np.int64)
    return rng, content, tbl, state, k, v, uk, uv, canon


@pytest.mark.parametrize("seed", [1, 2, 3, 4])
def test_sharing_against_a_model_with_sets_of_readers(oracle, seed):
    rng, content, tbl, state, k, v, uk, uv, canon = sharing_case(seed)
    n_uids, n_slots = len(tbl), len(k)
    model = SharingModel({u: int(tbl[u]) for u in range(n_uids) if state[u] & RES},
                         {u: ({"prot"} if state[u] & PROT else set()) for u in range(n_uids)})
    refs = np.zeros(n_slots, np.uint32)
    uids = rng.permutation(n_uids).astype(np.int64)
    uids = np.r_[uids, [-3, n_uids + 5]].astype(np.int64)          # two malformed entries
    cn = np.r_[canon[uids[:-2]], [0, 1]].astype(np.int64)
    bad = np.zeros(1, np.uint32)
    freed = oracle.dedup_share(tbl, state, n_slots, uids, cn, refs, n_bad=bad)
    want = [model.share(int(u), int(c), n_uids) for u, c in zip(uids, cn)]
    assert bad[0] == 2 == sum(1 for w in want if w == "bad")
    np.testing.assert_array_equal(freed, [w if isinstance(w, int) else -1 for w in want])
    assert (freed >= 0).sum() > 5                                   # the case does share
    for u in range(n_uids):
        if state[u] & RES:
            assert tbl[u] == model.frame_of[u]
            assert bool(state[u] & SHARED) == ("shared" in model.flags[u])
            # what a unit reads is still its own content
            assert k[tbl[u], 0] == content[u] * 3 + 1 and v[tbl[u], 0] == content[u] * 3 + 2
    for f in range(n_slots):
        r = len(model.readers.get(f, ()))
        assert refs[f] == (r if r >= 2 else 0), (f, refs[f], r)
    # a frame given up is read by nobody; frames in use + frames given up = frames in use before
    in_use = {int(tbl[u]) for u in range(n_uids) if state[u] & RES}
    assert not in_use & set(int(f) for f in freed if f >= 0)
    # a second call with the same list changes nothing: the duplicates are SHARED already
    t2, s2, r2 = tbl.copy(), state.copy(), refs.copy()
    again = oracle.dedup_share(tbl, state, n_slots, uids[:-2], cn[:-2], refs)
    assert (again == -1).all() and (tbl == t2).all() and (state == s2).all() and (refs == r2).all()

    # ---- and back: every shared unit gets a frame of its own, in a random order
    free = [f for f in range(n_slots) if f not in in_use]
    shared = np.array([u for u in range(n_uids) if state[u] & SHARED], np.int64)
    rng.shuffle(shared)
    extra = np.array([u for u in range(n_uids) if not (state[u] & SHARED)][:3], np.int64)     # not shared: skipped
    lst = np.r_[shared, extra, [n_uids + 1]].astype(np.int64)
    assert len(free) >= len(lst)
    nf = np.array(free[:len(lst)], np.int32)
    bad[:] = 0
    got = oracle.dedup_unshare(k, v, uk, uv, tbl, state, lst, nf, refs, n_bad=bad)
    assert bad[0] == 1
    for i, (u, f_new) in enumerate(zip(lst, nf)):
        kind, f = model.unshare(int(u), int(f_new), n_uids, n_slots)
        assert got[i] == f, (i, kind, got[i], f)
    assert not (state & SHARED).any() and not refs.any()
    frames = [int(tbl[u]) for u in range(n_uids) if state[u] & RES]
    assert len(frames) == len(set(frames))                            # every unit has a frame of its own again
    for u in range(n_uids):
        if state[u] & RES:
            assert (k[tbl[u]] == content[u] * 3 + 1).all() and (v[tbl[u]] == content[u] * 3 + 2).all()
    # frames free afterwards: the ones that came back + the ones never handed out = all frames not in use
    back = set(int(f) for f in got if f >= 0) | set(free[len(lst):])
    assert back == set(range(n_slots)) - set(frames)


def test_shared_units_are_never_victims_and_cannot_be_packed(oracle):
    """A frame that several units read must not be handed out: the selection skips SHARED units even at the
    lowest priority, pack and the outgoing half of an exchange refuse them."""
    n = 12
    prio = np.arange(n, dtype=np.float32)
    state = np.full(n, RES | SCORED, np.uint8)
    state[[0, 1, 5]] |= SHARED
    got = oracle.select_victims(prio, state, k=4)
    np.testing.assert_array_equal(got, [2, 3, 4, 6])
    got = oracle.select_victims(prio, state, k=-1, budget_units=2)      # 12 in HBM, 9 may go: all that are eligible
    np.testing.assert_array_equal(got, [2, 3, 4, 6, 7, 8, 9, 10, 11])
    uk = uv = 64
    k = np.arange(n * uk, dtype=np.uint8).reshape(n, uk).copy()
    v = k[::-1].copy()
    tbl = np.arange(n, dtype=np.int32)
    tbl[1] = 0                                                            # units 0 and 1 read frame 0
    bad = np.zeros(1, np.uint32)
    staging, freed = oracle.pack(k, v, uk, uv, tbl, state, np.array([1, 2], np.int64), np.array([7, 8], np.int32), n_bad=bad)
    np.testing.assert_array_equal(freed, [-1, 2])
    assert bad[0] == 1 and tbl[1] == 0 and state[1] == RES | SCORED | SHARED and tbl[2] == -9
    tier = np.zeros((4, uk + uv), np.uint8)
    state[3], tbl[3] = HOST, -1 - 1                                        # unit 3 on the host in slot 1
    oracle.exchange(k, v, uk, uv, tbl, state, np.array([5], np.int64), np.array([3], np.int64), tier, n_bad=bad)
    assert bad[0] == 2 and tbl[5] == 5 and state[3] == HOST
