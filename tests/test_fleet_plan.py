"""Host logic of the trace-driven workloads (no GPU): the seeded request generator and the replay that turns a
trace into per-step arrays.  The replay decides nothing the method computes; what is checked here is that the
arrays it hands to both the library and the oracle describe one consistent history."""
import numpy as np
import pytest

from paper_2604_26968_amd import fleet, synth

BLOCK = synth.BLOCK


def small_fleet(seed=90, n_requests=260, rate=0.3, start=350, n_steps=14):
    shapes = [synth.Shape(2, 4, 4, 128, synth.BF16, True, []), synth.Shape(2, 32, 1, 128, synth.BF16, True, [])]
    cats = [synth.fleet_catalogue(8, seed), synth.fleet_catalogue(8, seed + 1)]
    reqs = synth.fleet_requests(n_requests, seed + 2, rate, 8, cats, mean_decode=20, mean_gap=30, mu=5.5, hi=4096)
    plan = fleet.build_plan(shapes, cats, reqs, start, n_steps, capacity_units=12000, max_tokens=4096)
    return shapes, cats, reqs, plan


def test_trace_generator_follows_its_recipe():
    cats = [synth.fleet_catalogue(64, 11), synth.fleet_catalogue(64, 12)]
    reqs = synth.fleet_requests(20000, 13, 0.5, 64, cats)
    arr = np.array([r.arrival for r in reqs])
    assert (np.diff(arr) >= 0).all()
    assert abs(arr[-1] / len(reqs) - 2.0) < 0.1                      # Poisson arrivals, 0.5 per step
    assert abs(np.mean([r.model for r in reqs]) - 0.5) < 0.02
    lens = np.array([r.prompt_len for r in reqs])
    assert lens.min() >= 16 and lens.max() <= 32768
    inner = lens[(lens > 16) & (lens < 32768)]
    assert abs(np.log(inner).mean() - 7.0) < 0.05 and abs(np.log(inner).std() - 1.0) < 0.05   # lognormal(7, 1)
    # prefix ids: Zipf(1.1) over 64 ranks
    counts = np.bincount([r.prefix for r in reqs], minlength=64).astype(float)
    want = np.arange(1, 65) ** -1.1
    want = want / want.sum() * len(reqs)
    assert np.all(np.abs(counts[:8] - want[:8]) < 5 * np.sqrt(want[:8]))
    for r in reqs[:2000]:
        assert r.prefix_len % BLOCK == 0 and 0 <= r.prefix_len <= r.prompt_len
        assert len(r.gap) == len(r.decode) - 1 and min(r.decode) >= 1 and all(g >= 1 for g in r.gap)
    assert abs(np.mean([len(r.decode) for r in reqs]) - 3.0) < 0.1
    # same seed, same trace; another seed, another trace
    again = synth.fleet_requests(200, 13, 0.5, 64, cats)
    assert [(r.arrival, r.model, r.prefix, r.prompt_len) for r in again] == \
           [(r.arrival, r.model, r.prefix, r.prompt_len) for r in reqs[:200]]
    other = synth.fleet_requests(200, 14, 0.5, 64, cats)
    assert [(r.arrival, r.prompt_len) for r in other] != [(r.arrival, r.prompt_len) for r in again]


def test_plan_is_one_consistent_history():
    shapes, cats, reqs, plan = small_fleet()
    n = plan.n_uids
    upb = [s.n_layers * s.n_kv_heads for s in shapes]
    # ---- the arena: every row owns a uid range of its own, long enough for the row's last length
    spans = []
    for a, r in enumerate(plan.rows):
        n_rows = len(r["off"])
        assert n_rows % upb[a] == 0 and r["ntok"].shape == (plan.n_steps, n_rows)
        last_nb = (r["ntok"].max(axis=0).astype(np.int64) + BLOCK - 1) // BLOCK
        spans += [(int(o), int(o + nb)) for o, nb in zip(r["off"], last_nb)]
        # rows of one entry (all layers and heads of a sequence) have the same length and decode together
        ent = r["ntok"].reshape(plan.n_steps, -1, upb[a])
        assert (ent == ent[:, :, :1]).all()
        act = r["active"].reshape(plan.n_steps, -1, upb[a])
        assert (act == act[:, :, :1]).all()
        np.testing.assert_array_equal(r["layer"], np.tile(np.arange(upb[a]) // shapes[a].n_kv_heads, n_rows // upb[a]))
        np.testing.assert_array_equal(r["q_off"], np.arange(n_rows) * shapes[a].g * shapes[a].dim)
    spans.sort()
    assert spans[0][0] >= 0 and spans[-1][1] <= n
    assert all(a[1] <= b[0] for a, b in zip(spans, spans[1:]))          # no two rows share a uid
    # ---- lengths: a decoding row appends exactly one token per step, an idle one keeps its length unless a
    # request continues its entry (then it grows by that request's new part, at a step where it decodes again)
    for a, r in enumerate(plan.rows):
        nt, act = r["ntok"].astype(np.int64), r["active"]
        for j in range(1, plan.n_steps):
            grew = nt[j] - nt[j - 1]
            assert (grew >= 0).all()
            was_decoding = act[j - 1] == 1
            assert (grew[was_decoding & (act[j] == 1)] >= 1).all()
            still = (act[j - 1] == 0) & (act[j] == 0)
            assert (grew[still] == 0).all()
            came_to_be = (nt[j - 1] == 0) & (nt[j] > 0)
            assert (act[j][came_to_be] == 1).all()                       # a new entry decodes at once
        pos = r["pos"]
        assert ((pos == -1) == (act == 0)).all() and (pos[act == 1] == nt[act == 1]).all()
    # ---- units: what exists = what existed + what came into existence, exactly the blocks the lengths imply
    exists = np.zeros(n, bool)
    exists[plan.init_units] = True
    assert len(np.unique(plan.init_units)) == len(plan.init_units)
    for a, r in enumerate(plan.rows):
        nb0 = (plan.init_ntok[a].astype(np.int64) + BLOCK - 1) // BLOCK
        want = np.concatenate([o + np.arange(k) for o, k in zip(r["off"], nb0)]) if len(nb0) else np.zeros(0, np.int64)
        assert exists[want].all()
    assert exists.sum() == sum(int((((plan.init_ntok[a].astype(np.int64) + BLOCK - 1) // BLOCK)).sum())
                               for a in range(len(shapes)))
    for j in range(plan.n_steps):
        new = plan.new_uids[j]
        assert len(np.unique(new)) == len(new) and not exists[new].any()
        exists[new] = True
        for a, r in enumerate(plan.rows):
            nb = (r["ntok"][j].astype(np.int64) + BLOCK - 1) // BLOCK
            want = np.concatenate([o + np.arange(k) for o, k in zip(r["off"], nb)]) if len(nb) else np.zeros(0, np.int64)
            assert exists[want].all(), j
        assert exists.sum() == sum(int(((r["ntok"][j].astype(np.int64) + BLOCK - 1) // BLOCK).sum()) for r in plan.rows)
    assert plan.stats["new_units_per_step"] == [len(u) for u in plan.new_uids] and sum(plan.stats["new_units_per_step"]) > 0
    # ---- the block being written: after a step's prot_clear / prot_set exactly the last blocks of the decoding
    # rows are protected
    prot = np.zeros(n, bool)
    for j in range(plan.n_steps):
        assert prot[plan.prot_clear[j]].all() and not prot[plan.prot_set[j]].any()
        prot[plan.prot_clear[j]] = False
        prot[plan.prot_set[j]] = True
        want = []
        for r in plan.rows:
            on = r["active"][j] == 1
            want.append(r["off"][on] + (r["ntok"][j][on].astype(np.int64) + BLOCK - 1) // BLOCK - 1)
        want = np.concatenate(want)
        np.testing.assert_array_equal(np.flatnonzero(prot), np.sort(want))
        assert exists[np.flatnonzero(prot)].all()
    # ---- events: pairs in range, outcomes 0 / 1; pair bytes of the units: 4 * block type + transition
    for p, o in plan.events:
        assert p.dtype == np.uint8 and o.dtype == np.uint8 and len(p) == len(o)
        assert (p < 16).all() and (o <= 1).all()
    assert plan.pair.max() < 16
    assert plan.stats["hits"] > 0 and plan.stats["misses"] > 0
    assert plan.stats["hits"] + plan.stats["misses"] == plan.stats["requests_replayed"]


def test_plan_is_deterministic_and_independent_of_the_window_length():
    _, _, _, a = small_fleet(n_steps=14)
    _, _, _, b = small_fleet(n_steps=14)
    assert a.n_uids == b.n_uids and (a.pair == b.pair).all()
    for x, y in zip(a.new_uids, b.new_uids):
        np.testing.assert_array_equal(x, y)
    # a shorter window is a prefix of the longer one in everything that does not depend on the arena's layout
    _, _, _, c = small_fleet(n_steps=9)
    assert c.stats["new_units_per_step"] == a.stats["new_units_per_step"][:9]
    assert c.stats["events_per_step"] == a.stats["events_per_step"][:9]
    assert c.stats["active_per_step"] == a.stats["active_per_step"][:9]
    assert c.stats["init_units"] == a.stats["init_units"]


def test_growing_batch_is_the_fleet_replay_of_sequences_that_only_decode():
    lens = [700, 2100, 333, 17, 1500, 1023]
    shape = synth.Shape(2, 8, 2, 128, synth.BF16, True, lens)
    plan = fleet.build_plan([shape], [[synth.FleetPrefix(0.0, 2, 0)]], synth.growing_batch_requests(lens), 1, 24,
                            capacity_units=1 << 62)
    upb = shape.n_layers * shape.n_kv_heads
    r = plan.rows[0]
    assert len(r["off"]) == len(lens) * upb and (r["active"] == 1).all()
    for j in range(24):
        np.testing.assert_array_equal(r["ntok"][j].reshape(len(lens), upb)[:, 0], np.array(lens) + 1 + j)
        crossing = [(n + j) % BLOCK == 0 for n in lens]                 # the token appended before this step opened a block
        assert len(plan.new_uids[j]) == upb * sum(crossing)
    assert len(plan.events[0][0]) == 0 and plan.stats["hits"] == 0
    assert plan.n_uids == upb * sum((n + 24 + BLOCK) // BLOCK for n in lens) or plan.n_uids >= plan.stats["init_units"]
