"""GPU parity on a heterogeneous fleet (twin of the fifth workload): MHA and MQA
sequences share one HBM pool and one uid space, each architecture is one row
group (its own g), sessions go idle and resume, and every step runs scoring,
posterior updates, eviction to a budget and prefetch of resuming sessions on
both the HIP path and the oracle."""
import numpy as np
import pytest
import torch

from paper_2604_26968_amd import synth
from tests.harness import gpu_row_weight, ref_row_weight

pytestmark = pytest.mark.gpu

RES, HOST, PROT, SCORED = 1, 2, 4, 8


def lognormal_lengths(n, seed, mu=5.5, sigma=1.0, lo=16, hi=4096):
    rng = np.random.default_rng(seed)
    return [int(v) for v in np.clip(rng.lognormal(mu, sigma, n), lo, hi)]


class Fleet:
    """Two architectures over one pool: per-unit arrays are concatenated, slots of the second
    group are shifted behind the first group's frames."""

    def __init__(self, shape_a, shape_b, seed):
        a = synth.make_case(shape_a, seed, pair_weights=synth.categorical_weights(seed + 5), uid_gap=1)
        b = synth.make_case(shape_b, seed + 1, pair_weights=synth.categorical_weights(seed + 5), uid_gap=2)
        assert shape_a.dim == shape_b.dim and shape_a.dtype == shape_b.dtype
        self.groups = [a, b]
        self.dim, self.dtype = shape_a.dim, shape_a.dtype
        self.n_slots = a.n_slots + b.n_slots
        self.k_pool = np.concatenate([a.k_pool, b.k_pool])
        self.v_pool = np.concatenate([a.v_pool, b.v_pool])
        self.uid_base = [0, a.n_uids]
        self.n_uids = a.n_uids + b.n_uids
        tb = b.slot_tbl.copy()
        tb[tb >= 0] += a.n_slots
        self.slot_tbl = np.concatenate([a.slot_tbl, tb]).astype(np.int32)
        self.state = np.concatenate([a.state, b.state])
        self.pair = np.concatenate([a.pair, b.pair])
        self.rows = []
        for grp, base in zip(self.groups, self.uid_base):
            self.rows.append(dict(ntok=grp.row_ntok, off=(grp.row_off + base).astype(np.int64), q_off=grp.row_q_off,
                                  seq=grp.row_seq, g=grp.shape.g,
                                  q_elems=grp.n_rows * grp.shape.g * grp.shape.dim))


def run_fleet(oracle, shape_a, shape_b, steps=5, seed=40):
    from paper_2604_26968_amd import kvm
    fl = Fleet(shape_a, shape_b, seed)
    dev = "cuda"
    t = lambda x: torch.from_numpy(np.ascontiguousarray(x)).to(dev)
    k_pool, v_pool = t(fl.k_pool.view(np.int16)), t(fl.v_pool.view(np.int16))
    pool = kvm.make_pool(k_pool, v_pool, fl.dim, fl.dtype)
    slot_tbl, state, pair = t(fl.slot_tbl), t(fl.state), t(fl.pair)
    n = fl.n_uids
    mass = torch.zeros(n, dtype=torch.float32, device=dev)
    S = torch.zeros(n, dtype=torch.float32, device=dev)
    prio = torch.zeros(n, dtype=torch.float32, device=dev)
    hits = torch.zeros(16, dtype=torch.int32, device=dev)
    misses = torch.zeros(16, dtype=torch.int32, device=dev)
    p_hat = torch.zeros(16, dtype=torch.float32, device=dev)
    victims = torch.zeros(n, dtype=torch.int64, device=dev)
    n_victims = torch.zeros(1, dtype=torch.int64, device=dev)
    n_bad = torch.zeros(1, dtype=torch.int32, device=dev)
    ws_bytes = max([kvm.kvm_workspace_bytes(kvm.OP_SCORE, n, len(r["ntok"]), r["g"], fl.dim) for r in fl.rows]
                   + [kvm.kvm_workspace_bytes(kvm.OP_SELECT, n)])
    ws = torch.full((ws_bytes,), 0x7F, dtype=torch.uint8, device=dev)
    # head weights: the library's sizing call for the GPU side, the oracle's sizing function for the oracle
    dev_rows = [dict(ntok=t(r["ntok"]), off=t(r["off"]), q_off=t(r["q_off"]),
                     weight=t(gpu_row_weight(kvm, grp.shape, grp.n_rows))) for r, grp in zip(fl.rows, fl.groups)]
    for r, grp in zip(fl.rows, fl.groups):
        r["weight"] = ref_row_weight(oracle, grp)
    rec = 2 * 16 * fl.dim * 2

    # oracle state (host)
    o_tbl, o_state = fl.slot_tbl.copy(), fl.state.copy()
    o_S, o_prio = np.zeros(n, np.float32), np.zeros(n, np.float32)
    o_hits, o_misses = np.zeros(16, np.uint32), np.zeros(16, np.uint32)
    k8 = fl.k_pool.view(np.uint8).reshape(fl.n_slots, -1).copy()
    v8 = fl.v_pool.view(np.uint8).reshape(fl.n_slots, -1).copy()
    host_store = {}

    rng = np.random.default_rng(seed + 9)
    n_res0 = int(np.sum((fl.state & RES) != 0))
    budget = int(0.7 * n_res0)
    n_seq = [len(g.shape.seq_lens) for g in fl.groups]
    idle_left = [np.zeros(k, np.int64) for k in n_seq]          # steps until a session resumes
    scale = 1.0 / np.sqrt(fl.dim)
    w_ev = synth.categorical_weights(seed + 5)

    for step in range(steps):
        # sessions: an active one goes idle with probability 0.3 for an Exp(2)-distributed number of steps
        actives = []
        for gi in range(2):
            idle_left[gi] = np.maximum(idle_left[gi] - 1, 0)
            go_idle = (idle_left[gi] == 0) & (rng.random(n_seq[gi]) < 0.3) & (step > 0)
            idle_left[gi][go_idle] = 1 + rng.exponential(2.0, int(go_idle.sum())).astype(np.int64)
            actives.append((idle_left[gi] == 0))
        ev = synth.make_events(300, seed + 100 + step, pair_weights=w_ev, reuse_prob=np.linspace(0.1, 0.9, 16))

        kvm.kvm_beta_update(t(ev[0]), t(ev[1]), hits, misses, p_hat, n_bad=n_bad)
        o_p = oracle.beta_update(ev[0], ev[1], o_hits, o_misses)
        np.testing.assert_array_equal(hits.cpu().numpy().view(np.uint32), o_hits)
        np.testing.assert_array_equal(misses.cpu().numpy().view(np.uint32), o_misses)

        o_mass = np.zeros(n, np.float32)
        mass.zero_()
        row_active = []
        for gi, (r, dr, grp) in enumerate(zip(fl.rows, dev_rows, fl.groups)):
            ra = actives[gi][r["seq"]].astype(np.uint8)
            row_active.append(ra)
            q = synth.make_queries(grp, seed + 1000 * gi + step)
            rows = kvm.make_rows(dr["ntok"], dr["off"], dr["q_off"], slot_tbl, r["g"], r["q_elems"], t(ra))
            kvm.kvm_score_step(pool, rows, t(q.view(np.int16)), scale, mass, ws)
            oracle.score_step(k8.view(np.uint16).reshape(fl.n_slots, -1), fl.dim, fl.dtype, r["ntok"], r["off"],
                              r["q_off"], o_tbl, q, r["g"], scale, o_mass, row_active=ra)
        torch.cuda.synchronize()
        np.testing.assert_allclose(mass.cpu().numpy(), o_mass, rtol=1e-3, atol=1e-9)

        # identical masses on both sides from here on, so that the states stay comparable
        mass.copy_(torch.from_numpy(o_mass))
        for gi, (r, dr) in enumerate(zip(fl.rows, dev_rows)):
            rows = kvm.make_rows(dr["ntok"], dr["off"], dr["q_off"], slot_tbl, r["g"], r["q_elems"], t(row_active[gi]))
            kvm.kvm_ema_update(rows, mass, 0.9, dr["weight"], pair, p_hat, state, S, prio)
            oracle.ema_update(r["ntok"], r["off"], o_mass, 0.9, r["weight"], fl.pair, o_p, o_state, o_S, o_prio,
                              row_active=row_active[gi])
        torch.cuda.synchronize()
        np.testing.assert_array_equal(state.cpu().numpy(), o_state)
        np.testing.assert_allclose(S.cpu().numpy(), o_S, rtol=3e-6)
        fin = np.isfinite(o_prio)
        np.testing.assert_allclose(prio.cpu().numpy()[fin], o_prio[fin], rtol=3e-6)

        # select on the oracle's priorities (bit-identical keys) -> identical victim sets
        prio.copy_(torch.from_numpy(o_prio))
        kvm.kvm_select_victims(prio, state, victims, n_victims, ws, k=-1, budget_units=budget)
        ov = oracle.select_victims(o_prio, o_state, k=-1, budget_units=budget)
        nv = int(n_victims.item())
        np.testing.assert_array_equal(victims[:nv].cpu().numpy(), ov)
        if step == 0:
            assert nv == n_res0 - budget
        # victims are units of both architectures unless one has none eligible
        if nv:
            hs = (np.arange(nv) + 10000 * step).astype(np.int32)
            freed = torch.full((nv,), -1, dtype=torch.int32, device=dev)
            host = torch.zeros(nv * rec, dtype=torch.uint8, pin_memory=True)
            sdev = torch.zeros(min(nv, 64) * rec, dtype=torch.uint8, device=dev)
            kvm.kvm_pack(pool, slot_tbl, state, victims, nv, t(hs), freed, sdev, host, n_bad=n_bad, n_dev=n_victims)
            o_stag, o_freed = oracle.pack(k8, v8, rec // 2, rec // 2, o_tbl, o_state, ov, hs)
            torch.cuda.synchronize()
            np.testing.assert_array_equal(host.numpy().reshape(nv, rec), o_stag)
            np.testing.assert_array_equal(freed.cpu().numpy(), o_freed)
            for u, r_ in zip(ov, o_stag):
                host_store[int(u)] = r_.copy()
            # prefetch: up to 30 host units come back into the frames just freed
            back = rng.choice(np.array(sorted(host_store)), size=min(30, nv), replace=False).astype(np.int64)
            recs = np.stack([host_store.pop(int(u)) for u in back])
            dst = o_freed[:len(back)].astype(np.int32)
            hb = torch.from_numpy(recs.reshape(-1)).pin_memory()
            kvm.kvm_unpack(pool, slot_tbl, state, t(back), len(back), t(dst), sdev, hb, n_bad=n_bad)
            oracle.unpack(k8, v8, rec // 2, rec // 2, o_tbl, o_state, back, dst, recs)
            torch.cuda.synchronize()
        np.testing.assert_array_equal(slot_tbl.cpu().numpy(), o_tbl)
        np.testing.assert_array_equal(state.cpu().numpy(), o_state)
        assert int(n_bad.item()) == 0
    res_slots = o_tbl[(o_state & RES) != 0]
    np.testing.assert_array_equal(k_pool.cpu().numpy().view(np.uint8).reshape(fl.n_slots, -1)[res_slots], k8[res_slots])
    np.testing.assert_array_equal(v_pool.cpu().numpy().view(np.uint8).reshape(fl.n_slots, -1)[res_slots], v8[res_slots])
    # units left the pool (with head weights proportional to the group size the MHA units go first)
    assert ((o_state & HOST) != 0).any()


def test_fleet_mha_plus_mqa_g8(oracle):
    """MHA (4 heads, g 1) and MQA (1 KV head, g 8) sessions with lognormal lengths."""
    a = synth.Shape(2, 4, 4, 128, synth.BF16, True, lognormal_lengths(10, 1))
    b = synth.Shape(2, 8, 1, 128, synth.BF16, True, lognormal_lengths(14, 2))
    run_fleet(oracle, a, b)


def test_fleet_mha_plus_mqa_g32(oracle):
    """Same with the real MQA group size 32 (matrix-core scorer) next to g 1."""
    a = synth.Shape(1, 2, 2, 128, synth.BF16, True, lognormal_lengths(8, 3))
    b = synth.Shape(2, 32, 1, 128, synth.BF16, True, lognormal_lengths(8, 4))
    run_fleet(oracle, a, b, steps=4, seed=60)


# ------------------------------------------------------------------ trace-driven fleet (fifth workload)
def fleet_twin_inputs(seed, n_requests, rate):
    shapes = [synth.Shape(2, 4, 4, 128, synth.BF16, True, []), synth.Shape(2, 32, 1, 128, synth.BF16, True, [])]
    cats = [synth.fleet_catalogue(8, seed), synth.fleet_catalogue(8, seed + 1)]
    reqs = synth.fleet_requests(n_requests, seed + 2, rate, 8, cats, mean_decode=20, mean_gap=30, mu=5.5, hi=4096)
    return shapes, cats, reqs


def run_trace_fleet(oracle, seed, n_requests=260, rate=0.3, start=350, n_steps=14, P=24, keep_all=True, inputs=None,
                    pool_target_units=12000, expect=None, ahead=False, ride_max=1 << 20):
    """The fleet as the benchmark drives it, at a size the oracle follows step by step: one pool sized by
    kvm_size shared by an MHA and an MQA model, a seeded request trace (Zipf prefix ids, lognormal lengths,
    multi-turn sessions with idle gaps), warm start (everything scored once, bulk eviction to the budget),
    then per step: arrivals and growth into the frames the last step made room in, posteriors from the
    step's lookups, scoring of the decoding rows of both architectures, EMA + priority with the head weight
    of each architecture, position-aware prefetch list, ONE victim selection over the shared pool, exchange
    and pack.  Every stage is compared with the oracle; the oracle's floating-point outputs are then handed
    to the GPU side so that both stay on the same trajectory and the integer outputs can be compared exactly.
    `inputs` = (shapes, catalogues, requests) replaces the two-model trace (the growing single-model batch).
    `ahead`: the victims' bytes leave inside the next step's scoring launch (kvm_pack_begin +
    kvm_score_step_xfer) instead of in line, at most `ride_max` units per step."""
    from paper_2604_26968_amd import kvm, fleet
    from tests.fleet_ref import FleetRef
    shapes, cats, reqs = inputs if inputs is not None else fleet_twin_inputs(seed, n_requests, rate)
    target = pool_target_units * 8192 + 100
    sizing = [kvm.kvm_size(**sh.model_args(), n_max=4096, mem_target=target) for sh in shapes]
    for s, sh in zip(sizing, shapes):
        assert s == oracle.size(**sh.model_args(), n_max=4096, mem_target=target)
    assert all(s["pool_units"] == pool_target_units for s in sizing)            # same unit bytes, one pool
    if inputs is None:
        assert [s["head_weight"] for s in sizing] == [1, 32] and [s["units_per_block"] for s in sizing] == [8, 2]
    pool_units = sizing[0]["pool_units"]
    plan = fleet.build_plan(shapes, cats, reqs, start, n_steps, capacity_units=int(0.9 * pool_units), max_tokens=4096)
    st = plan.stats
    print("fleet plan", {k: st[k] for k in ("entries_by_model", "hits", "misses", "retired", "init_units")},
          "active", st["active_per_step"], "new", st["new_units_per_step"], "events", st["events_per_step"], flush=True)
    assert st["init_units"] <= pool_units and min(st["entries_by_model"]) > 0
    assert sum(st["new_units_per_step"]) > 0
    rec = 8192
    tier_slots = st["init_units"] + sum(st["new_units_per_step"]) + 8
    tier = torch.zeros(tier_slots * rec, dtype=torch.uint8).pin_memory()
    dev = fleet.FleetDevice(plan, kvm, torch, pool_units, [float(s["head_weight"]) for s in sizing], tier, tier_slots,
                            prefetch_cap=P, window_tokens=512, seed=seed, fresh_records=64, ahead=ahead, ride_max=ride_max)
    ref = FleetRef(oracle, dev, plan)
    n = plan.n_uids
    cpu = lambda x: x.detach().cpu().numpy()

    def same_tables(tag):
        np.testing.assert_array_equal(cpu(dev.slot_tbl), ref.tbl, err_msg=tag)
        np.testing.assert_array_equal(cpu(dev.state), ref.state, err_msg=tag)

    def ride_slots(n_ride):
        """Host slots of the one-way pairs (evictions) of the list that waits for a scoring launch."""
        h = cpu(dev.ride_host)[:n_ride]
        h = h[(h >= 0) & ((h & kvm.XFER_OUT_ONLY) != 0)]
        return (h & ~kvm.XFER_OUT_ONLY).astype(np.int64)

    def floats_then_align(tag, j, q_set):
        dev.score(j, q_set)
        ref.score(j, q_set)
        torch.cuda.synchronize()
        np.testing.assert_allclose(cpu(dev.mass), ref.mass, rtol=1e-3, atol=1e-9, err_msg=tag)
        dev.mass.copy_(torch.from_numpy(ref.mass))
        dev.ema(j)
        ref.ema(j)
        torch.cuda.synchronize()
        same_tables(tag + " ema")
        np.testing.assert_allclose(cpu(dev.S), ref.S, rtol=3e-6, err_msg=tag)
        fin = np.isfinite(ref.prio)
        np.testing.assert_allclose(cpu(dev.prio)[fin], ref.prio[fin], rtol=3e-6, err_msg=tag)
        assert np.array_equal(np.isfinite(cpu(dev.prio)), fin)
        dev.S.copy_(torch.from_numpy(ref.S))
        dev.prio.copy_(torch.from_numpy(ref.prio))

    # ---- warm start ---------------------------------------------------------------------------------------
    dev.beta_none()
    ref.beta(None)
    floats_then_align("first pass", None, 0)
    n_res = int((ref.state & RES).sum())
    assert n_res == st["init_units"]
    budget = int(0.6 * n_res)
    order = np.random.default_rng(seed + 7).permutation(n_res - budget)
    keep = (n_res - budget) if keep_all else (n_res - budget) // 2
    scratch = torch.zeros(tier_slots * rec, dtype=torch.uint8).pin_memory()
    k0, _ = dev.evict_to_budget(budget, keep, order, scratch, chunk=500)
    k0_ref, _ = ref.evict_to_budget(budget, keep, order)
    assert k0 == k0_ref == n_res - budget
    same_tables("bulk eviction")
    np.testing.assert_array_equal(tier.numpy().reshape(tier_slots, rec)[:keep], ref.tier[:keep])
    np.testing.assert_array_equal(cpu(dev.free), ref.free)
    assert (dev.free_head, dev.free_ready, dev.free_tail) == (ref.free_head, ref.free_ready, ref.free_tail)
    assert dev.budget == dev.resident == ref.budget == ref.resident == budget

    # ---- the window -----------------------------------------------------------------------------------------
    n_pf_seen = n_moved = n_rode = n_to_ride = 0
    over_budget = []
    for j in range(n_steps):
        tag = "step %d" % j
        dev.arrive(j)
        ref.arrive(j)
        same_tables(tag + " arrive")
        dev.beta(j)
        ref.beta(j)
        np.testing.assert_array_equal(cpu(dev.hits).view(np.uint32), ref.hits)
        np.testing.assert_array_equal(cpu(dev.misses).view(np.uint32), ref.misses)
        np.testing.assert_allclose(cpu(dev.p_hat), ref.p_hat, rtol=1e-6)
        dev.p_hat.copy_(torch.from_numpy(ref.p_hat))
        riding = dev.ride
        floats_then_align(tag, j, j)
        if riding is not None:                  # the records of the last step's moves were written by the scoring launch
            r_slots = ride_slots(riding[0])
            assert dev.ride is None and len(r_slots) == dev.evicted[j - 1] and (len(r_slots) == 0 or r_slots.min() >= 0)
            np.testing.assert_array_equal(tier.numpy().reshape(tier_slots, rec)[r_slots], ref.tier[r_slots], err_msg=tag)
            n_rode += len(r_slots)
        dev.settle()
        ref.settle()
        same_tables(tag + " settle")
        dev.prefetch_keys(j)
        ref.prefetch_keys(j)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(cpu(dev.cand), ref.cand, err_msg=tag)
        fin = np.isfinite(ref.key)
        # key = 1 - p * decay^d in fp32: the power, the product and the difference each round once, on values
        # of at most 1 (half an ulp of 1 = 6e-8 for each, 1.2e-7 where the exp2 is off by one ulp): 4e-7 in all
        np.testing.assert_allclose(cpu(dev.key)[fin], ref.key[fin], atol=4e-7, rtol=0, err_msg=tag)
        dev.key.copy_(torch.from_numpy(ref.key))
        dev.select(j)
        ref.select(j)
        torch.cuda.synchronize()
        assert dev.evict_now == ref.evict_now == (min(max(dev.resident - budget, 0), ride_max) if ahead
                                                   else max(dev.resident - budget, 0))
        k = dev.evict_now + P
        assert int(dev.n_v.item()) == len(ref.victims) == k, (tag, int(dev.n_v.item()), len(ref.victims), k)
        np.testing.assert_array_equal(cpu(dev.victims)[:k], ref.victims, err_msg=tag)
        n_pf = int(dev.n_pf.item())
        assert n_pf == len(ref.pf_list)
        np.testing.assert_array_equal(cpu(dev.pf_list)[:n_pf], ref.pf_list, err_msg=tag)
        n_pf_seen += n_pf
        dev.move(j)
        ref.move(j)
        torch.cuda.synchronize()
        same_tables(tag + " move")
        m = dev.evicted[j]
        np.testing.assert_array_equal(cpu(dev.free)[:dev.free_tail], ref.free[:ref.free_tail], err_msg=tag)
        assert (dev.free_head, dev.free_tail, dev.resident) == (ref.free_head, ref.free_tail, ref.resident)
        # (units an exchange in three parts brings in are not in HBM until it is settled in the next step)
        assert int((ref.state & RES).sum()) == ref.resident - (len(ref.pending_in[0]) if ref.pending_in else 0)
        assert (dev.ride is not None) == (ahead and m + P > 0)
        n_to_ride += m if ahead else 0
        over_budget.append(dev.resident - budget)
        assert dev.next_slot == ref.next_slot
        n_moved += m
        assert int(dev.n_bad.item()) == 0 and int(ref.n_bad[0]) == 0, tag
    if dev.ride is not None:                    # the last step's bytes move in a launch of their own
        r_slots = ride_slots(dev.ride[0])
        dev.flush()
        ref.score_none()
        ref.settle()
        torch.cuda.synchronize()
        same_tables("flush")
        np.testing.assert_array_equal(tier.numpy().reshape(tier_slots, rec)[r_slots], ref.tier[r_slots])
        n_rode += len(r_slots)
    assert (dev.free_head, dev.free_ready, dev.free_tail) == (ref.free_head, ref.free_ready, ref.free_tail)
    # ---- bytes: pools of the units in HBM and the tier records of the units on the host -----------------------
    res = (ref.state & RES) != 0
    frames = ref.tbl[res]
    gk = cpu(dev.k_pool.view(torch.int16)).view(np.uint8).reshape(pool_units, -1)
    gv = cpu(dev.v_pool.view(torch.int16)).view(np.uint8).reshape(pool_units, -1)
    np.testing.assert_array_equal(gk[frames], ref.k8[frames])
    np.testing.assert_array_equal(gv[frames], ref.v8[frames])
    on_host = (ref.state & HOST) != 0
    slots = -1 - ref.tbl[on_host]
    assert slots.min() >= 0 and len(np.unique(slots)) == len(slots)
    np.testing.assert_array_equal(tier.numpy().reshape(tier_slots, rec)[slots], ref.tier[slots])
    # the trace made the pass do all of its work: units were created and evicted, prefetch candidates were found
    # and traded (where a prefetch cap is set), both outcomes of a lookup occurred (two-model trace)
    assert n_moved > 0 and (n_pf_seen > 0 or P == 0)
    assert dev.ride is None and n_rode == n_to_ride and (n_rode > 0) == ahead
    if ahead and ride_max < (1 << 20):
        assert max(over_budget) > 0, "no arrival was large enough to leave HBM over the budget for a while"
    else:
        assert max(over_budget) == 0
    if inputs is None:
        assert ref.hits.sum() > 0 and ref.misses.sum() > 0
    return dict(n_pf=n_pf_seen, moved=n_moved, steps_with_new=sum(1 for m in dev.n_new[:n_steps] if m),
                over_budget=over_budget)


def test_fleet_trace_twin_matches_oracle_step_by_step(oracle):
    run_trace_fleet(oracle, seed=90)


def test_fleet_trace_twin_with_records_dropped_below_tier_one(oracle):
    """Half of the bulk eviction's records are not kept in tier 1 (demoted further down): those units must
    never come back as prefetch candidates and never be scored."""
    run_trace_fleet(oracle, seed=131, rate=0.4, start=300, n_steps=10, P=16, keep_all=False)


def test_fleet_trace_twin_evictions_in_two_parts(oracle):
    """The same trace with every eviction in two parts: the victims leave the table when they are chosen, their
    bytes leave inside the next step's scoring launch, their frames are handed out again after that."""
    run_trace_fleet(oracle, seed=90, ahead=True)


def test_fleet_trace_twin_evictions_in_two_parts_at_a_bounded_rate(oracle):
    """As above with at most 150 units evicted per step: after a prompt has arrived HBM stays over the budget
    for some steps and comes back to it."""
    out = run_trace_fleet(oracle, seed=90, ahead=True, ride_max=150)
    assert out["moved"] > 0 and out["over_budget"][-1] < max(out["over_budget"])


@pytest.mark.parametrize("P,ahead", [(0, False), (12, False), (0, True), (12, True)])
def test_growing_batch_twin_matches_oracle_over_24_steps(oracle, P, ahead):
    """Twin of the Llama-3-8B-shaped configuration as it decodes: every sequence appends one token per step, new
    blocks (hence new units in every layer and head) appear at block boundaries in the frames the previous step's
    victims left, the block being written is PROTECTED and the one before it no longer is; 24 steps, so every
    sequence crosses a boundary at least once.  With P > 0 host-resident blocks near the decode position are also
    prefetched each step."""
    shape = synth.Shape(2, 8, 2, 128, synth.BF16, True, [700, 2100, 333, 17, 1500, 1023])
    inputs = ([shape], [[synth.FleetPrefix(0.0, 2, 0)]], synth.growing_batch_requests(shape.seq_lens))
    out = run_trace_fleet(oracle, seed=7 + P, start=1, n_steps=24, P=P, inputs=inputs, pool_target_units=1600,
                          ahead=ahead)
    assert out["steps_with_new"] >= 6
