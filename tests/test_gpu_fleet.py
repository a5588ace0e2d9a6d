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
