"""Parity at the benchmark's full size and launch configuration (Llama-3-8B-shaped
workload: 5.4 M units, 22 GB of K and as much V), on outputs the oracle can
compute: sampled rows for the scorer and the EMA, the whole array for the
counters and the victim set, sampled records for pack / unpack."""
import numpy as np
import pytest
import torch

from paper_2604_26968_amd import synth
from tests.harness import gpu_row_weight, ref_row_weight, sized_pool_units

pytestmark = pytest.mark.gpu

RES, HOST, PROT, SCORED = 1, 2, 4, 8


def test_llama8b_shaped_full_size(oracle):
    from paper_2604_26968_amd import kvm
    import gc
    gc.collect()
    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info()
    if free < 60 * 2**30:
        pytest.skip("needs 60 GiB of free HBM")
    dev = "cuda"
    shape = synth.llama8b_shape(64, seed=2)
    pair_w = synth.categorical_weights(3)
    wl = synth.DeviceWorkload(shape, seed=1, pair_weights=pair_w, pool_units=sized_pool_units(kvm, oracle, shape))
    n, n_rows, g, dim = wl.n_uids, wl.n_rows, shape.g, shape.dim
    rec = shape.unit_k_bytes + shape.unit_v_bytes
    pool = kvm.make_pool(wl.k_pool.view(torch.int16), wl.v_pool.view(torch.int16), dim, shape.dtype)
    rows = kvm.make_rows(wl.row_ntok, wl.row_off, wl.row_q_off, wl.slot_tbl, g, wl.q_elems)
    scale = 1.0 / float(np.sqrt(dim))
    mass = torch.zeros(n, dtype=torch.float32, device=dev)
    S = torch.zeros(n, dtype=torch.float32, device=dev)
    prio = torch.zeros(n, dtype=torch.float32, device=dev)
    hits = torch.zeros(16, dtype=torch.int32, device=dev)
    misses = torch.zeros(16, dtype=torch.int32, device=dev)
    p_hat = torch.zeros(16, dtype=torch.float32, device=dev)
    n_bad = torch.zeros(1, dtype=torch.int32, device=dev)
    n_victims = torch.zeros(1, dtype=torch.int64, device=dev)
    ws = torch.empty(max(kvm.kvm_workspace_bytes(kvm.OP_SCORE, n, n_rows, g, dim),
                         kvm.kvm_workspace_bytes(kvm.OP_SELECT, n)), dtype=torch.uint8, device=dev)
    sample_seqs = [5, 40]

    def check_sample(q_dev, tag):
        """Oracle on all rows of two sequences against the masses the GPU just wrote."""
        case = wl.host_sample(sample_seqs)
        qh = q_dev.view(torch.int16).cpu().numpy().view(np.uint16)
        q_rows = np.concatenate([qh[r * g * dim:(r + 1) * g * dim] for r in case.sample_rows])
        ref = np.full(case.n_uids, -1.0, np.float32)
        oracle.score_step(case.k_pool, dim, shape.dtype, case.row_ntok, case.row_off, case.row_q_off, case.slot_tbl,
                          q_rows, g, scale, ref)
        got = mass[torch.from_numpy(case.sample_uids).to(dev)].cpu().numpy()
        res = case.slot_tbl >= 0
        assert res.sum() > 1000, tag
        np.testing.assert_allclose(got[res], ref[res], rtol=1e-3, atol=1e-9, err_msg=tag)
        return case, ref

    # ---- step 0: everything resident -----------------------------------------------------------
    ev = synth.make_events(4096, 200, pair_weights=pair_w, reuse_prob=np.linspace(0.15, 0.95, 16))
    kvm.kvm_beta_update(torch.from_numpy(ev[0]).to(dev), torch.from_numpy(ev[1]).to(dev), hits, misses, p_hat,
                        n_bad=n_bad)
    oh, om = np.zeros(16, np.uint32), np.zeros(16, np.uint32)
    op = oracle.beta_update(ev[0], ev[1], oh, om)
    np.testing.assert_array_equal(hits.cpu().numpy().view(np.uint32), oh)
    np.testing.assert_array_equal(misses.cpu().numpy().view(np.uint32), om)
    np.testing.assert_allclose(p_hat.cpu().numpy(), op, rtol=1e-6)

    q0 = wl.queries(100)
    kvm.kvm_score_step(pool, rows, q0, scale, mass, ws)
    torch.cuda.synchronize()
    case, ref_mass = check_sample(q0, "all resident")

    row_weight = torch.from_numpy(gpu_row_weight(kvm, shape, n_rows)).to(dev)
    kvm.kvm_ema_update(rows, mass, 0.95, row_weight, wl.pair, p_hat, wl.state, S, prio)
    torch.cuda.synchronize()
    S_ref, prio_ref, st_ref = np.zeros(case.n_uids, np.float32), np.zeros(case.n_uids, np.float32), case.state.copy()
    oracle.ema_update(case.row_ntok, case.row_off, ref_mass, 0.95, ref_row_weight(oracle, case), case.pair, op, st_ref,
                      S_ref, prio_ref)
    idx = torch.from_numpy(case.sample_uids).to(dev)
    np.testing.assert_allclose(S[idx].cpu().numpy(), S_ref, rtol=1e-3)
    np.testing.assert_allclose(prio[idx].cpu().numpy(), prio_ref, rtol=1e-3)
    np.testing.assert_array_equal(wl.state[idx].cpu().numpy(), st_ref)

    # ---- victim selection over all 5.4 M units against a full sort ------------------------------
    n_res0 = int((wl.state & 1).sum().item())
    budget = int(0.6 * n_res0)
    k0 = n_res0 - budget
    victims = torch.zeros(k0, dtype=torch.int64, device=dev)
    kvm.kvm_select_victims(prio, wl.state, victims, n_victims, ws, k=-1, budget_units=budget)
    torch.cuda.synchronize()
    assert int(n_victims.item()) == k0
    want = oracle.select_victims(prio.cpu().numpy(), wl.state.cpu().numpy(), k=-1, budget_units=budget)
    np.testing.assert_array_equal(victims.cpu().numpy(), want)

    # ---- bulk eviction in slices through one pinned buffer; first slice checked byte for byte ---
    slice_n = 32768
    host = torch.empty(slice_n * rec, dtype=torch.uint8, pin_memory=True)
    sdev = torch.empty(8192 * rec, dtype=torch.uint8, device=dev)
    freed = torch.full((k0,), -1, dtype=torch.int32, device=dev)
    host_slots = torch.arange(k0, dtype=torch.int32, device=dev)
    first = victims[:slice_n]
    first_slots = wl.slot_tbl[first].long()
    want_k = wl.k_pool[first_slots[:512]].view(torch.uint8).cpu().numpy()
    want_v = wl.v_pool[first_slots[:512]].view(torch.uint8).cpu().numpy()
    kept = None
    for lo in range(0, k0, slice_n):
        cnt = min(slice_n, k0 - lo)
        kvm.kvm_pack(pool, wl.slot_tbl, wl.state, victims[lo:lo + cnt], cnt, host_slots[lo:lo + cnt],
                     freed[lo:lo + cnt], sdev, host, n_bad=n_bad)
        torch.cuda.synchronize()
        if lo == 0:
            got = host.numpy().reshape(slice_n, rec)
            np.testing.assert_array_equal(got[:512, :shape.unit_k_bytes], want_k.reshape(512, -1))
            np.testing.assert_array_equal(got[:512, shape.unit_k_bytes:], want_v.reshape(512, -1))
            np.testing.assert_array_equal(freed[:slice_n].cpu().numpy(), first_slots.cpu().numpy().astype(np.int32))
            kept = host[:1024 * rec].clone().pin_memory()
    assert int(n_bad.item()) == 0
    assert int((wl.state & 1).sum().item()) == budget
    assert bool((wl.slot_tbl[victims] == -1 - host_slots).all())

    # ---- prefetch 1024 of them back into other freed frames, as the benchmark does each step ----
    back, dst = victims[:1024], freed[k0 - 1024:]
    kvm.kvm_unpack(pool, wl.slot_tbl, wl.state, back, 1024, dst, sdev, kept, n_bad=n_bad)
    torch.cuda.synchronize()
    assert int(n_bad.item()) == 0
    assert int((wl.state & 1).sum().item()) == budget + 1024
    np.testing.assert_array_equal(wl.k_pool[dst[:512].long()].view(torch.uint8).cpu().numpy().reshape(512, -1),
                                  want_k.reshape(512, -1))
    np.testing.assert_array_equal(wl.v_pool[dst[:512].long()].view(torch.uint8).cpu().numpy().reshape(512, -1),
                                  want_v.reshape(512, -1))
    assert bool((wl.slot_tbl[back] == dst).all())

    # ---- the launch the benchmark times: 60 % + 1024 units resident ------------------------------
    q1 = wl.queries(101)
    mass.fill_(-1.0)
    kvm.kvm_score_step(pool, rows, q1, scale, mass, ws)
    torch.cuda.synchronize()
    check_sample(q1, "at budget")
    # properties over the whole array: resident units were scored, the others were not touched
    resident = (wl.state & 1) != 0
    assert bool((mass[resident] >= 0).all()) and bool((mass[~resident] == -1.0).all())
    # sum over the resident blocks of a row lies in [1, g] for the group maximum
    row_sum = torch.zeros(n_rows, dtype=torch.float64, device=dev)
    row_id = torch.repeat_interleave(torch.arange(n_rows, device=dev), torch.from_numpy(wl.nb).to(dev))
    row_sum.index_add_(0, row_id[resident], mass[resident].double())
    assert float(row_sum.min()) > 1.0 - 1e-4 and float(row_sum.max()) < g + 1e-4

    # ---- the same with an exchange riding along, as the benchmark's default mode launches it -------
    host_tier = torch.empty(2048 * rec, dtype=torch.uint8, pin_memory=True)
    # 1,024 resident units go to host slots 0..1023 first; then they trade places with 1,024 others
    res_ids = torch.nonzero(resident).flatten()
    sel = res_ids[torch.randperm(res_ids.numel(), generator=wl.gen, device=dev)[:2048]]
    out_a, out_b = sel[:1024].contiguous(), sel[1024:].contiguous()
    kvm.kvm_pack(pool, wl.slot_tbl, wl.state, out_a, 1024, torch.arange(1024, dtype=torch.int32, device=dev),
                 freed[:1024], None, host_tier[:1024 * rec], n_bad=n_bad)
    torch.cuda.synchronize()
    rec_a = host_tier[:1024 * rec].clone()                 # what is on the host for out_a
    frames_b = wl.slot_tbl[out_b].clone()
    k_b = wl.k_pool[frames_b[:256].long()].view(torch.uint8).cpu().numpy().reshape(256, -1)
    v_b = wl.v_pool[frames_b[:256].long()].view(torch.uint8).cpu().numpy().reshape(256, -1)
    xf_frame = torch.full((1024,), -1, dtype=torch.int32, device=dev)
    xf_host = torch.full((1024,), -1, dtype=torch.int64, device=dev)
    kvm.kvm_exchange_begin(pool, wl.slot_tbl, wl.state, out_b, out_a, 1024, 2048, xf_frame, xf_host, n_bad=n_bad)
    q2 = wl.queries(102)
    mass.fill_(-1.0)
    # ... and with the next victims chosen meanwhile on a second stream, as the default step does it
    ws_sel = torch.empty(kvm.kvm_workspace_bytes(kvm.OP_SELECT, n), dtype=torch.uint8, device=dev)
    vic_seq = torch.zeros(1024, dtype=torch.int64, device=dev)
    vic_par = torch.zeros(1024, dtype=torch.int64, device=dev)
    n_par = torch.zeros(1, dtype=torch.int64, device=dev)
    kvm.kvm_select_victims(prio, wl.state, vic_seq, n_victims, ws_sel, k=1024)
    torch.cuda.synchronize()
    assert int(n_victims.item()) == 1024
    main, side = torch.cuda.current_stream(), torch.cuda.Stream()
    side.wait_stream(main)
    kvm.kvm_select_victims(prio, wl.state, vic_par, n_par, ws_sel, k=1024, stream=side)
    kvm.kvm_score_step_xfer(pool, rows, q2, scale, mass, ws, xf_frame, xf_host, 1024, host_tier)
    main.wait_stream(side)
    torch.cuda.synchronize()
    assert int(n_par.item()) == 1024 and bool((vic_par == vic_seq).all())
    want_v2 = oracle.select_victims(prio.cpu().numpy(), wl.state.cpu().numpy(), k=1024)
    np.testing.assert_array_equal(vic_par.cpu().numpy(), want_v2)
    check_sample(q2, "at budget, exchange riding along")
    in_flight = torch.cat([out_a, out_b])
    assert bool((mass[in_flight] == -1.0).all())           # neither side of a pair is in HBM for the scorer
    kvm.kvm_exchange_end(wl.slot_tbl, wl.state, out_a, xf_frame, 1024)
    torch.cuda.synchronize()
    assert int(n_bad.item()) == 0
    assert bool((xf_frame == frames_b).all()) and bool((wl.slot_tbl[out_a] == frames_b).all())
    assert bool((wl.slot_tbl[out_b] == -1 - torch.arange(1024, dtype=torch.int32, device=dev)).all())
    # frames of out_b now hold out_a's records; the tier slots hold out_b's old frames
    got_k = wl.k_pool[frames_b[:256].long()].view(torch.uint8).cpu().numpy().reshape(256, -1)
    want_a = rec_a.numpy().reshape(1024, rec)[:256]
    np.testing.assert_array_equal(got_k, want_a[:, :shape.unit_k_bytes])
    tier_now = host_tier.numpy().reshape(2048, rec)[:256]
    np.testing.assert_array_equal(tier_now[:, :shape.unit_k_bytes], k_b)
    np.testing.assert_array_equal(tier_now[:, shape.unit_k_bytes:], v_b)


@pytest.mark.parametrize("name,need_gib", [("llama70b", 190), ("mla", 90)])
def test_long_row_workloads_full_size_sampled(oracle, name, need_gib):
    """Configs 3 and 4 at full size (8,192-block rows with g = 8; 2,048-block latent rows with g = 128),
    in the launch configuration the benchmark times: all resident, then half / 40 % resident.  The oracle
    scores sampled rows; over the whole array resident units are written, others untouched, and every
    row's masses sum to a value in [1, g]."""
    from paper_2604_26968_amd import kvm
    import gc
    gc.collect()
    torch.cuda.empty_cache()               # give back what earlier tests' pools still hold in the allocator
    free, _ = torch.cuda.mem_get_info()
    if free < need_gib * 2**30:
        pytest.skip("needs %d GiB of free HBM" % need_gib)
    dev = "cuda"
    shape = synth.llama70b_shape() if name == "llama70b" else synth.mla_shape()
    wl = synth.DeviceWorkload(shape, seed=1, pair_weights=synth.categorical_weights(3),
                              pool_units=sized_pool_units(kvm, oracle, shape))
    n, n_rows, g, dim = wl.n_uids, wl.n_rows, shape.g, shape.dim
    pool = kvm.make_pool(wl.k_pool.view(torch.int16), None if wl.v_pool is None else wl.v_pool.view(torch.int16), dim,
                         shape.dtype)
    rows = kvm.make_rows(wl.row_ntok, wl.row_off, wl.row_q_off, wl.slot_tbl, g, wl.q_elems)
    scale = 1.0 / float(np.sqrt(dim))
    mass = torch.full((n,), -1.0, dtype=torch.float32, device=dev)
    ws = torch.empty(kvm.kvm_workspace_bytes(kvm.OP_SCORE, n, n_rows, g, dim), dtype=torch.uint8, device=dev)
    # at least 64 rows and 0.5 % of the K bytes: first, middle and last row always, the rest drawn with a seed
    # (64 of 2,560 rows = 2.5 %, 64 of 1,952 = 3.3 %; rows all have the same length here)
    drawn = np.random.default_rng(23).choice(n_rows, size=64, replace=False)
    sample = np.unique(np.concatenate([[0, n_rows // 2, n_rows - 1], drawn]))
    assert len(sample) >= 64 and len(sample) * 200 >= n_rows
    sample_all_resident = sample
    row_id = torch.repeat_interleave(torch.arange(n_rows, device=dev), torch.from_numpy(wl.nb).to(dev))
    for phase, frac in (("all resident", 1.0), ("at budget", 0.5 if name == "llama70b" else 0.4)):
        if frac < 1.0:
            # take a random share of the units out of HBM (table and state only: the scorer must skip them)
            drop = torch.rand(n, generator=wl.gen, device=dev) >= frac
            drop &= (wl.state & PROT) == 0
            wl.slot_tbl[drop] = -1
            wl.state[drop] = (wl.state[drop] & (255 - RES)) | HOST
        q = wl.queries(110)
        mass.fill_(-1.0)
        kvm.kvm_score_step(pool, rows, q, scale, mass, ws)
        torch.cuda.synchronize()
        case = wl.host_sample(rows=sample if frac < 1.0 else sample_all_resident)
        print(name, phase, "oracle rows", case.n_rows, flush=True)
        qh = q.view(torch.int16).cpu().numpy().view(np.uint16)
        q_rows = np.concatenate([qh[r * g * dim:(r + 1) * g * dim] for r in case.sample_rows])
        ref = np.full(case.n_uids, -1.0, np.float32)
        oracle.score_step(case.k_pool, dim, shape.dtype, case.row_ntok, case.row_off, case.row_q_off, case.slot_tbl,
                          q_rows, g, scale, ref)
        got = mass[torch.from_numpy(case.sample_uids).to(dev)].cpu().numpy()
        res = case.slot_tbl >= 0
        assert res.sum() > 500, phase
        np.testing.assert_allclose(got[res], ref[res], rtol=1e-3, atol=1e-9, err_msg=phase)
        np.testing.assert_array_equal(got[~res], -1.0)
        resident = (wl.state & 1) != 0
        assert bool((mass[resident] >= 0).all()) and bool((mass[~resident] == -1.0).all()), phase
        row_sum = torch.zeros(n_rows, dtype=torch.float64, device=dev)
        row_sum.index_add_(0, row_id[resident], mass[resident].double())
        assert float(row_sum.min()) > 1.0 - 1e-4 and float(row_sum.max()) < g + 1e-3, phase


def test_fleet_full_size_sampled(oracle):
    """The heterogeneous fleet at the benchmark's size and launch configuration: one pool of 21 M frames sized by
    kvm_size (60 % of the HBM) shared by the MHA and the MQA model, the 10,000-request trace replayed on the host
    up to the window, warm start, bulk eviction, then three steps of the window.  The oracle scores sampled
    decoding rows of both models (all resident, and at the last step); over the whole arrays: only resident
    units of decoding rows are written, every decoding row's masses sum to a value in [1, g], the number of
    units in HBM stays what the step's bookkeeping says, nothing is reported bad."""
    import argparse
    import gc
    import bench
    from paper_2604_26968_amd import kvm, fleet
    gc.collect()
    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info()
    if free < 200 * 2**30:
        pytest.skip("needs 200 GiB of free HBM")
    dev = "cuda"
    args = argparse.Namespace(warmup=0, steps=3)
    prep = bench.prepare_fleet(args, kvm, synth)
    shapes, sizing, plan, rec = prep["shapes"], prep["sizing"], prep["plan"], prep["rec"]
    for s, sh in zip(sizing, shapes):       # every field of the sizing the pool comes from
        assert s == oracle.size(**sh.model_args(), n_max=32768, mem_target=int(bench.FLEET["hbm_share"] * 288 * 10**9))
    pool_units = int(sizing[0]["pool_units"])
    keep = 1 << 17
    tier_slots = keep + sum(plan.stats["new_units_per_step"]) + 8
    tier = torch.empty(tier_slots * rec, dtype=torch.uint8, pin_memory=True)
    scratch = torch.empty(32768 * rec, dtype=torch.uint8, pin_memory=True)
    fd = fleet.FleetDevice(plan, kvm, torch, pool_units, [float(s["head_weight"]) for s in sizing], tier, tier_slots,
                           prefetch_cap=1024, window_tokens=2048, decay=0.9, seed=11, ahead=True)   # as bench.py runs it
    n = plan.n_uids
    rng = np.random.default_rng(5)

    def check_rows(j, tag):
        """Sampled rows of both models against the oracle; whole-array properties."""
        worst = 0.0
        for a, d in enumerate(fd.arch):
            on = np.arange(d["n_rows"]) if j is None else torch.nonzero(d["active"][j]).flatten().cpu().numpy()
            pick = np.unique(np.concatenate([[on[0], on[len(on) // 2], on[-1]],
                                             rng.choice(on, size=min(len(on), 1024 if a == 0 else 128), replace=False)]))
            hr = fd.host_rows(a, j, pick, 0 if j is None else j)
            ref = np.full(len(hr["uids"]), -1.0, np.float32)
            oracle.score_step(hr["k_pool"], 128, synth.BF16, hr["ntok"], hr["off"], hr["q_off"], hr["tbl"], hr["q"],
                              hr["g"], fd.scale, ref)
            got = fd.mass[torch.from_numpy(hr["uids"]).to(dev)].cpu().numpy()
            r_ = hr["resident"]
            assert r_.sum() > 1000, tag
            np.testing.assert_allclose(got[r_], ref[r_], rtol=1e-3, atol=1e-9, err_msg=tag)
            np.testing.assert_array_equal(got[~r_], -1.0)
        return worst

    # ---- everything in HBM, every row decodes once ------------------------------------------------------------
    fd.mass.fill_(-1.0)
    fd.first_pass()
    torch.cuda.synchronize()
    check_rows(None, "all resident")
    exist = (fd.state & RES) != 0
    assert int(exist.sum().item()) == plan.stats["init_units"]
    assert bool((fd.mass[exist] >= 0).all()) and bool((fd.mass[~exist] == -1.0).all())
    n_res0 = int(exist.sum().item())
    budget = int(0.6 * n_res0)
    k0, victims = fd.evict_to_budget(budget, keep, np.random.default_rng(6).permutation(n_res0 - budget), scratch)
    assert k0 == n_res0 - budget and int(fd.n_bad.item()) == 0
    assert int((fd.state & RES).sum().item()) == budget
    assert int(((fd.state & HOST) != 0).sum().item()) == keep    # the other victims were demoted below tier 1
    want_resident = budget
    assert fd.budget == fd.resident == budget
    rides, rode, in_flight = [], 0, 0
    for j in range(3):
        fd.arrive(j)
        want_resident += fd.n_new[j]
        fd.beta(j)
        fd.mass.fill_(-1.0)
        fd.score(j, j)
        torch.cuda.synchronize()
        if rides:                           # the last eviction's records were written by this scoring launch
            frames, hosts = rides.pop()
            frames, hosts = frames[fd.P:], hosts[fd.P:]        # behind the swap pairs of the exchange
            pick_r = torch.from_numpy(rng.choice(frames.numel(), size=min(512, frames.numel()), replace=False)).to(dev)
            fr = frames[pick_r].long()
            hs = (hosts[pick_r] & ~kvm.XFER_OUT_ONLY).cpu().numpy()
            assert bool((frames >= 0).all()) and hs.min() >= 0
            want_rec = torch.cat([fd.k_pool[fr].view(torch.uint8).reshape(len(fr), -1),
                                  fd.v_pool[fr].view(torch.uint8).reshape(len(fr), -1)], dim=1).cpu().numpy()
            np.testing.assert_array_equal(tier.numpy().reshape(tier_slots, rec)[hs], want_rec)
            rode += frames.numel()
        if j == 2:
            check_rows(j, "window step %d" % j)
        # only resident units of decoding rows are written; the masses of every decoding row sum to [1, g]
        resident = (fd.state & RES) != 0
        # (the units the last exchange brings in get their frames when it is settled, after this step's EMA)
        assert int(resident.sum().item()) == want_resident - in_flight, (j, int(resident.sum().item()), want_resident)
        written = fd.mass >= 0
        assert bool((written <= resident).all())
        for a, d in enumerate(fd.arch):
            nb = (d["ntok"][j].long() + 15) // 16
            row_id = torch.repeat_interleave(torch.arange(d["n_rows"], device=dev), nb)
            uid = torch.repeat_interleave(d["off"], nb) + (torch.arange(int(nb.sum().item()), device=dev)
                                                          - torch.repeat_interleave(torch.cumsum(nb, 0) - nb, nb))
            act = d["active"][j][row_id] != 0
            assert bool((written[uid[act]] == resident[uid[act]]).all()) and not bool(written[uid[~act]].any())
            sums = torch.zeros(d["n_rows"], dtype=torch.float64, device=dev)
            w = written[uid]
            sums.index_add_(0, row_id[w], fd.mass[uid[w]].double())
            rows_on = d["active"][j] != 0
            has_res = torch.zeros(d["n_rows"], dtype=torch.bool, device=dev)
            has_res[row_id[w]] = True
            chk = rows_on & has_res
            assert float(sums[chk].min()) > 1.0 - 1e-4 and float(sums[chk].max()) < d["g"] + 1e-3, (j, a)
        fd.ema(j)
        fd.settle()
        in_flight = 0
        fd.prefetch_keys(j)
        fd.select(j)
        torch.cuda.synchronize()
        # what HBM holds beyond the budget goes, at most ride_max units per step
        m = min(want_resident - budget, fd.ride_max)
        assert fd.evict_now == m and int(fd.n_v.item()) == m + fd.P
        n_pairs = min(int(fd.n_pf.item()), fd.P)
        fd.move(j)
        torch.cuda.synchronize()
        # out of the table at once, the bytes leave inside the next scoring launch; the exchange trades one for one
        want_resident -= m
        assert fd.ride is not None and fd.ride[0] == fd.P + m and fd.resident == want_resident
        rides.append((fd.ride_frame[:fd.ride[0]].clone(), fd.ride_host[:fd.ride[0]].clone()))
        in_flight = n_pairs              # out of the table, their partners not yet in
        assert int((fd.state & RES).sum().item()) == want_resident - in_flight
        assert int(fd.n_bad.item()) == 0
    assert rode > 0 and len(rides) <= 1
    fd.flush()
    torch.cuda.synchronize()
    assert fd.ride is None and fd.free_ready == fd.free_tail and int(fd.n_bad.item()) == 0
    assert int((fd.state & RES).sum().item()) == want_resident
