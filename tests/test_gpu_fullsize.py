"""Parity at the benchmark's full size and launch configuration (Llama-3-8B-shaped
workload: 5.4 M units, 22 GB of K and as much V), on outputs the oracle can
compute: sampled rows for the scorer and the EMA, the whole array for the
counters and the victim set, sampled records for pack / unpack."""
import numpy as np
import pytest
import torch

from paper_2604_26968_amd import synth

pytestmark = pytest.mark.gpu

RES, HOST, PROT, SCORED = 1, 2, 4, 8


def test_llama8b_shaped_full_size(oracle):
    from paper_2604_26968_amd import kvm
    free, _ = torch.cuda.mem_get_info()
    if free < 60 * 2**30:
        pytest.skip("needs 60 GiB of free HBM")
    dev = "cuda"
    shape = synth.llama8b_shape(64, seed=2)
    pair_w = synth.categorical_weights(3)
    wl = synth.DeviceWorkload(shape, seed=1, pair_weights=pair_w)
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

    kvm.kvm_ema_update(rows, mass, 0.95, wl.row_weight, wl.pair, p_hat, wl.state, S, prio)
    torch.cuda.synchronize()
    S_ref, prio_ref, st_ref = np.zeros(case.n_uids, np.float32), np.zeros(case.n_uids, np.float32), case.state.copy()
    oracle.ema_update(case.row_ntok, case.row_off, ref_mass, 0.95, case.row_weight, case.pair, op, st_ref, S_ref,
                      prio_ref)
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
