"""The scorer's path for launches made of long rows (at least 256 rows of 2,048 blocks on average: one large
workgroup per row, block values kept in LDS, no plan and no row merge), against the oracle on rows of every kind:
one to 9,000 blocks, ragged tails, half evicted, fully resident (more block values than the LDS holds: the
spill path), fully evicted, inactive; every group size of the path, both aggregations, and with the bytes of a
deferred exchange riding along."""
import numpy as np
import pytest
import torch

from paper_2604_26968_amd import synth

pytestmark = pytest.mark.gpu

RES, HOST, PROT = 1, 2, 4


def _lengths(n_seq, seed):
    """Token counts: mostly 30k-70k, plus the special cases; mean above 2,048 blocks."""
    rng = np.random.default_rng(seed)
    lens = [int(v) for v in rng.integers(30000, 70000, size=n_seq)]
    lens[0], lens[1], lens[2], lens[3], lens[4] = 1, 17, 16 * 4096, 16 * 4096 + 1, 144000
    lens[5] = 70001
    return lens


@pytest.mark.parametrize("n_q,dim,dtype,agg", [(64, 128, synth.BF16, 0), (32, 64, synth.FP16, 1), (8, 64, synth.BF16, 0),
                                               (16, 32, synth.FP16, 0)],
                         ids=["g8-d128-bf16-max", "g4-d64-fp16-mean", "g1-d64-bf16-max", "g2-d32-fp16-max"])
def test_long_rows_in_one_workgroup_each(oracle, n_q, dim, dtype, agg):
    from paper_2604_26968_amd import kvm
    dev = "cuda"
    n_kv = 8
    shape = synth.Shape(1, n_q, n_kv, dim, dtype, True, _lengths(36, 3))
    wl = synth.DeviceWorkload(shape, seed=4)
    n, n_rows, g = wl.n_uids, wl.n_rows, shape.g
    assert n_rows >= 256 and n // n_rows >= 2048          # what sends the launch down this path
    pool = kvm.make_pool(wl.k_pool.view(torch.int16), wl.v_pool.view(torch.int16), dim, dtype)
    scale = float(np.float32(1.0 / np.sqrt(dim)))
    # residency: half of everything out at random; sequence 7 stays whole (more resident blocks than fit the LDS
    # for g 8), sequence 8 leaves completely, the 144,000-token rows keep everything (several segments + spill)
    drop = torch.rand(n, generator=wl.gen, device=dev) < 0.5
    row_seq = torch.from_numpy(wl.row_seq).to(dev)
    uid_row = torch.repeat_interleave(torch.arange(n_rows, device=dev), torch.from_numpy(wl.nb).to(dev))
    uid_seq = row_seq[uid_row]
    drop[(uid_seq == 7) | (uid_seq == 4)] = False
    drop[uid_seq == 8] = True
    wl.slot_tbl[drop] = -1
    wl.state[drop] = HOST
    active = np.ones(n_rows, np.uint8)
    active[n_kv * 9:n_kv * 10] = 0                        # sequence 9 does not decode
    row_active = torch.from_numpy(active).to(dev)
    rows = kvm.make_rows(wl.row_ntok, wl.row_off, wl.row_q_off, wl.slot_tbl, g, wl.q_elems, row_active)
    ws = torch.full((kvm.kvm_workspace_bytes(kvm.OP_SCORE, n, n_rows, g, dim),), 0x7F, dtype=torch.uint8, device=dev)
    q = wl.queries(21)
    mass = torch.full((n,), -1.0, dtype=torch.float32, device=dev)
    kvm.kvm_score_step(pool, rows, q, scale, mass, ws, agg=agg)
    torch.cuda.synchronize()

    # the oracle on every second row plus the special ones
    pick = np.unique(np.concatenate([np.arange(0, n_rows, 2), np.arange(0, n_kv * 10)]))
    case = wl.host_sample(rows=pick)
    qh = q.view(torch.int16).cpu().numpy().view(np.uint16)
    q_rows = np.concatenate([qh[r * g * dim:(r + 1) * g * dim] for r in case.sample_rows])
    ref = np.full(case.n_uids, -1.0, np.float32)
    oracle.score_step(case.k_pool, dim, dtype, case.row_ntok, case.row_off, case.row_q_off, case.slot_tbl, q_rows, g,
                      scale, ref, agg=agg, row_active=active[pick])
    got = mass[torch.from_numpy(case.sample_uids).to(dev)].cpu().numpy()
    res = ref >= 0
    assert res.sum() > 100000
    np.testing.assert_allclose(got[res], ref[res], rtol=1e-3, atol=1e-9)
    np.testing.assert_array_equal(got[~res], -1.0)
    # over the whole array: exactly the resident units of decoding rows were written
    resident = wl.slot_tbl >= 0
    decoding = row_active[uid_row] != 0
    assert bool(((mass >= 0) == (resident & decoding)).all())
    if agg == 1:            # per-query masses sum to 1 over the resident blocks of a row, so does their mean
        sums = torch.zeros(n_rows, dtype=torch.float64, device=dev)
        w = mass >= 0
        sums.index_add_(0, uid_row[w], mass[w].double())
        has = torch.zeros(n_rows, dtype=torch.bool, device=dev)
        has[uid_row[w]] = True
        assert float((sums[has] - 1.0).abs().max()) < 1e-4

    # ---- the same launch with the bytes of a deferred exchange riding along -----------------------------------
    rec = shape.unit_k_bytes + shape.unit_v_bytes
    m = 700
    res_ids = torch.nonzero(resident & ((wl.state & PROT) == 0)).flatten()
    sel = res_ids[torch.randperm(res_ids.numel(), generator=wl.gen, device=dev)[:2 * m]]
    out_a, out_b = sel[:m].contiguous(), sel[m:].contiguous()
    tier = torch.zeros(2 * m * rec, dtype=torch.uint8).pin_memory()
    n_bad = torch.zeros(1, dtype=torch.int32, device=dev)
    freed = torch.full((m,), -1, dtype=torch.int32, device=dev)
    kvm.kvm_pack(pool, wl.slot_tbl, wl.state, out_a, m, torch.arange(m, dtype=torch.int32, device=dev), freed, None,
                 tier[:m * rec], n_bad=n_bad)
    torch.cuda.synchronize()
    rec_a = tier[:m * rec].clone().numpy().reshape(m, rec)
    frames_b = wl.slot_tbl[out_b].clone()
    k_b = wl.k_pool[frames_b.long()].view(torch.uint8).cpu().numpy().reshape(m, -1)
    v_b = wl.v_pool[frames_b.long()].view(torch.uint8).cpu().numpy().reshape(m, -1)
    xf_frame = torch.full((m,), -1, dtype=torch.int32, device=dev)
    xf_host = torch.full((m,), -1, dtype=torch.int64, device=dev)
    kvm.kvm_exchange_begin(pool, wl.slot_tbl, wl.state, out_b, out_a, m, 2 * m, xf_frame, xf_host, n_bad=n_bad)
    mass2 = torch.full((n,), -1.0, dtype=torch.float32, device=dev)
    ws.fill_(0x7F)
    kvm.kvm_score_step_xfer(pool, rows, q, scale, mass2, ws, xf_frame, xf_host, m, tier, agg=agg)
    kvm.kvm_exchange_end(wl.slot_tbl, wl.state, out_a, xf_frame, m)
    torch.cuda.synchronize()
    assert int(n_bad.item()) == 0
    # frames of out_b now hold out_a's records, the tier slots hold out_b's old frames
    got_k = wl.k_pool[frames_b.long()].view(torch.uint8).cpu().numpy().reshape(m, -1)
    got_v = wl.v_pool[frames_b.long()].view(torch.uint8).cpu().numpy().reshape(m, -1)
    np.testing.assert_array_equal(got_k, rec_a[:, :shape.unit_k_bytes])
    np.testing.assert_array_equal(got_v, rec_a[:, shape.unit_k_bytes:])
    tier_now = tier.numpy().reshape(2 * m, rec)[:m]
    np.testing.assert_array_equal(tier_now[:, :shape.unit_k_bytes], k_b)
    np.testing.assert_array_equal(tier_now[:, shape.unit_k_bytes:], v_b)
    # neither side of a pair was in HBM for the scorer; every other unit got the same mass as before (rows that
    # lost a unit to the exchange are renormalised over what is left: compare the untouched rows bit for bit)
    touched_rows = torch.zeros(n_rows, dtype=torch.bool, device=dev)
    touched_rows[uid_row[torch.cat([out_a, out_b])]] = True
    same = ~touched_rows[uid_row]
    assert bool((mass2[torch.cat([out_a, out_b])] == -1.0).all())
    assert bool((mass2[same] == mass[same]).all())
    assert int(same.sum().item()) > 0

    # ---- and with evictions in two parts: kvm_pack_begin, the frames copied out by the scoring launch ---------
    m2 = 300
    res2 = torch.nonzero((wl.slot_tbl >= 0) & ((wl.state & PROT) == 0)).flatten()
    out_c = res2[torch.randperm(res2.numel(), generator=wl.gen, device=dev)[:m2]].contiguous()
    frames_c = wl.slot_tbl[out_c].clone()
    k_c = wl.k_pool[frames_c.long()].view(torch.uint8).cpu().numpy().reshape(m2, -1)
    v_c = wl.v_pool[frames_c.long()].view(torch.uint8).cpu().numpy().reshape(m2, -1)
    slots_c = torch.arange(m, m + m2, dtype=torch.int32, device=dev)
    pf_frame = torch.full((m2,), -1, dtype=torch.int32, device=dev)
    pf_host = torch.full((m2,), -1, dtype=torch.int64, device=dev)
    kvm.kvm_pack_begin(pool, wl.slot_tbl, wl.state, out_c, m2, slots_c, 2 * m, pf_frame, pf_host, n_bad=n_bad)
    mass3 = torch.full((n,), -1.0, dtype=torch.float32, device=dev)
    ws.fill_(0x7F)
    kvm.kvm_score_step_xfer(pool, rows, q, scale, mass3, ws, pf_frame, pf_host, m2, tier, agg=agg)
    torch.cuda.synchronize()
    assert int(n_bad.item()) == 0
    assert bool((pf_frame == frames_c).all()) and bool((pf_host == (slots_c.long() | kvm.XFER_OUT_ONLY)).all())
    assert bool((wl.slot_tbl[out_c] == -1 - slots_c).all())
    assert bool(((wl.state[out_c] & 3) == 2).all())
    tier_c = tier.numpy().reshape(2 * m, rec)[m:m + m2]
    np.testing.assert_array_equal(tier_c[:, :shape.unit_k_bytes], k_c)
    np.testing.assert_array_equal(tier_c[:, shape.unit_k_bytes:], v_c)
    assert bool((mass3[out_c] == -1.0).all())
    touched3 = torch.zeros(n_rows, dtype=torch.bool, device=dev)
    touched3[uid_row[out_c]] = True
    same3 = ~(touched3 | touched_rows)[uid_row]         # rows none of the three lists touched
    assert bool((mass3[same3] == mass[same3]).all()) and int(same3.sum().item()) > 0
