"""Run-to-run determinism: every entry point is run twice from the same inputs, in fresh device
buffers, and all outputs are compared bit for bit: counters, tables, state bytes, victim lists,
staging and pool bytes, spans and windows, digests and store contents, and the floating-point outputs
as well (masses, EMA, priorities, keys), since no kernel accumulates floats with atomics."""
import numpy as np
import pytest
import torch

from paper_2604_26968_amd import synth
from tests.harness import DeviceCase

pytestmark = pytest.mark.gpu

RES, HOST, PROT, SCORED = 1, 2, 4, 8


def _t(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _whole_path(shape, seed):
    """One pass over every entry point; returns {name: numpy array} of everything that was written."""
    from paper_2604_26968_amd import kvm
    out = {}
    case = synth.make_case(shape, seed=seed, pair_weights=synth.categorical_weights(seed + 1), poison_tail=True)
    dev = DeviceCase(case)
    n, n_rows = case.n_uids, case.n_rows
    L = shape.n_layers
    rec = dev.rec
    rng = np.random.default_rng(seed + 2)
    ev = synth.make_events(5000, seed + 3, pair_weights=synth.categorical_weights(seed + 4),
                           reuse_prob=np.linspace(0.1, 0.9, 16))
    ev_p, ev_o = _t(ev[0]), _t(ev[1])

    # posteriors, plain and blended
    kvm.kvm_beta_update(ev_p, ev_o, dev.hits, dev.misses, dev.p_hat, n_bad=dev.n_bad)
    out["hits"], out["misses"], out["p_hat"] = dev.hits, dev.misses, dev.p_hat.clone()
    win = torch.full((16, 64), 255, dtype=torch.uint8, device="cuda")
    win_head = torch.zeros(16, dtype=torch.int32, device="cuda")
    conf, p_blend = torch.zeros(16, device="cuda"), torch.zeros(16, device="cuda")
    h2, m2 = torch.zeros(16, dtype=torch.int32, device="cuda"), torch.zeros(16, dtype=torch.int32, device="cuda")
    kvm.kvm_beta_blend_update(ev_p, ev_o, h2, m2, win, win_head, 32.0, dev.p_hat, conf, p_blend, n_bad=dev.n_bad)
    out.update(win=win, win_head=win_head, conf=conf, p_blend=p_blend, hits2=h2, misses2=m2)

    # scoring with a third of the units out of HBM, then both EMA kernels
    gone = rng.random(n) < 0.33
    gone &= (case.state & PROT) == 0
    tbl = case.slot_tbl.copy()
    st = case.state.copy()
    host_slot = np.cumsum(gone) - 1
    tbl[gone] = (-1 - host_slot[gone]).astype(np.int32)
    st[gone] = (st[gone] & ~np.uint8(RES)) | HOST
    frames_gone = case.slot_tbl[gone]
    dev.slot_tbl.copy_(_t(tbl))
    dev.state.copy_(_t(st))
    q = _t(synth.make_queries(case, seed + 5).view(np.int16))
    scale = 1.0 / float(np.sqrt(shape.dim))
    dev.mass.fill_(-1.0)
    kvm.kvm_score_step(dev.pool, dev.rows(), q, scale, dev.mass, dev.ws)
    out["mass"] = dev.mass.clone()
    kvm.kvm_ema_update(dev.rows(), dev.mass, 0.9, dev.row_weight, dev.pair, dev.p_hat, dev.state, dev.S, dev.prio)
    out["S"], out["prio"], out["state_after_ema"] = dev.S.clone(), dev.prio.clone(), dev.state.clone()
    head_idx = _t(synth.row_head_index(case))
    ex = kvm.make_ema_ex(0.999, _t(case.row_seq), head_idx,
                         _t(rng.choice(np.array([0, 1, 2, 3, 255], np.uint8), len(shape.seq_lens))),
                         _t((0.5 + rng.random((4, L * shape.n_kv_heads))).astype(np.float32)))
    S2, prio2 = dev.S.clone(), dev.prio.clone()
    kvm.kvm_ema_update_ex(dev.rows(), dev.mass, 0.9, ex, dev.row_weight, dev.pair, p_blend, dev.state, S2, prio2)
    out["S_ex"], out["prio_ex"] = S2, prio2

    # spans, windows, prefetch keys
    row_layer = _t(synth.row_layer_index(case))
    span_sum = torch.zeros(L, dtype=torch.int64, device="cuda")
    span_cnt = torch.zeros(L, dtype=torch.int32, device="cuda")
    window = torch.full((L,), 64, dtype=torch.int32, device="cuda")
    ws_span = torch.full((max(kvm.kvm_workspace_bytes(kvm.OP_SPAN, n, n_rows), 256),), 0x7F, dtype=torch.uint8,
                         device="cuda")
    kvm.kvm_span_update(dev.rows(), row_layer, dev.mass, dev.state, 9, 10, span_sum, span_cnt, 16, 4096, window,
                        ws_span)
    out.update(span_sum=span_sum, span_cnt=span_cnt, window=window)
    key = torch.zeros(n, device="cuda")
    cand = torch.zeros(n, dtype=torch.uint8, device="cuda")
    kvm.kvm_prefetch_keys(dev.rows(), row_layer, dev.row_ntok, window, dev.state, dev.pair, p_blend, 0.999, key, cand)
    out.update(key=key, cand=cand)

    # selections: victims (workspace and built-in scratch), prefetch list
    k = int((st & RES).sum()) // 5
    vic = torch.full((n,), -1, dtype=torch.int64, device="cuda")
    vic_s = torch.full((n,), -1, dtype=torch.int64, device="cuda")
    n_s = torch.zeros(1, dtype=torch.int64, device="cuda")
    kvm.kvm_select_victims(dev.prio, dev.state, vic, dev.n_victims, dev.ws, k=k)
    kvm.kvm_select_victims_static(dev.prio, dev.state, vic_s, n_s, k=k)
    pf = torch.full((n,), -1, dtype=torch.int64, device="cuda")
    n_pf = torch.zeros(1, dtype=torch.int64, device="cuda")
    kvm.kvm_select_victims(key, cand, pf, n_pf, dev.ws, k=k)
    torch.cuda.synchronize()
    nv, npf = int(dev.n_victims.item()), int(n_pf.item())
    assert nv == k and npf > 0 and bool((vic == vic_s).all())
    out.update(victims=vic, prefetch_list=pf, n_prefetch=n_pf)

    # the host tier holds the records of the units taken out above (their frames' bytes)
    n_tier = int(gone.sum())
    tier = torch.empty(n_tier * rec, dtype=torch.uint8).pin_memory()
    tv = tier.numpy().reshape(n_tier, rec)
    tv[:, :shape.unit_k_bytes] = case.k_pool.view(np.uint8).reshape(case.n_slots, -1)[frames_gone]
    if shape.unit_v_bytes:
        tv[:, shape.unit_k_bytes:] = case.v_pool.view(np.uint8).reshape(case.n_slots, -1)[frames_gone]

    # hashes of the victims and the content store
    digests = torch.zeros((nv, 32), dtype=torch.uint8, device="cuda")
    kvm.kvm_hash_units(dev.pool, dev.slot_tbl, dev.state, vic[:nv].contiguous(), nv, digests, n_bad=dev.n_bad)
    store = kvm.make_store(1 << 12)
    canon = torch.zeros(nv, dtype=torch.int64, device="cuda")
    kvm.kvm_dedup_insert(store, digests, vic[:nv].contiguous(), nv, canon, torch.zeros(nv, dtype=torch.int64, device="cuda"))
    kvm.kvm_dedup_release(store, digests[: nv // 2].contiguous(), nv // 2, n_bad=dev.n_bad)
    # Which place of the open-addressing table an entry lands in depends on which of two colliding
    # digests claims a place first; what the store holds does not: compare it as a set ordered by tag.
    order = torch.argsort(store.tensors["tag"])
    out.update(digests=digests, canon=canon, store_tag=store.tensors["tag"][order],
               store_refs=store.tensors["refs"][order], store_canon=store.tensors["canon"][order])

    # exchange in one call (first half of the pairs), then in three parts riding along with a scoring launch
    m = min(nv, npf) // 2
    a_out, a_in = vic[:m].contiguous(), pf[:m].contiguous()
    kvm.kvm_exchange(dev.pool, dev.slot_tbl, dev.state, a_out, a_in, m, tier, n_bad=dev.n_bad)
    b_out, b_in = vic[m:2 * m].contiguous(), pf[m:2 * m].contiguous()
    xf_frame = torch.full((m,), -1, dtype=torch.int32, device="cuda")
    xf_host = torch.full((m,), -1, dtype=torch.int64, device="cuda")
    kvm.kvm_exchange_begin(dev.pool, dev.slot_tbl, dev.state, b_out, b_in, m, n_tier, xf_frame, xf_host,
                           n_bad=dev.n_bad)
    dev.mass.fill_(-1.0)
    kvm.kvm_score_step_xfer(dev.pool, dev.rows(), q, scale, dev.mass, dev.ws, xf_frame, xf_host, m, tier)
    kvm.kvm_exchange_end(dev.slot_tbl, dev.state, b_in, xf_frame, m)
    torch.cuda.synchronize()
    out.update(mass_xfer=dev.mass.clone(), xf_frame=xf_frame, xf_host=xf_host, tbl_after_exchange=dev.slot_tbl.clone(),
               state_after_exchange=dev.state.clone(), tier_after_exchange=torch.from_numpy(tier.numpy().copy()))

    # pack / unpack (staged and zero-copy) and the fused swap on what is resident now
    res_now = torch.nonzero(dev.state & RES).flatten()
    res_now = res_now[(dev.state[res_now] & PROT) == 0]
    p_uids = res_now[: 3 * 37].contiguous()
    cnt = 37
    hs = torch.arange(cnt, dtype=torch.int32, device="cuda")
    freed = torch.full((3 * cnt,), -9, dtype=torch.int32, device="cuda")
    host_a = torch.zeros(cnt * rec, dtype=torch.uint8).pin_memory()
    host_b = torch.zeros(cnt * rec, dtype=torch.uint8).pin_memory()
    host_c = torch.zeros(cnt * rec, dtype=torch.uint8).pin_memory()
    sdev = torch.zeros(8 * rec, dtype=torch.uint8, device="cuda")
    kvm.kvm_pack(dev.pool, dev.slot_tbl, dev.state, p_uids[:cnt].contiguous(), cnt, hs, freed[:cnt], sdev, host_a,
                 n_bad=dev.n_bad)
    kvm.kvm_pack(dev.pool, dev.slot_tbl, dev.state, p_uids[cnt:2 * cnt].contiguous(), cnt, hs, freed[cnt:2 * cnt],
                 None, host_b, n_bad=dev.n_bad)
    torch.cuda.synchronize()
    # swap: the third group leaves, the first comes back into the frames it frees
    kvm.kvm_swap(dev.pool, dev.slot_tbl, dev.state, p_uids[2 * cnt:].contiguous(), p_uids[:cnt].contiguous(), cnt, hs,
                 freed[2 * cnt:], host_c, host_a, n_bad=dev.n_bad)
    # the second group comes back into its own old frames through device staging
    kvm.kvm_unpack(dev.pool, dev.slot_tbl, dev.state, p_uids[cnt:2 * cnt].contiguous(), cnt,
                   freed[cnt:2 * cnt].contiguous(), sdev, host_b, n_bad=dev.n_bad)
    torch.cuda.synchronize()
    out.update(staging_a=torch.from_numpy(host_a.numpy().copy()), staging_b=torch.from_numpy(host_b.numpy().copy()),
               staging_c=torch.from_numpy(host_c.numpy().copy()), freed=freed.clone(), tbl_swapped=dev.slot_tbl.clone(),
               state_swapped=dev.state.clone())

    # eviction in two parts riding in a scoring launch, the selection with the built-in scratch
    res_now = torch.nonzero(dev.state & RES).flatten()
    res_now = res_now[(dev.state[res_now] & PROT) == 0]
    e_uids = res_now[-29:].contiguous()
    e_slots = torch.arange(n_tier - 29, n_tier, dtype=torch.int32, device="cuda")       # records nobody needs any more
    e_frame = torch.full((29,), -1, dtype=torch.int32, device="cuda")
    e_host = torch.full((29,), -1, dtype=torch.int64, device="cuda")
    kvm.kvm_pack_begin(dev.pool, dev.slot_tbl, dev.state, e_uids, 29, e_slots, n_tier, e_frame, e_host, n_bad=dev.n_bad)
    dev.mass.fill_(-1.0)
    kvm.kvm_score_step_xfer(dev.pool, dev.rows(), q, scale, dev.mass, dev.ws, e_frame, e_host, 29, tier)
    v2 = torch.full((n,), -1, dtype=torch.int64, device="cuda")
    nv2 = torch.zeros(1, dtype=torch.int64, device="cuda")
    kvm.kvm_select_victims_static(dev.prio, dev.state, v2, nv2, k=n // 7)
    torch.cuda.synchronize()
    out.update(e_frame=e_frame, e_host=e_host, mass_evict=dev.mass.clone(), victims_static=v2, n_victims_static=nv2,
               tier_after_evict=torch.from_numpy(tier.numpy().copy()))

    # frames shared by duplicates: copy the frames of a few units over others, hash, insert, share, unshare
    res_now = torch.nonzero(dev.state & RES).flatten()
    res_now = res_now[(dev.state[res_now] & PROT) == 0][:40].contiguous()
    fr = dev.slot_tbl[res_now].long()
    for grp in range(8):                                   # groups of five units with the content of their first
        dev.k_pool[fr[5 * grp + 1:5 * grp + 5]] = dev.k_pool[fr[5 * grp]].clone()
        if dev.v_pool is not None:
            dev.v_pool[fr[5 * grp + 1:5 * grp + 5]] = dev.v_pool[fr[5 * grp]].clone()
    d2 = torch.zeros((40, 32), dtype=torch.uint8, device="cuda")
    kvm.kvm_hash_units(dev.pool, dev.slot_tbl, dev.state, res_now, 40, d2, n_bad=dev.n_bad)
    store2 = kvm.make_store(1 << 8)
    canon2 = torch.zeros(40, dtype=torch.int64, device="cuda")
    kvm.kvm_dedup_insert(store2, d2, res_now, 40, canon2, torch.zeros(40, dtype=torch.int64, device="cuda"))
    refs = torch.zeros(case.n_slots, dtype=torch.int32, device="cuda")
    given = torch.full((40,), -9, dtype=torch.int32, device="cuda")
    kvm.kvm_dedup_share(dev.slot_tbl, dev.state, case.n_slots, res_now, canon2, 40, refs, given, n_bad=dev.n_bad)
    torch.cuda.synchronize()
    out.update(canon2=canon2, given=given.clone(), refs_shared=refs.clone(), tbl_shared=dev.slot_tbl.clone(),
               state_shared=dev.state.clone())
    sharers = torch.nonzero((dev.state & 16) != 0).flatten().contiguous()
    ns = sharers.numel()
    new_frames = given[given >= 0]
    extra = e_frame[e_frame >= 0]                          # frames the eviction above left free
    new_frames = torch.cat([new_frames, extra])[:ns].contiguous()
    back = torch.full((ns,), -9, dtype=torch.int32, device="cuda")
    kvm.kvm_dedup_unshare(dev.pool, dev.slot_tbl, dev.state, sharers, new_frames, ns, refs, back, n_bad=dev.n_bad)
    torch.cuda.synchronize()
    # which of a frame's last readers reports it free may differ from run to run: compare the frames as a set
    out.update(back_sorted=torch.sort(back).values, refs_final=refs, tbl_final=dev.slot_tbl, state_final=dev.state,
               k_pool_final=dev.k_pool, n_bad=dev.n_bad)
    assert ns == 40 and int((given >= 0).sum().item()) == 32 and not bool(refs.any().item())
    if dev.v_pool is not None:
        out["v_pool_final"] = dev.v_pool
    torch.cuda.synchronize()
    return {name: t.detach().cpu().numpy().copy() for name, t in out.items()}


@pytest.mark.parametrize("shape", [
    synth.Shape(2, 8, 2, 128, synth.BF16, True, [3000, 777, 9100]),       # rows of several tiles (g 4)
    synth.Shape(2, 32, 1, 128, synth.BF16, True, [2500, 640]),            # matrix-core scorer (g 32)
    synth.Shape(2, 128, 1, 576, synth.BF16, False, [1500, 333]),          # latent rows, no V
], ids=["gqa", "mqa", "mla"])
def test_two_runs_give_identical_bits(shape):
    first = _whole_path(shape, seed=70)
    second = _whole_path(shape, seed=70)
    assert first.keys() == second.keys()
    assert int(first["n_bad"][0]) == 0
    for name in first:
        a, b = first[name], second[name]
        assert a.shape == b.shape and a.dtype == b.dtype, name
        assert np.array_equal(a.view(np.uint8), b.view(np.uint8)), name
    assert (first["victims"] >= 0).sum() > 10 and first["hits"].sum() > 0
