#!/usr/bin/env python3
"""Benchmark of the per-decode-step KV-cache management pass on one MI355X.

One step = beta update -> scoring of every resident unit -> EMA + priority ->
budget victim selection -> pack of the victims to pinned host -> unpack of an
equal number of host units into the freed frames, all through the C ABI.  The
kernels run on one stream; the host-link copies of the swapped records run on a
side stream and overlap the scoring of the same / the following step.  Workload: the Llama-3-8B-shaped configuration (32 layers, 32 q / 8 KV
heads, d 128, bf16, 64 sequences of uniform [2048, 8192] tokens, block 16,
EMA decay 0.95, budget = 60 % of the initially resident units, 4096 reuse
events per step).  Prints one JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0        # MI355X HBM3E published peak

# name -> (description, shape builder, default sequences, budget fraction, EMA decay, swap units per step,
#          rows sampled for the CPU baseline (None = all rows of `sample_seqs` sequences), sample_seqs)
WORKLOADS = {
    "llama8b": ("llama3-8b-shaped GQA: 32 layers, 32q/8kv heads, d128, bf16, %d seqs U[2048,8192] tok",
                lambda synth, n: synth.llama8b_shape(n, seed=2), 64, 0.60, 0.95, 1024, None, 32),
    "llama70b": ("llama3-70b-shaped GQA (one GPU's share): 80 layers, 64q/8kv heads, d128, bf16, %d x 131072 tok",
                 lambda synth, n: synth.llama70b_shape(n), 4, 0.50, 0.95, 4096, 64, 0),
    "mla": ("deepseek-v3-shaped MLA: 61 layers, 576-channel latent, 128 absorbed queries, bf16, %d x 32768 tok",
            lambda synth, n: synth.mla_shape(n), 32, 0.40, 0.90, 1024, 2, 0),
    # the two halves of the fleet configuration, each on its own (prompt lengths lognormal(7, 1))
    "mha": ("fleet, MHA half: 32 layers, 32q/32kv heads (g 1), d128, bf16, %d seqs lognormal(7,1) tok",
            lambda synth, n: synth.mha_fleet_shape(n), 72, 0.60, 0.90, 1024, 32768, 0),
    "mqa": ("fleet, MQA half: 32 layers, 32q/1kv head (g 32), d128, bf16, %d seqs lognormal(7,1) tok",
            lambda synth, n: synth.mqa_fleet_shape(n), 1536, 0.60, 0.90, 1024, 8192, 0),
}
# HBM bytes per launch of the tile kernel from rocprofv3 --pmc (FETCH_SIZE x 2 KiB + WRITE_SIZE x 1 KiB), with the
# transfer workgroups of --swap-mode pipelined / overlap riding along; one entry per workload at its default size
# (profiles/score_tile_dot2_llama8b_pmc.md, score_tile_dot2_llama70b_pmc.md, score_tile_wide_mla_pmc.md,
# score_tile_dot2_mha_pmc.md, score_tile_mfma_mqa_pmc.md).
SCORE_TILE_TRAFFIC_BYTES = {
    "llama8b": int(6624641.7 * 2048 + 37636.7 * 1024),       # score_tile_dot2_kernel<4, 128, bf16, 512>
    "llama70b": int(21135248.4 * 2048 + 394499.4 * 1024),    # score_tile_dot2_kernel<8, 128, bf16, 512>
    "mla": int(14707914.7 * 2048 + 840307.0 * 1024),         # score_tile_wide_kernel<576, bf16, 512>
    "mha": int(8385917.2 * 2048 + 38958.0 * 1024),           # score_tile_dot2_kernel<1, 128, bf16, 512>
    "mqa": int(7100460.9 * 2048 + 77685.8 * 1024),           # score_tile_mfma_kernel<2, 128, bf16, 256>
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", choices=sorted(WORKLOADS), default="llama8b",
                    help="llama8b is the named benchmark workload; the others are the larger configurations")
    ap.add_argument("--n-seq", type=int, default=0, help="sequences in the batch (0 = the workload's own number)")
    ap.add_argument("--swap-units", type=int, default=0, help="units evicted and prefetched per step (0 = workload default)")
    ap.add_argument("--swap-mode", choices=["pipelined", "overlap", "fused", "staged", "direct", "side-stream"], default="pipelined",
                    help="how the per-step victims / prefetch records cross the host link: in-place exchange whose "
                         "bytes move inside the next step's scoring launch (kvm_exchange_begin / "
                         "kvm_score_step_xfer / kvm_exchange_end), with the selection on a second stream beside "
                         "the scoring launch; the same with the selection in line after the EMA; "
                         "one fused two-way zero-copy kernel after the "
                         "selection (kvm_swap); kvm_pack then kvm_unpack through device staging and hipMemcpyAsync; "
                         "the same with zero-copy kernels; or gather / scatter in line with the copies on a side "
                         "stream")
    ap.add_argument("--refined", action="store_true",
                    help="run the pass with the refinements switched on: blended reuse estimate, EMA with "
                         "positional decay and transition multipliers, attention-span windows, and a prefetch list "
                         "chosen on the device (keys + select) and served by the in-place exchange with a "
                         "slot-addressed host tier")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB read + 1 GiB write elementwise kernel (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only (the pass has no cross-GPU step); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2604_26968_amd import kvm, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = "cuda"
    t_setup = time.time()
    wdesc, wshape, w_nseq, w_budget, decay, w_swap, w_sample_rows, w_sample_seqs = WORKLOADS[args.workload]
    n_seq = args.n_seq or w_nseq
    shape = wshape(synth, n_seq)
    pair_w = synth.categorical_weights(3)
    reuse_p = np.linspace(0.15, 0.95, 16)
    # the pool is dimensioned by the sizing call: units per token block x blocks of the batch, at the unit
    # bytes it reports
    blocks = sum((int(t) + 15) // 16 for t in shape.seq_lens)
    sizing = kvm.kvm_size(**shape.model_args(), n_max=max(shape.seq_lens))
    sizing = kvm.kvm_size(**shape.model_args(), n_max=max(shape.seq_lens),
                          mem_target=blocks * sizing["units_per_block"] * (sizing["unit_k_bytes"] + sizing["unit_v_bytes"]))
    assert (sizing["unit_k_bytes"], sizing["unit_v_bytes"], sizing["group_size"]) == \
        (shape.unit_k_bytes, shape.unit_v_bytes, shape.g)
    wl = synth.DeviceWorkload(shape, seed=1, pair_weights=pair_w, pool_units=sizing["pool_units"])
    n, n_rows, g, dim = wl.n_uids, wl.n_rows, shape.g, shape.dim
    assert n == sizing["pool_units"]
    rec = shape.unit_k_bytes + shape.unit_v_bytes
    pool = kvm.make_pool(wl.k_pool.view(torch.int16), None if wl.v_pool is None else wl.v_pool.view(torch.int16), dim,
                         shape.dtype)
    rows = kvm.make_rows(wl.row_ntok, wl.row_off, wl.row_q_off, wl.slot_tbl, g, wl.q_elems)
    scale = 1.0 / float(np.sqrt(dim))
    row_weight = torch.full((n_rows,), float(sizing["head_weight"]), dtype=torch.float32, device=dev)

    mass = torch.zeros(n, dtype=torch.float32, device=dev)
    S = torch.zeros(n, dtype=torch.float32, device=dev)
    prio = torch.zeros(n, dtype=torch.float32, device=dev)
    hits = torch.zeros(16, dtype=torch.int32, device=dev)
    misses = torch.zeros(16, dtype=torch.int32, device=dev)
    p_hat = torch.zeros(16, dtype=torch.float32, device=dev)
    n_bad = torch.zeros(1, dtype=torch.int32, device=dev)
    n_victims = torch.zeros(1, dtype=torch.int64, device=dev)
    ws_bytes = max(kvm.kvm_workspace_bytes(kvm.OP_SCORE, n, n_rows, g, dim),
                   kvm.kvm_workspace_bytes(kvm.OP_SELECT, n))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    # a selection that runs beside a scoring launch needs a workspace of its own
    ws_select = torch.empty(max(kvm.kvm_workspace_bytes(kvm.OP_SELECT, n), 256), dtype=torch.uint8, device=dev)

    n_q_sets = 4
    qs = [wl.queries(100 + i) for i in range(n_q_sets)]
    evs = []
    for i in range(n_q_sets):
        p, o = synth.make_events(4096, 200 + i, pair_weights=pair_w, reuse_prob=reuse_p)
        evs.append((torch.from_numpy(p).to(dev), torch.from_numpy(o).to(dev)))

    n_res0 = int((wl.state & 1).sum().item())
    budget = int(w_budget * n_res0)
    k0 = n_res0 - budget
    swap = args.swap_units or w_swap
    total_steps = args.warmup + args.steps
    assert swap * (total_steps + 2) <= k0, "not enough host-resident units for this many steps"
    # Tier 1 keeps the records the later steps prefetch (all of them when they fit 24 GiB of pinned memory);
    # the rest of the bulk eviction goes through a scratch buffer and is dropped, as if demoted further down.
    chunk = min(k0, 32768)
    keep = k0 if k0 * rec <= 24 * 2**30 else ((swap * (total_steps + 2) + chunk - 1) // chunk) * chunk

    victims = torch.zeros(k0, dtype=torch.int64, device=dev)
    freed = torch.full((k0,), -1, dtype=torch.int32, device=dev)
    host_slots = torch.arange(k0, dtype=torch.int32, device=dev)
    host_tier = torch.empty(keep * rec, dtype=torch.uint8, pin_memory=True)    # tier 1
    host_scratch = torch.empty(chunk * rec, dtype=torch.uint8, pin_memory=True) if keep < k0 else None
    staging_dev = torch.empty(chunk * rec, dtype=torch.uint8, device=dev)

    if args.refined:
        L, lh = shape.n_layers, shape.n_layers * shape.n_kv_heads
        rng = np.random.default_rng(17)
        head_idx = (np.arange(n_rows) % lh).astype(np.int32)
        row_layer = torch.from_numpy(head_idx // shape.n_kv_heads).to(dev)
        n_seqs = len(shape.seq_lens)
        ex = kvm.make_ema_ex(0.9995, torch.from_numpy(wl.row_seq).to(dev), torch.from_numpy(head_idx).to(dev),
                             torch.from_numpy(rng.choice(np.array([0, 1, 2, 3, 255], np.uint8), n_seqs)).to(dev),
                             torch.from_numpy((0.5 + rng.random((4, lh))).astype(np.float32)).to(dev))
        win = torch.full((16, 256), 255, dtype=torch.uint8, device=dev)
        win_head = torch.zeros(16, dtype=torch.int32, device=dev)
        conf = torch.zeros(16, dtype=torch.float32, device=dev)
        p_blend = torch.zeros(16, dtype=torch.float32, device=dev)
        span_sum = torch.zeros(L, dtype=torch.int64, device=dev)
        span_cnt = torch.zeros(L, dtype=torch.int32, device=dev)
        layer_window = torch.full((L,), 1 << 30, dtype=torch.int32, device=dev)
        ws_span = torch.empty(max(kvm.kvm_workspace_bytes(kvm.OP_SPAN, n, n_rows), 256), dtype=torch.uint8, device=dev)
        pf_key = torch.zeros(n, dtype=torch.float32, device=dev)
        pf_cand = torch.zeros(n, dtype=torch.uint8, device=dev)
        n_pf = torch.zeros(1, dtype=torch.int64, device=dev)
        swap_units = args.swap_units or w_swap
        store = kvm.make_store(1 << 22)
        digests = torch.zeros((swap_units, 32), dtype=torch.uint8, device=dev)
        canon = torch.zeros(swap_units, dtype=torch.int64, device=dev)
        dedup_ws = torch.zeros(swap_units, dtype=torch.int64, device=dev)

    def management_pass(i, k_arg, budget_arg):
        ev = evs[i % n_q_sets]
        kvm.kvm_beta_update(ev[0], ev[1], hits, misses, p_hat, n_bad=n_bad)
        kvm.kvm_score_step(pool, rows, qs[i % n_q_sets], scale, mass, ws)
        kvm.kvm_ema_update(rows, mass, decay, row_weight, wl.pair, p_hat, wl.state, S, prio)
        kvm.kvm_select_victims(prio, wl.state, victims, n_victims, ws, k=k_arg, budget_units=budget_arg)

    # ---- step 0: everything resident; evict down to the budget in one go ------------------------
    # one untimed scoring pass first: it loads the code objects and leaves no state behind (masses are overwritten)
    kvm.kvm_score_step(pool, rows, qs[0], scale, mass, ws)
    torch.cuda.synchronize()
    setup_s = time.time() - t_setup
    t0 = time.time()
    management_pass(0, -1, budget)
    torch.cuda.synchronize()
    t_pass0 = time.time() - t0
    assert int(n_victims.item()) == k0, (int(n_victims.item()), k0)
    # shuffle the victim list so that later prefetch segments are random samples of the host tier
    perm = torch.randperm(k0, generator=wl.gen, device=dev)
    victims.copy_(victims[perm])
    torch.cuda.synchronize()
    t0 = time.time()
    for lo in range(0, k0, chunk):
        cnt = min(chunk, k0 - lo)
        dst = host_tier[lo * rec:(lo + cnt) * rec] if lo + cnt <= keep else host_scratch
        kvm.kvm_pack(pool, wl.slot_tbl, wl.state, victims[lo:lo + cnt], cnt, host_slots[lo:lo + cnt],
                     freed[lo:lo + cnt], staging_dev, dst, n_bad=n_bad)
    torch.cuda.synchronize()
    t_bulk_pack = time.time() - t0
    host_uids = victims.clone()                 # uid stored in host record i
    free_frames = freed.clone()
    assert int(n_bad.item()) == 0
    assert int((wl.state & 1).sum().item()) == budget

    # bring the first `swap` units back so that every timed step starts `swap` over budget
    def prefetch(seg):
        lo = seg * swap
        kvm.kvm_unpack(pool, wl.slot_tbl, wl.state, host_uids[lo:lo + swap], swap, free_frames[lo:lo + swap],
                       staging_dev, host_tier[lo * rec:(lo + swap) * rec], n_bad=n_bad)

    step_victims = torch.zeros(swap, dtype=torch.int64, device=dev)
    step_freed = torch.full((swap,), -1, dtype=torch.int32, device=dev)
    # Per-step swap traffic goes over a side stream: the prefetch records of step i travel host -> device
    # while step i is being scored, the victims' records device -> host while step i + 1 is being scored.
    # Two staging buffers per direction alternate between steps; events order the buffer reuse.
    main = torch.cuda.current_stream()
    side = torch.cuda.Stream()
    out_dev = [torch.empty(swap * rec, dtype=torch.uint8, device=dev) for _ in range(2)]
    in_dev = [torch.empty(swap * rec, dtype=torch.uint8, device=dev) for _ in range(2)]
    ev_gathered = [torch.cuda.Event() for _ in range(2)]
    ev_d2h = [torch.cuda.Event() for _ in range(2)]
    ev_h2d = [torch.cuda.Event() for _ in range(2)]
    ev_scattered = [torch.cuda.Event() for _ in range(2)]
    for e in ev_d2h + ev_scattered:
        e.record(main)

    pf_list = torch.full((swap,), -1, dtype=torch.int64, device=dev)
    arrived = torch.full((swap,), -1, dtype=torch.int64, device=dev)      # the units that came in one step ago

    xf_frame = torch.full((swap,), -1, dtype=torch.int32, device=dev)
    xf_host = torch.full((swap,), -1, dtype=torch.int64, device=dev)
    xf_in = [host_uids[0:swap]]                 # the in-list of the transfer that is under way
    tier_slots = host_tier.numel() // rec

    def step_overlap(i):
        """The pass with the host-link bytes of step i - 1 moving inside step i's scoring launch.  Units on
        their way in or out are in HBM for nobody meanwhile: the victims of step i - 1 left the table when they
        were chosen, the units fetched for them join it after this step's EMA."""
        ev = evs[i % n_q_sets]
        kvm.kvm_beta_update(ev[0], ev[1], hits, misses, p_hat, n_bad=n_bad)
        kvm.kvm_score_step_xfer(pool, rows, qs[i % n_q_sets], scale, mass, ws, xf_frame, xf_host, swap, host_tier)
        kvm.kvm_ema_update(rows, mass, decay, row_weight, wl.pair, p_hat, wl.state, S, prio)
        kvm.kvm_exchange_end(wl.slot_tbl, wl.state, xf_in[0], xf_frame, swap)
        kvm.kvm_select_victims(prio, wl.state, step_victims, n_victims, ws, k=-1, budget_units=budget)
        nxt = (i + 1) * swap
        xf_in[0] = host_uids[nxt:nxt + swap]
        kvm.kvm_exchange_begin(pool, wl.slot_tbl, wl.state, step_victims, xf_in[0], swap, tier_slots, xf_frame,
                               xf_host, n_out_dev=n_victims, n_bad=n_bad)

    def step_pipelined(i):
        """step_overlap with the selection moved off the critical path: the victims are chosen, from the
        priorities the previous step left, on a second stream beside this step's scoring launch (a small
        kernel there costs the scorer next to nothing; the posterior update goes with it).  They leave HBM
        inside the next step's scoring launch, one step later than in step_overlap.  While the selection
        runs the units of the last exchange are still on their way, so the budget it is given is the
        budget minus what is in flight."""
        ev = evs[i % n_q_sets]
        side.wait_stream(main)
        kvm.kvm_beta_update(ev[0], ev[1], hits, misses, p_hat, n_bad=n_bad, stream=side)
        kvm.kvm_select_victims(prio, wl.state, step_victims, n_victims, ws_select, k=-1, budget_units=budget - swap,
                               stream=side)
        kvm.kvm_score_step_xfer(pool, rows, qs[i % n_q_sets], scale, mass, ws, xf_frame, xf_host, swap, host_tier)
        main.wait_stream(side)
        kvm.kvm_ema_update(rows, mass, decay, row_weight, wl.pair, p_hat, wl.state, S, prio)
        kvm.kvm_exchange_end(wl.slot_tbl, wl.state, xf_in[0], xf_frame, swap)
        nxt = (i + 1) * swap
        xf_in[0] = host_uids[nxt:nxt + swap]
        kvm.kvm_exchange_begin(pool, wl.slot_tbl, wl.state, step_victims, xf_in[0], swap, tier_slots, xf_frame,
                               xf_host, n_out_dev=n_victims, n_bad=n_bad)

    def finish_overlap():
        """Lets the last transfer land (untimed) so that the final state can be checked like the other modes'."""
        kvm.kvm_score_step_xfer(pool, rows, qs[0], scale, mass, ws, xf_frame, xf_host, swap, host_tier)
        kvm.kvm_exchange_end(wl.slot_tbl, wl.state, xf_in[0], xf_frame, swap)

    def step_refined(i):
        """The pass with every refinement on.  The prefetch list comes from the device (candidates inside the
        per-layer window behind the decode position, ranked by blended reuse estimate x positional decay); its
        records and the victims' trade places in the slot-addressed tier while the next step is scored."""
        ev = evs[i % n_q_sets]
        # Content addressing of the units that entered HBM in the previous step (stands in for newly allocated
        # blocks): one SHA-256 chain per unit is 0.5 ms of latency for 16 wavefronts of work, so it runs on a
        # second stream beside the scoring launch (a small compute kernel there costs the scorer 0.01 ms; it
        # was copies on a second stream that slowed it down).  Nobody writes those units meanwhile: they were
        # not yet scored when the last victims were chosen.  Before the first transfer the list holds -1s and
        # every digest is the zero of a skipped unit.
        # The reuse estimates and the victims (from the priorities the previous step left, as in
        # step_pipelined) are worked out on the same stream.
        side.wait_stream(main)
        kvm.kvm_beta_blend_update(ev[0], ev[1], hits, misses, win, win_head, 64.0, p_hat, conf, p_blend, n_bad=n_bad,
                                  stream=side)
        kvm.kvm_select_victims(prio, wl.state, step_victims, n_victims, ws_select, k=-1, budget_units=budget - swap,
                               stream=side)
        kvm.kvm_hash_units(pool, wl.slot_tbl, wl.state, arrived, swap, digests, stream=side)
        kvm.kvm_score_step_xfer(pool, rows, qs[i % n_q_sets], scale, mass, ws, xf_frame, xf_host, swap, host_tier)
        main.wait_stream(side)
        kvm.kvm_dedup_insert(store, digests, arrived, swap, canon, dedup_ws)
        kvm.kvm_ema_update_ex(rows, mass, decay, ex, row_weight, wl.pair, p_blend, wl.state, S, prio)
        kvm.kvm_span_update(rows, row_layer, mass, wl.state, 9, 10, span_sum, span_cnt, 256, 1 << 30, layer_window,
                            ws_span)
        kvm.kvm_exchange_end(wl.slot_tbl, wl.state, pf_list, xf_frame, swap)
        arrived.copy_(pf_list)
        kvm.kvm_prefetch_keys(rows, row_layer, wl.row_ntok, layer_window, wl.state, wl.pair, p_blend, 0.9995,
                              pf_key, pf_cand)
        kvm.kvm_select_victims(pf_key, pf_cand, pf_list, n_pf, ws, k=swap)
        kvm.kvm_exchange_begin(pool, wl.slot_tbl, wl.state, step_victims, pf_list, swap, tier_slots, xf_frame, xf_host,
                               n_out_dev=n_victims, n_in_dev=n_pf, n_bad=n_bad)

    def finish_refined():
        kvm.kvm_score_step_xfer(pool, rows, qs[0], scale, mass, ws, xf_frame, xf_host, swap, host_tier)
        kvm.kvm_exchange_end(wl.slot_tbl, wl.state, pf_list, xf_frame, swap)

    def step_serial(i):
        """One full pass, everything in line on one stream.  Resident units at entry: budget + swap."""
        ev = evs[i % n_q_sets]
        kvm.kvm_beta_update(ev[0], ev[1], hits, misses, p_hat, n_bad=n_bad)
        kvm.kvm_score_step(pool, rows, qs[i % n_q_sets], scale, mass, ws)
        kvm.kvm_ema_update(rows, mass, decay, row_weight, wl.pair, p_hat, wl.state, S, prio)
        kvm.kvm_select_victims(prio, wl.state, step_victims, n_victims, ws, k=-1, budget_units=budget)
        lo = i * swap
        # the segment's old records were prefetched by the previous step, so it is free to take the victims
        if args.swap_mode == "fused":
            nxt = (i + 1) * swap
            kvm.kvm_swap(pool, wl.slot_tbl, wl.state, step_victims, host_uids[nxt:nxt + swap], swap,
                         host_slots[lo:lo + swap], step_freed, host_tier[lo * rec:(lo + swap) * rec],
                         host_tier[nxt * rec:(nxt + swap) * rec], n_bad=n_bad, n_dev=n_victims)
            return
        sd = None if args.swap_mode == "direct" else staging_dev
        kvm.kvm_pack(pool, wl.slot_tbl, wl.state, step_victims, swap, host_slots[lo:lo + swap], step_freed,
                     sd, host_tier[lo * rec:(lo + swap) * rec], n_bad=n_bad, n_dev=n_victims)
        nxt = (i + 1) * swap
        kvm.kvm_unpack(pool, wl.slot_tbl, wl.state, host_uids[nxt:nxt + swap], swap, step_freed, sd,
                       host_tier[nxt * rec:(nxt + swap) * rec], n_bad=n_bad, n_dev=n_victims)

    def step_overlapped(i):
        """Same pass with the host-link copies on the side stream."""
        b = i & 1
        nxt = (i + 1) * swap
        with torch.cuda.stream(side):
            side.wait_event(ev_scattered[b])                         # in_dev[b] was last read two steps ago
            in_dev[b].copy_(host_tier[nxt * rec:(nxt + swap) * rec], non_blocking=True)
            ev_h2d[b].record(side)
        ev = evs[i % n_q_sets]
        kvm.kvm_beta_update(ev[0], ev[1], hits, misses, p_hat, n_bad=n_bad)
        kvm.kvm_score_step(pool, rows, qs[i % n_q_sets], scale, mass, ws)
        kvm.kvm_ema_update(rows, mass, decay, row_weight, wl.pair, p_hat, wl.state, S, prio)
        kvm.kvm_select_victims(prio, wl.state, step_victims, n_victims, ws, k=-1, budget_units=budget)
        lo = i * swap
        main.wait_event(ev_d2h[b])                                   # out_dev[b] has left for the host
        kvm.kvm_pack(pool, wl.slot_tbl, wl.state, step_victims, swap, host_slots[lo:lo + swap], step_freed,
                     out_dev[b], None, n_bad=n_bad, n_dev=n_victims)
        ev_gathered[b].record(main)
        with torch.cuda.stream(side):
            side.wait_event(ev_gathered[b])
            # the segment's old records were prefetched by the previous step, so it is free to take the victims
            host_tier[lo * rec:(lo + swap) * rec].copy_(out_dev[b], non_blocking=True)
            ev_d2h[b].record(side)
        main.wait_event(ev_h2d[b])
        kvm.kvm_unpack(pool, wl.slot_tbl, wl.state, host_uids[nxt:nxt + swap], swap, step_freed, in_dev[b], None,
                       n_bad=n_bad, n_dev=n_victims)
        ev_scattered[b].record(main)

    step = step_overlapped if args.swap_mode == "side-stream" else step_overlap if args.swap_mode == "overlap" \
        else step_pipelined if args.swap_mode == "pipelined" \
        else step_serial
    if args.refined:
        assert keep == k0, "the refined pass addresses the whole host tier by slot"
        step = step_refined
    prefetch(0)
    # the frames of segment 0 came from the bulk list; from now on each step reuses the frames it frees
    torch.cuda.synchronize()
    # The warm-up steps are run with every kernel bracketed by events: that is where the durations of the
    # small kernels come from (the first warm-up step is left out when there are several).  The timed steps
    # bracket the dominant kernel only: an event pair costs a few microseconds on the stream and twenty of
    # them per step were 3 % of the step.
    KERNEL_NAMES = ("score_plan", "score_partial", "score_finalize", "ema_prio", "beta", "select_hist", "select_emit",
                    "pack", "unpack", "swap", "span", "prefetch_keys", "hash", "dedup", "exchange_flip")
    kvm.kvm_timing_only(None)
    kvm.kvm_timing_reset()
    kvm.kvm_timing_enable(True)
    for i in range(args.warmup):
        if i == 1:
            torch.cuda.synchronize()
            kvm.kvm_timing_reset()
        step(i)
    torch.cuda.synchronize()
    kvm.kvm_timing_enable(False)
    warm_kernels = {}
    for name in KERNEL_NAMES:
        cnt, ms = kvm.kvm_timing_read(name)
        warm_kernels[name] = {"launches": cnt, "avg_ms": (ms / cnt) if cnt else None}
    overlap = step is step_overlap or step is step_refined or step is step_pipelined
    resident = int((wl.state & 1).sum().item())
    # with the transfer overlapped the victims have left the table and their replacements are still on their way
    assert resident == (budget if overlap else budget + swap), (resident, budget, swap)
    assert int(n_bad.item()) == 0, int(n_bad.item())

    kvm.kvm_timing_reset()
    kvm.kvm_timing_only("score_partial")
    kvm.kvm_timing_enable(True)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]   # one per step boundary
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record(main)
    for i in range(args.warmup, total_steps):
        step(i)
        marks[i - args.warmup + 1].record(main)
    torch.cuda.synchronize()                      # both streams: the last victims have reached the host
    elapsed = time.perf_counter() - t0
    per_step = sorted(marks[j].elapsed_time(marks[j + 1]) for j in range(args.steps))
    kvm.kvm_timing_enable(False)
    kvm.kvm_timing_only(None)
    assert int(n_bad.item()) == 0, int(n_bad.item())
    assert int(n_victims.item()) == swap
    if overlap:
        (finish_refined if args.refined else finish_overlap)()
        torch.cuda.synchronize()
        assert int(n_bad.item()) == 0, int(n_bad.item())
    assert int((wl.state & 1).sum().item()) == budget + swap

    ms_per_step = elapsed / args.steps * 1e3
    scored_units = budget if overlap else budget + swap      # units in HBM when the scorer runs
    scored_bytes = scored_units * shape.unit_k_bytes
    value = scored_bytes / (elapsed / args.steps) / 1e9

    kernels = dict(warm_kernels)
    cnt, ms = kvm.kvm_timing_read("score_partial")       # the timed steps' launches of the dominant kernel
    kernels["score_partial"] = {"launches": cnt, "avg_ms": (ms / cnt) if cnt else None}
    kvm.kvm_timing_reset()
    # Dominant kernel: score_partial (the tile kernel).  Algorithmic bytes per launch = what the method has to
    # move whatever the kernel design: per resident unit its K frame (16 * dim * 2) and its mass (4); per block
    # of an active row its table entry (4); per row its g queries.  The per-block partial values that long rows
    # pass from the tile kernel to the row merge are the design's own traffic and are not counted.
    n_blocks_active = n
    algo_bytes = scored_units * (shape.unit_k_bytes + 4) + n_blocks_active * 4 + n_rows * g * dim * 2
    sp = kernels["score_partial"]["avg_ms"]
    achieved = algo_bytes / (sp * 1e-3) / 1e9
    # measured HBM bytes per launch: only for the sizes the counters were taken at
    traffic = SCORE_TILE_TRAFFIC_BYTES.get(args.workload) if (n_seq == w_nseq and swap == w_swap
                                                              and args.swap_mode in ("overlap", "pipelined")
                                                              and not args.refined) else None
    roofline = {"kernel": "score_partial", "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
                "algorithmic_bytes_per_launch": algo_bytes, "avg_ms": round(sp, 4)}

    out = {
        "metric": "KV scored GB/s (frac of HBM peak) + evicted/prefetched blocks/s, 1 MI355X",
        "metric_parts": "value = K bytes scored per second over the whole management pass; frac_of_hbm_peak = "
                        "value / 8000; evicted_units_per_s, prefetched_units_per_s = the per-step exchange",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "ms_per_step_median": round(per_step[len(per_step) // 2], 4),
        "ms_per_step_min_max": [round(per_step[0], 4), round(per_step[-1], 4)], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": (wdesc % n_seq) + ", block 16, decay %g, budget %d%%, 4096 events/step"
                               % (decay, round(100 * w_budget)),
                   "units_total": n, "units_scored_per_step": scored_units, "rows": n_rows,
                   "swap_units_per_step": swap, "resident_fraction": round(scored_units / n, 4),
                   "swap_mode": "exchange" if args.refined else args.swap_mode, "refined": bool(args.refined)},
        "frac_of_hbm_peak": round(value / HBM_PEAK_GBPS, 4),
        "evicted_units_per_s": round(swap / (elapsed / args.steps), 1),
        "prefetched_units_per_s": round(swap / (elapsed / args.steps), 1),
        "roofline": roofline,
        "kernels_avg_ms": {k: (round(v["avg_ms"], 4) if v["avg_ms"] is not None else None) for k, v in kernels.items()},
        "kernels_avg_ms_from": "score_partial: the timed steps; the others: the warm-up steps (all kernels bracketed)",
        "step0": {"pass_ms_all_resident": round(t_pass0 * 1e3, 3),
                  "scored_GBps_all_resident": round(n_res0 * shape.unit_k_bytes / t_pass0 / 1e9, 1),
                  "bulk_evict_units": k0, "bulk_pack_s": round(t_bulk_pack, 4),
                  "bulk_pack_GBps": round(k0 * rec / t_bulk_pack / 1e9, 2),
                  "bulk_pack_units_per_s": round(k0 / t_bulk_pack, 1)},
        "setup_s": round(setup_s, 1),
    }

    if args.refined:
        # bulk hashing rate (checkpoint-style pass over many units): integer-ALU bound, one lane per unit
        n_bulk = min(1 << 18, budget)
        bulk_uids = torch.nonzero(wl.state & 1).flatten()[:n_bulk].contiguous()
        bulk_digests = torch.zeros((n_bulk, 32), dtype=torch.uint8, device=dev)
        kvm.kvm_hash_units(pool, wl.slot_tbl, wl.state, bulk_uids, n_bulk, bulk_digests)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        kvm.kvm_hash_units(pool, wl.slot_tbl, wl.state, bulk_uids, n_bulk, bulk_digests)
        torch.cuda.synchronize()
        t_hash = time.perf_counter() - t0
        out["hash_bulk"] = {"units": n_bulk, "ms": round(t_hash * 1e3, 3),
                            "GBps": round(n_bulk * rec / t_hash / 1e9, 1)}
        del bulk_uids, bulk_digests

    if args.calibrate_copy:
        src = torch.zeros(1 << 28, dtype=torch.int32, device=dev)
        dst = torch.empty_like(src)
        torch.add(src, 1, out=dst)              # reads 2^30 bytes, writes 2^30 bytes
        torch.cuda.synchronize()
        del src, dst

    # ---- plain read ceiling of this chip over the K pool (what a kernel that only reads could reach) ----
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    probe_bytes = min(wl.k_pool.numel() * wl.k_pool.element_size(), 16 * 2**30)
    probe_buf = wl.k_pool.view(torch.uint8).flatten()[:probe_bytes]
    kvm.kvm_probe_read(probe_buf, sink)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(3):
        kvm.kvm_probe_read(probe_buf, sink)
    torch.cuda.synchronize()
    ceiling = 3 * probe_bytes / (time.perf_counter() - t0) / 1e9
    out["read_ceiling_GBps"] = round(ceiling, 1)
    out["roofline"]["frac_of_read_ceiling"] = round(out["roofline"]["achieved"] / ceiling, 4)

    # ---- host link measured in the same run (pinned, 1 GiB, both directions) -----------------------
    link_n = 1 << 30
    hbuf = host_tier[:link_n] if host_tier.numel() >= link_n else torch.empty(link_n, dtype=torch.uint8, pin_memory=True)
    dbuf = torch.empty(link_n, dtype=torch.uint8, device=dev)
    link = {}
    for name, dst, src in (("d2h", hbuf, dbuf), ("h2d", dbuf, hbuf)):
        dst.copy_(src, non_blocking=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(3):
            dst.copy_(src, non_blocking=True)
        torch.cuda.synchronize()
        link[name + "_GBps"] = round(3 * link_n / (time.perf_counter() - t0) / 1e9, 2)
    # both directions at once, each on a stream of its own (needs a second pair of buffers)
    if host_tier.numel() >= 2 * link_n:
        hbuf2 = host_tier[link_n:2 * link_n]
    else:
        hbuf2 = torch.empty(link_n, dtype=torch.uint8, pin_memory=True)
    dbuf2 = torch.empty(link_n, dtype=torch.uint8, device=dev)
    s_out, s_in = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(3):
        with torch.cuda.stream(s_out):
            hbuf.copy_(dbuf, non_blocking=True)
        with torch.cuda.stream(s_in):
            dbuf2.copy_(hbuf2, non_blocking=True)
    torch.cuda.synchronize()
    link["both_at_once_GBps"] = round(2 * 3 * link_n / (time.perf_counter() - t0) / 1e9, 2)
    del dbuf2
    out["host_link"] = link
    out["step0"]["bulk_pack_frac_of_link"] = round(out["step0"]["bulk_pack_GBps"] / link["d2h_GBps"], 3)

    # ---- CPU baseline: the oracle on a bounded sample of the same workload -------------------------
    if not args.no_cpu_baseline:
        import oracle
        oracle.build()
        # score once more (untimed) so that the masses belong to the table as it stands now
        kvm.kvm_score_step(pool, rows, qs[0], scale, mass, ws)
        torch.cuda.synchronize()
        if w_sample_rows is None:
            case = wl.host_sample(seq_ids=list(range(min(w_sample_seqs, n_seq))))
        else:
            pick = np.random.default_rng(7).choice(n_rows, size=min(w_sample_rows, n_rows), replace=False)
            case = wl.host_sample(rows=np.sort(pick))
        q_host = qs[0].view(torch.int16).cpu().numpy().view(np.uint16)
        q_rows = np.concatenate([q_host[r * g * dim:(r + 1) * g * dim] for r in case.sample_rows])
        ref_mass = np.zeros(case.n_uids, np.float32)
        t0 = time.perf_counter()
        oracle.score_step(case.k_pool, dim, shape.dtype, case.row_ntok, case.row_off, case.row_q_off, case.slot_tbl,
                          q_rows, g, scale, ref_mass)
        S_ref = np.zeros(case.n_uids, np.float32)
        prio_ref = np.zeros(case.n_uids, np.float32)
        st_ref = case.state.copy()
        ph = p_hat.cpu().numpy()
        ref_weight = np.full(case.n_rows, float(oracle.size(**shape.model_args())["head_weight"]), np.float32)
        oracle.ema_update(case.row_ntok, case.row_off, ref_mass, decay, ref_weight, case.pair, ph, st_ref, S_ref,
                          prio_ref)
        oracle.select_victims(prio_ref, st_ref, k=-1, budget_units=int(w_budget * case.n_uids))
        t_cpu = time.perf_counter() - t0
        res = case.slot_tbl >= 0
        cpu_bytes = int(res.sum()) * shape.unit_k_bytes
        gpu_mass = mass[torch.from_numpy(case.sample_uids).to(dev)].cpu().numpy()
        rel = np.abs(gpu_mass[res] - ref_mass[res]) / np.maximum(np.abs(ref_mass[res]), 1e-9)
        out["cpu_baseline"] = {"value": round(cpu_bytes / t_cpu / 1e9, 4), "unit": "GB/s", "cores": oracle.threads(),
                               "kind": "oracle",
                               "sample": "%d of %d rows (%d resident units, %.2f GB of K): score + ema + select, "
                                         "%.1f s" % (case.n_rows, n_rows, int(res.sum()), cpu_bytes / 1e9, t_cpu)}
        out["parity_sample_max_rel_err"] = float(rel.max())
        # the same oracle on one core, on a sixteenth of the sample's rows
        n_all = oracle.threads()
        sub = max(1, case.n_rows // 16)
        sub_units = int(case.row_off[sub]) if sub < case.n_rows else case.n_uids
        oracle.set_threads(1)
        try:
            one_mass = np.zeros(case.n_uids, np.float32)
            t0 = time.perf_counter()
            oracle.score_step(case.k_pool, dim, shape.dtype, case.row_ntok[:sub], case.row_off[:sub],
                              case.row_q_off[:sub], case.slot_tbl, q_rows, g, scale, one_mass)
            t_one = time.perf_counter() - t0
        finally:
            oracle.set_threads(n_all)
        one_bytes = int((case.slot_tbl[:sub_units] >= 0).sum()) * shape.unit_k_bytes
        try:
            model = next(l.split(":", 1)[1].strip() for l in open("/proc/cpuinfo") if l.startswith("model name"))
        except Exception:
            model = "unknown"
        out["cpu_baseline"]["cpu_model"] = model
        out["cpu_baseline"]["nproc"] = os.cpu_count()
        out["cpu_baseline"]["one_core"] = {"value": round(one_bytes / t_one / 1e9, 4), "unit": "GB/s",
                                           "sample": "scoring of the first %d rows of that sample, %.1f s" % (sub, t_one)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
