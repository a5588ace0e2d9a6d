#!/usr/bin/env python3
"""Benchmark of the per-decode-step KV-cache management pass on one MI355X.

One step = Beta update of the 16 reuse posteriors -> scoring of every resident unit of the decoding
rows -> EMA + priority -> victim selection under the capacity budget -> victims out to pinned host,
an equal number of host units in, all through the C ABI with every input resident in HBM.

The default run measures the Llama-3-70B-shaped configuration (the largest that one GPU holds:
4 x 131,072 tokens, 80 layers, 8 KV heads, g 8; 86 GB of K) and prints ONE JSON line for it, which
also carries, under "workloads", the same record for the Llama-3-8B-shaped, the DeepSeek-V3-shaped
(MLA) and the heterogeneous-fleet configurations.  `--workload NAME` measures one configuration only.

Per workload the line reports: the step in the order the stages are defined in (selection after this
step's EMA; `value`, `ms_per_step`), the same step with the selection moved beside the scoring launch
(`pipelined`) and with the host-link bytes moved in line by one fused kernel (`in_line`); the
all-resident first pass with a per-kernel breakdown; bulk eviction, bulk prefetch, bulk two-way swap
and exchange against the host link measured in the same run; the roofline of the dominant kernel; the
CPU oracle on a row sample, and the GPU masses of that sample against it.
"""
import argparse
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0        # MI355X HBM3E published peak

# name -> (description, shape builder, sequences, budget fraction, EMA decay, units exchanged per step,
#          rows sampled for the CPU oracle)
WORKLOADS = {
    "llama70b": ("llama3-70b-shaped GQA (one GPU's share): 80 layers, 64q/8kv heads, d128, bf16, %d x 131072 tok",
                 lambda synth, n: synth.llama70b_shape(n), 4, 0.50, 0.95, 4096, 256),
    # config 2 proper ("llama8b") is the growing batch, driven by a plan; this is the same batch with static rows
    "llama8b_static": ("llama3-8b-shaped GQA, static rows: 32 layers, 32q/8kv heads, d128, bf16, %d seqs U[2048,8192] tok",
                lambda synth, n: synth.llama8b_shape(n, seed=2), 64, 0.60, 0.95, 1024, 4096),
    "mla": ("deepseek-v3-shaped MLA: 61 layers, 576-channel latent, 128 absorbed queries, bf16, %d x 32768 tok",
            lambda synth, n: synth.mla_shape(n), 32, 0.40, 0.90, 1024, 64),
    # the two halves of the fleet configuration on their own, one architecture per pool
    "mha": ("fleet, MHA half alone: 32 layers, 32q/32kv heads (g 1), d128, bf16, %d seqs lognormal(7,1) tok",
            lambda synth, n: synth.mha_fleet_shape(n), 72, 0.60, 0.90, 1024, 16384),
    "mqa": ("fleet, MQA half alone: 32 layers, 32q/1kv head (g 32), d128, bf16, %d seqs lognormal(7,1) tok",
            lambda synth, n: synth.mqa_fleet_shape(n), 1536, 0.60, 0.90, 1024, 4096),
}
DEFAULT_ORDER = ["llama70b", "llama8b", "mla", "fleet"]

# HBM bytes per scoring launch from rocprofv3 --pmc (FETCH_SIZE x 2 KiB + WRITE_SIZE x 1 KiB, mean over the 20
# timed steps, all scoring kernels of a step divided by its scoring launches), one entry per workload at its
# default size and default --steps/--warmup.  Each entry names the summary it comes from and the library version
# whose kernels were profiled: a run of any other version, size or step count reports traffic null, because the
# counters no longer describe what it launches.
PROFILED_TRAFFIC = {
    "llama70b": ("0.4", "profiles/score_row_llama70b.md", int(21056580.6 * 2048 + 147102.6 * 1024)),
    "llama8b": ("0.4", "profiles/score_tile_dot2_llama8b_growing.md", int(6616992.0 * 2048 + 29938.1 * 1024)),
    "mla": ("0.4", "profiles/score_tile_wide_mla.md", int(15123149.8 * 2048 + 855654.0 * 1024)),
    "fleet": ("0.4", "profiles/score_tile_fleet.md", int((12314068.4 * 2048 + 201429.7 * 1024) / 2)),
}
KERNEL_NAMES = ("score_plan", "score_partial", "score_finalize", "ema_prio", "beta", "select_hist", "select_emit",
                "pack", "unpack", "swap", "span", "prefetch_keys", "hash", "dedup", "exchange_flip")


class Pinned:
    """One pinned host arena for the whole run, carved per workload (page-locking tens of GB takes seconds)."""

    def __init__(self, torch, nbytes):
        self.buf = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
        self.at = 0

    def reset(self):
        self.at = 0

    def take(self, nbytes):
        nbytes = (nbytes + 4095) // 4096 * 4096
        assert self.at + nbytes <= self.buf.numel(), "pinned arena too small: %d + %d > %d" % (
            self.at, nbytes, self.buf.numel())
        v = self.buf[self.at:self.at + nbytes]
        self.at += nbytes
        return v


def host_link(torch, pinned, dev):
    """hipMemcpyAsync rates of the host link with 1 GiB pinned buffers: each direction, then both at once."""
    n = 1 << 30
    pinned.reset()
    hbuf, hbuf2 = pinned.take(n), pinned.take(n)
    dbuf = torch.empty(n, dtype=torch.uint8, device=dev)
    dbuf2 = torch.empty(n, dtype=torch.uint8, device=dev)
    link = {}
    for name, dst, src in (("d2h", hbuf, dbuf), ("h2d", dbuf, hbuf)):
        dst.copy_(src, non_blocking=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(3):
            dst.copy_(src, non_blocking=True)
        torch.cuda.synchronize()
        link[name + "_GBps"] = round(3 * n / (time.perf_counter() - t0) / 1e9, 2)
    # both directions at once, each on a stream of its own; the best of three trials (the first pair of
    # copies on fresh streams sometimes runs one direction after the other)
    s_out, s_in = torch.cuda.Stream(), torch.cuda.Stream()
    best = 0.0
    for _ in range(3):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(3):
            with torch.cuda.stream(s_out):
                hbuf.copy_(dbuf, non_blocking=True)
            with torch.cuda.stream(s_in):
                dbuf2.copy_(hbuf2, non_blocking=True)
        torch.cuda.synchronize()
        best = max(best, 2 * 3 * n / (time.perf_counter() - t0) / 1e9)
    link["both_at_once_GBps"] = round(best, 2)
    return link


def read_ceiling(torch, kvm, k_pool, dev):
    """Rate of a kernel that only reads the K pool (16-byte non-temporal loads): what this chip gives a pure read."""
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    nbytes = min(k_pool.numel() * k_pool.element_size(), 16 * 2**30)
    buf = k_pool.view(torch.uint8).flatten()[:nbytes]
    kvm.kvm_probe_read(buf, sink)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(3):
        kvm.kvm_probe_read(buf, sink)
    torch.cuda.synchronize()
    return 3 * nbytes / (time.perf_counter() - t0) / 1e9


def timed(torch, fn, reps=1):
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / reps


def read_kernel_times(kvm):
    out = {}
    for name in KERNEL_NAMES:
        cnt, ms = kvm.kvm_timing_read(name)
        out[name] = round(ms / cnt, 4) if cnt else None
    return out


def cpu_model():
    try:
        return next(l.split(":", 1)[1].strip() for l in open("/proc/cpuinfo") if l.startswith("model name"))
    except Exception:
        return "unknown"


def run_refined(args, torch, np, kvm, v):
    """The pass with every refinement switched on (blended reuse estimate, EMA with positional decay and
    transition multipliers, attention-span windows, a prefetch list chosen on the device by position and
    served by the in-place exchange, content hashes of the units that entered HBM and the reference-counted
    store), continued from the state the other step orders left.  `v`: the locals of run_uniform."""
    dev = "cuda"
    shape, wl, rows, pool, swap, budget = v["shape"], v["wl"], v["rows"], v["pool"], v["swap"], v["budget"]
    n, n_rows, decay, row_weight = v["n"], v["n_rows"], v["decay"], v["row_weight"]
    mass, S, prio, hits, misses, p_hat, n_bad, n_victims = (v[k] for k in ("mass", "S", "prio", "hits", "misses",
                                                                           "p_hat", "n_bad", "n_victims"))
    ws, ws_select, qs, evs, scale, host_tier = v["ws"], v["ws_select"], v["qs"], v["evs"], v["scale"], v["host_tier"]
    step_victims, xf_frame, xf_host, tier_slots = v["step_victims"], v["xf_frame"], v["xf_host"], v["tier_slots"]
    main, side, n_q_sets = v["main"], v["side"], v["n_q_sets"]
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
    pf_list = torch.full((swap,), -1, dtype=torch.int64, device=dev)
    arrived = torch.full((swap,), -1, dtype=torch.int64, device=dev)      # the units that came in one step ago
    store = kvm.make_store(1 << 22)
    digests = torch.zeros((swap, 32), dtype=torch.uint8, device=dev)
    canon = torch.zeros(swap, dtype=torch.int64, device=dev)
    dedup_ws = torch.zeros(swap, dtype=torch.int64, device=dev)
    frame_refs = torch.zeros(int(pool.n_slots), dtype=torch.int32, device=dev)
    given_up = torch.full((swap,), -1, dtype=torch.int32, device=dev)

    def step(i):
        ev = evs[i % n_q_sets]
        # The hash of the units that entered HBM in the previous step (one SHA-256 chain per unit: 0.5 ms of
        # latency for 16 wavefronts of work), the reuse estimates and the victims (from the priorities the
        # previous step left) are worked out on a second stream beside the scoring launch.
        side.wait_stream(main)
        kvm.kvm_beta_blend_update(ev[0], ev[1], hits, misses, win, win_head, 64.0, p_hat, conf, p_blend, n_bad=n_bad,
                                  stream=side)
        kvm.kvm_select_victims(prio, wl.state, step_victims, n_victims, ws_select, k=-1, budget_units=budget - swap,
                               stream=side)
        kvm.kvm_hash_units(pool, wl.slot_tbl, wl.state, arrived, swap, digests, stream=side)
        kvm.kvm_score_step_xfer(pool, rows, qs[i % n_q_sets], scale, mass, ws, xf_frame, xf_host, swap, host_tier)
        main.wait_stream(side)
        kvm.kvm_dedup_insert(store, digests, arrived, swap, canon, dedup_ws)
        # duplicates would give up their frames here (the synthetic K and V are random: there are none)
        kvm.kvm_dedup_share(wl.slot_tbl, wl.state, int(pool.n_slots), arrived, canon, swap, frame_refs, given_up)
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

    res = v["run_mode"](step, 0)
    kvm.kvm_score_step_xfer(pool, rows, qs[0], scale, mass, ws, xf_frame, xf_host, swap, host_tier)
    kvm.kvm_exchange_end(wl.slot_tbl, wl.state, pf_list, xf_frame, swap)
    torch.cuda.synchronize()
    assert int(n_bad.item()) == 0, int(n_bad.item())
    res["value"] = round(budget * shape.unit_k_bytes / (res["ms_per_step"] * 1e-3) / 1e9, 1)
    res["frames_shared"] = int((frame_refs > 0).sum().item())
    res["note"] = "all refinements on; selection, estimates and content hashes beside the scoring launch"
    # bulk hashing rate (checkpoint-style pass over many units): integer-ALU bound, one lane per unit
    n_bulk = min(1 << 18, budget)
    rec = shape.unit_k_bytes + shape.unit_v_bytes
    bulk_uids = torch.nonzero(wl.state & 1).flatten()[:n_bulk].contiguous()
    bulk_digests = torch.zeros((n_bulk, 32), dtype=torch.uint8, device=dev)
    kvm.kvm_hash_units(pool, wl.slot_tbl, wl.state, bulk_uids, n_bulk, bulk_digests)
    t_hash = timed(torch, lambda: kvm.kvm_hash_units(pool, wl.slot_tbl, wl.state, bulk_uids, n_bulk, bulk_digests))
    res["hash_bulk"] = {"units": n_bulk, "ms": round(t_hash * 1e3, 3), "GBps": round(n_bulk * rec / t_hash / 1e9, 1)}
    return res


def run_uniform(name, args, torch, np, kvm, synth, pinned, link):
    """One configuration whose rows all belong to one architecture (configurations 2, 3, 4)."""
    dev = "cuda"
    t_setup = time.time()
    wdesc, wshape, w_nseq, w_budget, decay, w_swap, w_sample_rows = WORKLOADS[name]
    n_seq = args.n_seq or w_nseq
    shape = wshape(synth, n_seq)
    pair_w = synth.categorical_weights(3)
    reuse_p = np.linspace(0.15, 0.95, 16)
    # the pool is dimensioned by the sizing call: units per token block x blocks of the batch, at the unit
    # bytes it reports; the head weight of the priority comes from the same call
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
    n_modes = 4 if args.refined else 3
    steps_all = n_modes * (args.warmup + args.steps) + 4          # segments of the tier the stepping consumes
    n_bulk = min((1 << 30) // rec, k0 // 4)                       # records of the bulk transfer measurements (1 GiB)
    keep = swap * (steps_all + 2) + n_bulk                        # tier records that are read again later
    assert keep <= k0, "not enough host-resident units for this many steps"
    if args.refined:
        keep = k0          # a prefetch list chosen on the device can name any unit of tier 1: all records are kept
    chunk = min(k0, 32768)

    # Tier 1 keeps the records that later steps prefetch; the rest of the bulk eviction goes through a
    # scratch chunk and is dropped, as if demoted further down.
    pinned.reset()
    host_tier = pinned.take(keep * rec)[:keep * rec]
    host_scratch = pinned.take(chunk * rec)[:chunk * rec]
    bulk_out = pinned.take(n_bulk * rec)[:n_bulk * rec]
    victims = torch.zeros(k0, dtype=torch.int64, device=dev)
    freed = torch.full((k0,), -1, dtype=torch.int32, device=dev)
    host_slots = torch.arange(k0, dtype=torch.int32, device=dev)
    staging_dev = torch.empty(chunk * rec, dtype=torch.uint8, device=dev)

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
    t_pass0 = timed(torch, lambda: management_pass(0, -1, budget))
    assert int(n_victims.item()) == k0, (int(n_victims.item()), k0)
    # the same pass again with every launch bracketed by events: where the all-resident pass spends its time
    # (the EMA folds the same masses in a second time, which changes no count)
    kvm.kvm_timing_only(None)
    kvm.kvm_timing_reset()
    kvm.kvm_timing_enable(True)
    management_pass(0, -1, budget)
    torch.cuda.synchronize()
    kvm.kvm_timing_enable(False)
    pass0_kernels = read_kernel_times(kvm)
    kvm.kvm_timing_reset()
    assert int(n_victims.item()) == k0
    # shuffle the victim list so that later prefetch segments are random samples of the host tier
    perm = torch.randperm(k0, generator=wl.gen, device=dev)
    victims.copy_(victims[perm])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for lo in range(0, k0, chunk):
        cnt = min(chunk, k0 - lo)
        dst = host_tier[lo * rec:(lo + cnt) * rec] if lo + cnt <= keep else host_scratch
        kvm.kvm_pack(pool, wl.slot_tbl, wl.state, victims[lo:lo + cnt], cnt, host_slots[lo:lo + cnt],
                     freed[lo:lo + cnt], staging_dev, dst, n_bad=n_bad)
    torch.cuda.synchronize()
    t_bulk_pack = time.perf_counter() - t0
    host_uids = victims.clone()                 # uid stored in host record i
    free_frames = freed.clone()
    assert int(n_bad.item()) == 0
    assert int((wl.state & 1).sum().item()) == budget

    step_victims = torch.zeros(swap, dtype=torch.int64, device=dev)
    main = torch.cuda.current_stream()
    side = torch.cuda.Stream()
    xf_frame = torch.full((swap,), -1, dtype=torch.int32, device=dev)
    xf_host = torch.full((swap,), -1, dtype=torch.int64, device=dev)
    xf_in = [host_uids[0:swap]]                 # the in-list of the transfer that is under way
    tier_slots = keep

    def step_in_order(i):
        """The pass in the order its stages are defined in: posteriors, scoring, EMA + priority, then the
        selection on this step's priorities.  The host-link bytes of the exchange chosen in step i - 1 move
        inside step i's scoring launch; units on their way in or out are in HBM for nobody meanwhile: the
        victims left the table when they were chosen, the units fetched for them join it after this step's EMA."""
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
        """step_in_order with the selection moved off the critical path: the victims are chosen, from the
        priorities the previous step left, on a second stream beside this step's scoring launch (the posterior
        update goes with it).  They leave HBM inside the next step's scoring launch, one step later than in
        step_in_order.  While the selection runs the units of the last exchange are still on their way, so
        the budget it is given is the budget minus what is in flight."""
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

    def land_exchange():
        """Lets the last deferred transfer land (untimed)."""
        kvm.kvm_score_step_xfer(pool, rows, qs[0], scale, mass, ws, xf_frame, xf_host, swap, host_tier)
        kvm.kvm_exchange_end(wl.slot_tbl, wl.state, xf_in[0], xf_frame, swap)
        xf_frame.fill_(-1)

    def step_in_line(i):
        """Everything in line on one stream, the bytes included: the victims of this step and the next prefetch
        segment trade places in the slot-addressed tier through one two-way kernel after the selection.
        Resident units at entry: budget + swap."""
        ev = evs[i % n_q_sets]
        kvm.kvm_beta_update(ev[0], ev[1], hits, misses, p_hat, n_bad=n_bad)
        kvm.kvm_score_step(pool, rows, qs[i % n_q_sets], scale, mass, ws)
        kvm.kvm_ema_update(rows, mass, decay, row_weight, wl.pair, p_hat, wl.state, S, prio)
        kvm.kvm_select_victims(prio, wl.state, step_victims, n_victims, ws, k=-1, budget_units=budget)
        nxt = (i + 1) * swap
        kvm.kvm_exchange(pool, wl.slot_tbl, wl.state, step_victims, host_uids[nxt:nxt + swap], swap, host_tier,
                         n_out_dev=n_victims, n_bad=n_bad)

    def run_mode(step_fn, first, dominant=False):
        """args.warmup untimed + args.steps timed steps of step_fn, step numbers from `first`."""
        kvm.kvm_timing_only(None)
        kvm.kvm_timing_reset()
        kvm.kvm_timing_enable(dominant)
        for i in range(first, first + args.warmup):
            if dominant and i == first + 1:
                torch.cuda.synchronize()
                kvm.kvm_timing_reset()
            step_fn(i)
        torch.cuda.synchronize()
        warm = read_kernel_times(kvm) if dominant else None
        assert int(n_bad.item()) == 0, int(n_bad.item())
        kvm.kvm_timing_reset()
        if dominant:
            # the timed steps bracket the dominant kernel only: an event pair costs a few microseconds on the
            # stream, and twenty of them per step were 3 % of a step
            kvm.kvm_timing_only("score_partial")
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        marks[0].record(main)
        for j in range(args.steps):
            step_fn(first + args.warmup + j)
            marks[j + 1].record(main)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        per_step = sorted(marks[j].elapsed_time(marks[j + 1]) for j in range(args.steps))
        kvm.kvm_timing_enable(False)
        kvm.kvm_timing_only(None)
        assert int(n_bad.item()) == 0, int(n_bad.item())
        assert int(n_victims.item()) == swap
        res = {"ms_per_step": round(elapsed / args.steps * 1e3, 4),
               "ms_per_step_median": round(per_step[len(per_step) // 2], 4),
               "ms_per_step_min_max": [round(per_step[0], 4), round(per_step[-1], 4)]}
        if dominant:
            cnt, ms = kvm.kvm_timing_read("score_partial")
            warm["score_partial"] = round(ms / cnt, 4)
            res["kernels_avg_ms"] = warm
            kvm.kvm_timing_reset()
        return res

    # bring the first `swap` units back so that the stepping starts `swap` over budget
    kvm.kvm_unpack(pool, wl.slot_tbl, wl.state, host_uids[0:swap], swap, free_frames[0:swap], staging_dev,
                   host_tier[0:swap * rec], n_bad=n_bad)
    torch.cuda.synchronize()
    per = args.warmup + args.steps
    in_order = run_mode(step_in_order, 0, dominant=True)
    assert int((wl.state & 1).sum().item()) == budget       # victims gone, replacements on their way
    pipelined = run_mode(step_pipelined, per)
    land_exchange()
    torch.cuda.synchronize()
    assert int((wl.state & 1).sum().item()) == budget + swap
    in_line = run_mode(step_in_line, 2 * per + 1)
    assert int((wl.state & 1).sum().item()) == budget + swap

    scored_units = budget                                    # units in HBM when the scorer runs (in_order, pipelined)
    scored_bytes = scored_units * shape.unit_k_bytes
    value = scored_bytes / (in_order["ms_per_step"] * 1e-3) / 1e9

    # Dominant kernel: score_partial (the tile kernel).  Algorithmic bytes per launch = what the method has to
    # move whatever the kernel design: per resident unit its K frame (16 * dim * 2) and its mass (4); per block
    # of an active row its table entry (4); per row its g queries.  The per-block partial values that long rows
    # pass from the tile kernel to the row merge are the design's own traffic and are not counted.
    algo_bytes = scored_units * (shape.unit_k_bytes + 4) + n * 4 + n_rows * g * dim * 2
    sp = in_order["kernels_avg_ms"]["score_partial"]
    achieved = algo_bytes / (sp * 1e-3) / 1e9
    prof = PROFILED_TRAFFIC.get(name)
    traffic = prof[2] if (prof and prof[0] == kvm.kvm_version() and n_seq == w_nseq and swap == w_swap) else None
    roofline = {"kernel": "score_partial", "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
                "traffic_from": (prof[1] + " (library " + prof[0] + ")") if traffic else None,
                "algorithmic_bytes_per_launch": algo_bytes, "avg_ms": round(sp, 4)}

    out = {
        "value": round(value, 1), "unit": "GB/s", "ms_per_step": in_order["ms_per_step"],
        "ms_per_step_median": in_order["ms_per_step_median"], "ms_per_step_min_max": in_order["ms_per_step_min_max"],
        "config": {"workload": (wdesc % n_seq) + ", block 16, decay %g, budget %d%%, 4096 events/step"
                               % (decay, round(100 * w_budget)),
                   "units_total": n, "units_scored_per_step": scored_units, "rows": n_rows,
                   "exchange_units_per_step": swap, "resident_fraction": round(scored_units / n, 4),
                   "step_order": "beta, score (+ bytes of the previous exchange), ema+priority, select, exchange",
                   "pool_units_from_kvm_size": int(sizing["pool_units"]), "head_weight": int(sizing["head_weight"])},
        "frac_of_hbm_peak": round(value / HBM_PEAK_GBPS, 4),
        "in_order_ms_per_step": in_order["ms_per_step"],
        "step_orders": {
            "in_order": {k: in_order[k] for k in ("ms_per_step", "ms_per_step_median", "ms_per_step_min_max")},
            "pipelined": dict(pipelined, value=round(scored_bytes / (pipelined["ms_per_step"] * 1e-3) / 1e9, 1),
                              note="victims chosen beside the scoring launch from the previous step's priorities"),
            "in_line": dict(in_line, value=round((budget + swap) * shape.unit_k_bytes / (in_line["ms_per_step"] * 1e-3) / 1e9, 1),
                            note="bytes moved in line by kvm_exchange after the selection"),
        },
        "roofline": roofline,
        "kernels_avg_ms": in_order["kernels_avg_ms"],
        "kernels_avg_ms_from": "score_partial: the timed steps; the others: the warm-up steps (all kernels bracketed)",
        "step0": {"pass_ms_all_resident": round(t_pass0 * 1e3, 3),
                  "scored_GBps_all_resident": round(n_res0 * shape.unit_k_bytes / t_pass0 / 1e9, 1),
                  "frac_of_hbm_peak": round(n_res0 * shape.unit_k_bytes / t_pass0 / 1e9 / HBM_PEAK_GBPS, 4),
                  "kernels_avg_ms": pass0_kernels,
                  "bulk_evict_units": k0},
        "setup_s": round(setup_s, 1),
    }

    # ---- the host link's side of the metric: bulk transfers of n_bulk records (1 GiB) each way ---------
    # Tier segment [a, a + n_bulk) is untouched since the bulk eviction: record a + i belongs to host_uids[a + i],
    # and the frames those units left are still free.
    a = keep - n_bulk
    b_uids, b_frames, b_slots = host_uids[a:keep].contiguous(), free_frames[a:keep].contiguous(), host_slots[a:keep]
    b_tier = host_tier[a * rec:keep * rec]
    b_freed = torch.full((n_bulk,), -1, dtype=torch.int32, device=dev)
    gb = n_bulk * rec / 1e9
    t_unpack = timed(torch, lambda: kvm.kvm_unpack(pool, wl.slot_tbl, wl.state, b_uids, n_bulk, b_frames, None, b_tier,
                                                   n_bad=n_bad))
    t_pack = timed(torch, lambda: kvm.kvm_pack(pool, wl.slot_tbl, wl.state, b_uids, n_bulk, b_slots, b_freed, None,
                                               b_tier, n_bad=n_bad))
    assert bool((b_freed == b_frames).all())
    # two-way: n_bulk resident units leave for bulk_out while the segment's units enter the frames they free;
    # then the reverse, which restores tables, pools and tier
    res_ids = torch.nonzero(((wl.state & 5) == 1)).flatten()
    pick = res_ids[torch.randperm(res_ids.numel(), generator=wl.gen, device=dev)[:n_bulk]].contiguous()
    out_slots = torch.arange(keep, keep + n_bulk, dtype=torch.int32, device=dev)     # labels outside the kept tier
    t_swap = timed(torch, lambda: kvm.kvm_swap(pool, wl.slot_tbl, wl.state, pick, b_uids, n_bulk, out_slots, b_freed,
                                               bulk_out, b_tier, n_bad=n_bad))
    t_swap_back = timed(torch, lambda: kvm.kvm_swap(pool, wl.slot_tbl, wl.state, b_uids, pick, n_bulk, b_slots, b_freed,
                                                    b_tier, bulk_out, n_bad=n_bad))
    # in-place exchange against the slot-addressed tier, there and back
    t_exch = timed(torch, lambda: kvm.kvm_exchange(pool, wl.slot_tbl, wl.state, pick, b_uids, n_bulk,
                                                   host_tier, n_bad=n_bad))
    t_exch_back = timed(torch, lambda: kvm.kvm_exchange(pool, wl.slot_tbl, wl.state, b_uids, pick, n_bulk,
                                                        host_tier, n_bad=n_bad))
    assert int(n_bad.item()) == 0, int(n_bad.item())
    assert int((wl.state & 1).sum().item()) == budget + swap
    t_swap2, t_exch2 = min(t_swap, t_swap_back), min(t_exch, t_exch_back)
    out["host_link"] = link
    out["transfers"] = {
        "record_bytes": rec, "bulk_records": n_bulk,
        "evict_staged": {"GBps": round(k0 * rec / t_bulk_pack / 1e9, 2), "units_per_s": round(k0 / t_bulk_pack, 1),
                         "frac_of_link": round(k0 * rec / t_bulk_pack / 1e9 / link["d2h_GBps"], 3),
                         "what": "kvm_pack of the %d units of the step-0 eviction, gather kernel + hipMemcpyAsync" % k0},
        "evict": {"GBps": round(gb / t_pack, 2), "units_per_s": round(n_bulk / t_pack, 1),
                  "frac_of_link": round(gb / t_pack / link["d2h_GBps"], 3), "what": "kvm_pack, zero-copy, device to host"},
        "prefetch": {"GBps": round(gb / t_unpack, 2), "units_per_s": round(n_bulk / t_unpack, 1),
                     "frac_of_link": round(gb / t_unpack / link["h2d_GBps"], 3),
                     "what": "kvm_unpack, zero-copy, host to device"},
        "swap": {"GBps": round(2 * gb / t_swap2, 2), "units_per_s_each_way": round(n_bulk / t_swap2, 1),
                 "frac_of_link": round(2 * gb / t_swap2 / link["both_at_once_GBps"], 3),
                 "what": "kvm_swap, both directions at once, bytes of both directions counted"},
        "exchange": {"GBps": round(2 * gb / t_exch2, 2), "units_per_s_each_way": round(n_bulk / t_exch2, 1),
                     "frac_of_link": round(2 * gb / t_exch2 / link["both_at_once_GBps"], 3),
                     "what": "kvm_exchange, in place against the slot-addressed tier"},
    }
    out["evicted_units_per_s"] = out["transfers"]["evict"]["units_per_s"]
    out["prefetched_units_per_s"] = out["transfers"]["prefetch"]["units_per_s"]

    ceiling = read_ceiling(torch, kvm, wl.k_pool, dev)
    out["read_ceiling_GBps"] = round(ceiling, 1)
    out["roofline"]["frac_of_read_ceiling"] = round(achieved / ceiling, 4)

    if args.refined:
        out["step_orders"]["refined"] = run_refined(args, torch, np, kvm, locals())

    # ---- CPU baseline: the oracle on a bounded sample of the same workload -------------------------
    if not args.no_cpu_baseline:
        import oracle
        oracle.build()
        # score once more (untimed) so that the masses belong to the table as it stands now
        kvm.kvm_score_step(pool, rows, qs[0], scale, mass, ws)
        torch.cuda.synchronize()
        # first, middle and last row always, the rest drawn with a seed
        want = min(w_sample_rows, n_rows)
        drawn = np.random.default_rng(7).choice(n_rows, size=want, replace=False)
        pick_rows = np.unique(np.concatenate([[0, n_rows // 2, n_rows - 1], drawn]))
        case = wl.host_sample(rows=pick_rows)
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
                               "sample": "%d of %d rows (%d resident units, %.2f GB of K = %.2f %% of the K in HBM): "
                                         "score + ema + select, %.1f s"
                                         % (case.n_rows, n_rows, int(res.sum()), cpu_bytes / 1e9,
                                            100.0 * cpu_bytes / scored_bytes, t_cpu)}
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
        out["cpu_baseline"]["cpu_model"] = cpu_model()
        out["cpu_baseline"]["nproc"] = os.cpu_count()
        out["cpu_baseline"]["one_core"] = {"value": round(one_bytes / t_one / 1e9, 4), "unit": "GB/s",
                                           "sample": "scoring of the first %d rows of that sample, %.1f s" % (sub, t_one)}
    return out


FLEET = dict(n_requests=10000, rate=0.5, n_prefixes=64, start=15000, hbm_share=0.6, budget=0.60, decay=0.90,
             prefetch_cap=1024, window_tokens=2048, keep_records=1 << 19, seed=11)
GROWING = dict(n_seq=64, budget=0.60, decay=0.95, events_per_step=4096, seed=2)


def prepare_fleet(args, kvm, synth):
    """Sizing of the shared pool and the host replay of the trace (no GPU work)."""
    from paper_2604_26968_amd import fleet
    F = FLEET
    shapes = [synth.Shape(32, 32, 32, 128, synth.BF16, True, []), synth.Shape(32, 32, 1, 128, synth.BF16, True, [])]
    target = int(F["hbm_share"] * 288 * 10**9)
    sizing = [kvm.kvm_size(**sh.model_args(), n_max=32768, mem_target=target) for sh in shapes]
    assert sizing[0]["pool_units"] == sizing[1]["pool_units"]               # same unit bytes: one pool serves both
    cats = [synth.fleet_catalogue(F["n_prefixes"], F["seed"]), synth.fleet_catalogue(F["n_prefixes"], F["seed"] + 1)]
    reqs = synth.fleet_requests(F["n_requests"], F["seed"] + 2, F["rate"], F["n_prefixes"], cats)
    n_steps = args.warmup + args.steps
    plan = fleet.build_plan(shapes, cats, reqs, F["start"], n_steps, capacity_units=int(0.97 * sizing[0]["pool_units"]))
    rec = int(sizing[0]["unit_k_bytes"] + sizing[0]["unit_v_bytes"])
    tier_slots = F["keep_records"] + sum(plan.stats["new_units_per_step"]) + 8
    pool_units = int(sizing[0]["pool_units"])
    desc = ("heterogeneous fleet: MHA (32 layers, 32 KV heads, g 1) + MQA (32 layers, 1 KV head, g 32), d128, bf16, one "
            "pool of %d frames from kvm_size(%.0f %% of 288 GB); trace of %d requests, Zipf(1.1) over %d prefixes per "
            "model, lengths lognormal(7,1) clipped to 32768, window = steps %d..%d, budget %d%%, decay %g"
            % (pool_units, 100 * F["hbm_share"], F["n_requests"], F["n_prefixes"], F["start"], F["start"] + n_steps - 1,
               round(100 * F["budget"]), F["decay"]))
    return dict(shapes=shapes, sizing=sizing, plan=plan, rec=rec, tier_slots=tier_slots, pool_units=pool_units,
                pinned_bytes=(tier_slots + 32768) * rec + 2 * 4096, desc=desc, budget=F["budget"], decay=F["decay"],
                prefetch_cap=F["prefetch_cap"], window_tokens=F["window_tokens"], keep_records=F["keep_records"],
                seed=F["seed"], sample_rows=[2048, 256],
                step_order="arrivals into free frames, beta, score (2 launches), ema+priority (2), "
                           "prefetch keys (2) + list, ONE victim selection, exchange, pack")


def prepare_growing(args, kvm, synth, np):
    """The Llama-3-8B-shaped batch as it decodes: every sequence appends one token per step, a sequence that
    crosses a block boundary gets a new block (256 new units: 32 layers x 8 KV heads) whose frames the previous
    step's victims left, the block being written is PROTECTED, the budget stays 60 % of the initial units."""
    from paper_2604_26968_amd import fleet
    G = GROWING
    shape = synth.llama8b_shape(args.n_seq or G["n_seq"], seed=G["seed"])
    n_steps = args.warmup + args.steps
    cats = [[synth.FleetPrefix(0.0, 2, 0)]]
    plan = fleet.build_plan([shape], cats, synth.growing_batch_requests(shape.seq_lens), 1, n_steps,
                            capacity_units=1 << 62)
    # pair bytes and events as in the static configurations: seeded categoricals
    pair_w = synth.categorical_weights(3)
    # one pair per (sequence, block), shared by the block's units over all layers and heads
    rng = np.random.default_rng(G["seed"] + 1)
    off = plan.rows[0]["off"]
    caps = np.diff(np.append(off, plan.n_uids))                      # uids per row = blocks the sequence can reach
    upb = shape.n_layers * shape.n_kv_heads
    row_of_uid = np.repeat(np.arange(len(off)), caps)
    block = np.arange(plan.n_uids) - off[row_of_uid]
    seq_caps = caps[::upb]
    seq_base = np.concatenate([[0], np.cumsum(seq_caps)[:-1]])
    per_block = rng.choice(16, size=int(seq_caps.sum()), p=pair_w).astype(np.uint8)
    plan.pair[:] = per_block[seq_base[row_of_uid // upb] + block]
    plan.events[:] = [synth.make_events(G["events_per_step"], 200 + j, pair_weights=pair_w,
                                        reuse_prob=np.linspace(0.15, 0.95, 16)) for j in range(n_steps)]
    probe = kvm.kvm_size(**shape.model_args(), n_max=max(shape.seq_lens) + n_steps + 1)
    rec = int(probe["unit_k_bytes"] + probe["unit_v_bytes"])
    sizing = [kvm.kvm_size(**shape.model_args(), n_max=max(shape.seq_lens) + n_steps + 1, mem_target=plan.n_uids * rec)]
    pool_units = int(sizing[0]["pool_units"])
    assert pool_units == plan.n_uids                    # every unit the window will ever hold has a frame to its name
    tier_slots = sum(plan.stats["new_units_per_step"]) + 8
    desc = ("llama3-8b-shaped GQA, decoding: 32 layers, 32q/8kv heads, d128, bf16, %d seqs U[2048,8192] tok growing one "
            "token per step (new blocks at block boundaries, newest block PROTECTED), block 16, decay %g, budget %d%% of "
            "the initial units, %d events/step"
            % (len(shape.seq_lens), G["decay"], round(100 * G["budget"]), G["events_per_step"]))
    return dict(shapes=[shape], sizing=sizing, plan=plan, rec=rec, tier_slots=tier_slots, pool_units=pool_units,
                pinned_bytes=(tier_slots + 32768) * rec + 2 * 4096, desc=desc, budget=G["budget"], decay=G["decay"],
                prefetch_cap=0, window_tokens=0, keep_records=0, seed=G["seed"], sample_rows=[4096],
                step_order="new blocks into free frames, beta, score, ema+priority, ONE victim selection, eviction")


def run_fleet(args, torch, np, kvm, synth, pinned, link, prep, ahead=True, brief=False):
    """A trace-driven workload (the heterogeneous fleet, or the growing Llama-3-8B-shaped batch): rows of one
    or two architectures in ONE pool sized by kvm_size, per-step inputs from a plan replayed on the host.
    New units take free frames of the pool at once; every step then evicts what HBM holds beyond the budget.
    ahead: the victims leave the table when chosen and their bytes leave inside the next scoring launch, at most
    16,384 units per step (after a whole prompt has arrived HBM is back at the budget some steps later);
    otherwise they are packed out in line, all at once.  brief: the stepping only."""
    from paper_2604_26968_amd import fleet
    dev = "cuda"
    t_setup = time.time()
    shapes, sizing, plan, rec, tier_slots = prep["shapes"], prep["sizing"], prep["plan"], prep["rec"], prep["tier_slots"]
    pool_units = prep["pool_units"]
    unit_k = int(sizing[0]["unit_k_bytes"])
    n_steps = args.warmup + args.steps
    st = plan.stats
    assert st["init_units"] <= pool_units
    pinned.reset()
    tier = pinned.take(tier_slots * rec)[:tier_slots * rec]
    scratch = pinned.take(32768 * rec)[:32768 * rec]
    fd = fleet.FleetDevice(plan, kvm, torch, pool_units, [float(s["head_weight"]) for s in sizing], tier, tier_slots,
                           prefetch_cap=prep["prefetch_cap"], window_tokens=prep["window_tokens"], decay=prep["decay"],
                           seed=prep["seed"], ahead=ahead, ride_max=args.ride_max or 16384)
    n = plan.n_uids
    # per step: which uids belong to rows that decode (to count the units the scorer reads)
    act_uid = []
    for j in range(n_steps):
        m = torch.zeros(n, dtype=torch.uint8, device=dev)
        for a, d in enumerate(fd.arch):
            rows_on = torch.nonzero(d["active"][j]).flatten()
            nb = (d["ntok"][j][rows_on].long() + 15) // 16
            starts = d["off"][rows_on]
            tot = int(nb.sum().item())
            if tot:
                rep = torch.repeat_interleave(torch.arange(rows_on.numel(), device=dev), nb)
                within = torch.arange(tot, device=dev) - torch.repeat_interleave(torch.cumsum(nb, 0) - nb, nb)
                m[starts[rep] + within] = 1
        act_uid.append(m)
    torch.cuda.synchronize()
    setup_s = time.time() - t_setup

    # ---- warm start: everything in HBM, every row decodes once; then bulk eviction to the budget ----------
    fd.score(None, 0)                       # untimed: loads the code objects
    torch.cuda.synchronize()
    t_pass0 = timed(torch, fd.first_pass)
    kvm.kvm_timing_only(None)
    kvm.kvm_timing_reset()
    kvm.kvm_timing_enable(True)
    fd.first_pass()
    torch.cuda.synchronize()
    kvm.kvm_timing_enable(False)
    pass0_kernels = read_kernel_times(kvm)
    kvm.kvm_timing_reset()
    n_res0 = int((fd.state & 1).sum().item())
    budget = int(prep["budget"] * n_res0)
    order = np.random.default_rng(prep["seed"] + 5).permutation(n_res0 - budget)
    t0 = time.perf_counter()
    k0, _ = fd.evict_to_budget(budget, prep["keep_records"], order, scratch)
    t_bulk = time.perf_counter() - t0

    # ---- the window -------------------------------------------------------------------------------------
    main = torch.cuda.current_stream()
    scored = torch.zeros(n_steps, dtype=torch.int64, device=dev)
    pairs = torch.zeros(n_steps, dtype=torch.int64, device=dev)

    pass_marks = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_steps)]

    def step(j):
        fd.arrive(j)
        pass_marks[j][0].record(main)
        fd.beta(j)
        fd.score(j, j)
        fd.ema(j)
        fd.settle()
        fd.prefetch_keys(j)
        fd.select(j)
        pass_marks[j][1].record(main)
        scored[j] = ((fd.state & 1) * act_uid[j]).sum()          # units the two scoring launches just read
        if fd.P:
            pairs[j] = torch.minimum(fd.n_pf[0], fd.n_v[0]).clamp(max=fd.P)
        fd.move(j)
        over_h.append(fd.resident - fd.budget)

    over_h = []
    kvm.kvm_timing_only(None)
    kvm.kvm_timing_reset()
    kvm.kvm_timing_enable(True)
    for j in range(args.warmup):
        if j == 1:
            torch.cuda.synchronize()
            kvm.kvm_timing_reset()
        step(j)
    torch.cuda.synchronize()
    warm = read_kernel_times(kvm)
    kvm.kvm_timing_reset()
    kvm.kvm_timing_only("score_partial")
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record(main)
    for j in range(args.warmup, n_steps):
        step(j)
        marks[j - args.warmup + 1].record(main)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    kvm.kvm_timing_enable(False)
    kvm.kvm_timing_only(None)
    cnt, sp_ms = kvm.kvm_timing_read("score_partial")
    kvm.kvm_timing_reset()
    fd.flush()
    torch.cuda.synchronize()
    assert int(fd.n_bad.item()) == 0, int(fd.n_bad.item())
    per_step = [marks[j].elapsed_time(marks[j + 1]) for j in range(args.steps)]
    scored_h = scored.cpu().numpy()[args.warmup:]
    pairs_h = pairs.cpu().numpy()[args.warmup:]
    new_next = np.asarray(fd.evicted[args.warmup:n_steps])      # units each timed step evicts
    arrived = np.asarray(fd.n_new[args.warmup:n_steps])
    scored_bytes = float(scored_h.sum()) * unit_k
    value = scored_bytes / elapsed / 1e9
    pass_ms = [pass_marks[j][0].elapsed_time(pass_marks[j][1]) for j in range(args.warmup, n_steps)]
    pass_value = scored_bytes / (sum(pass_ms) * 1e-3) / 1e9
    # steps without an arrival of a whole prompt: growth of the decoding sequences only
    quiet = [t for t, m in zip(per_step, arrived) if m < 65536]
    quiet_bytes = [b * unit_k for b, m in zip(scored_h, arrived) if m < 65536]
    # roofline of the two scoring launches of a step together (g 1 rows on the dot-product kernel, g 32 rows on
    # the matrix-core kernel): algorithmic bytes = K frames + masses of the units read, table entries of the
    # decoding rows' blocks, their queries
    blocks_active = sum(int(act_uid[j].sum().item()) for j in range(args.warmup, n_steps))
    q_bytes = sum(int(fd.arch[a]["active"][j].sum().item()) * shapes[a].g * 128 * 2
                  for j in range(args.warmup, n_steps) for a in range(len(shapes)))
    algo = float(scored_h.sum()) * (unit_k + 4) + blocks_active * 4 + q_bytes
    achieved = algo / (sp_ms * 1e-3) / 1e9
    prof = PROFILED_TRAFFIC.get(prep["name"])
    at_defaults = args.steps == 20 and args.warmup == 5 and not args.n_seq and not args.ride_max and ahead
    traffic = prof[2] if (prof and prof[0] == kvm.kvm_version() and at_defaults) else None
    warm["score_partial"] = round(sp_ms / max(cnt, 1), 4)
    out = {
        "value": round(value, 1), "unit": "GB/s", "ms_per_step": round(elapsed / args.steps * 1e3, 4),
        "ms_per_step_median": round(sorted(per_step)[len(per_step) // 2], 4),
        "ms_per_step_min_max": [round(min(per_step), 4), round(max(per_step), 4)],
        "config": {"workload": prep["desc"],
                   "units_total": int(st["init_units"]), "pool_units_from_kvm_size": pool_units,
                   "head_weights": [int(s["head_weight"]) for s in sizing], "entries_by_model": st["entries_by_model"],
                   "rows": [d["n_rows"] for d in fd.arch], "requests_replayed": st["requests_replayed"],
                   "lookup_hits": st["hits"], "lookup_misses": st["misses"], "retired_before_window": st["retired"],
                   "decoding_sequences_per_step": [int(min(st["active_per_step"])), int(max(st["active_per_step"]))],
                   "units_scored_per_step": [int(scored_h.min()), int(scored_h.max())],
                   "new_units_per_step": [int(arrived.min()), int(arrived.max())],
                   "evicted_units_per_step": [int(new_next.min()), int(new_next.max())],
                   "events_per_step": [min(len(e[0]) for e in plan.events), max(len(e[0]) for e in plan.events)],
                   "prefetch_pairs_per_step": [int(pairs_h.min()), int(pairs_h.max())],
                   "step_order": prep["step_order"] + (
                       "; new units take free frames of the pool, what HBM then holds beyond the budget is evicted: the "
                       "victims leave the table at once (kvm_pack_begin), their bytes leave inside the next scoring "
                       "launch, at most %d units per step" % fd.ride_max if ahead else
                       "; new units take free frames of the pool, what HBM then holds beyond the budget is packed out "
                       "in line"),
                   "units_over_budget_after_step": [int(x) for x in over_h[args.warmup:]]},
        "frac_of_hbm_peak": round(value / HBM_PEAK_GBPS, 4),
        "in_order_ms_per_step": round(elapsed / args.steps * 1e3, 4),
        "pass_without_transfers": {
            "ms": round(sum(pass_ms) / len(pass_ms), 4), "value": round(pass_value, 1),
            "frac_of_hbm_peak": round(pass_value / HBM_PEAK_GBPS, 4),
            "what": "beta + scoring + ema/priority + prefetch keys + the selections, from events on "
                    "the stream (with the victims' bytes of the last eviction inside the scoring launch); the "
                    "arrivals' scatter, the in-line exchange and in-line evictions left out"},
        "steps_without_prompt_arrival": {
            "count": len(quiet), "ms_per_step": round(sum(quiet) / max(len(quiet), 1), 4),
            "value": round(sum(quiet_bytes) / max(sum(quiet), 1e-9) / 1e6, 1),
            "note": "steps whose eviction only makes room for the growth of decoding sequences; a step that makes "
                    "room for a whole arriving prompt is bound by the host link (its victims' bytes go out in line)"},
        "eviction": "bytes inside the next scoring launch, at most %d units per step" % fd.ride_max if ahead
                    else "in line, all at once",
        "link_bytes_per_step_mean": int((new_next.sum() + 2 * pairs_h.sum()) * rec / args.steps),
        "roofline": {"kernel": "score_partial (all scoring launches of a step)", "bound": "hbm", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
                     "traffic_from": (prof[1] + " (library " + prof[0] + ")") if traffic else None,
                     "algorithmic_bytes_per_launch": int(algo / max(cnt, 1)), "avg_ms": round(sp_ms / max(cnt, 1), 4)},
        "kernels_avg_ms": warm,
        "kernels_avg_ms_from": "score_partial: the timed steps (one launch per architecture and step); the others: the "
                               "warm-up steps",
        "step0": {"pass_ms_all_resident": round(t_pass0 * 1e3, 3),
                  "scored_GBps_all_resident": round(n_res0 * unit_k / t_pass0 / 1e9, 1),
                  "frac_of_hbm_peak": round(n_res0 * unit_k / t_pass0 / 1e9 / HBM_PEAK_GBPS, 4),
                  "kernels_avg_ms": pass0_kernels, "bulk_evict_units": k0,
                  "bulk_evict_GBps": round(k0 * rec / t_bulk / 1e9, 2),
                  "bulk_evict_frac_of_link": round(k0 * rec / t_bulk / 1e9 / link["d2h_GBps"], 3)},
        "host_link": link, "setup_s": round(setup_s, 1),
    }
    if brief:
        return out
    ceiling = read_ceiling(torch, kvm, fd.k_pool, dev)
    out["read_ceiling_GBps"] = round(ceiling, 1)
    out["roofline"]["frac_of_read_ceiling"] = round(achieved / ceiling, 4)

    # ---- CPU baseline and parity: sampled decoding rows of both architectures at the last step ---------------
    if not args.no_cpu_baseline:
        import oracle
        oracle.build()
        j = n_steps - 1
        fd.mass.fill_(-1.0)
        fd.score(j, j)                      # untimed, on the tables as they stand now
        torch.cuda.synchronize()
        rng = np.random.default_rng(7)
        t_cpu, cpu_bytes, worst, n_rows_s = 0.0, 0, 0.0, 0
        for a, d in enumerate(fd.arch):
            on = torch.nonzero(d["active"][j]).flatten().cpu().numpy()
            pick = np.unique(np.concatenate([[on[0], on[len(on) // 2], on[-1]],
                                             rng.choice(on, size=min(len(on), prep["sample_rows"][a]), replace=False)]))
            hr = fd.host_rows(a, j, pick, j)
            uids, u_dev, g = hr["uids"], torch.from_numpy(hr["uids"]).to(dev), hr["g"]
            ref = np.full(len(uids), -1.0, np.float32)
            t0 = time.perf_counter()
            oracle.score_step(hr["k_pool"], 128, synth.BF16, hr["ntok"], hr["off"], hr["q_off"], hr["tbl"], hr["q"], g,
                              fd.scale, ref)
            t_cpu += time.perf_counter() - t0
            got = fd.mass[u_dev].cpu().numpy()
            r_ = hr["resident"]
            rel = np.abs(got[r_] - ref[r_]) / np.maximum(np.abs(ref[r_]), 1e-9)
            worst = max(worst, float(rel.max()))
            assert np.all(got[~r_] == -1.0)
            cpu_bytes += int(r_.sum()) * unit_k
            n_rows_s += len(pick)
        out["cpu_baseline"] = {"value": round(cpu_bytes / t_cpu / 1e9, 4), "unit": "GB/s", "cores": oracle.threads(),
                               "kind": "oracle",
                               "sample": "%d decoding rows at the last step (%.2f GB of K): scoring, %.1f s"
                                         % (n_rows_s, cpu_bytes / 1e9, t_cpu),
                               "cpu_model": cpu_model(), "nproc": os.cpu_count()}
        out["parity_sample_max_rel_err"] = worst
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", choices=sorted(WORKLOADS) + ["llama8b", "fleet", "all"], default="all",
                    help="all = the Llama-3-70B-shaped configuration as the headline, with the records of the "
                         "Llama-3-8B-shaped, MLA and fleet configurations under 'workloads'")
    ap.add_argument("--n-seq", type=int, default=0, help="sequences in the batch (0 = the workload's own number)")
    ap.add_argument("--swap-units", type=int, default=0, help="units evicted and prefetched per step (0 = workload default)")
    ap.add_argument("--refined", action="store_true",
                    help="also time the pass with every refinement switched on (single-architecture workloads; "
                         "keeps all of tier 1 in pinned memory)")
    ap.add_argument("--ride-max", type=int, default=0,
                    help="trace-driven workloads: units evicted per step at most, their bytes inside the next scoring "
                         "launch (0 = 16384)")
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
    names = DEFAULT_ORDER if args.workload == "all" else [args.workload]
    # pinned arena: the tier segments the stepping consumes (8 KiB records, up to 4,096 per step; 18 KiB
    # records, 1,024 per step), a scratch chunk, and 1 GiB buffers for the bulk transfers and the link probes
    per_step_bytes = max(args.swap_units or 4096, 1024) * 18432
    arena = 4 * 2**30 + per_step_bytes * (3 * (args.warmup + args.steps) + 8)
    if args.refined:
        arena = max(arena, 24 * 2**30)
    preps = {}
    if "fleet" in names:
        # tier records kept from the bulk eviction + room for the victims the window's arrivals push out
        preps["fleet"] = dict(prepare_fleet(args, kvm, synth), name="fleet")
    if "llama8b" in names:
        preps["llama8b"] = dict(prepare_growing(args, kvm, synth, np), name="llama8b")
    for pr in preps.values():
        arena = max(arena, pr["pinned_bytes"], 2 * 2**30 + 8192)
    pinned = Pinned(torch, arena)
    link = host_link(torch, pinned, "cuda")

    records = []
    for name in names:
        t0 = time.time()
        if name in preps:
            rec = run_fleet(args, torch, np, kvm, synth, pinned, link, preps[name])
            gc.collect()
            torch.cuda.empty_cache()
            alt = run_fleet(args, torch, np, kvm, synth, pinned, link, preps[name], ahead=False, brief=True)
            keys = ("ms_per_step", "ms_per_step_median", "ms_per_step_min_max", "value", "frac_of_hbm_peak",
                    "pass_without_transfers", "steps_without_prompt_arrival", "eviction")
            rec["step_orders"] = {"ahead": {k: rec[k] for k in keys}, "in_line": {k: alt[k] for k in keys}}
            rec["in_order_ms_per_step"] = rec["ms_per_step"]
            del alt
        else:
            rec = run_uniform(name, args, torch, np, kvm, synth, pinned, link)
        rec["name"] = name
        rec["wall_s"] = round(time.time() - t0, 1)
        records.append(rec)
        gc.collect()
        torch.cuda.empty_cache()

    if args.calibrate_copy:
        src = torch.zeros(1 << 28, dtype=torch.int32, device="cuda")
        dst = torch.empty_like(src)
        torch.add(src, 1, out=dst)              # reads 2^30 bytes, writes 2^30 bytes
        torch.cuda.synchronize()
        del src, dst

    head = records[0]
    out = {
        "metric": "KV scored GB/s (frac of HBM peak) + evicted/prefetched blocks/s, 1 MI355X",
        "metric_parts": "value = K bytes scored per second over the whole management pass (stages in their defined "
                        "order); frac_of_hbm_peak = value / 8000; evicted_units_per_s, prefetched_units_per_s = bulk "
                        "kvm_pack / kvm_unpack rates over the host link (transfers.* gives them against the link "
                        "measured in the same run)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic", "library_version": kvm.kvm_version(),
    }
    out.update(head)
    if len(records) > 1:
        out["workloads"] = records[1:]
    print(json.dumps(out))


if __name__ == "__main__":
    main()
