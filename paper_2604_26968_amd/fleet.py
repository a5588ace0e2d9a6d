"""Driver of the heterogeneous-fleet workload: sequences of an MHA model and of an MQA model share
one HBM pool and one uid space, a seeded request trace decides who decodes, who idles, who arrives
and what is looked up, and every decode step runs the whole management pass over the shared pool.

Two parts, neither of which holds any arithmetic of the method:

* :func:`build_plan` replays the request trace on the host (sessions, shared-prefix lookups, cached
  entries, growth of decoding sequences) and lays the result down as plain arrays: an arena of rows
  in one uid space and, per decode step of the measured window, the row lengths, the rows that
  decode, the reuse events, the units that come into existence and the blocks that are being
  written.  Nothing in it depends on what the GPU decides (which units are in HBM), so the same plan
  drives the library and a reference.
* :class:`FleetDevice` keeps the per-unit state on the GPU and issues the step's library calls in
  stages (arrive, beta, score, ema, prefetch, select, move).

Model of the trace.  A request names a model, a prefix id (Zipf-distributed over a catalogue) and a
prompt length.  Its lookup finds either a cached entry of that (model, prefix) — a finished session
kept in the cache; the request continues it, appending only the part of its prompt beyond the shared
prefix — or nothing, and then a new entry is prefilled in full.  One event per looked-up prefix block
records the outcome under the pair (block type, transition type) of the catalogue entry.  A session
alternates decode turns (one token per step) and idle gaps; resuming looks up its most recent blocks
(events with outcome 1).  After its last turn the entry stays cached under its key.  Before the
measured window the replay retires least-recently-used cached entries whenever the content exceeds
the logical capacity; inside the window nothing is retired.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np

from . import synth

BLOCK = synth.BLOCK
ACTIVE, IDLE, CACHED, RETIRED = 0, 1, 2, 3
RES, HOST, PROT, SCORED = 1, 2, 4, 8
USER_CONTEXT, REASONING = 2, 3          # block types of prompt text and of decoded text


@dataclass
class _Entry:
    model: int
    prefix: int
    transition: int
    ntok: int = 0
    status: int = ACTIVE
    decode_left: int = 0
    turns: List[int] = field(default_factory=list)
    gaps: List[int] = field(default_factory=list)
    last_used: int = 0
    blk_pair: List[int] = field(default_factory=list)      # pair byte of every block that exists
    in_window: bool = False
    start_nb: int = 0                                      # blocks and tokens that exist when the window starts
    start_ntok: int = 0
    nb_seen: int = 0                                       # blocks the window replay has already laid down
    # arena placement (window entries only)
    base: int = 0
    cap: int = 0
    row0: int = 0

    @property
    def nb(self) -> int:
        return len(self.blk_pair)


@dataclass
class FleetPlan:
    shapes: List[synth.Shape]
    n_uids: int
    n_steps: int
    pair: np.ndarray                      # uint8 [n_uids]
    init_units: np.ndarray                # int64: uids that exist when the window starts
    rows: List[dict]                      # per architecture: off, q_off, layer (static); ntok, active, pos [n_steps, n_rows]
    events: List[Tuple[np.ndarray, np.ndarray]]
    new_uids: List[np.ndarray]            # units that come into existence at the start of each step
    prot_set: List[np.ndarray]
    prot_clear: List[np.ndarray]
    init_ntok: List[np.ndarray]           # per architecture: row lengths when the window starts
    n_entries: int
    stats: dict


def build_plan(shapes: List[synth.Shape], catalogues, requests: List[synth.FleetRequest], start: int, n_steps: int,
               capacity_units: int, lookup_blocks: int = 64, max_tokens: int = 32768) -> FleetPlan:
    """Replay `requests` from step 0; steps [start, start + n_steps) are the window that is laid down."""
    upb = [s.n_layers * s.n_kv_heads for s in shapes]           # units per token block = rows per entry
    entries: List[_Entry] = []
    cached: Dict[Tuple[int, int], List[int]] = {}
    active: set = set()
    wake: Dict[int, List[int]] = {}
    content = 0
    req_i = 0
    n_hit = n_miss = n_retired = 0
    win_steps = []

    def grow(e: _Entry, ntok: int, kind: int, n_prefix_blocks: int = 0, prefix_type: int = 0) -> int:
        """Extends the entry to ntok tokens; returns the units that its new blocks add."""
        before = e.nb
        for b in range(before, (ntok + BLOCK - 1) // BLOCK):
            e.blk_pair.append(4 * (prefix_type if b < n_prefix_blocks else kind) + e.transition)
        e.ntok = ntok
        return (e.nb - before) * upb[e.model]

    for t in range(start + n_steps):
        in_win = t >= start
        if t == start:
            for e in entries:
                if e.status != RETIRED:
                    e.in_window = True
                    e.start_nb = e.nb_seen = e.nb
                    e.start_ntok = e.ntok
        ev_pair: List[int] = []
        ev_out: List[int] = []
        # ---- arrivals ------------------------------------------------------------------------------------
        while req_i < len(requests) and requests[req_i].arrival <= t:
            r = requests[req_i]
            req_i += 1
            cat = catalogues[r.model][r.prefix]
            n_pb = r.prefix_len // BLOCK
            new_part = max(r.prompt_len - r.prefix_len, 1)
            idx = -1
            lst = cached.get((r.model, r.prefix), [])
            while lst:
                c = entries[lst[-1]]
                if c.status == CACHED:
                    if c.ntok + new_part + sum(r.decode) + 1 <= max_tokens:
                        idx = lst.pop()
                    break
                lst.pop()
            ev_pair += [4 * cat.block_type + cat.transition] * n_pb
            ev_out += [1 if idx >= 0 else 0] * n_pb
            if idx >= 0:
                n_hit += 1
                e = entries[idx]
                content += grow(e, e.ntok + new_part, USER_CONTEXT)
            else:
                n_miss += 1
                e = _Entry(r.model, r.prefix, cat.transition)
                e.in_window = in_win
                entries.append(e)
                idx = len(entries) - 1
                content += grow(e, r.prompt_len, USER_CONTEXT, n_pb, cat.block_type)
            e.status = ACTIVE
            e.decode_left = r.decode[0]
            e.turns = list(r.decode[1:])
            e.gaps = list(r.gap)
            e.last_used = t
            active.add(idx)
        # ---- resumes: the session looks its most recent blocks up ------------------------------------------
        for i in wake.pop(t, []):
            e = entries[i]
            if e.status != IDLE:
                continue
            e.status = ACTIVE
            e.decode_left = e.turns.pop(0)
            e.last_used = t
            active.add(i)
            recent = e.blk_pair[max(0, e.nb - lookup_blocks):]
            ev_pair += recent
            ev_out += [1] * len(recent)
        # ---- what the window step sees -------------------------------------------------------------------
        if in_win:
            rec = dict(active=sorted(active), events=(np.asarray(ev_pair, np.uint8), np.asarray(ev_out, np.uint8)),
                       new_blocks=[], ntok={}, prot={i: entries[i].nb - 1 for i in active})
            for i, e in enumerate(entries):
                if not e.in_window or e.status == RETIRED:
                    continue
                rec["ntok"][i] = e.ntok
                if e.nb > e.nb_seen:
                    rec["new_blocks"].append((i, e.nb_seen, e.nb))
                    e.nb_seen = e.nb
            win_steps.append(rec)
        # ---- decode: every active entry appends one token after this step's scoring -----------------------
        done = []
        for i in active:
            e = entries[i]
            content += grow(e, e.ntok + 1, REASONING)
            e.decode_left -= 1
            if e.decode_left <= 0:
                done.append(i)
        for i in done:
            e = entries[i]
            active.discard(i)
            if e.turns:
                e.status = IDLE
                wake.setdefault(t + 1 + e.gaps.pop(0), []).append(i)
            else:
                e.status = CACHED
                cached.setdefault((e.model, e.prefix), []).append(i)
        # ---- before the window: retire least-recently-used cached entries beyond the capacity ------------
        if not in_win and content > capacity_units:
            order = sorted((entries[i].last_used, i) for lst in cached.values() for i in lst
                           if entries[i].status == CACHED)
            for _, i in order:
                if content <= capacity_units:
                    break
                e = entries[i]
                e.status = RETIRED
                content -= e.nb * upb[e.model]
                n_retired += 1

    # ---- arena: window entries only, rows of an entry adjacent, one uid range per row ---------------------
    win_entries = [i for i, e in enumerate(entries) if e.in_window and e.status != RETIRED]
    n_arch = len(shapes)
    n_rows = [0] * n_arch
    base = 0
    for i in win_entries:
        e = entries[i]
        e.cap = e.nb
        e.base = base
        e.row0 = n_rows[e.model]
        n_rows[e.model] += upb[e.model]
        base += upb[e.model] * e.cap
    n_uids = base

    def unit_ids(e: _Entry, b_lo: int, b_hi: int) -> np.ndarray:
        r = np.arange(upb[e.model], dtype=np.int64)[:, None] * e.cap
        return (e.base + r + np.arange(b_lo, b_hi, dtype=np.int64)[None, :]).reshape(-1)

    pair = np.zeros(n_uids, np.uint8)
    init_parts = []
    init_ntok = [np.zeros(n_rows[a], np.int32) for a in range(n_arch)]
    for i in win_entries:
        e = entries[i]
        pair[unit_ids(e, 0, e.cap)] = np.tile(np.asarray(e.blk_pair[:e.cap], np.uint8), upb[e.model])
        if e.start_nb > 0:
            init_parts.append(unit_ids(e, 0, e.start_nb))
        init_ntok[e.model][e.row0:e.row0 + upb[e.model]] = e.start_ntok
    init_units = np.concatenate(init_parts) if init_parts else np.zeros(0, np.int64)

    rows = []
    for a, sh in enumerate(shapes):
        ents = [entries[i] for i in win_entries if entries[i].model == a]
        off = np.concatenate([e.base + np.arange(upb[a], dtype=np.int64) * e.cap for e in ents]) if ents else \
            np.zeros(0, np.int64)
        layer = np.tile(np.arange(upb[a], dtype=np.int32) // sh.n_kv_heads, len(ents))
        rows.append(dict(off=off, layer=layer.astype(np.int32),
                         q_off=np.arange(n_rows[a], dtype=np.int64) * sh.g * sh.dim,
                         ntok=np.zeros((n_steps, n_rows[a]), np.int32),
                         active=np.zeros((n_steps, n_rows[a]), np.uint8),
                         pos=np.full((n_steps, n_rows[a]), -1, np.int32)))

    events, new_uids, prot_set, prot_clear = [], [], [], []
    prev_prot: Dict[int, int] = {}
    for j, rec in enumerate(win_steps):
        events.append(rec["events"])
        parts = [unit_ids(entries[i], lo, hi) for (i, lo, hi) in rec["new_blocks"]]
        new_uids.append(np.concatenate(parts) if parts else np.zeros(0, np.int64))
        act = set(rec["active"])
        for i, nt in rec["ntok"].items():
            e = entries[i]
            sl = slice(e.row0, e.row0 + upb[e.model])
            rows[e.model]["ntok"][j, sl] = nt
            if i in act:
                rows[e.model]["active"][j, sl] = 1
                rows[e.model]["pos"][j, sl] = nt
        cur = rec["prot"]
        sets = [unit_ids(entries[i], b, b + 1) for i, b in cur.items() if prev_prot.get(i) != b]
        clears = [unit_ids(entries[i], b, b + 1) for i, b in prev_prot.items() if cur.get(i) != b]
        prot_set.append(np.concatenate(sets) if sets else np.zeros(0, np.int64))
        prot_clear.append(np.concatenate(clears) if clears else np.zeros(0, np.int64))
        prev_prot = dict(cur)

    stats = dict(requests_replayed=req_i, hits=n_hit, misses=n_miss, retired=n_retired, entries=len(win_entries),
                 entries_by_model=[sum(1 for i in win_entries if entries[i].model == a) for a in range(n_arch)],
                 active_per_step=[len(r["active"]) for r in win_steps],
                 new_units_per_step=[int(len(u)) for u in new_uids], init_units=int(len(init_units)),
                 events_per_step=[int(len(e[0])) for e in events])
    return FleetPlan(shapes, n_uids, n_steps, pair, init_units, rows, events, new_uids, prot_set, prot_clear, init_ntok,
                     len(win_entries), stats)


class FleetDevice:
    """Per-unit state of the fleet on the GPU and the library calls of one step, in stages.

    `pool_units` frames (from the sizing call) hold the K and V of every unit that is in HBM; `tier` is
    the pinned host tier addressed by slot.  The pool has more frames than the budget lets units stay in
    HBM, so a unit that comes into existence takes a frame from the free frames at once (a log of frame
    numbers: arrivals read it from the front, evictions append to it), and each step then evicts what HBM
    holds beyond the budget, plus up to `prefetch_cap` units that trade places with prefetched ones.

    `ahead` False: the victims are packed out in line, after the selection.
    `ahead` True: the victims leave the table at once (kvm_pack_begin, kvm_exchange_begin) and the bytes
    of both move inside the next step's first scoring launch, so the host link works beside the scoring; a
    step evicts at most `ride_max` units (what the link moves during one scoring launch), so after a whole
    prompt has arrived HBM is back at the budget some steps later.  The frames are handed out again from
    the step after that launch, and the prefetched units are in HBM from that step's selection on
    (kvm_exchange_end after its EMA: they were not scored in that launch).
    """

    def __init__(self, plan: FleetPlan, kvm, torch, pool_units: int, head_weights: List[float], tier, tier_slots: int,
                 prefetch_cap: int, window_tokens: int, decay: float = 0.9, pos_decay: float = 0.9995, seed: int = 1,
                 fresh_records: int = 65536, k_pool=None, v_pool=None, ahead: bool = False,
                 ride_max: int = 16384):
        self.plan, self.kvm, self.torch = plan, kvm, torch
        dev = "cuda"
        sh0 = plan.shapes[0]
        assert all(s.dim == sh0.dim and s.dtype == sh0.dtype and s.has_v == sh0.has_v for s in plan.shapes)
        self.dim, self.dtype = sh0.dim, sh0.dtype
        self.rec = sh0.unit_k_bytes + sh0.unit_v_bytes
        self.pool_units = int(pool_units)
        n = plan.n_uids
        self.n = n
        gen = torch.Generator(device=dev)
        gen.manual_seed(seed)
        self.gen = gen
        tdt = torch.bfloat16 if self.dtype == synth.BF16 else torch.float16
        unit_elems = BLOCK * self.dim

        def filled(m):
            t = torch.empty((m, unit_elems), dtype=tdt, device=dev)
            step = max(1, (1 << 27) // unit_elems)
            for i in range(0, m, step):
                j = min(m, i + step)
                t[i:j] = torch.randn((j - i, unit_elems), generator=gen, device=dev, dtype=torch.float32).to(tdt)
            return t

        self.k_pool = filled(self.pool_units) if k_pool is None else k_pool
        self.v_pool = filled(self.pool_units) if v_pool is None else v_pool
        self.pool = kvm.make_pool(self.k_pool.view(torch.int16), self.v_pool.view(torch.int16), self.dim, self.dtype)
        n_init = len(plan.init_units)
        assert n_init <= self.pool_units, (n_init, self.pool_units)
        perm = torch.randperm(self.pool_units, generator=gen, device=dev).to(torch.int32)
        self.slot_tbl = torch.full((n,), -1, dtype=torch.int32, device=dev)
        self.state = torch.zeros(n, dtype=torch.uint8, device=dev)
        init = torch.from_numpy(plan.init_units).to(dev)
        self.slot_tbl[init] = perm[:n_init]
        self.state[init] = RES
        self.free_frames = perm[n_init:].contiguous()           # frames no unit holds yet
        self.pair = torch.from_numpy(plan.pair).to(dev)
        self.mass = torch.zeros(n, dtype=torch.float32, device=dev)
        self.S = torch.zeros(n, dtype=torch.float32, device=dev)
        self.prio = torch.zeros(n, dtype=torch.float32, device=dev)
        self.key = torch.zeros(n, dtype=torch.float32, device=dev)
        self.cand = torch.zeros(n, dtype=torch.uint8, device=dev)
        self.hits = torch.zeros(16, dtype=torch.int32, device=dev)
        self.misses = torch.zeros(16, dtype=torch.int32, device=dev)
        self.p_hat = torch.zeros(16, dtype=torch.float32, device=dev)
        self.n_bad = torch.zeros(1, dtype=torch.int32, device=dev)
        self.n_v = torch.zeros(1, dtype=torch.int64, device=dev)
        self.n_pf = torch.zeros(1, dtype=torch.int64, device=dev)
        self.P = int(prefetch_cap)
        # the library takes these as fp32: keep the values it will really see, so that a reference fed the
        # same numbers computes with the same constants
        self.decay, self.pos_decay = float(np.float32(decay)), float(np.float32(pos_decay))
        self.scale = float(np.float32(1.0 / np.sqrt(self.dim)))
        self.tier, self.tier_slots = tier, int(tier_slots)
        self.next_slot = 0
        self.arch = []
        ws_bytes = [kvm.kvm_workspace_bytes(kvm.OP_SELECT, n), 256]
        for a, sh in enumerate(plan.shapes):
            r = plan.rows[a]
            n_rows = len(r["off"])
            d = dict(shape=sh, n_rows=n_rows, g=sh.g, q_elems=n_rows * sh.g * sh.dim,
                     off=torch.from_numpy(r["off"]).to(dev), q_off=torch.from_numpy(r["q_off"]).to(dev),
                     layer=torch.from_numpy(r["layer"]).to(dev),
                     ntok=torch.from_numpy(r["ntok"]).to(dev), active=torch.from_numpy(r["active"]).to(dev),
                     pos=torch.from_numpy(r["pos"]).to(dev),
                     init_ntok=torch.from_numpy(plan.init_ntok[a]).to(dev),
                     weight=torch.full((max(n_rows, 1),), float(head_weights[a]), dtype=torch.float32, device=dev)[:n_rows],
                     window=torch.full((sh.n_layers,), int(window_tokens), dtype=torch.int32, device=dev))
            d["q"] = [torch.randn(max(d["q_elems"], 8), generator=gen, device=dev, dtype=torch.float32).to(tdt)
                      for _ in range(4)]
            ws_bytes.append(kvm.kvm_workspace_bytes(kvm.OP_SCORE, n, n_rows, sh.g, sh.dim))
            self.arch.append(d)
        self.ws = torch.full((max(ws_bytes),), 0x7F, dtype=torch.uint8, device=dev)
        self.events = [(torch.from_numpy(p).to(dev), torch.from_numpy(o).to(dev)) for p, o in plan.events]
        self.new_uids = [torch.from_numpy(u).to(dev) for u in plan.new_uids]
        self.prot_set = [torch.from_numpy(u).to(dev) for u in plan.prot_set]
        self.prot_clear = [torch.from_numpy(u).to(dev) for u in plan.prot_clear]
        self.ahead = bool(ahead)
        self.ride_max = int(ride_max)
        self.n_new = [len(u) for u in plan.new_uids]
        k_max = sum(self.n_new) + self.P
        self.victims = torch.full((max(k_max, 1),), -1, dtype=torch.int64, device=dev)
        self.pf_list = torch.full((max(self.P, 1),), -1, dtype=torch.int64, device=dev)
        # the log of free frames: [free_head, free_ready) may be handed to arrivals, [free_ready, free_tail)
        # belong to victims whose bytes have not left yet; evict_to_budget() fills it first
        self.free = None
        self.free_head = self.free_ready = self.free_tail = 0
        self.budget = self.resident = 0
        self.evict_now = 0                                     # victims of the current step beyond the exchange
        self.evicted = []                                      # per step, for whoever accounts for the link
        n_ride = max(sum(self.n_new), 1) + self.P
        self.ride_frame = torch.full((n_ride,), -1, dtype=torch.int32, device=dev)
        self.ride_host = torch.full((n_ride,), -1, dtype=torch.int64, device=dev)
        self.ride = None               # (pairs, log position behind the freed frames) waiting for a scoring launch
        self.settle_pairs = 0          # swap pairs whose prefetched units still wait for their table entries
        self.fresh_records = int(min(fresh_records, max(max(self.n_new), 1)))
        self.fresh = torch.randn(self.fresh_records * self.rec // 2, generator=gen, device=dev,
                                 dtype=torch.float32).to(tdt).view(torch.uint8)
        self.host_slot_ids = None

    # ---- descriptors ------------------------------------------------------------------------------------
    def rows(self, a: int, j: Optional[int]):
        """Row descriptor of architecture `a` at window step j (None: the lengths before the window, all rows decoding)."""
        d = self.arch[a]
        ntok = d["init_ntok"] if j is None else d["ntok"][j]
        act = None if j is None else d["active"][j]
        return self.kvm.make_rows(ntok, d["off"], d["q_off"], self.slot_tbl, d["g"], d["q_elems"], act)

    # ---- stages -------------------------------------------------------------------------------------------
    def arrive(self, j: int):
        """The units that come into existence at step j take free frames, with freshly written K and V; the
        blocks being written are marked PROTECTED, the ones no longer written to are released."""
        kvm = self.kvm
        n = self.n_new[j]
        assert self.free_head + n <= self.free_ready, "no free frame for a new unit"
        frames = self.free[self.free_head:self.free_head + n]
        self.free_head += n
        self.resident += n
        for lo in range(0, n, self.fresh_records):
            cnt = min(self.fresh_records, n - lo)
            kvm.kvm_unpack(self.pool, self.slot_tbl, self.state, self.new_uids[j][lo:lo + cnt], cnt,
                           frames[lo:lo + cnt], self.fresh, None, n_bad=self.n_bad)
        if len(self.prot_clear[j]):
            self.state[self.prot_clear[j]] &= 255 - PROT
        if len(self.prot_set[j]):
            self.state[self.prot_set[j]] |= PROT

    def beta(self, j: int):
        p, o = self.events[j]
        self.kvm.kvm_beta_update(p if len(p) else None, o if len(o) else None, self.hits, self.misses, self.p_hat,
                                 n_bad=self.n_bad)

    def score(self, j: Optional[int], q_set: int = 0):
        ride, self.ride = self.ride, None
        for a, d in enumerate(self.arch):
            if d["n_rows"]:
                if ride is not None:                       # the bytes of the last step's moves travel inside this launch
                    self.kvm.kvm_score_step_xfer(self.pool, self.rows(a, j), d["q"][q_set % 4], self.scale, self.mass,
                                                 self.ws, self.ride_frame, self.ride_host, ride[0], self.tier)
                    self.free_ready = ride[1]          # later launches on the stream may reuse those frames
                    ride = None
                else:
                    self.kvm.kvm_score_step(self.pool, self.rows(a, j), d["q"][q_set % 4], self.scale, self.mass,
                                            self.ws)
        assert ride is None, "an eviction in two parts needs a scoring launch to carry its bytes"

    def ema(self, j: Optional[int]):
        for a, d in enumerate(self.arch):
            if d["n_rows"]:
                self.kvm.kvm_ema_update(self.rows(a, j), self.mass, self.decay, d["weight"], self.pair, self.p_hat,
                                        self.state, self.S, self.prio)

    def settle(self):
        """The units prefetched by the exchange whose bytes the last scoring launch moved get their frames."""
        if self.settle_pairs:
            self.kvm.kvm_exchange_end(self.slot_tbl, self.state, self.pf_list, self.ride_frame, self.settle_pairs)
            self.settle_pairs = 0

    def prefetch_keys(self, j: int):
        if not self.P:
            return
        for a, d in enumerate(self.arch):
            if d["n_rows"]:
                self.kvm.kvm_prefetch_keys(self.rows(a, j), d["layer"], d["pos"][j], d["window"], self.state, self.pair,
                                           self.p_hat, self.pos_decay, self.key, self.cand)

    def select(self, j: int):
        """One selection of victims over the shared pool (what HBM holds beyond the budget + the units that
        trade places with prefetched ones) and one of the prefetch list."""
        kvm = self.kvm
        if self.P:
            kvm.kvm_select_victims(self.key, self.cand, self.pf_list, self.n_pf, self.ws, k=self.P)
        over = max(self.resident - self.budget, 0)
        self.evict_now = min(over, self.ride_max) if self.ahead else over
        k = self.evict_now + self.P
        self.victims.fill_(-1)
        kvm.kvm_select_victims(self.prio, self.state, self.victims[:max(k, 1)], self.n_v, self.ws, k=k)

    def move(self, j: int):
        """The first P victims trade places with the prefetch list in the slot-addressed tier; the others go
        to fresh tier slots and their frames to the free log: packed out here, or (`ahead`) taken out of the
        table here and copied out by the next scoring launch."""
        kvm = self.kvm
        P = self.P
        assert self.ride is None and self.settle_pairs == 0
        if P and self.ahead:
            kvm.kvm_exchange_begin(self.pool, self.slot_tbl, self.state, self.victims[:P], self.pf_list, P,
                                   self.tier_slots, self.ride_frame[:P], self.ride_host[:P], n_out_dev=self.n_v,
                                   n_in_dev=self.n_pf, n_bad=self.n_bad)
        elif P:
            kvm.kvm_exchange(self.pool, self.slot_tbl, self.state, self.victims[:P], self.pf_list, P, self.tier,
                             n_out_dev=self.n_v, n_in_dev=self.n_pf, n_bad=self.n_bad)
        m = self.evict_now
        self.evicted.append(m)
        if m:
            assert self.next_slot + m <= self.tier_slots, "host tier full"
            assert self.free_tail + m <= self.free.numel(), "free log full"
            slots = self.torch.arange(self.next_slot, self.next_slot + m, dtype=self.torch.int32, device="cuda")
            freed = self.free[self.free_tail:self.free_tail + m]
            if self.ahead:
                kvm.kvm_pack_begin(self.pool, self.slot_tbl, self.state, self.victims[P:P + m], m, slots,
                                   self.tier_slots, self.ride_frame[P:P + m], self.ride_host[P:P + m],
                                   n_bad=self.n_bad)
                freed.copy_(self.ride_frame[P:P + m])
            else:
                kvm.kvm_pack(self.pool, self.slot_tbl, self.state, self.victims[P:P + m], m, slots, freed, None,
                             self.tier[self.next_slot * self.rec:(self.next_slot + m) * self.rec], n_bad=self.n_bad)
                self.free_ready = self.free_tail + m
            self.free_tail += m
            self.next_slot += m
            self.resident -= m
        if self.ahead and P + m:
            self.ride = (P + m, self.free_tail)
            self.settle_pairs = P

    def flush(self):
        """Bytes that no scoring launch has carried yet move in a launch of their own."""
        if self.ride is not None:
            ride, self.ride = self.ride, None
            d = self.arch[0]
            none = self.kvm.make_rows(d["init_ntok"][:0], d["off"][:0], d["q_off"][:0], self.slot_tbl, d["g"], 0)
            self.kvm.kvm_score_step_xfer(self.pool, none, d["q"][0], self.scale, self.mass, self.ws, self.ride_frame,
                                         self.ride_host, ride[0], self.tier)
            self.free_ready = ride[1]
        self.settle()

    def step(self, j: int):
        self.arrive(j)
        self.beta(j)
        self.score(j, j)
        self.ema(j)
        self.settle()
        self.prefetch_keys(j)
        self.select(j)
        self.move(j)

    # ---- warm start -----------------------------------------------------------------------------------------
    def first_pass(self):
        """Everything that exists when the window starts is in HBM and every row decodes once: scoring and
        EMA of all units (which makes them eligible for eviction afterwards)."""
        self.beta_none()
        self.score(None, 0)
        self.ema(None)

    def beta_none(self):
        self.kvm.kvm_beta_update(None, None, self.hits, self.misses, self.p_hat, n_bad=self.n_bad)

    def evict_to_budget(self, budget_units: int, keep_records: int, order: np.ndarray, scratch, chunk: int = 32768):
        """Bulk eviction down to `budget_units` units in HBM.  `order` permutes the victim list (uid ascending
        as selected); the first `keep_records` victims of the permuted list keep their records in the tier
        (slots 0 ..), the others go through `scratch` and are dropped from tier 1 as well (ON_HOST cleared:
        demoted below the tiers this path handles; they are neither scored nor prefetched again).
        Returns the number of victims."""
        torch, kvm = self.torch, self.kvm
        n_res = int((self.state & RES).sum().item())
        k0 = max(n_res - budget_units, 0)
        victims = torch.full((max(k0, 1),), -1, dtype=torch.int64, device="cuda")
        kvm.kvm_select_victims(self.prio, self.state, victims, self.n_v, self.ws, k=-1, budget_units=budget_units)
        torch.cuda.synchronize()
        assert int(self.n_v.item()) == k0, (int(self.n_v.item()), k0)
        victims = victims[torch.from_numpy(order[:k0]).to("cuda")].contiguous() if k0 else victims[:0]
        freed = torch.full((max(k0, 1),), -1, dtype=torch.int32, device="cuda")
        slots = torch.arange(max(k0, 1), dtype=torch.int32, device="cuda")
        keep = min(keep_records, k0)
        assert keep <= self.tier_slots
        for lo in range(0, k0, chunk):
            cnt = min(chunk, k0 - lo)
            if lo + cnt <= keep:
                dst = self.tier[lo * self.rec:(lo + cnt) * self.rec]
            elif lo >= keep:
                dst = scratch[:cnt * self.rec]
            else:                                   # the chunk straddles the boundary: split it
                a = keep - lo
                kvm.kvm_pack(self.pool, self.slot_tbl, self.state, victims[lo:lo + a], a, slots[lo:lo + a],
                             freed[lo:lo + a], None, self.tier[lo * self.rec:keep * self.rec], n_bad=self.n_bad)
                kvm.kvm_pack(self.pool, self.slot_tbl, self.state, victims[keep:lo + cnt], cnt - a, slots[keep:lo + cnt],
                             freed[keep:lo + cnt], None, scratch[:(cnt - a) * self.rec], n_bad=self.n_bad)
                continue
            kvm.kvm_pack(self.pool, self.slot_tbl, self.state, victims[lo:lo + cnt], cnt, slots[lo:lo + cnt],
                         freed[lo:lo + cnt], None, dst, n_bad=self.n_bad)
        if k0 > keep:
            self.state[victims[keep:]] &= 255 - HOST
        self.next_slot = keep
        # the free log starts with the frames just freed, then the frames never used; room behind them for
        # every frame the window's evictions can free
        frames = torch.cat([freed[:k0], self.free_frames]) if k0 else self.free_frames
        self.free = torch.full((frames.numel() + sum(self.n_new) + 8,), -1, dtype=torch.int32, device="cuda")
        self.free[:frames.numel()] = frames
        self.free_head, self.free_ready, self.free_tail = 0, frames.numel(), frames.numel()
        self.budget = self.resident = n_res - k0
        torch.cuda.synchronize()
        return k0, victims

    # ---- row samples for a reference ---------------------------------------------------------------------------
    def host_rows(self, a: int, j: Optional[int], pick: np.ndarray, q_set: int = 0) -> dict:
        """Host copy of rows `pick` of architecture `a` as they stand at window step j: lengths, a compact
        table and pool holding only their units that are in HBM, their queries, and their uids."""
        torch = self.torch
        d = self.arch[a]
        ntok_all = d["init_ntok"] if j is None else d["ntok"][j]
        ntok = ntok_all.cpu().numpy()[pick]
        off = d["off"].cpu().numpy()[pick]
        nb = (ntok.astype(np.int64) + BLOCK - 1) // BLOCK
        uids = np.concatenate([o + np.arange(k) for o, k in zip(off, nb)]) if len(pick) else np.zeros(0, np.int64)
        u_dev = torch.from_numpy(uids).to("cuda")
        slots = self.slot_tbl[u_dev]
        res = slots >= 0
        k_host = self.k_pool[slots[res].long()].view(torch.int16).cpu().numpy().view(np.uint16)
        tbl = np.full(len(uids), -1, np.int32)
        tbl[res.cpu().numpy()] = np.arange(int(res.sum().item()), dtype=np.int32)
        new_off = np.zeros(len(pick), np.int64)
        new_off[1:] = np.cumsum(nb[:-1])
        gd = d["g"] * self.dim
        q_all = d["q"][q_set % 4].view(torch.int16).cpu().numpy().view(np.uint16)
        q_rows = np.concatenate([q_all[r * gd:(r + 1) * gd] for r in pick])
        return dict(k_pool=k_host, ntok=ntok, off=new_off, q_off=np.arange(len(pick), dtype=np.int64) * gd, tbl=tbl,
                    q=q_rows, g=d["g"], uids=uids, resident=res.cpu().numpy())
