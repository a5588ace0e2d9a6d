"""The fleet step on the CPU oracle: the same stages as paper_2604_26968_amd.fleet.FleetDevice, on
numpy arrays, through the oracle's functions only.  Inputs (pools, tables, queries, fresh records) are
copied from the device driver once, before any stage runs; from then on the two sides only meet where
a test compares them."""
from __future__ import annotations

import numpy as np

RES, HOST, PROT, SCORED = 1, 2, 4, 8


class FleetRef:
    def __init__(self, o, dev, plan):
        """`dev`: a freshly constructed FleetDevice (nothing run yet)."""
        self.o, self.plan = o, plan
        t = lambda x: x.detach().cpu().numpy().copy()
        self.k16 = t(dev.k_pool.view(dev.torch.int16)).view(np.uint16)
        self.v16 = t(dev.v_pool.view(dev.torch.int16)).view(np.uint16)
        self.k8 = self.k16.view(np.uint8).reshape(dev.pool_units, -1)
        self.v8 = self.v16.view(np.uint8).reshape(dev.pool_units, -1)
        self.uk, self.uv = self.k8.shape[1], self.v8.shape[1]
        self.rec = self.uk + self.uv
        self.tbl, self.state, self.pair = t(dev.slot_tbl), t(dev.state), plan.pair.copy()
        self.free_frames = t(dev.free_frames)
        n = plan.n_uids
        self.mass = np.zeros(n, np.float32)
        self.S, self.prio = np.zeros(n, np.float32), np.zeros(n, np.float32)
        self.key, self.cand = np.zeros(n, np.float32), np.zeros(n, np.uint8)
        self.hits, self.misses = np.zeros(16, np.uint32), np.zeros(16, np.uint32)
        self.p_hat = np.zeros(16, np.float32)
        self.n_bad = np.zeros(1, np.uint32)
        self.P, self.decay, self.pos_decay, self.scale = dev.P, dev.decay, dev.pos_decay, dev.scale
        self.dim, self.dtype = dev.dim, dev.dtype
        self.tier = np.zeros((dev.tier_slots, self.rec), np.uint8)
        self.next_slot = 0
        self.fresh = t(dev.fresh).reshape(-1, self.rec)
        self.n_new = list(dev.n_new)
        # the free-frame log and the residency bookkeeping, kept here independently of the driver's
        self.ahead, self.ride_max = dev.ahead, dev.ride_max
        self.free = np.zeros(0, np.int32)
        self.free_head = self.free_ready = self.free_tail = 0
        self.pending_ready = None
        self.pending_in = None          # (prefetched uids, their frames): in HBM once the driver settles the exchange
        self.budget = self.resident = 0
        self.evict_now = 0
        self.arch = []
        for a, d in enumerate(dev.arch):
            sh = d["shape"]
            args = sh.model_args()
            self.arch.append(dict(g=sh.g, n_rows=d["n_rows"], off=plan.rows[a]["off"], q_off=plan.rows[a]["q_off"],
                                  layer=plan.rows[a]["layer"], ntok=plan.rows[a]["ntok"], active=plan.rows[a]["active"],
                                  pos=plan.rows[a]["pos"], init_ntok=plan.init_ntok[a],
                                  weight=np.full(d["n_rows"], float(o.size(**args)["head_weight"]), np.float32),
                                  window=t(d["window"]),
                                  q=[t(q.view(dev.torch.int16)).view(np.uint16) for q in d["q"]]))
        self.victims = np.zeros(0, np.int64)
        self.pf_list = np.zeros(0, np.int64)

    def _rows(self, a, j):
        d = self.arch[a]
        return (d["init_ntok"], None) if j is None else (d["ntok"][j], d["active"][j])

    def arrive(self, j):
        n = self.n_new[j]
        uids = self.plan.new_uids[j]
        assert self.free_head + n <= self.free_ready
        frames = self.free[self.free_head:self.free_head + n]
        self.free_head += n
        self.resident += n
        step = len(self.fresh)
        for lo in range(0, n, step):
            cnt = min(step, n - lo)
            self.o.unpack(self.k8, self.v8, self.uk, self.uv, self.tbl, self.state, uids[lo:lo + cnt],
                          frames[lo:lo + cnt], self.fresh[:cnt], n_bad=self.n_bad)
        self.state[self.plan.prot_clear[j]] &= 255 - PROT
        self.state[self.plan.prot_set[j]] |= PROT

    def beta(self, j):
        p, o_ = (np.zeros(0, np.uint8), np.zeros(0, np.uint8)) if j is None else self.plan.events[j]
        self.p_hat = self.o.beta_update(p, o_, self.hits, self.misses)

    def score(self, j, q_set=0):
        if self.pending_ready is not None:          # the driver's scoring launch carries the last eviction's bytes
            self.free_ready, self.pending_ready = self.pending_ready, None
        for a, d in enumerate(self.arch):
            if d["n_rows"]:
                ntok, act = self._rows(a, j)
                self.o.score_step(self.k16, self.dim, self.dtype, ntok, d["off"], d["q_off"], self.tbl,
                                  d["q"][q_set % 4], d["g"], self.scale, self.mass, row_active=act)

    def score_none(self):
        """The driver's flush: bytes move, nothing is scored."""
        if self.pending_ready is not None:
            self.free_ready, self.pending_ready = self.pending_ready, None

    def ema(self, j):
        for a, d in enumerate(self.arch):
            if d["n_rows"]:
                ntok, act = self._rows(a, j)
                self.o.ema_update(ntok, d["off"], self.mass, self.decay, d["weight"], self.pair, self.p_hat, self.state,
                                  self.S, self.prio, row_active=act)

    def settle(self):
        """The prefetched units of an exchange in three parts get their frames (what kvm_exchange_end does)."""
        if self.pending_in is not None:
            uids, frames = self.pending_in
            self.tbl[uids] = frames
            self.state[uids] = (self.state[uids] & (255 - HOST)) | RES
            self.pending_in = None

    def prefetch_keys(self, j):
        if not self.P:
            return
        for a, d in enumerate(self.arch):
            if d["n_rows"]:
                self.o.prefetch_keys(d["ntok"][j], d["off"], d["layer"], d["pos"][j], d["window"], self.state, self.pair,
                                     self.p_hat, self.pos_decay, self.key, self.cand)

    def select(self, j):
        self.pf_list = self.o.select_victims(self.key, self.cand, k=self.P) if self.P else np.zeros(0, np.int64)
        over = max(self.resident - self.budget, 0)
        self.evict_now = min(over, self.ride_max) if self.ahead else over
        self.victims = self.o.select_victims(self.prio, self.state, k=self.evict_now + self.P)

    def move(self, j):
        P = self.P
        n_pairs = min(P, len(self.victims), len(self.pf_list))
        if n_pairs:
            ins = self.pf_list[:n_pairs]
            before = self.tbl[ins].copy()
            self.o.exchange(self.k8, self.v8, self.uk, self.uv, self.tbl, self.state, self.victims[:n_pairs],
                            ins, self.tier, n_bad=self.n_bad)
            if self.ahead:
                # in three parts the bytes move inside the next scoring launch and the prefetched units get their
                # table entries after that step's EMA: until then they read as on the host, at their old slot
                # (nothing looks at the frames or the records meanwhile: neither unit of a pair is in HBM)
                done = self.tbl[ins] >= 0
                self.pending_in = (ins[done], self.tbl[ins[done]].copy())
                self.tbl[ins[done]] = before[done]
                self.state[ins[done]] = (self.state[ins[done]] & (255 - RES)) | HOST
        # whether the bytes leave now or inside the next scoring launch, tables, state and tier end up as a
        # plain pack leaves them, and nothing reads the records or reuses the frames in between
        m = self.evict_now
        if m:
            out = self.victims[P:P + m]
            assert len(out) == m, "fewer eligible victims than HBM holds units beyond the budget"
            slots = np.arange(self.next_slot, self.next_slot + m, dtype=np.int32)
            staging, freed = self.o.pack(self.k8, self.v8, self.uk, self.uv, self.tbl, self.state, out, slots,
                                         n_bad=self.n_bad)
            self.tier[self.next_slot:self.next_slot + m] = staging
            self.free[self.free_tail:self.free_tail + m] = freed
            if self.ahead:
                self.pending_ready = self.free_tail + m
            else:
                self.free_ready = self.free_tail + m
            self.free_tail += m
            self.next_slot += m
            self.resident -= m

    # ---- warm start ------------------------------------------------------------------------------------------
    def first_pass(self):
        self.beta(None)
        self.score(None, 0)
        self.ema(None)

    def evict_to_budget(self, budget_units, keep_records, order):
        victims = self.o.select_victims(self.prio, self.state, k=-1, budget_units=budget_units)
        k0 = len(victims)
        victims = victims[order[:k0]]
        slots = np.arange(k0, dtype=np.int32)
        staging, freed = self.o.pack(self.k8, self.v8, self.uk, self.uv, self.tbl, self.state, victims, slots,
                                     n_bad=self.n_bad)
        keep = min(keep_records, k0)
        self.tier[:keep] = staging[:keep]
        self.state[victims[keep:]] &= 255 - HOST
        self.next_slot = keep
        frames = np.concatenate([freed[:k0], self.free_frames])
        self.free = np.full(len(frames) + sum(self.n_new) + 8, -1, np.int32)
        self.free[:len(frames)] = frames
        self.free_head, self.free_ready, self.free_tail = 0, len(frames), len(frames)
        self.budget = self.resident = int((self.state & RES).sum())
        return k0, victims
