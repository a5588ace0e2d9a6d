"""Seeded synthetic inputs for the KV-cache management pass.

This module only *makes data*: random pools, queries, block tables, event
streams, with the shapes of the benchmark configurations.  It contains none of
the method's arithmetic (no softmax, EMA, posterior, selection) and is the one
module that both the GPU tests and the CPU oracle tests draw inputs from.

16-bit floating point data is carried as ``uint16`` bit patterns in numpy.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

BF16, FP16 = 0, 1
BLOCK = 16


# ----------------------------------------------------------------- formats
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns, round to nearest even (NaN kept quiet)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    rounded = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    nan = np.isnan(x)
    out = rounded.astype(np.uint16)
    if np.any(nan):
        out = np.where(nan, np.uint16(0x7FC0), out)
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32)


def to_bits(x: np.ndarray, dtype: int) -> np.ndarray:
    if dtype == BF16:
        return f32_to_bf16_bits(x)
    return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16).view(np.uint16)


def from_bits(b: np.ndarray, dtype: int) -> np.ndarray:
    if dtype == BF16:
        return bf16_bits_to_f32(b)
    return b.view(np.float16).astype(np.float32)


def unit_from_tokens(tok_bits: np.ndarray) -> np.ndarray:
    """[16, dim] token-major bit patterns -> one K unit in pool layout [dim/8][16][8], flattened."""
    t, dim = tok_bits.shape
    assert t == BLOCK and dim % 8 == 0
    return np.ascontiguousarray(tok_bits.reshape(BLOCK, dim // 8, 8).transpose(1, 0, 2)).reshape(-1)


def tokens_from_unit(unit_bits: np.ndarray, dim: int) -> np.ndarray:
    """Inverse of :func:`unit_from_tokens`: flattened unit -> [16, dim]."""
    return np.ascontiguousarray(unit_bits.reshape(dim // 8, BLOCK, 8).transpose(1, 0, 2)).reshape(BLOCK, dim)


# ------------------------------------------------------------------- cases
@dataclass
class Shape:
    """One architecture's share of a workload."""
    n_layers: int
    n_q_heads: int
    n_kv_heads: int          # 1 for MLA (the single latent head)
    dim: int                 # head_dim, or d_latent + d_rope for MLA
    dtype: int = BF16
    has_v: bool = True
    seq_lens: List[int] = field(default_factory=list)

    @property
    def g(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def unit_k_bytes(self) -> int:
        return BLOCK * self.dim * 2

    def model_args(self) -> dict:
        """The shape as the keyword arguments the sizing calls take (a latent row of 576 channels is
        512 latent + 64 rope channels; any other latent width is passed as latent only)."""
        if self.has_v:
            return dict(n_layers=self.n_layers, n_q_heads=self.n_q_heads, n_kv_heads=self.n_kv_heads,
                        head_dim=self.dim)
        rope = 64 if self.dim == 576 else 0
        return dict(n_layers=self.n_layers, n_q_heads=self.n_q_heads, n_kv_heads=self.n_q_heads,
                    head_dim=self.dim, d_latent=self.dim - rope, d_rope=rope)

    @property
    def unit_v_bytes(self) -> int:
        return BLOCK * self.dim * 2 if self.has_v else 0


@dataclass
class Case:
    shape: Shape
    n_slots: int
    k_pool: np.ndarray        # uint16 [n_slots, 16*dim]
    v_pool: Optional[np.ndarray]  # uint16 [n_slots, 16*dim] or None
    row_ntok: np.ndarray      # int32 [n_rows]
    row_off: np.ndarray       # int64 [n_rows]
    row_q_off: np.ndarray     # int64 [n_rows]
    row_seq: np.ndarray       # int32 [n_rows] sequence index of the row
    slot_tbl: np.ndarray      # int32 [n_uids]
    state: np.ndarray         # uint8 [n_uids]
    pair: np.ndarray          # uint8 [n_uids]
    n_uids: int

    @property
    def n_rows(self) -> int:
        return len(self.row_ntok)


def make_case(shape: Shape, seed: int, spare_slots: int = 0, uid_gap: int = 0,
              pair_weights: Optional[np.ndarray] = None, protect_last: bool = True,
              poison_tail: bool = False) -> Case:
    """Build a fully resident paged cache for ``shape``.

    Rows are ordered (sequence, layer, kv head).  Every unit gets a random pool
    slot (a random permutation, so neighbouring blocks are scattered).  K and V
    are i.i.d. N(0, 1) rounded to the element type.  ``uid_gap`` leaves that
    many unused uids after every row.  ``pair`` is drawn per (sequence, block)
    and shared by the units of that block.  The last block of every sequence
    is marked PROTECTED when ``protect_last``.  With ``poison_tail`` the token
    positions past a row's length hold NaN bit patterns.
    """
    rng = np.random.default_rng(seed)
    L, H, dim = shape.n_layers, shape.n_kv_heads, shape.dim
    n_seq = len(shape.seq_lens)
    rows_ntok, rows_seq = [], []
    for s, n in enumerate(shape.seq_lens):
        for _ in range(L * H):
            rows_ntok.append(n)
            rows_seq.append(s)
    row_ntok = np.asarray(rows_ntok, np.int32)
    row_seq = np.asarray(rows_seq, np.int32)
    nb = (row_ntok.astype(np.int64) + BLOCK - 1) // BLOCK
    row_off = np.zeros(len(nb), np.int64)
    if len(nb):
        row_off[1:] = np.cumsum(nb[:-1] + uid_gap)
    n_uids = int((nb + uid_gap).sum()) if len(nb) else 0
    n_units = int(nb.sum())
    n_slots = n_units + spare_slots
    unit_elems = BLOCK * dim

    k_pool = to_bits(rng.standard_normal((n_slots, unit_elems), dtype=np.float32), shape.dtype)
    v_pool = (to_bits(rng.standard_normal((n_slots, unit_elems), dtype=np.float32), shape.dtype)
              if shape.has_v else None)

    perm = rng.permutation(n_slots)[:n_units].astype(np.int32)
    slot_tbl = np.full(n_uids, -1, np.int32)
    state = np.zeros(n_uids, np.uint8)
    pair = np.zeros(n_uids, np.uint8)
    if pair_weights is None:
        pair_weights = np.full(16, 1.0 / 16)
    seq_pairs = [rng.choice(16, size=(n + BLOCK - 1) // BLOCK, p=pair_weights).astype(np.uint8)
                 for n in shape.seq_lens]
    u = 0
    for r in range(len(nb)):
        o, k = int(row_off[r]), int(nb[r])
        slot_tbl[o:o + k] = perm[u:u + k]
        u += k
        state[o:o + k] = 1
        pair[o:o + k] = seq_pairs[row_seq[r]]
        if protect_last and k:
            state[o + k - 1] |= 4
        tail = int(row_ntok[r]) % BLOCK
        if poison_tail and tail:
            unit = k_pool[slot_tbl[o + k - 1]].reshape(dim // 8, BLOCK, 8)
            unit[:, tail:, :] = 0x7FC1 if shape.dtype == BF16 else 0x7E01
    g = shape.g
    row_q_off = (np.arange(len(nb), dtype=np.int64) * g * dim)
    return Case(shape, n_slots, k_pool, v_pool, row_ntok, row_off, row_q_off, row_seq, slot_tbl,
                state, pair, n_uids)


def row_head_index(case: Case) -> np.ndarray:
    """layer * n_kv_heads + head of every row (rows are ordered sequence, layer, head)."""
    lh = case.shape.n_layers * case.shape.n_kv_heads
    return (np.arange(case.n_rows) % lh).astype(np.int32)


def row_layer_index(case: Case) -> np.ndarray:
    return (row_head_index(case) // case.shape.n_kv_heads).astype(np.int32)


def make_queries(case: Case, seed: int, scale: float = 1.0) -> np.ndarray:
    """Fresh N(0, scale^2) queries for every row: uint16 [n_rows * g * dim]."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal(case.n_rows * case.shape.g * case.shape.dim, dtype=np.float32) * scale
    return to_bits(x, case.shape.dtype)


def make_events(n: int, seed: int, pair_weights: Optional[np.ndarray] = None,
                reuse_prob: Optional[np.ndarray] = None):
    """n reuse events: pair ~ categorical(pair_weights) (uniform by default),
    outcome ~ Bernoulli(reuse_prob[pair]) (0.5 by default)."""
    rng = np.random.default_rng(seed)
    if pair_weights is None:
        pair_weights = np.full(16, 1.0 / 16)
    if reuse_prob is None:
        reuse_prob = np.full(16, 0.5)
    p = rng.choice(16, size=n, p=pair_weights).astype(np.uint8)
    o = (rng.random(n) < reuse_prob[p]).astype(np.uint8)
    return p, o


def categorical_weights(seed: int, n: int = 16) -> np.ndarray:
    """A fixed seeded probability vector (normalised gamma draws)."""
    rng = np.random.default_rng(seed)
    w = rng.gamma(1.0, 1.0, size=n)
    return w / w.sum()


def uniform_lengths(n_seq: int, lo: int, hi: int, seed: int) -> List[int]:
    rng = np.random.default_rng(seed)
    return [int(v) for v in rng.integers(lo, hi + 1, size=n_seq)]


# ------------------------------------------------------- named workloads
def tiny_gqa(seed: int = 1) -> Case:
    """1 layer, 4 q / 2 KV heads, d 64, fp16, one 512-token sequence."""
    return make_case(Shape(1, 4, 2, 64, FP16, True, [512]), seed, protect_last=False)


def llama8b_twin(seed: int = 11, n_seq: int = 3, n_layers: int = 2) -> Case:
    """Row shapes of the Llama-3-8B-shaped workload (8 KV heads, g 4, d 128, lengths in
    [2048, 8192]) with few sequences and layers."""
    lens = uniform_lengths(n_seq, 2048, 8192, seed + 1)
    return make_case(Shape(n_layers, 32, 8, 128, BF16, True, lens), seed,
                     pair_weights=categorical_weights(seed + 2), spare_slots=64)


def llama70b_twin(seed: int = 21, n_tok: int = 131072, n_layers: int = 1, n_kv: int = 1) -> Case:
    """One very long row family (8192 blocks per row, g 8, d 128)."""
    return make_case(Shape(n_layers, 8 * n_kv, n_kv, 128, BF16, True, [n_tok]), seed,
                     pair_weights=categorical_weights(seed + 2))


def mla_twin(seed: int = 31, n_seq: int = 1, n_tok: int = 4096, n_layers: int = 1) -> Case:
    """Latent KV of 576 channels scored by 128 absorbed queries, no V."""
    return make_case(Shape(n_layers, 128, 1, 576, BF16, False, [n_tok] * n_seq), seed,
                     pair_weights=categorical_weights(seed + 2))


# ------------------------------------------------- full-size device workloads
class DeviceWorkload:
    """A fully resident paged cache of a given Shape built directly in GPU memory.

    Same structure as :func:`make_case` (rows ordered (sequence, layer, kv head),
    random slot permutation, pair bytes per (sequence, block), last block of
    every sequence PROTECTED) but K and V are drawn on the device with a seeded
    torch generator, so pools of tens of GB never pass through the host.
    """

    def __init__(self, shape: Shape, seed: int, pair_weights: Optional[np.ndarray] = None,
                 spare_slots: int = 0, device: str = "cuda", pool_units: Optional[int] = None):
        import torch
        self.torch = torch
        self.shape = shape
        rng = np.random.default_rng(seed)
        L, H, dim = shape.n_layers, shape.n_kv_heads, shape.dim
        lens = np.asarray(shape.seq_lens, np.int64)
        rows_per_seq = L * H
        row_ntok = np.repeat(lens, rows_per_seq).astype(np.int32)
        self.row_seq = np.repeat(np.arange(len(lens)), rows_per_seq).astype(np.int32)
        nb = (row_ntok.astype(np.int64) + BLOCK - 1) // BLOCK
        row_off = np.zeros(len(nb), np.int64)
        row_off[1:] = np.cumsum(nb[:-1])
        self.n_rows = len(nb)
        self.n_uids = int(nb.sum())
        self.n_slots = self.n_uids + spare_slots
        if pool_units is not None:          # frame count decided by the caller (from the sizing call)
            assert pool_units >= self.n_uids, (pool_units, self.n_uids)
            self.n_slots = int(pool_units)
        self.nb = nb
        g = shape.g
        if pair_weights is None:
            pair_weights = np.full(16, 1.0 / 16)
        pair = np.empty(self.n_uids, np.uint8)
        state = np.full(self.n_uids, 1, np.uint8)
        for s, n in enumerate(lens):
            k = int((n + BLOCK - 1) // BLOCK)
            sp = rng.choice(16, size=k, p=pair_weights).astype(np.uint8)
            r0 = s * rows_per_seq
            o = int(row_off[r0])
            pair[o:o + k * rows_per_seq] = np.tile(sp, rows_per_seq)
            state[o + k - 1:o + k * rows_per_seq:k] |= 4
        self.host = dict(row_ntok=row_ntok, row_off=row_off, pair=pair, state=state)
        gen = torch.Generator(device=device)
        gen.manual_seed(seed)
        self.gen = gen
        unit_elems = BLOCK * dim
        tdt = torch.bfloat16 if shape.dtype == BF16 else torch.float16
        self.tdtype = tdt

        def filled(n):
            t = torch.empty((n, unit_elems), dtype=tdt, device=device)
            step = max(1, (1 << 27) // unit_elems)
            for i in range(0, n, step):
                j = min(n, i + step)
                t[i:j] = torch.randn((j - i, unit_elems), generator=gen, device=device, dtype=torch.float32).to(tdt)
            return t

        self.k_pool = filled(self.n_slots)
        self.v_pool = filled(self.n_slots) if shape.has_v else None
        perm = torch.randperm(self.n_slots, generator=gen, device=device)[: self.n_uids].to(torch.int32)
        self.slot_tbl = perm.contiguous()
        self.row_ntok = torch.from_numpy(row_ntok).to(device)
        self.row_off = torch.from_numpy(row_off).to(device)
        self.row_q_off = (torch.arange(self.n_rows, dtype=torch.int64, device=device) * (g * dim))
        self.state = torch.from_numpy(state).to(device)
        self.pair = torch.from_numpy(pair).to(device)
        self.q_elems = self.n_rows * g * dim

    def queries(self, seed: int):
        torch = self.torch
        gen = torch.Generator(device=self.k_pool.device)
        gen.manual_seed(seed)
        return torch.randn(self.q_elems, generator=gen, device=self.k_pool.device,
                           dtype=torch.float32).to(self.tdtype)

    def host_sample(self, seq_ids=None, rows=None) -> "Case":
        """Host copy of some rows (all rows of the given sequences, or the given row indices) with
        their units compacted into a small pool (slot ids renumbered), for the CPU oracle."""
        torch = self.torch
        if rows is None:
            rows = np.nonzero(np.isin(self.row_seq, np.asarray(seq_ids)))[0]
        rows = np.asarray(rows, np.int64)
        seq_ids = sorted(set(int(s) for s in self.row_seq[rows]))
        nb = self.nb[rows]
        new_off = np.zeros(len(rows), np.int64)
        new_off[1:] = np.cumsum(nb[:-1])
        n_u = int(nb.sum())
        old_uids = np.concatenate([np.arange(self.host["row_off"][r], self.host["row_off"][r] + k)
                                   for r, k in zip(rows, nb)])
        uids_dev = torch.from_numpy(old_uids).to(self.k_pool.device)
        slots = self.slot_tbl[uids_dev]
        res = slots >= 0
        res_slots = slots[res].long()
        k_host = self.k_pool[res_slots].view(torch.int16).cpu().numpy().view(np.uint16)
        new_tbl = np.full(n_u, -1, np.int32)
        new_tbl[res.cpu().numpy()] = np.arange(int(res.sum().item()), dtype=np.int32)
        state = self.state[uids_dev].cpu().numpy()
        pair = self.pair[uids_dev].cpu().numpy()
        g, dim = self.shape.g, self.shape.dim
        sample_shape = Shape(self.shape.n_layers, self.shape.n_q_heads, self.shape.n_kv_heads, dim,
                             self.shape.dtype, self.shape.has_v, [self.shape.seq_lens[s] for s in seq_ids])
        case = Case(sample_shape, k_host.shape[0], k_host, None, self.host["row_ntok"][rows].copy(), new_off,
                    np.arange(len(rows), dtype=np.int64) * g * dim, self.row_seq[rows].copy(), new_tbl, state,
                    pair, n_u)
        case.sample_rows = rows
        case.sample_uids = old_uids
        return case


def llama8b_shape(n_seq: int = 64, seed: int = 2) -> Shape:
    """32 layers, 32 q / 8 KV heads, d 128, bf16, n_seq sequences of uniform [2048, 8192] tokens."""
    return Shape(32, 32, 8, 128, BF16, True, uniform_lengths(n_seq, 2048, 8192, seed))


def llama70b_shape(n_seq: int = 4, n_tok: int = 131072) -> Shape:
    """One GPU's share of the Llama-3-70B-shaped workload: 80 layers, 64 q / 8 KV heads, d 128, bf16."""
    return Shape(80, 64, 8, 128, BF16, True, [n_tok] * n_seq)


def mla_shape(n_seq: int = 32, n_tok: int = 32768) -> Shape:
    """DeepSeek-V3-shaped MLA: 61 layers, one 576-channel latent head scored by 128 queries, no V."""
    return Shape(61, 128, 1, 576, BF16, False, [n_tok] * n_seq)


def lognormal_lengths(n_seq: int, seed: int, mu: float = 7.0, sigma: float = 1.0, lo: int = 16, hi: int = 32768):
    """Prompt lengths of the fleet workload: lognormal(mu, sigma) tokens clipped to [lo, hi]."""
    rng = np.random.default_rng(seed)
    return [int(x) for x in np.clip(np.exp(rng.normal(mu, sigma, n_seq)), lo, hi)]


def mha_fleet_shape(n_seq: int = 48, seed: int = 5) -> Shape:
    """MHA half of the fleet workload: 32 layers, 32 q = 32 KV heads (g = 1), d 128, bf16, lognormal lengths."""
    return Shape(32, 32, 32, 128, BF16, True, lognormal_lengths(n_seq, seed))


def mqa_fleet_shape(n_seq: int = 1536, seed: int = 6) -> Shape:
    """MQA half of the fleet workload: 32 layers, 32 q / 1 KV head (g = 32), d 128, bf16, lognormal lengths."""
    return Shape(32, 32, 1, 128, BF16, True, lognormal_lengths(n_seq, seed))


# ------------------------------------------------------------ fleet request trace
@dataclass
class FleetRequest:
    """One request of the heterogeneous-fleet trace (all times in decode steps)."""
    arrival: int
    model: int               # 0 = the MHA model, 1 = the MQA model
    prefix: int              # id in that model's shared-prefix catalogue (0 = most popular)
    prompt_len: int          # tokens, lognormal clipped
    prefix_len: int          # leading tokens shared with every request of the same prefix id (whole blocks)
    decode: List[int]        # decode steps of each turn of the session
    gap: List[int]           # idle steps after each turn but the last


@dataclass
class FleetPrefix:
    frac: float              # share of a prompt that the prefix makes up
    block_type: int          # 0 system_prompt or 1 tool_context
    transition: int          # transition type of the requests that use it, 0..3


def fleet_catalogue(n_prefixes: int, seed: int) -> List[FleetPrefix]:
    rng = np.random.default_rng(seed)
    w = categorical_weights(seed + 1, 4)
    return [FleetPrefix(float(rng.uniform(0.2, 0.9)), int(rng.integers(0, 2)), int(rng.choice(4, p=w)))
            for _ in range(n_prefixes)]


def fleet_requests(n_requests: int, seed: int, rate: float, n_prefixes: int, catalogues, zipf_a: float = 1.1,
                   mean_turns: float = 3.0, mean_decode: float = 80.0, mean_gap: float = 150.0, mu: float = 7.0,
                   sigma: float = 1.0, lo: int = 16, hi: int = 32768) -> List[FleetRequest]:
    """A seeded request trace: Poisson arrivals (`rate` per decode step), model ~ Bernoulli(0.5), prefix id
    ~ Zipf(zipf_a) over a catalogue of n_prefixes per model, prompt length ~ lognormal(mu, sigma) clipped to
    [lo, hi], sessions of 1 + Poisson(mean_turns - 1) turns of 1 + Geometric(mean_decode) decode steps with
    exponential idle gaps (mean mean_gap steps) between turns."""
    rng = np.random.default_rng(seed)
    ranks = np.arange(1, n_prefixes + 1, dtype=np.float64)
    zipf = ranks ** (-zipf_a)
    zipf /= zipf.sum()
    t = 0.0
    out = []
    for _ in range(n_requests):
        t += rng.exponential(1.0 / rate)
        model = int(rng.random() < 0.5)
        prefix = int(rng.choice(n_prefixes, p=zipf))
        prompt = int(np.clip(np.exp(rng.normal(mu, sigma)), lo, hi))
        plen = int(catalogues[model][prefix].frac * prompt) // BLOCK * BLOCK
        turns = 1 + int(rng.poisson(max(mean_turns - 1.0, 0.0)))
        decode = [1 + int(rng.geometric(1.0 / mean_decode)) for _ in range(turns)]
        gap = [1 + int(rng.exponential(mean_gap)) for _ in range(turns - 1)]
        out.append(FleetRequest(int(t), model, prefix, prompt, plen, decode, gap))
    return out


def growing_batch_requests(seq_lens: List[int]) -> List[FleetRequest]:
    """A batch that only decodes: every sequence is there from step 0 with its prompt and appends one token
    per step for ever (no prefix, one endless turn).  Replayed by the fleet's plan builder this gives the
    Llama-3-8B-shaped configuration's growth: a new block, hence new units, whenever a sequence crosses a block
    boundary, the block being written PROTECTED."""
    return [FleetRequest(0, 0, 0, int(n), 0, [1 << 30], []) for n in seq_lens]
