"""ctypes binding of libkvm (see ``include/kvm.h`` for the contract of every call).

Argument marshalling only: each function here takes torch tensors (for device
and pinned memory) or plain integers, checks dtype / device / contiguity, and
passes raw pointers to the C entry point of the same name.  There is no
fallback: if the shared library has not been built, importing this module
raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

from ._build import LIB_PATH, build  # noqa: F401  (re-exported)

OK, EINVAL, ESHAPE, ENOSPC, EHIP = 0, -1, -2, -3, -4
BF16, FP16 = 0, 1
ARCH_MHA, ARCH_GQA, ARCH_MQA, ARCH_MLA = 0, 1, 2, 3
ST_RESIDENT, ST_ON_HOST, ST_PROTECTED, ST_SCORED, ST_SHARED = 1, 2, 4, 8, 16
AGG_MAX, AGG_MEAN = 0, 1
OP_SCORE, OP_SELECT, OP_SPAN = 0, 1, 2
SELECT_STATIC_MAX_UIDS = 1 << 26
XFER_OUT_ONLY = 1 << 62

EXPORTS = ["kvm_size", "kvm_score_step", "kvm_score_step_xfer", "kvm_exchange_begin", "kvm_exchange_end", "kvm_pack_begin", "kvm_beta_update", "kvm_beta_blend_update", "kvm_ema_update",
           "kvm_ema_update_ex", "kvm_select_victims", "kvm_select_victims_static", "kvm_pack", "kvm_unpack", "kvm_swap", "kvm_exchange", "kvm_span_update",
           "kvm_prefetch_keys", "kvm_hash_units", "kvm_dedup_insert", "kvm_dedup_release", "kvm_dedup_share", "kvm_dedup_unshare", "kvm_workspace_bytes", "kvm_last_error", "kvm_version", "kvm_probe_read",
           "kvm_timing_enable", "kvm_timing_only", "kvm_timing_reset", "kvm_timing_read"]


class KvmError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"kvm error {code}: {msg}")
        self.code = code


class Model(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "n_layers", "n_q_heads", "n_kv_heads", "head_dim", "d_latent", "d_rope",
        "bits_per_elem", "block_tokens", "head_divisor")]


class Sizing(C.Structure):
    _fields_ = [("arch", C.c_int32), ("group_size", C.c_int32),
                ("bytes_per_token_layer", C.c_uint64), ("bytes_per_token", C.c_uint64),
                ("bytes_per_seq", C.c_uint64), ("max_batch", C.c_uint64),
                ("units_per_block", C.c_uint32), ("unit_k_bytes", C.c_uint32),
                ("unit_v_bytes", C.c_uint32), ("head_weight", C.c_uint32), ("pool_units", C.c_uint64)]


class Pool(C.Structure):
    _fields_ = [("k_pool", C.c_void_p), ("v_pool", C.c_void_p), ("n_slots", C.c_uint64),
                ("dim", C.c_int32), ("dtype", C.c_int32),
                ("unit_k_bytes", C.c_uint32), ("unit_v_bytes", C.c_uint32)]


class Rows(C.Structure):
    _fields_ = [("n_rows", C.c_int32), ("g", C.c_int32), ("n_uids", C.c_int64), ("q_elems", C.c_int64),
                ("row_ntok", C.c_void_p), ("row_off", C.c_void_p), ("row_q_off", C.c_void_p),
                ("row_active", C.c_void_p), ("slot_tbl", C.c_void_p)]


class EmaEx(C.Structure):
    _fields_ = [("pos_decay", C.c_float), ("n_seq", C.c_int32), ("n_heads", C.c_int32),
                ("row_seq", C.c_void_p), ("row_head", C.c_void_p), ("seq_transition", C.c_void_p),
                ("head_mult", C.c_void_p)]


class Store(C.Structure):
    _fields_ = [("tag", C.c_void_p), ("digest", C.c_void_p), ("canon", C.c_void_p), ("refs", C.c_void_p),
                ("pending", C.c_void_p), ("cap", C.c_uint64)]


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run __graft_entry__.build() (hipcc) first")
    lib = C.CDLL(LIB_PATH)
    lib.kvm_last_error.restype = C.c_char_p
    lib.kvm_version.restype = C.c_char_p
    lib.kvm_workspace_bytes.restype = C.c_size_t
    lib.kvm_workspace_bytes.argtypes = [C.c_int, C.c_int64, C.c_int32, C.c_int32, C.c_int32]
    lib.kvm_size.argtypes = [C.POINTER(Model), C.c_uint64, C.c_uint64, C.POINTER(Sizing)]
    lib.kvm_score_step.argtypes = [C.POINTER(Pool), C.POINTER(Rows), C.c_void_p, C.c_float, C.c_int,
                                   C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.kvm_beta_update.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p,
                                    C.c_float, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.kvm_ema_update.argtypes = [C.POINTER(Rows), C.c_void_p, C.c_float, C.c_void_p, C.c_void_p,
                                   C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.kvm_select_victims.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64,
                                       C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.kvm_select_victims_static.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64,
                                              C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
    lib.kvm_pack.argtypes = [C.POINTER(Pool), C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p,
                             C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t,
                             C.c_void_p, C.c_void_p]
    lib.kvm_unpack.argtypes = [C.POINTER(Pool), C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p,
                               C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t,
                               C.c_void_p, C.c_void_p]
    lib.kvm_swap.argtypes = [C.POINTER(Pool), C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_int64,
                             C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t,
                             C.c_void_p, C.c_void_p]
    lib.kvm_beta_blend_update.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_float,
                                          C.c_float, C.c_void_p, C.c_void_p, C.c_int32, C.c_float, C.c_void_p,
                                          C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.kvm_ema_update_ex.argtypes = [C.POINTER(Rows), C.c_void_p, C.c_float, C.POINTER(EmaEx), C.c_void_p,
                                      C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.kvm_span_update.argtypes = [C.POINTER(Rows), C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_uint32,
                                    C.c_uint32, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                    C.c_size_t, C.c_void_p]
    lib.kvm_prefetch_keys.argtypes = [C.POINTER(Rows), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p,
                                      C.c_void_p, C.c_void_p, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.kvm_exchange.argtypes = [C.POINTER(Pool), C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_int64,
                                 C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p]
    lib.kvm_hash_units.argtypes = [C.POINTER(Pool), C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64,
                                   C.c_void_p, C.c_void_p, C.c_void_p]
    lib.kvm_dedup_insert.argtypes = [C.POINTER(Store), C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p,
                                     C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.kvm_dedup_release.argtypes = [C.POINTER(Store), C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
    lib.kvm_score_step_xfer.argtypes = [C.POINTER(Pool), C.POINTER(Rows), C.c_void_p, C.c_float, C.c_int, C.c_void_p,
                                        C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p,
                                        C.c_uint64, C.c_void_p]
    lib.kvm_exchange_begin.argtypes = [C.POINTER(Pool), C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p,
                                       C.c_int64, C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p,
                                       C.c_void_p, C.c_void_p]
    lib.kvm_dedup_share.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_uint64, C.c_void_p, C.c_void_p, C.c_int64,
                                    C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.kvm_dedup_unshare.argtypes = [C.POINTER(Pool), C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p,
                                      C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.kvm_pack_begin.argtypes = [C.POINTER(Pool), C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p,
                                   C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.kvm_exchange_end.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
    lib.kvm_probe_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
    lib.kvm_timing_read.argtypes = [C.c_char_p, C.POINTER(C.c_double)]
    lib.kvm_timing_only.argtypes = [C.c_char_p]
    return lib


lib = _load()


def _check(rc: int):
    if rc != 0:
        raise KvmError(rc, lib.kvm_last_error().decode())


def _ptr(t: Optional[torch.Tensor], dtype=None, device_type: Optional[str] = "cuda") -> Optional[int]:
    if t is None:
        return None
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {t.dtype}")
    if device_type is not None and t.device.type != device_type:
        raise TypeError(f"expected a {device_type} tensor, got {t.device}")
    if not t.is_contiguous():
        raise TypeError("tensor must be contiguous")
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else None
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


# ---------------------------------------------------------------- descriptors
def make_pool(k_pool: torch.Tensor, v_pool: Optional[torch.Tensor], dim: int, dtype: int) -> Pool:
    """k_pool / v_pool: device tensors [n_slots, unit elements] of any 2-byte dtype."""
    n_slots = k_pool.shape[0]
    unit_k = k_pool[0].numel() * k_pool.element_size() if n_slots else 16 * dim * 2
    unit_v = 0 if v_pool is None else (v_pool[0].numel() * v_pool.element_size() if n_slots else 0)
    p = Pool(_ptr(k_pool), _ptr(v_pool), n_slots, dim, dtype, unit_k, unit_v)
    p._keep = (k_pool, v_pool)
    return p


def make_rows(row_ntok, row_off, row_q_off, slot_tbl, g: int, q_elems: int, row_active=None) -> Rows:
    r = Rows(row_ntok.numel(), g, slot_tbl.numel(), q_elems,
             _ptr(row_ntok, torch.int32), _ptr(row_off, torch.int64), _ptr(row_q_off, torch.int64),
             _ptr(row_active, torch.uint8), _ptr(slot_tbl, torch.int32))
    r._keep = (row_ntok, row_off, row_q_off, slot_tbl, row_active)
    return r


# --------------------------------------------------------------- entry points
def kvm_size(n_layers, n_q_heads, n_kv_heads, head_dim, d_latent=0, d_rope=0, bits_per_elem=16,
             block_tokens=16, head_divisor=1, n_max=0, mem_target=0) -> dict:
    m = Model(n_layers, n_q_heads, n_kv_heads, head_dim, d_latent, d_rope, bits_per_elem, block_tokens,
              head_divisor)
    s = Sizing()
    _check(lib.kvm_size(C.byref(m), n_max, mem_target, C.byref(s)))
    return {n: getattr(s, n) for n, _ in Sizing._fields_}


def kvm_workspace_bytes(op: int, n_uids: int, n_rows: int = 0, g: int = 1, dim: int = 0) -> int:
    return int(lib.kvm_workspace_bytes(op, n_uids, n_rows, g, dim))


def kvm_score_step(pool: Pool, rows: Rows, q: torch.Tensor, softmax_scale: float, mass: torch.Tensor,
                   ws: torch.Tensor, agg: int = AGG_MAX, stream=None):
    _check(lib.kvm_score_step(C.byref(pool), C.byref(rows), _ptr(q), softmax_scale, agg,
                              _ptr(mass, torch.float32), _ptr(ws), ws.numel() * ws.element_size(),
                              _stream(stream)))


def kvm_beta_update(ev_pair, ev_outcome, hits, misses, p_hat, alpha0: float = 1.0, beta0: float = 1.0,
                    n_bad=None, stream=None):
    n = 0 if ev_pair is None else ev_pair.numel()
    _check(lib.kvm_beta_update(_ptr(ev_pair, torch.uint8), _ptr(ev_outcome, torch.uint8), n,
                               _ptr(hits, torch.int32), _ptr(misses, torch.int32), alpha0, beta0,
                               _ptr(p_hat, torch.float32), _ptr(n_bad, torch.int32), _stream(stream)))


def kvm_beta_blend_update(ev_pair, ev_outcome, hits, misses, win, win_head, kappa: float, p_hat, conf, p_blend,
                          alpha0: float = 1.0, beta0: float = 1.0, n_bad=None, stream=None):
    """win: uint8 device tensor [16, window], filled with 255 before first use; win_head: int32 [16]."""
    n = 0 if ev_pair is None else ev_pair.numel()
    _check(lib.kvm_beta_blend_update(_ptr(ev_pair, torch.uint8), _ptr(ev_outcome, torch.uint8), n,
                                     _ptr(hits, torch.int32), _ptr(misses, torch.int32), alpha0, beta0,
                                     _ptr(win, torch.uint8), _ptr(win_head, torch.int32), win.shape[1], kappa,
                                     _ptr(p_hat, torch.float32), _ptr(conf, torch.float32),
                                     _ptr(p_blend, torch.float32), _ptr(n_bad, torch.int32), _stream(stream)))


def make_ema_ex(pos_decay: float = 1.0, row_seq=None, row_head=None, seq_transition=None, head_mult=None) -> EmaEx:
    """head_mult: float32 device tensor [4, n_heads] or None."""
    e = EmaEx(pos_decay, 0 if seq_transition is None else seq_transition.numel(),
              0 if head_mult is None else head_mult.shape[1],
              _ptr(row_seq, torch.int32), _ptr(row_head, torch.int32), _ptr(seq_transition, torch.uint8),
              _ptr(head_mult, torch.float32))
    e._keep = (row_seq, row_head, seq_transition, head_mult)
    return e


def kvm_ema_update_ex(rows: Rows, mass, ema_decay: float, ex: EmaEx, row_weight, pair, p_hat, state, S, prio,
                      stream=None):
    _check(lib.kvm_ema_update_ex(C.byref(rows), _ptr(mass, torch.float32), ema_decay, C.byref(ex),
                                 _ptr(row_weight, torch.float32), _ptr(pair, torch.uint8),
                                 _ptr(p_hat, torch.float32), _ptr(state, torch.uint8),
                                 _ptr(S, torch.float32), _ptr(prio, torch.float32), _stream(stream)))


def kvm_span_update(rows: Rows, row_layer, mass, state, theta_num: int, theta_den: int, span_sum, span_cnt,
                    w_min: int, w_max: int, layer_window, ws, stream=None):
    """span_sum: int64 [n_layers] (read as unsigned), span_cnt / layer_window: int32 [n_layers];
    ws: uint8 scratch of kvm_workspace_bytes(OP_SPAN, 0, n_rows) bytes (None when there are no rows)."""
    _check(lib.kvm_span_update(C.byref(rows), _ptr(row_layer, torch.int32), layer_window.numel(),
                               _ptr(mass, torch.float32), _ptr(state, torch.uint8), theta_num, theta_den,
                               _ptr(span_sum, torch.int64), _ptr(span_cnt, torch.int32), w_min, w_max,
                               _ptr(layer_window, torch.int32), _ptr(ws, torch.uint8) if ws is not None else None,
                               ws.numel() if ws is not None else 0, _stream(stream)))


def kvm_prefetch_keys(rows: Rows, row_layer, row_pos, layer_window, state, pair, p_est, pos_decay: float, key, cand,
                      stream=None):
    _check(lib.kvm_prefetch_keys(C.byref(rows), _ptr(row_layer, torch.int32), _ptr(row_pos, torch.int32),
                                 _ptr(layer_window, torch.int32), layer_window.numel(), _ptr(state, torch.uint8),
                                 _ptr(pair, torch.uint8), _ptr(p_est, torch.float32), pos_decay,
                                 _ptr(key, torch.float32), _ptr(cand, torch.uint8), _stream(stream)))


def kvm_ema_update(rows: Rows, mass, ema_decay: float, row_weight, pair, p_hat, state, S, prio, stream=None):
    _check(lib.kvm_ema_update(C.byref(rows), _ptr(mass, torch.float32), ema_decay,
                              _ptr(row_weight, torch.float32), _ptr(pair, torch.uint8),
                              _ptr(p_hat, torch.float32), _ptr(state, torch.uint8),
                              _ptr(S, torch.float32), _ptr(prio, torch.float32), _stream(stream)))


def kvm_select_victims(prio, state, victims, n_victims, ws, k: int = -1, budget_units: int = 0, stream=None):
    _check(lib.kvm_select_victims(_ptr(prio, torch.float32), _ptr(state, torch.uint8), state.numel(), k,
                                  budget_units, _ptr(victims, torch.int64), victims.numel(),
                                  _ptr(n_victims, torch.int64), _ptr(ws), ws.numel() * ws.element_size(),
                                  _stream(stream)))


def kvm_select_victims_static(prio, state, victims, n_victims, k: int = -1, budget_units: int = 0, stream=None):
    _check(lib.kvm_select_victims_static(_ptr(prio, torch.float32), _ptr(state, torch.uint8), state.numel(), k,
                                         budget_units, _ptr(victims, torch.int64), victims.numel(),
                                         _ptr(n_victims, torch.int64), _stream(stream)))


def _nbytes(t: Optional[torch.Tensor]) -> int:
    return 0 if t is None else t.numel() * t.element_size()


def kvm_pack(pool: Pool, slot_tbl, state, uids, n: int, host_slots, freed_slots, staging_dev,
             staging_host, n_bad=None, n_dev=None, stream=None):
    _check(lib.kvm_pack(C.byref(pool), _ptr(slot_tbl, torch.int32), _ptr(state, torch.uint8), state.numel(),
                        _ptr(uids, torch.int64), n, _ptr(n_dev, torch.int64), _ptr(host_slots, torch.int32),
                        _ptr(freed_slots, torch.int32), _ptr(staging_dev), _nbytes(staging_dev),
                        _ptr(staging_host, None, "cpu"), _nbytes(staging_host),
                        _ptr(n_bad, torch.int32), _stream(stream)))


def kvm_unpack(pool: Pool, slot_tbl, state, uids, n: int, dst_slots, staging_dev, staging_host,
               n_bad=None, n_dev=None, stream=None):
    _check(lib.kvm_unpack(C.byref(pool), _ptr(slot_tbl, torch.int32), _ptr(state, torch.uint8), state.numel(),
                          _ptr(uids, torch.int64), n, _ptr(n_dev, torch.int64), _ptr(dst_slots, torch.int32),
                          _ptr(staging_dev), _nbytes(staging_dev),
                          _ptr(staging_host, None, "cpu"), _nbytes(staging_host),
                          _ptr(n_bad, torch.int32), _stream(stream)))


def kvm_swap(pool: Pool, slot_tbl, state, out_uids, in_uids, n: int, host_slots, freed_slots, host_out, host_in,
             n_bad=None, n_dev=None, stream=None):
    _check(lib.kvm_swap(C.byref(pool), _ptr(slot_tbl, torch.int32), _ptr(state, torch.uint8), state.numel(),
                        _ptr(out_uids, torch.int64), _ptr(in_uids, torch.int64), n, _ptr(n_dev, torch.int64),
                        _ptr(host_slots, torch.int32), _ptr(freed_slots, torch.int32),
                        _ptr(host_out, None, "cpu"), _nbytes(host_out), _ptr(host_in, None, "cpu"), _nbytes(host_in),
                        _ptr(n_bad, torch.int32), _stream(stream)))


def kvm_exchange(pool: Pool, slot_tbl, state, out_uids, in_uids, n: int, host_tier, n_out_dev=None, n_in_dev=None,
                 n_bad=None, stream=None):
    """host_tier: pinned uint8 tensor holding whole records, record of host slot h at h * record bytes."""
    rec = pool.unit_k_bytes + pool.unit_v_bytes
    _check(lib.kvm_exchange(C.byref(pool), _ptr(slot_tbl, torch.int32), _ptr(state, torch.uint8), state.numel(),
                            _ptr(out_uids, torch.int64), _ptr(in_uids, torch.int64), n, _ptr(n_out_dev, torch.int64),
                            _ptr(n_in_dev, torch.int64), _ptr(host_tier, None, "cpu"), _nbytes(host_tier) // rec,
                            _ptr(n_bad, torch.int32), _stream(stream)))


def kvm_hash_units(pool: Pool, slot_tbl, state, uids, n: int, digests, n_bad=None, stream=None):
    """digests: uint8 device tensor [n, 32]."""
    _check(lib.kvm_hash_units(C.byref(pool), _ptr(slot_tbl, torch.int32), _ptr(state, torch.uint8), state.numel(),
                              _ptr(uids, torch.int64), n, _ptr(digests, torch.uint8), _ptr(n_bad, torch.int32),
                              _stream(stream)))


def make_store(cap: int, device="cuda") -> Store:
    """An empty content store with `cap` places (a power of two)."""
    t = dict(tag=torch.zeros(cap, dtype=torch.int64, device=device),
             digest=torch.zeros((cap, 32), dtype=torch.uint8, device=device),
             canon=torch.full((cap,), -1, dtype=torch.int64, device=device),
             refs=torch.zeros(cap, dtype=torch.int32, device=device),
             pending=torch.full((cap,), -1, dtype=torch.int32, device=device))
    s = Store(t["tag"].data_ptr(), t["digest"].data_ptr(), t["canon"].data_ptr(), t["refs"].data_ptr(),
              t["pending"].data_ptr(), cap)
    s.tensors = t
    return s


def kvm_dedup_insert(store: Store, digests, uids, n: int, canon_out, ws, n_full=None, n_collide=None, stream=None):
    _check(lib.kvm_dedup_insert(C.byref(store), _ptr(digests, torch.uint8), _ptr(uids, torch.int64), n,
                                _ptr(canon_out, torch.int64), _ptr(n_full, torch.int32), _ptr(n_collide, torch.int32),
                                _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)))


def kvm_dedup_release(store: Store, digests, n: int, n_bad=None, stream=None):
    _check(lib.kvm_dedup_release(C.byref(store), _ptr(digests, torch.uint8), n, _ptr(n_bad, torch.int32),
                                 _stream(stream)))


def kvm_score_step_xfer(pool: Pool, rows: Rows, q, softmax_scale: float, mass, ws, xfer_frame, xfer_host, n_pairs: int,
                        host_tier, agg: int = AGG_MAX, stream=None):
    """host_tier: pinned uint8 tensor of whole records; its record count is passed on as tier_slots."""
    rec = pool.unit_k_bytes + pool.unit_v_bytes
    tier_slots = 0 if host_tier is None else host_tier.numel() * host_tier.element_size() // rec
    _check(lib.kvm_score_step_xfer(C.byref(pool), C.byref(rows), _ptr(q), softmax_scale, agg,
                                   _ptr(mass, torch.float32), _ptr(ws), ws.numel() * ws.element_size(),
                                   _ptr(xfer_frame, torch.int32), _ptr(xfer_host, torch.int64), n_pairs,
                                   _ptr(host_tier, None, "cpu"), tier_slots, _stream(stream)))


def kvm_exchange_begin(pool: Pool, slot_tbl, state, out_uids, in_uids, n: int, tier_slots: int, frame, host,
                       n_out_dev=None, n_in_dev=None, n_bad=None, stream=None):
    _check(lib.kvm_exchange_begin(C.byref(pool), _ptr(slot_tbl, torch.int32), _ptr(state, torch.uint8), state.numel(),
                                  _ptr(out_uids, torch.int64), _ptr(in_uids, torch.int64), n,
                                  _ptr(n_out_dev, torch.int64), _ptr(n_in_dev, torch.int64), tier_slots,
                                  _ptr(frame, torch.int32), _ptr(host, torch.int64), _ptr(n_bad, torch.int32),
                                  _stream(stream)))


def kvm_pack_begin(pool: Pool, slot_tbl, state, uids, n: int, host_slots, tier_slots: int, frame, host, n_dev=None,
                   n_bad=None, stream=None):
    _check(lib.kvm_pack_begin(C.byref(pool), _ptr(slot_tbl, torch.int32), _ptr(state, torch.uint8), state.numel(),
                              _ptr(uids, torch.int64), n, _ptr(n_dev, torch.int64), _ptr(host_slots, torch.int32),
                              tier_slots, _ptr(frame, torch.int32), _ptr(host, torch.int64), _ptr(n_bad, torch.int32),
                              _stream(stream)))


def kvm_exchange_end(slot_tbl, state, in_uids, frame, n: int, stream=None):
    _check(lib.kvm_exchange_end(_ptr(slot_tbl, torch.int32), _ptr(state, torch.uint8), state.numel(),
                                _ptr(in_uids, torch.int64), _ptr(frame, torch.int32), n, _stream(stream)))


def kvm_dedup_share(slot_tbl, state, n_slots: int, uids, canon, n: int, frame_refs, freed, n_bad=None, stream=None):
    _check(lib.kvm_dedup_share(_ptr(slot_tbl, torch.int32), _ptr(state, torch.uint8), state.numel(), n_slots,
                               _ptr(uids, torch.int64), _ptr(canon, torch.int64), n, _ptr(frame_refs, torch.int32),
                               _ptr(freed, torch.int32), _ptr(n_bad, torch.int32), _stream(stream)))


def kvm_dedup_unshare(pool: Pool, slot_tbl, state, uids, new_frames, n: int, frame_refs, freed, n_bad=None,
                      stream=None):
    _check(lib.kvm_dedup_unshare(C.byref(pool), _ptr(slot_tbl, torch.int32), _ptr(state, torch.uint8), state.numel(),
                                 _ptr(uids, torch.int64), _ptr(new_frames, torch.int32), n,
                                 _ptr(frame_refs, torch.int32), _ptr(freed, torch.int32), _ptr(n_bad, torch.int32),
                                 _stream(stream)))


def kvm_probe_read(buf, sink, stream=None):
    _check(lib.kvm_probe_read(_ptr(buf), buf.numel() * buf.element_size(), _ptr(sink, torch.int32), _stream(stream)))


def kvm_last_error() -> str:
    return lib.kvm_last_error().decode()


def kvm_version() -> str:
    return lib.kvm_version().decode()


def kvm_timing_enable(on: bool):
    lib.kvm_timing_enable(1 if on else 0)


def kvm_timing_only(name):
    lib.kvm_timing_only(name.encode() if name is not None else None)


def kvm_timing_reset():
    lib.kvm_timing_reset()


def kvm_timing_read(name: str):
    """(launch count, total milliseconds) of the named kernel since the last reset."""
    ms = C.c_double(0.0)
    n = lib.kvm_timing_read(name.encode(), C.byref(ms))
    return int(n), float(ms.value)
