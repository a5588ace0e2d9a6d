"""CPU oracle for the KV-cache management pass — TEST INFRASTRUCTURE ONLY.

A ctypes front end over ``kvm_oracle.c`` (plain C, fp64, written from the
paper's definitions).  Only tests, the smoke check and the benchmark's CPU
baseline leg may import this package; the product never does.  It imports
nothing from the GPU package.

All arguments are numpy arrays on the host; 16-bit floating point data (K
pool, queries) travels as ``uint16`` bit patterns.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kvm_oracle.c")
_LIB = os.path.join(_HERE, "libkvm_oracle.so")

BF16, FP16 = 0, 1
AGG_MAX, AGG_MEAN = 0, 1
ST_RESIDENT, ST_ON_HOST, ST_PROTECTED, ST_SCORED = 1, 2, 4, 8


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (``-O2 -fopenmp``); returns the library path.  With KVM_ORACLE_LIB
    set, that file (a sanitizer build, see :func:`build_sanitized`) is used as it is."""
    override = os.environ.get("KVM_ORACLE_LIB")
    if override:
        return override
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


def build_sanitized(out: str) -> str:
    """The oracle compiled with AddressSanitizer and UndefinedBehaviorSanitizer (gcc), for the CPU test
    that reruns the pins under them; returns ``out``.  A process loading it needs gcc's libasan preloaded."""
    subprocess.check_call(
        ["gcc", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
         "-shared", "-fPIC", "-Wall", "-Wextra", "-o", out, _SRC, "-lm"])
    return out


def asan_runtime() -> str:
    return subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()


class _Model(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "n_layers", "n_q_heads", "n_kv_heads", "head_dim", "d_latent", "d_rope",
        "bits_per_elem", "block_tokens", "head_divisor")]


class _Sizing(C.Structure):
    _fields_ = [("arch", C.c_int32), ("group_size", C.c_int32),
                ("bytes_per_token_layer", C.c_uint64), ("bytes_per_token", C.c_uint64),
                ("bytes_per_seq", C.c_uint64), ("max_batch", C.c_uint64),
                ("units_per_block", C.c_uint32), ("unit_k_bytes", C.c_uint32),
                ("unit_v_bytes", C.c_uint32), ("head_weight", C.c_uint32), ("pool_units", C.c_uint64)]


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
    return _lib


def _p(a, dtype):
    """Pointer to a C-contiguous numpy array of the given dtype (None -> NULL)."""
    if a is None:
        return None
    assert isinstance(a, np.ndarray) and a.dtype == dtype and a.flags["C_CONTIGUOUS"], (a.dtype, dtype)
    return a.ctypes.data_as(C.c_void_p)


class OracleError(RuntimeError):
    pass


def _check(rc, what):
    if rc != 0:
        raise OracleError(f"{what} returned {rc}")


def threads() -> int:
    return int(lib().kvm_ref_threads())


def set_threads(n: int) -> int:
    """Number of threads the row loops use from now on; returns what is in force."""
    return int(lib().kvm_ref_set_threads(int(n)))


def size(n_layers, n_q_heads, n_kv_heads, head_dim, d_latent=0, d_rope=0, bits_per_elem=16,
         block_tokens=16, head_divisor=1, n_max=0, mem_target=0) -> dict:
    m = _Model(n_layers, n_q_heads, n_kv_heads, head_dim, d_latent, d_rope, bits_per_elem,
               block_tokens, head_divisor)
    s = _Sizing()
    rc = lib().kvm_ref_size(C.byref(m), C.c_uint64(n_max), C.c_uint64(mem_target), C.byref(s))
    _check(rc, "kvm_ref_size")
    return {n: getattr(s, n) for n, _ in _Sizing._fields_}


def score_step(k_pool, dim, dtype, row_ntok, row_off, row_q_off, slot_tbl, q, g, scale, mass,
               agg=AGG_MAX, row_active=None, block_tokens=16, mass_q=None):
    """Writes ``mass`` (float32 [n_uids]) in place; optionally ``mass_q`` (float64 [n_uids * g])."""
    k_pool = k_pool.reshape(-1)
    unit_elems = block_tokens * dim
    n_slots = k_pool.size // unit_elems
    rc = lib().kvm_ref_score_step(
        _p(k_pool, np.uint16), C.c_uint64(n_slots), C.c_int(dim), C.c_int(dtype), C.c_int(block_tokens),
        C.c_int(len(row_ntok)), C.c_int(g), C.c_int64(len(slot_tbl)),
        _p(row_ntok, np.int32), _p(row_off, np.int64), _p(row_q_off, np.int64),
        _p(row_active, np.uint8), _p(slot_tbl, np.int32), _p(q.reshape(-1), np.uint16),
        C.c_double(scale), C.c_int(agg), _p(mass, np.float32), _p(mass_q, np.float64))
    _check(rc, "kvm_ref_score_step")
    return mass


def beta_update(ev_pair, ev_outcome, hits, misses, alpha0=1.0, beta0=1.0, p_hat=None, n_bad=None):
    if p_hat is None:
        p_hat = np.zeros(16, np.float32)
    rc = lib().kvm_ref_beta_update(
        _p(ev_pair, np.uint8), _p(ev_outcome, np.uint8), C.c_int64(len(ev_pair)),
        _p(hits, np.uint32), _p(misses, np.uint32), C.c_double(alpha0), C.c_double(beta0),
        _p(p_hat, np.float32), _p(n_bad, np.uint32))
    _check(rc, "kvm_ref_beta_update")
    return p_hat


def beta_blend_update(ev_pair, ev_outcome, hits, misses, win, win_head, kappa, alpha0=1.0, beta0=1.0, n_bad=None):
    """Returns (p_hat, conf, p_blend); win is uint8 [16, window] (255 = never written)."""
    window = win.shape[1]
    p_hat, conf, p_blend = (np.zeros(16, np.float32) for _ in range(3))
    rc = lib().kvm_ref_beta_blend_update(
        _p(ev_pair, np.uint8), _p(ev_outcome, np.uint8), C.c_int64(len(ev_pair)),
        _p(hits, np.uint32), _p(misses, np.uint32), C.c_double(alpha0), C.c_double(beta0),
        _p(win, np.uint8), _p(win_head, np.uint32), C.c_int(window), C.c_double(kappa),
        _p(p_hat, np.float32), _p(conf, np.float32), _p(p_blend, np.float32), _p(n_bad, np.uint32))
    _check(rc, "kvm_ref_beta_blend_update")
    return p_hat, conf, p_blend


def ema_update(row_ntok, row_off, mass, decay, row_weight, pair, p_hat, state, S, prio,
               row_active=None, block_tokens=16):
    rc = lib().kvm_ref_ema_update(
        C.c_int(len(row_ntok)), C.c_int(block_tokens), C.c_int64(len(state)),
        _p(row_ntok, np.int32), _p(row_off, np.int64), _p(row_active, np.uint8),
        _p(mass, np.float32), C.c_double(decay), _p(row_weight, np.float32), _p(pair, np.uint8),
        _p(p_hat, np.float32), _p(state, np.uint8), _p(S, np.float32), _p(prio, np.float32))
    _check(rc, "kvm_ref_ema_update")


def ema_update_ex(row_ntok, row_off, mass, decay, pos_decay, row_weight, pair, p_hat, state, S, prio,
                  row_seq=None, row_head=None, seq_transition=None, head_mult=None,
                  row_active=None, block_tokens=16):
    """head_mult: float32 [4, n_heads] or None."""
    n_seq = 0 if seq_transition is None else len(seq_transition)
    n_heads = 0 if head_mult is None else head_mult.shape[1]
    rc = lib().kvm_ref_ema_update_ex(
        C.c_int(len(row_ntok)), C.c_int(block_tokens), C.c_int64(len(state)),
        _p(row_ntok, np.int32), _p(row_off, np.int64), _p(row_active, np.uint8),
        _p(mass, np.float32), C.c_double(decay), C.c_double(pos_decay), _p(row_weight, np.float32),
        _p(row_seq, np.int32), _p(row_head, np.int32), _p(seq_transition, np.uint8), C.c_int(n_seq),
        _p(head_mult, np.float32), C.c_int(n_heads),
        _p(pair, np.uint8), _p(p_hat, np.float32), _p(state, np.uint8), _p(S, np.float32), _p(prio, np.float32))
    _check(rc, "kvm_ref_ema_update_ex")


def span_update(row_ntok, row_off, row_layer, mass, state, theta_num, theta_den, span_sum, span_cnt,
                w_min, w_max, layer_window, row_active=None, block_tokens=16):
    rc = lib().kvm_ref_span_update(
        C.c_int(len(row_ntok)), C.c_int(block_tokens), C.c_int64(len(state)),
        _p(row_ntok, np.int32), _p(row_off, np.int64), _p(row_active, np.uint8), _p(row_layer, np.int32),
        C.c_int(len(layer_window)), _p(mass, np.float32), _p(state, np.uint8),
        C.c_uint32(theta_num), C.c_uint32(theta_den), _p(span_sum, np.uint64), _p(span_cnt, np.uint32),
        C.c_int32(w_min), C.c_int32(w_max), _p(layer_window, np.int32))
    _check(rc, "kvm_ref_span_update")


def prefetch_keys(row_ntok, row_off, row_layer, row_pos, layer_window, state, pair, p_est, pos_decay,
                  key, cand, block_tokens=16):
    rc = lib().kvm_ref_prefetch_keys(
        C.c_int(len(row_ntok)), C.c_int(block_tokens), C.c_int64(len(state)),
        _p(row_ntok, np.int32), _p(row_off, np.int64), _p(row_layer, np.int32), _p(row_pos, np.int32),
        _p(layer_window, np.int32), C.c_int(len(layer_window)), _p(state, np.uint8), _p(pair, np.uint8),
        _p(p_est, np.float32), C.c_double(pos_decay), _p(key, np.float32), _p(cand, np.uint8))
    _check(rc, "kvm_ref_prefetch_keys")


def select_victims(prio, state, k=-1, budget_units=0, victims_cap=None):
    n = len(prio)
    cap = n if victims_cap is None else victims_cap
    victims = np.zeros(max(cap, 1), np.int64)
    nv = np.zeros(1, np.int64)
    rc = lib().kvm_ref_select_victims(
        _p(prio, np.float32), _p(state, np.uint8), C.c_int64(n), C.c_int64(k),
        C.c_int64(budget_units), _p(victims, np.int64), C.c_int64(cap), _p(nv, np.int64))
    _check(rc, "kvm_ref_select_victims")
    return victims[: int(nv[0])].copy()


def pack(k_pool, v_pool, unit_k_bytes, unit_v_bytes, slot_tbl, state, uids, host_slots, n_bad=None):
    """k_pool / v_pool: uint8 views of the pools.  Returns (staging uint8 [n, rec], freed_slots)."""
    n = len(uids)
    rec = unit_k_bytes + unit_v_bytes
    staging = np.zeros((max(n, 1), rec), np.uint8)
    freed = np.zeros(max(n, 1), np.int32)
    n_slots = k_pool.size // unit_k_bytes
    rc = lib().kvm_ref_pack(
        _p(k_pool.reshape(-1), np.uint8), _p(None if v_pool is None else v_pool.reshape(-1), np.uint8),
        C.c_uint64(n_slots), C.c_uint32(unit_k_bytes), C.c_uint32(unit_v_bytes),
        _p(slot_tbl, np.int32), _p(state, np.uint8), C.c_int64(len(state)),
        _p(uids, np.int64), C.c_int64(n), _p(host_slots, np.int32), _p(freed, np.int32),
        _p(staging.reshape(-1), np.uint8), _p(n_bad, np.uint32))
    _check(rc, "kvm_ref_pack")
    return staging[:n], freed[:n]


def unpack(k_pool, v_pool, unit_k_bytes, unit_v_bytes, slot_tbl, state, uids, dst_slots, staging,
           n_bad=None):
    n = len(uids)
    n_slots = k_pool.size // unit_k_bytes
    rc = lib().kvm_ref_unpack(
        _p(k_pool.reshape(-1), np.uint8), _p(None if v_pool is None else v_pool.reshape(-1), np.uint8),
        C.c_uint64(n_slots), C.c_uint32(unit_k_bytes), C.c_uint32(unit_v_bytes),
        _p(slot_tbl, np.int32), _p(state, np.uint8), C.c_int64(len(state)),
        _p(uids, np.int64), C.c_int64(n), _p(dst_slots, np.int32),
        _p(np.ascontiguousarray(staging).reshape(-1), np.uint8), _p(n_bad, np.uint32))
    _check(rc, "kvm_ref_unpack")


def exchange(k_pool, v_pool, unit_k_bytes, unit_v_bytes, slot_tbl, state, out_uids, in_uids, tier, n_bad=None):
    """tier: uint8 [tier_slots, rec], modified in place like the pools and tables."""
    n_slots = k_pool.size // unit_k_bytes
    rc = lib().kvm_ref_exchange(
        _p(k_pool.reshape(-1), np.uint8), _p(None if v_pool is None else v_pool.reshape(-1), np.uint8),
        C.c_uint64(n_slots), C.c_uint32(unit_k_bytes), C.c_uint32(unit_v_bytes),
        _p(slot_tbl, np.int32), _p(state, np.uint8), C.c_int64(len(state)),
        _p(out_uids, np.int64), _p(in_uids, np.int64), C.c_int64(len(out_uids)),
        _p(tier.reshape(-1), np.uint8), C.c_uint64(tier.shape[0]), _p(n_bad, np.uint32))
    _check(rc, "kvm_ref_exchange")


def sha256(msg: bytes) -> bytes:
    a = np.frombuffer(msg, np.uint8).copy() if len(msg) else np.zeros(1, np.uint8)
    out = np.zeros(32, np.uint8)
    _check(lib().kvm_ref_sha256(_p(a, np.uint8), C.c_uint64(len(msg)), _p(out, np.uint8)), "kvm_ref_sha256")
    return out.tobytes()


def hash_units(k_pool, v_pool, unit_k_bytes, unit_v_bytes, slot_tbl, state, uids, n_bad=None):
    """Returns uint8 [n, 32]."""
    n = len(uids)
    digests = np.zeros((max(n, 1), 32), np.uint8)
    n_slots = k_pool.size // unit_k_bytes
    rc = lib().kvm_ref_hash_units(
        _p(k_pool.reshape(-1), np.uint8), _p(None if v_pool is None else v_pool.reshape(-1), np.uint8),
        C.c_uint64(n_slots), C.c_uint32(unit_k_bytes), C.c_uint32(unit_v_bytes),
        _p(slot_tbl, np.int32), _p(state, np.uint8), C.c_int64(len(state)),
        _p(uids, np.int64), C.c_int64(n), _p(digests.reshape(-1), np.uint8), _p(n_bad, np.uint32))
    _check(rc, "kvm_ref_hash_units")
    return digests[:n]


class DedupStore:
    """The oracle's store: a list of (digest, canonical uid, references)."""

    def __init__(self, cap):
        self.digest = np.zeros((cap, 32), np.uint8)
        self.canon = np.full(cap, -1, np.int64)
        self.refs = np.zeros(cap, np.uint32)
        self.n = np.zeros(1, np.int64)
        self.cap = cap

    def insert(self, digests, uids):
        n = len(uids)
        out = np.zeros(max(n, 1), np.int64)
        rc = lib().kvm_ref_dedup_insert(
            _p(self.digest.reshape(-1), np.uint8), _p(self.canon, np.int64), _p(self.refs, np.uint32),
            _p(self.n, np.int64), C.c_int64(self.cap), _p(np.ascontiguousarray(digests).reshape(-1), np.uint8),
            _p(uids, np.int64), C.c_int64(n), _p(out, np.int64))
        _check(rc, "kvm_ref_dedup_insert")
        return out[:n]

    def release(self, digests, n_bad=None):
        rc = lib().kvm_ref_dedup_release(
            _p(self.digest.reshape(-1), np.uint8), _p(self.refs, np.uint32), C.c_int64(int(self.n[0])),
            _p(np.ascontiguousarray(digests).reshape(-1), np.uint8), C.c_int64(len(digests)), _p(n_bad, np.uint32))
        _check(rc, "kvm_ref_dedup_release")

    def as_dict(self):
        """digest bytes -> (canonical uid, references)."""
        return {self.digest[e].tobytes(): (int(self.canon[e]), int(self.refs[e])) for e in range(int(self.n[0]))}


def decode(bits: int, dtype: int) -> float:
    f = lib().kvm_ref_decode
    f.restype = C.c_double
    return float(f(C.c_uint16(bits), C.c_int(dtype)))


def dedup_share(slot_tbl, state, n_slots, uids, canon, frame_refs, n_bad=None):
    """Duplicates give up their frames and read their canonical unit's.  Returns freed frames per item (-1: none)."""
    n = len(uids)
    freed = np.zeros(max(n, 1), np.int32)
    rc = lib().kvm_ref_dedup_share(_p(slot_tbl, np.int32), _p(state, np.uint8), C.c_int64(len(state)),
                                   C.c_uint64(n_slots), _p(uids, np.int64), _p(canon, np.int64), C.c_int64(n),
                                   _p(frame_refs, np.uint32), _p(freed, np.int32), _p(n_bad, np.uint32))
    _check(rc, "kvm_ref_dedup_share")
    return freed[:n]


def dedup_unshare(k_pool, v_pool, unit_k_bytes, unit_v_bytes, slot_tbl, state, uids, new_frames, frame_refs,
                  n_bad=None):
    """Units get frames of their own again.  Returns per item the frame that is free afterwards (-1: none)."""
    n = len(uids)
    freed = np.zeros(max(n, 1), np.int32)
    n_slots = k_pool.size // unit_k_bytes
    rc = lib().kvm_ref_dedup_unshare(
        _p(k_pool.reshape(-1), np.uint8), _p(None if v_pool is None else v_pool.reshape(-1), np.uint8),
        C.c_uint64(n_slots), C.c_uint32(unit_k_bytes), C.c_uint32(unit_v_bytes), _p(slot_tbl, np.int32),
        _p(state, np.uint8), C.c_int64(len(state)), _p(uids, np.int64), _p(new_frames, np.int32), C.c_int64(n),
        _p(frame_refs, np.uint32), _p(freed, np.int32), _p(n_bad, np.uint32))
    _check(rc, "kvm_ref_dedup_unshare")
    return freed[:n]
