"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header
declares, sizes like the paper's tables, and rejects bad arguments before
touching the GPU."""
import os
import re

import pytest

from tests.test_oracle_size import G, MODELS

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def kvm():
    from paper_2604_26968_amd import kvm as k
    return k


def test_every_declared_symbol_is_exported(kvm):
    header = open(os.path.join(ROOT, "include", "kvm.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(kvm_[a-z_]+)\s*\(", header))
    assert declared == set(kvm.EXPORTS)
    for name in declared:
        assert getattr(kvm.lib, name) is not None
    assert re.fullmatch(r"\d+\.\d+", kvm.kvm_version())


def test_struct_layouts_match_header(kvm):
    import ctypes as C
    assert C.sizeof(kvm.Model) == 36
    assert C.sizeof(kvm.Sizing) == 64
    assert C.sizeof(kvm.Pool) == 40
    assert C.sizeof(kvm.Rows) == 64
    assert C.sizeof(kvm.EmaEx) == 48
    assert C.sizeof(kvm.Store) == 48


@pytest.mark.parametrize("name", list(G["table3"]))
def test_kvm_size_reproduces_paper_tables(kvm, oracle, name):
    m = MODELS[name]
    mha_batch, arch_batch = map(int, G["table3"][name])
    kw = dict(n_max=4096, mem_target=30 * 10**9)
    a = kvm.kvm_size(m["L"], m["h_q"], m["h_q"], m["d"], head_divisor=8, **kw)
    b = kvm.kvm_size(m["L"], m["h_q"], m["h_kv"], m["d"], m["d_latent"], m["d_rope"], **kw)
    assert a["max_batch"] == mha_batch and b["max_batch"] == arch_batch
    mha, actual, _ = map(int, G["table1"][name])
    assert kvm.kvm_size(m["L"], m["h_q"], m["h_q"], m["d"])["bytes_per_token_layer"] == mha
    assert b["bytes_per_token_layer"] == actual
    # every field equals the oracle's
    assert b == oracle.size(m["L"], m["h_q"], m["h_kv"], m["d"], m["d_latent"], m["d_rope"], **kw)
    assert a == oracle.size(m["L"], m["h_q"], m["h_q"], m["d"], head_divisor=8, **kw)


def test_kvm_size_matches_oracle_on_a_sweep(kvm, oracle):
    for L in (1, 32):
        for hq, hkv in ((8, 8), (8, 2), (8, 1), (1, 1)):
            for d in (64, 128):
                for bits in (4, 8, 16):
                    for lat in (0, 512):
                        kw = dict(d_latent=lat, d_rope=64 if lat else 0, bits_per_elem=bits, n_max=1000,
                                  mem_target=10**9)
                        assert kvm.kvm_size(L, hq, hkv, d, **kw) == oracle.size(L, hq, hkv, d, **kw)


def test_kvm_size_errors(kvm):
    for bad in (dict(n_layers=0), dict(n_q_heads=6, n_kv_heads=4), dict(bits_per_elem=7),
                dict(head_divisor=3), dict(block_tokens=0), dict(head_dim=0)):
        kw = dict(n_layers=2, n_q_heads=8, n_kv_heads=4, head_dim=64)
        kw.update(bad)
        with pytest.raises(kvm.KvmError) as e:
            kvm.kvm_size(**kw)
        assert e.value.code == kvm.EINVAL and "kvm_size" in str(e.value)


def test_device_entry_points_validate_before_launching(kvm):
    """Null descriptors / buffers and bad scalars return an error code on the host."""
    import ctypes as C
    lib = kvm.lib
    pool = kvm.Pool(None, None, 4, 128, kvm.BF16, 4096, 4096)
    rows = kvm.Rows(1, 4, 8, 512, None, None, None, None, None)
    assert lib.kvm_score_step(None, None, None, 1.0, 0, None, None, 0, None) == kvm.EINVAL
    assert lib.kvm_score_step(C.byref(pool), C.byref(rows), None, 1.0, 0, None, None, 0, None) == kvm.EINVAL
    assert "null buffer" in kvm.kvm_last_error()
    bad_dim = kvm.Pool(None, None, 4, 100, kvm.BF16, 3200, 3200)
    assert lib.kvm_score_step(C.byref(bad_dim), C.byref(rows), None, 1.0, 0, None, None, 0, None) == kvm.ESHAPE
    bad_g = kvm.Rows(1, 200, 8, 512, None, None, None, None, None)
    assert lib.kvm_score_step(C.byref(pool), C.byref(bad_g), None, 1.0, 0, None, None, 0, None) == kvm.ESHAPE
    assert lib.kvm_score_step(C.byref(pool), C.byref(rows), None, 1.0, 7, None, None, 0, None) == kvm.EINVAL
    empty = kvm.Rows(0, 4, 0, 0, None, None, None, None, None)
    assert lib.kvm_score_step(C.byref(pool), C.byref(empty), None, 1.0, 0, None, None, 0, None) == kvm.OK
    assert lib.kvm_beta_update(None, None, -1, None, None, 1.0, 1.0, None, None, None) == kvm.EINVAL
    assert lib.kvm_beta_update(None, None, 0, None, None, 1.0, 1.0, None, None, None) == kvm.EINVAL
    assert lib.kvm_ema_update(None, None, 0.9, None, None, None, None, None, None, None) == kvm.EINVAL
    assert lib.kvm_ema_update(C.byref(rows), None, 1.5, None, None, None, None, None, None, None) == kvm.EINVAL
    ex = kvm.EmaEx(0.0, 0, 0, None, None, None, None)
    assert lib.kvm_ema_update_ex(C.byref(rows), None, 0.9, None, None, None, None, None, None, None, None) == kvm.EINVAL
    assert lib.kvm_ema_update_ex(C.byref(rows), None, 0.9, C.byref(ex), None, None, None, None, None, None, None) \
        == kvm.EINVAL
    assert "positional decay" in kvm.kvm_last_error()
    ex = kvm.EmaEx(0.5, 0, 0, None, None, None, 1)          # multipliers without the index arrays
    assert lib.kvm_ema_update_ex(C.byref(rows), None, 0.9, C.byref(ex), None, None, None, None, None, None, None) \
        == kvm.EINVAL
    blend = lambda n, window, kappa, ptr: lib.kvm_beta_blend_update(
        None, None, n, ptr, ptr, 1.0, 1.0, ptr, ptr, window, kappa, ptr, ptr, ptr, None, None)
    assert blend(0, 8, 1.0, None) == kvm.EINVAL             # null counters
    assert blend(0, 0, 1.0, 1) == kvm.EINVAL and "window" in kvm.kvm_last_error()
    assert blend(0, 1 << 20, 1.0, 1) == kvm.EINVAL
    assert blend(0, 8, -1.0, 1) == kvm.EINVAL and "kappa" in kvm.kvm_last_error()
    assert blend(5, 8, 1.0, 1) == kvm.EINVAL                # events without arrays
    span = lambda n_layers, num, den, w_min, w_max, ptr: lib.kvm_span_update(
        C.byref(rows), None, n_layers, None, None, num, den, ptr, ptr, w_min, w_max, ptr, None, 0, None)
    assert span(0, 9, 10, 0, 100, 1) == kvm.EINVAL
    assert span(4, 11, 10, 0, 100, 1) == kvm.EINVAL and "theta" in kvm.kvm_last_error()
    assert span(4, 9, 0, 0, 100, 1) == kvm.EINVAL
    assert span(4, 9, 10, 50, 10, 1) == kvm.EINVAL
    assert span(4, 9, 10, 0, 100, None) == kvm.EINVAL
    assert span(4, 9, 10, 0, 100, 1) == kvm.EINVAL and "null row array" in kvm.kvm_last_error()
    keys = lambda n_layers, decay: lib.kvm_prefetch_keys(
        C.byref(rows), None, None, None, n_layers, None, None, None, decay, None, None, None)
    assert keys(0, 0.9) == kvm.EINVAL
    assert keys(4, 0.0) == kvm.EINVAL and keys(4, 1.5) == kvm.EINVAL
    assert keys(4, 0.9) == kvm.EINVAL
    assert lib.kvm_hash_units(None, None, None, 8, None, 1, None, None, None) == kvm.EINVAL
    odd = kvm.Pool(1, 1, 4, 128, kvm.BF16, 4096, 4000)
    assert lib.kvm_hash_units(C.byref(odd), None, None, 8, None, 1, None, None, None) == kvm.ESHAPE
    assert lib.kvm_hash_units(C.byref(pool), None, None, 8, None, 0, None, None, None) == kvm.OK
    assert lib.kvm_hash_units(C.byref(pool), None, None, 8, None, 1, None, None, None) == kvm.EINVAL
    st = kvm.Store(1, 1, 1, 1, 1, 12)
    assert lib.kvm_dedup_insert(C.byref(st), None, None, 1, None, None, None, None, 0, None) == kvm.EINVAL
    assert "power of two" in kvm.kvm_last_error()
    st = kvm.Store(1, 1, 1, 1, 1, 16)
    assert lib.kvm_dedup_insert(C.byref(st), None, None, 0, None, None, None, None, 0, None) == kvm.OK
    assert lib.kvm_dedup_insert(C.byref(st), 4, 8, 5, 8, None, None, 8, 16, None) == kvm.ENOSPC
    assert lib.kvm_dedup_release(None, None, 1, None, None) == kvm.EINVAL
    assert lib.kvm_dedup_release(C.byref(st), None, 1, None, None) == kvm.EINVAL
    assert lib.kvm_probe_read(None, 16, None, None) == kvm.EINVAL
    assert lib.kvm_probe_read(16, 24, 16, None) == kvm.EINVAL          # size not a multiple of 16
    assert lib.kvm_probe_read(16, 0, 16, None) == kvm.OK
    assert lib.kvm_score_step_xfer(C.byref(pool), C.byref(empty), None, 1.0, 0, None, None, 0, None, None, -1, None,
                                   0, None) == kvm.EINVAL
    assert lib.kvm_score_step_xfer(C.byref(pool), C.byref(empty), None, 1.0, 0, None, None, 0, None, None, 5, None,
                                   0, None) == kvm.EINVAL                   # pairs without buffers
    assert lib.kvm_score_step_xfer(C.byref(pool), C.byref(empty), None, 1.0, 0, None, None, 0, None, None, 0, None,
                                   0, None) == kvm.OK
    assert lib.kvm_exchange(None, None, None, 0, None, None, 0, None, None, None, 0, None, None) == kvm.EINVAL
    assert lib.kvm_exchange(C.byref(pool), None, None, 8, None, None, 4, None, None, None, 4, None, None) == kvm.EINVAL
    assert lib.kvm_exchange_begin(C.byref(pool), None, None, 8, None, None, 4, None, None, 4, None, None, None,
                                  None) == kvm.EINVAL
    assert lib.kvm_dedup_share(None, None, 8, 4, None, None, 3, None, None, None, None) == kvm.EINVAL
    assert lib.kvm_dedup_share(None, None, 8, 4, None, None, 0, None, None, None, None) == kvm.OK
    assert lib.kvm_dedup_share(None, None, 8, 1 << 40, None, None, 0, None, None, None, None) == kvm.EINVAL
    assert lib.kvm_dedup_unshare(None, None, None, 8, None, None, 3, None, None, None, None) == kvm.EINVAL
    assert lib.kvm_dedup_unshare(C.byref(pool), None, None, 8, None, None, 3, None, None, None, None) == kvm.EINVAL
    assert lib.kvm_dedup_unshare(C.byref(pool), None, None, 8, None, None, 0, None, None, None, None) == kvm.OK
    assert lib.kvm_pack_begin(None, None, None, 8, None, 4, None, None, 4, None, None, None, None) == kvm.EINVAL
    assert lib.kvm_pack_begin(C.byref(pool), None, None, 8, None, 4, None, None, 4, None, None, None, None) == kvm.EINVAL
    assert lib.kvm_pack_begin(C.byref(pool), None, None, 8, None, 0, None, None, 4, None, None, None, None) == kvm.OK
    assert lib.kvm_pack_begin(C.byref(pool), None, None, 8, None, -1, None, None, 4, None, None, None, None) == kvm.EINVAL
    assert lib.kvm_exchange_end(None, None, 8, None, None, 4, None) == kvm.EINVAL
    assert lib.kvm_exchange_end(None, None, 8, None, None, 0, None) == kvm.OK
    assert lib.kvm_select_victims(None, None, -1, 0, 0, None, 0, None, None, 0, None) == kvm.EINVAL
    assert lib.kvm_select_victims(None, None, 10, -2, 0, None, 0, None, None, 0, None) == kvm.EINVAL
    assert lib.kvm_pack(None, None, None, 0, None, 0, None, None, None, None, 0, None, 0, None, None) == kvm.EINVAL
    assert lib.kvm_pack(C.byref(pool), None, None, 0, None, 0, None, None, None, None, 0, None, 0, None, None) == kvm.OK
    assert lib.kvm_pack(C.byref(pool), None, None, 8, None, 3, None, None, None, None, 0, None, 0, None, None) == kvm.EINVAL
    assert lib.kvm_unpack(C.byref(pool), None, None, 8, None, -3, None, None, None, 0, None, 0, None, None) == kvm.EINVAL
    assert kvm.kvm_workspace_bytes(kvm.OP_SCORE, 1000, 10, 4, 128) >= 1000 * 4 * 4
    assert kvm.kvm_workspace_bytes(kvm.OP_SELECT, 1000) > 0
    assert kvm.kvm_workspace_bytes(kvm.OP_SPAN, 0, 1000) >= 4000
    assert kvm.kvm_workspace_bytes(99, 1000) == 0
