"""Sizing on the path (section 3.1, Eq. 3 and Eq. 4; head weights of section 3.4): for each attention
architecture the pool is dimensioned with kvm_size (units per token block, unit bytes, frames for a
byte budget), every field of the result is compared with the oracle's sizing function, and one step of
scoring + EMA + priority + selection runs in that pool with the head weight the sizing call returned,
against the oracle with the head weight of its own sizing function."""
import numpy as np
import pytest
import torch

from paper_2604_26968_amd import synth
from tests.harness import DeviceCase, oracle_score, ref_row_weight, sized_pool_units

pytestmark = pytest.mark.gpu

ARCHS = {
    # name: (shape, expected architecture code, expected head weight)
    "mha": (synth.Shape(2, 4, 4, 128, synth.BF16, True, [300, 77]), 0, 1),
    "gqa": (synth.Shape(2, 8, 2, 128, synth.BF16, True, [300, 77]), 1, 4),
    "mqa": (synth.Shape(2, 32, 1, 128, synth.BF16, True, [300, 77]), 2, 32),
    "mla": (synth.Shape(2, 128, 1, 576, synth.BF16, False, [300, 77]), 3, 1),
}


@pytest.mark.parametrize("name", list(ARCHS))
def test_pool_sized_by_kvm_size_and_step_in_it(oracle, name):
    from paper_2604_26968_amd import kvm
    shape, arch, weight = ARCHS[name]
    spare = 5
    pool_units = sized_pool_units(kvm, oracle, shape, spare_units=spare)
    args = dict(shape.model_args(), n_max=4096, mem_target=30 * 10**9)
    s, r = kvm.kvm_size(**args), oracle.size(**args)
    assert s == r and s["arch"] == arch and s["head_weight"] == weight
    for field in ("bytes_per_token_layer", "bytes_per_token", "bytes_per_seq", "max_batch", "units_per_block",
                  "unit_k_bytes", "unit_v_bytes", "pool_units", "group_size"):
        assert s[field] == r[field], field
    # bytes of one token over all layers = units of one token block x unit bytes / 16 tokens
    assert s["bytes_per_token"] * 16 == s["units_per_block"] * (s["unit_k_bytes"] + s["unit_v_bytes"])

    case = synth.make_case(shape, seed=61, spare_slots=spare, pair_weights=synth.categorical_weights(4),
                           poison_tail=True)
    assert case.n_slots == pool_units
    dev = DeviceCase(case)
    assert float(dev.row_weight[0]) == weight
    scale = 1.0 / np.sqrt(shape.dim)
    q = synth.make_queries(case, 62)
    ev = synth.make_events(300, 63)
    hits, misses = np.zeros(16, np.uint32), np.zeros(16, np.uint32)
    gh, gm, gp = dev.beta(*ev)
    p_hat = oracle.beta_update(ev[0], ev[1], hits, misses)
    np.testing.assert_array_equal(gh, hits)
    gmass = dev.score(q, scale)
    omass = oracle_score(oracle, case, q, scale)
    np.testing.assert_allclose(gmass, omass, rtol=1e-3, atol=1e-9)
    S, prio = np.zeros(case.n_uids, np.float32), np.zeros(case.n_uids, np.float32)
    state = case.state.copy()
    oracle.ema_update(case.row_ntok, case.row_off, omass, 0.9, ref_row_weight(oracle, case), case.pair, p_hat, state,
                      S, prio)
    gS, gprio, gstate = dev.ema(0.9)
    np.testing.assert_array_equal(gstate, state)
    np.testing.assert_allclose(gprio, prio, rtol=1e-3)
    # the priority carries the head weight: weight x S x posterior mean
    np.testing.assert_allclose(gprio, weight * gS * gp[case.pair], rtol=1e-6)
    # selection on the oracle's keys inside the sized pool: identical sets
    dev.prio.copy_(torch.from_numpy(prio).cuda())
    budget = int(0.6 * pool_units)
    np.testing.assert_array_equal(dev.select(k=-1, budget=budget),
                                  oracle.select_victims(prio, state, k=-1, budget_units=budget))
