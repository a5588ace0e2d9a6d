"""kvm_select_victims_static (the selection with the library's built-in scratch, for callers that
cannot allocate) against kvm_select_victims on the same inputs: bit-identical victim lists and
counts, two calls in a row, the second on a smaller input (the scratch keeps the first call's
contents, none of which may leak into the second)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _inputs(n, seed):
    rng = np.random.default_rng(seed)
    prio = rng.random(n, dtype=np.float32)
    prio[rng.integers(0, n, n // 50)] = prio[0]                       # ties across the cutoff
    prio[rng.integers(0, n, n // 100)] = np.inf
    prio[rng.integers(0, n, n // 200)] = np.nan
    state = rng.choice(np.array([0, 1, 2, 9, 9, 9, 13, 8], np.uint8), n)
    return torch.from_numpy(prio).cuda(), torch.from_numpy(state).cuda()


def _both(kvm, prio, state, k, budget):
    n = state.numel()
    out = []
    for static in (False, True):
        victims = torch.full((n,), -7, dtype=torch.int64, device="cuda")
        n_v = torch.full((1,), -7, dtype=torch.int64, device="cuda")
        if static:
            kvm.kvm_select_victims_static(prio, state, victims, n_v, k=k, budget_units=budget)
        else:
            ws = torch.full((max(kvm.kvm_workspace_bytes(kvm.OP_SELECT, n), 256),), 0x7F, dtype=torch.uint8,
                            device="cuda")
            kvm.kvm_select_victims(prio, state, victims, n_v, ws, k=k, budget_units=budget)
        torch.cuda.synchronize()
        out.append((int(n_v.item()), victims.cpu().numpy()))
    return out


def test_static_select_equals_workspace_select_twice():
    from paper_2604_26968_amd import kvm
    torch.cuda.set_device(0)
    # first call: 1.3 M units (318 chunks, ragged last chunk); second: 70,001 units (18 chunks)
    for n, seed, k, budget in ((1_300_037, 5, -1, 400_000), (70_001, 6, 9_000, 0), (70_001, 6, -1, 12_345)):
        prio, state = _inputs(n, seed)
        (n_a, v_a), (n_b, v_b) = _both(kvm, prio, state, k, budget)
        print("n", n, "k", k, "budget", budget, "victims", n_a, flush=True)
        assert n_a == n_b and n_a > 0
        np.testing.assert_array_equal(v_a, v_b)          # the untouched tail (-7) included
    # empty input and a size beyond the built-in scratch
    e_p, e_s = torch.zeros(0, dtype=torch.float32, device="cuda"), torch.zeros(0, dtype=torch.uint8, device="cuda")
    victims = torch.zeros(4, dtype=torch.int64, device="cuda")
    n_v = torch.full((1,), -7, dtype=torch.int64, device="cuda")
    kvm.kvm_select_victims_static(e_p, e_s, victims, n_v, k=3)
    torch.cuda.synchronize()
    assert int(n_v.item()) == 0
    rc = kvm.lib.kvm_select_victims_static(prio.data_ptr(), state.data_ptr(), kvm.SELECT_STATIC_MAX_UIDS + 1, -1, 0,
                                           victims.data_ptr(), 4, n_v.data_ptr(), None)
    assert rc == kvm.ENOSPC and "limit" in kvm.kvm_last_error()
