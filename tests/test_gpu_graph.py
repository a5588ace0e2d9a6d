"""One step of the pass captured in a HIP graph (the library only launches kernels on the stream it is given:
no allocation, no memset, no synchronisation) and replayed: every replay, with eager work of the program and
synchronisations in between, must leave exactly what the same calls leave when issued eagerly."""
import numpy as np
import pytest
import torch

from paper_2604_26968_amd import synth
from tests.harness import DeviceCase

pytestmark = pytest.mark.gpu
RES, HOST, PROT, SCORED = 1, 2, 4, 8


@pytest.mark.parametrize("shape", [
    synth.Shape(2, 8, 2, 128, synth.BF16, True, [700, 77, 9000]),        # dot2 tile kernel, rows of one and several tiles
    synth.Shape(2, 32, 1, 128, synth.FP16, True, [900, 40]),             # matrix-core tile kernel
])
def test_step_in_a_graph_replays_like_the_eager_step(shape):
    from paper_2604_26968_amd import kvm
    torch.cuda.set_device(0)
    case = synth.make_case(shape, seed=61)
    dev = DeviceCase(case)
    n = case.n_uids
    rng = np.random.default_rng(3)
    q = torch.from_numpy(synth.make_queries(case, 5).view(np.int16)).cuda()
    ev_p = torch.from_numpy(rng.integers(0, 16, 500).astype(np.uint8)).cuda()
    ev_o = torch.from_numpy(rng.integers(0, 2, 500).astype(np.uint8)).cuda()
    scale = float(1.0 / np.sqrt(shape.dim))
    k = int((case.state & RES).sum()) // 5
    rows = dev.rows()
    rec = dev.rec
    tier = torch.zeros(k * rec, dtype=torch.uint8).pin_memory()
    slots = torch.arange(k, dtype=torch.int32, device="cuda")
    freed = torch.full((k,), -1, dtype=torch.int32, device="cuda")

    def step():
        kvm.kvm_beta_update(ev_p, ev_o, dev.hits, dev.misses, dev.p_hat, n_bad=dev.n_bad)
        kvm.kvm_score_step(dev.pool, rows, q, scale, dev.mass, dev.ws)
        kvm.kvm_ema_update(rows, dev.mass, 0.9, dev.row_weight, dev.pair, dev.p_hat, dev.state, dev.S, dev.prio)
        kvm.kvm_select_victims_static(dev.prio, dev.state, dev.victims, dev.n_victims, k=k)
        # zero-copy pack of the victims (the list's length comes from the device)
        kvm.kvm_pack(dev.pool, dev.slot_tbl, dev.state, dev.victims, k, slots, freed, None, tier, n_bad=dev.n_bad,
                     n_dev=dev.n_victims)

    names = ("mass", "S", "prio", "state", "slot_tbl", "hits", "misses", "p_hat", "victims", "n_victims", "n_bad")
    start = {a: getattr(dev, a).clone() for a in names}

    def restore():
        for a in names:
            getattr(dev, a).copy_(start[a])
        freed.fill_(-1)
        tier.zero_()
        dev.ws.fill_(0x7F)

    def snapshot():
        torch.cuda.synchronize()
        out = {a: getattr(dev, a).cpu().numpy().copy() for a in names}
        out["freed"] = freed.cpu().numpy().copy()
        out["tier"] = tier.numpy().copy()
        return out

    step()                                   # loads the code objects, sets kernel attributes
    torch.cuda.synchronize()
    restore()
    step()
    want = snapshot()
    assert int(want["n_victims"][0]) == k and (want["freed"] >= 0).all() and want["tier"].any()
    assert int(want["n_bad"][0]) == 0

    restore()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for replay in range(4):
        restore()                            # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        got = snapshot()
        for a in want:
            np.testing.assert_array_equal(got[a], want[a], err_msg="replay %d: %s" % (replay, a))
        if replay == 1:                      # more eager work: an unrelated scoring call on the same stream
            kvm.kvm_score_step(dev.pool, rows, q, scale, dev.mass, dev.ws)
            torch.cuda.synchronize()
