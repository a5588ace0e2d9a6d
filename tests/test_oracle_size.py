"""Pins for the sizing oracle: the values the paper prints (Tables 1, 3, 6 and the
text of section 2.1), read from tests/golden/paper_tables.txt, plus the
architecture-inference rule of section 3.1."""
import os

import pytest

GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_tables.txt")


def load_golden():
    rows = {}
    with open(GOLD) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = [p.strip() for p in line.split("|")]
            rows.setdefault(parts[0], {})[parts[1]] = parts[2:]
    return rows


G = load_golden()
MODELS = {name: dict(zip(("L", "h_q", "h_kv", "d", "d_latent", "d_rope"), map(int, v)))
          for name, v in G["model"].items()}


def sized(o, name, mha_equiv=False, divisor=1, **kw):
    m = MODELS[name]
    if mha_equiv:   # pretend every query head has its own KV head
        return o.size(m["L"], m["h_q"], m["h_q"], m["d"], 0, 0, head_divisor=divisor, **kw)
    return o.size(m["L"], m["h_q"], m["h_kv"], m["d"], m["d_latent"], m["d_rope"],
                  head_divisor=divisor, **kw)


@pytest.mark.parametrize("name", list(G["table1"]))
def test_table1_bytes_per_token_layer(oracle, name):
    mha, actual, ratio = map(int, G["table1"][name])
    assert sized(oracle, name, mha_equiv=True)["bytes_per_token_layer"] == mha
    assert sized(oracle, name)["bytes_per_token_layer"] == actual
    assert round(mha / actual) == ratio


@pytest.mark.parametrize("name", list(G["table3"]))
def test_table3_max_batch(oracle, name):
    mha_batch, arch_batch = map(int, G["table3"][name])
    kw = dict(n_max=4096, mem_target=30 * 10**9)
    assert sized(oracle, name, mha_equiv=True, divisor=8, **kw)["max_batch"] == mha_batch
    assert sized(oracle, name, **kw)["max_batch"] == arch_batch


@pytest.mark.parametrize("name", list(G["table6"]))
def test_table6_raw_checkpoint(oracle, name):
    (raw_mb,) = G["table6"][name]
    s = sized(oracle, name, n_max=1000)
    assert f"{s['bytes_per_seq'] / 1e6:.1f}" == raw_mb


def test_section21_llama_128k(oracle):
    tokens, mha_gb, gqa_gb = map(int, G["text21"]["Llama-3-70B"])
    assert round(sized(oracle, "Llama-3-70B", mha_equiv=True, n_max=tokens)["bytes_per_seq"] / 1e9) == mha_gb
    assert round(sized(oracle, "Llama-3-70B", n_max=tokens)["bytes_per_seq"] / 1e9) == gqa_gb
    # one 131072-token context of this model is exactly 40 GiB, the tier-0 capacity the paper quotes
    assert sized(oracle, "Llama-3-70B", n_max=131072)["bytes_per_seq"] == 40 * 2**30


def test_arch_inference_and_units(oracle):
    assert oracle.size(4, 8, 8, 64)["arch"] == 0            # MHA
    assert oracle.size(4, 8, 2, 64)["arch"] == 1            # GQA
    assert oracle.size(4, 8, 1, 64)["arch"] == 2            # MQA
    assert oracle.size(4, 8, 8, 64, d_latent=32, d_rope=8)["arch"] == 3   # latent wins
    assert oracle.size(4, 1, 1, 64)["arch"] == 0            # h_q == h_kv == 1: first rule that matches
    s = oracle.size(32, 32, 8, 128, mem_target=8192 * 1000 + 5)
    assert (s["group_size"], s["units_per_block"], s["unit_k_bytes"], s["unit_v_bytes"]) == (4, 256, 4096, 4096)
    assert s["pool_units"] == 1000
    m = oracle.size(61, 128, 128, 128, d_latent=512, d_rope=64, mem_target=18432 * 7)
    assert (m["group_size"], m["units_per_block"], m["unit_k_bytes"], m["unit_v_bytes"], m["pool_units"]) == \
        (128, 61, 18432, 0, 7)
    # Eq. 3 cases written out
    assert oracle.size(1, 8, 8, 64)["bytes_per_token_layer"] == 2 * 8 * 64 * 2
    assert oracle.size(1, 8, 1, 64)["bytes_per_token_layer"] == 2 * 1 * 64 * 2
    assert oracle.size(1, 8, 8, 64, d_latent=96, d_rope=32)["bytes_per_token_layer"] == (96 + 32) * 2
    # 4-bit elements are half a byte each (p = 0.5)
    assert oracle.size(1, 8, 2, 64, bits_per_elem=4)["bytes_per_token_layer"] == 2 * 2 * 64 // 2


def test_head_weight_rule_per_architecture(oracle):
    """Section 3.4: the aggregate importance weights heads uniformly for MHA and in proportion to the
    group size for GQA; MQA is the group of all query heads; the MLA matrix has one head per layer."""
    assert oracle.size(32, 32, 32, 128)["head_weight"] == 1                      # MHA: uniform
    assert oracle.size(4, 1, 1, 64)["head_weight"] == 1                          # one head each way is MHA
    assert oracle.size(32, 32, 8, 128)["head_weight"] == 4                       # GQA, 4 query heads per KV head
    assert oracle.size(80, 64, 8, 128)["head_weight"] == 8
    assert oracle.size(1, 4, 2, 64, bits_per_elem=16)["head_weight"] == 2
    assert oracle.size(32, 32, 1, 128)["head_weight"] == 32                      # MQA: all query heads in one group
    assert oracle.size(61, 128, 128, 128, d_latent=512, d_rope=64)["head_weight"] == 1   # MLA: single latent head
    # proportional: doubling the group doubles the weight; the tensor-parallel divisor does not enter
    for hq, hkv in ((16, 8), (32, 8), (64, 8), (64, 2)):
        assert oracle.size(2, hq, hkv, 64)["head_weight"] * hkv == hq
    assert oracle.size(2, 64, 8, 64, head_divisor=8)["head_weight"] == 8


def test_size_rejects_bad_models(oracle):
    for bad in (dict(n_layers=0), dict(n_q_heads=6, n_kv_heads=4), dict(bits_per_elem=7),
                dict(head_divisor=3), dict(block_tokens=0), dict(head_dim=0)):
        kw = dict(n_layers=2, n_q_heads=8, n_kv_heads=4, head_dim=64)
        kw.update(bad)
        with pytest.raises(oracle.OracleError):
            oracle.size(**kw)
