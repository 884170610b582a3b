"""The shared input generators: determinism, shapes, and bf16 rounding of inputs."""
import numpy as np
import torch

from paper_2407_00952_amd import synth


def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(0)
    a = np.concatenate([rng.standard_normal(5000).astype(np.float32) * 10.0 ** rng.integers(-6, 6, 5000),
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38], dtype=np.float32)])
    a = a.astype(np.float32)
    mine = synth.round_bf16(a)
    ref = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(mine, ref)
    bits = synth.bf16_bits(a)
    assert np.array_equal(torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).float().numpy(), ref)
    assert np.array_equal(synth.round_bf16(mine), mine)


def test_stack_inputs_are_seeded_and_shaped():
    cfg = synth.tiny_config(lora_proj=("q", "v", "pr"))
    a = synth.make_stack_inputs(cfg)
    b = synth.make_stack_inputs(cfg)
    assert len(a["blocks"]) == cfg.n_blocks and len(a["clients"]) == cfg.n_clients
    assert a["clients"][0].shape == (cfg.batch, cfg.seq_len, cfg.d_model)
    assert a["dY"].shape == (cfg.n_seq, cfg.seq_len, cfg.d_model)
    assert a["blocks"][0]["Wqkv"].shape == (3 * cfg.d_model, cfg.d_model)
    assert a["adapters"][1]["pr"][0].shape == (cfg.lora_r, cfg.d_ff)
    assert a["adapters"][1]["pr"][1].shape == (cfg.d_model, cfg.lora_r)
    for k in a["blocks"][0]:
        assert np.array_equal(a["blocks"][0][k], b["blocks"][0][k])
        assert np.array_equal(synth.round_bf16(a["blocks"][0][k]), a["blocks"][0][k])
    assert np.array_equal(a["dY"], b["dY"])
    A = a["adapters"][0]["q"][0]
    assert np.abs(A).max() <= 1 / np.sqrt(cfg.d_model) * 1.01


def test_workload_table():
    c = synth.CONFIGS
    assert (c[2].tokens, c[3].tokens, c[4].tokens, c[5].tokens) == (10240, 32768, 32768, 65536)
    assert all(cfg.d_model // cfg.n_head == 64 for cfg in c.values())
    vecs, counts = synth.make_fedavg_inputs(n_clients=3, n_params=10)
    assert counts.min() >= 100 and counts.max() <= 1000 and vecs[0].dtype == np.float32
