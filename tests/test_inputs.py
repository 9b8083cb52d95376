"""Seeded input generators: definition checks, determinism, statistics."""
import numpy as np
import pytest
import torch

import asynclm_inputs as ai
from asynclm_inputs import generator as gen


def test_splitmix64_published_vector():
    # First outputs of SplitMix64 from state 1234567, as printed with the reference C code
    # that accompanies xoshiro/xoroshiro (Vigna) and used in many ports' unit tests.
    got = ai.splitmix64_draws_py(1234567, 5)
    assert got == [6457827717110365317, 3203168211198807973, 9817491932198370423,
                   4593380528125082431, 16408922859458223821]


def test_torch_mixer_matches_python_bigint():
    rng = np.random.default_rng(0)
    vals = [0, 1, 2**63 - 1, 2**63, 2**64 - 1] + [int(v) for v in rng.integers(0, 2**63, size=64)]
    t = torch.tensor([gen._signed(v) for v in vals], dtype=torch.int64)
    out = gen._mix64_t(t).tolist()
    for v, o in zip(vals, out):
        assert (o & gen._MASK64) == gen._mix64_py(v)


def test_element_definition_by_hand():
    seed, tid = 77, 5
    key = ai.tensor_key(seed, tid)
    draws = ai.splitmix64_draws_py(key, 3 * 40)
    want = []
    for i in range(40):
        s = 0
        for z in draws[3 * i:3 * i + 3]:
            s += sum((z >> (16 * j)) & 0xFFFF for j in range(4))
        want.append(np.float32(s - 393210) * (np.float32(0.02) * np.float32(2.0 ** -16)))
    got = ai.gaussian_tensor(seed, tid, (40,), 0.02, "fp32").numpy()
    assert np.array_equal(got, np.array(want, dtype=np.float32))


def test_slices_and_chunks_agree():
    full = ai.gaussian_tensor(3, 9, (1000, 37), chunk=1 << 24)
    small_chunks = ai.gaussian_tensor(3, 9, (1000, 37), chunk=997)
    assert torch.equal(full, small_chunks)
    part = gen.gaussian_flat(3, 9, 12345, 500, 0.02)
    assert torch.equal(full.view(-1)[12345:12845], part)


def test_statistics_match_normal():
    x = ai.gaussian_tensor(11, 2, (1 << 20,)).double().numpy()
    assert abs(x.mean()) < 4 * 0.02 / np.sqrt(x.size)
    assert abs(x.std() / 0.02 - 1) < 5e-3
    assert abs(np.mean(x ** 4) / 0.02 ** 4 - 2.9) < 0.05   # Irwin-Hall(12): kurtosis 3 - 0.1
    assert np.abs(x).max() <= 6 * 0.02 * (1 + 1e-6)
    # different tensors and different seeds are uncorrelated
    y = ai.gaussian_tensor(11, 3, (1 << 20,)).double().numpy()
    z = ai.gaussian_tensor(12, 2, (1 << 20,)).double().numpy()
    for o in (y, z):
        assert abs(np.corrcoef(x, o)[0, 1]) < 5e-3


def test_bf16_is_rne_of_fp32():
    a = ai.gaussian_tensor(5, 7, (4096,), dtype="fp32")
    b = ai.gaussian_tensor(5, 7, (4096,), dtype="bf16")
    assert b.dtype == torch.bfloat16
    assert torch.equal(a.to(torch.bfloat16), b)


def test_weights_layout_and_truncation():
    wl = ai.preset("tiny")
    w = ai.make_weights(wl.model, seed=1)
    m = wl.model
    assert w["wqkv"][0].shape == (m.q_dim + 2 * m.kv_dim, m.d_model)
    assert w["wgate_up"][1].shape == (2 * m.ffn, m.d_model)
    assert w["wdown"][1].shape == (m.d_model, m.ffn)
    assert torch.equal(w["attn_norm"][0], torch.ones(m.d_model))
    w1 = ai.make_weights(ai.truncated(m, 1), seed=1)
    assert len(w1["wqkv"]) == 1 and torch.equal(w1["wqkv"][0], w["wqkv"][0])
    assert torch.equal(w1["lm_head"], w["lm_head"])
    wn = ai.weights_to_numpy(w)
    assert wn["embed"].dtype == np.float32 and isinstance(wn["wo"], list)


def test_model_byte_counts():
    m = ai.preset("8b").model
    assert m.weight_bytes_per_step() == 15_009_316_864   # 32 x 436.2 MB + 1.05 GB output head
    assert m.kv_bytes_per_position() == 131072
    m70 = ai.preset("70b").model
    assert m70.kv_bytes_per_position() == 327680
    assert abs(m70.weight_bytes_per_step() / 1e9 - 139.0) < 0.05


@pytest.mark.parametrize("name", ["tiny", "8b", "8b-long", "70b"])
def test_single_sequence_workloads(name):
    wl = ai.preset(name)
    a, b = ai.build_workload(name), ai.build_workload(name)
    assert np.array_equal(a["prompt"], b["prompt"]) and a["prompt"].dtype == np.int32
    assert len(a["prompt"]) == wl.prompt_len
    assert a["prompt"].min() >= 0 and a["prompt"].max() < wl.model.vocab
    steps = [n for n, _ in a["events"]]
    assert steps == sorted(set(steps)) and all(1 <= n < wl.n_decode for n in steps)
    if name == "tiny":
        assert steps == [16] and len(a["events"][0][1]) == 8
    if name == "8b":
        assert steps == [64, 128, 192] and all(len(t) == 24 for _, t in a["events"])
    if name == "8b-long":
        assert sum(len(t) for _, t in a["events"]) == 8 * 48
    if name == "70b":
        assert steps == list(range(32, 256, 32)) and all(len(t) == 32 for _, t in a["events"])
    other = ai.build_workload(name, seed=5)
    assert not np.array_equal(a["prompt"], other["prompt"])


def test_ragged_workload():
    a = ai.build_workload("8b-ragged16")
    assert len(a["prompts"]) == 16
    assert all(512 <= len(p) <= 4096 for p in a["prompts"])
    assert len(a["step_events"]) == 256 and a["step_events"][-1] == []
    n = sum(len(ev) for ev in a["step_events"])
    assert 120 < n < 300            # Bernoulli(0.05) over 16 x 255 slots, mean 204
    assert all(16 <= len(t) <= 32 for ev in a["step_events"] for _, t in ev)
