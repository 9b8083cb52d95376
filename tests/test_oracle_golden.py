"""The oracle on the tiny preset: frozen values, O1 == O2, and sensitivity of the pins to planted mistakes."""
import json
import os

import numpy as np
import pytest

import asynclm_inputs as ai
from oracle import asynclm_oracle as orc

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.fixture(scope="module")
def tiny():
    wl = ai.preset("tiny")
    w = ai.weights_to_numpy(ai.make_weights(wl.model, ai.MASTER_SEED))
    spec = ai.build_workload("tiny", ai.MASTER_SEED)
    sh = orc.Shape.of(wl.model)
    res = orc.run_stream(sh, w, spec["prompt"], spec["n_decode"], spec["events"])
    return wl, sh, w, spec, res


def test_tiny_stream_matches_frozen_values(tiny):
    wl, sh, w, spec, res = tiny
    with open(os.path.join(HERE, "golden", "tiny_stream.json")) as f:
        gold = json.load(f)
    assert gold["seed"] == ai.MASTER_SEED
    assert [int(t) for t in spec["prompt"][:8]] == gold["prompt_head"]
    assert [int(t) for t in spec["events"][0][1]] == gold["interrupt"]
    assert res["generated"] == gold["generated"]
    assert len(res["stream"]) == gold["stream_len"] == 64 + 32 + 8
    for l, head in zip(res["choose_logits"], gold["logit_heads"]):
        assert np.abs(l[:6] - np.array(head)).max() < 1e-8
    assert np.abs(res["final_logits"][:6] - np.array(gold["final_logit_head"])).max() < 1e-8


def test_tiny_cached_equals_from_scratch(tiny):
    wl, sh, w, spec, res = tiny
    ref = orc.full_logits(sh, w, res["stream"])
    P, k = len(spec["prompt"]), len(spec["events"][0][1])
    for j in range(32):
        at = P + j - 1 + (k if j >= 16 else 0)
        assert np.abs(res["choose_logits"][j] - ref[at]).max() < 1e-10
    assert np.abs(res["final_logits"] - ref[-1]).max() < 1e-10
    # the interrupt sits between generated tokens 16 and 17
    s = res["stream"]
    assert s[P + 16:P + 16 + k] == [int(t) for t in spec["events"][0][1]]
    assert s[P + 16 + k] == res["generated"][16]


def test_fp32_oracle_on_tiny_is_within_parity_budget(tiny):
    wl, sh, w, spec, res = tiny
    r32 = orc.run_stream(sh, w, spec["prompt"], 8, [], dtype=np.float32)
    r64 = orc.run_stream(sh, w, spec["prompt"], 8, [])
    for a, b in zip(r32["choose_logits"], r64["choose_logits"]):
        assert np.abs(a - b).max() < 2e-5


# Mistakes planted in the oracle (on the CPU) must trip the from-scratch / library pins.
@pytest.mark.parametrize("mistake", ["no_scale", "interleaved_rope", "eps_outside", "kv_head_map", "drop_gate"])
def test_planted_mistakes_are_caught(monkeypatch, mistake):
    import torch
    from tests.test_oracle_pins import _model, _tokens, _hf_model
    cfg, sh, w = _model(hq=4, hkv=2)
    toks = _tokens(23, cfg.vocab, seed=3)
    with torch.no_grad():
        want = _hf_model(cfg, w)(torch.from_numpy(toks)[None]).logits[0].numpy()
    assert np.abs(orc.full_logits(sh, w, toks) - want).max() < 2e-5
    if mistake == "no_scale":
        good_sm = orc.softmax_rows
        monkeypatch.setattr(orc, "softmax_rows", lambda sc: good_sm(sc * np.sqrt(cfg.head_dim)))
    elif mistake == "interleaved_rope":
        good = orc.rope_rotate
        half = cfg.head_dim // 2
        inter = np.arange(cfg.head_dim).reshape(half, 2).T.reshape(-1)     # pairs (2i, 2i+1) instead of (i, i+dh/2)
        back = np.argsort(inter)
        monkeypatch.setattr(orc, "rope_rotate", lambda u, pos, theta: good(u[..., inter], pos, theta)[..., back])
    elif mistake == "eps_outside":
        monkeypatch.setattr(orc, "rmsnorm", lambda x, g, eps: x * g / (np.sqrt(np.mean(x * x, -1, keepdims=True)) + 1e-2))
    elif mistake == "kv_head_map":
        w = dict(w)
        nq, nkv, dh = cfg.q_dim, cfg.kv_dim, cfg.head_dim
        swap = lambda blk: blk.reshape(2, dh, -1)[::-1].reshape(nkv, -1)   # exchange the two kv heads' keys
        w["wqkv"] = [np.concatenate([a[:nq], swap(a[nq:nq + nkv]), a[nq + nkv:]]) for a in w["wqkv"]]
    elif mistake == "drop_gate":
        monkeypatch.setattr(orc, "silu", lambda z: z)
    assert np.abs(orc.full_logits(sh, w, toks) - want).max() > 1e-3
