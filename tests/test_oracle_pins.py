"""Pins for the CPU oracle: things the paper and the mathematics fix, none computed by the oracle itself.

The paper (arXiv 2412.07017) prints no numeric model outputs, so the oracle is tied to
  (a) an independent library implementation of the Llama architecture (transformers),
  (b) library routines for attention, normalisation, activation, bf16 rounding (torch),
  (c) closed forms and invariants of the decoder,
  (d) the defining property of interrupt injection (Sec. 3.2 vs Sec. 5.5): appending a block
      to the live context gives the logits of a from-scratch pass over the concatenation.
"""
import numpy as np
import pytest
import torch

import asynclm_inputs as ai
from oracle import asynclm_oracle as orc

SEED = 20241207
HF_TOL = 2e-5


def _model(n_layers=2, d=64, hq=4, hkv=2, dh=16, ffn=88, vocab=97, theta=10000.0, seed=SEED):
    cfg = ai.ModelConfig(n_layers, d, hq, hkv, dh, ffn, vocab, 1e-5, theta, "fp32")
    w = ai.weights_to_numpy(ai.make_weights(cfg, seed=seed))
    # scale weights up so that attention is far from uniform and SiLU far from linear
    for k in ("wqkv", "wo", "wgate_up", "wdown"):
        w[k] = [a * np.float32(6.0) for a in w[k]]
    w["embed"] = w["embed"] * np.float32(20.0)
    w["lm_head"] = w["lm_head"] * np.float32(8.0)
    rng = np.random.default_rng(seed)
    w["attn_norm"] = [(1 + 0.3 * rng.standard_normal(d)).astype(np.float32) for _ in range(n_layers)]
    w["ffn_norm"] = [(1 + 0.3 * rng.standard_normal(d)).astype(np.float32) for _ in range(n_layers)]
    w["final_norm"] = (1 + 0.3 * rng.standard_normal(d)).astype(np.float32)
    return cfg, orc.Shape.of(cfg), w


def _tokens(n, vocab, seed=0):
    return np.random.default_rng(seed).integers(0, vocab, size=n)


# ---------------------------------------------------------------- (a) independent library model

def _hf_model(cfg, w):
    from transformers import LlamaConfig, LlamaForCausalLM
    hc = LlamaConfig(vocab_size=cfg.vocab, hidden_size=cfg.d_model, intermediate_size=cfg.ffn,
                     num_hidden_layers=cfg.n_layers, num_attention_heads=cfg.n_q_heads,
                     num_key_value_heads=cfg.n_kv_heads, head_dim=cfg.head_dim,
                     rms_norm_eps=cfg.rms_eps, rope_theta=cfg.rope_theta, tie_word_embeddings=False,
                     attention_bias=False, mlp_bias=False, max_position_embeddings=4096)
    hc._attn_implementation = "eager"
    m = LlamaForCausalLM(hc).double().eval()
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    sd = {"model.embed_tokens.weight": t(w["embed"]), "model.norm.weight": t(w["final_norm"]),
          "lm_head.weight": t(w["lm_head"])}
    nq, nkv, F = cfg.q_dim, cfg.kv_dim, cfg.ffn
    for l in range(cfg.n_layers):
        p = f"model.layers.{l}."
        sd[p + "self_attn.q_proj.weight"] = t(w["wqkv"][l][:nq])
        sd[p + "self_attn.k_proj.weight"] = t(w["wqkv"][l][nq:nq + nkv])
        sd[p + "self_attn.v_proj.weight"] = t(w["wqkv"][l][nq + nkv:])
        sd[p + "self_attn.o_proj.weight"] = t(w["wo"][l])
        sd[p + "mlp.gate_proj.weight"] = t(w["wgate_up"][l][:F])
        sd[p + "mlp.up_proj.weight"] = t(w["wgate_up"][l][F:])
        sd[p + "mlp.down_proj.weight"] = t(w["wdown"][l])
        sd[p + "input_layernorm.weight"] = t(w["attn_norm"][l])
        sd[p + "post_attention_layernorm.weight"] = t(w["ffn_norm"][l])
    missing, unexpected = m.load_state_dict(sd, strict=False)
    assert not unexpected and all("rotary" in k or "inv_freq" in k for k in missing), (missing, unexpected)
    return m


@pytest.mark.parametrize("hq,hkv,theta", [(4, 2, 10000.0), (4, 4, 10000.0), (8, 2, 500000.0)])
def test_full_logits_match_library_llama(hq, hkv, theta):
    cfg, sh, w = _model(hq=hq, hkv=hkv, theta=theta)
    toks = _tokens(37, cfg.vocab, seed=1)
    hf = _hf_model(cfg, w)
    with torch.no_grad():
        want = hf(torch.from_numpy(toks)[None]).logits[0].numpy()
    got = orc.full_logits(sh, w, toks)
    assert np.abs(want).max() > 1.0
    # the library forms its rotary cos/sin tables in fp32, which caps agreement near 1e-6;
    # any structural mistake (pairing, scaling, masking, head mapping) shows up at O(1)
    assert np.abs(got - want).max() < HF_TOL


def test_cached_decoder_matches_library_llama_with_cache():
    cfg, sh, w = _model()
    toks = _tokens(30, cfg.vocab, seed=2)
    hf = _hf_model(cfg, w)
    with torch.no_grad():
        want = hf(torch.from_numpy(toks)[None]).logits[0].numpy()
    dec = orc.CachedDecoder(sh, w)
    assert np.abs(dec.prefill(toks[:11]) - want[10]).max() < HF_TOL
    dec.decode_step(forced=toks[11])
    assert np.abs(dec.logits - want[11]).max() < HF_TOL
    assert np.abs(dec.inject(toks[12:30]) - want[29]).max() < HF_TOL


# ---------------------------------------------------------------- (b) library routines

def test_elementwise_definitions_match_torch():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((5, 48)) * 3
    g = rng.standard_normal(48)
    want = torch.nn.functional.rms_norm(torch.from_numpy(x), (48,), torch.from_numpy(g), eps=1e-5).numpy()
    assert np.abs(orc.rmsnorm(x, g, 1e-5) - want).max() < 1e-12
    assert np.abs(orc.silu(x) - torch.nn.functional.silu(torch.from_numpy(x)).numpy()).max() < 1e-12
    assert orc.silu(np.zeros(3)).tolist() == [0, 0, 0]
    s = rng.standard_normal((7, 9)) * 10
    s[2, 5:] = -np.inf
    want = torch.softmax(torch.from_numpy(s), dim=-1).numpy()
    got = orc.softmax_rows(s)
    assert np.abs(got - want).max() < 1e-14 and np.all(got[2, 5:] == 0)
    assert np.abs(got.sum(-1) - 1).max() < 1e-14


def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(4)
    x = np.concatenate([rng.standard_normal(5000).astype(np.float32) * 3,
                        np.array([1.00390625, 1.01171875, -1.00390625, 0.0, 3.0e-39], dtype=np.float32)])
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(orc.round_to_bf16(x), want)


def test_attention_matches_library_sdpa():
    """One layer with identity-like surroundings: compare the oracle's probabilities with SDPA."""
    cfg, sh, w = _model(n_layers=1)
    toks = _tokens(19, cfg.vocab, seed=5)
    _, probs = orc.full_logits(sh, w, toks, return_probs=True)
    p = probs[0]
    assert np.abs(p.sum(-1) - 1).max() < 1e-12
    assert np.all(np.triu(p, k=1) == 0)            # no weight on future positions
    assert p[:, 0, 0].tolist() == [1.0] * cfg.n_q_heads
    # rebuild q, k with library ops and let SDPA produce the same weights applied to V = identity
    x = torch.from_numpy(w["embed"][toks].astype(np.float64))
    h = torch.nn.functional.rms_norm(x, (cfg.d_model,), torch.from_numpy(w["attn_norm"][0].astype(np.float64)), eps=cfg.rms_eps)
    qkv = h @ torch.from_numpy(w["wqkv"][0].astype(np.float64)).T
    T, dh = len(toks), cfg.head_dim
    q = qkv[:, :cfg.q_dim].view(T, cfg.n_q_heads, dh)
    k = qkv[:, cfg.q_dim:cfg.q_dim + cfg.kv_dim].view(T, cfg.n_kv_heads, dh)
    # rotary by complex multiplication (a different formulation from the oracle's)
    ang = torch.arange(T, dtype=torch.float64)[:, None] * cfg.rope_theta ** (-torch.arange(0, dh, 2, dtype=torch.float64) / dh)
    rot = torch.polar(torch.ones_like(ang), ang)[:, None, :]
    cplx = lambda u: torch.complex(u[..., :dh // 2], u[..., dh // 2:])
    unc = lambda z: torch.cat([z.real, z.imag], dim=-1)
    q, k = unc(cplx(q) * rot), unc(cplx(k) * rot)
    k = k.repeat_interleave(cfg.n_q_heads // cfg.n_kv_heads, dim=1)
    eye = torch.eye(T, dtype=torch.float64)[None].expand(cfg.n_q_heads, T, T)
    want = torch.nn.functional.scaled_dot_product_attention(q.transpose(0, 1), k.transpose(0, 1), eye, is_causal=True)
    assert np.abs(p - want.numpy()).max() < 1e-12


# ---------------------------------------------------------------- (c) closed forms and invariants

def test_rope_properties():
    rng = np.random.default_rng(6)
    u = rng.standard_normal((9, 3, 32))
    pos = np.array([0, 1, 2, 5, 17, 100, 1000, 16895, 17407])
    r = orc.rope_rotate(u, pos, 500000.0)
    assert np.array_equal(r[0], u[0])                                       # position 0 is the identity
    n_in = u[..., :16] ** 2 + u[..., 16:] ** 2
    n_out = r[..., :16] ** 2 + r[..., 16:] ** 2
    assert np.abs(n_in - n_out).max() < 1e-12                               # per-pair norm preserved
    # closed form for pair i at position t: angle t * theta^(-2i/dh)
    t, i = 17, 3
    phi = 17 * 500000.0 ** (-2 * 3 / 32)
    a, b = u[4, 1, i], u[4, 1, i + 16]
    assert abs(r[4, 1, i] - (a * np.cos(phi) - b * np.sin(phi))) < 1e-12
    assert abs(r[4, 1, i + 16] - (b * np.cos(phi) + a * np.sin(phi))) < 1e-12
    # scores depend on the position difference only
    q, k = rng.standard_normal((1, 1, 32)), rng.standard_normal((1, 1, 32))
    dot = lambda m, n: float(np.sum(orc.rope_rotate(q, np.array([m]), 1e4) * orc.rope_rotate(k, np.array([n]), 1e4)))
    assert abs(dot(7, 3) - dot(1007, 1003)) < 1e-10
    assert abs(dot(7, 3) - dot(3, 7)) > 1e-3


def test_position_shift_leaves_logits_unchanged():
    cfg, sh, w = _model()
    toks = _tokens(21, cfg.vocab, seed=7)
    a = orc.full_logits(sh, w, toks)
    b = orc.full_logits(sh, w, toks, pos0=333)
    assert np.abs(a - b).max() < 1e-9


def test_causality_is_bitwise():
    cfg, sh, w = _model()
    toks = _tokens(25, cfg.vocab, seed=8)
    other = toks.copy()
    other[15:] = (other[15:] + 1) % cfg.vocab
    a, b = orc.full_logits(sh, w, toks), orc.full_logits(sh, w, other)
    assert np.array_equal(a[:15], b[:15]) and np.abs(a[15:] - b[15:]).max() > 1e-3


def test_gqa_equals_mha_with_replicated_kv():
    cfg, sh, w = _model(hq=4, hkv=2)
    dh, g = cfg.head_dim, 2
    nq, nkv = cfg.q_dim, cfg.kv_dim
    cfg2 = ai.ModelConfig(cfg.n_layers, cfg.d_model, 4, 4, dh, cfg.ffn, cfg.vocab, cfg.rms_eps, cfg.rope_theta, "fp32")
    w2 = dict(w)
    rep = lambda blk: np.repeat(blk.reshape(2, dh, -1), g, axis=0).reshape(4 * dh, -1)
    w2["wqkv"] = [np.concatenate([a[:nq], rep(a[nq:nq + nkv]), rep(a[nq + nkv:])]) for a in w["wqkv"]]
    toks = _tokens(17, cfg.vocab, seed=9)
    a = orc.full_logits(sh, w, toks)
    b = orc.full_logits(orc.Shape.of(cfg2), w2, toks)
    assert np.abs(a - b).max() < 1e-10


def test_zero_projections_give_closed_form():
    cfg, sh, w = _model()
    toks = _tokens(12, cfg.vocab, seed=10)
    w0 = dict(w)
    w0["wo"] = [np.zeros_like(a) for a in w["wo"]]
    w0["wdown"] = [np.zeros_like(a) for a in w["wdown"]]
    got = orc.full_logits(sh, w0, toks)
    e = w["embed"][toks].astype(np.float64)
    hn = e / np.sqrt((e ** 2).mean(-1, keepdims=True) + cfg.rms_eps) * w["final_norm"]
    assert np.abs(got - hn @ w["lm_head"].astype(np.float64).T).max() < 1e-12
    # attention-only layers (zero down projection) still depend on context, FFN-only do not
    w1 = dict(w); w1["wo"] = w0["wo"]
    t2 = toks.copy(); t2[0] = (t2[0] + 1) % cfg.vocab
    assert np.array_equal(orc.full_logits(sh, w1, toks)[5:], orc.full_logits(sh, w1, t2)[5:])


def test_rmsnorm_closed_forms():
    x = np.random.default_rng(11).standard_normal(64) * 5
    h = orc.rmsnorm(x, np.ones(64), 1e-5)
    ms = np.mean(x ** 2)
    assert abs(np.mean(h ** 2) - ms / (ms + 1e-5)) < 1e-12
    assert np.abs(orc.rmsnorm(7.0 * x, np.ones(64), 0.0) - orc.rmsnorm(x, np.ones(64), 0.0)).max() < 1e-12


def test_greedy_takes_lowest_index_on_ties():
    assert orc.greedy(np.array([0.0, 3.0, -1.0, 3.0, 3.0])) == 1
    assert orc.greedy(np.array([2.0, 2.0])) == 0
    assert orc.top2_margin(np.array([0.0, 3.0, -1.0, 2.5])) == 0.5
    assert orc.top2_margin(np.array([3.0, 3.0, 1.0])) == 0.0


# ---------------------------------------------------------------- (d) interrupt injection

def test_inject_equals_prefill_of_concatenation():
    cfg, sh, w = _model()
    prompt = _tokens(13, cfg.vocab, seed=12)
    intr = _tokens(5, cfg.vocab, seed=13)
    res = orc.run_stream(sh, w, prompt, n_decode=9, events=[(4, intr)])
    stream = res["stream"]
    g = res["generated"]
    assert stream == list(prompt) + g[:4] + list(intr) + g[4:]
    ref = orc.full_logits(sh, w, stream)            # from scratch on the concatenated stream
    P = len(prompt)
    # logits each generated token was chosen from, at their stream positions
    for j in range(9):
        at = P + j - 1 + (len(intr) if j >= 4 else 0)
        assert np.abs(res["choose_logits"][j] - ref[at]).max() < 1e-9
        assert g[j] == int(np.argmax(ref[at]))
    assert np.abs(res["inject_logits"][4] - ref[P + 4 + len(intr) - 1]).max() < 1e-9
    assert np.abs(res["final_logits"] - ref[-1]).max() < 1e-9


def test_interrupts_may_be_batched_or_split():
    cfg, sh, w = _model()
    prompt = _tokens(10, cfg.vocab, seed=14)
    a, b = _tokens(4, cfg.vocab, seed=15), _tokens(7, cfg.vocab, seed=16)
    d1 = orc.CachedDecoder(sh, w); d1.prefill(prompt); d1.inject(a); d1.inject(b)
    d2 = orc.CachedDecoder(sh, w); d2.prefill(prompt); d2.inject(np.concatenate([a, b]))
    d3 = orc.CachedDecoder(sh, w); d3.prefill(prompt[:3]); d3.inject(prompt[3:])
    for t in np.concatenate([a, b]):
        d3.decode_step(forced=t)
    assert np.abs(d1.logits - d2.logits).max() < 1e-10
    assert np.abs(d3.logits - d2.logits).max() < 1e-10
    assert d1.tokens == d2.tokens == d3.tokens
    for l in range(cfg.n_layers):
        assert np.abs(d1.keys(l) - d3.keys(l)).max() < 1e-10
        assert np.abs(d1.values(l) - d2.values(l)).max() < 1e-10


def test_state_rules():
    cfg, sh, w = _model(n_layers=1)
    d = orc.CachedDecoder(sh, w)
    with pytest.raises(RuntimeError):
        d.decode_step()
    with pytest.raises(RuntimeError):
        d.inject([1])
    d.prefill([1, 2])
    with pytest.raises(RuntimeError):
        d.prefill([3])
    with pytest.raises(ValueError):
        d.append([])


def test_fp32_oracle_close_to_fp64():
    cfg, sh, w = _model()
    toks = _tokens(40, cfg.vocab, seed=17)
    a = orc.full_logits(sh, w, toks)
    b = orc.full_logits(sh, w, toks, dtype=np.float32)
    assert b.dtype == np.float32 and np.abs(a - b).max() < 2e-4 * np.abs(a).max()


def test_greedy_skips_banned_ids_and_keeps_the_lowest_index_on_ties():
    """The masked choice (token monitor, Sec. 5.1) against its definition written as a loop."""
    rng = np.random.default_rng(5)
    for trial in range(50):
        logits = rng.integers(-3, 4, size=40).astype(np.float64)        # many ties
        banned = list(rng.choice(40, size=int(rng.integers(0, 6)), replace=False))
        best, best_i = -np.inf, -1
        for i, v in enumerate(logits):
            if i in banned:
                continue
            if v > best:
                best, best_i = v, i
        assert orc.greedy(logits, banned) == best_i
    assert orc.greedy(np.array([1.0, 5.0, 5.0, 2.0])) == 1
    assert orc.greedy(np.array([1.0, 5.0, 5.0, 2.0]), [1]) == 2
    assert orc.greedy(np.array([1.0, 5.0, 5.0, 2.0]), [1, 2]) == 3
