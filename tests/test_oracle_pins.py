"""Pins for the CPU oracle: what the paper and the mathematics fix, checked on the CPU.

The oracle is compared with things other than itself: the Hugging Face Qwen3 model
(the architecture the paper builds on, Sec. 3.1), PyTorch library routines, brute-force
loops on tiny inputs, the paper's Fig. 3 walk-through, Eq. 7 and its printed values.
"""
import dataclasses
import math
import os

import numpy as np
import pytest
import torch

import dmtd_inputs as di
from oracle import dmtd_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")

TINY = di.ModelShape(4, 64, 4, 2, 16, 96, 50, dtype="fp32")


def make(shape=TINY, seed=3, std=0.2, gain_sigma=0.2, dtype=np.float64, **cfg_kw):
    blob = di.make_weight_blob(shape, seed=seed, std=std, gain_sigma=gain_sigma)
    cfg = O.OracleConfig(shape.n_layers, shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                         shape.intermediate, shape.vocab, shape.rms_eps, shape.rope_theta,
                         shape.tied_embeddings, **cfg_kw)
    return blob, cfg, O.unpack_weights(blob, cfg, dtype)


def run_forced(cfg, w, toks, P, tau, n_late, n, dtype=np.float64):
    o = O.DmtdOracle(cfg, w, 96, dtype)
    o.prefill(toks[:P], n_late)
    while o.n_tok < n:
        o.decode_cycle(tau, n_late, forced=toks[o.n_tok:o.n_tok + tau].tolist())
    return o


# ------------------------------------------------------------------ library pins

def hf_model(shape, w):
    from transformers import Qwen3Config, Qwen3ForCausalLM
    hc = Qwen3Config(vocab_size=shape.vocab, hidden_size=shape.hidden, intermediate_size=shape.intermediate,
                     num_hidden_layers=shape.n_layers, num_attention_heads=shape.n_q_heads,
                     num_key_value_heads=shape.n_kv_heads, head_dim=shape.head_dim, rms_norm_eps=shape.rms_eps,
                     rope_theta=shape.rope_theta, tie_word_embeddings=True, attention_bias=False,
                     max_position_embeddings=256, use_sliding_window=False)
    hc._attn_implementation = "eager"
    m = Qwen3ForCausalLM(hc).double().eval()
    sd = {"model.embed_tokens.weight": w["embed"], "lm_head.weight": w["embed"], "model.norm.weight": w["final_norm"]}
    names = {"attn_norm": "input_layernorm", "q": "self_attn.q_proj", "k": "self_attn.k_proj",
             "v": "self_attn.v_proj", "q_norm": "self_attn.q_norm", "k_norm": "self_attn.k_norm",
             "o": "self_attn.o_proj", "mlp_norm": "post_attention_layernorm", "gate": "mlp.gate_proj",
             "up": "mlp.up_proj", "down": "mlp.down_proj"}
    for l, lw in enumerate(w["layers"]):
        for k, hk in names.items():
            sd[f"model.layers.{l}.{hk}.weight"] = lw[k]
    missing = m.load_state_dict({k: torch.from_numpy(np.ascontiguousarray(v)) for k, v in sd.items()}, strict=True)
    assert not missing.missing_keys and not missing.unexpected_keys
    return m


@pytest.fixture(scope="module")
def hf_case():
    _, cfg, w = make()
    toks = di.make_prompts(TINY.vocab, 1, 24, seed=11)[0]
    m = hf_model(TINY, w)
    with torch.no_grad():
        ref = m(torch.from_numpy(toks.astype(np.int64))[None]).logits[0].numpy()
    return cfg, w, toks, m, ref


def test_vanilla_forward_matches_hf_qwen3(hf_case):
    """tau = 1 is ordinary decoding (Sec. 2.2), and the block is Qwen3's (Sec. 3.1)."""
    cfg, w, toks, _, ref = hf_case
    ours = O.vanilla_forward(toks, w, cfg)
    # the library keeps its norms and rotary tables in float32 even in a float64 model, hence 5e-6
    assert np.abs(ours - ref).max() < 5e-6 * np.abs(ref).max()


def test_incremental_tau1_matches_hf_cached_greedy(hf_case):
    cfg, w, toks, m, _ = hf_case
    P, G = 6, 12
    with torch.no_grad():
        step = m(torch.from_numpy(toks[:P].astype(np.int64))[None], use_cache=True)
        gen = [int(step.logits[0, -1].argmax())]
        while len(gen) < G:
            step = m(torch.tensor([[gen[-1]]]), past_key_values=step.past_key_values, use_cache=True)
            gen.append(int(step.logits[0, -1].argmax()))
    o = O.DmtdOracle(cfg, w, 64)
    out = [o.prefill(toks[:P])]
    while len(out) < G:
        out += o.decode_cycle(1, 1)
    assert out == gen


@pytest.mark.parametrize("mutation", ["rope_sign", "rope_interleaved", "gqa_mod", "norm_after_rope", "no_scale",
                                      "silu_on_up", "post_norm"])
def test_hf_pin_catches_planted_mistakes(hf_case, monkeypatch, mutation):
    """Each plausible slip in the block changes the logits far beyond the pin's tolerance."""
    cfg, w, toks, _, ref = hf_case
    if mutation == "rope_sign":
        orig = O.rope
        monkeypatch.setattr(O, "rope", lambda x, p, t: orig(x, -np.asarray(p), t))
    elif mutation == "rope_interleaved":
        def bad(x, positions, theta):
            hd = x.shape[-1]
            inv = theta ** (-2.0 * np.arange(hd // 2) / hd)
            ang = np.asarray(positions, float)[:, None] * inv[None]
            c, s = np.cos(ang)[:, None], np.sin(ang)[:, None]
            out = np.empty_like(x)
            out[..., 0::2] = x[..., 0::2] * c - x[..., 1::2] * s
            out[..., 1::2] = x[..., 1::2] * c + x[..., 0::2] * s
            return out
        monkeypatch.setattr(O, "rope", bad)
    elif mutation == "gqa_mod":
        orig = O.causal_attention

        def bad(q, qp, K, V):       # query heads read the wrong KV head
            return orig(q, qp, np.roll(K, 1, axis=1), np.roll(V, 1, axis=1))
        monkeypatch.setattr(O, "causal_attention", bad)
    elif mutation == "norm_after_rope":
        def bad(lw, X, positions, c):
            rows = X.shape[0]
            xh = O.rmsnorm(X, lw["attn_norm"], c.rms_eps)
            q = (xh @ lw["q"].T).reshape(rows, c.n_q_heads, c.head_dim)
            k = (xh @ lw["k"].T).reshape(rows, c.n_kv_heads, c.head_dim)
            v = (xh @ lw["v"].T).reshape(rows, c.n_kv_heads, c.head_dim)
            q = O.rmsnorm(O.rope(q, positions, c.rope_theta), lw["q_norm"], c.rms_eps)
            k = O.rmsnorm(O.rope(k, positions, c.rope_theta), lw["k_norm"], c.rms_eps)
            return q, k, v
        monkeypatch.setattr(O, "_project_qkv", bad)
    elif mutation == "no_scale":
        monkeypatch.setattr(O.math, "sqrt", lambda v: 1.0)
    elif mutation == "silu_on_up":
        def bad(lw, X, attn, c):
            a = X + attn.reshape(X.shape[0], -1) @ lw["o"].T
            ah = O.rmsnorm(a, lw["mlp_norm"], c.rms_eps)
            return a + ((ah @ lw["gate"].T) * O.silu(ah @ lw["up"].T)) @ lw["down"].T
        monkeypatch.setattr(O, "_finish_block", bad)
    elif mutation == "post_norm":
        def bad(lw, X, attn, c):
            a = X + attn.reshape(X.shape[0], -1) @ lw["o"].T
            ah = O.rmsnorm(a, lw["mlp_norm"], c.rms_eps)
            return ah + (O.silu(ah @ lw["gate"].T) * (ah @ lw["up"].T)) @ lw["down"].T
        monkeypatch.setattr(O, "_finish_block", bad)
    ours = O.vanilla_forward(toks, w, cfg)
    assert np.abs(ours - ref).max() > 1e-3 * np.abs(ref).max()


def test_primitives_match_torch_library_routines():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((5, 48))
    g = rng.standard_normal(48)
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x), (48,), torch.from_numpy(g), eps=1e-6).numpy()
    assert np.allclose(O.rmsnorm(x, g, 1e-6), ref, rtol=1e-12, atol=1e-14)
    t = rng.standard_normal(100) * 4
    assert np.allclose(O.silu(t), torch.nn.functional.silu(torch.from_numpy(t)).numpy(), rtol=1e-12, atol=1e-15)
    s = rng.standard_normal((7, 33)) * 5
    assert np.allclose(O.softmax_rows(s), torch.softmax(torch.from_numpy(s), -1).numpy(), rtol=1e-12, atol=1e-16)
    # grouped-query causal attention vs torch's scaled_dot_product_attention on a full sequence
    n, nh, nkv, hd = 9, 6, 2, 8
    q, k, v = rng.standard_normal((n, nh, hd)), rng.standard_normal((n, nkv, hd)), rng.standard_normal((n, nkv, hd))
    tq, tk, tv = (torch.from_numpy(a).permute(1, 0, 2)[None] for a in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(
        tq, tk.repeat_interleave(nh // nkv, dim=1), tv.repeat_interleave(nh // nkv, dim=1), is_causal=True)
    ref = ref[0].permute(1, 0, 2).numpy()
    assert np.allclose(O.causal_attention(q, np.arange(n), k, v), ref, rtol=1e-11, atol=1e-13)


def test_attention_with_ragged_positions_vs_loops():
    """Rows at arbitrary absolute positions against a longer cache: plain loops."""
    rng = np.random.default_rng(2)
    ctx, nh, nkv, hd = 13, 4, 2, 8
    K, V = rng.standard_normal((ctx, nkv, hd)), rng.standard_normal((ctx, nkv, hd))
    qpos = np.array([4, 9, 10, 12])
    q = rng.standard_normal((len(qpos), nh, hd))
    got = O.causal_attention(q, qpos, K, V)
    for i, p in enumerate(qpos):
        for j in range(nh):
            g = j // (nh // nkv)
            sc = [sum(q[i, j, e] * K[t, g, e] for e in range(hd)) / math.sqrt(hd) for t in range(p + 1)]
            m = max(sc)
            ex = [math.exp(s - m) for s in sc]
            tot = sum(ex)
            for e in range(hd):
                want = sum(ex[t] / tot * V[t, g, e] for t in range(p + 1))
                assert abs(got[i, j, e] - want) < 1e-12


# ---------------------------------------------------------------- closed forms

def test_rmsnorm_closed_forms():
    rng = np.random.default_rng(3)
    x = rng.standard_normal(64) * 3.0
    eps = 1e-6
    y = O.rmsnorm(x, np.ones(64), eps)
    ms = np.mean(x * x)
    assert abs(np.mean(y * y) - 1.0 / (1.0 + eps / ms)) < 1e-14
    assert np.allclose(O.rmsnorm(1000.0 * x, np.ones(64), 0.0), O.rmsnorm(x, np.ones(64), 0.0), rtol=1e-13)
    g = rng.standard_normal(64)
    assert np.allclose(O.rmsnorm(x, g, eps), y * g, rtol=1e-14)
    assert np.allclose(O.rmsnorm(np.full(8, 2.0), np.ones(8), 0.0), np.ones(8))


def test_rope_closed_forms():
    rng = np.random.default_rng(4)
    hd, theta = 16, 1e6
    x = rng.standard_normal((3, 2, hd))
    assert np.array_equal(O.rope(x, np.zeros(3), theta), x)
    y = O.rope(x, np.array([5, 17, 1000]), theta)
    assert np.allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-13)
    # as complex multiplication: pair (i, i+hd/2) is one complex number times exp(i p theta^(-2i/hd))
    z = x[..., : hd // 2] + 1j * x[..., hd // 2:]
    pos = np.array([5, 17, 1000])
    rot = np.exp(1j * pos[:, None] * theta ** (-2.0 * np.arange(hd // 2) / hd))[:, None, :]
    zz = z * rot
    assert np.allclose(y, np.concatenate([zz.real, zz.imag], -1), rtol=1e-12, atol=1e-13)
    # first pair turns by p radians exactly (frequency 1), last pair by p * theta^(-(hd-2)/hd)
    e = np.zeros((1, 1, hd)); e[0, 0, 0] = 1.0
    r = O.rope(e, np.array([2]), theta)[0, 0]
    assert abs(r[0] - math.cos(2.0)) < 1e-15 and abs(r[hd // 2] - math.sin(2.0)) < 1e-15
    # relative-position property of the scores
    q, k = rng.standard_normal((1, 1, hd)), rng.standard_normal((1, 1, hd))
    d1 = np.sum(O.rope(q, [40], theta) * O.rope(k, [33], theta))
    d2 = np.sum(O.rope(q, [107], theta) * O.rope(k, [100], theta))
    assert abs(d1 - d2) < 1e-11


def test_softmax_and_attention_special_cases():
    rng = np.random.default_rng(5)
    s = rng.standard_normal((4, 10)) * 30
    p = O.softmax_rows(s)
    assert np.allclose(p.sum(-1), 1.0, rtol=1e-14)
    assert np.allclose(O.softmax_rows(s + 1234.5), p, rtol=1e-10)
    assert np.allclose(O.softmax_rows(np.zeros((1, 8))), 1.0 / 8)
    # context of one key: output is that value; equal value rows: output is that row
    q = rng.standard_normal((1, 4, 8))
    K, V = rng.standard_normal((1, 2, 8)), rng.standard_normal((1, 2, 8))
    out = O.causal_attention(q, np.array([0]), K, V)
    assert np.allclose(out[0, :2], V[0, 0]) and np.allclose(out[0, 2:], V[0, 1])
    K = rng.standard_normal((6, 2, 8))
    V = np.broadcast_to(rng.standard_normal((1, 2, 8)), (6, 2, 8)).copy()
    out = O.causal_attention(q, np.array([5]), K, V)
    assert np.allclose(out[0, 0], V[0, 0], rtol=1e-13) and np.allclose(out[0, 3], V[0, 1], rtol=1e-13)
    # a key that scores far above the rest takes all the weight; keys after the query position are hidden
    K = np.zeros((5, 1, 4)); K[2, 0, 0] = 100.0; K[4, 0, 0] = 1000.0
    V = np.arange(20, dtype=float).reshape(5, 1, 4)
    qq = np.zeros((1, 1, 4)); qq[0, 0, 0] = 10.0
    assert np.allclose(O.causal_attention(qq, np.array([3]), K, V)[0, 0], V[2, 0])


def test_zero_output_projections_reduce_to_the_lm_head_of_the_embedding():
    """With W_o = W_d = 0 every block is the identity, so logits = E . norm(E[tok])."""
    blob, cfg, w = make()
    for lw in w["layers"]:
        lw["o"] = np.zeros_like(lw["o"])
        lw["down"] = np.zeros_like(lw["down"])
    toks = di.make_prompts(TINY.vocab, 1, 7, seed=2)[0]
    o = O.DmtdOracle(cfg, w, 32)
    o.prefill(toks[:4])
    o.decode_cycle(3, 2, forced=toks[4:7].tolist())
    E = w["embed"]
    for i, z in enumerate(o.step_logits):
        h = E[toks[3 + i]]
        want = E @ (h / math.sqrt(np.mean(h * h) + cfg.rms_eps) * w["final_norm"])
        assert np.allclose(z, want, rtol=1e-12, atol=1e-13)


def test_gqa_with_duplicated_kv_heads_equals_mha():
    sh_g = di.ModelShape(2, 32, 4, 2, 8, 48, 20, dtype="fp32")
    sh_m = dataclasses.replace(sh_g, n_kv_heads=4)
    _, cfg_g, wg = make(sh_g)
    cfg_m = dataclasses.replace(cfg_g, n_kv_heads=4)
    wm = {"embed": wg["embed"], "final_norm": wg["final_norm"], "lm_head": wg["lm_head"], "layers": []}
    for lw in wg["layers"]:
        m = dict(lw)
        for n in ("k", "v"):
            a = lw[n].reshape(2, 8, 32)
            m[n] = np.repeat(a, 2, axis=0).reshape(32, 32)
        wm["layers"].append(m)
    toks = di.make_prompts(20, 1, 10, seed=9)[0]
    assert np.allclose(O.vanilla_forward(toks, wg, cfg_g), O.vanilla_forward(toks, wm, cfg_m), rtol=1e-11, atol=1e-12)


# --------------------------------------------------------- the cycle machine

@pytest.mark.parametrize("literal", [False, True])
@pytest.mark.parametrize("tau,n_late", [(1, 1), (2, 1), (3, 1), (3, 2), (4, 3), (6, 2), (2, 4)])
def test_cycle_decode_equals_one_shot_masked_forward(tau, n_late, literal):
    """Incremental decoding with refilling (Sec. 2.2) == Eqs. 1-5 with the mask it realises."""
    _, cfg, w = make(full_pos_add_embed=literal)
    P, n = 5, 22
    toks = di.make_prompts(TINY.vocab, 1, n + 8, seed=5)[0]
    o = run_forced(cfg, w, toks, P, tau, n_late, n)
    assert o.tokens == toks[:o.n_tok].tolist()
    Z = np.stack(o.step_logits)
    ref = O.masked_forward(toks[:o.n_tok], O.inference_mask(o.n_tok, P, tau), n_late, w, cfg)
    assert np.abs(Z - ref[P - 1:P - 1 + len(Z)]).max() < 1e-11
    van = O.vanilla_forward(toks[:o.n_tok], w, cfg)
    same = np.abs(Z - van[P - 1:P - 1 + len(Z)]).max() < 1e-11
    assert same == ((tau == 1 or n_late == cfg.n_layers) and not literal)


def test_training_mask_of_eq3_is_the_inference_mask_for_aligned_prompts():
    """Eq. 3's m_i = [p_i mod tau == 0] coincides with the inference mask after the prompt when P-1 is a multiple of tau."""
    for tau in (2, 3, 4):
        P = 2 * tau + 1
        m = O.inference_mask(40, P, tau)
        eq3 = (np.arange(40) % tau == 0)
        assert np.array_equal(m[P:], eq3[P:])
    assert O.inference_mask(10, 1, 3).astype(int).tolist() == [1, 0, 0, 1, 0, 0, 1, 0, 0, 1]  # the pattern Eq. 3's text prints


def test_training_mask_is_eq3_and_prints_the_papers_pattern():
    """Sec. 2.1 prints the tau = 3 pattern [1,0,0,1,0,0,1,0,0,...] for Eq. 3."""
    assert O.training_mask(9, 3).astype(int).tolist() == [1, 0, 0, 1, 0, 0, 1, 0, 0]
    assert O.training_mask(5, 1).all()
    assert O.training_mask(6, 4).astype(int).tolist() == [1, 0, 0, 0, 1, 0]


def test_next_token_loss_of_eq6():
    """Eq. 6 against the library cross entropy, closed forms, and planted mistakes (unshifted or wrongly signed)."""
    rng = np.random.default_rng(5)
    n, V = 12, 37
    z = rng.normal(size=(n, V)) * 3.0
    toks = rng.integers(0, V, size=n)
    nll = O.next_token_nll(z, toks)
    assert nll.shape == (n - 1,)
    lib = torch.nn.functional.cross_entropy(torch.from_numpy(z[:-1]), torch.from_numpy(toks[1:].astype(np.int64)), reduction="none").numpy()
    assert np.abs(nll - lib).max() < 1e-12
    assert abs(O.next_token_loss(z, toks) - lib.mean()) < 1e-12
    # closed forms: equal logits give log V whatever the target; a shift of a row changes nothing;
    # a dominant target logit gives a loss near zero, a dominant wrong logit gives the gap
    assert np.abs(O.next_token_nll(np.zeros((4, V)), [0, 5, 9, 36]) - math.log(V)).max() < 1e-14
    assert np.abs(O.next_token_nll(z + 100.0 * rng.normal(size=(n, 1)), toks) - nll).max() < 1e-9
    big = np.zeros((2, V)); big[0, 7] = 50.0
    assert O.next_token_nll(big, [3, 7])[0] < 1e-15 + (V - 1) * math.exp(-50.0) * 1.0001
    assert abs(O.next_token_nll(big, [3, 8])[0] - 50.0) < 1e-12
    # the values survive large magnitudes (max subtraction)
    assert np.isfinite(O.next_token_nll(z * 1e3, toks)).all()
    # planted mistakes are visible to the library pin: target x_i instead of x_{i+1}; wrong sign
    unshifted = np.array([-np.log(np.exp(z[i] - z[i].max()).sum()) - z[i].max() + z[i][toks[i]] for i in range(n - 1)]) * -1.0
    assert np.abs(unshifted - lib).max() > 0.1
    assert np.abs(-nll - lib).max() > 0.1


def test_masked_forward_loss_uses_the_masked_logits():
    """Eq. 6 on the logits of Eqs. 1-5: with tau = 1 (every position full) it is the ordinary next-token loss of the
    Hugging Face model's logits; with tau > 1 it differs (in-cycle positions never saw the front layers)."""
    _, cfg, w = make()
    toks = di.make_prompts(TINY.vocab, 1, 24, seed=11)[0]
    z1 = O.masked_forward(toks, O.training_mask(len(toks), 1), 2, w, cfg)
    van = O.vanilla_forward(toks, w, cfg)
    assert np.abs(z1 - van).max() < 1e-11
    m = hf_model(TINY, w)
    with torch.no_grad():
        out = m(torch.from_numpy(toks.astype(np.int64))[None], labels=torch.from_numpy(toks.astype(np.int64))[None])
    assert abs(O.next_token_loss(z1, toks) - float(out.loss)) < 2e-6   # the library computes its loss in float32
    z3 = O.masked_forward(toks, O.training_mask(len(toks), 3), 2, w, cfg)
    assert abs(O.next_token_loss(z3, toks) - O.next_token_loss(z1, toks)) > 1e-3


def test_sampling_uniforms_are_the_generators_top_23_bits():
    u = O.sampling_uniforms(5, 2, 17, 1000)
    raw = di.raw_u64(5, (2 << 32) | 17, 0, 1000)
    assert np.array_equal(u * (1 << 23) - 0.5, (raw >> np.uint64(41)).astype(np.float64))
    assert u.min() > 0.0 and u.max() < 1.0
    assert np.array_equal(u.astype(np.float32).astype(np.float64), u)          # exactly representable in float32
    assert not np.array_equal(u, O.sampling_uniforms(5, 2, 18, 1000))           # another position: another draw
    assert not np.array_equal(u, O.sampling_uniforms(5, 3, 17, 1000))           # another sequence
    big = O.sampling_uniforms(1, 0, 0, 200000)
    assert abs(big.mean() - 0.5) < 3e-3 and abs(big.var() - 1.0 / 12.0) < 2e-3


def _draw_frequencies(z, temperature, top_k, n, mutate=None):
    counts = np.zeros(len(z))
    for pos in range(n):
        s = O.sampling_scores(z, temperature, top_k, 99, 0, pos)
        if mutate is not None:
            s = mutate(z, pos)
        counts[int(np.argmax(s))] += 1
    return counts


def test_sampling_draws_from_the_tempered_softmax_over_the_top_k():
    """Frequencies of 40000 draws (one per position counter) against softmax(z / T) over the k largest logits:
    Pearson's chi-square statistic below the 0.9999 quantile.  Planted mistakes (temperature multiplied instead of
    divided, restriction to the k smallest, no restriction) exceed it by far."""
    from scipy import stats
    z = np.array([2.0, 0.5, 1.5, -1.0, 0.0, 1.0, -2.0, 0.7])
    n = 40000
    for T, k in ((1.0, 0), (0.7, 0), (1.6, 5), (0.5, 3)):
        keep = np.ones(len(z), bool) if k == 0 else z >= np.sort(z)[len(z) - k]
        p = np.where(keep, np.exp(z / T), 0.0)
        p /= p.sum()
        counts = _draw_frequencies(z, T, k, n)
        assert counts[~keep].sum() == 0
        chi2 = (((counts - n * p) ** 2)[keep] / (n * p[keep])).sum()
        assert chi2 < stats.chi2.ppf(0.9999, keep.sum() - 1), (T, k, chi2)
    T, k = 0.5, 3
    keep = z >= np.sort(z)[len(z) - k]
    p = np.where(keep, np.exp(z / T), 0.0)
    p /= p.sum()
    limit = stats.chi2.ppf(0.9999, len(z) - 1)

    def chi2_of(counts):
        exp = np.maximum(n * p, 1e-9)
        return (((counts - n * p) ** 2) / exp).sum()

    g = lambda pos: -np.log(-np.log(O.sampling_uniforms(99, 0, pos, len(z))))
    wrong_temperature = _draw_frequencies(z, T, k, n, lambda zz, pos: np.where(keep, zz * T + g(pos), -np.inf))
    smallest_k = _draw_frequencies(z, T, k, n, lambda zz, pos: np.where(zz <= np.sort(zz)[k - 1], zz / T + g(pos), -np.inf))
    unrestricted = _draw_frequencies(z, T, k, n, lambda zz, pos: zz / T + g(pos))
    for wrong in (wrong_temperature, smallest_k, unrestricted):
        assert chi2_of(wrong) > 10 * limit


def test_sampling_special_cases_and_the_cycle_machine():
    """top_k = 1 and temperature -> 0 are greedy selection; k >= V is no restriction; ties at the k-th logit stay in;
    the cycle machine draws at the emitting row's position and sequences draw independently."""
    rng = np.random.default_rng(3)
    z = rng.normal(size=50) * 2
    for pos in range(20):
        assert O.sample_token(z, 1.3, 1, 7, 0, pos) == int(np.argmax(z))
        assert O.sample_token(z, 1e-4, 0, 7, 0, pos) == int(np.argmax(z))
        assert O.sample_token(z, 0.9, 50, 7, 0, pos) == O.sample_token(z, 0.9, 0, 7, 0, pos) == O.sample_token(z, 0.9, 80, 7, 0, pos)
    tied = np.array([1.0, 3.0, 2.0, 2.0, 0.0])
    assert np.isfinite(O.sampling_scores(tied, 1.0, 2, 0, 0, 0)).tolist() == [False, True, True, True, False]
    _, cfg, w = make()
    toks = di.make_prompts(TINY.vocab, 1, 9, seed=4)[0]
    runs = []
    for seq in (0, 0, 1):
        o = O.DmtdOracle(cfg, w, 64)
        o.set_sampling(1.5, 8, seed=11, seq=seq)
        out = [o.prefill(toks)]
        assert out[0] == O.sample_token(o.last_logits, 1.5, 8, 11, seq, len(toks) - 1)
        for _ in range(5):
            got = o.decode_cycle(3, 2)
            assert got[-1] == O.sample_token(o.last_logits, 1.5, 8, 11, seq, o.n_tok - 1)
            out += got
        runs.append(out)
    assert runs[0] == runs[1] and runs[0] != runs[2]
    greedy = O.DmtdOracle(cfg, w, 64)
    g_out = [greedy.prefill(toks)] + sum((greedy.decode_cycle(3, 2) for _ in range(5)), [])
    assert g_out != runs[0]
    o = O.DmtdOracle(cfg, w, 64)
    o.set_sampling(0.0)
    assert [o.prefill(toks)] + sum((o.decode_cycle(3, 2) for _ in range(5)), []) == g_out


def test_fig3_schedule():
    want = []
    for line in open(os.path.join(GOLDEN, "fig3_schedule.txt")):
        if line.strip() and not line.startswith("#"):
            f = line.split()
            want.append((int(f[0]), f[1], [int(x) for x in f[2:]]))
    _, cfg, w = make()
    o = O.DmtdOracle(cfg, w, 32)
    o.prefill([1, 2, 3, 4, 5])
    o.decode_cycle(3, 1)
    o.decode_cycle(3, 1)
    o.decode_cycle(3, 1, max_new=1)
    got = [(i + 1, grp, pos) for i, passes in enumerate(o.trace) for grp, pos in passes]
    assert got == want
    assert o.n_emitted == 2 + 3 + 1      # the first cycle's first token came from prefill


def test_plt_closed_form_and_printed_values():
    for line in open(os.path.join(GOLDEN, "plt_values.txt")):
        if line.strip() and not line.startswith("#"):
            L, Ld, tau, plt, inv = line.split()
            val = O.plt_closed_form(int(L), int(Ld), int(tau))
            assert abs(val - float(plt)) < 0.005
            assert abs(1.0 / val - float(inv)) < 0.005
    assert abs(O.plt_closed_form(36, 8, 3) - (1 / 3 + 2 / 3 * 8 / 36)) < 1e-15   # second form of Eq. 7


@pytest.mark.parametrize("tau,n_late", [(3, 1), (2, 2), (4, 1)])
def test_layer_visit_counters_match_eq7_and_total_load(tau, n_late):
    _, cfg, w = make()
    L = cfg.n_layers
    o = O.DmtdOracle(cfg, w, 64)
    o.prefill([3, 1, 4, 1, 5])
    o.decode_cycle(tau, n_late)                      # finishes cycle 1 (tau - 1 tokens)
    g0, e0 = o.gen_layer_visits, o.n_emitted
    cycles = 5
    for _ in range(cycles):
        assert len(o.decode_cycle(tau, n_late)) == tau
    gen = o.gen_layer_visits - g0
    assert gen / ((o.n_emitted - e0) * L) == pytest.approx(O.plt_closed_form(L, n_late, tau), abs=1e-15)
    # total load equals the vanilla model's (Sec. 2.2): every consumed token passes every layer once,
    # except the tau - 1 newest tokens, which still wait for their refill
    consumed_after_prefill = o.n_tok - 5
    total = o.gen_layer_visits + o.refill_layer_visits
    assert total == consumed_after_prefill * L - (o.n_tok - o.n_front) * (L - n_late)


# --------------------------------------------------------- ExDy variant (Sec. 2.1 / Sec. 3.3)

SIX = di.ModelShape(6, 64, 4, 2, 16, 96, 50, dtype="fp32")


def run_forced_exdy(cfg, w, toks, P, tau, n_late, n_early, n):
    o = O.DmtdOracle(cfg, w, 96)
    o.prefill(toks[:P], n_late, n_early)
    while o.n_tok < n:
        o.decode_cycle(tau, n_late, forced=toks[o.n_tok:o.n_tok + tau].tolist(), n_early=n_early)
    return o


@pytest.mark.parametrize("literal", [False, True])
@pytest.mark.parametrize("tau,n_early,n_late", [(3, 1, 1), (3, 2, 2), (2, 1, 3), (4, 3, 1), (3, 0, 2), (1, 2, 2), (5, 2, 1)])
def test_exdy_cycle_decode_equals_one_shot_masked_forward(tau, n_early, n_late, literal):
    """The incremental machine with stored encoding outputs and thinking-layer refill == Eqs. 1-5 with h_enc
    in place of h_emb (the last paragraph before Eq. 5), for both readings of Eq. 4."""
    _, cfg, w = make(SIX, full_pos_add_embed=literal)
    P, n = 5, 23
    toks = di.make_prompts(SIX.vocab, 1, n + 8, seed=6)[0]
    o = run_forced_exdy(cfg, w, toks, P, tau, n_late, n_early, n)
    assert o.tokens == toks[:o.n_tok].tolist()
    Z = np.stack(o.step_logits)
    ref = O.masked_forward(toks[:o.n_tok], O.inference_mask(o.n_tok, P, tau), n_late, w, cfg, n_early=n_early)
    assert np.abs(Z - ref[P - 1:P - 1 + len(Z)]).max() < 1e-11
    # the variant changes the function unless nothing is skipped (the literal reading adds h_enc at full positions too)
    plain = O.masked_forward(toks[:o.n_tok], O.inference_mask(o.n_tok, P, tau), n_late, w, cfg, n_early=0)
    differs = np.abs(ref - plain).max() > 1e-6
    assert differs == (n_early > 0 and (tau > 1 or literal))


@pytest.mark.parametrize("tau", [2, 3, 5])
@pytest.mark.parametrize("n_early", [1, 3, 5])
def test_exdy_without_thinking_layers_is_ordinary_decoding(tau, n_early):
    """x + y = L: every token passes every layer in its own step, nothing is left to refill, so any
    cycle length reproduces the ordinary causal forward (default reading of Eq. 4)."""
    _, cfg, w = make(SIX)
    n_late = SIX.n_layers - n_early
    P, n = 4, 18
    toks = di.make_prompts(SIX.vocab, 1, n + 8, seed=7)[0]
    o = run_forced_exdy(cfg, w, toks, P, tau, n_late, n_early, n)
    van = O.vanilla_forward(toks[:o.n_tok], w, cfg)
    Z = np.stack(o.step_logits)
    assert np.abs(Z - van[P - 1:P - 1 + len(Z)]).max() < 1e-11
    assert o.refill_layer_visits == 0
    # and the caches equal those of one causal pass over the whole string
    ref = O.DmtdOracle(cfg, w, 96)
    ref.prefill(toks[:o.n_tok])
    for l in range(SIX.n_layers):
        assert np.abs(o.K[l][:o.n_tok] - ref.K[l][:o.n_tok]).max() < 1e-12
        assert np.abs(o.V[l][:o.n_tok] - ref.V[l][:o.n_tok]).max() < 1e-12


def test_exdy_n_early_zero_is_the_plain_method_bit_for_bit():
    _, cfg, w = make(SIX)
    toks = di.make_prompts(SIX.vocab, 1, 40, seed=8)[0]
    a = run_forced_exdy(cfg, w, toks, 5, 3, 2, 0, 20)
    b = run_forced(cfg, w, toks, 5, 3, 2, 20)
    assert all(np.array_equal(x, y) for x, y in zip(a.step_logits, b.step_logits))
    assert a.trace == b.trace and a.gen_layer_visits == b.gen_layer_visits


def test_exdy_schedule_counters_and_refill_span():
    """Layers per generated token follow Eq. 7 with L_d = x + y; the refill rows traverse only the thinking
    layers; the total load stays that of ordinary decoding (Sec. 2.2)."""
    _, cfg, w = make(SIX)
    L, tau, x, y = SIX.n_layers, 3, 2, 1
    o = O.DmtdOracle(cfg, w, 64)
    o.prefill([3, 1, 4, 1, 5])
    o.decode_cycle(tau, y, n_early=x)
    g0, e0 = o.gen_layer_visits, o.n_emitted
    for _ in range(4):
        assert len(o.decode_cycle(tau, y, n_early=x)) == tau
    assert (o.gen_layer_visits - g0) / ((o.n_emitted - e0) * L) == pytest.approx(O.plt_closed_form(L, y, tau, x), abs=1e-15)
    assert O.plt_closed_form(L, y, tau, x) == pytest.approx((6 + 2 * 3) / 18)
    consumed = o.n_tok - 5
    assert o.gen_layer_visits + o.refill_layer_visits == consumed * L - (o.n_tok - o.n_front) * (L - x - y)
    # a full pass of a later cycle: newest token through the encoding layers, 3 rows through the thinking layers,
    # newest token through the decoding layers (Fig. 3 with the encoding block moved to the tokens' own passes)
    full = [t for t in o.trace if any(g == "front" for g, _ in t)][-1]
    p = full[-1][1][0]
    assert full == [("enc", [p]), ("front", [p - 2, p - 1, p]), ("late", [p])]
    late = o.trace[-1]
    assert late == [("enc", [o.n_tok - 1]), ("late", [o.n_tok - 1])]


@pytest.mark.parametrize("literal", [False, True])
def test_exdy_with_identity_upper_layers_equals_the_library_model_of_the_encoding_layers(literal):
    """A pin of the ExDy variant outside the oracle: with W_o = W_d = 0 in every thinking and decoding layer those layers are
    the identity, every token still passes the x encoding layers in its own step with its full causal context, and
    h_masked = h_enc (Sec. 2.1, before Eq. 5), so the logits at EVERY position - full or inside a cycle - are those of
    the Hugging Face Qwen3 model made of the encoding layers alone.  The plain method (x = 0) would give the LM head of
    the raw embedding at in-cycle positions instead (pinned above).  Under the literal reading of Eq. 4 full positions
    feed h_enc + h_think = 2 h_enc, which the final RMSNorm maps back up to its epsilon."""
    x, y, tau, P, n = 2, 1, 3, 5, 20
    _, cfg, w = make(full_pos_add_embed=literal)
    for lw in w["layers"][x:]:
        lw["o"] = np.zeros_like(lw["o"])
        lw["down"] = np.zeros_like(lw["down"])
    toks = di.make_prompts(TINY.vocab, 1, 24, seed=11)[0]
    enc_only = dict(w, layers=w["layers"][:x])
    m = hf_model(dataclasses.replace(TINY, n_layers=x), enc_only)
    with torch.no_grad():
        ref = m(torch.from_numpy(toks.astype(np.int64))[None]).logits[0].numpy()
    o = run_forced_exdy(cfg, w, toks, P, tau, y, x, n)
    assert len(o.step_logits) >= n - P + 1
    in_cycle = 0
    for i, z in enumerate(o.step_logits):                 # step i emits from position P - 1 + i
        pos = P - 1 + i
        tol = (2e-4 if literal else 5e-6) * np.abs(ref[pos]).max()
        assert np.abs(z - ref[pos]).max() < tol, (pos, np.abs(z - ref[pos]).max())
        in_cycle += (pos - (P - 1)) % tau != 0
        # the plain method's in-cycle logits (LM head of the raw embedding) are far away: the pin can tell the two apart
        E = w["embed"]
        h = E[toks[pos]]
        emb_only = E @ (h / math.sqrt(np.mean(h * h) + cfg.rms_eps) * w["final_norm"])
        assert np.abs(emb_only - ref[pos]).max() > 1e-2 * np.abs(ref[pos]).max()
    assert in_cycle >= 8


def test_literal_eq4_with_identity_decoding_layers_against_the_library_hidden_state():
    """A pin of the literal reading of Eq. 4 outside the oracle: with W_o = W_d = 0 in the decoding layers they are the
    identity, so a full position's logits are E . norm(h_emb + h_think) with h_think the hidden state the Hugging Face
    model reports after the front layers, and an in-cycle position's logits are E . norm(h_emb)."""
    y, tau, P, n = 2, 3, 5, 20
    F = TINY.n_layers - y
    _, cfg, w = make(full_pos_add_embed=True)
    for lw in w["layers"][F:]:
        lw["o"] = np.zeros_like(lw["o"])
        lw["down"] = np.zeros_like(lw["down"])
    toks = di.make_prompts(TINY.vocab, 1, 24, seed=11)[0]
    m = hf_model(TINY, w)
    with torch.no_grad():
        h_think = m(torch.from_numpy(toks.astype(np.int64))[None], output_hidden_states=True).hidden_states[F][0].numpy()
    o = run_forced(cfg, w, toks, P, tau, y, n)
    E = w["embed"]

    def head(h):
        return E @ (h / np.sqrt(np.mean(h * h) + cfg.rms_eps) * w["final_norm"])

    n_full = n_in = 0
    for i, z in enumerate(o.step_logits):
        pos = P - 1 + i
        full = (pos - (P - 1)) % tau == 0
        want = head(E[toks[pos]] + h_think[pos]) if full else head(E[toks[pos]])
        assert np.abs(z - want).max() < 5e-6 * np.abs(want).max(), (pos, full)
        if full:                                          # and the default reading's value is far away
            assert np.abs(head(h_think[pos]) - want).max() > 1e-2 * np.abs(want).max()
        n_full += full
        n_in += not full
    assert n_full >= 4 and n_in >= 8


def test_exdy_plt_against_hand_counted_cycles():
    """Eq. 7 with L_d = x + y against layer counts written out by hand (tests/golden/plt_exdy_hand_count.txt): the
    closed form, and the cycle machine's own counter on a model of that depth where it is small enough to run."""
    n_rows = 0
    for line in open(os.path.join(GOLDEN, "plt_exdy_hand_count.txt")):
        if line.startswith("#") or not line.strip():
            continue
        left, mid, right = [part.split() for part in line.split("|")]
        L, x, y, tau = map(int, left)
        per_token = list(map(int, mid))
        num, den = map(int, right)
        assert len(per_token) == tau and per_token[0] == L and all(v == x + y for v in per_token[1:])
        assert sum(per_token) == num and den == tau * L
        assert O.plt_closed_form(L, y, tau, x) == pytest.approx(num / den, abs=1e-15)
        n_rows += 1
        if L == 6:
            _, cfg, w = make(SIX)
            o = O.DmtdOracle(cfg, w, 64)
            o.prefill([3, 1, 4, 1, 5])
            o.decode_cycle(tau, y, n_early=x)                     # the rest of cycle 1
            g0 = o.gen_layer_visits
            for _ in range(3):
                o.decode_cycle(tau, y, n_early=x)
            assert o.gen_layer_visits - g0 == 3 * num
    assert n_rows >= 8


def test_exdy_state_errors():
    _, cfg, w = make(SIX)
    o = O.DmtdOracle(cfg, w, 64)
    o.prefill([1, 2, 3])
    with pytest.raises(ValueError):
        o.decode_cycle(3, 2, n_early=5)               # x + y > L
    o.decode_cycle(3, 2, n_early=1)                   # leaves tokens awaiting refill
    with pytest.raises(RuntimeError):
        o.decode_cycle(3, 2, n_early=2)               # their stored encoding outputs belong to x = 1
    o.decode_cycle(3, 2, max_new=1, n_early=1)        # the full step closes the gap
    assert o.n_front == o.n_tok
    o.decode_cycle(3, 2, n_early=2)


def test_exdy_catches_planted_mistakes(monkeypatch):
    """The masked-forward pin fails if the in-cycle tokens read the embedding instead of the encoding output,
    or if the refill starts from the embeddings again."""
    _, cfg, w = make(SIX)
    toks = di.make_prompts(SIX.vocab, 1, 40, seed=9)[0]
    P, tau, x, y = 5, 3, 2, 2
    good = run_forced_exdy(cfg, w, toks, P, tau, y, x, 20)
    ref = O.masked_forward(toks[:good.n_tok], O.inference_mask(good.n_tok, P, tau), y, w, cfg, n_early=x)
    Zg = np.stack(good.step_logits)
    assert np.abs(Zg - ref[P - 1:P - 1 + len(Zg)]).max() < 1e-11
    orig = O.DmtdOracle._full_step

    def refill_from_embeddings(self, n_late, n_early=0):
        self.pend_enc = [self.w["embed"][t] for t in self.tokens[self.n_front:self.n_tok]]
        return orig(self, n_late, n_early)
    monkeypatch.setattr(O.DmtdOracle, "_full_step", refill_from_embeddings)
    bad = run_forced_exdy(cfg, w, toks, P, tau, y, x, 20)
    Zb = np.stack(bad.step_logits)
    assert np.abs(Zb - ref[P - 1:P - 1 + len(Zb)]).max() > 1e-6


def test_refill_row_by_row_equals_refill_as_one_batch():
    """Feeding the pending tokens through the front layers one at a time gives the same caches and logits."""
    _, cfg, w = make()
    toks = di.make_prompts(TINY.vocab, 1, 16, seed=8)[0]
    a = run_forced(cfg, w, toks, 4, 3, 2, 10)
    b = O.DmtdOracle(cfg, w, 96)
    b.prefill(toks[:4])
    F = cfg.n_layers - 2
    # same schedule, but the front layers are advanced one position at a time with tau = 1-style rows
    for p in range(4, 10):
        full = (p - 3) % 3 == 0
        if full:
            for pp in range(b.n_front, p + 1):
                h = w["embed"][toks[pp]][None]
                for l in range(F):
                    h = b._block(l, h, np.array([pp]))
            b.n_front = p + 1
        else:
            h = w["embed"][toks[p]][None]
        for l in range(F, cfg.n_layers):
            h = b._block(l, h, np.array([p]))
        z = O.lm_logits(h[0], w, cfg)
        assert np.abs(z - a.step_logits[p - 3]).max() < 1e-11
    for l in range(cfg.n_layers):
        assert np.abs(a.K[l][:10] - b.K[l][:10]).max() < 1e-12


def test_changing_tau_between_cycles_and_truncated_cycles():
    _, cfg, w = make()
    toks = di.make_prompts(TINY.vocab, 1, 40, seed=12)[0]
    o = O.DmtdOracle(cfg, w, 96)
    o.prefill(toks[:6])
    mask = [True] * 6
    plan = [(3, 0), (2, 0), (4, 2), (4, 0), (1, 0), (5, 3), (5, 0)]   # (tau, max_new)
    for tau, cap in plan:
        before = o.phase
        got = o.decode_cycle(tau, 2, max_new=cap, forced=toks[o.n_tok:o.n_tok + tau].tolist())
        starts_full = before >= tau or before == 0
        mask += ([True] if starts_full else []) + [False] * (len(got) - (1 if starts_full else 0))
    Z = np.stack(o.step_logits)
    ref = O.masked_forward(toks[:o.n_tok], np.array(mask[:o.n_tok]), 2, w, cfg)
    assert np.abs(Z - ref[5:5 + len(Z)]).max() < 1e-11
    with pytest.raises(RuntimeError):
        o.decode_cycle(5, 3)          # n_late may not change while tokens await refill


def test_state_errors():
    _, cfg, w = make()
    o = O.DmtdOracle(cfg, w, 8)
    with pytest.raises(RuntimeError):
        o.decode_cycle(2, 1)
    o.prefill([1, 2, 3, 4, 5, 6])
    with pytest.raises(ValueError):
        o.decode_cycle(0, 1)
    with pytest.raises(ValueError):
        o.decode_cycle(2, 5)
    o.decode_cycle(2, 1)
    o.decode_cycle(1, 1)
    with pytest.raises(OverflowError):
        o.decode_cycle(1, 1)


def test_float32_mode_stays_close_to_float64():
    sh = di.WORKLOADS["C1"].shape
    blob, cfg, w64 = make(sh, seed=0, std=0.02, gain_sigma=0.0)
    w32 = O.unpack_weights(blob, cfg, np.float32)
    toks = di.make_prompts(sh.vocab, 1, 48, seed=1)[0]
    a = run_forced(cfg, w64, toks, 32, 2, 1, 40)
    b = run_forced(cfg, w32, toks, 32, 2, 1, 40, dtype=np.float32)
    za, zb = np.stack(a.step_logits), np.stack(b.step_logits)
    assert zb.dtype == np.float32
    assert np.abs(za - zb).max() / np.abs(za).max() < 2e-5
