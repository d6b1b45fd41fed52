"""GPU parity of token selection by sampling (temperature, top-k) and of cycle lengths that change per cycle.

A draw is the argmax of z_v / T - log(-log(u_v)) over the top-k logits: floating point decides an integer.  Two levels:
(1) decision level: the oracle's sampler applied to the very logits the GPU reports (float32 values, widened) must pick
    the GPU's token wherever its two best scores are more than 1e-3 apart (the GPU's scores differ from the oracle's by
    float32 rounding of z / T and of the logarithms, about 1e-6 of the scores' size); the top-k set is decided on the
    same float32 values on both sides, by exact comparisons, so it is identical;
(2) end to end: engine and oracle run the same seeded model teacher-forced, each sampling from its own logits; tokens
    must agree wherever the oracle's draw beats, by more than the greedy tests' 0.05, every other score in the top-k
    set and every entry whose logit lies within 0.05 of the set's boundary; logits obey the usual tolerance.
"""
import numpy as np
import pytest

import dmtd_inputs as di
import paper_2510_11958_amd as pkg
from oracle import dmtd_oracle as O
from parity_util import MARGIN, Pair, norm_err

pytestmark = pytest.mark.gpu

TOL_F32, TOL_BF16 = 1e-4, 2e-2


def forced_string(vocab, batch, prompts, total_len, seed=1001):
    cont = di.make_continuation(vocab, batch, total_len, seed=seed)
    return [np.concatenate([prompts[b], cont[b]])[:total_len] for b in range(batch)]


def top2_gap(s):
    f = np.sort(s[np.isfinite(s)])
    return float(f[-1] - f[-2]) if len(f) > 1 else np.inf


def robust_margin(z, scores, T, k, seed, b, pos):
    """How far the oracle's draw is from changing under small logit errors: its score minus the best other score inside
    the top-k set and minus the best score of any entry whose logit lies within MARGIN of the k-th largest (whose
    membership a small error could flip); -inf if the draw itself is such an entry."""
    win = int(np.argmax(scores))
    rest = np.delete(scores, win)
    margin = scores[win] - rest.max()
    if 0 < k < len(z):
        kth = np.sort(z)[len(z) - k]
        near = np.abs(z - kth) < MARGIN
        if near[win]:
            return -np.inf
        free = O.sampling_scores(z, T, 0, seed, b, pos)          # the same draw without the restriction
        if near.any():
            margin = min(margin, scores[win] - free[near].max())
    return float(margin)


CASES = {
    # name: (shape, batch, prompt_len, steps, tau, n_late, temperature, top_k, seed)
    "f32_t1_all": (di.ModelShape(3, 64, 4, 2, 64, 96, 61, dtype="fp32"), 2, 6, 24, 3, 1, 1.0, 0, 5),
    "f32_t07_k8": (di.ModelShape(3, 72, 2, 2, 64, 104, 93, dtype="fp32"), 1, 7, 24, 4, 2, 0.7, 8, 2**40 + 3),
    "f32_t2_k50_of_50": (di.ModelShape(3, 64, 2, 1, 64, 96, 50, dtype="fp32"), 1, 5, 16, 2, 1, 2.0, 50, 1),
    "bf16_t08_k40": (di.ModelShape(4, 256, 8, 2, 128, 512, 1000, dtype="bf16"), 3, 40, 18, 3, 2, 0.8, 40, 77),
    # the benchmark models' vocabulary (151936 entries: 148 full strides of the selection kernel's 1024 threads and a ragged one)
    "bf16_full_vocab_k50": (di.ModelShape(2, 64, 2, 1, 64, 128, 151936, dtype="bf16"), 2, 12, 10, 3, 1, 0.8, 50, 123),
    "bf16_t13_all_ragged_vocab": (di.ModelShape(3, 128, 4, 2, 64, 256, 515, dtype="bf16"), 1, 30, 16, 2, 1, 1.3, 0, 9),
}


@pytest.mark.parametrize("use_graphs", [True, False])
@pytest.mark.parametrize("name", list(CASES))
def test_sampled_decoding_teacher_forced(name, use_graphs):
    sh, batch, P, steps, tau, n_late, T, k, seed = CASES[name]
    tol = TOL_F32 if sh.dtype == "fp32" else TOL_BF16
    blob = di.make_weight_blob(sh, seed=13, std=0.08 if sh.dtype == "fp32" else 0.05, gain_sigma=0.2)
    prompts = di.make_prompts(sh.vocab, batch, P, seed=6)
    toks = forced_string(sh.vocab, batch, prompts, P + steps + 2)
    p = Pair(sh, blob, P + steps + 8, batch=batch, use_graphs=use_graphs)
    p.eng.set_sampling(T, k, seed)
    for b, o in enumerate(p.orcs):
        o.set_sampling(T, k, seed, seq=b)
    stats = {"decision": 0, "end_to_end": 0, "differs_from_greedy": 0}

    def check(gpu_tokens, pos):
        z = p.eng.logits()
        for b, o in enumerate(p.orcs):
            assert norm_err(z[b], o.last_logits) < tol
            # (1) the oracle's sampler on the GPU's own logits
            s_gpu = O.sampling_scores(z[b].astype(np.float64), T, k, seed, b, pos)
            assert np.isfinite(s_gpu[int(gpu_tokens[b])])             # the draw lies inside the top-k set
            if top2_gap(s_gpu) > 1e-3:
                assert int(gpu_tokens[b]) == int(np.argmax(s_gpu)), (b, pos)
                stats["decision"] += 1
            # (2) against the oracle's own model and draw
            if robust_margin(o.last_logits.astype(np.float64), o.last_scores, T, k, seed, b, pos) > MARGIN:
                assert int(gpu_tokens[b]) == int(np.argmax(o.last_scores)), (b, pos)
                stats["end_to_end"] += 1
            stats["differs_from_greedy"] += int(gpu_tokens[b]) != int(np.argmax(z[b]))

    first = p.eng.prefill(prompts)
    for b, o in enumerate(p.orcs):
        o.prefill(prompts[b])
    check(first, P - 1)
    for _ in range(steps):
        nt = p.eng.state()["n_tok"]
        f = np.stack([toks[b][nt:nt + 1] for b in range(batch)])
        out = p.eng.decode_cycle(tau, n_late, max_new=1, forced=f)
        for b, o in enumerate(p.orcs):
            o.decode_cycle(tau, n_late, max_new=1, forced=f[b].tolist())
        check(out[:, 0], nt)
    assert stats["decision"] >= (steps + 1) * batch * 0.9 and stats["end_to_end"] >= (steps + 1) * batch * 0.3, stats
    assert stats["differs_from_greedy"] > 0, stats        # the draws are not the greedy choice in disguise
    print(f"{name} graphs={use_graphs}: {stats}")


def test_sampling_is_reproducible_batch_independent_and_switchable():
    sh = di.ModelShape(3, 64, 4, 2, 64, 96, 61, dtype="fp32")
    blob = di.make_weight_blob(sh, seed=13, std=0.08, gain_sigma=0.2)
    prompts = di.make_prompts(sh.vocab, 3, 6, seed=6)
    prompts[2] = prompts[0]                                 # the same prompt at two batch indices
    eng = pkg.Engine(pkg.ModelConfig(sh.n_layers, sh.hidden, sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.intermediate,
                                     sh.vocab, dtype="fp32", max_seq_len=64, max_batch=3), blob)

    def run(temperature, top_k, seed):
        eng.reset()
        eng.set_sampling(temperature, top_k, seed)
        out = [eng.prefill(prompts)[:, None]]
        for _ in range(6):
            out.append(eng.decode_cycle(3, 1))
        return np.concatenate(out, 1)

    a, a2, other_seed, greedy = run(1.0, 10, 4), run(1.0, 10, 4), run(1.0, 10, 5), run(0.0, 0, 0)
    assert np.array_equal(a, a2) and not np.array_equal(a, other_seed) and not np.array_equal(a, greedy)
    assert not np.array_equal(a[0], a[2])                   # the sequence index enters the counter: independent draws
    assert np.array_equal(run(0.9, 1, 4), greedy)           # top_k = 1 is the greedy choice
    assert np.array_equal(greedy[0], greedy[2])
    for bad in ((float("nan"), 0), (1.0, -1)):
        with pytest.raises(pkg.DmtdError) as e:
            eng.set_sampling(bad[0], bad[1], 0)
        assert e.value.code == pkg.DMTD_EINVAL


def test_cycle_length_changes_every_cycle_with_sampling():
    """Table 5's setting taken further: the cycle length changes from one cycle to the next (2..6, then 1), with whole-cycle
    calls, graphs on, free running on sampled tokens; every call's last logits and the scheduler state against the oracle,
    which is fed the tokens the GPU drew."""
    sh = di.ModelShape(4, 64, 4, 2, 64, 96, 61, dtype="fp32")
    blob = di.make_weight_blob(sh, seed=5, std=0.08, gain_sigma=0.2)
    prompts = di.make_prompts(sh.vocab, 2, 6, seed=4)
    p = Pair(sh, blob, 96, batch=2)
    p.eng.set_sampling(1.1, 12, 21)
    first = p.eng.prefill(prompts)
    for b, o in enumerate(p.orcs):
        o.prefill(prompts[b])
    last = first
    for tau in (3, 2, 6, 4, 5, 1, 3, 6, 2):
        out = p.eng.decode_cycle(tau, 2)
        z = p.eng.logits()
        for b, o in enumerate(p.orcs):
            # the oracle consumes the GPU's tokens: step i's input is the token drawn before it
            inputs = [int(last[b])] + [int(t) for t in out[b, :-1]]
            o.decode_cycle(tau, 2, forced=inputs)
            assert norm_err(z[b], o.last_logits) < TOL_F32
        s = p.eng.state()
        assert (s["n_tok"], s["n_front"], s["phase"]) == (p.orcs[0].n_tok, p.orcs[0].n_front, p.orcs[0].phase)
        last = out[:, -1]
    p.compare_kv(1e-5)
