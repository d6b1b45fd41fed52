"""GPU parity: the HIP decode path against the CPU oracle on the same seeded inputs, through the C ABI.

Tolerances (max_i |z_gpu - z_ref| / max_j |z_ref|, per step and sequence): 1e-4 for the fp32
model, 2e-2 for bf16 models.  Token ids must agree wherever the oracle's top-2 margin exceeds 0.05.
"""
import numpy as np
import pytest

import dmtd_inputs as di
import paper_2510_11958_amd as pkg
from parity_util import Pair

pytestmark = pytest.mark.gpu

TOL_F32, TOL_BF16 = 1e-4, 2e-2


def forced_string(vocab, batch, prompts, total_len, seed=1001):
    cont = di.make_continuation(vocab, batch, total_len, seed=seed)
    return [np.concatenate([prompts[b], cont[b]])[:total_len] for b in range(batch)]


@pytest.mark.parametrize("use_graphs", [False, True])
@pytest.mark.parametrize("tau,n_late", [(2, 1), (1, 1)])
def test_c1_teacher_forced(tau, n_late, use_graphs):
    wl = di.WORKLOADS["C1"]
    sh = wl.shape
    blob = di.make_weight_blob(sh, seed=0)
    prompts = di.make_prompts(sh.vocab, 1, wl.prompt_len, seed=1)
    toks = forced_string(sh.vocab, 1, prompts, wl.prompt_len + wl.gen_len + 2)
    p = Pair(sh, blob, 64, use_graphs=use_graphs)
    p.prefill(prompts)
    for _ in range(wl.gen_len):
        p.step_forced(tau, n_late, toks)
    assert p.worst < TOL_F32, p.worst
    p.compare_kv(1e-5)
    print(f"C1 tau={tau} graphs={use_graphs}: worst {p.worst:.2e}, tokens checked {p.token_checks}, skipped {p.token_skips}")


def test_c1_free_running_greedy_matches():
    wl = di.WORKLOADS["C1"]
    sh = wl.shape
    blob = di.make_weight_blob(sh, seed=0)
    prompts = di.make_prompts(sh.vocab, 1, wl.prompt_len, seed=1)
    p = Pair(sh, blob, 64)
    first = p.eng.prefill(prompts)
    ofirst = p.orcs[0].prefill(prompts[0])
    got, want = [int(first[0])], [ofirst]
    margins = [np.sort(p.orcs[0].last_logits)[-1] - np.sort(p.orcs[0].last_logits)[-2]]
    while len(got) < wl.gen_len:
        got += p.eng.decode_cycle(wl.tau, wl.n_late, max_new=wl.gen_len - len(got))[0].tolist()
        n0 = len(p.orcs[0].step_logits)
        want += p.orcs[0].decode_cycle(wl.tau, wl.n_late, max_new=wl.gen_len - len(want))
        margins += [np.sort(z)[-1] - np.sort(z)[-2] for z in p.orcs[0].step_logits[n0:]]
    # free-running outputs can only be compared up to the first near-tie
    upto = next((i for i, m in enumerate(margins) if m <= 1e-3), len(margins))
    assert got[:upto + 1] == want[:upto + 1] or got[:upto] == want[:upto]
    assert upto >= 1


SHAPES = {
    # name: (shape, batch, prompt_len, steps, tau, n_late)
    "hd64_gq1_ragged": (di.ModelShape(3, 72, 2, 2, 64, 104, 93, dtype="fp32"), 1, 7, 12, 3, 1),
    "hd128_gq4": (di.ModelShape(3, 128, 4, 1, 128, 200, 130, dtype="fp32"), 1, 9, 12, 3, 2),
    "hd64_gq2_batch3": (di.ModelShape(4, 64, 4, 2, 64, 96, 61, dtype="fp32"), 3, 6, 14, 4, 2),
    "all_late": (di.ModelShape(3, 64, 2, 1, 64, 96, 50, dtype="fp32"), 1, 5, 8, 3, 3),
    "tau6": (di.ModelShape(3, 64, 4, 2, 64, 96, 50, dtype="fp32"), 2, 5, 20, 6, 1),
    "bf16_small": (di.ModelShape(4, 256, 8, 2, 128, 512, 1000, dtype="bf16"), 2, 300, 12, 3, 2),
    "bf16_hd64": (di.ModelShape(3, 128, 4, 2, 64, 256, 515, dtype="bf16"), 1, 270, 9, 2, 1),
    # many rows through the tiled projection kernel (36 rows in full steps, 18 in late steps and in the LM head), with tile
    # counts that leave waves and blocks partly empty (12, 20, 40 tiles) and a vocabulary that is no multiple of 16
    "bf16_batch18_ragged_tiles": (di.ModelShape(3, 192, 6, 2, 64, 320, 515, dtype="bf16"), 18, 20, 7, 2, 1),
    # 80 rows: two passes of the tiled kernel (64 + 16)
    "bf16_batch20_two_passes": (di.ModelShape(2, 128, 4, 2, 64, 256, 203, dtype="bf16"), 20, 18, 9, 4, 1),
}


@pytest.mark.parametrize("literal", [False, True])
@pytest.mark.parametrize("name", list(SHAPES))
def test_small_shapes_teacher_forced(name, literal):
    sh, batch, P, steps, tau, n_late = SHAPES[name]
    blob = di.make_weight_blob(sh, seed=7, std=0.05 if sh.dtype == "fp32" else 0.03, gain_sigma=0.2)
    prompts = di.make_prompts(sh.vocab, batch, P, seed=3)
    toks = forced_string(sh.vocab, batch, prompts, P + steps + 2)
    p = Pair(sh, blob, P + steps + 8, batch=batch, literal=literal)
    p.prefill(prompts, n_late if literal else 0)
    for _ in range(steps):
        p.step_forced(tau, n_late, toks)
    tol = TOL_F32 if sh.dtype == "fp32" else TOL_BF16
    assert p.worst < tol, p.worst
    p.compare_kv(1e-5 if sh.dtype == "fp32" else 2e-2)
    print(f"{name} literal={literal}: worst {p.worst:.2e}, tokens checked {p.token_checks}, skipped {p.token_skips}")


EXDY = {
    # name: (shape, batch, prompt_len, steps, tau, n_early, n_late)
    "f32_e2d2": (di.ModelShape(6, 64, 4, 2, 64, 96, 61, dtype="fp32"), 2, 6, 14, 3, 2, 2),
    "f32_e1d1_tau5": (di.ModelShape(5, 72, 2, 2, 64, 104, 93, dtype="fp32"), 1, 7, 16, 5, 1, 1),
    "f32_no_thinking": (di.ModelShape(4, 64, 4, 2, 64, 96, 50, dtype="fp32"), 1, 5, 9, 3, 1, 3),
    "bf16_e1d2": (di.ModelShape(6, 256, 8, 2, 128, 512, 1000, dtype="bf16"), 1, 200, 12, 3, 1, 2),
    "bf16_e2d2_batch2": (di.ModelShape(6, 128, 4, 2, 64, 256, 515, dtype="bf16"), 2, 130, 10, 4, 2, 2),
}


@pytest.mark.parametrize("literal", [False, True])
@pytest.mark.parametrize("name", list(EXDY))
def test_exdy_teacher_forced(name, literal):
    """ExDy variant (in-cycle tokens reuse the first n_early layers; the refill covers the thinking layers only):
    every step's logits and, at the end, all caches against the oracle."""
    sh, batch, P, steps, tau, n_early, n_late = EXDY[name]
    blob = di.make_weight_blob(sh, seed=11, std=0.05 if sh.dtype == "fp32" else 0.03, gain_sigma=0.2)
    prompts = di.make_prompts(sh.vocab, batch, P, seed=4)
    toks = forced_string(sh.vocab, batch, prompts, P + steps + 2)
    p = Pair(sh, blob, P + steps + 8, batch=batch, literal=literal, n_early=n_early)
    p.prefill(prompts, n_late if literal else 0)
    for _ in range(steps):
        p.step_forced(tau, n_late, toks)
    tol = TOL_F32 if sh.dtype == "fp32" else TOL_BF16
    assert p.worst < tol, p.worst
    p.compare_kv(1e-5 if sh.dtype == "fp32" else 2e-2)
    got = p.eng.state()
    o = p.orcs[0]
    assert got["gen_layer_visits"] == o.gen_layer_visits and got["refill_layer_visits"] == o.refill_layer_visits
    print(f"{name} literal={literal}: worst {p.worst:.2e}, tokens checked {p.token_checks}, skipped {p.token_skips}")


def test_exdy_switching_n_early_at_cycle_boundaries():
    """n_early may change whenever no token awaits refill (after a full step), not in between."""
    sh = di.ModelShape(6, 64, 4, 2, 64, 96, 61, dtype="fp32")
    blob = di.make_weight_blob(sh, seed=12, std=0.05, gain_sigma=0.2)
    prompts = di.make_prompts(sh.vocab, 1, 6, seed=2)
    toks = forced_string(sh.vocab, 1, prompts, 40)
    p = Pair(sh, blob, 64)
    p.prefill(prompts)
    for n_early in (2, 0, 3, 1):
        s = p.eng.state()
        assert s["n_tok"] == s["n_front"]
        p.eng.set_n_early(n_early)
        p.n_early = n_early
        for _ in range(3):                       # two late steps, then the full step that refills them
            p.step_forced(3, 2, toks)
    assert p.worst < TOL_F32, p.worst
    p.step_forced(3, 2, toks)                    # a late step: its token now awaits refill
    with pytest.raises(pkg.DmtdError):
        p.eng.set_n_early(0)
    with pytest.raises(pkg.DmtdError):
        p.eng.decode_cycle(3, 6)                 # n_early + n_late > n_layers


def test_changing_tau_and_whole_cycle_calls():
    """Whole-cycle calls (several steps per call) with a tau that changes between cycles."""
    sh = di.ModelShape(4, 64, 4, 2, 64, 96, 61, dtype="fp32")
    blob = di.make_weight_blob(sh, seed=5, std=0.05, gain_sigma=0.2)
    prompts = di.make_prompts(sh.vocab, 2, 6, seed=4)
    toks = forced_string(sh.vocab, 2, prompts, 64)
    p = Pair(sh, blob, 64, batch=2)
    p.prefill(prompts)
    for tau, cap in [(3, 0), (2, 0), (5, 3), (5, 0), (1, 0), (4, 0), (4, 0)]:
        nt = p.eng.state()["n_tok"]
        f = np.stack([toks[b][nt:nt + tau] for b in range(2)])
        out = p.eng.decode_cycle(tau, 2, max_new=cap, forced=f)
        for b, o in enumerate(p.orcs):
            want = o.decode_cycle(tau, 2, max_new=cap, forced=f[b].tolist())
            z = p.eng.logits()[b]
            assert np.abs(z - o.last_logits).max() / np.abs(o.last_logits).max() < TOL_F32
            assert out.shape[1] == len(want)
        s = p.eng.state()
        assert (s["n_tok"], s["n_front"], s["phase"]) == (p.orcs[0].n_tok, p.orcs[0].n_front, p.orcs[0].phase)
    p.compare_kv(1e-5)


def test_reset_and_rerun_is_bit_identical():
    sh = di.WORKLOADS["C1"].shape
    blob = di.make_weight_blob(sh, seed=0)
    prompts = di.make_prompts(sh.vocab, 1, 32, seed=1)
    p = Pair(sh, blob, 64)
    runs = []
    for _ in range(2):
        p.eng.prefill(prompts)
        outs = [p.eng.decode_cycle(2, 1) for _ in range(4)]
        runs.append((np.concatenate(outs, 1), p.eng.logits().copy()))
        p.eng.reset()
    assert np.array_equal(runs[0][0], runs[1][0]) and np.array_equal(runs[0][1], runs[1][1])
