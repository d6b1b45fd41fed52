"""GPU parity of the whole-sequence masked forward (Sec. 2.1, Eqs. 1-5) and the next-token loss (Eq. 6).

Three checks: (1) every position's logits, the per-position cross entropies, the loss and the argmax against the CPU
oracle's one-shot masked forward, for the training mask of Eq. 3 and for the mask cycle decoding realises;
(2) on the GPU alone, the masked forward against prefill + teacher-forced cycle decoding at the same positions (the
same identity that pins the oracle); (3) argument errors.

Tolerances: logits as in the decode parity tests (max-normalised, 1e-4 fp32 model, 2e-2 bf16 models).  A cross entropy is
log-sum-exp(z) - z[target]; an error of at most e on every logit moves the first term by at most e and the second by at
most e, so |nll_gpu - nll_ref| <= 2 e with e = tolerance * max|z_ref|; the loss, a mean of those, obeys the same bound.
"""
import numpy as np
import pytest

import dmtd_inputs as di
import paper_2510_11958_amd as pkg
from oracle import dmtd_oracle as O
from parity_util import MARGIN, engine_config, norm_err, oracle_config, top2_margin

pytestmark = pytest.mark.gpu

TOL_F32, TOL_BF16 = 1e-4, 2e-2

CASES = {
    # name: (shape, batch, n, tau, n_early, n_late, prompt_len or None (None: Eq. 3's mask))
    "f32_eq3_tau3": (di.ModelShape(4, 64, 4, 2, 64, 96, 61, dtype="fp32"), 2, 37, 3, 0, 2, None),
    "f32_infer_tau4_ragged": (di.ModelShape(3, 72, 2, 2, 64, 104, 93, dtype="fp32"), 1, 21, 4, 0, 1, 6),
    "f32_all_late": (di.ModelShape(3, 64, 2, 1, 64, 96, 50, dtype="fp32"), 1, 18, 2, 0, 3, None),
    "f32_tau1": (di.ModelShape(3, 64, 4, 2, 64, 96, 50, dtype="fp32"), 1, 17, 1, 0, 1, None),
    "f32_exdy_e2d2": (di.ModelShape(6, 64, 4, 2, 64, 96, 61, dtype="fp32"), 2, 33, 3, 2, 2, 7),
    "f32_exdy_no_thinking": (di.ModelShape(4, 64, 4, 2, 64, 96, 50, dtype="fp32"), 1, 19, 3, 1, 3, None),
    "bf16_eq3_tau3": (di.ModelShape(4, 256, 8, 2, 128, 512, 1000, dtype="bf16"), 2, 70, 3, 0, 2, None),
    "bf16_infer_hd64": (di.ModelShape(3, 128, 4, 2, 64, 256, 515, dtype="bf16"), 1, 45, 2, 0, 1, 30),
    "bf16_exdy_e1d2": (di.ModelShape(6, 256, 8, 2, 128, 512, 1000, dtype="bf16"), 1, 40, 3, 1, 2, 20),
    # 5 sequences x 25 positions = 125 rows per pass (one 128-row pass of the tiled projection kernel), ragged vocabulary
    "bf16_batch5_two_passes": (di.ModelShape(2, 128, 4, 2, 64, 256, 203, dtype="bf16"), 5, 35, 4, 0, 1, None),
    # 9 sequences x 16 positions = 144 rows per pass: two weight passes of the tiled kernel (128 + 16 rows)
    "bf16_batch9_two_weight_passes": (di.ModelShape(2, 128, 4, 2, 64, 256, 203, dtype="bf16"), 9, 35, 4, 0, 1, None),
}


def case_inputs(name):
    sh, batch, n, tau, n_early, n_late, P = CASES[name]
    blob = di.make_weight_blob(sh, seed=21, std=0.05 if sh.dtype == "fp32" else 0.03, gain_sigma=0.2)
    toks = di.make_prompts(sh.vocab, batch, n, seed=9)
    mask = O.training_mask(n, tau) if P is None else O.inference_mask(n, P, tau)
    return sh, batch, n, tau, n_early, n_late, P, blob, toks, mask


@pytest.mark.parametrize("literal", [False, True])
@pytest.mark.parametrize("name", list(CASES))
def test_masked_forward_against_oracle(name, literal):
    sh, batch, n, tau, n_early, n_late, P, blob, toks, mask = case_inputs(name)
    tol = TOL_F32 if sh.dtype == "fp32" else TOL_BF16
    eng = pkg.Engine(engine_config(sh, n + 3, batch, full_pos_add_embed=literal), blob)
    if n_early:
        eng.set_n_early(n_early)
    got = eng.masked_forward(toks, mask, n_late, want_logits=True)
    ocfg = oracle_config(sh, full_pos_add_embed=literal)
    w = O.unpack_weights(blob, ocfg)
    worst, worst_nll, checked = 0.0, 0.0, 0
    for b in range(batch):
        ref = O.masked_forward(toks[b], mask, n_late, w, ocfg, n_early=n_early)
        ref_nll = O.next_token_nll(ref, toks[b])
        for i in range(n):
            worst = max(worst, norm_err(got["logits"][b, i], ref[i]))
            assert int(got["best"][b, i]) == int(np.argmax(got["logits"][b, i]))
            if top2_margin(ref[i]) > MARGIN:
                assert int(got["best"][b, i]) == int(np.argmax(ref[i])), (b, i)
                checked += 1
        bound = 2 * tol * np.abs(ref).max()
        err = np.abs(got["nll"][b, :n - 1] - ref_nll).max()
        worst_nll = max(worst_nll, err / bound)
        assert err < bound, (b, err, bound)
        assert got["nll"][b, n - 1] == 0.0
        assert abs(got["loss"][b] - O.next_token_loss(ref, toks[b])) < bound
        # the device's loss is the mean of the device's own summands
        assert abs(got["loss"][b] - got["nll"][b, :n - 1].astype(np.float64).mean()) < 1e-5 * max(1.0, abs(got["loss"][b]))
    assert worst < tol, worst
    # the context is empty again: a prefill may follow, and a second call gives the same bits
    again = eng.masked_forward(toks, mask, n_late, want_logits=True)
    assert np.array_equal(again["logits"], got["logits"]) and np.array_equal(again["nll"], got["nll"])
    eng.prefill(toks[:, :5], n_late if literal else 0)
    print(f"{name} literal={literal}: worst logit error {worst:.2e}, nll error / bound {worst_nll:.2e}, tokens checked {checked}")


@pytest.mark.parametrize("name", ["f32_infer_tau4_ragged", "f32_exdy_e2d2", "bf16_infer_hd64", "bf16_exdy_e1d2"])
def test_masked_forward_equals_cycle_decoding_on_the_gpu(name):
    """Cycle decoding with refill (prefill, then teacher-forced steps) and the one-shot masked forward with the mask that
    decoding realises compute the same function (Sec. 2.1 vs Sec. 2.2).  The two GPU paths batch rows differently, so they
    agree to rounding (fp32 model) or to the bf16 storage noise, not bit for bit."""
    sh, batch, n, tau, n_early, n_late, P, blob, toks, mask = case_inputs(name)
    tol = TOL_F32 if sh.dtype == "fp32" else TOL_BF16
    eng = pkg.Engine(engine_config(sh, n + 3, batch), blob)
    if n_early:
        eng.set_n_early(n_early)
    one_shot = eng.masked_forward(toks, mask, n_late, want_logits=True)["logits"]
    eng.prefill(toks[:, :P])
    worst = max(norm_err(eng.logits()[b], one_shot[b, P - 1].astype(np.float64)) for b in range(batch))
    for pos in range(P, n):
        eng.decode_cycle(tau, n_late, max_new=1, forced=toks[:, pos:pos + 1])
        z = eng.logits()
        worst = max(worst, max(norm_err(z[b], one_shot[b, pos].astype(np.float64)) for b in range(batch)))
    assert worst < tol, worst
    print(f"{name}: cycle decoding vs one-shot masked forward on the GPU, worst {worst:.2e}")


def test_masked_forward_argument_errors():
    sh = di.ModelShape(3, 64, 4, 2, 64, 96, 50, dtype="fp32")
    blob = di.make_weight_blob(sh, seed=2, std=0.05)
    eng = pkg.Engine(engine_config(sh, 24, 2), blob)
    toks = di.make_prompts(sh.vocab, 2, 12, seed=3)
    mask = O.training_mask(12, 3)
    for bad in (dict(n_late=0), dict(n_late=4)):
        with pytest.raises(pkg.DmtdError) as e:
            eng.masked_forward(toks, mask, bad["n_late"])
        assert e.value.code == pkg.DMTD_EINVAL
    with pytest.raises(pkg.DmtdError) as e:
        eng.masked_forward(np.full((1, 12), sh.vocab), mask, 1)
    assert e.value.code == pkg.DMTD_EINVAL
    with pytest.raises(pkg.DmtdError) as e:
        eng.masked_forward(di.make_prompts(sh.vocab, 1, 25, seed=3), O.training_mask(25, 3), 1)
    assert e.value.code == pkg.DMTD_ECAPACITY
    with pytest.raises(pkg.DmtdError) as e:
        eng.masked_forward(di.make_prompts(sh.vocab, 3, 12, seed=3), mask, 1)
    assert e.value.code == pkg.DMTD_EINVAL
    eng.prefill(toks[:, :5])
    with pytest.raises(pkg.DmtdError) as e:
        eng.masked_forward(toks, mask, 1)
    assert e.value.code == pkg.DMTD_ESTATE
    eng.reset()
    assert eng.masked_forward(toks, mask, 1)["nll"].shape == (2, 12)
