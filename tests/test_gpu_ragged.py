"""GPU parity for batches whose prompts differ in length (dmtd_prefill_ragged): every sequence against its own
standalone oracle run.  Sequences decode in lockstep (same phase), each at its own positions; padding behind a
shorter prompt must not influence anything."""
import numpy as np
import pytest

import dmtd_inputs as di
import paper_2510_11958_amd as pkg
from oracle import dmtd_oracle as O
from parity_util import MARGIN, engine_config, norm_err, oracle_config, top2_margin

pytestmark = pytest.mark.gpu

TOL_F32, TOL_BF16 = 1e-4, 2e-2

CASES = {
    # name: (shape, lengths, steps, tau, n_early, n_late)
    "f32_three_chunks": (di.ModelShape(4, 64, 4, 2, 64, 96, 61, dtype="fp32"), [9, 20, 33, 17], 14, 3, 0, 2),
    "f32_one_token_prompt": (di.ModelShape(3, 72, 2, 2, 64, 104, 93, dtype="fp32"), [1, 16, 5], 10, 4, 0, 1),
    "f32_exdy": (di.ModelShape(6, 64, 4, 2, 64, 96, 61, dtype="fp32"), [7, 18, 12], 12, 3, 2, 2),
    "bf16_small": (di.ModelShape(4, 256, 8, 2, 128, 512, 1000, dtype="bf16"), [300, 270, 41], 10, 3, 0, 2),
    # 18 sequences: 36 rows in full steps (tiled projection kernel), context buckets differ by sequence
    "bf16_batch18": (di.ModelShape(3, 192, 6, 2, 64, 320, 515, dtype="bf16"), [20 + 29 * (b % 5) for b in range(18)], 7, 2, 0, 1),
}


@pytest.mark.parametrize("literal", [False, True])
@pytest.mark.parametrize("name", list(CASES))
def test_ragged_prompts_teacher_forced(name, literal):
    sh, lengths, steps, tau, n_early, n_late = CASES[name]
    B, P = len(lengths), max(lengths)
    tol = TOL_F32 if sh.dtype == "fp32" else TOL_BF16
    blob = di.make_weight_blob(sh, seed=17, std=0.05 if sh.dtype == "fp32" else 0.03, gain_sigma=0.2)
    full = di.make_prompts(sh.vocab, B, P + steps + 4, seed=8)     # each sequence's prompt and forced continuation
    padded = np.full((B, P), sh.vocab - 1, np.int32)                # padding: a valid id that must be ignored ...
    for b, n in enumerate(lengths):
        padded[b, :n] = full[b, :n]
    padded[0, lengths[0]:] = 10 ** 6 if lengths[0] < P else padded[0, lengths[0]:]   # ... or any junk at all
    eng = pkg.Engine(engine_config(sh, P + steps + 8, B, full_pos_add_embed=literal), blob)
    ocfg = oracle_config(sh, full_pos_add_embed=literal)
    w = O.unpack_weights(blob, ocfg)
    orcs = [O.DmtdOracle(ocfg, w, P + steps + 8) for _ in range(B)]
    if n_early:
        eng.set_n_early(n_early)
    worst, checked = 0.0, 0

    def compare(gpu_tokens):
        nonlocal worst, checked
        z = eng.logits()
        for b, o in enumerate(orcs):
            ref = o.last_logits.astype(np.float64)
            worst = max(worst, norm_err(z[b], ref))
            if top2_margin(ref) > MARGIN:
                assert int(gpu_tokens[b]) == int(np.argmax(ref)), (b, o.n_tok)
                checked += 1
            assert int(gpu_tokens[b]) == int(np.argmax(z[b]))

    first = eng.prefill(padded, n_late if literal else 0, lengths=lengths)
    for b, o in enumerate(orcs):
        o.prefill(full[b, :lengths[b]], n_late if literal else None, n_early)
    compare(first)
    for step in range(steps):
        f = np.stack([full[b, lengths[b] + step:lengths[b] + step + 1] for b in range(B)])
        out = eng.decode_cycle(tau, n_late, max_new=1, forced=f)
        for b, o in enumerate(orcs):
            o.decode_cycle(tau, n_late, max_new=1, forced=f[b].tolist(), n_early=n_early)
        compare(out[:, 0])
        s = eng.state()
        longest = orcs[int(np.argmax(lengths))]
        assert (s["n_tok"], s["n_front"], s["phase"]) == (longest.n_tok, longest.n_front, longest.phase)
    assert worst < tol, worst
    for l in range(sh.n_layers):
        for b, o in enumerate(orcs):
            kv = eng.read_kv(l, b, o.n_tok)
            late = l >= sh.n_layers - n_late
            upto = o.n_tok if (late or l < n_early) else o.n_front
            for which, ref in ((0, o.K[l]), (1, o.V[l])):
                r = np.transpose(ref[:upto], (1, 0, 2))
                err = np.abs(kv[which][:, :upto] - r).max() / max(np.abs(r).max(), 1e-30)
                assert err < (1e-5 if sh.dtype == "fp32" else 2e-2), (l, b, which, err)
    print(f"{name} literal={literal}: worst {worst:.2e}, tokens checked {checked}")


def test_ragged_free_running_whole_cycles_and_sampling():
    """Whole-cycle calls, free running, with sampled tokens: each sequence draws at its own positions, so a sequence
    decodes the same tokens inside a ragged batch (at any batch index with the same draw counter) as alone."""
    sh = di.ModelShape(4, 64, 4, 2, 64, 96, 61, dtype="fp32")
    blob = di.make_weight_blob(sh, seed=17, std=0.08, gain_sigma=0.2)
    lengths = [5, 19, 11]
    full = di.make_prompts(sh.vocab, 3, 19, seed=8)
    padded = np.zeros((3, 19), np.int32)
    for b, n in enumerate(lengths):
        padded[b, :n] = full[b, :n]
    eng = pkg.Engine(engine_config(sh, 64, 3), blob)
    ocfg = oracle_config(sh)
    w = O.unpack_weights(blob, ocfg)
    for sampling in (None, (1.2, 9, 5)):
        eng.reset()
        orcs = [O.DmtdOracle(ocfg, w, 64) for _ in range(3)]
        if sampling:
            eng.set_sampling(*sampling)
            for b, o in enumerate(orcs):
                o.set_sampling(*sampling, seq=b)
        last = eng.prefill(padded, lengths=lengths)
        for b, o in enumerate(orcs):
            o.prefill(full[b, :lengths[b]])
        for tau in (3, 3, 2, 4, 1, 3):
            out = eng.decode_cycle(tau, 2)
            z = eng.logits()
            for b, o in enumerate(orcs):
                o.decode_cycle(tau, 2, forced=[int(last[b])] + [int(t) for t in out[b, :-1]])
                assert norm_err(z[b], o.last_logits) < TOL_F32
            last = out[:, -1]


def test_ragged_argument_errors():
    sh = di.ModelShape(3, 64, 4, 2, 64, 96, 50, dtype="fp32")
    eng = pkg.Engine(engine_config(sh, 32, 3), di.make_weight_blob(sh, seed=2, std=0.05))
    toks = di.make_prompts(sh.vocab, 3, 12, seed=3)
    for lengths in ([12, 0, 5], [12, 13, 5], [11, 10, 5]):       # zero, beyond prompt_len, none reaches prompt_len
        with pytest.raises(pkg.DmtdError) as e:
            eng.prefill(toks, lengths=lengths)
        assert e.value.code == pkg.DMTD_EINVAL
    bad = toks.copy()
    bad[1, 3] = sh.vocab
    with pytest.raises(pkg.DmtdError):
        eng.prefill(bad, lengths=[12, 4, 5])                     # inside sequence 1's prompt: an error
    eng.prefill(bad, lengths=[12, 3, 5])                          # behind it: ignored
