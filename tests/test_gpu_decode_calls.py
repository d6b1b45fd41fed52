"""GPU tests of dmtd_decode (Sec. 2.2: cycles back to back, one host synchronisation per call).

(1) Against the oracle: every call's last step is compared (logits within the model's tolerance, token where the oracle's
    margin allows), the steps in between by their tokens, on teacher-forced strings so that near-ties cannot fork the
    two sides; KV caches at the end.
(2) Against repeated dmtd_decode_cycle calls on a second engine: the same kernels run in the same order on the same
    data, so tokens, logits and caches must be bit-identical - free-running (every token feeds the next step), with
    several sequences, with sampling, through graphs and without.
"""
import numpy as np
import pytest

import dmtd_inputs as di
import paper_2510_11958_amd as pkg
from parity_util import MARGIN, Pair, engine_config, norm_err, top2_margin

pytestmark = pytest.mark.gpu

TOL_F32, TOL_BF16 = 1e-4, 2e-2

SHAPES = {
    # name: (shape, batch, prompt_len, tau, n_late, calls (steps per dmtd_decode call))
    "f32_tau3": (di.ModelShape(3, 128, 4, 1, 128, 200, 130, dtype="fp32"), 1, 9, 3, 2, (7, 1, 6)),
    "f32_batch3_tau4": (di.ModelShape(4, 64, 4, 2, 64, 96, 61, dtype="fp32"), 3, 6, 4, 2, (9, 4, 2)),
    "f32_tau1": (di.ModelShape(3, 64, 2, 1, 64, 96, 50, dtype="fp32"), 2, 5, 1, 3, (5, 3)),
    "bf16_tau3": (di.ModelShape(4, 256, 8, 2, 128, 512, 1000, dtype="bf16"), 2, 300, 3, 2, (8, 5)),
    "bf16_rows": (di.ModelShape(3, 256, 4, 2, 64, 512, 700, dtype="bf16"), 6, 40, 4, 1, (11, 6)),
}


def forced_string(vocab, batch, prompts, total_len, seed=1001):
    cont = di.make_continuation(vocab, batch, total_len, seed=seed)
    return [np.concatenate([prompts[b], cont[b]])[:total_len] for b in range(batch)]


@pytest.mark.parametrize("name", list(SHAPES))
def test_back_to_back_cycles_against_the_oracle(name):
    sh, B, P, tau, n_late, calls = SHAPES[name]
    blob = di.make_weight_blob(sh, seed=3)
    prompts = di.make_prompts(sh.vocab, B, P, seed=5)
    total = P + sum(calls) + 1
    toks = forced_string(sh.vocab, B, prompts, total)
    p = Pair(sh, blob, total + 2, batch=B)
    p.prefill(prompts)
    tol = TOL_F32 if sh.dtype == "fp32" else TOL_BF16
    worst, checked = 0.0, 0
    for n in calls:
        nt = p.eng.state()["n_tok"]
        f = np.stack([toks[b][nt:nt + n] for b in range(B)])
        out = p.eng.decode(tau, n_late, n, forced=f)
        assert out.shape == (B, n)
        z = p.eng.logits()
        for b, o in enumerate(p.orcs):
            n0 = len(o.step_logits)
            done = 0
            while done < n:                                     # the oracle cycle by cycle, same forced inputs
                done += len(o.decode_cycle(tau, n_late, max_new=n - done, forced=f[b][done:].tolist()))
            refs = o.step_logits[n0:]
            assert len(refs) == n
            for i, ref in enumerate(refs):                      # every step's token, where the oracle's margin allows
                if top2_margin(ref.astype(np.float64)) > MARGIN:
                    assert int(out[b, i]) == int(np.argmax(ref)), (b, i)
                    checked += 1
            worst = max(worst, norm_err(z[b], refs[-1].astype(np.float64)))
            assert int(out[b, -1]) == int(np.argmax(z[b]))
        s, o = p.eng.state(), p.orcs[0]
        assert (s["n_tok"], s["n_front"], s["phase"]) == (o.n_tok, o.n_front, o.phase)
    assert worst < tol, worst
    assert checked > 0
    p.compare_kv(1e-5 if sh.dtype == "fp32" else 2e-2)
    print(f"{name}: worst {worst:.2e}, tokens checked {checked}")


@pytest.mark.parametrize("use_graphs", [True, False])
@pytest.mark.parametrize("name,sampling", [("f32_tau3", False), ("f32_batch3_tau4", True), ("bf16_tau3", False), ("bf16_rows", True)])
def test_back_to_back_cycles_equal_single_cycle_calls_bit_for_bit(name, sampling, use_graphs):
    sh, B, P, tau, n_late, calls = SHAPES[name]
    blob = di.make_weight_blob(sh, seed=3)
    prompts = di.make_prompts(sh.vocab, B, P, seed=5)
    total = P + sum(calls) + 4
    engs = [pkg.Engine(engine_config(sh, total, B, use_graphs=use_graphs), blob) for _ in range(2)]
    for e in engs:
        if sampling:
            e.set_sampling(0.8, 20, 1234)
        e.prefill(prompts)
    a, b = engs
    for n in calls:                                             # free-running: every token is the next step's input
        got = b.decode(tau, n_late, n)
        want = []
        while sum(w.shape[1] for w in want) < n:
            want.append(a.decode_cycle(tau, n_late, max_new=n - sum(w.shape[1] for w in want)))
        want = np.concatenate(want, axis=1)
        assert np.array_equal(got, want)
        assert np.array_equal(a.logits(), b.logits())
        assert a.state() == b.state()
    assert a.trace() == b.trace()
    nt = a.state()["n_tok"]
    for l in range(sh.n_layers):
        for s in range(B):
            assert np.array_equal(a.read_kv(l, s, nt), b.read_kv(l, s, nt))


@pytest.mark.parametrize("entry", ["decode_cycle", "decode"])
def test_a_failed_call_can_be_repeated(entry, monkeypatch):
    """The error path of a decode call (a launch that fails midway, here injected from the host before step 2 of the call:
    the two steps before it run to completion on the GPU): the call reports DMTD_EHIP, the scheduler state on the host
    is unchanged, and repeating the call gives tokens, logits and caches bit-identical to an engine that never failed."""
    sh = di.ModelShape(4, 256, 8, 2, 128, 512, 1000, dtype="bf16")
    B, P, tau, n_late = 2, 40, 4, 2
    blob = di.make_weight_blob(sh, seed=3)
    prompts = di.make_prompts(sh.vocab, B, P, seed=5)
    toks = forced_string(sh.vocab, B, prompts, P + 24)
    good = pkg.Engine(engine_config(sh, P + 24, B), blob)
    monkeypatch.setenv("DMTD_TEST_FAIL_STEP", "2")
    bad = pkg.Engine(engine_config(sh, P + 24, B), blob)
    monkeypatch.delenv("DMTD_TEST_FAIL_STEP")
    for e in (good, bad):
        e.prefill(prompts)

    def call(e, n, forced):
        return e.decode(tau, n_late, n, forced=forced) if entry == "decode" else e.decode_cycle(tau, n_late, forced=forced)

    f = np.stack([toks[b][P:P + 6] for b in range(B)])
    n = 6 if entry == "decode" else tau - 1
    before = bad.state()
    with pytest.raises(pkg.DmtdError) as err:
        call(bad, n, f)
    assert err.value.code == pkg.DMTD_EHIP and "injected" in str(err.value)
    assert bad.state() == before
    for forced in (f, None, None):                       # the repeated call, then free-running calls
        assert np.array_equal(call(bad, n, forced), call(good, n, forced))
        assert np.array_equal(bad.logits(), good.logits())
        assert bad.state() == good.state()
    nt = good.state()["n_tok"]
    for l in range(sh.n_layers):
        for b in range(B):
            assert np.array_equal(bad.read_kv(l, b, nt), good.read_kv(l, b, nt))
    assert bad.trace() == good.trace()


@pytest.mark.parametrize("dtype,max_seq_len,P", [("fp32", 45, 7), ("bf16", 531, 490)])
def test_decoding_into_the_last_cache_slot_and_not_beyond(dtype, max_seq_len, P):
    """The cache's maximum size: cycles run until the last position of the cache is written (bf16 case: the context
    crosses a 512-key bucket whose end lies beyond the cache), every call checked against the oracle; one more step is
    refused with DMTD_ECAPACITY and leaves the state alone; a cycle that does not fit whole is refused, its first step
    alone is not."""
    sh = (di.ModelShape(3, 128, 4, 1, 128, 200, 130, dtype="fp32") if dtype == "fp32"
          else di.ModelShape(3, 256, 4, 2, 64, 512, 700, dtype="bf16"))
    B, tau, n_late = 2, 3, 1
    blob = di.make_weight_blob(sh, seed=3)
    prompts = di.make_prompts(sh.vocab, B, P, seed=5)
    toks = forced_string(sh.vocab, B, prompts, max_seq_len + 1)
    p = Pair(sh, blob, max_seq_len, batch=B)
    p.prefill(prompts)
    tol = TOL_F32 if dtype == "fp32" else TOL_BF16
    worst = 0.0
    while p.eng.state()["n_tok"] < max_seq_len:
        nt = p.eng.state()["n_tok"]
        n = min(7, max_seq_len - nt)
        if max_seq_len - nt == 1:
            # one slot left: a whole cycle of tau steps does not fit (only when the next step opens a cycle), its first step does
            if p.eng.state()["phase"] >= tau:
                with pytest.raises(pkg.DmtdError) as e:
                    p.eng.decode_cycle(tau, n_late)
                assert e.value.code == pkg.DMTD_ECAPACITY
                assert p.eng.state()["n_tok"] == nt
        f = np.stack([toks[b][nt:nt + n] for b in range(B)])
        out = p.eng.decode(tau, n_late, n, forced=f)
        z = p.eng.logits()
        for b, o in enumerate(p.orcs):
            done = 0
            while done < n:
                done += len(o.decode_cycle(tau, n_late, max_new=n - done, forced=f[b][done:].tolist()))
            ref = o.last_logits.astype(np.float64)
            worst = max(worst, norm_err(z[b], ref))
            if top2_margin(ref) > MARGIN:
                assert int(out[b, -1]) == int(np.argmax(ref))
    s = p.eng.state()
    assert s["n_tok"] == max_seq_len == p.orcs[0].n_tok
    assert worst < tol, worst
    p.compare_kv(1e-5 if dtype == "fp32" else 2e-2)
    for call in (lambda: p.eng.decode(tau, n_late, 1), lambda: p.eng.decode_cycle(tau, n_late, max_new=1)):
        with pytest.raises(pkg.DmtdError) as e:
            call()
        assert e.value.code == pkg.DMTD_ECAPACITY
        assert p.eng.state() == s
    print(f"{dtype}: cache of {max_seq_len} positions filled, worst {worst:.2e}")
