"""GPU test of the measurement aid dmtd_time_kernel: it runs the decode path's kernels (and the read-only kinds that
stream the same weight bytes) on scratch buffers, and the model's state must come out of it untouched - the next
decode steps still agree with the oracle and the caches are bit-identical to those before the timing calls."""
import numpy as np
import pytest

import dmtd_inputs as di
import paper_2510_11958_amd as pkg
from parity_util import Pair

pytestmark = pytest.mark.gpu


def test_timing_calls_leave_the_model_state_untouched():
    sh = di.ModelShape(4, 256, 8, 2, 128, 512, 1000, dtype="bf16")
    B, P, tau, n_late = 2, 37, 3, 2
    blob = di.make_weight_blob(sh, seed=3)
    prompts = di.make_prompts(sh.vocab, B, P, seed=5)
    cont = di.make_continuation(sh.vocab, B, P + 16, seed=11)
    toks = [np.concatenate([prompts[b], cont[b]]) for b in range(B)]
    p = Pair(sh, blob, P + 20, batch=B)
    p.prefill(prompts)
    for _ in range(4):
        p.step_forced(tau, n_late, toks)
    before_state = p.eng.state()
    before_kv = [p.eng.read_kv(l, b, before_state["n_tok"]) for l in range(sh.n_layers) for b in range(B)]
    times = {}
    for kind in pkg.Engine.KERNEL_KINDS:
        rows = B if kind == "lmhead" else (3 if kind == "attn" else 3 * B)
        times[kind] = p.eng.time_kernel(kind, rows if not kind.startswith("read_") else 1, reps=2)
        assert np.isfinite(times[kind]) and times[kind] > 0.0, (kind, times[kind])
    assert p.eng.state() == before_state
    after_kv = [p.eng.read_kv(l, b, before_state["n_tok"]) for l in range(sh.n_layers) for b in range(B)]
    for a, b_ in zip(before_kv, after_kv):
        assert np.array_equal(a, b_)
    for _ in range(5):                      # the path goes on as if nothing had happened
        p.step_forced(tau, n_late, toks)
    assert p.worst < 2e-2, p.worst
    p.compare_kv(2e-2)
    print("us per launch:", {k: round(v, 2) for k, v in times.items()})


def test_read_only_kinds_are_refused_for_an_fp32_model():
    sh = di.ModelShape(3, 128, 4, 1, 128, 200, 130, dtype="fp32")
    blob = di.make_weight_blob(sh, seed=3)
    p = Pair(sh, blob, 32, batch=1)
    p.prefill(di.make_prompts(sh.vocab, 1, 9, seed=5))
    assert p.eng.time_kernel("gateup", 1, reps=1) > 0.0
    with pytest.raises(pkg.DmtdError):
        p.eng.time_kernel("read_gateup", 1, reps=1)
