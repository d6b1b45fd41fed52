"""dmtd_decode_cycle_noalloc (the entry point for callers that cannot allocate: partial results in the library's own
array, DEVICE token buffers, no synchronisation) against dmtd_decode_cycle on a second engine: the same kernels run in
the same order on the same data, so tokens, logits and caches must be bit-identical; the existing entry point is itself
compared with the oracle.  Two calls in a row on one context, the second with a smaller input (fewer steps, fewer forced
tokens), then whole free-running cycles; the scratch limit; host-side argument errors in a dry run."""
import numpy as np
import pytest
import torch

import dmtd_inputs as di
import paper_2510_11958_amd as pkg
from parity_util import MARGIN, Pair, engine_config, norm_err, top2_margin

TOL_F32, TOL_BF16 = 1e-4, 2e-2

SHAPES = {
    "bf16": (di.ModelShape(4, 256, 8, 2, 128, 512, 1000, dtype="bf16"), 2, 70, 4, 2),
    "bf16_rows": (di.ModelShape(3, 256, 4, 2, 64, 512, 700, dtype="bf16"), 6, 40, 4, 1),    # full steps through the tiled kernel
    "fp32": (di.ModelShape(3, 128, 4, 1, 128, 200, 130, dtype="fp32"), 1, 9, 3, 2),
}


def forced_string(vocab, batch, prompts, total_len, seed=1001):
    cont = di.make_continuation(vocab, batch, total_len, seed=seed)
    return [np.concatenate([prompts[b], cont[b]])[:total_len] for b in range(batch)]


@pytest.mark.gpu
@pytest.mark.parametrize("name", list(SHAPES))
def test_noalloc_equals_decode_cycle_and_the_oracle(name):
    sh, B, P, tau, n_late = SHAPES[name]
    tol = TOL_F32 if sh.dtype == "fp32" else TOL_BF16
    blob = di.make_weight_blob(sh, seed=3)
    prompts = di.make_prompts(sh.vocab, B, P, seed=5)
    total = P + 48
    toks = forced_string(sh.vocab, B, prompts, total)
    p = Pair(sh, blob, total, batch=B)                        # the existing entry point + one oracle per sequence
    new = pkg.Engine(engine_config(sh, total, B), blob)       # the entry point under test
    p.prefill(prompts)
    new.prefill(prompts)
    out_dev = torch.full((B, 8), -7, dtype=torch.int32, device="cuda")
    worst, checked = 0.0, 0
    # (max_new, forced tokens given): the rest of cycle 1, then a smaller call (2 steps), the rest of that cycle with more
    # forced tokens than steps, a single full step, whole cycles; the last two calls run free (no forced inputs)
    for max_new, n_forced in ((0, tau), (2, 2), (0, tau), (1, 1), (0, tau), (0, tau), (0, 0), (0, 0)):
        nt = p.eng.state()["n_tok"]
        f = np.stack([toks[b][nt:nt + max(n_forced, 1)] for b in range(B)]).astype(np.int32)
        want = p.eng.decode_cycle(tau, n_late, max_new=max_new, forced=f if n_forced else None)
        out_dev.fill_(-7)
        f_dev = torch.from_numpy(f).cuda() if n_forced else None
        torch.cuda.synchronize()
        n = new.decode_cycle_noalloc(tau, n_late, out_dev, max_new=max_new, forced_dev=f_dev)
        new.synchronize()
        got = out_dev.cpu().numpy()
        assert n == want.shape[1]
        assert np.array_equal(got[:, :n], want)
        assert (got[:, n:] == -7).all()                       # nothing written beyond the steps run
        z = new.logits()
        assert np.array_equal(z, p.eng.logits())
        assert new.state() == p.eng.state()
        if not n_forced:
            continue                                          # free-running: the two entry points against each other only
        assert n_forced >= n
        for b, o in enumerate(p.orcs):                        # and against the oracle (the existing entry point's own bar)
            n0 = len(o.step_logits)
            o.decode_cycle(tau, n_late, max_new=max_new, forced=f[b].tolist())
            refs = o.step_logits[n0:]
            assert len(refs) == n
            for i, ref in enumerate(refs):
                if top2_margin(ref.astype(np.float64)) > MARGIN:
                    assert int(got[b, i]) == int(np.argmax(ref))
                    checked += 1
            worst = max(worst, norm_err(z[b], refs[-1].astype(np.float64)))
    assert worst < tol, worst
    assert checked > 0
    nt = new.state()["n_tok"]
    for l in range(sh.n_layers):
        for b in range(B):
            assert np.array_equal(new.read_kv(l, b, nt), p.eng.read_kv(l, b, nt))
    assert new.trace() == p.eng.trace()
    print(f"noalloc {name}: worst vs oracle {worst:.2e}, tokens checked {checked}")


@pytest.mark.gpu
def test_noalloc_scratch_limit_is_an_error_and_leaves_the_state_alone():
    """Partial results beyond the library's array: 4 sequences x 16 refill rows of 8 query heads of 128 need 16.8 MB."""
    sh = di.ModelShape(2, 256, 8, 2, 128, 512, 300, dtype="bf16")
    B, P = 4, 12
    blob = di.make_weight_blob(sh, seed=3)
    eng = pkg.Engine(engine_config(sh, 80, B), blob)
    eng.prefill(di.make_prompts(sh.vocab, B, P, seed=5))
    out_dev = torch.zeros((B, 16), dtype=torch.int32, device="cuda")
    assert eng.decode_cycle_noalloc(16, 1, out_dev) == 15       # the rest of cycle 1: one row per sequence
    eng.synchronize()
    before = eng.state()
    with pytest.raises(pkg.DmtdError) as e:
        eng.decode_cycle_noalloc(16, 1, out_dev)                # the full step would carry 16 rows per sequence
    assert e.value.code == pkg.DMTD_ECAPACITY and "scratch" in str(e.value)
    assert eng.state() == before
    assert eng.decode_cycle(16, 1).shape == (B, 16)             # the workspace-backed entry point takes it


def test_noalloc_argument_errors_without_a_gpu():
    eng = pkg.Engine(pkg.ModelConfig(4, 64, 4, 2, 64, 96, 50, dtype="fp32", max_seq_len=16, dry_run=True))
    lib = eng.lib
    import ctypes as C
    n = C.c_int32(5)
    assert lib.dmtd_decode_cycle_noalloc(eng._h, 2, 1, 0, None, 0, None, 4, C.byref(n)) == pkg.DMTD_ESTATE   # before prefill
    assert n.value == 0
    eng.prefill(np.zeros((1, 5), np.int32))
    assert lib.dmtd_decode_cycle_noalloc(eng._h, 2, 1, 0, None, 0, None, 4, None) == pkg.DMTD_EINVAL
    assert lib.dmtd_decode_cycle_noalloc(eng._h, 0, 1, 0, None, 0, None, 4, C.byref(n)) == pkg.DMTD_EINVAL
    assert lib.dmtd_decode_cycle_noalloc(eng._h, 65, 1, 0, None, 0, None, 4, C.byref(n)) == pkg.DMTD_EINVAL
    assert lib.dmtd_decode_cycle_noalloc(eng._h, 3, 1, 0, None, 0, None, 1, C.byref(n)) == pkg.DMTD_ECAPACITY  # out_stride
    before = eng.state()
    assert lib.dmtd_decode_cycle_noalloc(eng._h, 3, 1, 0, None, 0, None, 4, C.byref(n)) == pkg.DMTD_OK and n.value == 2
    s = eng.state()
    assert (s["n_tok"], s["n_front"], s["phase"]) == (before["n_tok"] + 2, before["n_front"], 3)
    ref = pkg.Engine(pkg.ModelConfig(4, 64, 4, 2, 64, 96, 50, dtype="fp32", max_seq_len=16, dry_run=True))
    ref.prefill(np.zeros((1, 5), np.int32))
    ref.decode_cycle(3, 1)
    assert ref.state() == s and ref.trace() == eng.trace()
