"""GPU parity on the kernel paths the benchmark configurations take at their real sizes, through the C ABI with
graphs on (the launch configuration bench.py times).

* C4's attention launch shape (one key range per 8-wave block, chosen when the (KV head, sequence) pairs fill the
  chip) at C4's batch and context: 32 sequences x 2048 keys on a one-layer model with C4's head geometry, steps with
  one row and with four rows per sequence, against the float64 oracle.
* C4 itself (36 layers, B = 32, P = 2048, tau = 4, n_late = 12): sequences 0 and 31 against standalone float32 oracle
  runs over the first two cycles (batch rows are independent).
* C3's whole run (P = 1024, 511 decode steps) teacher-forced against the float32 oracle.
* Decoding across a 512-token context bucket (graph re-capture, split of a group of steps), against the oracle.
* A context reset and prefilled again with a different batch size (captured graphs bake the batch in).
"""
import time

import numpy as np
import pytest
import torch

import dmtd_inputs as di
from oracle import dmtd_oracle as O
from parity_util import MARGIN, Pair, engine_config, norm_err, oracle_config, top2_margin
import paper_2510_11958_amd as pkg

pytestmark = pytest.mark.gpu

TOL_F32, TOL_BF16 = 1e-4, 2e-2


def forced_string(vocab, batch, prompts, total_len, seed=1001):
    cont = di.make_continuation(vocab, batch, total_len, seed=seed)
    return [np.concatenate([prompts[b], cont[b]])[:total_len] for b in range(batch)]


def _step_and_compare(eng, orcs, toks, tau, n_late, worst, checked):
    """One teacher-forced step of the whole batch; the sequences in orcs against their oracles."""
    B = len(toks)
    nt = eng.state()["n_tok"]
    f = np.stack([toks[b][nt:nt + 1] for b in range(B)])
    out = eng.decode_cycle(tau, n_late, max_new=1, forced=f)
    z = eng.logits()
    assert np.array_equal(out[:, 0], np.argmax(z, axis=1))          # every sequence: token = argmax of its logits
    for b, o in orcs.items():
        o.decode_cycle(tau, n_late, max_new=1, forced=f[b].tolist())
        ref = o.last_logits.astype(np.float64)
        worst = max(worst, norm_err(z[b], ref))
        if top2_margin(ref) > MARGIN:
            assert int(out[b, 0]) == int(np.argmax(ref)), (b, nt)
            checked += 1
    s, o = eng.state(), next(iter(orcs.values()))
    assert (s["n_tok"], s["n_front"], s["phase"]) == (o.n_tok, o.n_front, o.phase)
    return worst, checked


def test_c4_attention_launch_shape_at_full_context():
    """32 sequences x 2048-token prompts, one layer with C4's head geometry (32 query / 8 KV heads of 128): the 8 x 32
    (KV head, sequence) pairs fill the chip, so attention runs as one key range per 8-wave block, 16+ trips of its key
    loop with every wave busy.  tau = 4: three steps with one row per sequence, then a full step with four rows, twice.
    Sequences 0, 13 and 31 against float64 oracles; caches of those sequences element-wise."""
    sh = di.ModelShape(1, 512, 32, 8, 128, 1024, 2048, dtype="bf16")
    blob = di.make_weight_blob(sh, seed=4, std=0.05, gain_sigma=0.2)
    B, P, tau, n_late = 32, 2048, 4, 1
    prompts = di.make_prompts(sh.vocab, B, P, seed=11)
    toks = forced_string(sh.vocab, B, prompts, P + 16)
    eng = pkg.Engine(engine_config(sh, P + 16, B), blob)
    ocfg = oracle_config(sh)
    w = O.unpack_weights(blob, ocfg, np.float64)
    picks = (0, 13, B - 1)
    orcs = {b: O.DmtdOracle(ocfg, w, P + 16, np.float64) for b in picks}
    first = eng.prefill(prompts)
    z = eng.logits()
    worst, checked = 0.0, 0
    for b, o in orcs.items():
        o.prefill(prompts[b])
        ref = o.last_logits.astype(np.float64)
        worst = max(worst, norm_err(z[b], ref))
        if top2_margin(ref) > MARGIN:
            assert int(first[b]) == int(np.argmax(ref))
    rows_seen = set()
    for _ in range(8):
        st = eng.state()
        rows_seen.add(st["n_tok"] - st["n_front"] + 1 if st["phase"] >= tau else 1)
        worst, checked = _step_and_compare(eng, orcs, toks, tau, n_late, worst, checked)
    assert rows_seen == {1, 4}
    assert worst < TOL_BF16, worst
    n = eng.state()["n_tok"]
    for b, o in orcs.items():
        kv = eng.read_kv(0, b, n)
        for which, ref in ((0, o.K[0]), (1, o.V[0])):
            r = np.transpose(ref[:n], (1, 0, 2))
            assert np.abs(kv[which][:, :n] - r).max() / np.abs(r).max() < 1e-2
    print(f"C4 attention shape (B={B}, P={P}): worst {worst:.2e}, tokens checked {checked}")


@pytest.fixture(scope="module")
def model_4b():
    sh = di.WORKLOADS["C3"].shape
    blob = di.make_weight_blob(sh, seed=0)
    ocfg = oracle_config(sh)
    w32 = O.unpack_weights(blob, ocfg, np.float32)      # float32 oracle for the 4B shape (float64 would be 32 GB)
    dev = torch.from_numpy(blob.view(np.int16)).cuda()
    return sh, blob, ocfg, w32, dev


def test_c4_real_prompt_first_two_cycles(model_4b):
    """C4 as configured (36 layers, B = 32, P = 2048, tau = 4, n_late = 12): prefill logits and the first two cycles
    (3 + 4 decode steps, teacher-forced) of sequences 0 and 31 against standalone float32 oracle runs.  Not verified
    against the oracle: the other 30 sequences (their tokens must still be the argmax of their logits) and the cycles
    after the second - a float32 oracle prefill of one 2048-token prompt alone takes most of a minute on the host."""
    wl = di.WORKLOADS["C4"]
    sh, blob, ocfg, w32, dev = model_4b
    B, P = wl.batch, wl.prompt_len
    prompts = di.make_prompts(sh.vocab, B, P, seed=1)
    toks = forced_string(sh.vocab, B, prompts, P + 16)
    eng = pkg.Engine(engine_config(sh, P + 16, B), dev)
    first = eng.prefill(prompts)
    z = eng.logits()
    picks = (0, B - 1)
    orcs = {b: O.DmtdOracle(ocfg, w32, P + 16, np.float32) for b in picks}
    worst, checked = 0.0, 0
    t0 = time.time()
    for b, o in orcs.items():
        o.prefill(prompts[b])
        ref = o.last_logits.astype(np.float64)
        worst = max(worst, norm_err(z[b], ref))
        if top2_margin(ref) > MARGIN:
            assert int(first[b]) == int(np.argmax(ref))
    t_prefill = time.time() - t0
    for _ in range((wl.tau - 1) + wl.tau):
        worst, checked = _step_and_compare(eng, orcs, toks, wl.tau, wl.n_late, worst, checked)
    assert worst < TOL_BF16, worst
    print(f"C4 (B={B}, P={P}): worst {worst:.2e}, tokens checked {checked}, oracle prefill of two sequences {t_prefill:.0f} s")


def test_c3_whole_run_teacher_forced(model_4b):
    """C3 as configured (P = 1024, G = 512, tau = 3, n_late = 8): all 511 decode steps teacher-forced against the float32
    oracle, every step's logits and (where the oracle's margin allows) token; the generation crosses the 512-token
    attention bucket boundary at position 1536 only at its very end, so the bucket test below covers that case."""
    wl = di.WORKLOADS["C3"]
    sh, blob, ocfg, w32, dev = model_4b
    P, G = wl.prompt_len, wl.gen_len
    prompts = di.make_prompts(sh.vocab, 1, P, seed=1)
    toks = forced_string(sh.vocab, 1, prompts, P + G + 2)
    eng = pkg.Engine(engine_config(sh, P + G + 8), dev)
    orc = O.DmtdOracle(ocfg, w32, P + G + 8, np.float32)
    first = eng.prefill(prompts)
    orc.prefill(prompts[0])
    worst = norm_err(eng.logits()[0], orc.last_logits.astype(np.float64))
    checked = 0
    t0 = time.time()
    for _ in range(G - 1):
        worst, checked = _step_and_compare(eng, {0: orc}, toks, wl.tau, wl.n_late, worst, checked)
    assert worst < TOL_BF16, worst
    s = eng.state()
    assert s["n_tok"] == P + G - 1 and s["n_emitted"] == G - 1
    print(f"C3 whole run: worst {worst:.2e}, tokens checked {checked} of {G - 1}, {time.time() - t0:.0f} s")


@pytest.mark.parametrize("use_graphs", [True, False])
def test_decode_across_a_context_bucket(use_graphs):
    """A prompt of 505 tokens, 28 decode steps through dmtd_decode (cycles captured as one graph each): the context
    grows from 506 to 533 keys, so the attention launch shape changes at 512 - a new graph per step kind, and the group
    of steps that straddles the boundary is split.  Every step's token and each call's last logits against the float64
    oracle, the caches at the end; then the same decoding on a second engine through single-step calls, bit for bit."""
    sh = di.ModelShape(4, 256, 8, 2, 128, 512, 1000, dtype="bf16")
    B, P, tau, n_late, calls = 2, 505, 3, 2, (5, 6, 9, 8)
    blob = di.make_weight_blob(sh, seed=3)
    prompts = di.make_prompts(sh.vocab, B, P, seed=5)
    total = P + sum(calls) + 1
    toks = forced_string(sh.vocab, B, prompts, total)
    p = Pair(sh, blob, total + 2, batch=B, use_graphs=use_graphs)
    p.prefill(prompts)
    single = pkg.Engine(engine_config(sh, total + 2, B, use_graphs=use_graphs), blob)
    single.prefill(prompts)
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
            while done < n:
                done += len(o.decode_cycle(tau, n_late, max_new=n - done, forced=f[b][done:].tolist()))
            refs = o.step_logits[n0:]
            for i, ref in enumerate(refs):
                if top2_margin(ref.astype(np.float64)) > MARGIN:
                    assert int(out[b, i]) == int(np.argmax(ref)), (b, i)
                    checked += 1
            worst = max(worst, norm_err(z[b], refs[-1].astype(np.float64)))
        want = np.concatenate([single.decode_cycle(tau, n_late, max_new=1, forced=f[:, i:i + 1]) for i in range(n)], axis=1)
        assert np.array_equal(out, want)
        assert np.array_equal(z, single.logits())
    assert p.eng.state()["n_tok"] > 512 + 16
    assert worst < TOL_BF16, worst
    assert checked > 0
    p.compare_kv(2e-2)
    print(f"bucket crossing (graphs={use_graphs}): worst {worst:.2e}, tokens checked {checked}")


@pytest.mark.parametrize("order", [(4, 2), (2, 4), (3, 1, 4)])
@pytest.mark.parametrize("name", ["bf16", "fp32"])
def test_reset_then_prefill_with_another_batch(name, order):
    """One context (max_batch = 4, graphs on) used for batches of different sizes in turn, with dmtd_reset in between:
    every batch decodes through dmtd_decode_cycle and through dmtd_decode and is compared with per-sequence oracles.
    A captured step carries the batch size in its grids and in the layout of the emitted tokens, so a graph captured
    for one batch must not be replayed for another."""
    sh = (di.ModelShape(3, 256, 4, 2, 64, 512, 700, dtype="bf16") if name == "bf16"
          else di.ModelShape(3, 128, 4, 2, 64, 192, 130, dtype="fp32"))
    tol = TOL_BF16 if name == "bf16" else TOL_F32
    P, tau, n_late = 24, 3, 1
    blob = di.make_weight_blob(sh, seed=7)
    ocfg = oracle_config(sh)
    w = O.unpack_weights(blob, ocfg, np.float64)
    eng = pkg.Engine(engine_config(sh, P + 40, 4), blob)
    worst, checked = 0.0, 0
    for round_no, B in enumerate(order):
        if round_no:
            eng.reset()
        prompts = di.make_prompts(sh.vocab, B, P, seed=20 + round_no)
        toks = forced_string(sh.vocab, B, prompts, P + 40, seed=500 + round_no)
        orcs = [O.DmtdOracle(ocfg, w, P + 40, np.float64) for _ in range(B)]
        first = eng.prefill(prompts)
        z = eng.logits()
        assert z.shape[0] == B
        for b, o in enumerate(orcs):
            o.prefill(prompts[b])
            worst = max(worst, norm_err(z[b], o.last_logits.astype(np.float64)))
            if top2_margin(o.last_logits.astype(np.float64)) > MARGIN:
                assert int(first[b]) == int(np.argmax(o.last_logits))
        for call, n in enumerate((tau - 1, tau, 2 * tau + 1, tau)):
            nt = eng.state()["n_tok"]
            f = np.stack([toks[b][nt:nt + n] for b in range(B)])
            out = eng.decode(tau, n_late, n, forced=f) if call >= 2 else eng.decode_cycle(tau, n_late, forced=f)
            assert out.shape == (B, n)
            z = eng.logits()
            for b, o in enumerate(orcs):
                n0 = len(o.step_logits)
                done = 0
                while done < n:
                    done += len(o.decode_cycle(tau, n_late, max_new=n - done, forced=f[b][done:].tolist()))
                refs = o.step_logits[n0:]
                for i, ref in enumerate(refs):
                    if top2_margin(ref.astype(np.float64)) > MARGIN:
                        assert int(out[b, i]) == int(np.argmax(ref)), (round_no, b, i)
                        checked += 1
                worst = max(worst, norm_err(z[b], refs[-1].astype(np.float64)))
                assert int(out[b, -1]) == int(np.argmax(z[b]))
    assert worst < tol, worst
    assert checked > 0
    print(f"reset with batches {order} ({name}): worst {worst:.2e}, tokens checked {checked}")
