"""Host-side checks of the C ABI that need no GPU: exported symbols, argument validation,
and the cycle scheduler (run in the library's dry-run mode, which launches nothing)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2510_11958_amd as pkg
from paper_2510_11958_amd.binding import _Config

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLDEN = os.path.join(ROOT, "tests", "golden")


def dry(n_layers=4, max_seq_len=64, max_batch=1, **kw):
    return pkg.Engine(pkg.ModelConfig(n_layers, 64, 4, 2, 64, 96, 50, dtype="fp32", max_seq_len=max_seq_len,
                                      max_batch=max_batch, dry_run=True, **kw))


def test_every_declared_symbol_is_exported():
    header = open(os.path.join(ROOT, "include", "dmtd.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(dmtd_[a-z_]+)\s*\(", header))
    assert {"dmtd_create", "dmtd_prefill", "dmtd_decode_cycle", "dmtd_logits"} <= names
    lib = pkg.load_library()
    for n in names:
        assert hasattr(lib, n), n


def test_config_struct_matches_header_order():
    header = open(os.path.join(ROOT, "include", "dmtd.h")).read()
    body = header[header.index("typedef struct dmtd_config {"):header.index("} dmtd_config;")]
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"\b(?:int32_t|float|void\*)\s+([a-z_]+);", body)
    assert fields == [f[0] for f in _Config._fields_]


def test_invalid_configurations_are_rejected():
    lib = pkg.load_library()
    good = pkg.ModelConfig(4, 64, 4, 2, 64, 96, 50, dtype="fp32", dry_run=True)
    assert lib.dmtd_workspace_bytes(C.byref(good.to_c())) > 0
    for field, val in [("n_layers", 0), ("hidden", 60), ("head_dim", 48), ("n_q_heads", 3), ("max_seq_len", 1),
                       ("max_batch", 0), ("intermediate", 100), ("vocab", 1)]:
        bad = pkg.ModelConfig(**{**good.__dict__, field: val})
        assert lib.dmtd_workspace_bytes(C.byref(bad.to_c())) == 0, field
        with pytest.raises(pkg.DmtdError) as e:
            pkg.Engine(bad)
        assert e.value.code == pkg.DMTD_EINVAL
    # without dry_run, null device pointers are an argument error (no HIP call is made)
    h = C.c_void_p()
    real = pkg.ModelConfig(**{**good.__dict__, "dry_run": False})
    assert lib.dmtd_create(C.byref(real.to_c()), None, 0, None, 0, C.byref(h)) == pkg.DMTD_EINVAL
    assert b"null" in lib.dmtd_last_error(None)


def test_fig3_schedule_from_the_library_scheduler():
    want = []
    for line in open(os.path.join(GOLDEN, "fig3_schedule.txt")):
        if line.strip() and not line.startswith("#"):
            f = line.split()
            want.append((int(f[0]), f[1], [int(x) for x in f[2:]]))
    e = dry()
    e.prefill([[1, 2, 3, 4, 5]])
    assert e.decode_cycle(3, 1).shape == (1, 2)     # cycle 1: prefill's token + two late-only steps
    assert e.decode_cycle(3, 1).shape == (1, 3)
    assert e.decode_cycle(3, 1, max_new=1).shape == (1, 1)
    assert e.trace() == want
    s = e.state()
    assert (s["n_tok"], s["n_front"], s["phase"], s["n_emitted"], s["n_full_steps"]) == (11, 11, 1, 6, 2)


@pytest.mark.parametrize("L,n_late,tau", [(36, 8, 3), (36, 8, 4), (28, 4, 2), (4, 1, 2), (36, 12, 4), (36, 8, 1)])
def test_layer_visit_counters_give_eq7(L, n_late, tau):
    e = dry(n_layers=L, max_seq_len=256)
    e.prefill([[1, 2, 3]])
    e.decode_cycle(tau, n_late)
    s0 = e.state()
    for _ in range(7):
        assert e.decode_cycle(tau, n_late).shape[1] == tau
    s1 = e.state()
    toks = s1["n_emitted"] - s0["n_emitted"]
    plt = (s1["gen_layer_visits"] - s0["gen_layer_visits"]) / (toks * L)
    assert plt == pytest.approx((L + (tau - 1) * n_late) / (tau * L), abs=1e-15)
    if (L, n_late, tau) == (36, 8, 3):      # the values the paper prints for MTD3 (Sec. 3.4)
        assert abs(plt - 0.48) < 0.005 and abs(1 / plt - 2.08) < 0.005
    # same total load as the vanilla model (Sec. 2.2): each consumed token crosses every layer once
    consumed = s1["n_tok"] - 3
    total = s1["gen_layer_visits"] + s1["refill_layer_visits"]
    assert total == consumed * L - (s1["n_tok"] - s1["n_front"]) * (L - n_late)


@pytest.mark.parametrize("tau,n_early,n_late", [(3, 2, 1), (4, 1, 2), (2, 3, 3), (3, 0, 2), (5, 2, 2)])
def test_exdy_schedule_matches_the_oracle_machine(tau, n_early, n_late):
    """ExDy variant: the library's scheduler (dry run) and the oracle's cycle machine visit the same
    (pass, layer group, positions), count the same layer visits, and give Eq. 7 with L_d = x + y."""
    import dmtd_inputs as di
    from oracle import dmtd_oracle as O
    L = 6
    sh = di.ModelShape(L, 64, 4, 2, 16, 96, 50, dtype="fp32")
    ocfg = O.OracleConfig(L, 64, 4, 2, 16, 96, 50)
    orc = O.DmtdOracle(ocfg, O.unpack_weights(di.make_weight_blob(sh, seed=1, std=0.1), ocfg), 64)
    e = dry(n_layers=L)
    e.set_n_early(n_early)
    e.prefill([[1, 2, 3, 4]])
    orc.prefill([1, 2, 3, 4], n_early=n_early)
    for _ in range(4):
        n = e.decode_cycle(tau, n_late).shape[1]
        assert len(orc.decode_cycle(tau, n_late, n_early=n_early)) == n
    want = [(i + 1, g, pos) for i, passes in enumerate(orc.trace) for g, pos in passes]
    got = e.trace()
    order = {"enc": 0, "front": 1, "late": 2}
    assert sorted(got, key=lambda t: (t[0], order[t[1]])) == sorted(want, key=lambda t: (t[0], order[t[1]]))
    s = e.state()
    assert (s["n_tok"], s["n_front"], s["gen_layer_visits"], s["refill_layer_visits"]) == \
        (orc.n_tok, orc.n_front, orc.gen_layer_visits, orc.refill_layer_visits)


def test_exdy_setting_errors():
    e = dry(n_layers=6)
    with pytest.raises(pkg.DmtdError) as ei:
        e.set_n_early(6)
    assert ei.value.code == pkg.binding.DMTD_EINVAL
    with pytest.raises(pkg.DmtdError):
        e.set_n_early(-1)
    e.set_n_early(2)
    e.prefill([[1, 2, 3]])
    with pytest.raises(pkg.DmtdError) as ei:
        e.decode_cycle(3, 5)                      # 2 + 5 > 6
    assert ei.value.code == pkg.binding.DMTD_EINVAL and e.state()["n_tok"] == 3
    e.decode_cycle(3, 2)                          # two late steps: tokens await refill
    with pytest.raises(pkg.DmtdError) as ei:
        e.set_n_early(1)
    assert ei.value.code == pkg.binding.DMTD_ESTATE
    e.decode_cycle(3, 2, max_new=1)               # the full step refills them
    e.set_n_early(1)
    e.reset()
    e.prefill([[1, 2, 3]])
    e.decode_cycle(2, 4)
    assert ("enc", [3]) in [(g, p) for _, g, p in e.trace()]      # the setting survived the reset


def test_state_and_argument_errors_leave_state_unchanged():
    e = dry(max_seq_len=8)
    with pytest.raises(pkg.DmtdError) as ex:
        e.decode_cycle(2, 1)
    assert ex.value.code == pkg.DMTD_ESTATE
    with pytest.raises(pkg.DmtdError) as ex:
        e.prefill([[1, 2, 99]])
    assert ex.value.code == pkg.DMTD_EINVAL and e.state()["n_tok"] == 0
    with pytest.raises(pkg.DmtdError) as ex:
        e.prefill([[1] * 8])
    assert ex.value.code == pkg.DMTD_ECAPACITY
    with pytest.raises(pkg.DmtdError) as ex:
        e.prefill([[1, 2], [3, 4]])          # batch above max_batch
    assert ex.value.code == pkg.DMTD_EINVAL
    e.prefill([[1, 2, 3, 4, 5, 6]])
    with pytest.raises(pkg.DmtdError) as ex:
        e.prefill([[1, 2, 3]])
    assert ex.value.code == pkg.DMTD_ESTATE
    before = e.state()
    for tau, n_late, code in [(0, 1, pkg.DMTD_EINVAL), (2, 0, pkg.DMTD_EINVAL), (2, 5, pkg.DMTD_EINVAL),
                              (65, 1, pkg.DMTD_EINVAL), (4, 1, pkg.DMTD_ECAPACITY)]:
        with pytest.raises(pkg.DmtdError) as ex:
            e.decode_cycle(tau, n_late)
        assert ex.value.code == code
        assert e.state() == before
    with pytest.raises(pkg.DmtdError) as ex:
        e.decode_cycle(2, 1, forced=[[77]])
    assert ex.value.code == pkg.DMTD_EINVAL and e.state() == before
    with pytest.raises(pkg.DmtdError) as ex:
        e.logits()
    assert ex.value.code == pkg.DMTD_ESTATE
    e.decode_cycle(2, 1)                      # one late step: a token now awaits refill
    with pytest.raises(pkg.DmtdError) as ex:
        e.decode_cycle(2, 2)                  # n_late may not change now
    assert ex.value.code == pkg.DMTD_ESTATE
    e.decode_cycle(1, 1)
    with pytest.raises(pkg.DmtdError) as ex:
        e.decode_cycle(1, 1)
    assert ex.value.code == pkg.DMTD_ECAPACITY
    e.reset()
    assert e.state()["n_tok"] == 0 and e.trace() == []
    e.prefill([[1, 2, 3]])
    e.decode_cycle(1, 2)                      # after a reset n_late is free again


def test_out_stride_and_null_outputs():
    lib = pkg.load_library()
    e = dry()
    e.prefill([[1, 2, 3]])
    out = np.empty(2, np.int32)
    n = C.c_int32()
    p = out.ctypes.data_as(C.POINTER(C.c_int32))
    assert lib.dmtd_decode_cycle(e._h, 4, 1, 0, None, 0, p, 2, C.byref(n)) == pkg.DMTD_ECAPACITY
    assert lib.dmtd_decode_cycle(e._h, 4, 1, 0, None, 0, None, 4, C.byref(n)) == pkg.DMTD_EINVAL
    assert lib.dmtd_decode_cycle(e._h, 4, 1, 2, None, 0, p, 2, C.byref(n)) == pkg.DMTD_OK and n.value == 2
    assert e.state()["phase"] == 3


def test_long_cycles_refill_all_pending_rows():
    e = dry(max_seq_len=128)
    e.prefill([[1, 2, 3]])
    e.decode_cycle(12, 1)          # 11 late steps: 11 tokens await refill
    assert e.state()["n_tok"] - e.state()["n_front"] == 11
    e.decode_cycle(12, 1, max_new=1)
    assert e.trace()[-2:] == [(13, "front", list(range(3, 15))), (13, "late", [14])]
    assert e.state()["n_tok"] == e.state()["n_front"] == 15


def test_masked_forward_argument_checks_without_a_gpu():
    """Argument validation of dmtd_masked_forward runs before any device work (dry-run context)."""
    e = dry(max_seq_len=16, max_batch=2)
    ok_t, ok_m = np.ones((2, 8), np.int32), np.ones(8, np.uint8)
    for toks, mask, n_late, code in [
            (ok_t, ok_m, 0, pkg.DMTD_EINVAL), (ok_t, ok_m, 5, pkg.DMTD_EINVAL),
            (np.full((2, 8), 50, np.int32), ok_m, 1, pkg.DMTD_EINVAL),
            (np.ones((3, 8), np.int32), ok_m, 1, pkg.DMTD_EINVAL),
            (np.ones((1, 17), np.int32), np.ones(17, np.uint8), 1, pkg.DMTD_ECAPACITY),
            (ok_t, ok_m, 1, pkg.DMTD_ESTATE)]:             # valid arguments: only the dry run itself is refused
        with pytest.raises(pkg.DmtdError) as err:
            e.masked_forward(toks, mask, n_late)
        assert err.value.code == code
    e.set_n_early(2)
    with pytest.raises(pkg.DmtdError) as err:
        e.masked_forward(ok_t, ok_m, 3)                   # n_early + n_late > n_layers
    assert err.value.code == pkg.DMTD_EINVAL
    e.set_n_early(0)
    e.prefill([[1, 2, 3], [4, 5, 6]])
    with pytest.raises(pkg.DmtdError) as err:
        e.masked_forward(ok_t, ok_m, 1)
    assert err.value.code == pkg.DMTD_ESTATE


def test_ragged_prefill_argument_checks_and_schedule_without_a_gpu():
    e = dry(max_seq_len=32, max_batch=3)
    toks = np.ones((3, 8), np.int32)
    for lengths in ([8, 0, 3], [8, 9, 3], [7, 7, 3]):
        with pytest.raises(pkg.DmtdError) as err:
            e.prefill(toks, lengths=lengths)
        assert err.value.code == pkg.DMTD_EINVAL
    e.prefill(toks, lengths=[8, 2, 5])
    e.decode_cycle(3, 1)
    s = e.state()
    assert (s["n_tok"], s["n_front"], s["phase"]) == (10, 8, 3)     # the longest sequence's counters


def test_build_refuses_spilling_matrix_core_kernels():
    """build_library() reads the compiler's resource-usage remarks: a *_mfma_kernel with scratch is reported, others are not."""
    from paper_2510_11958_amd.build import spilling_mfma_kernels
    remarks = "\n".join([
        "x.hip:1:1: remark: Function Name: _ZN4dmtd16gemv_mfma_kernelILi1ELb0ELi4ELi16ELb1EEEv [-Rpass-analysis=kernel-resource-usage]",
        "x.hip:1:1: remark:     VGPRs: 128 [-Rpass-analysis=kernel-resource-usage]",
        "x.hip:1:1: remark:     ScratchSize [bytes/lane]: 516 [-Rpass-analysis=kernel-resource-usage]",
        "x.hip:2:1: remark: Function Name: _ZN4dmtd16gemv_rows_kernelIfLi1EEEv [-Rpass-analysis=kernel-resource-usage]",
        "x.hip:2:1: remark:     ScratchSize [bytes/lane]: 32 [-Rpass-analysis=kernel-resource-usage]",
        "x.hip:3:1: remark: Function Name: _ZN4dmtd22attn_split_mfma_kernelILi128EEEv [-Rpass-analysis=kernel-resource-usage]",
        "x.hip:3:1: remark:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis=kernel-resource-usage]",
    ])
    bad = spilling_mfma_kernels(remarks)
    assert len(bad) == 1 and "gemv_mfma_kernel" in bad[0] and "516" in bad[0]
    assert spilling_mfma_kernels("") == []


@pytest.mark.parametrize("tau,n_steps,chunks", [(3, 7, (7,)), (3, 11, (4, 1, 6)), (1, 5, (2, 3)), (4, 64, (64,)), (2, 9, (3, 3, 3))])
def test_cycles_back_to_back_schedule_like_single_cycle_calls(tau, n_steps, chunks):
    """dmtd_decode (Sec. 2.2, cycles back to back) runs the steps repeated dmtd_decode_cycle calls would run: same
    schedule trace (Fig. 3), same counters, same state, also when a call ends inside a cycle."""
    a, b = dry(max_seq_len=128), dry(max_seq_len=128)
    for e in (a, b):
        e.prefill([[1, 2, 3, 4, 5]])
    done = 0
    while done < n_steps:                      # reference: one call per cycle
        done += a.decode_cycle(tau, 2, max_new=n_steps - done).shape[1]
    assert sum(chunks) == n_steps
    for c in chunks:
        assert b.decode(tau, 2, c).shape == (1, c)
    assert a.state() == b.state() and a.trace() == b.trace()
    # and the two kinds of call continue each other's cycles
    a.decode(tau, 2, 2); b.decode_cycle(tau, 2, max_new=1); b.decode_cycle(tau, 2, max_new=1)
    assert a.state() == b.state() and a.trace() == b.trace()


def test_cycles_back_to_back_errors_leave_the_state_alone():
    e = dry(max_seq_len=12)
    e.prefill([[1, 2, 3, 4]])
    before, tr = e.state(), e.trace()
    for n_steps, code in [(0, pkg.DMTD_EINVAL), (65, pkg.DMTD_EINVAL), (9, pkg.DMTD_ECAPACITY)]:
        with pytest.raises(pkg.DmtdError) as ex:
            e.decode(3, 1, n_steps)            # 9 steps would pass max_seq_len in the third cycle: nothing may run
        assert ex.value.code == code and e.state() == before and e.trace() == tr
    with pytest.raises(pkg.DmtdError) as ex:
        e.decode(0, 1, 2)
    assert ex.value.code == pkg.DMTD_EINVAL
    lib = pkg.load_library()
    out = np.empty(4, np.int32); n = C.c_int32()
    p = out.ctypes.data_as(C.POINTER(C.c_int32))
    assert lib.dmtd_decode(e._h, 3, 1, 5, None, 0, p, 4, C.byref(n)) == pkg.DMTD_ECAPACITY      # out_stride < n_steps
    assert e.state() == before
    assert e.decode(3, 1, 8).shape == (1, 8) and e.state()["n_tok"] == 12


def test_per_sequence_cycle_lengths_schedule_like_one_oracle_per_sequence():
    """dmtd_decode_per_seq in a dry run: every sequence's phase and refill point follow a standalone oracle machine run with
    that sequence's cycle lengths; the single-phase calls are refused while the sequences differ and accepted once they
    agree again; the counters and the trace follow sequence 0."""
    import dmtd_inputs as di
    from oracle import dmtd_oracle as O
    sh = di.ModelShape(5, 32, 2, 1, 16, 48, 40, dtype="fp32")
    cfg = O.OracleConfig(sh.n_layers, sh.hidden, sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.intermediate, sh.vocab)
    w = O.unpack_weights(di.make_weight_blob(sh, seed=1, std=0.2), cfg)
    B, P, n_late = 3, 4, 2
    eng = dry(n_layers=sh.n_layers, max_batch=B)          # only the schedule is compared: the engine's shape need not be the oracle's
    eng.prefill(np.zeros((B, P), np.int32))
    orcs = [O.DmtdOracle(cfg, w, 64) for _ in range(B)]
    for o in orcs:
        o.prefill([1, 2, 3, 4])
    for taus, n in (([2, 3, 5], 7), ([2, 3, 5], 2), ([4, 4, 4], 6), ([1, 6, 2], 5)):
        out = eng.decode_per_seq(taus, n_late, n)
        assert out.shape == (B, n)
        for b, o in enumerate(orcs):
            done = 0
            while done < n:
                done += len(o.decode_cycle(taus[b], n_late, max_new=n - done))
            s = eng.seq_state(b)
            assert (eng.state()["n_tok"], s["n_front"], s["phase"]) == (o.n_tok, o.n_front, o.phase), (taus, b)
    s0, o0 = eng.state(), orcs[0]
    assert (s0["gen_layer_visits"], s0["refill_layer_visits"], s0["n_emitted"]) == (o0.gen_layer_visits, o0.refill_layer_visits, o0.n_emitted)
    assert eng.trace() == [(p + 1, g, pos) for p, t in enumerate(o0.trace) for g, pos in t]
    with pytest.raises(pkg.DmtdError) as e:
        eng.decode_cycle(3, n_late)
    assert e.value.code == pkg.DMTD_ESTATE
    # argument errors leave everything alone
    before = [eng.seq_state(b) for b in range(B)]
    for bad_taus, n, code in (([2, 0, 3], 3, pkg.DMTD_EINVAL), ([2, 3, 65], 3, pkg.DMTD_EINVAL), ([2, 3, 4], 0, pkg.DMTD_EINVAL),
                              ([2, 3, 4], 65, pkg.DMTD_EINVAL), ([30, 30, 30], 40, pkg.DMTD_ECAPACITY)):
        with pytest.raises(pkg.DmtdError) as e:
            eng.decode_per_seq(bad_taus, n_late, n)
        assert e.value.code == code, bad_taus
    assert [eng.seq_state(b) for b in range(B)] == before
    # a cycle longer than the rows a pass can carry (16) cannot be refilled in one pass
    eng.reset()
    eng.prefill(np.zeros((B, P), np.int32))
    eng.decode_per_seq([20, 2, 2], n_late, 19)
    with pytest.raises(pkg.DmtdError) as e:
        eng.decode_per_seq([20, 2, 2], n_late, 1)
    assert e.value.code == pkg.DMTD_ECAPACITY
