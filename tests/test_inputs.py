"""The seeded input generators: determinism, independence of chunking, value distributions."""
import numpy as np
import torch

import dmtd_inputs as di


def test_splitmix_reference_values():
    # SplitMix64 with state 0: the first outputs are the widely published test vector.
    z = di._mix(np.uint64(0) + np.arange(1, 4, dtype=np.uint64) * di._GOLDEN)
    assert [int(v) for v in z] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]


def test_slices_are_independent_of_chunking():
    a = di.raw_u64(7, 3, 0, 1000)
    b = np.concatenate([di.raw_u64(7, 3, 0, 333), di.raw_u64(7, 3, 333, 667)])
    assert np.array_equal(a, b)
    n1 = di._normal_chunk(7, 3, 0, 1000)
    n2 = np.concatenate([di._normal_chunk(7, 3, 0, 400), di._normal_chunk(7, 3, 400, 600)])
    assert np.array_equal(n1, n2)
    assert not np.array_equal(di.raw_u64(7, 3, 0, 16), di.raw_u64(7, 4, 0, 16))
    assert not np.array_equal(di.raw_u64(7, 3, 0, 16), di.raw_u64(8, 3, 0, 16))


def test_blob_is_reproducible_and_thread_independent():
    sh = di.ModelShape(2, 64, 4, 2, 16, 96, 50, dtype="bf16")
    a = di.make_weight_blob(sh, seed=0, threads=1)
    b = di.make_weight_blob(sh, seed=0, threads=4)
    assert a.dtype == np.uint16 and np.array_equal(a, b)
    assert a.size == di.blob_elems(sh)
    assert not np.array_equal(a, di.make_weight_blob(sh, seed=1))


def test_normal_statistics_and_gains():
    sh = di.WORKLOADS["C1"].shape
    blob = di.make_weight_blob(sh, seed=0)
    emb = blob[: sh.vocab * sh.hidden]
    assert abs(float(emb.mean())) < 3e-4
    assert abs(float(emb.std()) - 0.02) < 3e-4
    # kurtosis of a normal is 3
    assert abs(float(np.mean((emb / emb.std()) ** 4)) - 3.0) < 0.1
    # first gain vector follows the table and is all ones in the benchmark configurations
    g = blob[sh.vocab * sh.hidden: sh.vocab * sh.hidden + sh.hidden]
    assert np.all(g == 1.0)
    blob2 = di.make_weight_blob(sh, seed=0, gain_sigma=0.1)
    g2 = blob2[sh.vocab * sh.hidden: sh.vocab * sh.hidden + sh.hidden]
    assert abs(float(g2.mean()) - 1.0) < 0.03 and 0.07 < float(g2.std()) < 0.13


def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(100000).astype(np.float32) * 0.02,
                        np.array([1.0, -1.0, 0.0, 1.00390625, 1.01171875, 3.0e38, 1e-40], np.float32)])
    ours = di.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, ref)
    back = di.bf16_bits_to_f32(ours)
    assert np.array_equal(back, torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_prompts_uniform_and_per_sequence():
    p = di.make_prompts(1024, 3, 4096, seed=1)
    assert p.shape == (3, 4096) and p.dtype == np.int32
    assert p.min() >= 0 and p.max() < 1024
    assert not np.array_equal(p[0], p[1])
    assert np.array_equal(p[1], di.make_prompts(1024, 1, 4096, seed=2)[0])
    counts = np.bincount(p.ravel(), minlength=1024)
    assert counts.min() > 0 and counts.max() < 40   # mean 12


def test_workload_sizes_match_the_named_configurations():
    assert di.blob_elems(di.WORKLOADS["C1"].shape) == 3_410_688
    assert di.blob_elems(di.WORKLOADS["C2"].shape) == 596_049_920
    s = di.WORKLOADS["C3"].shape
    per_layer = 2 * s.hidden + 2 * s.head_dim + s.hidden * (s.n_q_heads + 2 * s.n_kv_heads) * s.head_dim \
        + s.hidden * s.n_q_heads * s.head_dim + 3 * s.hidden * s.intermediate
    assert di.blob_elems(s) == s.vocab * s.hidden + s.n_layers * per_layer + s.hidden
