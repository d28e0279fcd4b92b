"""The shared input generators: numpy and torch versions produce the same bits; basic distribution sanity."""
import numpy as np
import torch

from synth_inputs import prng, prng_torch
from synth_inputs.workloads import build_config


def test_torch_generator_matches_numpy_bit_for_bit():
    for tid, seed in ((0, 241002684), (3, 7)):
        a = prng.uniform_pm1(seed, tid, 5000)
        b = prng_torch.uniform_pm1(seed, tid, 5000, device="cpu").numpy()
        assert np.array_equal(a, b)
        a = prng.normal(seed, tid, 5000, 0.02)
        b = prng_torch.normal(seed, tid, 5000, 0.02, device="cpu").numpy()
        # log/cos may differ in the last ulp between numpy and torch; after rounding to the bf16 storage
        # dtype the workloads use, a handful of ties at most may differ, and never by more than one ulp
        assert np.allclose(a, b, rtol=1e-6, atol=0)
        ab, bb = prng.f32_to_bf16_bits(a), prng.f32_to_bf16_bits(b)
        assert np.mean(ab != bb) < 1e-3
        oh = prng.onehot(seed, tid, 300, 17)
        ot = prng_torch.onehot(seed, tid, 300, 17, device="cpu").numpy()
        assert np.array_equal(oh, ot)
    m = prng.causal_mask(6, 6)
    mt = prng_torch.make_tensor({"dist": "causal_mask"}, (6, 6), "f32", 0, 0, device="cpu").numpy()
    assert np.array_equal(m, mt)


def test_bf16_rounding_matches_torch():
    x = prng.normal(1, 2, 4096, 3.0)
    bits = prng.f32_to_bf16_bits(x)
    t = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, t)


def test_subrange_regeneration_and_moments():
    full = prng.uniform_pm1(5, 1, 10000)
    part = prng.uniform_pm1(5, 1, 100, start=1234)
    assert np.array_equal(full[1234:1334], part)
    g = prng.normal(5, 2, 200000, 2.0)
    assert abs(g.mean()) < 0.02 and abs(g.std() - 2.0) < 0.02
    assert abs(full.mean()) < 0.02 and full.min() >= -1 and full.max() < 1
    ints = prng.small_ints(5, 3, 1000)
    assert set(np.unique(ints)) <= {-2.0, -1.0, 0.0, 1.0, 2.0}


def test_every_config_builds_at_full_and_small_size():
    for n in range(1, 8):
        for small in (False, True):
            w = build_config(n, small=small)
            assert w.outputs and w.partitionings
            names = [v.name for v in w.vertices]
            for v in w.einsum_vertices():
                assert all(i in names[:names.index(v.name)] for i in v.inputs)     # topological order
