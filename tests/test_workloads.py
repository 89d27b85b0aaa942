"""The seeded input generators (no GPU, no oracle arithmetic): same seed -> same bits, the shapes
the benchmark is quoted on, and the one-time bf16 rounding against an independent conversion."""
import numpy as np
import torch

from paper_2602_11812_amd import workloads as wl


def test_bf16_rounding_is_nearest_even_and_widening_is_exact():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(4096).astype(np.float32) * np.float32(10.0) ** rng.integers(-6, 6, 4096),
                        np.array([0.0, -0.0, 1.0, 1.0 + 2.0 ** -8, 1.0 + 2.0 ** -7, 1.0 + 3 * 2.0 ** -8, 65504.0, 3.0e38],
                                 dtype=np.float32)])
    bits = wl.to_bf16_bits(x)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, want)
    # ties go to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7 -> 1; 1 + 3*2^-8 -> 1 + 2^-6
    assert wl.bf16_bits_to_f32(wl.to_bf16_bits(np.array([1.0 + 2.0 ** -8], np.float32)))[0] == 1.0
    assert wl.bf16_bits_to_f32(wl.to_bf16_bits(np.array([1.0 + 3 * 2.0 ** -8], np.float32)))[0] == 1.0 + 2.0 ** -6
    back = wl.bf16_bits_to_f32(bits)
    assert np.array_equal(back, torch.from_numpy(want.view(np.int16)).view(torch.bfloat16).float().numpy())


def test_same_seed_same_bits_and_different_seed_differs():
    spec = wl.scaled(wl.SPECS["mid"], B=4, d=64, V=300, d_h=16)
    a, b = wl.make(spec), wl.make(spec)
    for name in ("lengths", "hidden", "w_lm", "w1", "w2"):
        assert np.array_equal(getattr(a, name), getattr(b, name)), name
    c = wl.make(wl.scaled(spec, seed=spec.seed + 1))
    assert not np.array_equal(a.hidden[:8], c.hidden[:8])


def test_workload_shapes_and_the_benchmark_batch():
    t = wl.make(wl.SPECS["tiny"])
    assert t.lengths.tolist() == [17, 64, 100, 128] and t.T == 309
    assert t.hidden.dtype == np.float32 and t.hidden.shape == (309, 256) and t.w_lm.shape == (4096, 256)
    s = wl.SPECS["serving"]
    lens = wl.draw_lengths(s, np.random.default_rng(s.seed))
    assert lens.size == 128 and int(lens.sum()) == 137720            # the batch the throughput is quoted on
    assert lens.min() >= 32 and lens.max() <= 8192
    assert (s.d, s.V, s.d_h, s.dtype) == (4096, 151936, 1024, "bf16")
    m = wl.make(wl.scaled(wl.SPECS["mid"], B=3, d=64, V=200, d_h=8))
    assert m.hidden.dtype == np.uint16 and m.w_lm.dtype == np.uint16 and m.hidden.shape == (m.T, 64)


def test_decode_and_continuation_draws():
    spec = wl.scaled(wl.SPECS["plp_decode"], B=8, d=64, V=100, d_h=8, lengths=tuple([1] * 8))
    a, b = wl.decode_hidden(spec, 3), wl.decode_hidden(spec, 3)
    assert a.shape == (8, 64) and np.array_equal(a, b)
    assert not np.array_equal(a, wl.decode_hidden(spec, 4))
    c = wl.rl_continuations(wl.SPECS["rl_prompts"], 16)
    assert c.size == 64 * 16 and c.min() >= 1 and c.max() <= 16384
    assert 0 < np.mean(c < 64) < 0.5 and np.mean(c >= 128) > 0.5     # some samples end early, most go on


def test_training_set_recipe():
    a = wl.make_train(5, B=40, d=32, d_h=16, K=20)
    b = wl.make_train(5, B=40, d=32, d_h=16, K=20)
    assert np.array_equal(a.x, b.x) and np.array_equal(a.y, b.y) and np.array_equal(a.w1, b.w1)
    assert a.bins.min() >= 0 and a.bins.max() < 20 and a.y.min() >= 1.0 and a.y.max() <= 2047.0
    width = 2048.0 / 20
    assert np.array_equal(a.bins, np.minimum((a.y / np.float32(width)).astype(np.int32), 19))
    assert np.allclose(a.centers, (np.arange(20) + 0.5) * width)
    p = wl.make_train(5, B=40, d=32, d_h=16, K=20, plp_seqs=7)
    assert p.n_seqs == 7 and p.steps.min() >= 1 and abs(float(np.sum(1.0 / (7 * p.steps))) - 1.0) < 1e-6
