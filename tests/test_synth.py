"""The synthetic workloads have the shapes and structure the benchmark names."""
import numpy as np
import pytest

from paper_2605_00392_amd import synth


def test_workload_shapes_and_determinism():
    b1 = synth.gen_batch(1)
    assert b1.tokens.dtype == np.float32 and b1.tokens.shape == (64, 1280) and b1.batch == 1
    b2 = synth.gen_batch(2, images=[0, 5])
    assert b2.tokens.dtype == np.uint16 and b2.tokens.shape == (512, 1280)
    again = synth.gen_batch(2, images=[5])
    np.testing.assert_array_equal(again.tokens, b2.tokens[256:])
    b4 = synth.gen_batch(4, images=range(12))
    counts = np.diff(b4.offsets)
    assert ((counts - 256) % 100 == 0).all() and counts.min() >= 456 and counts.max() <= 1156
    assert b4.offsets[0] == 0 and b4.offsets.dtype == np.int32
    assert [synth.image_token_count(4, i) for i in range(12)] == list(counts)
    assert (b4.density >= 0.1).all() and (b4.density <= 0.9).all()
    assert synth.WORKLOADS[5].batch == 1024 and synth.WORKLOADS[5].params["iters"] == 100


def test_value_structure():
    x, _ = synth.gen_image(2, 3)
    n = np.linalg.norm(x, axis=1)
    assert (n > 3.0).sum() == 25                      # floor(0.1 * 256) outliers x4
    assert abs(np.median(n) - np.sqrt(1 + 0.04)) < 0.02
    x5, rho = synth.gen_image(5, 0)
    u = x5 / np.linalg.norm(x5, axis=1, keepdims=True)
    c = u @ u.T
    np.fill_diagonal(c, 0)
    assert (c.max(axis=1) > 0.98).sum() >= 120        # 30 % near-copies (and their sources)
    assert 0.1 <= rho <= 0.9
    x1, _ = synth.gen_image(1, 0)
    assert x1.shape == (64, 1280) and (np.linalg.norm(x1, axis=1) > 0).all()


def test_bf16_encoding_round_trip():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(0)
    x = rng.standard_normal(10000).astype(np.float32)
    bits = synth.f32_to_bf16_bits(x)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(bits, want)
    np.testing.assert_array_equal(synth.bf16_bits_to_f32(bits),
                                  torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_subset_repacks():
    b = synth.gen_batch(4, images=range(4))
    s = synth.subset(b, [2, 0])
    assert s.batch == 2 and s.images == [2, 0]
    np.testing.assert_array_equal(s.tokens[: s.offsets[1]], b.tokens[b.offsets[2]: b.offsets[3]])


def test_parallel_generation_gives_the_same_batch():
    """Every image is drawn from its own seed, so spreading the drawing over worker
    processes changes nothing (workload 4: 128 ragged pages)."""
    a = synth.gen_batch(4)
    b = synth.gen_batch_parallel(4, workers=3)
    np.testing.assert_array_equal(a.offsets, b.offsets)
    np.testing.assert_array_equal(a.tokens, b.tokens)
    np.testing.assert_array_equal(a.density, b.density)
    assert a.params == b.params and a.images == b.images
