"""Pins for the oracle's 16-bit float converters: every code point against numpy / the format's definition."""
import numpy as np
import pytest

F16, BF16 = 0, 1


def test_f16_decode_all_words(oracle):
    words = np.arange(65536, dtype=np.uint16)
    got = oracle.to_f32(words, F16)
    want = words.view(np.float16).astype(np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))


def test_bf16_decode_all_words(oracle):
    words = np.arange(65536, dtype=np.uint16)
    got = oracle.to_f32(words, BF16)
    want = (words.astype(np.uint32) << 16).view(np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))


def _probe_values(rng):
    x = np.concatenate([
        rng.standard_normal(20000).astype(np.float32) * 10,
        rng.standard_normal(5000).astype(np.float32) * 1e-6,      # binary16 subnormal range
        rng.standard_normal(5000).astype(np.float32) * 3e4,
        np.array([0.0, -0.0, 65504.0, 65519.9, 65520.0, 1e9, -1e9, 2.0 ** -24, 2.0 ** -25, 1.5 * 2.0 ** -25,
                  2.0 ** -14, 2.0 ** -14 - 2.0 ** -25, 1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11,
                  1.0 + 2.0 ** -11 + 2.0 ** -20], dtype=np.float32),
    ])
    # exact halfway cases between every pair of neighbouring binary16 values in [1, 2)
    h = np.arange(0x3C00, 0x4000, dtype=np.uint16).view(np.float16).astype(np.float32)
    return np.concatenate([x, (h[:-1] + h[1:]) / 2])


def test_f16_encode_rne(oracle):
    x = _probe_values(np.random.default_rng(1))
    got = oracle.from_f32(x, F16)
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    assert np.array_equal(got, want)


def test_bf16_encode_rne(oracle):
    torch = pytest.importorskip("torch")
    x = _probe_values(np.random.default_rng(2))
    h = (np.arange(0x3F80, 0x4000, dtype=np.uint32) << 16).view(np.float32)
    x = np.concatenate([x, (h[:-1] + h[1:]) / 2])
    got = oracle.from_f32(x, BF16)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, want)


def test_generator_rounding_matches_oracle_words(oracle):
    """The input generator's 16-bit rounding yields words the oracle decodes to the nearest value."""
    from paper_2508_08256_amd import synth

    x = np.random.default_rng(3).standard_normal(4096).astype(np.float32) * 5
    for dt in (F16, BF16):
        w = synth.f32_to_words(x, dt)
        assert np.array_equal(w, oracle.from_f32(x, dt))
        assert np.array_equal(synth.words_to_f32(w, dt), oracle.to_f32(w, dt))
