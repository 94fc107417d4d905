"""Pins of the oracle's draft-head input projection (Eq. 3: h = Linear(concat[e, f])).  CPU only."""
import numpy as np

from oracle import s4c_oracle as O
from paper_2506_14158_amd import synth


def test_equals_a_library_matmul_of_the_concatenation():
    rng = np.random.default_rng(0)
    for T, H, Hout in ((5, 16, 16), (33, 48, 20), (1, 8, 64)):
        e, f = rng.standard_normal((T, H)).astype(np.float32), rng.standard_normal((T, H)).astype(np.float32)
        W = rng.standard_normal((Hout, 2 * H)).astype(np.float32)
        b = rng.standard_normal(Hout).astype(np.float32)
        want = np.concatenate([e, f], axis=1).astype(np.float64) @ W.astype(np.float64).T + b
        np.testing.assert_allclose(O.draft_linear(e, f, W, b), want, rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(O.draft_linear(e, f, W), want - b, rtol=1e-12, atol=1e-12)


def test_selector_weights_and_bf16_decoding():
    rng = np.random.default_rng(1)
    T, H = 7, 32
    e, f = rng.standard_normal((T, H)).astype(np.float32), rng.standard_normal((T, H)).astype(np.float32)
    I, Z = np.eye(H, dtype=np.float32), np.zeros((H, H), dtype=np.float32)
    assert np.array_equal(O.draft_linear(e, f, np.hstack([I, Z])), e.astype(np.float64))       # picks e
    assert np.array_equal(O.draft_linear(e, f, np.hstack([Z, I])), f.astype(np.float64))       # picks f
    assert np.array_equal(O.draft_linear(e, f, np.hstack([I, -I])), e.astype(np.float64) - f)  # a swapped half would flip the sign
    eb, fb = synth.f32_to_bf16_bits(e), synth.f32_to_bf16_bits(f)
    Wb = synth.f32_to_bf16_bits(rng.standard_normal((H, 2 * H)).astype(np.float32))
    want = np.concatenate([synth.bf16_bits_to_f32(eb), synth.bf16_bits_to_f32(fb)], 1).astype(np.float64) @ \
        synth.bf16_bits_to_f32(Wb).astype(np.float64).T
    np.testing.assert_allclose(O.draft_linear(eb, fb, Wb), want, rtol=1e-12, atol=1e-12)
