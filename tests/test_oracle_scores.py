"""Pins of the oracle's activation magnitudes and layer scores (paper, Algorithm 1)."""
import numpy as np

import oracle


def test_token_norms_closed_forms():
    a = np.array([[3.0, 4.0, 0.0], [1.0, 2.0, 2.0]], np.float32)
    assert np.array_equal(oracle.token_norms(a), [5.0, 3.0])
    # two vectors side by side: the squares add
    b = np.array([[12.0], [4.0]], np.float32)
    assert np.array_equal(oracle.token_norms(a, b), [13.0, 5.0])
    # homogeneity and the order of the two parts
    rng = np.random.default_rng(1)
    x = rng.standard_normal((5, 40)).astype(np.float32)
    y = rng.standard_normal((5, 24)).astype(np.float32)
    n = oracle.token_norms(x, y)
    assert np.allclose(oracle.token_norms(y, x), n, rtol=1e-15)
    assert np.allclose(oracle.token_norms(2 * x, 2 * y), 2 * n, rtol=1e-15)
    assert np.allclose(n, np.sqrt((x.astype(np.float64) ** 2).sum(1) +
                                  (y.astype(np.float64) ** 2).sum(1)), rtol=1e-14)
    # bf16 inputs are read as the numbers they encode
    xb = (x.view(np.uint32) >> 16).astype(np.uint16)
    xf = (xb.astype(np.uint32) << 16).view(np.float32)
    assert np.allclose(oracle.token_norms(xb), oracle.token_norms(xf), rtol=1e-15)


def test_scores_average_tokens_inside_a_prompt_first():
    # one layer, two prompts: one token of magnitude 10, three tokens of magnitude 2 (ffn 0):
    # the mean over prompts of the means over tokens is (10 + 2) / 2 = 6; the plain mean over
    # all four tokens would be 4
    attn = np.array([[10.0, 2.0, 2.0, 2.0]])
    ffn = np.zeros((1, 4))
    assert oracle.mcap_scores(attn, ffn, [1, 3])[0] == 6.0
    # both magnitudes enter, with weight one each
    assert oracle.mcap_scores(attn, attn, [1, 3])[0] == 12.0
    # layers are independent of each other; a constant layer scores its constant
    attn2 = np.vstack([attn[0], np.full(4, 7.0)])
    ffn2 = np.vstack([np.zeros(4), np.full(4, 0.5)])
    assert np.array_equal(oracle.mcap_scores(attn2, ffn2, [2, 2]), [4.0, 7.5])


def test_scores_feed_the_assignment():
    # three layers, the middle one with an outlying feed-forward magnitude: only it goes to W4A16
    attn = np.ones((3, 6))
    ffn = np.array([[1.0] * 6, [9.0] * 6, [1.5] * 6])
    s = oracle.mcap_scores(attn, ffn, [6])
    assert np.array_equal(s, [2.0, 10.0, 2.5])
    bits, shat = oracle.precision_from_scores(s, tau=0.7)
    assert list(bits) == [0, 1, 0] and shat[1] == 1.0 and shat[0] == 0.0
