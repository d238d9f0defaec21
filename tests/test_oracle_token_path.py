"""Pins of the token-path oracle (embedding, LM head, greedy sampling)."""
import numpy as np

from oracle import token_path as tp


def test_embedding_is_a_row_lookup():
    table = np.arange(12.0).reshape(4, 3)
    np.testing.assert_array_equal(tp.embedding(table, [2, 0, 2]), [[6, 7, 8], [0, 1, 2], [6, 7, 8]])


def test_lm_head_with_one_hot_rows_reads_the_normalised_activation():
    """W = identity rows picks single normalised coordinates: logit j = x_j / rms(x) * g_j."""
    rng = np.random.default_rng(1)
    x = rng.standard_normal((3, 8))
    g = 1 + 0.1 * rng.standard_normal(8)
    w = np.eye(8)[[5, 0, 7]]
    got = tp.lm_head_logits(x, g, w, 1e-5)
    rms = np.sqrt((x ** 2).mean(axis=1, keepdims=True) + 1e-5)
    np.testing.assert_allclose(got, (x / rms * g)[:, [5, 0, 7]], rtol=1e-12)
    # scaling the activation leaves the logits (almost) unchanged: the norm removes it
    np.testing.assert_allclose(tp.lm_head_logits(1000 * x, g, w, 1e-5), got, rtol=1e-4)  # eps / (2 mean x^2) ~ 1e-5


def test_greedy_takes_the_first_of_equal_maxima():
    logits = np.array([[0.0, 3.0, 3.0, -1.0], [2.0, 2.0, 2.0, 2.0], [-5.0, -7.0, -5.0, -9.0]])
    np.testing.assert_array_equal(tp.greedy(logits), [1, 0, 0])
    # the token whose LM-head row is the normalised activation itself wins (Cauchy-Schwarz)
    rng = np.random.default_rng(2)
    x = rng.standard_normal((1, 16))
    w = rng.standard_normal((10, 16))
    w /= np.linalg.norm(w, axis=1, keepdims=True)
    w[6] = x[0] / np.linalg.norm(x[0])
    assert tp.greedy(tp.lm_head_logits(x, np.ones(16), w, 0.0))[0] == 6
