"""Oracle of the ends of the iteration (paper Sec. 2.1: the input tokens are embedded, run
through the decoder layers, and the last layer's output goes through the LM head and
sampling to give the next token).  Plain numpy float64.  TEST INFRASTRUCTURE ONLY.

Readings: the final normalisation is an RMSNorm with its own gain (LLaMA), the LM head a
dense operation without bias on the normalised rows, sampling is greedy (the largest logit,
the lowest index among equal ones).
"""
import numpy as np

from . import decoder_layer as layer


def embedding(table, token_ids):
    """Row token_ids[t] of the embedding table [vocab, D] for every t."""
    return layer.widen(table)[np.asarray(token_ids, dtype=np.int64)]


def lm_head_logits(x_rows, g_final, w_lm, eps):
    """Logits [n, vocab] of the rows that need a next token."""
    return layer.dense(layer.rmsnorm(np.asarray(x_rows, dtype=np.float64), layer.widen(g_final), eps),
                       layer.widen(w_lm))


def greedy(logits):
    """Index of the largest logit per row; np.argmax returns the first of equal maxima."""
    return np.argmax(np.asarray(logits), axis=-1)
