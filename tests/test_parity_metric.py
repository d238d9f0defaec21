"""What the GPU parity measures can and cannot see - shown on the CPU.

The GPU tests compare the layer output z, the appended K/V rows, the attention output (per
tensor and per token row), the attention block y - x, SiLU(gate)*up and the FFN block z - y
with the oracle (tests/parity_metrics.py).  Here the mistakes are planted in the ORACLE's
attention, the corrupted layer is rounded to bf16 where the GPU path stores bf16, and the
same checking code runs on it:

  * the unmodified oracle, rounded to bf16, passes every check (the rounding allowances are
    not exceeded by rounding itself);
  * zero attention output, uniform softmax weights, a dropped self key, a wrong score scale
    and a wrong q-head -> kv-head map are each rejected on the long-context case, the
    single decode row and the chunked-prefill case;
  * the layer-output measure alone ACCEPTS uniform softmax weights on the long-context
    case - which is why it is not the only measure.
"""
import numpy as np
import pytest

from oracle import decoder_layer as orc
from paper_2408_12757_amd import workloads as wl

from cases import edge_case_batch
from parity_metrics import REL_TOL, check_intermediates, row_rel_err, tensor_rel_err


def to_bf16(a: np.ndarray) -> np.ndarray:
    return wl.f32_to_bf16_bits(np.asarray(a, np.float32))


def run_oracle(name, monkeypatch=None, mistake=None):
    model, b, seed = edge_case_batch(name)
    w = wl.make_weights(model, seed)
    x = wl.make_x(b.n_tokens, model.hidden, seed + 1)
    pages = wl.make_kv_pages_host(model, b.num_pages, seed + 3)
    if mistake is not None:
        mistake(monkeypatch, model)
    z, k, v, parts = orc.layer_forward(model, w, pages, b, x, return_parts=True)
    parts["x"] = orc.widen(x)
    return model, b, z, parts


def as_stored(z, parts):
    """The tensors the GPU path leaves behind, as bf16 bits."""
    B = z.shape[0]
    regions = {"attn": to_bf16(parts["attn"].reshape(B, -1)), "y": to_bf16(parts["y"]), "f": to_bf16(parts["inner"])}
    return to_bf16(z), regions


# ---- mistakes, planted in the oracle ------------------------------------------------

def zero_output(mp, model):
    mp.setattr(orc, "softmax_attention", lambda q, K, V: np.zeros_like(q))


def uniform_weights(mp, model):
    mp.setattr(orc, "softmax_attention", lambda q, K, V: np.mean(V, axis=0))


def dropped_self_key(mp, model):
    true = orc.softmax_attention
    mp.setattr(orc, "softmax_attention", lambda q, K, V: true(q, K[:-1], V[:-1]) if len(K) > 1 else np.zeros_like(q))


def wrong_scale(mp, model):
    def f(q, K, V):
        s = (K @ q) / float(q.shape[0])
        p = np.exp(s - np.max(s))
        return (p / np.sum(p)) @ V
    mp.setattr(orc, "softmax_attention", f)


def wrong_head_map(mp, model):
    # kv heads taken in reverse order (cached and fresh): q head h reads kv head Hkv - 1 - h // G
    true_stage, true_gather = orc.attention_stage, orc.gather_kv

    def gather(*a):
        K, V = true_gather(*a)
        return K[:, ::-1], V[:, ::-1]

    def stage(model_, batch, pages, q, k, v):
        qr, kr, attn = true_stage(model_, batch, pages, q, k[:, ::-1], v[:, ::-1])
        return qr, kr[:, ::-1], attn
    mp.setattr(orc, "gather_kv", gather)
    mp.setattr(orc, "attention_stage", stage)


MISTAKES = [zero_output, uniform_weights, dropped_self_key, wrong_scale, wrong_head_map]
CASES = ["long_ctx", "one_decode", "prefill_prior"]


@pytest.mark.parametrize("name", CASES + ["page_edges", "gqa8", "mha64", "prefill_only"])
def test_rounded_oracle_passes_every_measure(name):
    model, b, z, parts = run_oracle(name)
    z_bits, regions = as_stored(z, parts)
    report = check_intermediates(model, regions, z_bits, np.arange(b.n_tokens), z, parts)
    assert report["attn_row"] < 5e-3 and tensor_rel_err(orc.widen(z_bits), z) < 5e-3


@pytest.mark.parametrize("name", CASES)
@pytest.mark.parametrize("mistake", MISTAKES, ids=lambda f: f.__name__)
def test_planted_attention_mistakes_are_rejected(name, mistake, monkeypatch):
    model, b, z_ref, parts_ref = run_oracle(name)
    _, _, z_bad, parts_bad = run_oracle(name, monkeypatch, mistake)
    z_bits, regions = as_stored(z_bad, parts_bad)
    tok = np.arange(b.n_tokens)
    bad = orc.widen(regions["attn"]).reshape(parts_ref["attn"].shape)
    if mistake is dropped_self_key and name in ("long_ctx", "one_decode"):
        # one key of >= 500 moves a row by about 1/n: below any bf16 tolerance.  Dropped keys
        # at long contexts are the business of the planted-key ("needle") test, whose closed
        # form (output row = the planted key's V row) has no such limit.
        assert row_rel_err(bad, parts_ref["attn"]) < REL_TOL
        return
    with pytest.raises(AssertionError, match="attention"):
        check_intermediates(model, regions, z_bits, tok, z_ref, parts_ref)
    # the measure of the single-operation attention test on its own
    assert row_rel_err(bad, parts_ref["attn"]) > REL_TOL


def test_planted_key_closed_form_sees_a_dropped_key_at_any_length():
    """One key with a score 30 above the rest takes the whole softmax weight: the output is
    its V row.  Dropping that key from 9000 gives a completely different row."""
    rng = np.random.default_rng(3)
    n, dh = 9000, 128
    K, V, q = rng.standard_normal((n, dh)), rng.standard_normal((n, dh)), rng.standard_normal(dh)
    K[n - 1] = q * (36.0 * np.sqrt(dh) / float(q @ q))
    out = orc.softmax_attention(q, K, V)
    assert np.max(np.abs(out - V[n - 1])) < 1e-6
    assert np.max(np.abs(orc.softmax_attention(q, K[:-1], V[:-1]) - V[n - 1])) > 1.0


def test_layer_output_alone_accepts_a_wrong_softmax_at_long_contexts(monkeypatch):
    model, b, z_ref, parts_ref = run_oracle("long_ctx")
    _, _, z_bad, parts_bad = run_oracle("long_ctx", monkeypatch, uniform_weights)
    z_bits, _ = as_stored(z_bad, parts_bad)
    assert tensor_rel_err(orc.widen(z_bits), z_ref) < REL_TOL          # the blind spot
    bad = parts_bad["attn"]
    assert row_rel_err(bad, parts_ref["attn"]) > 10 * REL_TOL          # what the row measure says


def test_block_allowance_is_smaller_than_every_block():
    """The rounding allowance of the block checks (half a bf16 ulp of the stored operands)
    stays below the magnitude of the block it guards, so a missing block is always seen."""
    from parity_metrics import block_tol
    for name in CASES:
        model, b, z, parts = run_oracle(name)
        blk = parts["y"] - parts["x"]
        ffn = z - parts["y"]
        assert block_tol(blk, parts["y"]) < 0.5 * np.max(np.abs(blk)), name
        assert block_tol(ffn, z, parts["y"]) < 0.5 * np.max(np.abs(ffn)), name
