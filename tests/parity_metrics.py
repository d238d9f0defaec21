"""Error measures of the GPU parity tests (pure numpy; importable without a GPU).

The tolerance asked of bf16 with fp32 accumulation is max |gpu - ref| / max |ref| <= 2e-2
per output tensor.  Applied to the layer output z = x + attention block + FFN block alone
it cannot see a block whose magnitude is below 2e-2 * max |z|: with x ~ N(0, 1) that is
the attention block of every row with more than about 2 k cached tokens.  So every
intermediate is compared on its own scale:

  tensor_rel_err   max |gpu - ref| / max |ref| over one tensor;
  row_rel_err      the same per row (one token's values), maximum over the rows - a long-context
                   attention row is then measured against its own, small, magnitude;
  block_tol        bound for a block that is only seen as the difference of two bf16
                   tensors (attention block = y - x, FFN block = z - y): 2e-2 * max |block|
                   plus half a bf16 ulp of every stored operand of the difference;
  rms_report       the element-wise figure: max |gpu - ref| / rms(ref) and the share of
                   elements within 2e-2 * rms(ref).

tests/test_parity_metric.py plants mistakes in the oracle's attention (zero output,
uniform weights, a dropped key, a wrong scale, a wrong kv head) and shows on the CPU
that these measures reject every one of them on the cases the GPU tests run, while the
z-only measure accepts several.
"""
import numpy as np

from oracle.decoder_layer import widen

REL_TOL = 2e-2
BF16_HALF_ULP = 2.0 ** -8       # relative rounding error of one bf16 store (8 significant bits)


def tensor_rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    return float(np.max(np.abs(got.astype(np.float64) - ref)) / max(np.max(np.abs(ref)), 1e-30))


def row_rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """Maximum over rows (first axis) of max |gpu - ref| / max |ref| within the row."""
    g = got.astype(np.float64).reshape(got.shape[0], -1)
    r = ref.reshape(ref.shape[0], -1)
    if r.shape[0] == 0:
        return 0.0
    d = np.max(np.abs(g - r), axis=1)
    s = np.maximum(np.max(np.abs(r), axis=1), 1e-30)
    return float(np.max(d / s))


def block_tol(block_ref: np.ndarray, *stored_operands: np.ndarray, tol: float = REL_TOL) -> float:
    """Absolute bound for |(a - b)_gpu - block_ref| when a, b are stored in bf16."""
    t = tol * float(np.max(np.abs(block_ref)))
    for op in stored_operands:
        t += BF16_HALF_ULP * float(np.max(np.abs(op)))
    return t


def rms_report(got: np.ndarray, ref: np.ndarray) -> "tuple[float, float]":
    """(max |gpu - ref| / rms(ref), share of elements with |gpu - ref| <= 2e-2 * rms(ref))."""
    d = np.abs(got.astype(np.float64) - ref)
    rms = max(float(np.sqrt(np.mean(ref * ref))), 1e-30)
    return float(np.max(d) / rms), float(np.mean(d <= REL_TOL * rms))


def check_intermediates(model, regions, z_bits, tok, z_ref, parts, tol=REL_TOL):
    """attn (per tensor and per token row), the attention block y - x, SiLU(gate)*up and the
    FFN block z - y of the rows `tok` against the oracle's parts.  Returns the figures."""
    B = len(tok)
    attn = widen(regions["attn"][tok]).reshape(B, model.n_q_heads, model.head_dim)
    e_attn = tensor_rel_err(attn, parts["attn"])
    e_attn_row = row_rel_err(attn, parts["attn"])
    assert e_attn <= tol and e_attn_row <= tol, ("attention output", e_attn, e_attn_row)
    y = widen(regions["y"][tok])
    blk = parts["y"] - parts["x"]
    d_blk = float(np.max(np.abs((y - parts["x"]) - blk)))
    assert d_blk <= block_tol(blk, parts["y"], tol=tol), ("attention block y - x", d_blk, float(np.max(np.abs(blk))))
    report = {"attn": e_attn, "attn_row": e_attn_row, "attn_block": d_blk / float(np.max(np.abs(blk))),
              "attn_rms": rms_report(attn, parts["attn"])}
    if parts.get("inner") is not None and "f" in regions:
        e_f = tensor_rel_err(widen(regions["f"][tok]), parts["inner"])
        assert e_f <= tol, ("SiLU(gate)*up", e_f)
        report["inner"] = e_f
    ffn = z_ref - parts["y"]
    d_ffn = float(np.max(np.abs((widen(z_bits[tok]) - y) - ffn)))
    assert d_ffn <= block_tol(ffn, z_ref, parts["y"], tol=tol), ("FFN block z - y", d_ffn, float(np.max(np.abs(ffn))))
    report["ffn_block"] = d_ffn / float(np.max(np.abs(ffn)))
    return report


def routing_exemptions(ids_gpu: np.ndarray, logits: np.ndarray, h2: np.ndarray, w_router: np.ndarray, top_k: int):
    """Tokens whose expert choice on the GPU (fp32 dot products of bf16 inputs) differs from the
    float64 choice.  A difference is accepted only at a near-tie, with the threshold taken from
    the arithmetic: the GPU forms its logits from activations that were rounded to bf16 twice
    (y, then the normalised row), a relative error of about 2^-8 per element, so the difference
    of two logits d = sum_k h_k (w_ak - w_bk) carries an error of standard deviation
    2^-8 * sqrt(sum_k h_k^2 (w_ak - w_bk)^2); four of these is the bound.  Every expert the GPU
    chose and the float64 top-k did not must lie within that bound of the k-th float64 logit.
    Returns the indices of the exempted tokens (the others must match the float64 choice)."""
    T, E = logits.shape
    exempt = []
    for t in range(T):
        order = sorted(range(E), key=lambda e: (-logits[t, e], e))
        top = order[:top_k]
        if sorted(ids_gpu[t]) == sorted(top):
            continue
        assert len(set(int(e) for e in ids_gpu[t])) == top_k, (t, ids_gpu[t])
        kth = top[-1]
        for e in ids_gpu[t]:
            if e in top:
                continue
            dw = w_router[e] - w_router[kth]
            bound = 4.0 * 2.0 ** -8 * float(np.sqrt(np.sum(h2[t] ** 2 * dw ** 2)))
            gap = float(logits[t, kth] - logits[t, e])
            assert 0.0 <= gap <= bound, ("expert choice is not a near-tie", t, int(e), gap, bound)
        exempt.append(t)
    return np.asarray(exempt, np.int64)
