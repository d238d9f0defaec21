"""CPU oracle: the plain definition of one LLaMA-style decoder-layer iteration
over a dense batch of prefill and decode tokens, in float64.

TEST INFRASTRUCTURE ONLY.  This file is the yardstick the HIP path is checked
against.  It is imported by the tests, by the smoke check and by the bench's
``cpu_baseline`` leg, never by the product path, and it shares no code with
the HIP kernels or their Python binding.

What it computes follows the paper's description of the inference workflow
(Sec. 2.1): the input is multiplied by W_Q, W_K, W_V; Key and Value are
appended to the request's KV cache; the Query is multiplied with all Keys of
the request, normalised (softmax), and used to average the Values; the result
goes through the O projection and a normalisation; the feed-forward stage
multiplies by W_up and W_gate, applies SiLU to the gate branch, multiplies
elementwise, and applies W_down.  Nano-batching (Sec. 3.7) performs "the exact
same projection" on sub-ranges of the batch and only re-orders independent
work, so the result the method must reach is this plain whole-batch result:
there are no nano-batches, tiles, streams or chunked softmax here.

Readings taken where the paper is silent (each one is listed in the design
notes of the repository):
  * normalisation = RMSNorm, applied before the KQV projection and before the
    feed-forward stage (LLaMA pre-norm), with residual connections around the
    attention block and the feed-forward block;
  * position embedding (an "other operation", Sec. 2.2) = rotary embedding in
    the half-split pairing (element i rotates with element i + dh/2), applied
    to Q and K before K is appended;
  * softmax scale 1/sqrt(head_dim), computed with the maximum subtracted;
  * a token attends to every cached token of its request, to the earlier
    tokens of its own prefill chunk, and to itself (K/V are appended first);
  * grouped-query attention: q head h reads kv head h // R_GQA (Sec. 3.1);
  * MoE feed-forward (Sec. 4.1.4): router logits W_r.h, the top_k largest
    logits (ties to the lower expert index), softmax over the selected
    logits, weighted sum of the selected experts' SwiGLU outputs;
  * KV pages hold page_size = 16 tokens; pages[p, 0, h] is the K block and
    pages[p, 1, h] the V block of kv head h.  The paper gives no layout; the one
    read here is the library's interface: K block [dh/32][16 tokens][32], V block
    [4][dh/32][16][2][4] with element (t, d) at index
    ((((t//4)*(dh//32) + d//32)*16 + d%16)*2 + (d//16)%2)*4 + t%4  (see unpack_page_blocks).

Inputs are bf16 bit patterns (uint16) or float arrays; every bf16 value is
widened exactly and all arithmetic is float64.  Values produced in this
iteration (Q, K, V, activations) are never rounded back to bf16.

Parity pins for these functions live in tests/test_oracle_*.py.  The paper
prints no numeric example of a layer output, so "parity versus values printed
in the paper" is unpinned; the pins are closed forms, brute force, invariants
and reductions to textbook routines.
"""
from __future__ import annotations

import numpy as np


# ----------------------------------------------------------------------------
# data widening
# ----------------------------------------------------------------------------

def widen(a) -> np.ndarray:
    """bf16 bit patterns (uint16) -> float64, exactly; floats pass through."""
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


# ----------------------------------------------------------------------------
# the operations of the layer (Sec. 2.1, 2.2)
# ----------------------------------------------------------------------------

def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    """h[t] = x[t] / sqrt(mean_j x[t,j]^2 + eps) * g   (an "other operation")."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * g


def dense(x: np.ndarray, w: np.ndarray) -> np.ndarray:
    """Dense operation (Sec. 2.2): y[t, n] = sum_k x[t, k] * w[n, k]."""
    return x @ w.T


def rope(v: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """Rotary position embedding on v[T, H, dh] at integer positions pos[T].

    For i in [0, dh/2): angle = pos * theta^(-2i/dh); the pair (v[i], v[i+dh/2])
    is rotated by that angle.
    """
    T, H, dh = v.shape
    half = dh // 2
    i = np.arange(half, dtype=np.float64)
    freq = np.power(float(theta), -2.0 * i / dh)
    ang = pos.astype(np.float64)[:, None] * freq[None, :]          # [T, half]
    c = np.cos(ang)[:, None, :]
    s = np.sin(ang)[:, None, :]
    a = v[:, :, :half]
    b = v[:, :, half:]
    return np.concatenate([a * c - b * s, a * s + b * c], axis=-1)


def silu(a: np.ndarray) -> np.ndarray:
    return a / (1.0 + np.exp(-a))


def swiglu_inner(h: np.ndarray, w_gate_up: np.ndarray) -> np.ndarray:
    """silu(gate(h)) * up(h); w_gate_up[2I, D] holds gate rows then up rows."""
    inner = w_gate_up.shape[0] // 2
    og = dense(h, w_gate_up[:inner])
    ou = dense(h, w_gate_up[inner:])
    return silu(og) * ou


def swiglu_ffn(h: np.ndarray, w_gate_up: np.ndarray, w_down: np.ndarray) -> np.ndarray:
    """down( silu(gate(h)) * up(h) )."""
    return dense(swiglu_inner(h, w_gate_up), w_down)


def softmax_attention(q: np.ndarray, K: np.ndarray, V: np.ndarray) -> np.ndarray:
    """One query vector q[dh] over keys K[n, dh], values V[n, dh]."""
    dh = q.shape[0]
    s = (K @ q) / np.sqrt(float(dh))
    s = s - np.max(s)
    p = np.exp(s)
    p = p / np.sum(p)
    return p @ V


def route_topk(logits: np.ndarray, top_k: int):
    """Per token: indices of the top_k largest logits (ties -> lower index, in
    descending-logit order) and the softmax weights over those logits."""
    T, E = logits.shape
    idx = np.zeros((T, top_k), np.int64)
    wts = np.zeros((T, top_k), np.float64)
    for t in range(T):
        order = sorted(range(E), key=lambda e: (-logits[t, e], e))[:top_k]
        sel = logits[t, order]
        p = np.exp(sel - np.max(sel))
        idx[t] = order
        wts[t] = p / np.sum(p)
    return idx, wts


def moe_ffn(h, w_router, w_gate_up, w_down, top_k, expert_choice=None):
    """Mixture-of-experts feed-forward.  ``expert_choice`` [T, top_k], when
    given, replaces the argmax decision (used when the caller has taken the
    decision in another precision); the weights are then the softmax over the
    logits of the given experts."""
    logits = dense(h, w_router)
    idx, wts = route_topk(logits, top_k)
    if expert_choice is not None:
        idx = np.asarray(expert_choice, np.int64)
        sel = np.take_along_axis(logits, idx, axis=1)
        p = np.exp(sel - np.max(sel, axis=1, keepdims=True))
        wts = p / np.sum(p, axis=1, keepdims=True)
    out = np.zeros_like(h)
    for e in range(len(w_gate_up)):
        for k in range(top_k):
            rows = np.nonzero(idx[:, k] == e)[0]
            if rows.size:
                out[rows] += wts[rows, k][:, None] * swiglu_ffn(h[rows], widen(w_gate_up[e]), widen(w_down[e]))
    return out, idx, wts, logits


# ----------------------------------------------------------------------------
# paged KV cache access
# ----------------------------------------------------------------------------

def unpack_page_blocks(kblk, vblk, head_dim: int, page_size: int):
    """K and V of one page and kv head as [page_size, head_dim] arrays.

    kblk: [head_dim/32, 16, 32]        kblk[s, t, e]       = K[t, 32s + e]
    vblk: [4, head_dim/32, 16, 2, 4]   vblk[g, q, c, h, j] = V[4g + j, 32q + 16h + c]
    """
    assert page_size == 16
    K = kblk.reshape(head_dim // 32, 16, 32).transpose(1, 0, 2).reshape(16, head_dim)
    V = vblk.reshape(4, head_dim // 32, 16, 2, 4).transpose(0, 4, 1, 3, 2).reshape(16, head_dim)
    return K, V


def gather_kv(pages, page_list, n_tokens: int, n_kv_heads: int, head_dim: int, page_size: int):
    """Read the first n_tokens cached tokens of a request from its pages.

    pages: [num_pages, 2*Hkv*page_size*dh] (uint16 or float).  Returns
    K[n_tokens, Hkv, dh], V[n_tokens, Hkv, dh] in float64.
    """
    K = np.zeros((n_tokens, n_kv_heads, head_dim))
    V = np.zeros((n_tokens, n_kv_heads, head_dim))
    for pi in range((n_tokens + page_size - 1) // page_size):
        page = widen(pages[page_list[pi]]).reshape(2, n_kv_heads, page_size * head_dim)
        n_here = min(page_size, n_tokens - pi * page_size)
        for h in range(n_kv_heads):
            Kp, Vp = unpack_page_blocks(page[0, h], page[1, h], head_dim, page_size)
            K[pi * page_size: pi * page_size + n_here, h] = Kp[:n_here]
            V[pi * page_size: pi * page_size + n_here, h] = Vp[:n_here]
    return K, V


def attention_stage(model, batch, pages, q, k, v):
    """Position embedding, KV concatenation and attention of the whole dense batch
    (Sec. 2.1: "Key and Value [are] concatenated into the existing KV-cache.  The Query
    is then multiplied with the existing Keys", normalised, and used to average the Values).

    q[B, Hq, dh], k[B, Hkv, dh], v[B, Hkv, dh]: this iteration's projections BEFORE the
    rotary embedding.  pages: the KV pool before the iteration.  The token with index t of
    request r sits at position ctx_len[r] + (t - q_indptr[r]) and reads keys 0 .. position.

    Returns (q after rotary embedding, k after rotary embedding, attn[B, Hq, dh]).
    """
    Hq, Hkv, dh, P = model.n_q_heads, model.n_kv_heads, model.head_dim, model.page_size
    G = Hq // Hkv
    B = q.shape[0]
    n_reqs = len(batch.ctx_len)
    pos = np.zeros(B, np.int64)
    for r in range(n_reqs):
        t0, t1 = int(batch.q_indptr[r]), int(batch.q_indptr[r + 1])
        pos[t0:t1] = int(batch.ctx_len[r]) + np.arange(t1 - t0)
    q = rope(q, pos, model.rope_theta)
    k = rope(k, pos, model.rope_theta)

    attn = np.zeros((B, Hq, dh))
    for r in range(n_reqs):
        t0, t1 = int(batch.q_indptr[r]), int(batch.q_indptr[r + 1])
        c = int(batch.ctx_len[r])
        plist = batch.page_ids[int(batch.page_indptr[r]): int(batch.page_indptr[r + 1])]
        Kc, Vc = gather_kv(pages, plist, c, Hkv, dh, P)
        # cached prefix + this iteration's rows of the request
        Kall = np.concatenate([Kc, k[t0:t1]], axis=0)
        Vall = np.concatenate([Vc, v[t0:t1]], axis=0)
        for t in range(t0, t1):
            n_keys = c + (t - t0) + 1
            for hq in range(Hq):
                hk = hq // G
                attn[t, hq] = softmax_attention(q[t, hq], Kall[:n_keys, hk], Vall[:n_keys, hk])
    return q, k, attn


# ----------------------------------------------------------------------------
# the layer
# ----------------------------------------------------------------------------

def layer_forward(model, weights, pages, batch, x, expert_choice=None, return_parts=False):
    """One decoder-layer iteration over the whole dense batch.

    model   : object with hidden, n_q_heads, n_kv_heads, head_dim, ffn_inner,
              n_experts, top_k, page_size, rms_eps, rope_theta
    weights : dict with g_attn_norm, w_qkv, w_o, g_ffn_norm, w_gate_up [E,2I,D],
              w_down [E,D,I], w_router [E,D] or None  (bf16 bits or floats)
    pages   : KV pool before the iteration [num_pages, page_elems]
    batch   : object with q_indptr, ctx_len, page_indptr, page_ids,
              n_prefill_reqs, n_decode_reqs
    x       : [B, D] layer input

    Returns z[B, D] and the K, V rows appended for every token
    (k_new[B, Hkv, dh] after rotary embedding, v_new[B, Hkv, dh]).
    """
    D, Hq, Hkv, dh = model.hidden, model.n_q_heads, model.n_kv_heads, model.head_dim
    x = widen(x)
    B = x.shape[0]

    # attention stage
    h = rmsnorm(x, widen(weights["g_attn_norm"]), model.rms_eps)
    qkv = dense(h, widen(weights["w_qkv"]))
    q = qkv[:, : Hq * dh].reshape(B, Hq, dh)
    k = qkv[:, Hq * dh: (Hq + Hkv) * dh].reshape(B, Hkv, dh)
    v = qkv[:, (Hq + Hkv) * dh:].reshape(B, Hkv, dh)

    q, k, attn = attention_stage(model, batch, pages, q, k, v)

    y = x + dense(attn.reshape(B, Hq * dh), widen(weights["w_o"]))

    # feed-forward stage
    h2 = rmsnorm(y, widen(weights["g_ffn_norm"]), model.rms_eps)
    wgu = weights["w_gate_up"]
    wd = weights["w_down"]
    route = None
    inner = None
    if model.n_experts > 1:
        f, idx, wts, logits = moe_ffn(h2, widen(weights["w_router"]), wgu, wd,
                                      model.top_k, expert_choice)
        route = (idx, wts, logits)
    else:
        inner = swiglu_inner(h2, widen(wgu[0]))
        f = dense(inner, widen(wd[0]))
    z = y + f
    if return_parts:
        return z, k, v, dict(h=h, q=q, attn=attn, y=y, h2=h2, inner=inner, route=route)
    return z, k, v


def layers_forward(model, weights_list, pages_list, batch, x):
    """Consecutive decoder layers on one dense batch (Sec. 2.1: the output of the
    down-projection "serves as the input to the next layer").  Layer l has its own weights
    and its own KV pool; the batch (requests, positions, page table) is the same for all.

    Returns the last layer's output and, per layer, the K and V rows it appended.
    Nothing is rounded between layers.
    """
    ks, vs = [], []
    z = np.asarray(x)
    for w, pages in zip(weights_list, pages_list):
        z, k, v = layer_forward(model, w, pages, batch, z)
        ks.append(k)
        vs.append(v)
    return z, ks, vs


def kv_slot(batch, model, t_req: int, pos: int):
    """(physical page id, slot) where the token at position pos of request
    t_req is stored (append rule: page = page list[pos // page_size])."""
    P = model.page_size
    return int(batch.page_ids[int(batch.page_indptr[t_req]) + pos // P]), pos % P
