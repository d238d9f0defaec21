"""The allocation-free attention entry point (nf_op_attention_static: partial results in an
array built into the library) against nf_op_attention (partials in a caller workspace):
same bits, on two calls in a row, the second with a smaller input; a plan whose partials
exceed the built-in array is refused before anything runs."""
import numpy as np
import pytest
import torch

from paper_2408_12757_amd import binding as nf
from paper_2408_12757_amd import harness as hz
from paper_2408_12757_amd import workloads as wl

from cases import edge_case_batch, small_gqa_model

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(*a):
    print(*a, flush=True)


def both_entry_points(ctx, model, b, seed, bounds, attn_wgs):
    args = hz.upload_batch(b, DEV)
    rng = np.random.default_rng(seed)
    pages = hz.bf16_tensor(wl.make_kv_pages_host(model, b.num_pages, seed + 3), DEV)
    qkv = hz.bf16_tensor(wl.f32_to_bf16_bits(rng.standard_normal((b.n_tokens, model.n_qkv)).astype(np.float32)), DEV)
    plan = nf.nf_plan_manual(ctx, model, args, bounds, False, 0, 0, attn_wgs)
    nf.nf_op_rope_append(ctx, model, pages.data_ptr(), b.num_pages, args, plan, qkv.data_ptr(), 0, b.n_tokens)
    ws = torch.empty(plan.workspace_bytes, dtype=torch.uint8, device=DEV)
    want = torch.full((b.n_tokens, model.q_dim), 7.0, dtype=torch.bfloat16, device=DEV)
    got = torch.full((b.n_tokens, model.q_dim), 9.0, dtype=torch.bfloat16, device=DEV)
    torch.cuda.synchronize()
    for i in range(len(bounds) - 1):
        nf.nf_op_attention(ctx, model, pages.data_ptr(), b.num_pages, args, plan, qkv.data_ptr(), want.data_ptr(),
                           ws.data_ptr(), ws.numel(), i)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    for i in range(len(bounds) - 1):
        nf.nf_op_attention_static(ctx, model, pages.data_ptr(), b.num_pages, args, plan, qkv.data_ptr(),
                                  got.data_ptr(), i)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    plan.close()
    w, g = hz.bf16_bits(want), hz.bf16_bits(got)
    return w, g


def test_static_scratch_attention_gives_the_bits_of_the_workspace_form_twice_in_a_row():
    ctx = nf.Context(0)
    assert nf.nf_attention_static_bytes() == 64 << 20
    # first call: multi-chunk rows (partials and merges in use), several nano-batches
    model, b, seed = edge_case_batch("long_ctx")
    say("long_ctx through both entry points")
    w, g = both_entry_points(ctx, model, b, seed, [0, 5, b.n_tokens], 0)
    assert np.array_equal(w, g)
    assert not np.any(g == hz.bf16_bits(torch.tensor([9.0], dtype=torch.bfloat16))[0])
    # second call, smaller: fewer and shorter rows; the array still holds the first call's partials
    model2, b2, seed2 = edge_case_batch("prefill_prior")
    say("prefill_prior through both entry points")
    w2, g2 = both_entry_points(ctx, model2, b2, seed2, [0, b2.n_tokens], -1)
    assert np.array_equal(w2, g2)
    # and a third, smaller still (one multi-chunk row only)
    m3 = small_gqa_model()
    b3 = wl.batch_from_lengths([1, 1], [2100, 30], 0, np.random.default_rng(2))
    w3, g3 = both_entry_points(ctx, m3, b3, 5, [0, 2], 0)
    assert np.array_equal(w3, g3)
    ctx.close()


def test_static_scratch_attention_refuses_a_plan_that_does_not_fit():
    """1300 rows of two chunks each with 8 kv heads of 128 need 165 MiB of partials.  The page
    table points into a small pool (every id valid), and the call must return NF_ESCRATCH
    before launching anything."""
    ctx = nf.Context(0)
    model = small_gqa_model(n_q_heads=8, n_kv_heads=8)
    n = 1300
    b = wl.batch_from_lengths([1] * n, [2100] * n, 0, np.random.default_rng(3))
    pool = 256
    b.page_ids[:] = b.page_ids % pool
    b.num_pages = pool
    args = hz.upload_batch(b, DEV)
    pages = torch.zeros((pool, model.page_elems), dtype=torch.bfloat16, device=DEV)
    qkv = torch.zeros((n, model.n_qkv), dtype=torch.bfloat16, device=DEV)
    out = torch.zeros((n, model.q_dim), dtype=torch.bfloat16, device=DEV)
    plan = nf.nf_plan_manual(ctx, model, args, [0, n])
    need = 2 * n * model.n_kv_heads * (16 * model.head_dim + 32) * 4
    assert need > nf.nf_attention_static_bytes()
    with pytest.raises(nf.NfError) as e:
        nf.nf_op_attention_static(ctx, model, pages.data_ptr(), pool, args, plan, qkv.data_ptr(), out.data_ptr(), 0)
    assert e.value.status == nf.NF_ESCRATCH
    torch.cuda.synchronize()
    assert float(out.abs().max()) == 0.0
    plan.close()
    ctx.close()
