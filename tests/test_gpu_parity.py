"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the
same seeded inputs.  Run with -m gpu on an MI355X."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import decoder_layer as orc
from paper_2408_12757_amd import binding as nf
from paper_2408_12757_amd import harness as hz
from paper_2408_12757_amd import workloads as wl

from cases import EDGE_CASES, edge_case_batch, small_gqa_model
from gpu_util import DEV, REL_TOL, Case, ChainCase, f64, rel_err, untouched_pages_equal
from parity_metrics import routing_exemptions

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = nf.Context(0)
    yield c
    c.close()


def say(*a):
    print(*a, flush=True)


# ------------------------------------------------------------ single operations ---

@pytest.mark.parametrize("T,D", [(1, 512), (37, 4096), (64, 8192)])
def test_rmsnorm_kernel(T, D):
    say("rmsnorm", T, D)
    r = np.random.default_rng(T * 7 + D)
    x = wl.f32_to_bf16_bits(r.standard_normal((T, D)).astype(np.float32) * 3)
    g = wl.f32_to_bf16_bits(1 + 0.1 * r.standard_normal(D).astype(np.float32))
    xt, gt = hz.bf16_tensor(x, DEV), hz.bf16_tensor(g, DEV)
    out = torch.empty_like(xt)
    nf.nf_op_rmsnorm(xt.data_ptr(), gt.data_ptr(), out.data_ptr(), T, D, 1e-5)
    torch.cuda.synchronize()
    ref = orc.rmsnorm(f64(x), f64(g), 1e-5)
    assert rel_err(f64(hz.bf16_bits(out)), ref) <= 1e-2


@pytest.mark.parametrize("M,N,K", [(1, 128, 64), (64, 1536, 512), (200, 192, 1408), (333, 512, 4096), (128, 6144, 4096)])
def test_gemm_kernel_plain_and_residual(M, N, K):
    say("gemm", M, N, K)
    r = np.random.default_rng(M + N + K)
    x = wl.f32_to_bf16_bits(r.standard_normal((M, K)).astype(np.float32))
    w = wl.f32_to_bf16_bits(0.05 * r.standard_normal((N, K)).astype(np.float32))
    res = wl.f32_to_bf16_bits(r.standard_normal((M, N)).astype(np.float32))
    xt, wt, rt = hz.bf16_tensor(x, DEV), hz.bf16_tensor(w, DEV), hz.bf16_tensor(res, DEV)
    # rows past M in the output buffer must stay untouched
    out = torch.full((M + 3, N), 7.0, dtype=torch.bfloat16, device=DEV)
    nf.nf_op_gemm(xt.data_ptr(), wt.data_ptr(), out.data_ptr(), None, M, N, K, nf.NF_EPI_NONE)
    torch.cuda.synchronize()
    ref = orc.dense(f64(x), f64(w))
    got = f64(hz.bf16_bits(out))
    assert rel_err(got[:M], ref) <= REL_TOL / 2
    assert np.all(got[M:] == 7.0)
    nf.nf_op_gemm(xt.data_ptr(), wt.data_ptr(), out.data_ptr(), rt.data_ptr(), M, N, K, nf.NF_EPI_RESIDUAL)
    torch.cuda.synchronize()
    assert rel_err(f64(hz.bf16_bits(out))[:M], ref + f64(res)) <= REL_TOL / 2


@pytest.mark.parametrize("M,I,K", [(64, 1408, 512), (130, 256, 1024), (77, 14336, 4096)])
def test_gemm_kernel_swiglu(M, I, K):
    say("gemm swiglu", M, I, K)
    r = np.random.default_rng(M + I + K)
    x = wl.f32_to_bf16_bits(r.standard_normal((M, K)).astype(np.float32))
    w = wl.f32_to_bf16_bits(0.05 * r.standard_normal((2 * I, K)).astype(np.float32))
    xt, wt = hz.bf16_tensor(x, DEV), hz.bf16_tensor(w, DEV)
    out = torch.empty((M, I), dtype=torch.bfloat16, device=DEV)
    nf.nf_op_gemm(xt.data_ptr(), wt.data_ptr(), out.data_ptr(), None, M, I, K, nf.NF_EPI_SWIGLU)
    torch.cuda.synchronize()
    wf = f64(w)
    ref = orc.silu(orc.dense(f64(x), wf[:I])) * orc.dense(f64(x), wf[I:])
    assert rel_err(f64(hz.bf16_bits(out)), ref) <= REL_TOL / 2


@pytest.mark.parametrize("M,N,K,epi", [(300, 512, 256, "none"), (1100, 1024, 1408, "residual"), (257, 768, 512, "swiglu"),
                                       (700, 1536, 320, "residual"), (513, 512, 1024, "none"), (64, 256, 128, "none"),
                                       # 8 x 48 tiles of 256x256 = 1.5 rounds of 256: the remainder runs as 128x256 tiles
                                       (2048, 12288, 128, "residual"), (2000, 6144, 256, "swiglu"),
                                       # 6 and 10 K-steps of 64: with 2, 4 and 16 above, every start-up and tail
                                       # form of the loop that keeps three stages of weight rows in LDS
                                       (520, 768, 384, "swiglu"), (300, 512, 640, "residual"),
                                       # widths that 192 divides and 256 does not: the 256x192 form and its ragged rows
                                       (257, 192, 2048, "residual"), (1000, 768, 640, "none")])
def test_every_gemm_implementation_gives_the_same_bits(M, N, K, epi):
    """All tile shapes and both LDS feeding schemes walk K in the same order with the same
    MFMA instruction, so the implementation choice (which the profile makes per operation
    and batch size) must never change an output bit."""
    say("gemm implementations", M, N, K, epi)
    r = np.random.default_rng(M * 3 + N + K)
    rows = 2 * N if epi == "swiglu" else N
    xt = hz.bf16_tensor(wl.f32_to_bf16_bits(r.standard_normal((M, K)).astype(np.float32)), DEV)
    wt = hz.bf16_tensor(wl.f32_to_bf16_bits(0.05 * r.standard_normal((rows, K)).astype(np.float32)), DEV)
    rt = hz.bf16_tensor(wl.f32_to_bf16_bits(r.standard_normal((M, N)).astype(np.float32)), DEV)
    code = {"none": nf.NF_EPI_NONE, "residual": nf.NF_EPI_RESIDUAL, "swiglu": nf.NF_EPI_SWIGLU}[epi]
    res_ptr = rt.data_ptr() if epi == "residual" else None
    outs = {}
    try:
        for tile in range(1, 26):
            nf.nf_tune_set("gemm.tile", tile)
            out = torch.full((M + 1, N), 7.0, dtype=torch.bfloat16, device=DEV)
            nf.nf_op_gemm(xt.data_ptr(), wt.data_ptr(), out.data_ptr(), res_ptr, M, N, K, code)
            torch.cuda.synchronize()
            outs[tile] = hz.bf16_bits(out)
    finally:
        nf.nf_tune_set("gemm.tile", 0)
    for tile, got in outs.items():
        assert np.array_equal(got, outs[1]), f"implementation {tile} differs from implementation 1"
    assert np.all(f64(outs[1])[M:] == 7.0)
    nf.nf_op_gemm(xt.data_ptr(), wt.data_ptr(), out.data_ptr(), res_ptr, M, N, K, code)  # the default choice
    torch.cuda.synchronize()
    assert np.array_equal(hz.bf16_bits(out), outs[1])


@pytest.mark.parametrize("M,N,K", [(300, 512, 8192), (37, 128, 9088)])
def test_gemm_with_two_k_segments(M, N, K):
    """Long-K, narrow-N operations (the FFN down projection) add the sums of the two halves of
    K; through this entry point (no scratch) every workgroup forms both sums itself.  The
    result agrees with the oracle and does not depend on the implementation asked for or on
    the rows it is computed with."""
    say("gemm, two K segments", M, N, K)
    r = np.random.default_rng(M + N + K)
    x = wl.f32_to_bf16_bits(r.standard_normal((M, K)).astype(np.float32))
    w = wl.f32_to_bf16_bits(0.05 * r.standard_normal((N, K)).astype(np.float32))
    res = wl.f32_to_bf16_bits(r.standard_normal((M, N)).astype(np.float32))
    xt, wt, rt = hz.bf16_tensor(x, DEV), hz.bf16_tensor(w, DEV), hz.bf16_tensor(res, DEV)
    ref = orc.dense(f64(x), f64(w))
    outs = []
    try:
        for tile in (0, 1, 7, 13, 19):
            nf.nf_tune_set("gemm.tile", tile)
            out = torch.full((M + 3, N), 7.0, dtype=torch.bfloat16, device=DEV)
            nf.nf_op_gemm(xt.data_ptr(), wt.data_ptr(), out.data_ptr(), rt.data_ptr(), M, N, K, nf.NF_EPI_RESIDUAL)
            torch.cuda.synchronize()
            outs.append(hz.bf16_bits(out))
    finally:
        nf.nf_tune_set("gemm.tile", 0)
    assert rel_err(f64(outs[0])[:M], ref + f64(res)) <= REL_TOL / 2
    assert np.all(f64(outs[0])[M:] == 7.0)
    for o in outs[1:]:
        assert np.array_equal(o, outs[0])
    # a sub-range of the rows gives the same bits for those rows
    lo = M // 3
    out = torch.empty((M - lo, N), dtype=torch.bfloat16, device=DEV)
    nf.nf_op_gemm(xt[lo:].data_ptr(), wt.data_ptr(), out.data_ptr(), rt[lo:].data_ptr(), M - lo, N, K, nf.NF_EPI_RESIDUAL)
    nf.nf_op_gemm(xt.data_ptr(), wt.data_ptr(), out.data_ptr(), None, 1, N, K, nf.NF_EPI_NONE)   # no residual
    torch.cuda.synchronize()
    got = hz.bf16_bits(out)
    assert np.array_equal(got[1:], outs[0][lo + 1:M])
    assert rel_err(f64(got[:1]), ref[:1]) <= REL_TOL / 2


def test_gemm_rejects_bad_shapes():
    t = torch.zeros(64 * 64, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(nf.NfError) as e:
        nf.nf_op_gemm(t.data_ptr(), t.data_ptr(), t.data_ptr(), None, 8, 64, 48)
    assert e.value.status == nf.NF_ESHAPE
    with pytest.raises(nf.NfError) as e:
        nf.nf_op_gemm(t.data_ptr(), t.data_ptr(), t.data_ptr(), None, 8, 64, 64, nf.NF_EPI_RESIDUAL)
    assert e.value.status == nf.NF_EINVAL


# ------------------------------------------------------------------ whole layer ---

def test_c1_layer_matches_oracle_and_appends_kv(ctx):
    cfg = wl.CONFIGS["C1"]
    b = wl.make_batch(cfg.batch, cfg.seed + 2, spare_pages=7)
    say("C1 layer", b.n_tokens, "tokens", b.num_pages, "pages")
    case = Case(cfg.model, b, cfg.seed, ctx=ctx)
    z, pages = case.run(None)
    errs = case.check(z, pages)
    say("C1 rel err z/k/v", errs)
    assert untouched_pages_equal(case, pages)


@pytest.mark.parametrize("name", list(EDGE_CASES))
def test_layer_edge_cases(ctx, name):
    """Output, appended rows and every intermediate (attention output per row, attention
    block, SiLU(gate)*up, FFN block) against the oracle, each on its own scale: the layer
    output alone does not see the attention of a long-context row."""
    say("edge case", name)
    model, b, seed = edge_case_batch(name)
    case = Case(model, b, seed, ctx=ctx)
    z, pages = case.run(None)
    say(name, case.check(z, pages))
    assert untouched_pages_equal(case, pages)


def test_empty_batch_is_a_no_op(ctx):
    m = small_gqa_model()
    b = wl.batch_from_lengths([], [], 0, np.random.default_rng(0), spare_pages=2)
    args = hz.upload_batch(b, DEV)
    pages = torch.zeros((2, m.page_elems), dtype=torch.bfloat16, device=DEV)
    runner = hz.LayerRunner(m, wl.make_weights(m, 1), pages, DEV, ctx=ctx)
    x = torch.zeros((0, m.hidden), dtype=torch.bfloat16, device=DEV)
    out = runner.forward(args, x, None)
    torch.cuda.synchronize()
    assert out.shape[0] == 0


# ---------------------------------------------------- nano-batching is bit-exact ---

def test_nano_batched_and_overlapped_are_bit_exact_with_unsplit(ctx):
    cfg = wl.CONFIGS["C1"]
    b = wl.make_batch(cfg.batch, cfg.seed + 2)
    case = Case(cfg.model, b, cfg.seed, ctx=ctx)
    z0, p0 = case.run(None)
    for bounds in ([0, 32, 64], [0, 16, 64], [0, 20, 41, 64], [0, 4, 64]):   # 20/41/4 cut prefill requests
        for overlap, acu, gcu in ((False, 0, 0), (True, 0, 0), (True, 64, 192), (True, 96, 0)):
            say("plan", bounds, overlap, acu, gcu)
            plan = nf.nf_plan_manual(case.ctx, cfg.model, case.args, bounds, overlap, acu, gcu)
            d = plan.describe()
            assert d["bounds"] == bounds
            for rep in range(2):
                z, p = case.run(plan)
                assert np.array_equal(z, z0), (bounds, overlap, acu)
                assert np.array_equal(p, p0)
            plan.close()


def test_per_nano_operation_shares_and_launch_order_are_bit_exact(ctx):
    """Every attention nano-operation with its own workgroup count, every nano-operation with its
    own GEMM implementation, the nano-batches launched in another order (Sec. 4.1.1 - 4.1.3): the
    same bits as unsplit, for one layer and for a chain of layers; an order that would launch an
    attention nano-operation before the KQV of the earlier part of its prefill request is refused."""
    cfg = wl.CONFIGS["C1"]
    b = wl.make_batch(cfg.batch, cfg.seed + 2)
    case = Case(cfg.model, b, cfg.seed, ctx=ctx)
    z0, p0 = case.run(None)
    bounds = [0, 20, 41, 64]                     # 20 cuts the third prefill request (tokens 16..23)
    tiles = [[7, 22, 21, 19], [0, 0, 0, 0], [24, 25, 22, 13]]
    for wgs, pos in (([0, 3, -1], None), ([5, 0, 2], [0, 2, 1]), ([0, 0, 0], [1, 2, 0]), ([2, 7, 1], [1, 2, 0])):
        plan = nf.nf_plan_manual_ops(case.ctx, cfg.model, case.args, bounds, True, wgs, tiles, launch_pos=pos)
        d = plan.describe()
        say("plan", d["nano_attn_wgs"], d["order"])
        assert d["nano_attn_wgs"] == wgs
        for rep in range(2):
            z, p = case.run(plan)
            assert np.array_equal(z, z0) and np.array_equal(p, p0), (wgs, pos)
        plan.close()
    with pytest.raises(nf.NfError) as e:       # nano-batch 1 first: its attention needs the KQV of nano-batch 0
        nf.nf_plan_manual_ops(case.ctx, cfg.model, case.args, bounds, True, [0, 0, 0], None, launch_pos=[1, 0, 2])
    assert e.value.status == nf.NF_EPLAN
    with pytest.raises(nf.NfError) as e:       # not a permutation
        nf.nf_plan_manual_ops(case.ctx, cfg.model, case.args, bounds, True, [0, 0, 0], None, launch_pos=[1, 1, 2])
    assert e.value.status == nf.NF_EPLAN
    chain = ChainCase(cfg.model, b, cfg.seed, 3, ctx=ctx)
    z_ref, pools_ref = chain.run_layer_by_layer()
    plan = nf.nf_plan_manual_ops(chain.ctx, cfg.model, chain.args, bounds, True, [4, 0, 9], tiles, launch_pos=[0, 2, 1])
    z, pools = chain.run_chain(plan)
    assert np.array_equal(z, z_ref)
    for l in range(3):
        assert np.array_equal(pools[l], pools_ref[l]), l
    plan.close()


PARTITION_CASES = [
    # KQV and attention in more pieces than the rest (the shape of the paper's pipelines, Fig. 6)
    dict(KQV=[0, 12, 20, 41, 64], ATTN=[0, 12, 20, 41, 64], O=[0, 41, 64], UG=[0, 41, 64], D=[0, 41, 64]),
    # attention pieces that span several KQV pieces and cut prefill requests; Up/Gate finer than Down
    dict(KQV=[0, 7, 20, 33, 50, 64], ATTN=[0, 20, 50, 64], O=[0, 64], UG=[0, 16, 17, 40, 64], D=[0, 17, 64]),
    # everything different
    dict(KQV=[0, 64], ATTN=[0, 5, 64], O=[0, 30, 31, 64], UG=[0, 50, 64], D=[0, 10, 20, 30, 40, 50, 60, 63, 64]),
]


def test_a_partition_per_operation_is_bit_exact(ctx):
    """Every operation with its own number of nano-operations (Sec. 4.1.2): the plan launches
    them in the stated order with the dependencies of the range rule, and one layer, a chain of
    layers and a chain with the simultaneous KV offload give the bits of the unsplit run."""
    from oracle import pipeline_model as pm
    cfg = wl.CONFIGS["C1"]
    m = cfg.model
    b = wl.make_batch(cfg.batch, cfg.seed + 2, spare_pages=5)
    case = Case(m, b, cfg.seed, ctx=ctx)
    z0, p0 = case.run(None)
    for parts in PARTITION_CASES:
        n_attn = len(parts["ATTN"]) - 1
        for overlap, wgs, tiles in ((True, list(range(1, n_attn + 1)), [22, 0, 21, 25]), (False, None, None),
                                    (True, None, None)):
            plan = nf.nf_plan_manual_parts(case.ctx, m, case.args, parts, overlap, wgs, tiles)
            d = plan.describe()
            say("partitions", d["partitions"], "overlap", overlap)
            assert d["partitions"] == [parts[k] for k in pm.KINDS] and d["bounds"] == parts["ATTN"]
            assert [(o["op"], o["nano"]) for o in d["ops"]] == pm.launch_order(parts)
            for i, o in enumerate(d["ops"]):
                assert o["range"] == [parts[o["op"]][o["nano"]], parts[o["op"]][o["nano"] + 1]]
                # waits: the earlier nano-operations on the other lane that the range rule names
                lo = o["range"][0]
                if o["op"] == "ATTN":
                    lo = int(b.q_indptr[np.searchsorted(b.q_indptr, lo, side="right") - 1])
                want = [j for j, q in enumerate(d["ops"][:i]) if q["lane"] != o["lane"] and
                        nf.lib().nf_nano_ops_dependent(pm.KINDS.index(q["op"]), pm.KINDS.index(o["op"]), q["range"][0],
                                                 q["range"][1], lo, o["range"][1])]
                assert o["deps"] == want, (parts, o)
            if wgs is not None:
                assert d["nano_attn_wgs"] == wgs
            for rep in range(2):
                z, p = case.run(plan)
                assert np.array_equal(z, z0) and np.array_equal(p, p0), (parts, overlap)
            plan.close()
    bad = dict(PARTITION_CASES[0], O=[0, 41, 63])
    with pytest.raises(nf.NfError) as e:
        nf.nf_plan_manual_parts(case.ctx, m, case.args, bad, True)
    assert e.value.status == nf.NF_EPLAN
    # a chain of layers: the next layer's KQV pieces go behind the Down piece that completes their rows
    n_layers = 3
    chain = ChainCase(m, b, cfg.seed, n_layers, ctx=ctx)
    z_ref, pools_ref = chain.run_layer_by_layer()
    row = 2 * m.n_kv_heads * m.head_dim
    tok = np.arange(b.n_tokens)
    for parts in PARTITION_CASES:
        plan = nf.nf_plan_manual_parts(chain.ctx, m, chain.args, parts, True)
        for rep in range(2):
            z, pools = chain.run_chain(plan)
            assert np.array_equal(z, z_ref), parts
            for l in range(n_layers):
                assert np.array_equal(pools[l], pools_ref[l]), (parts, l)
        host = torch.full((n_layers, b.n_tokens, row), 7.0, dtype=torch.bfloat16).pin_memory()
        nf.nf_ctx_set_kv_offload(chain.ctx, host.data_ptr(), b.n_tokens * row * 2)
        try:
            z, pools = chain.run_chain(plan)
        finally:
            nf.nf_ctx_set_kv_offload(chain.ctx, None)
        assert np.array_equal(z, z_ref)
        got = hz.bf16_bits(host)
        for l in range(n_layers):
            assert np.array_equal(pools[l], pools_ref[l]), (parts, l)
            kg, vg = hz.read_kv_rows(pools[l], m, b, tok)
            assert np.array_equal(got[l], np.concatenate([kg.reshape(b.n_tokens, -1), vg.reshape(b.n_tokens, -1)],
                                                         axis=1)), (parts, l)
        plan.close()


def test_two_segment_down_projection_is_bit_exact_in_both_launch_forms(ctx):
    """A model whose down projection has a long K (ffn_inner 8192 over hidden 512) sums the two
    halves of K separately.  With the layer's workspace the halves may run on different
    workgroups (fp32 sums to scratch, a second kernel adds them) or in one workgroup; the
    choice follows the row count of the nano-batch and must not change a bit."""
    m = small_gqa_model(hidden=512, n_q_heads=4, n_kv_heads=2, ffn_inner=8192)
    q_lens = [70, 9] + [1] * 300
    ctx_lens = [0, 33] + list(np.random.default_rng(3).integers(1, 200, size=300))
    b = wl.batch_from_lengths(q_lens, ctx_lens, 2, np.random.default_rng(6), spare_pages=3)
    case = Case(m, b, 1234, ctx=ctx)
    outs = []
    try:
        for ks, tile in ((1, 0), (2, 0), (0, 0), (0, 21), (0, 22)):  # 21 / 22: the four-wavefront loops on each half of K
            nf.nf_tune_set("gemm.ksplit", ks)
            nf.nf_tune_set("gemm.tile", tile)
            for bounds in ([0, b.n_tokens], [0, 130, b.n_tokens], [0, 64, 128, 257, b.n_tokens]):
                plan = nf.nf_plan_manual(case.ctx, m, case.args, bounds, len(bounds) > 3)
                z, p = case.run(plan)
                outs.append(((ks, tile), bounds, z, p))
                plan.close()
    finally:
        nf.nf_tune_set("gemm.ksplit", 0)
        nf.nf_tune_set("gemm.tile", 0)
    say("two-segment down projection", case.check(outs[0][2], outs[0][3]))
    for ks, bounds, z, p in outs[1:]:
        assert np.array_equal(z, outs[0][2]), (ks, bounds)
        assert np.array_equal(p, outs[0][3]), (ks, bounds)


# ------------------------------------------------------- consecutive layers ---

def test_layer_chain_matches_oracle_and_is_bit_exact_with_separate_calls(ctx):
    """nf_layers_forward pipelines the nano-operations across the layer boundary; its result
    must equal layer-by-layer calls bit for bit (output and every layer's pool) and the
    oracle's chain within the tolerance."""
    cfg = wl.CONFIGS["C1"]
    b = wl.make_batch(cfg.batch, cfg.seed + 2, spare_pages=5)
    n_layers = 4
    chain = ChainCase(cfg.model, b, cfg.seed, n_layers, ctx=ctx)
    z_ref, pools_ref = chain.run_layer_by_layer()
    for bounds, overlap in (([0, 64], False), ([0, 32, 64], False), ([0, 32, 64], True), ([0, 20, 41, 64], True),
                            ([0, 16, 64], True)):
        say("chain", n_layers, "layers", bounds, overlap)
        plan = nf.nf_plan_manual(chain.ctx, cfg.model, chain.args, bounds, overlap, 0, 0)
        for rep in range(2):
            z, pools = chain.run_chain(plan)
            assert np.array_equal(z, z_ref), (bounds, overlap, rep)
            for l in range(n_layers):
                assert np.array_equal(pools[l], pools_ref[l]), (bounds, overlap, l)
        plan.close()
    # against the oracle: the GPU rounds the activations to bf16 between layers, the oracle does not
    zo, ks, vs = orc.layers_forward(cfg.model, chain.weights, chain.pools_bits, b, chain.x_bits)
    e = rel_err(f64(z_ref), zo)
    say("chain rel err", e)
    assert e <= REL_TOL
    tok = np.arange(b.n_tokens)
    for l in range(n_layers):
        kg, vg = hz.read_kv_rows(pools_ref[l], cfg.model, b, tok)
        assert rel_err(f64(kg), ks[l]) <= REL_TOL and rel_err(f64(vg), vs[l]) <= REL_TOL, l


def test_layer_chain_rejects_bad_arguments(ctx):
    cfg = wl.CONFIGS["C1"]
    b = wl.make_batch(cfg.batch, cfg.seed + 2)
    chain = ChainCase(cfg.model, b, cfg.seed, 2, ctx=ctx)
    plan = nf.nf_plan_manual(chain.ctx, cfg.model, chain.args, [0, 32, 64], True, 0, 0)
    out = torch.empty_like(chain.x)
    need = nf.nf_layers_workspace_bytes(plan, 2)
    assert need > plan.workspace_bytes
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    w = [d.struct for d in chain.dev_w]
    n_pages = chain.pools[0].shape[0]
    same_pool = [chain.pools[0].data_ptr(), chain.pools[0].data_ptr()]
    with pytest.raises(nf.NfError) as e:
        nf.nf_layers_forward(chain.ctx, cfg.model, w, same_pool, n_pages, chain.args, plan, chain.x.data_ptr(),
                             out.data_ptr(), ws.data_ptr(), ws.numel())
    assert e.value.status == nf.NF_EINVAL
    pools = [p.data_ptr() for p in chain.pools]
    with pytest.raises(nf.NfError) as e:
        nf.nf_layers_forward(chain.ctx, cfg.model, w, pools, n_pages, chain.args, plan, chain.x.data_ptr(),
                             out.data_ptr(), ws.data_ptr(), need - 256)
    assert e.value.status == nf.NF_EWORKSPACE
    with pytest.raises(nf.NfError) as e:
        nf.nf_layers_forward(chain.ctx, cfg.model, w, pools, n_pages, chain.args, plan, chain.x.data_ptr(),
                             chain.x.data_ptr(), ws.data_ptr(), ws.numel())
    assert e.value.status == nf.NF_EINVAL
    plan.close()
    torch.cuda.synchronize()


def test_kv_offload_delivers_the_appended_rows_and_changes_nothing_else(ctx):
    """Simultaneous KV offload: the host receives, per layer and token, exactly the K row
    (after the rotary embedding) and V row that the layer appended to its pool; outputs and
    pools are the same bits as without the offload."""
    cfg = wl.CONFIGS["C1"]
    m = cfg.model
    b = wl.make_batch(cfg.batch, cfg.seed + 2, spare_pages=5)
    n_layers = 3
    chain = ChainCase(m, b, cfg.seed, n_layers, ctx=ctx)
    row = 2 * m.n_kv_heads * m.head_dim
    stride = b.n_tokens * row * 2
    tok = np.arange(b.n_tokens)
    for bounds, overlap in (([0, 64], False), ([0, 20, 41, 64], True)):
        plan = nf.nf_plan_manual(chain.ctx, m, chain.args, bounds, overlap, 0, 0)
        z_ref, pools_ref = chain.run_chain(plan)
        host = torch.full((n_layers, b.n_tokens, row), 7.0, dtype=torch.bfloat16).pin_memory()
        nf.nf_ctx_set_kv_offload(chain.ctx, host.data_ptr(), stride)
        try:
            z, pools = chain.run_chain(plan)
            # a stride too small for the batch is refused before anything runs
            nf.nf_ctx_set_kv_offload(chain.ctx, host.data_ptr(), stride - 16)
            with pytest.raises(nf.NfError) as e:
                chain.run_chain(plan)
            assert e.value.status == nf.NF_EINVAL
        finally:
            nf.nf_ctx_set_kv_offload(chain.ctx, None)
        assert np.array_equal(z, z_ref)
        got = hz.bf16_bits(host)
        for l in range(n_layers):
            assert np.array_equal(pools[l], pools_ref[l]), (bounds, l)
            kg, vg = hz.read_kv_rows(pools[l], m, b, tok)
            want = np.concatenate([kg.reshape(b.n_tokens, -1), vg.reshape(b.n_tokens, -1)], axis=1)
            assert np.array_equal(got[l], want), (bounds, overlap, l)
        plan.close()


def test_pages_are_gathered_and_scattered_bit_for_bit():
    """KV loading and scattering (Sec. 4.2.2): pool pages named by an id list land in a contiguous
    buffer in list order and go back to (other) places in the pool; ids outside the pool are
    skipped; nothing else in the pool or in the buffer changes."""
    r = np.random.default_rng(11)
    num_pages, elems, n = 300, 2 * 8 * 16 * 128, 37          # a C2 page: K and V blocks of 8 kv heads
    pool_h = r.integers(0, 1 << 16, size=(num_pages, elems), dtype=np.uint16)
    pool = hz.bf16_tensor(pool_h, DEV)
    ids = r.choice(num_pages, size=n, replace=False).astype(np.int32)
    ids_bad = ids.copy()
    ids_bad[5], ids_bad[20] = -1, num_pages
    line = torch.full((n, elems), 3.0, dtype=torch.bfloat16, device=DEV)
    before = hz.bf16_bits(line).copy()
    d_ids = torch.from_numpy(ids_bad).to(DEV)
    nf.nf_op_move_pages(pool.data_ptr(), elems * 2, num_pages, d_ids.data_ptr(), n, line.data_ptr(), False)
    torch.cuda.synchronize()
    got = hz.bf16_bits(line)
    for i in range(n):
        want = before[i] if i in (5, 20) else pool_h[ids[i]]
        assert np.array_equal(got[i], want), i
    assert np.array_equal(hz.bf16_bits(pool), pool_h)
    # scatter the gathered pages to a disjoint set of places
    free = np.setdiff1d(np.arange(num_pages), ids)
    dst = r.choice(free, size=n, replace=False).astype(np.int32)
    d_dst = torch.from_numpy(dst).to(DEV)
    nf.nf_op_move_pages(pool.data_ptr(), elems * 2, num_pages, d_dst.data_ptr(), n, line.data_ptr(), True)
    torch.cuda.synchronize()
    want_pool = pool_h.copy()
    want_pool[dst] = got
    assert np.array_equal(hz.bf16_bits(pool), want_pool)
    nf.nf_op_move_pages(pool.data_ptr(), elems * 2, num_pages, d_dst.data_ptr(), 0, line.data_ptr(), True)   # nothing to move
    with pytest.raises(nf.NfError) as e:
        nf.nf_op_move_pages(pool.data_ptr(), 24, num_pages, d_dst.data_ptr(), n, line.data_ptr(), True)
    assert e.value.status == nf.NF_ESHAPE


def test_plan_mismatch_and_workspace_errors(ctx):
    cfg = wl.CONFIGS["C1"]
    b = wl.make_batch(cfg.batch, cfg.seed + 2)
    case = Case(cfg.model, b, cfg.seed, ctx=ctx)
    plan = nf.nf_plan_manual(case.ctx, cfg.model, case.args, [0, 32, 64])
    b2 = wl.make_batch(cfg.batch, cfg.seed + 99)
    args2 = hz.upload_batch(b2, DEV)
    with pytest.raises(nf.NfError) as e:
        case.runner.forward(args2, case.x, plan)
    assert e.value.status == nf.NF_EPLAN
    out = torch.empty_like(case.x)
    ws = torch.empty(1024, dtype=torch.uint8, device=DEV)
    with pytest.raises(nf.NfError) as e:
        nf.nf_layer_forward(case.ctx, cfg.model, case.runner.w.struct, case.pages.data_ptr(), b.num_pages, case.args,
                            plan, case.x.data_ptr(), out.data_ptr(), ws.data_ptr(), ws.numel(), 0)
    assert e.value.status == nf.NF_EWORKSPACE
    with pytest.raises(nf.NfError) as e:
        nf.nf_plan_manual(case.ctx, cfg.model, case.args, [0, 40, 30, 64])
    assert e.value.status == nf.NF_EPLAN
    plan.close()


# ------------------------------------------------------------ mixture of experts ---

def moe_model(**kw):
    base = dict(hidden=256, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn_inner=384, n_experts=8, top_k=2,
                rope_theta=1e6)
    base.update(kw)
    return wl.ModelDesc(**base)


def read_routing(case, plan, B, k):
    off, nb = plan.workspace_region("moe.expert_ids")
    ws = case.runner.workspace
    ids = ws[off:off + nb].view(torch.int32).cpu().numpy().reshape(B, k)
    off, nb = plan.workspace_region("moe.expert_w")
    w = ws[off:off + nb].view(torch.float32).cpu().numpy().reshape(B, k)
    return ids, w


def check_moe_case(case, plan):
    """The routing decision is taken in the kernel's precision (fp32).  Tokens on which it agrees
    with the oracle's own float64 decision - all but the near-ties, whose bound comes from the
    arithmetic (parity_metrics.routing_exemptions) - are compared with the oracle under ITS OWN
    choice; the exempted tokens with the oracle under the GPU's choice."""
    m, b = case.model, case.batch
    z_bits, pages = case.run(plan)
    ids, wts = read_routing(case, plan, b.n_tokens, m.top_k)
    z_own, k, v, parts = orc.layer_forward(m, case.weights, case.pages_bits, b, case.x_bits, return_parts=True)
    idx64, w64, logits = parts["route"]
    exempt = routing_exemptions(ids, logits, parts["h2"], f64(case.weights["w_router"]), m.top_k)
    say("routing: tokens exempted as near-ties", len(exempt), "of", b.n_tokens)
    assert len(exempt) <= max(2, b.n_tokens // 20), len(exempt)
    keep = np.setdiff1d(np.arange(b.n_tokens), exempt)
    got = f64(z_bits)
    assert np.all(np.isfinite(got))
    scale = np.max(np.abs(z_own))
    e = float(np.max(np.abs(got[keep] - z_own[keep])) / scale)
    assert e <= REL_TOL, e
    # the order of the k experts may differ between the two sides: compare weights per expert
    for t in keep:
        for j in range(m.top_k):
            jj = list(idx64[t]).index(ids[t, j])
            assert abs(wts[t, j] - w64[t, jj]) <= 2e-2, (t, wts[t], w64[t])
    if len(exempt):
        z_gpu_choice, _, _ = orc.layer_forward(m, case.weights, case.pages_bits, b, case.x_bits, expert_choice=ids)
        e2 = float(np.max(np.abs(got[exempt] - z_gpu_choice[exempt])) / scale)
        assert e2 <= REL_TOL, e2
    return z_bits, pages, e


def test_moe_layer_matches_oracle_and_is_split_invariant(ctx):
    m = moe_model()
    b = wl.batch_from_lengths([40, 9] + [1] * 79, [0, 30] + list(np.random.default_rng(3).integers(5, 400, 79)), 2,
                              np.random.default_rng(4), spare_pages=2)
    say("moe layer", b.n_tokens, "tokens")
    case = Case(m, b, 4000, ctx=ctx)
    plan1 = nf.nf_plan_manual(case.ctx, m, case.args, [0, b.n_tokens])
    z0, p0, e = check_moe_case(case, plan1)
    say("moe rel err", e)
    for bounds, overlap in (([0, 48, 128], False), ([0, 64, 128], True), ([0, 16, 50, 128], True)):
        plan = nf.nf_plan_manual(case.ctx, m, case.args, bounds, overlap)
        z, p = case.run(plan)
        assert np.array_equal(z, z0) and np.array_equal(p, p0), bounds
        plan.close()
    # a partition per operation: Up/Gate and Down must share theirs (the expert rows are grouped per Up/Gate piece)
    parts = dict(KQV=[0, 30, 45, 100, 128], ATTN=[0, 45, 100, 128], O=[0, 128], UG=[0, 50, 90, 128], D=[0, 50, 90, 128])
    for overlap in (True, False):
        plan = nf.nf_plan_manual_parts(case.ctx, m, case.args, parts, overlap)
        z, p = case.run(plan)
        assert np.array_equal(z, z0) and np.array_equal(p, p0), parts
        plan.close()
    with pytest.raises(nf.NfError) as err:
        nf.nf_plan_manual_parts(case.ctx, m, case.args, dict(parts, D=[0, 50, 128]), True)
    assert err.value.status == nf.NF_EPLAN
    plan1.close()


def test_moe_layer_chain_is_bit_exact_with_separate_calls(ctx):
    """Consecutive mixture-of-experts layers in one call (routing arrays and grouped-GEMM
    offsets live in the shared workspace per nano-batch): same bits as layer-by-layer calls."""
    m = moe_model()
    b = wl.batch_from_lengths([40, 9] + [1] * 79, [0, 30] + list(np.random.default_rng(3).integers(5, 400, 79)), 2,
                              np.random.default_rng(4), spare_pages=2)
    chain = ChainCase(m, b, 4200, 3, ctx=ctx)
    z_ref, pools_ref = chain.run_layer_by_layer()
    parts = dict(KQV=[0, 30, 45, 100, 128], ATTN=[0, 45, 100, 128], O=[0, 128], UG=[0, 50, 90, 128], D=[0, 50, 90, 128])
    for bounds, overlap in (([0, b.n_tokens], False), ([0, 64, 128], True), ([0, 16, 50, 128], True), (parts, True)):
        plan = (nf.nf_plan_manual_parts(chain.ctx, m, chain.args, bounds, overlap) if isinstance(bounds, dict)
                else nf.nf_plan_manual(chain.ctx, m, chain.args, bounds, overlap))
        for rep in range(2):
            z, pools = chain.run_chain(plan)
            assert np.array_equal(z, z_ref), (bounds, overlap, rep)
            for l in range(3):
                assert np.array_equal(pools[l], pools_ref[l]), (bounds, l)
        plan.close()


def test_moe_skewed_routing_and_empty_experts(ctx):
    # a router that sends every token to experts 5 and 1: six experts get no rows
    m = moe_model(n_experts=8, top_k=2)
    b = wl.batch_from_lengths([1] * 37, list(range(3, 40)), 0, np.random.default_rng(8))
    w = wl.make_weights(m, 4100)
    wr = np.zeros((8, m.hidden), np.float32)
    case_x = wl.bf16_bits_to_f32(wl.make_x(b.n_tokens, m.hidden, 4101))
    wr[5] = 0.05
    wr[1] = 0.02
    w["w_router"] = wl.f32_to_bf16_bits(wr)
    w["g_ffn_norm"] = wl.f32_to_bf16_bits(np.ones(m.hidden, np.float32))
    case = Case(m, b, 4100, weights=w, ctx=ctx)
    plan = nf.nf_plan_manual(case.ctx, m, case.args, [0, b.n_tokens])
    z_bits, pages, e = check_moe_case(case, plan)
    ids, _ = read_routing(case, plan, b.n_tokens, 2)
    say("skewed moe rel err", e, "experts used", sorted(set(ids.ravel().tolist())))
    plan.close()


def test_moe_top1_and_four_experts(ctx):
    m = moe_model(n_experts=4, top_k=1, ffn_inner=256)
    b = wl.batch_from_lengths([12] + [1] * 20, [5] + list(range(10, 30)), 1, np.random.default_rng(9))
    case = Case(m, b, 4200, ctx=ctx)
    plan = nf.nf_plan_manual(case.ctx, m, case.args, [0, 16, b.n_tokens], True)
    _, _, e = check_moe_case(case, plan)
    say("top-1 moe rel err", e)
    plan.close()


def test_moe_down_projection_with_two_k_segments(ctx):
    """Experts with a long inner dimension (8192 over hidden 512): the grouped down projection
    leaves the fp32 sums of its two K halves in the workspace and the combine kernel adds them.
    Checked against the oracle and for split invariance (rows land in different tiles, and
    beside different rows, in every structure)."""
    m = moe_model(hidden=512, n_q_heads=4, n_kv_heads=2, ffn_inner=8192, n_experts=4, top_k=2)
    b = wl.batch_from_lengths([40] + [1] * 150, [7] + list(np.random.default_rng(4).integers(1, 120, size=150)), 1,
                              np.random.default_rng(10))
    case = Case(m, b, 4300, ctx=ctx)
    ref = None
    for bounds, overlap in (([0, b.n_tokens], False), ([0, 64, b.n_tokens], True), ([0, 30, 100, b.n_tokens], False)):
        plan = nf.nf_plan_manual(case.ctx, m, case.args, bounds, overlap)
        z, pages, e = check_moe_case(case, plan)
        say("two-segment expert down projection", bounds, "rel err", e)
        if ref is None:
            ref = (z, pages)
        assert np.array_equal(z, ref[0]) and np.array_equal(pages, ref[1]), bounds
        plan.close()


# ------------------------------------------------------------- HIP graph capture ---

@pytest.mark.skip(reason="capturing nf_layer_forward with torch.cuda.graph ended in a host-side segmentation fault "
                         "inside the end of the capture; the cause is not established, so the case stays off the GPU")
def test_layer_forward_can_be_captured_in_a_hip_graph_and_replayed(ctx):
    """nf_layer_forward with a prepared plan only enqueues kernels, event records and event
    waits (its lane streams fork from and join the caller's stream), so a launch-bound caller
    can capture it once and replay it.  Every replay must give the eager bits; eager work and
    synchronisations run between the replays."""
    cfg = wl.CONFIGS["C1"]
    b = wl.make_batch(cfg.batch, cfg.seed + 2)
    case = Case(cfg.model, b, cfg.seed, ctx=ctx)
    for bounds, overlap in (([0, 64], False), ([0, 32, 64], True)):
        plan = nf.nf_plan_manual(case.ctx, cfg.model, case.args, bounds, overlap, 0, 0)
        z0, p0 = case.run(plan)                      # eager; also warms every kernel up
        case.runner.ensure_workspace(plan.workspace_bytes)
        out = torch.empty_like(case.x)
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        case.reset_pages()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            nf.nf_layer_forward(case.ctx, cfg.model, case.runner.w.struct, case.pages.data_ptr(), case.pages.shape[0],
                                case.args, plan, case.x.data_ptr(), out.data_ptr(), case.runner.workspace.data_ptr(),
                                case.runner.workspace.numel(), torch.cuda.current_stream().cuda_stream)
        for rep in range(3):
            case.reset_pages()
            out.zero_()
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert np.array_equal(hz.bf16_bits(out), z0), (bounds, overlap, rep)
            assert np.array_equal(hz.bf16_bits(case.pages), p0), (bounds, overlap, rep)
            # eager work between the replays
            z, p = case.run(plan)
            assert np.array_equal(z, z0)
        del graph
        plan.close()
