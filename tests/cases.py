"""Small layer problems shared by the GPU parity tests and by the CPU demonstration of what
the parity measures can see (shapes and lengths only; no arithmetic)."""
import numpy as np

from paper_2408_12757_amd import workloads as wl


def small_gqa_model(**kw):
    base = dict(hidden=256, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn_inner=512, rope_theta=5e5)
    base.update(kw)
    return wl.ModelDesc(**base)


# name -> (model, q_lens, ctx_lens, number of prefill requests)
EDGE_CASES = {
    # contexts around page boundaries, single-token batch pieces
    "page_edges": (small_gqa_model(), [1] * 8, [0, 1, 14, 15, 16, 17, 31, 32], 0),
    # contexts around the 64-page groups of the kernel's page-id registers (1024 keys each) and
    # several attention chunks per request (chunk = 2048 keys) incl. exact multiples
    "long_ctx": (small_gqa_model(), [1] * 12,
                 [1023, 1024, 1025, 2046, 2047, 2048, 3000, 4094, 4095, 4096, 8191, 9000], 0),
    # chunked prefill with cached prefix, chunk crossing pages, a page-id group and the 2048-key chunk edge
    "prefill_prior": (small_gqa_model(), [37, 5, 40, 40, 1, 1], [1000, 0, 2030, 4080, 77, 200], 4),
    # G = 8 (two tokens per row group), dh = 128
    "gqa8": (small_gqa_model(n_q_heads=16, n_kv_heads=2), [19, 1, 1, 1], [3, 40, 129, 16], 1),
    # G = 1, dh = 64 (sixteen tokens per row group)
    "mha64": (small_gqa_model(n_q_heads=4, n_kv_heads=4, head_dim=64), [33, 1, 1], [0, 65, 300], 1),
    # prefill only, ragged lengths; 3 kv heads exercise the partial head group of a workgroup
    "prefill_only": (small_gqa_model(n_q_heads=6, n_kv_heads=3), [1, 16, 17, 50], [0, 0, 0, 0], 4),
    # decode only, one request
    "one_decode": (small_gqa_model(), [1], [500], 0),
}


def edge_case_batch(name: str, spare_pages: int = 3):
    model, q_lens, ctx_lens, n_pf = EDGE_CASES[name]
    b = wl.batch_from_lengths(q_lens, ctx_lens, n_pf, np.random.default_rng(5), spare_pages=spare_pages)
    return model, b, 900 + len(q_lens)
