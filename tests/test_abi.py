"""The C-ABI library loads without a GPU and exports every symbol include/nf.h declares;
host-side validation returns the documented status codes (CPU only)."""
import os
import re

import numpy as np
import pytest

from paper_2408_12757_amd import binding as nf
from paper_2408_12757_amd import workloads as wl

HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "nf.h")


def declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(nf_[a-z_0-9]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    L = nf.lib()
    names = declared_functions()
    assert len(names) >= 20
    for n in names:
        assert hasattr(L, n), n
    assert set(nf.EXPORTS) <= set(names)


def test_strerror_and_context_without_gpu():
    L = nf.lib()
    assert L.nf_strerror(0) == b"ok"
    assert b"workspace" in L.nf_strerror(nf.NF_EWORKSPACE)
    import torch
    if not torch.cuda.is_available():
        with pytest.raises(nf.NfError) as e:
            nf.Context(0)
        assert e.value.status == nf.NF_EHIP


def host_args(b):
    dev = {"q_indptr": 1, "ctx_len": 1, "page_indptr": 1, "page_ids": 1}
    return nf.BatchArgs(b.n_tokens, b.n_prefill_reqs, b.n_decode_reqs, b.q_indptr, b.ctx_len, b.page_indptr,
                        b.page_ids, dev)


def test_host_validation_status_codes():
    m = wl.CONFIGS["C1"].model
    b = wl.make_batch(wl.CONFIGS["C1"].batch, 5)
    assert nf.nf_check_batch(m, host_args(b), b.num_pages) == nf.NF_OK
    # page id out of range
    assert nf.nf_check_batch(m, host_args(b), int(b.page_ids.max())) == nf.NF_EPAGES
    # page list too short for ctx_len + q_len
    import dataclasses
    short = dataclasses.replace(b, ctx_len=b.ctx_len + 64)
    assert nf.nf_check_batch(m, host_args(short), b.num_pages) == nf.NF_EPAGES
    # a decode request must carry exactly one token
    bad = dataclasses.replace(b, n_prefill_reqs=b.n_prefill_reqs - 1, n_decode_reqs=b.n_decode_reqs + 1)
    assert nf.nf_check_batch(m, host_args(bad), b.num_pages) == nf.NF_ESHAPE
    # unsupported shapes
    assert nf.nf_check_batch(dataclasses.replace(m, head_dim=96), host_args(b), b.num_pages) == nf.NF_ESHAPE
    assert nf.nf_check_batch(dataclasses.replace(m, page_size=32), host_args(b), b.num_pages) == nf.NF_ESHAPE
    assert nf.nf_check_batch(dataclasses.replace(m, n_q_heads=7), host_args(b), b.num_pages) == nf.NF_ESHAPE
    assert nf.nf_workspace_bytes(dataclasses.replace(m, head_dim=96), 64, 128) == 0
    assert nf.nf_workspace_bytes(m, 64, 128) > 64 * m.hidden * 2 * 3


def test_argument_errors_are_reported_before_anything_touches_the_gpu():
    """Calls with null pointers, bad shapes or unknown keys return a status on a machine
    without a GPU (nothing is launched)."""
    for args, status in (((None, None, None, None, 10, None, 4, 64), nf.NF_EINVAL),):
        with pytest.raises(nf.NfError) as e:
            nf.nf_op_embedding(*args)
        assert e.value.status == status
    with pytest.raises(nf.NfError) as e:
        nf.nf_op_embedding(1, None, None, 1, 10, 1, 4, 60)      # row width not a multiple of 8
    assert e.value.status == nf.NF_ESHAPE
    with pytest.raises(nf.NfError) as e:
        nf.nf_op_embedding(1, 1, None, 1, 10, 1, 4, 64)         # slot indirection needs both arrays
    assert e.value.status == nf.NF_EINVAL
    with pytest.raises(nf.NfError) as e:
        nf.nf_op_argmax(None, 4, 64, None, None)
    assert e.value.status == nf.NF_EINVAL
    with pytest.raises(nf.NfError) as e:
        nf.nf_op_argmax(1, 4, 60, None, 1)
    assert e.value.status == nf.NF_ESHAPE
    for key, value in (("no.such.key", 1), ("gemm.tile", 99), ("gemm.tile", 26), ("gemm.tile", -1), ("search.layers", 0), ("search.rank", -1),
                       ("gemm.grouped_tile", 3), ("attention.variant", 8), ("search.refine", 3), ("search.refine", -1),
                       ("search.max_parts", 9), ("search.max_parts", -1)):
        with pytest.raises(nf.NfError) as e:
            nf.nf_tune_set(key, value)
        assert e.value.status == nf.NF_EINVAL, key
    for key, value in (("gemm.tile", 25), ("gemm.tile", 0), ("search.layers", 1), ("search.rank", 0), ("gemm.grouped_tile", 0),
                       ("search.refine", 0), ("search.refine", 2), ("search.max_parts", 8), ("search.max_parts", 0)):
        nf.nf_tune_set(key, value)


def test_k_segment_rule_looks_at_the_shape_only():
    """Which dense operations add the sums of the two halves of K is part of the numerics
    contract (a row's bits must not depend on the nano-batch it is computed in, so the rule may
    not involve M): the down projections of the 8B layer and of long-K toy models do, the
    other operations of the configurations here do not."""
    E = (nf.NF_EPI_NONE, nf.NF_EPI_RESIDUAL, nf.NF_EPI_SWIGLU)
    assert nf.nf_gemm_segments(4096, 14336, nf.NF_EPI_RESIDUAL) == 2        # 8B Down
    assert nf.nf_gemm_segments(512, 8192, nf.NF_EPI_NONE) == 2
    assert nf.nf_gemm_segments(8192, 28672, nf.NF_EPI_RESIDUAL) == 1        # 70B Down: N = 8192 fills the chip anyway
    assert nf.nf_gemm_segments(6144, 4096, nf.NF_EPI_NONE) == 1             # KQV
    assert nf.nf_gemm_segments(4096, 4096, nf.NF_EPI_RESIDUAL) == 1         # O
    assert nf.nf_gemm_segments(14336, 4096, nf.NF_EPI_SWIGLU) == 1          # Up/Gate
    assert nf.nf_gemm_segments(128, 8192, nf.NF_EPI_SWIGLU) == 1            # never with the SwiGLU epilogue
    assert nf.nf_gemm_segments(4096, 8128, nf.NF_EPI_NONE) == 1             # K below 8192
    assert nf.nf_gemm_segments(4160, 8320, nf.NF_EPI_NONE) == 1             # N, K not multiples of 128
    assert nf.nf_gemm_segments(4096, 8192, nf.NF_EPI_NONE) == 2 and nf.nf_gemm_segments(4224, 8192, nf.NF_EPI_NONE) == 1  # K >= 2 N
    for bad in ((0, 64, 0), (64, 0, 0), (64, 64, 7), (60, 64, 0), (64, 100, 0)):
        assert nf.nf_gemm_segments(*bad) == 0
    assert all(nf.nf_gemm_segments(256, 16384, e) in (1, 2) for e in E)
