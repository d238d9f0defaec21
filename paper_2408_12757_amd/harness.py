"""Device-memory plumbing for tests and the bench: uploads synthetic inputs with
PyTorch, calls the C-ABI binding with raw pointers, and copies results back.
No layer arithmetic happens here."""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np
import torch

from . import binding as nf
from . import workloads as wl


def bf16_tensor(bits: np.ndarray, device) -> torch.Tensor:
    """uint16 bf16 bit patterns -> torch.bfloat16 tensor on device (bit-exact)."""
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16))
    return t.to(device).view(torch.bfloat16)


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


class DeviceWeights:
    def __init__(self, weights: Dict[str, Optional[np.ndarray]], device="cuda:0"):
        self.t = {k: (bf16_tensor(v, device) if v is not None else None) for k, v in weights.items()}
        self.struct = nf.weights_struct({k: (v.data_ptr() if v is not None else None) for k, v in self.t.items()})


def upload_batch(b: wl.Batch, device="cuda:0") -> nf.BatchArgs:
    dev_t = {
        "q_indptr": torch.from_numpy(b.q_indptr.astype(np.int32)).to(device),
        "ctx_len": torch.from_numpy(b.ctx_len.astype(np.int32)).to(device),
        "page_indptr": torch.from_numpy(b.page_indptr.astype(np.int32)).to(device),
        "page_ids": torch.from_numpy(np.concatenate([b.page_ids, [0]]).astype(np.int32)).to(device),
    }
    dev = {k: v.data_ptr() for k, v in dev_t.items()}
    return nf.BatchArgs(b.n_tokens, b.n_prefill_reqs, b.n_decode_reqs, b.q_indptr, b.ctx_len, b.page_indptr,
                        b.page_ids, dev, keepalive=dev_t)


class LayerRunner:
    """Holds a context, device weights, a KV pool and a workspace for one model."""

    def __init__(self, model: wl.ModelDesc, weights: Dict[str, Optional[np.ndarray]], pages: torch.Tensor,
                 device="cuda:0", ctx: Optional[nf.Context] = None):
        self.device = torch.device(device)
        self.model = model
        self.ctx = ctx or nf.Context(self.device.index or 0)
        self.w = DeviceWeights(weights, device)
        self.pages = pages
        self.num_pages = pages.shape[0]
        self.workspace = None

    def ensure_workspace(self, nbytes: int):
        if self.workspace is None or self.workspace.numel() < nbytes:
            self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)

    def forward(self, batch: nf.BatchArgs, x: torch.Tensor, plan: Optional[nf.Plan], out: Optional[torch.Tensor] = None,
                stream: Optional[int] = None) -> torch.Tensor:
        if out is None:
            out = torch.empty_like(x)
        if plan is not None:
            need = plan.workspace_bytes
        else:
            need = nf.nf_workspace_bytes(self.model, int(x.shape[0]), int(batch.h_c.max(initial=0)) + 4096)
        self.ensure_workspace(need)
        s = torch.cuda.current_stream(self.device).cuda_stream if stream is None else stream
        nf.nf_layer_forward(self.ctx, self.model, self.w.struct, self.pages.data_ptr(), self.num_pages, batch, plan,
                            x.data_ptr(), out.data_ptr(), self.workspace.data_ptr(), self.workspace.numel(), s)
        return out


def read_kv_rows(pages_bits: np.ndarray, model: wl.ModelDesc, batch: wl.Batch, tokens) -> "tuple[np.ndarray, np.ndarray]":
    """K and V rows (bf16 bits, [n, Hkv, dh]) stored at the page slots of the given
    batch tokens.  Pure indexing of the page layout."""
    P, Hkv, dh = model.page_size, model.n_kv_heads, model.head_dim
    pg = pages_bits.reshape(pages_bits.shape[0], 2, Hkv, P * dh)
    tok_req = np.repeat(np.arange(batch.n_reqs), np.diff(batch.q_indptr))
    K = np.zeros((len(tokens), Hkv, dh), np.uint16)
    V = np.zeros((len(tokens), Hkv, dh), np.uint16)
    kidx, vidx = wl.page_block_index(dh, P)
    for i, t in enumerate(tokens):
        r = int(tok_req[t])
        pos = int(batch.ctx_len[r]) + int(t - batch.q_indptr[r])
        page = int(batch.page_ids[int(batch.page_indptr[r]) + pos // P])
        slot = pos % P
        K[i] = pg[page, 0][:, kidx[slot]]
        V[i] = pg[page, 1][:, vidx[slot]]
    return K, V


class DeviceCase:
    """A full-size synthetic layer problem on the GPU: weights (several copies, so that
    consecutive steps read cold weights), a seeded KV pool generated on the device,
    the uploaded batch and the layer input."""

    def __init__(self, cfg: wl.Config, n_weight_copies: int = 1, device="cuda:0", sort_decode="none",
                 keep_host_weights: bool = True):
        self.cfg = cfg
        self.model = cfg.model
        self.device = torch.device(device)
        self.batch = wl.make_batch(cfg.batch, cfg.seed + 2, sort_decode=sort_decode)
        self.host_weights = []
        self.runners = []
        gen = torch.Generator(device=self.device)
        gen.manual_seed(cfg.seed + 3)
        # KV pool ~ N(0,1) in bf16, every slot filled (also the slots past each context)
        self.pages = torch.empty((self.batch.num_pages, self.model.page_elems), dtype=torch.bfloat16,
                                 device=self.device)
        step = 1 << 14
        for s in range(0, self.batch.num_pages, step):
            self.pages[s:s + step].normal_(0.0, 1.0, generator=gen)
        self.ctx = nf.Context(self.device.index or 0)
        for c in range(n_weight_copies):
            w = wl.make_weights(self.model, cfg.seed + 100 * c)
            self.runners.append(LayerRunner(self.model, w, self.pages, device, ctx=self.ctx))
            if keep_host_weights and c == 0:
                self.host_weights.append(w)
        self.x_bits = wl.make_x(self.batch.n_tokens, self.model.hidden, cfg.seed + 1)
        self.x = bf16_tensor(self.x_bits, device)
        self.args = upload_batch(self.batch, device)
        self.out = torch.empty_like(self.x)
        self._ws = None

    def forward(self, plan: Optional[nf.Plan], copy: int = 0) -> torch.Tensor:
        r = self.runners[copy % len(self.runners)]
        if self._ws is not None:
            r.workspace = self._ws
        out = r.forward(self.args, self.x, plan, out=self.out)
        self._ws = r.workspace
        return out

    def layer_pools(self, n_layers: int) -> "list[torch.Tensor]":
        """KV pools for n_layers consecutive layers: the case's own pool first, then pools of
        the same shape filled from the same seeded generator stream."""
        pools = [self.pages]
        gen = torch.Generator(device=self.device)
        gen.manual_seed(self.cfg.seed + 7)
        step = 1 << 14
        for _ in range(1, n_layers):
            p = torch.empty_like(self.pages)
            for s in range(0, p.shape[0], step):
                p[s:s + step].normal_(0.0, 1.0, generator=gen)
            pools.append(p)
        return pools

    def pages_of_requests(self, reqs) -> np.ndarray:
        """bf16 bits of the physical pages of the listed requests (device -> host)."""
        b = self.batch
        phys = np.concatenate([b.page_ids[b.page_indptr[r]:b.page_indptr[r + 1]] for r in reqs]).astype(np.int64)
        idx = torch.from_numpy(phys).to(self.device)
        return bf16_bits(self.pages.index_select(0, idx))


def time_plan(case: DeviceCase, plan: Optional[nf.Plan], warmup: int, steps: int) -> float:
    """Average milliseconds per nf_layer_forward over `steps` calls (weights rotate)."""
    for i in range(warmup):
        case.forward(plan, i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(steps):
        case.forward(plan, warmup + i)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps
