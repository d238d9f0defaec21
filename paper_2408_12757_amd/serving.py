"""Multi-layer iteration loop with continuous batching (paper Sec. 4.2: request scheduling
and asynchronous scheduling) around the library's scheduler and nf_layers_forward.

This module is plumbing: it owns device memory (weights of every layer, one KV pool per
layer, workspace), two HIP streams and the host copies of swapped-out requests, and it
moves the scheduler's batches to the GPU.  Every decision (which tokens run, which pages
they use, who is swapped) is taken by the library's scheduler; every arithmetic step runs
in the library's kernels.

What is not here: embedding lookup, final norm, LM head and sampling.  The layer input of
an iteration is supplied by the caller (synthetic activations), and "the model emitted
EOS" is the request's output length, which the scheduler learns one iteration late when
async_lag = 1 (the paper's asynchronous scheduling).
"""
from __future__ import annotations

from collections import deque
from typing import Callable, Dict, List, Optional

import numpy as np
import torch

from . import binding as nf
from . import harness as hz
from . import workloads as wl


def device_random_weights(model: wl.ModelDesc, seed: int, device, std: float = 0.02) -> hz.DeviceWeights:
    """Random-init bf16 weights drawn on the device (same shapes and distributions as
    workloads.make_weights; used where a host copy of 32 layers would only cost time)."""
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    E = model.experts

    def normal(shape, mean=0.0):
        t = torch.empty(shape, dtype=torch.float32, device=device)
        t.normal_(mean, std, generator=gen)
        return t.to(torch.bfloat16)
    t = {"g_attn_norm": normal((model.hidden,), 1.0), "w_qkv": normal((model.n_qkv, model.hidden)),
         "w_o": normal((model.hidden, model.q_dim)), "g_ffn_norm": normal((model.hidden,), 1.0),
         "w_gate_up": normal((E, 2 * model.ffn_inner, model.hidden)),
         "w_down": normal((E, model.hidden, model.ffn_inner)),
         "w_router": normal((E, model.hidden)) if model.is_moe else None}
    w = hz.DeviceWeights.__new__(hz.DeviceWeights)
    w.t = t
    w.struct = nf.weights_struct({k: (v.data_ptr() if v is not None else None) for k, v in t.items()})
    return w


class ServingEngine:
    def __init__(self, model: wl.ModelDesc, n_layers: int, num_pages: int, dense_batch: int, max_requests: int,
                 host_weights: Optional[List[Dict[str, Optional[np.ndarray]]]] = None, weight_seed: int = 0,
                 device="cuda:0", async_lag: int = 1, avg_decode_len: float = 256.0, max_chunk: int = 0,
                 reserve_pages: int = 0, zero_pools: bool = False, ctx: Optional[nf.Context] = None,
                 bounds_fn: Optional[Callable[[int], List[int]]] = None, overlap: bool = False, attn_wgs: int = 0):
        self.model, self.n_layers, self.device = model, n_layers, torch.device(device)
        self.dense_batch, self.async_lag = dense_batch, async_lag
        self.ctx = ctx or nf.Context(self.device.index or 0)
        self.sched = nf.Scheduler(dense_batch, model.page_size, num_pages, max_requests, max_chunk, reserve_pages,
                                  avg_decode_len)
        if host_weights is not None:
            self.weights = [hz.DeviceWeights(w, device) for w in host_weights]
        else:
            self.weights = [device_random_weights(model, weight_seed + l, self.device) for l in range(n_layers)]
        alloc = torch.zeros if zero_pools else torch.empty
        self.pools = [alloc((num_pages, model.page_elems), dtype=torch.bfloat16, device=self.device)
                      for _ in range(n_layers)]
        self.num_pages = num_pages
        self.stream = torch.cuda.Stream(device=self.device)       # the iterations
        self.copy_stream = torch.cuda.Stream(device=self.device)  # batch arrays, while an iteration runs
        self.workspace: Optional[torch.Tensor] = None
        self.bounds_fn, self.overlap, self.attn_wgs = bounds_fn, overlap, attn_wgs
        self.host_store: Dict[int, List[torch.Tensor]] = {}       # swapped-out request -> pages per layer (pinned)
        self.pending = deque()                                    # (iteration, event, things to keep alive)
        self.iteration = 0
        self.tokens_launched = 0

    # ---- requests ---------------------------------------------------------------------
    def submit(self, prompt_len: int, output_len: int) -> int:
        return self.sched.submit(prompt_len, output_len)

    # ---- one iteration ------------------------------------------------------------------
    def _swap(self, fb: nf.FormedBatch):
        for rid in fb.released:
            self.host_store.pop(rid, None)
        with torch.cuda.stream(self.stream):
            for rid, pages in fb.swap_out:
                idx = torch.from_numpy(pages.astype(np.int64)).to(self.device)
                saved = []
                for pool in self.pools:
                    host = torch.empty((len(pages), pool.shape[1]), dtype=pool.dtype, pin_memory=True)
                    host.copy_(pool.index_select(0, idx), non_blocking=True)
                    saved.append(host)
                self.host_store[rid] = saved
            for rid, pages in fb.swap_in:
                idx = torch.from_numpy(pages.astype(np.int64)).to(self.device)
                saved = self.host_store.pop(rid)
                for pool, host in zip(self.pools, saved):
                    pool.index_copy_(0, idx, host.to(self.device, non_blocking=True))

    def _upload(self, fb: nf.FormedBatch) -> nf.BatchArgs:
        # pinned staging + a copy stream of its own: the arrays of iteration k + 1 cross the bus
        # while iteration k computes
        host = {"q_indptr": fb.q_indptr, "ctx_len": fb.ctx_len, "page_indptr": fb.page_indptr,
                "page_ids": np.concatenate([fb.page_ids, np.zeros(1, np.int32)])}
        dev_t, keep = {}, []
        with torch.cuda.stream(self.copy_stream):
            for k, a in host.items():
                pinned = torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).pin_memory()
                dev_t[k] = pinned.to(self.device, non_blocking=True)
                keep.append(pinned)
            done = torch.cuda.Event()
            done.record(self.copy_stream)
        self.stream.wait_event(done)
        dev = {k: v.data_ptr() for k, v in dev_t.items()}
        return nf.BatchArgs(fb.n_tokens, fb.n_prefill_reqs, fb.n_decode_reqs, fb.q_indptr, fb.ctx_len, fb.page_indptr,
                            fb.page_ids, dev, keepalive=(dev_t, keep))

    def step(self, x, out: Optional[torch.Tensor] = None):
        """Forms the next batch and launches it.  x: bf16 [>= n_tokens, D] layer input (rows
        in batch order) resident on the device, or a function of the formed batch that
        returns it.  Returns (formed batch, output tensor or None when the batch is empty);
        the output is valid once the engine's stream reaches this iteration (see drain())."""
        fb = self.sched.next_batch()
        self._swap(fb)
        z = None
        keep = None
        if fb.n_tokens > 0:
            if callable(x):
                x = x(fb)
            args = self._upload(fb)
            bounds = self.bounds_fn(fb.n_tokens) if self.bounds_fn else [0, fb.n_tokens]
            plan = nf.nf_plan_manual(self.ctx, self.model, args, bounds, self.overlap and len(bounds) > 2, 0, 0,
                                     self.attn_wgs)
            need = nf.nf_layers_workspace_bytes(plan, self.n_layers)
            if self.workspace is None or self.workspace.numel() < need:
                # grows rarely; the old buffer stays alive until the iterations using it are done
                old = self.workspace
                self.workspace = torch.empty(int(need * 1.25) + (1 << 20), dtype=torch.uint8, device=self.device)
                keep = old
            z = out if out is not None else torch.empty((fb.n_tokens, self.model.hidden), dtype=torch.bfloat16,
                                                        device=self.device)
            nf.nf_layers_forward(self.ctx, self.model, [w.struct for w in self.weights],
                                 [p.data_ptr() for p in self.pools], self.num_pages, args, plan, x.data_ptr(),
                                 z.data_ptr(), self.workspace.data_ptr(), self.workspace.numel(),
                                 self.stream.cuda_stream)
            keep = (keep, args, plan, x, z)
            self.tokens_launched += fb.n_tokens
        ev = torch.cuda.Event()
        ev.record(self.stream)
        self.pending.append((fb.iteration, ev, keep))
        # end-of-sequence news arrives async_lag iterations late: iteration k - lag must have
        # finished on the GPU before its outputs can be looked at
        while self.pending and self.pending[0][0] <= fb.iteration - self.async_lag:
            it, e, k = self.pending.popleft()
            e.synchronize()
            self.sched.complete(it)
            if k is not None and k[2] is not None:
                k[2].close()
        self.iteration += 1
        return fb, z

    def drain(self):
        """Waits for everything launched and reports the remaining iterations to the scheduler."""
        while self.pending:
            it, e, k = self.pending.popleft()
            e.synchronize()
            self.sched.complete(it)
            if k is not None and k[2] is not None:
                k[2].close()
        self.stream.synchronize()

    def stats(self) -> dict:
        return self.sched.stats()

    def close(self):
        self.drain()
        self.sched.close()
