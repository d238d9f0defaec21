"""Multi-layer iteration loop with continuous batching (paper Sec. 4.2: request scheduling
and asynchronous scheduling) around the library's scheduler and nf_layers_forward.

This module is plumbing: it owns device memory (weights of every layer, one KV pool per
layer, workspace), two HIP streams and the host copies of swapped-out requests, and it
moves the scheduler's batches to the GPU.  Every decision (which tokens run, which pages
they use, who is swapped) is taken by the library's scheduler; every arithmetic step runs
in the library's kernels.

Two ways to feed an iteration: the caller supplies the layer input (synthetic activations),
or, with a TokenPath, tokens flow through the model: embedding -> layers -> final norm ->
LM head -> greedy sampling, the sampled token of a decode request staying on the device
for the next iteration.  Prompt tokens are synthetic (a hash of request and position), and
"the model emitted EOS" is the request's output length, which the scheduler learns one
iteration late when async_lag = 1 (the paper's asynchronous scheduling).
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


def prompt_token(request_id: int, position: int, vocab: int) -> int:
    """Synthetic prompt: token at `position` of request `request_id`."""
    return (request_id * 7919 + position * 104729 + 17) % vocab


class TokenPath:
    """Embedding table, final norm gain and LM head on the device, plus the buffers of the
    sampling step.  Host arrays (bf16 bits) are given by tests; otherwise drawn on the device."""

    def __init__(self, model: wl.ModelDesc, vocab: int, dense_batch: int, max_requests: int, device,
                 host: Optional[Dict[str, np.ndarray]] = None, seed: int = 0, std: float = 0.02):
        if vocab % 64:
            raise ValueError("vocabulary size must be a multiple of 64 (LM head GEMM)")
        self.vocab, D = vocab, model.hidden
        if host is not None:
            self.table = hz.bf16_tensor(host["embedding"], device)
            self.g_final = hz.bf16_tensor(host["g_final"], device)
            self.w_lm = hz.bf16_tensor(host["w_lm"], device)
        else:
            gen = torch.Generator(device=device)
            gen.manual_seed(seed)

            def normal(shape, mean, sd):
                t = torch.empty(shape, dtype=torch.float32, device=device)
                t.normal_(mean, sd, generator=gen)
                return t.to(torch.bfloat16)
            self.table = normal((vocab, D), 0.0, 1.0)
            self.g_final = normal((D,), 1.0, std)
            self.w_lm = normal((vocab, D), 0.0, std)
        self.slot_tokens = torch.zeros(max_requests, dtype=torch.int32, device=device)
        self.x = torch.empty((dense_batch, D), dtype=torch.bfloat16, device=device)
        self.rows = torch.empty((dense_batch, D), dtype=torch.bfloat16, device=device)
        self.normed = torch.empty((dense_batch, D), dtype=torch.bfloat16, device=device)
        self.logits = torch.empty((dense_batch, vocab), dtype=torch.bfloat16, device=device)
        self.free_slots = list(range(max_requests - 1, -1, -1))
        self.slot_of: Dict[int, int] = {}


def make_token_weights(model: wl.ModelDesc, vocab: int, seed: int, std: float = 0.02) -> Dict[str, np.ndarray]:
    """Host-side (bf16 bits) embedding table ~ N(0,1), final norm gain ~ 1 + N(0, std^2), LM head ~ N(0, std^2)."""
    rng = np.random.default_rng(seed)
    f = wl.f32_to_bf16_bits
    return {"embedding": f(rng.standard_normal((vocab, model.hidden)).astype(np.float32)),
            "g_final": f((1 + std * rng.standard_normal(model.hidden)).astype(np.float32)),
            "w_lm": f((std * rng.standard_normal((vocab, model.hidden))).astype(np.float32))}


class ServingEngine:
    def __init__(self, model: wl.ModelDesc, n_layers: int, num_pages: int, dense_batch: int, max_requests: int,
                 host_weights: Optional[List[Dict[str, Optional[np.ndarray]]]] = None, weight_seed: int = 0,
                 device="cuda:0", async_lag: int = 1, avg_decode_len: float = 256.0, max_chunk: int = 0,
                 reserve_pages: int = 0, zero_pools: bool = False, ctx: Optional[nf.Context] = None,
                 bounds_fn: Optional[Callable[[int], List[int]]] = None, overlap: bool = False, attn_wgs: int = 0,
                 token_path: Optional[TokenPath] = None, auto_search: bool = False, granule: int = 128):
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
        self.tok = token_path
        self.prompt_len: Dict[int, int] = {}
        # auto-search (Sec. 4.1): profile the kernels once, then search the pipeline of every batch
        # with the time per layer of a run of consecutive layers as the objective
        self.auto_search, self.granule = auto_search, granule
        if auto_search:
            nf.nf_profile(self.ctx, model, dense_batch, granule, None)

    # ---- requests ---------------------------------------------------------------------
    def submit(self, prompt_len: int, output_len: int) -> int:
        rid = self.sched.submit(prompt_len, output_len)
        self.prompt_len[rid] = prompt_len
        return rid

    # ---- one iteration ------------------------------------------------------------------
    def _swap(self, fb: nf.FormedBatch):
        for rid in fb.released:
            self.host_store.pop(rid, None)
        # pages are gathered into / scattered from a contiguous device buffer by the library
        # (nf_op_move_pages); torch only allocates the buffers and copies them across the bus
        with torch.cuda.stream(self.stream):
            s = self.stream.cuda_stream
            for rid, pages in fb.swap_out:
                idx = torch.from_numpy(np.ascontiguousarray(pages, dtype=np.int32)).to(self.device)
                saved = []
                for pool in self.pools:
                    line = torch.empty((len(pages), pool.shape[1]), dtype=pool.dtype, device=self.device)
                    nf.nf_op_move_pages(pool.data_ptr(), pool.shape[1] * pool.element_size(), pool.shape[0],
                                        idx.data_ptr(), len(pages), line.data_ptr(), False, s)
                    host = torch.empty((len(pages), pool.shape[1]), dtype=pool.dtype, pin_memory=True)
                    host.copy_(line, non_blocking=True)
                    saved.append(host)
                self.host_store[rid] = saved
            for rid, pages in fb.swap_in:
                idx = torch.from_numpy(np.ascontiguousarray(pages, dtype=np.int32)).to(self.device)
                saved = self.host_store.pop(rid)
                for pool, host in zip(self.pools, saved):
                    line = host.to(self.device, non_blocking=True)
                    nf.nf_op_move_pages(pool.data_ptr(), pool.shape[1] * pool.element_size(), pool.shape[0],
                                        idx.data_ptr(), len(pages), line.data_ptr(), True, s)

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

    def _token_arrays(self, fb: nf.FormedBatch):
        """Host arrays of the token path for one batch: prompt token ids, the slot a decode
        token is read from (-1: use the id), the rows that need a next token and their slots."""
        tp = self.tok
        for rid in fb.finished:
            slot = tp.slot_of.pop(rid, None)
            if slot is not None:
                tp.free_slots.append(slot)
            self.prompt_len.pop(rid, None)
        ids = np.zeros(fb.n_tokens, np.int32)
        from_slot = np.full(fb.n_tokens, -1, np.int32)
        rows, slots = [], []
        for i in range(fb.n_prefill_reqs + fb.n_decode_reqs):
            rid, t0, t1, ctx = int(fb.request_ids[i]), int(fb.q_indptr[i]), int(fb.q_indptr[i + 1]), int(fb.ctx_len[i])
            if rid not in tp.slot_of:
                tp.slot_of[rid] = tp.free_slots.pop()
            slot = tp.slot_of[rid]
            if i >= fb.n_prefill_reqs:
                from_slot[t0] = slot
                rows.append(t0)
                slots.append(slot)
            else:
                for t in range(t0, t1):
                    ids[t] = prompt_token(rid, ctx + t - t0, tp.vocab)
                if ctx + (t1 - t0) == self.prompt_len[rid]:  # the chunk ends the prompt: first token comes out
                    rows.append(t1 - 1)
                    slots.append(slot)
        return ids, from_slot, np.array(rows, np.int32), np.array(slots, np.int32)

    def _to_device(self, arrays: List[np.ndarray]):
        """Pinned staging on the copy stream; the iteration stream waits for the copies."""
        dev, keep = [], []
        with torch.cuda.stream(self.copy_stream):
            for a in arrays:
                pinned = torch.from_numpy(np.ascontiguousarray(a if a.size else np.zeros(1, a.dtype))).pin_memory()
                dev.append(pinned.to(self.device, non_blocking=True))
                keep.append(pinned)
            done = torch.cuda.Event()
            done.record(self.copy_stream)
        self.stream.wait_event(done)
        return dev, keep

    def step(self, x=None, out: Optional[torch.Tensor] = None):
        """Forms the next batch and launches it.  x: bf16 [>= n_tokens, D] layer input (rows
        in batch order) resident on the device, or a function of the formed batch that
        returns it.  Returns (formed batch, output tensor or None when the batch is empty);
        the output is valid once the engine's stream reaches this iteration (see drain())."""
        fb = self.sched.next_batch()
        self._swap(fb)
        z = None
        keep = None
        tok_keep = None
        if fb.n_tokens > 0:
            if self.tok is not None:
                tp = self.tok
                ids, from_slot, rows, slots = self._token_arrays(fb)
                (d_ids, d_from, d_rows, d_slots), pinned = self._to_device([ids, from_slot, rows, slots])
                nf.nf_op_embedding(d_ids.data_ptr(), d_from.data_ptr(), tp.slot_tokens.data_ptr(), tp.table.data_ptr(),
                                   tp.vocab, tp.x.data_ptr(), fb.n_tokens, self.model.hidden, self.stream.cuda_stream)
                x = tp.x
                tok_keep = (d_ids, d_from, d_rows, d_slots, pinned, len(rows))
            elif callable(x):
                x = x(fb)
            args = self._upload(fb)
            if self.auto_search and fb.n_tokens >= 2 * self.granule:
                # per-iteration planning stays cheap: common boundaries (4 ms of host time, hidden behind
                # the previous iteration); the partition pass (13 ms) gains nothing on this loop's batches
                plan = nf.nf_plan_search(self.ctx, self.model, args, 0, self.granule,
                                         layers=max(1, min(16, self.n_layers)), refine=1)
            else:
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
            if tok_keep is not None and tok_keep[5] > 0:
                tp, n_rows, st = self.tok, tok_keep[5], self.stream.cuda_stream
                D = self.model.hidden
                # rows that need a next token -> final norm -> LM head -> greedy sampling into the slots
                nf.nf_op_embedding(tok_keep[2].data_ptr(), None, None, z.data_ptr(), fb.n_tokens, tp.rows.data_ptr(),
                                   n_rows, D, st)
                nf.nf_op_rmsnorm(tp.rows.data_ptr(), tp.g_final.data_ptr(), tp.normed.data_ptr(), n_rows, D,
                                 self.model.rms_eps, st)
                nf.nf_op_gemm(tp.normed.data_ptr(), tp.w_lm.data_ptr(), tp.logits.data_ptr(), None, n_rows, tp.vocab, D,
                              nf.NF_EPI_NONE, st)
                nf.nf_op_argmax(tp.logits.data_ptr(), n_rows, tp.vocab, tok_keep[3].data_ptr(),
                                tp.slot_tokens.data_ptr(), st)
            keep = (keep, args, plan, x, z, tok_keep)
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
