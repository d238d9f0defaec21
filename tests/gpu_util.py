"""Helpers for the GPU parity tests: build a case from the seeded generators, run the
HIP path through the C-ABI binding and the CPU oracle on the same inputs."""
import numpy as np
import torch

from oracle import decoder_layer as orc
from paper_2408_12757_amd import binding as nf
from paper_2408_12757_amd import harness as hz
from paper_2408_12757_amd import workloads as wl

from parity_metrics import REL_TOL, check_intermediates, tensor_rel_err

# REL_TOL: tolerance for bf16 with fp32 accumulation, max |gpu - ref| / max |ref| per tensor
DEV = "cuda:0"
rel_err = tensor_rel_err


def f64(bits: np.ndarray) -> np.ndarray:
    return orc.widen(bits)


def regions_from_workspace(ws: torch.Tensor, plan, model, B: int, rows=None):
    """bf16 bits of the attention output, y and (dense models) SiLU(gate)*up that the last
    call with this plan's layout left in the workspace; rows: optional row subset."""
    got = {}
    for name, cols in (("attn", model.q_dim), ("y", model.hidden), ("f", model.ffn_inner)):
        if name == "f" and model.is_moe:
            continue        # rows sorted by expert: compared through z only
        off, nb = plan.workspace_region(name)
        t = ws[off:off + nb].view(torch.bfloat16).view(B, cols)
        if rows is not None:
            t = t[torch.as_tensor(np.asarray(rows), device=t.device)]
        got[name] = hz.bf16_bits(t)
    return got


class Case:
    """One synthetic layer problem resident on the GPU, with host copies for the oracle."""

    def __init__(self, model, batch: wl.Batch, seed: int, weights=None, ctx=None):
        self.model = model
        self.batch = batch
        self.weights = weights if weights is not None else wl.make_weights(model, seed)
        self.x_bits = wl.make_x(batch.n_tokens, model.hidden, seed + 1)
        self.pages_bits = wl.make_kv_pages_host(model, batch.num_pages, seed + 3)
        self.pages = hz.bf16_tensor(self.pages_bits, DEV)
        self.runner = hz.LayerRunner(model, self.weights, self.pages, DEV, ctx=ctx)
        self.ctx = self.runner.ctx
        self.args = hz.upload_batch(batch, DEV)
        self.x = hz.bf16_tensor(self.x_bits, DEV)

    def reset_pages(self):
        self.pages.copy_(hz.bf16_tensor(self.pages_bits, DEV))

    def run(self, plan=None):
        """Returns (z bits [B, D], pages bits after the call); keeps the bf16 bits of the
        intermediates the call left in the workspace (attention output, y, SiLU(gate)*up)."""
        self.reset_pages()
        out = self.runner.forward(self.args, self.x, plan)
        torch.cuda.synchronize()
        self.last_regions = self.read_regions(plan)
        return hz.bf16_bits(out), hz.bf16_bits(self.pages)

    def read_regions(self, plan=None):
        """The activation regions lie in front of everything whose size depends on the plan,
        so an unsplit plan of the same batch names the offsets of any run."""
        m, B = self.model, self.batch.n_tokens
        if B == 0:
            return {}
        tmp = plan if plan is not None else nf.nf_plan_manual(self.ctx, m, self.args, [0, B])
        got = regions_from_workspace(self.runner.workspace, tmp, m, B)
        if plan is None:
            tmp.close()
        return got

    def oracle(self, reqs=None):
        b, x, pages = self.batch, self.x_bits, self.pages_bits
        tok = np.arange(b.n_tokens)
        if reqs is not None:
            b, tok, phys = wl.subset_batch(self.batch, reqs)
            x, pages = x[tok], pages[phys]
        z, k, v, parts = orc.layer_forward(self.model, self.weights, pages, b, x, return_parts=True)
        parts["x"] = orc.widen(x)
        return z, k, v, tok, parts

    def check(self, z_bits, pages_bits, reqs=None, tol=REL_TOL, regions=None):
        """Layer output, appended K/V rows and every intermediate the call left in the
        workspace against the oracle, each on its own scale (see parity_metrics)."""
        z, k, v, tok, parts = self.oracle(reqs)
        e_z = rel_err(f64(z_bits[tok]), z)
        kg, vg = hz.read_kv_rows(pages_bits, self.model, self.batch, tok)
        e_k = rel_err(f64(kg), k)
        e_v = rel_err(f64(vg), v)
        assert np.all(np.isfinite(f64(z_bits))), "non-finite output"
        assert e_z <= tol and e_k <= tol and e_v <= tol, (e_z, e_k, e_v)
        regions = self.last_regions if regions is None else regions
        report = check_intermediates(self.model, regions, z_bits, tok, z, parts, tol)
        return (e_z, e_k, e_v), report


def untouched_pages_equal(case: Case, pages_after: np.ndarray) -> bool:
    """Every page slot not written by the append must be unchanged."""
    m, b = case.model, case.batch
    P, Hkv, dh = m.page_size, m.n_kv_heads, m.head_dim
    before = case.pages_bits.reshape(-1, 2, Hkv, P * dh).copy()
    after = pages_after.reshape(-1, 2, Hkv, P * dh).copy()
    tok_req = np.repeat(np.arange(b.n_reqs), np.diff(b.q_indptr))
    kidx, vidx = wl.page_block_index(dh, P)
    for t in range(b.n_tokens):
        r = int(tok_req[t])
        pos = int(b.ctx_len[r]) + int(t - b.q_indptr[r])
        page, slot = int(b.page_ids[int(b.page_indptr[r]) + pos // P]), pos % P
        for arr in (before, after):
            arr[page, 0][:, kidx[slot]] = 0
            arr[page, 1][:, vidx[slot]] = 0
    return bool(np.array_equal(before, after))


class ChainCase:
    """n_layers consecutive layers with their own weights and KV pools on one batch."""

    def __init__(self, model, batch: wl.Batch, seed: int, n_layers: int, ctx=None):
        self.model, self.batch, self.n_layers = model, batch, n_layers
        self.weights = [wl.make_weights(model, seed + 17 * l) for l in range(n_layers)]
        self.pools_bits = [wl.make_kv_pages_host(model, batch.num_pages, seed + 3 + 29 * l) for l in range(n_layers)]
        self.x_bits = wl.make_x(batch.n_tokens, model.hidden, seed + 1)
        self.ctx = ctx or nf.Context(0)
        self.dev_w = [hz.DeviceWeights(w, DEV) for w in self.weights]
        self.pools = [hz.bf16_tensor(p, DEV) for p in self.pools_bits]
        self.args = hz.upload_batch(batch, DEV)
        self.x = hz.bf16_tensor(self.x_bits, DEV)

    def reset(self):
        for t, bits in zip(self.pools, self.pools_bits):
            t.copy_(hz.bf16_tensor(bits, DEV))

    def run_chain(self, plan):
        """One nf_layers_forward call.  Returns (z bits, [pool bits per layer])."""
        self.reset()
        out = torch.empty_like(self.x)
        need = nf.nf_layers_workspace_bytes(plan, self.n_layers)
        ws = torch.empty(need, dtype=torch.uint8, device=DEV)
        nf.nf_layers_forward(self.ctx, self.model, [w.struct for w in self.dev_w], [p.data_ptr() for p in self.pools],
                             self.pools[0].shape[0], self.args, plan, self.x.data_ptr(), out.data_ptr(),
                             ws.data_ptr(), ws.numel(), torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        return hz.bf16_bits(out), [hz.bf16_bits(p) for p in self.pools]

    def run_layer_by_layer(self):
        """n_layers separate nf_layer_forward calls (unsplit), the output of one fed to the next."""
        self.reset()
        cur = self.x
        for l in range(self.n_layers):
            runner = hz.LayerRunner(self.model, self.weights[l], self.pools[l], DEV, ctx=self.ctx)
            runner.w = self.dev_w[l]
            cur = runner.forward(self.args, cur, None)
        torch.cuda.synchronize()
        return hz.bf16_bits(cur), [hz.bf16_bits(p) for p in self.pools]
