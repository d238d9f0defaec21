"""Co-run measurements behind the resource-mapping table (paper Sec. 4.1.1): what the GEMM
nano-operations and the decode-attention kernel cost each other on one MI355X.  Run through
``python bench.py --corun-report``; prints a plain-text report.

rocprofv3 cannot provide per-kernel counters of two kernels that overlap: with --pmc it
serialises the dispatches (see profiles/corun_c2.txt), so everything here is timed with HIP
events on the streams the kernels run on, plus a probe kernel of the library
(nf_probe_load_latency) that reports what an L2-resident load waits for beside the attention
kernel.  Only plumbing and timing: every kernel is the library's.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as nf
from . import harness as hz
from . import workloads as wl


def _ev():
    return torch.cuda.Event(enable_timing=True)


def run(config: str = "C2", out=print):
    cfg = wl.CONFIGS[config]
    case = hz.DeviceCase(cfg, n_weight_copies=4, keep_host_weights=False)
    m, B, ctx, dev = cfg.model, case.batch.n_tokens, case.ctx, case.device
    sa = torch.cuda.ExternalStream(ctx.lane_stream(1, 0, 0))
    sb = torch.cuda.ExternalStream(ctx.lane_stream(0, 0, 0))
    D, I, NQ, QD = m.hidden, m.ffn_inner, m.n_qkv, m.q_dim
    g = torch.Generator(device=dev)
    g.manual_seed(1)

    def rnd(*shape, scale=1.0):
        return (scale * torch.randn(*shape, device=dev, generator=g, dtype=torch.float32)).to(torch.bfloat16)
    qkv_full, attn_full = rnd(B, NQ), torch.empty(B, QD, dtype=torch.bfloat16, device=dev)
    W = [r.w.t for r in case.runners]

    def attention_launcher(wgs):
        plan = nf.nf_plan_manual(ctx, m, case.args, [0, B], False, 0, 0, wgs)
        ws = torch.empty(plan.workspace_bytes, dtype=torch.uint8, device=dev)

        def launch(stream):
            nf.nf_op_attention(ctx, m, case.pages.data_ptr(), case.batch.num_pages, case.args, plan, qkv_full.data_ptr(),
                               attn_full.data_ptr(), ws.data_ptr(), ws.numel(), 0, stream)
        return launch, (plan, ws)

    out(f"# co-run report, workload {cfg.name}: {cfg.description}; {case.batch.n_decode_reqs} decode requests, "
        f"{int(case.batch.ctx_len.sum())} cached tokens; device with {ctx.num_cus} CUs")

    # ---- A. what a cache-resident load waits for -------------------------------------------------
    out("\n## A. latency of L2-resident loads (nf_probe_load_latency: 64 single-wavefront workgroups, 4000 dependent "
        "loads each; nanoseconds per load)")
    n_probe, iters = 64, 4000
    res = torch.zeros(2 * n_probe, dtype=torch.float32, device=dev)
    nf.nf_probe_load_latency(ctx, n_probe, 200, res.data_ptr(), sb.cuda_stream)
    torch.cuda.synchronize()

    def probe_stats():
        v = res.cpu().numpy()[0::2]
        return float(np.percentile(v, 10)), float(np.median(v)), float(np.percentile(v, 90))
    nf.nf_probe_load_latency(ctx, n_probe, iters, res.data_ptr(), sb.cuda_stream)
    torch.cuda.synchronize()
    out("   beside nothing:                        p10 %7.0f  median %7.0f  p90 %7.0f" % probe_stats())
    for wgs in (128, 176, 256):
        launch, keep = attention_launcher(wgs)
        launch(sa.cuda_stream)
        torch.cuda.synchronize()
        e0 = _ev()
        e0.record(sa)
        for _ in range(4):
            launch(sa.cuda_stream)
        sb.wait_event(e0)
        nf.nf_probe_load_latency(ctx, n_probe, iters, res.data_ptr(), sb.cuda_stream)
        torch.cuda.synchronize()
        out("   beside attention on %3d workgroups:    p10 %7.0f  median %7.0f  p90 %7.0f   (p10: probes on CUs without "
            "attention wavefronts, p90: on CUs that host them)" % ((wgs,) + probe_stats()))
        keep[0].close()

    # ---- B. fixed work, two lanes -------------------------------------------------------------------
    out("\n## B. fixed work on two streams: 2 attention launches over the whole batch beside GEMM groups (O, Up/Gate, "
        "Down, KQV at M rows, cold weights) worth half the attention time - the layer's own ratio")
    out("   columns: M, attention workgroups, GEMM implementation (0 = automatic), attention alone ms, GEMM groups alone ms, "
        "end of attention ms, end of GEMMs ms, best sequential / makespan")
    best_seq = {}
    for M in (1024, 512):
        x, a_in, f_in = rnd(M, D), rnd(M, QD), rnd(M, I, scale=0.1)
        qkv_o, y_o = torch.empty(M, NQ, dtype=torch.bfloat16, device=dev), torch.empty(M, D, dtype=torch.bfloat16, device=dev)
        f_o, z_o = torch.empty(M, I, dtype=torch.bfloat16, device=dev), torch.empty(M, D, dtype=torch.bfloat16, device=dev)

        def group(i, s):
            w = W[i % len(W)]
            nf.nf_op_gemm(a_in.data_ptr(), w["w_o"].data_ptr(), y_o.data_ptr(), x.data_ptr(), M, D, QD, nf.NF_EPI_RESIDUAL, s)
            nf.nf_op_gemm(x.data_ptr(), w["w_gate_up"].data_ptr(), f_o.data_ptr(), None, M, I, D, nf.NF_EPI_SWIGLU, s)
            nf.nf_op_gemm(f_in.data_ptr(), w["w_down"].data_ptr(), z_o.data_ptr(), y_o.data_ptr(), M, D, I, nf.NF_EPI_RESIDUAL, s)
            nf.nf_op_gemm(x.data_ptr(), w["w_qkv"].data_ptr(), qkv_o.data_ptr(), None, M, NQ, D, nf.NF_EPI_NONE, s)

        def timed(launch, n_attn, n_groups, tile):
            nf.nf_tune_set("gemm.tile", tile)
            try:
                torch.cuda.synchronize()
                e0, ea, eb = _ev(), _ev(), _ev()
                e0.record(torch.cuda.current_stream())
                sa.wait_event(e0)
                sb.wait_event(e0)
                for _ in range(n_attn):
                    launch(sa.cuda_stream)
                ea.record(sa)
                for i in range(n_groups):
                    group(i, sb.cuda_stream)
                eb.record(sb)
                torch.cuda.synchronize()
            finally:
                nf.nf_tune_set("gemm.tile", 0)
            return e0.elapsed_time(ea), e0.elapsed_time(eb)
        rows = []
        for wgs in (128, 176, 256):
            launch, keep = attention_launcher(wgs)
            for tile in (0, 22, 19, 8):
                timed(launch, 1, 1, tile)
                a_solo, _ = timed(launch, 2, 0, tile)
                _, g4 = timed(launch, 0, 4, tile)
                n_groups = max(1, int(round(0.5 * a_solo / (g4 / 4))))
                _, g_solo = timed(launch, 0, n_groups, tile)
                ta, tb = timed(launch, 2, n_groups, tile)
                rows.append((M, wgs, tile, a_solo, g_solo, n_groups, ta, tb))
            keep[0].close()
        # the yardstick: the fastest attention and the fastest GEMM form, one after the other
        a_best = min(r[3] for r in rows)
        for r in rows:
            g_ref = min(q[4] / q[5] for q in rows) * r[5]
            out("   %5d %4d %3d   %7.3f %7.3f   %7.3f %7.3f   %5.3f" % (r[0], r[1], r[2], r[3], r[4], r[6], r[7],
                                                                     (a_best + g_ref) / max(r[6], r[7])))
        best_seq[M] = a_best

    # ---- C. the layer's own timeline ------------------------------------------------------------------
    out("\n## C. kernel timeline of one layer iteration (HIP events around every kernel; start, end, duration in "
        "microseconds; lane 0 = GEMM lane, lane 1 = attention lane)")
    specs = [("unsplit", [0, B], [0], None, False),
             ("two nano-batches overlapped, automatic attention grid", [0, B // 2, B], [0, 0], None, True),
             ("two nano-batches overlapped, attention of the second on 128 workgroups", [0, B // 2, B], [0, 128], None, True),
             ("two nano-batches overlapped, 256 attention workgroups, 128x256 GEMM tiles beside them", [0, B // 2, B],
              [0, 256], [[22] * 4, [0] * 4], True)]
    # a partition per operation (the shape the search's last pass proposes for this layer): KQV and
    # Down whole, attention / O / Up-Gate cut at three quarters of the batch, so that only the
    # second attention nano-operation has GEMMs (O and Up/Gate of the first rows) beside it
    cut = max(1, B * 3 // 4)
    split = [0, cut, B] if cut < B else [0, B]
    specs.append(("a partition per operation: attention, O and Up/Gate cut at 3/4 of the batch, KQV and Down whole; "
                  "attention on 192 then 128 workgroups, O and Up/Gate as 128x256 tiles (with O as 256x256 tiles, which take whole CUs and "
                  "start together with the second attention piece, that piece lands two workgroups to a CU: 980 instead of 615 us)",
                  dict(KQV=[0, B], ATTN=split, O=split, UG=split, D=[0, B]), [192, 128][:len(split) - 1], [0, 21, 21, 0],
                  True))
    for name, bounds, wgs, tiles, overlap in specs:
        if isinstance(bounds, dict):
            p = nf.nf_plan_manual_parts(ctx, m, case.args, bounds, overlap, wgs, tiles)
        else:
            p = nf.nf_plan_manual_ops(ctx, m, case.args, bounds, overlap, wgs, tiles)
        t = hz.time_plan(case, p, 3, 10)
        out(f"   -- {name}: bounds {bounds}, {t:.3f} ms per step untraced")
        ctx.set_trace(2)
        case.forward(p, 0)
        torch.cuda.synchronize()
        recs = ctx.read_trace()
        ctx.set_trace(0)
        for r in recs:
            st, ms = r["start_ms"] * 1e3, r["ms"] * 1e3
            out("      %8.1f %8.1f %7.1f  %-12s %-4s piece %d, tokens [%d, %d)" % (st, st + ms, ms, r["kernel"], r["op"],
                                                                              r["nano"], r["tok_begin"], r["tok_end"]))
        p.close()
    case.ctx.close()
