#!/usr/bin/env python3
"""Benchmark of one device's Astra attention layer on one MI355X.

A step is one astra_layer_forward call: grouped VQ encode of the local rows, K-hat/V-hat projection of
the rows rebuilt from the peers' codes (decode fused into the operand load), Q/K/V projection of the
local rows, mixed-precision attention (Eq. 1) and the output projection.  Inputs are seeded synthetic
tensors already resident in HBM; the peers' codes are produced by the library's own encode.  Prints
ONE JSON line: tokens/s per layer (local rows per second), the MFMA roofline of the dominant kernel
(the grouped projection launch, which at the benchmark shape also carries the encode as extra
workgroups) from HIP-event stage timing, and the CPU oracle timed on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}       # MI355X: dense bf16 MFMA peak; fp32 vector-ALU peak
STAGES = ("vq_encode", "projections", "attention", "out_projection")
N_EVENT_CALLS = 24      # calls that carry stage events, run after the timed region, whatever --steps is


def layer_flops(cfg, n_before):
    """Algorithmic FLOPs of one call, per stage (masked-out causal work is not counted)."""
    D, dq, dkv, dh = cfg.d_model, cfg.n_q_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim, cfg.head_dim
    tl, tq = cfg.n_local, cfg.n_local + cfg.n_cls
    t_vis = n_before if cfg.causal else cfg.n_nonlocal
    pairs = tl * t_vis + tl * (tl + 1) // 2 if cfg.causal else tq * (tq + t_vis)
    return {
        "vq_encode": 2.0 * tl * cfg.codebook_size * D,
        "projections": 2.0 * D * (tq * (dq + 2 * dkv) + t_vis * 2 * dkv),
        "attention": 4.0 * dh * cfg.n_q_heads * pairs,
        "out_projection": 2.0 * tq * dq * D,
    }


def counter_from_profile(path, counter, kernel_substr):
    """Mean value per dispatch of `counter` for the first kernel whose name contains kernel_substr, read from a summary
    that paper_2505_19342_amd.rocprof_summary wrote under profiles/ (None when the file or the line is missing)."""
    try:
        lines = open(path).read().splitlines()
    except OSError:
        return None
    for ln in lines:
        parts = ln.split(None, 2)
        if len(parts) == 3 and parts[0] == counter and kernel_substr in parts[2]:
            try:
                return float(parts[1])
            except ValueError:
                return None
    return None


def traffic_from_profiles(stem, kernel_substr, copy_kib=262144.0):
    """HBM-side bytes per dispatch of a kernel from the two rocprofv3 --pmc summaries profiles/<stem>_pmc_fetch_size.txt and
    ..._write_size.txt (KiB per dispatch), each scaled by what the same counter reads for the plain 256 MiB copy kernel the
    same run launched (torch's AUnaryFunctor elementwise kernel: reads and writes copy_kib KiB)."""
    total = 0.0
    for kind in ("fetch", "write"):
        path = os.path.join(ROOT, "profiles", f"{stem}_pmc_{kind}_size.txt")
        name = "FETCH_SIZE" if kind == "fetch" else "WRITE_SIZE"
        v, cal = counter_from_profile(path, name, kernel_substr), counter_from_profile(path, name, "AUnaryFunctor")
        if v is None or not cal:
            return None
        total += v * (copy_kib / cal) * 1024.0
    return total


def make_layer_call(cfg, rank, data=None):
    """Device-resident tensors of one astra_layer_forward call of a workload on simulated device `rank`; the peers' codes are
    produced by the library's own encode of their rows (what they would have transmitted)."""
    import torch
    from paper_2505_19342_amd import binding as B
    from paper_2505_19342_amd import workloads as wl
    dev = "cuda:0"
    data = wl.generate(cfg) if data is None else data
    view = wl.device_view(cfg, data, rank)
    dt = cfg.dtype
    G, K, D = cfg.n_groups, cfg.codebook_size, cfg.d_model

    def to_dev(a):
        a = np.ascontiguousarray(a, dtype=np.float32)
        if dt == "bf16":
            return torch.from_numpy(wl.bf16_bits(a).view(np.int16)).to(dev).view(torch.bfloat16)
        return torch.from_numpy(a).to(dev)

    code_t = torch.uint8 if K <= 256 else torch.int16
    vq = B.vq_desc(dt, D, G, K)
    codebook = to_dev(data["codebook"])
    cnorm = torch.empty((G, K), dtype=torch.float32, device=dev)
    B.astra_vq_prepare(vq, codebook, cnorm)
    x_nl = to_dev(view["x_nonlocal"])
    tn = x_nl.shape[0]
    codes_nl = torch.empty((tn, G), dtype=code_t, device=dev)
    B.astra_vq_encode(vq, x_nl, tn, codebook, cnorm, codes_nl)
    del x_nl
    x_local = to_dev(view["x_local"])
    tq = x_local.shape[0]
    desc = B.LayerDesc(vq, B.attn_desc(dt, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.n_cls, tq - cfg.n_cls, tn,
                                       cfg.causal, view["n_before"]))
    w = [to_dev(np.ascontiguousarray(data[n].T)) for n in ("wq", "wk", "wv", "wo")]
    y = torch.empty((tq, D), dtype=torch.float32, device=dev)
    codes_local = torch.empty((tq - cfg.n_cls, G), dtype=code_t, device=dev)
    ws = torch.empty(max(B.astra_layer_workspace_bytes(desc), 256), dtype=torch.uint8, device=dev)
    call_args = (desc, x_local, codes_nl, codebook, cnorm, *w, None, None, None, None, y, codes_local, ws)
    return {"cfg": cfg, "rank": rank, "data": data, "view": view, "to_dev": to_dev, "code_t": code_t, "vq": vq, "codebook": codebook,
            "cnorm": cnorm, "codes_nl": codes_nl, "x_local": x_local, "tq": tq, "tn": tn, "desc": desc, "w": w, "y": y,
            "codes_local": codes_local, "ws": ws, "call_args": call_args}


def preheat(fn, min_ms, sync):
    """Calls fn back to back for at least min_ms of wall clock (in runs of 64 calls, each followed by a synchronisation, so
    the host never gets far ahead): after host-side set-up the chip sits at an idle clock and needs a few hundred
    milliseconds of load to settle at the clock it holds under this work.  Returns (calls made, seconds)."""
    t0, n = time.perf_counter(), 0
    while (time.perf_counter() - t0) * 1e3 < min_ms:
        for _ in range(64):
            fn()
        n += 64
        sync()
    return n, time.perf_counter() - t0


def stage_times(lc, n_calls):
    """Per-stage HIP-event spans (ms) of n_calls back-to-back astra_layer_forward_profiled calls: median and mean per stage,
    and the sorted whole-call spans.  Events: 0 entry, 1 projection launch done, 5/6 around the encode if it ran as a kernel of
    its own (otherwise it ran inside the projection launch and 5..6 is empty), 2 attention done, 3 output projection done,
    4 exit.  Back to back, a span starts when the previous kernel ends, so it is the kernel's duration plus one launch gap."""
    import torch
    from paper_2505_19342_amd import binding as B
    evs = [B.HipEvents(7) for _ in range(n_calls)]
    for _ in range(8):
        B.astra_layer_forward(*lc["call_args"])
    for ev in evs:
        B.astra_layer_forward_profiled(*lc["call_args"], ev.handles)
    torch.cuda.synchronize()
    spans = {"vq_encode": (5, 6), "projections": (0, 1), "attention": (6, 2), "out_projection": (2, 3)}
    per = {s: [ev.elapsed_ms(*spans[s]) for ev in evs] for s in STAGES}
    whole = sorted(ev.elapsed_ms(0, 4) for ev in evs)
    return {s: float(np.median(v)) for s, v in per.items()}, {s: float(np.mean(v)) for s, v in per.items()}, whole


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=200, help="untimed calls right before the timed region")
    ap.add_argument("--preheat-ms", type=float, default=400.0,
                    help="before the --warmup calls, run the same call back to back for at least this long: after the host-side "
                         "set-up the chip needs some hundred milliseconds of load to reach the clock it holds under this work, "
                         "and a warm-up given as a call count alone would make the result depend on --steps / --warmup")
    ap.add_argument("--workload", default="llama3_8b_bf16")
    ap.add_argument("--rank", type=int, default=-1, help="simulated device (default: last = critical path under causal masking)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the measurements outside the timed region")
    ap.add_argument("--extras", default="all",
                    help="comma list of the measurements outside the timed region to run: ranks, preprojected, workloads, sweep, uneven, lost, block, "
                         "stack (needs block), kv, kvcache, train, decode, gather, gather_x8, vendor, probe (default all)")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="before the warm-up, run one plain elementwise copy kernel reading and writing this many MiB "
                         "(fp32): the reference that scales rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one device's share on ONE GPU; the exchange of codes between devices is not "
              "part of this build, so --gpus must be 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2505_19342_amd import binding as B
    from paper_2505_19342_amd import workloads as wl

    if not torch.cuda.is_available():
        print("no GPU visible: the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(1)
    B.load(build_if_missing=True)
    dev = "cuda:0"
    cfg = wl.CONFIGS[args.workload]
    rank = args.rank if args.rank >= 0 else cfg.n_dev - 1
    lc = make_layer_call(cfg, rank)
    data, view, to_dev, code_t, vq = lc["data"], lc["view"], lc["to_dev"], lc["code_t"], lc["vq"]
    codebook, cnorm, codes_nl, x_local, tq, tn = lc["codebook"], lc["cnorm"], lc["codes_nl"], lc["x_local"], lc["tq"], lc["tn"]
    desc, w, y, codes_local, ws, call_args = lc["desc"], lc["w"], lc["y"], lc["codes_local"], lc["ws"], lc["call_args"]
    dt = cfg.dtype
    G, K, D = cfg.n_groups, cfg.codebook_size, cfg.d_model

    if args.calibration_copy_mib > 0:
        n = args.calibration_copy_mib * (1 << 20) // 4
        src = torch.ones(n, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.mul(src, 1.0, out=dst)          # one elementwise kernel: reads n*4 bytes, writes n*4 bytes
        torch.cuda.synchronize()
        del src, dst

    step = lambda: B.astra_layer_forward(*call_args)
    preheat_calls, preheat_s = preheat(step, args.preheat_ms, torch.cuda.synchronize) if args.preheat_ms > 0 else (0, 0.0)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # ---- timed region: exactly `steps` calls of astra_layer_forward, back to back, wall clock between two synchronisations.
    # Up to ten torch events on the launch stream cut the region into blocks of equal length (an event record between two
    # calls costs no measurable gap): the spread of the per-call time over the region.
    n_blocks = min(10, args.steps)
    edges = [round(i * args.steps / n_blocks) for i in range(n_blocks + 1)]
    marks = [torch.cuda.Event(enable_timing=True) for _ in edges]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    nxt = 0
    for i in range(args.steps):
        if i == edges[nxt]:
            marks[nxt].record()
            nxt += 1
        step()
    marks[-1].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    block_ms = sorted(marks[i].elapsed_time(marks[i + 1]) / (edges[i + 1] - edges[i]) for i in range(n_blocks))

    # ---- stage times: a fixed number of event-carrying calls after the timed region
    stage_ms, stage_ms_mean, per_step = stage_times(lc, N_EVENT_CALLS)

    flops = layer_flops(cfg, view["n_before"])
    total_flops = sum(flops.values())
    peak = PEAK_TFLOPS[dt]
    dom = "projections"
    # where the shape allows, the projection launch also runs the encode of the local rows (extra workgroups on
    # compute units its tiles leave idle): the launch's algorithmic work is then both
    enc_fused = B.astra_layer_encode_fused(desc)
    dom_flops = flops[dom] + (flops["vq_encode"] if enc_fused else 0.0)
    achieved = dom_flops / (stage_ms[dom] * 1e-3) / 1e12

    def timed(fn, n, warm=0):
        for _ in range(1 + warm):
            fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(n):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / n          # ms

    if enc_fused:
        # no span of its own inside the layer: time the same encode as a kernel of its own, for reference
        x_enc = x_local[cfg.n_cls:]
        stage_ms["vq_encode"] = timed(lambda: B.astra_vq_encode(vq, x_enc, tq - cfg.n_cls, codebook, cnorm, codes_local), 20, warm=5)
    is_bench_shape = cfg.name == "llama3_8b_bf16" and rank == cfg.n_dev - 1
    result = {
        "metric": "tokens/sec per layer (VQ encode + mixed attention) and % of MFMA roofline",
        "value": tq / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dt, "data": "synthetic",
        "config": {"workload": cfg.name, "rank": rank, "n_dev": cfg.n_dev, "local_rows": tq, "nonlocal_rows": tn,
                   "visible_nonlocal_rows": view["n_before"] if cfg.causal else tn, "d_model": D,
                   "heads": [cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim], "vq": {"G": G, "K": K, "dg": cfg.group_dim},
                   "causal": cfg.causal, "seed": cfg.seed},
        "preheat": {"ms_requested": args.preheat_ms, "calls": preheat_calls, "seconds": preheat_s,
                    "what": "the same call back to back before the --warmup calls, so that the timed region runs at the clock "
                            "the chip holds under this work"},
        "layer_tflops": total_flops / (ms_per_step * 1e-3) / 1e12,
        "layer_mfma_frac": total_flops / (ms_per_step * 1e-3) / 1e12 / peak,
        "ms_per_step_blocks_p10_p50_p90": [block_ms[int(q * (len(block_ms) - 1))] for q in (0.1, 0.5, 0.9)],
        "steps_with_events": N_EVENT_CALLS,
        "gpu_ms_per_step_events_p10_p50_p90": [per_step[int(q * (len(per_step) - 1))] for q in (0.1, 0.5, 0.9)],
        "encode_fused_into_projection_launch": bool(enc_fused),
        "stage_us": {s: stage_ms[s] * 1e3 for s in STAGES},
        "stage_us_mean": {s: stage_ms_mean[s] * 1e3 for s in STAGES},
        "stage_tflops": {s: (dom_flops if s == dom else flops[s]) / (stage_ms[s] * 1e-3) / 1e12 for s in STAGES},
        "stage_mfma_frac": {s: (dom_flops if s == dom else flops[s]) / (stage_ms[s] * 1e-3) / 1e12 / peak for s in STAGES},
        "roofline": {"kernel": ("gemm_nt_bf16_kernel (grouped Q/K/V/K-hat/V-hat projections" +
                                (" + VQ encode of the local rows as extra workgroups)" if enc_fused else ")")) if dt == "bf16"
                     else "gemm_nt_f32_kernel (grouped projections)",
                     "bound": "mfma" if dt == "bf16" else "alu", "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
                     "frac": achieved / peak,
                     # HBM-side bytes per launch from the rocprofv3 --pmc summaries kept under profiles/
                     "traffic": traffic_from_profiles("layer_llama3_8b", "gemm_nt_bf16_kernel<256, 256") if is_bench_shape else None,
                     "flops_per_launch": dom_flops, "us_per_launch": stage_ms[dom] * 1e3,
                     "how": f"median HIP-event span (entry of the call to the end of the launch) over {N_EVENT_CALLS} back-to-back calls "
                            "after the timed region"},
    }

    extras = set() if args.no_extras else set(("ranks,preprojected,workloads,sweep,uneven,lost,block,stack,kv,kvcache,train,decode,gather,gather_x8,vendor,probe" if args.extras == "all" else args.extras).split(","))
    if extras:
        # (1) the other simulated devices (under causal masking they see fewer non-local rows)
        if "ranks" in extras and cfg.causal and args.rank < 0:
            per_rank = {}
            for r in range(cfg.n_dev):
                vr = wl.device_view(cfg, data, r)
                xr = to_dev(vr["x_local"])
                dr = B.LayerDesc(vq, B.attn_desc(dt, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.n_cls, xr.shape[0] - cfg.n_cls,
                                                 tn, cfg.causal, vr["n_before"]))
                # the peers' codes in this rank's order: encode its non-local rows with the library
                xn = to_dev(vr["x_nonlocal"])
                cn = torch.empty((tn, G), dtype=code_t, device=dev)
                B.astra_vq_encode(vq, xn, tn, codebook, cnorm, cn)
                a_r = (dr, xr, cn, codebook, cnorm, *w, None, None, None, None, y, codes_local, ws)
                per_rank[r] = timed(lambda: B.astra_layer_forward(*a_r), 100, warm=100)
                del xr, xn, cn
            result["per_rank_ms"] = per_rank
            result["rank_mean_tokens_per_s"] = tq / (sum(per_rank.values()) / len(per_rank) * 1e-3)
        # (1b) the other named workloads (tiny ViT fp32, ViT-Base bf16 with class rows, GPT-2-small bf16 causal): per layer call on the
        # last simulated device, tokens/s, TFLOP/s, fraction of the peak of their arithmetic, and the oracle timed beside them
        def oracle_layer_seconds(lcw, budget_s, max_calls):
            import oracle
            c, d, v = lcw["cfg"], lcw["data"], lcw["view"]
            ch = lcw["codes_nl"].cpu().numpy()
            ch = (ch.view(np.uint16) if c.codebook_size > 256 else ch).astype(np.int32)
            oracle.num_threads()
            n, c0 = 0, time.perf_counter()
            while n < max_calls and (n == 0 or time.perf_counter() - c0 < budget_s):
                oracle.layer_forward(v["x_local"], ch, d["codebook"], d["wq"], d["wk"], d["wv"], d["wo"], n_q_heads=c.n_q_heads,
                                     n_kv_heads=c.n_kv_heads, n_cls=c.n_cls, causal=c.causal, n_before=v["n_before"])
                n += 1
            return (time.perf_counter() - c0) / n, n, oracle.num_threads()

        def measure_layer(lcw, n=300, warm=100):
            c = lcw["cfg"]
            ms = timed(lambda: B.astra_layer_forward(*lcw["call_args"]), n, warm=warm)
            fl = layer_flops(c, lcw["view"]["n_before"])
            tot = sum(fl.values())
            return ms, fl, tot

        def preprojected_tables(lcw):
            c = lcw["cfg"]
            dkv_ = c.n_kv_heads * c.head_dim
            pk = torch.empty((c.n_groups, c.codebook_size, dkv_), dtype=torch.float32, device=dev)
            pv = torch.empty_like(pk)
            B.astra_vq_project_codebook(lcw["vq"], lcw["codebook"], lcw["w"][1], dkv_, pk)
            B.astra_vq_project_codebook(lcw["vq"], lcw["codebook"], lcw["w"][2], dkv_, pv)
            return pk, pv

        # (1a) the benchmark shape with one or two groups (the paper's strongest compression, G = 1): the layer with K-hat, V-hat
        # projected from rebuilt rows, and with K-hat, V-hat looked up in pre-projected codebooks
        if "preprojected" in extras and args.workload == "llama3_8b_bf16":
            import dataclasses
            out_p = []
            for g_ in (1, 2):
                c = dataclasses.replace(cfg, name=f"llama3_8b_bf16_G{g_}", n_groups=g_)
                d_ = dict(data)
                d_["codebook"] = wl.round_to_bf16(np.random.default_rng(cfg.seed + 900 + g_).standard_normal(
                    (g_, c.codebook_size, c.group_dim), dtype=np.float32))
                lcw = make_layer_call(c, rank, data=d_)
                ms_gemm = timed(lambda: B.astra_layer_forward(*lcw["call_args"]), 100, warm=30)
                pk, pv = preprojected_tables(lcw)
                a_ = lcw["call_args"]
                pa = (a_[0], a_[1], a_[2], None, a_[3], a_[4], pk, pv, *a_[5:])
                ms_pre = timed(lambda: B.astra_layer_forward_preprojected(*pa), 100, warm=30)
                x_enc = lcw["x_local"]
                ms_enc = timed(lambda: B.astra_vq_encode(lcw["vq"], x_enc, lcw["tq"], lcw["codebook"], lcw["cnorm"], lcw["codes_local"]), 20, warm=5)
                ms_tab = timed(lambda: preprojected_tables(lcw), 5, warm=1)
                out_p.append({"G": g_, "K": c.codebook_size, "dg": c.group_dim, "ms_projecting_rebuilt_rows": ms_gemm, "ms_preprojected": ms_pre,
                              "encode_alone_ms": ms_enc, "tables_once_ms": ms_tab, "table_bytes": 2 * pk.numel() * 4,
                              "tokens_per_s_preprojected": lcw["tq"] / (ms_pre * 1e-3)})
                del pk, pv, lcw
            result["preprojected_codebooks"] = {"cases": out_p, "what": "the benchmark shape with G = 1 and G = 2 (K 1024): astra_layer_forward against "
                                                "astra_layer_forward_preprojected (K-hat, V-hat = sums of G rows of tables built once per codebook and weights)"}
        if "workloads" in extras and args.workload == "llama3_8b_bf16":
            out_w = {}
            for name in ("tiny_vit_f32", "vit_base_bf16", "gpt2_small_bf16"):
                c = wl.CONFIGS[name]
                lcw = make_layer_call(c, c.n_dev - 1)
                ms, fl, tot = measure_layer(lcw)
                st_med, _, _ = stage_times(lcw, N_EVENT_CALLS)
                x_enc = lcw["x_local"][c.n_cls:]
                enc_ms = timed(lambda: B.astra_vq_encode(lcw["vq"], x_enc, lcw["tq"] - c.n_cls, lcw["codebook"], lcw["cnorm"],
                                                         lcw["codes_local"]), 100, warm=20)
                pk = PEAK_TFLOPS[c.dtype]
                entry = {"rank": c.n_dev - 1, "local_rows": lcw["tq"], "nonlocal_rows": lcw["tn"], "dtype": c.dtype, "us_per_call": ms * 1e3,
                         "tokens_per_s": lcw["tq"] / (ms * 1e-3), "flops": tot, "tflops": tot / (ms * 1e-3) / 1e12,
                         "peak_tflops": pk, "frac_of_peak": tot / (ms * 1e-3) / 1e12 / pk,
                         "bound": "mfma" if c.dtype == "bf16" else "alu",
                         "encode_fused_into_projection_launch": bool(B.astra_layer_encode_fused(lcw["desc"])),
                         "stage_us_with_events": {s_: st_med[s_] * 1e3 for s_ in STAGES},
                         "encode_standalone_us": enc_ms * 1e3, "encode_tflops": fl["vq_encode"] / (enc_ms * 1e-3) / 1e12}
                if not args.no_cpu_baseline:
                    sec, n_or, cores = oracle_layer_seconds(lcw, 2.0, 20)
                    entry["cpu_oracle"] = {"s_per_call": sec, "tokens_per_s": lcw["tq"] / sec, "cores": cores, "calls": n_or}
                out_w[name] = entry
                del lcw
            result["workloads"] = {**out_w, "what": "astra_layer_forward of the other named workloads, last simulated device, "
                                   "300 back-to-back calls after 100 warm-up calls; stage_us_with_events are HIP-event spans "
                                   "(each includes one launch gap)"}
        # (1c) the sweep on the ViT-Base shape: G x K x simulated devices (36 points): time per layer call and the encode alone;
        # the oracle timed at the three device counts for G = 16, K = 256
        if "sweep" in extras and args.workload == "llama3_8b_bf16":
            pts = []
            for i_dev in range(len(wl.SWEEP_DEVICES)):
                for i_g in range(len(wl.SWEEP_GROUPS)):
                    for i_k in range(len(wl.SWEEP_CODEBOOK_SIZES)):
                        c = wl.sweep_config(i_g, i_k, i_dev)
                        lcw = make_layer_call(c, c.n_dev - 1)
                        ms, fl, tot = measure_layer(lcw, n=100, warm=30)
                        x_enc = lcw["x_local"]
                        enc_ms = timed(lambda: B.astra_vq_encode(lcw["vq"], x_enc, lcw["tq"], lcw["codebook"], lcw["cnorm"],
                                                                 lcw["codes_local"]), 50, warm=10)
                        need_ws = B.astra_vq_encode_workspace_bytes(lcw["vq"], lcw["tq"])
                        if need_ws > 256:
                            # wide groups: the encode with a workspace (score products + an argmin pass) is the one the layer itself runs
                            ews = torch.empty(need_ws, dtype=torch.uint8, device=dev)
                            enc_ms = timed(lambda: B.astra_vq_encode_ws(lcw["vq"], x_enc, lcw["tq"], lcw["codebook"], lcw["cnorm"],
                                                                        lcw["codes_local"], ews), 50, warm=10)
                            del ews
                        pt = {"G": c.n_groups, "K": c.codebook_size, "n_dev": c.n_dev, "local_rows": lcw["tq"], "us_per_call": ms * 1e3,
                              "tokens_per_s": lcw["tq"] / (ms * 1e-3), "tflops": tot / (ms * 1e-3) / 1e12,
                              "frac_of_peak": tot / (ms * 1e-3) / 1e12 / PEAK_TFLOPS["bf16"],
                              "encode_us": enc_ms * 1e3, "encode_tflops": fl["vq_encode"] / (enc_ms * 1e-3) / 1e12}
                        if c.group_dim % 64 == 0:
                            # K-hat / V-hat from pre-projected codebooks (tables built once, outside the timed calls)
                            pk, pv = preprojected_tables(lcw)
                            a_ = lcw["call_args"]
                            pa = (a_[0], a_[1], a_[2], None, a_[3], a_[4], pk, pv, *a_[5:])
                            pt["us_per_call_preprojected"] = timed(lambda: B.astra_layer_forward_preprojected(*pa), 100, warm=30) * 1e3
                            del pk, pv
                        if not args.no_cpu_baseline and c.n_groups == 16 and c.codebook_size == 256:
                            sec, n_or, cores = oracle_layer_seconds(lcw, 1.0, 10)
                            pt["cpu_oracle"] = {"s_per_call": sec, "tokens_per_s": lcw["tq"] / sec, "cores": cores, "calls": n_or}
                        pts.append(pt)
                        del lcw
            result["sweep"] = {"points": pts, "what": "ViT-Base shape (D 768, 12 heads of 64, N 1024, non-causal, bf16), last simulated "
                               "device; codes of the peers from the library's own encode; 100 back-to-back calls each"}
        # an uneven split of the same sequence (App. "heterogeneous devices": token counts in proportion to device speed,
        # FPAR = the fraction of (query, key) pairs that stay at full precision = sum_i n_i^2 / N^2): every device's call
        if "uneven" in extras and cfg.causal and cfg.n_cls == 0 and cfg.n_dev == 4:
            n_tot = cfg.n_dev * cfg.n_local
            shares = [n_tot // 8, n_tot // 4, n_tot // 4, n_tot - n_tot // 8 - 2 * (n_tot // 4)]       # 1 : 2 : 2 : 3
            xs_all = to_dev(data["x"])
            c_all = torch.empty((n_tot, G), dtype=code_t, device=dev)
            B.astra_vq_encode(vq, xs_all, n_tot, codebook, cnorm, c_all)
            per_dev, lo = [], 0
            for n_i in shares:
                # causal: the rows before the chunk are visible as codes, the rows after it are not needed at all
                d_i = B.LayerDesc(vq, B.attn_desc(dt, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, 0, n_i, lo, True, lo))
                x_i = xs_all[lo:lo + n_i].contiguous()
                cn_i = c_all[:lo].contiguous() if lo > 0 else torch.empty((0, G), dtype=code_t, device=dev)
                y_i = torch.empty((n_i, D), dtype=torch.float32, device=dev)
                cl_i = torch.empty((n_i, G), dtype=code_t, device=dev)
                ws_i = torch.empty(max(B.astra_layer_workspace_bytes(d_i), 256), dtype=torch.uint8, device=dev)
                a_i = (d_i, x_i, cn_i, codebook, cnorm, *w, None, None, None, None, y_i, cl_i, ws_i)
                per_dev.append(timed(lambda: B.astra_layer_forward(*a_i), 100, warm=50))
                lo += n_i
                del x_i, cn_i, y_i, cl_i, ws_i
            result["uneven_split"] = {"tokens_per_device": shares, "fpar": sum(n * n for n in shares) / float(n_tot) ** 2,
                                      "fpar_even_split": 1.0 / cfg.n_dev, "ms_per_device": per_dev,
                                      "slowest_device_ms": max(per_dev),
                                      "what": "astra_layer_forward of every device of a 1:2:2:3 split of the same sequence "
                                              "(under causal masking a device sees the codes of the rows before its chunk)"}
            del xs_all, c_all
        # the layer with 5 % of the peers' tokens lost (Sec. 4.5, packet loss without retransmission): same launches,
        # the attention additionally masks the lost keys of every non-local tile
        if "lost" in extras and tn > 0:
            lost_rng = np.random.default_rng(cfg.seed + 500)
            bits = torch.from_numpy(B.pack_valid_bits(lost_rng.random(tn) >= 0.05).view(np.int64).copy()).to(dev)
            a_v = (desc, x_local, codes_nl, bits, codebook, cnorm, *w, None, None, None, None, y, codes_local, ws)
            result["lost_codes_5pct_ms"] = timed(lambda: B.astra_layer_forward_valid(*a_v), 100, warm=50)
        # the whole Transformer block around the layer (Sec. 3.1: norm, layer, residual, norm, local MLP, residual) for
        # the model this workload stands in for; the peers' codes are reused as they are (their values do not change the work)
        bcfg = next((b for b in wl.BLOCK_CONFIGS.values() if b.layer.name == cfg.name), None)
        if "block" in extras and bcfg is not None:
            bdata = wl.generate_block(bcfg)
            bview = wl.device_view(cfg, bdata, rank)
            f32dev = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dev)
            bt = {"codebook": codebook, "cnorm": cnorm, "wq": w[0], "wk": w[1], "wv": w[2], "wo": w[3],
                  "w1": to_dev(np.ascontiguousarray(bdata["w1"].T)), "w2": to_dev(np.ascontiguousarray(bdata["w2"].T)),
                  "norm1_gain": f32dev(bdata["g1"]), "norm2_gain": f32dev(bdata["g2"])}
            if bcfg.norm_kind == "layernorm":
                bt.update(norm1_bias=f32dev(bdata["be1"]), norm2_bias=f32dev(bdata["be2"]))
            for n in ("bq", "bk", "bv", "bo", "b1", "b2"):
                if bdata.get(n) is not None:
                    bt[n] = to_dev(bdata[n])
            bdesc = B.block_desc(desc, bcfg.norm_kind, bcfg.mlp_kind, bcfg.d_ff, bcfg.eps)
            bw = B.block_weights(**bt)
            bx = f32dev(bview["x_local"])
            bout = torch.empty_like(bx)
            bws = torch.empty(max(B.astra_block_workspace_bytes(bdesc), 256), dtype=torch.uint8, device=dev)
            b_args = (bdesc, bw, bx, codes_nl, None, bout, codes_local, None, bws)
            ms = timed(lambda: B.astra_block_forward(*b_args), 200, warm=100)
            n1 = 2 * bcfg.d_ff if bcfg.mlp_kind == "swiglu" else bcfg.d_ff
            mlp_flops = 2.0 * tq * D * n1 + 2.0 * tq * bcfg.d_ff * D
            result["block"] = {"workload": bcfg.name, "ms": ms, "tokens_per_s": tq / (ms * 1e-3),
                               "flops": total_flops + mlp_flops, "tflops": (total_flops + mlp_flops) / (ms * 1e-3) / 1e12,
                               "mfma_frac": (total_flops + mlp_flops) / (ms * 1e-3) / 1e12 / peak,
                               "mlp_and_norms_ms": ms - ms_per_step, "mlp_tflops": mlp_flops / ((ms - ms_per_step) * 1e-3) / 1e12}
            if cfg.causal:
                # the same block with rotary positions inside the layer (optional, outside the paper): three in-place passes
                rdesc = B.block_desc(desc, bcfg.norm_kind, bcfg.mlp_kind, bcfg.d_ff, bcfg.eps, 500000.0)
                ms_r = timed(lambda: B.astra_block_forward(rdesc, *b_args[1:]), 200, warm=100)
                result["block"]["with_rotary_positions_ms"] = ms_r
            # L such blocks in sequence = this device's share of the whole model's prefill (12 blocks for the ViT-Base and
            # GPT-2 shapes, 32 for Llama-3-8B): distinct random weights and codes per block, generated on the device
            if "stack" in extras:
                n_layers = 32 if "llama" in cfg.name else 12
                gen = torch.Generator(device=dev).manual_seed(cfg.seed + 77)
                tdt = torch.bfloat16 if dt == "bf16" else torch.float32
                rnd = lambda *shape: (0.02 * torch.randn(*shape, generator=gen, device=dev, dtype=torch.float32)).to(tdt)
                dq, dkv = cfg.n_q_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim
                keep, w_list, codes_in, codes_out = [], [], [], []
                for l in range(n_layers):
                    lt = dict(bt)
                    lt.update(wq=rnd(dq, D), wk=rnd(dkv, D), wv=rnd(dkv, D), wo=rnd(D, dq), w1=rnd(n1, D), w2=rnd(D, bcfg.d_ff))
                    keep.append(lt)
                    w_list.append(B.block_weights(**lt))
                    codes_in.append(torch.randint(0, K, (tn, G), generator=gen, device=dev, dtype=torch.int32).to(code_t))
                    codes_out.append(torch.empty_like(codes_local))
                s_args = (bdesc, w_list, bx, codes_in, None, bout, codes_out, bws)
                ms_stack = timed(lambda: B.astra_stack_forward(*s_args), 10, warm=3)
                result["stack"] = {"workload": bcfg.name, "n_layers": n_layers, "ms": ms_stack, "ms_per_block": ms_stack / n_layers,
                                   "tokens_per_s": tq / (ms_stack * 1e-3),
                                   "tflops": n_layers * (total_flops + mlp_flops) / (ms_stack * 1e-3) / 1e12,
                                   "what": "astra_stack_forward: this device's share of one prefill pass through all blocks "
                                           "(the exchange of codes between blocks is not timed: they are resident inputs)"}
                del keep, w_list, codes_in, codes_out
            del bt, bw, bx, bout, bws, bdata
        # the variant that quantises K and V after projection (App. memory cost: C = 2 codebooks of dimension H_kv * dh; the
        # paper's Llama configuration): local projections only, two encodes, the peers' K-hat / V-hat looked up from codes
        if "kv" in extras and tn > 0:
            kdata = wl.generate_kv(cfg)
            gk = kdata["codebook_k"].shape[0]
            dkv = cfg.n_kv_heads * cfg.head_dim
            vqk = B.vq_desc(dt, dkv, gk, K)
            cbk, cbv = to_dev(kdata["codebook_k"]), to_dev(kdata["codebook_v"])
            cnk = torch.empty((gk, K), dtype=torch.float32, device=dev)
            cnv = torch.empty_like(cnk)
            B.astra_vq_prepare(vqk, cbk, cnk)
            B.astra_vq_prepare(vqk, cbv, cnv)
            kgen = torch.Generator(device=dev).manual_seed(cfg.seed + 78)
            ck_nl = torch.randint(0, K, (tn, gk), generator=kgen, device=dev, dtype=torch.int32).to(code_t)
            cv_nl = torch.randint(0, K, (tn, gk), generator=kgen, device=dev, dtype=torch.int32).to(code_t)
            kdesc = B.LayerKvDesc(vqk, desc.attn, D)
            ck_l = torch.empty((tq - cfg.n_cls, gk), dtype=code_t, device=dev)
            cv_l = torch.empty_like(ck_l)
            kws = torch.empty(max(B.astra_layer_kv_workspace_bytes(kdesc), 256), dtype=torch.uint8, device=dev)
            k_args = (kdesc, x_local, ck_nl, cv_nl, None, cbk, cnk, cbv, cnv, *w, None, None, None, None, y, ck_l, cv_l, None, None, kws)
            ms = timed(lambda: B.astra_layer_forward_kv(*k_args), 300, warm=100)
            kv_flops = (2.0 * tq * D * (cfg.n_q_heads * cfg.head_dim + 2 * dkv) + 2 * 2.0 * (tq - cfg.n_cls) * dkv * K
                        + flops["attention"] + flops["out_projection"])
            result["kv_variant"] = {"G_kv": gk, "bits_per_token_per_block": 2 * gk * int(np.ceil(np.log2(K))), "ms": ms,
                                    "tokens_per_s": tq / (ms * 1e-3), "flops": kv_flops, "tflops": kv_flops / (ms * 1e-3) / 1e12,
                                    "vs_embedding_space_layer": ms / ms_per_step,
                                    "what": "astra_layer_forward_kv at the same shape: no projection of rebuilt rows"}
            del cbk, cbv, ck_nl, cv_nl, kws
        # one decoding step over an index KV cache (App. memory cost; Sec. 3.1 hand-off to single-device decoding), per layer:
        # the cache a prefill of this workload leaves on the last device, and a 32 times longer one
        if "kvcache" in extras and tn > 0:
            kdata = wl.generate_kv(cfg)
            gk = kdata["codebook_k"].shape[0]
            dkv = cfg.n_kv_heads * cfg.head_dim
            vqk = B.vq_desc(dt, dkv, gk, K)
            cbk, cbv = to_dev(kdata["codebook_k"]), to_dev(kdata["codebook_v"])
            dgen = torch.Generator(device=dev).manual_seed(cfg.seed + 79)
            tdt = torch.bfloat16 if dt == "bf16" else torch.float32
            eb = 2 if dt == "bf16" else 4
            steps_out = []
            for mult in (1, 32):
                nl_rows, loc_rows = tn * mult, (tq - cfg.n_cls) * mult + 1
                kc = torch.randn((loc_rows, cfg.n_kv_heads, cfg.head_dim), generator=dgen, device=dev, dtype=torch.float32).to(tdt)
                vc = torch.randn((loc_rows, cfg.n_kv_heads, cfg.head_dim), generator=dgen, device=dev, dtype=torch.float32).to(tdt)
                qd = torch.randn((cfg.n_q_heads, cfg.head_dim), generator=dgen, device=dev, dtype=torch.float32).to(tdt)
                ckd = torch.randint(0, K, (nl_rows, gk), generator=dgen, device=dev, dtype=torch.int32).to(code_t)
                cvd = torch.randint(0, K, (nl_rows, gk), generator=dgen, device=dev, dtype=torch.int32).to(code_t)
                ddesc = B.DecodeDesc(vqk, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, loc_rows, nl_rows, 0.0)
                od = torch.empty((cfg.n_q_heads, cfg.head_dim), dtype=tdt, device=dev)
                dws = torch.empty(max(B.astra_decode_attention_workspace_bytes(ddesc), 256), dtype=torch.uint8, device=dev)
                d_args = (ddesc, qd, kc, vc, ckd, cvd, None, cbk, cbv, od, None, dws)
                ms = timed(lambda: B.astra_decode_attention(*d_args), 300, warm=50)
                cache_bytes = 2 * loc_rows * dkv * eb + 2 * nl_rows * gk * ckd.element_size()
                nbytes = cache_bytes + 2 * gk * K * (dkv // gk) * eb + 2 * cfg.n_q_heads * cfg.head_dim * eb
                steps_out.append({"cached_tokens": loc_rows + nl_rows, "local_rows": loc_rows, "index_rows": nl_rows, "us": ms * 1e3,
                                  "algorithmic_bytes": nbytes, "GBps": nbytes / (ms * 1e-3) / 1e9,
                                  "frac_of_hbm_8TBps": nbytes / (ms * 1e-3) / 8e12,
                                  "cache_bytes_per_layer": cache_bytes,
                                  "cache_vs_full_precision": cache_bytes / (2.0 * (loc_rows + nl_rows) * dkv * eb)})
                del kc, vc, ckd, cvd, dws
            result["decode_step_index_kv_cache"] = {"G_kv": gk, "steps": steps_out,
                                                    "what": "astra_decode_attention: one query over full-precision local K/V plus code streams; "
                                                            "bytes = cache + both codebooks + q + out"}
        # one codebook-learning step on a training-sized batch (Sec. 3.2: K-means initialisation / EMA updates with the
        # commitment sum of Eq. 2): encode, per-codeword statistics, update; 16384 tokens of this workload's width
        if "train" in extras:
            tt = 16384
            tgen = torch.Generator(device=dev).manual_seed(cfg.seed + 80)
            tdt = torch.bfloat16 if dt == "bf16" else torch.float32
            eb = 2 if dt == "bf16" else 4
            xt = torch.randn((tt, D), generator=tgen, device=dev, dtype=torch.float32).to(tdt)
            ct = torch.empty((tt, G), dtype=code_t, device=dev)
            cnt = torch.empty((G, K), dtype=torch.int32, device=dev)
            sm = torch.empty((G, K, cfg.group_dim), dtype=torch.float32, device=dev)
            sq = torch.empty(G, dtype=torch.float32, device=dev)
            en, em = torch.ones((G, K), dtype=torch.float32, device=dev), torch.zeros((G, K, cfg.group_dim), dtype=torch.float32, device=dev)
            cb2 = torch.empty_like(codebook)
            tws = torch.empty(max(B.astra_codebook_stats_workspace_bytes(vq, tt), 256), dtype=torch.uint8, device=dev)
            ms_e = timed(lambda: B.astra_vq_encode(vq, xt, tt, codebook, cnorm, ct), 30, warm=5)
            ms_s = timed(lambda: B.astra_codebook_stats(vq, xt, ct, tt, codebook, cnt, sm, sq, tws), 30, warm=5)
            ms_u = timed(lambda: B.astra_codebook_update(vq, cnt, sm, 0.99, en, em, codebook, cb2), 30, warm=5)
            stat_bytes = tt * D * eb + 2 * tt * G * ct.element_size() + G * K * cfg.group_dim * (eb + 4) + G * K * 4
            result["codebook_learning_step"] = {
                "tokens": tt, "encode_us": ms_e * 1e3, "encode_tflops": 2.0 * tt * K * D / (ms_e * 1e-3) / 1e12,
                "stats_us": ms_s * 1e3, "stats_algorithmic_bytes": stat_bytes, "stats_GBps": stat_bytes / (ms_s * 1e-3) / 1e9,
                "stats_frac_of_hbm_8TBps": stat_bytes / (ms_s * 1e-3) / 8e12, "update_us": ms_u * 1e3,
                "what": "astra_vq_encode + astra_codebook_stats (deterministic: counting sort by code, rows added in a fixed order) + "
                        "astra_codebook_update (EMA)"}
            del xt, ct, sm, em, cb2, tws
        # (2) the decode as a kernel of its own (inside the layer it is fused into the projection's operand load):
        #     the HBM-bound step; algorithmic bytes = codes + codebook + rebuilt rows
        t_v = view["n_before"] if cfg.causal else tn
        if "decode" in extras and t_v > 0:
            x_hat = torch.empty((t_v, D), dtype=x_local.dtype, device=dev)
            ms = timed(lambda: B.astra_vq_decode(vq, codes_nl, t_v, codebook, x_hat), 200, warm=50)
            eb = 2 if dt == "bf16" else 4
            nbytes = t_v * G * codes_nl.element_size() + G * K * cfg.group_dim * eb + t_v * D * eb
            result["decode_standalone"] = {"us": ms * 1e3, "algorithmic_bytes": nbytes, "GBps": nbytes / (ms * 1e-3) / 1e9,
                                           "frac_of_hbm_8TBps": nbytes / (ms * 1e-3) / 8e12, "rows": t_v}
            del x_hat
        # (2b) the same decode over buffers that rotate through more than the 256 MB last-level cache: every call reads its own copy
        #      of the codes and of the codebook and writes its own output, so that the rate is an HBM rate
        if "gather" in extras and t_v > 0:
            eb = 2 if dt == "bf16" else 4
            per_call = t_v * G * codes_nl.element_size() + G * K * cfg.group_dim * eb + t_v * D * eb
            n_sets = max(4, int(np.ceil(768e6 / per_call)))
            sets = [(codes_nl[:t_v].clone(), codebook.clone(), torch.empty((t_v, D), dtype=x_local.dtype, device=dev)) for _ in range(n_sets)]
            state = {"i": 0}

            def rot():
                c_, cb_, o_ = sets[state["i"] % n_sets]
                state["i"] += 1
                B.astra_vq_decode(vq, c_, t_v, cb_, o_)
            ms = timed(rot, 10 * n_sets, warm=2 * n_sets)
            gather = {"us": ms * 1e3, "algorithmic_bytes": per_call, "GBps": per_call / (ms * 1e-3) / 1e9,
                      "frac_of_hbm_8TBps": per_call / (ms * 1e-3) / 8e12, "rows": t_v, "buffer_sets": n_sets,
                      "rotating_bytes": n_sets * per_call,
                      "what": "astra_vq_decode, each call on its own copy of codes, codebook and output (the working set exceeds the "
                              "256 MB last-level cache)"}
            if is_bench_shape:
                tr = traffic_from_profiles("vq_decode_llama3_8b", "vq_decode_kernel")
                gather["traffic_bytes_from_counters"] = tr
                # the kernel's average duration in the kernel trace kept under profiles/, and the HBM rate that goes with the counters
                us_prof = None
                try:
                    for ln in open(os.path.join(ROOT, "profiles", "vq_decode_llama3_8b_kernel_trace.txt")):
                        f_ = ln.split()
                        if len(f_) >= 6 and "vq_decode_kernel" in ln and f_[0].isdigit():
                            us_prof = float(f_[1])
                            break
                except OSError:
                    pass
                gather["kernel_us_in_profile"] = us_prof
                if tr and us_prof:
                    gather["hbm_GBps_from_counters"] = tr / (us_prof * 1e-6) / 1e9
                    gather["hbm_frac_from_counters"] = tr / (us_prof * 1e-6) / 8e12
            del sets
            result["decode_rotating_buffers"] = gather
        if "gather_x8" in extras and t_v > 0:
            eb = 2 if dt == "bf16" else 4
            gather = result.setdefault("decode_rotating_buffers", {})
            # the same kernel on 8 times the rows (one call moves more than the last-level cache holds): its streaming rate
            # without the fixed cost of a launch that a 10-microsecond kernel is dominated by
            t_big = 8 * t_v
            codes_big = codes_nl[:t_v].repeat(8, 1).contiguous()
            out_big = torch.empty((t_big, D), dtype=x_local.dtype, device=dev)
            ms_big = timed(lambda: B.astra_vq_decode(vq, codes_big, t_big, codebook, out_big), 20, warm=5)
            big_bytes = t_big * G * codes_nl.element_size() + G * K * cfg.group_dim * eb + t_big * D * eb
            gather["rows_x8"] = {"rows": t_big, "us": ms_big * 1e3, "algorithmic_bytes": big_bytes, "GBps": big_bytes / (ms_big * 1e-3) / 1e9,
                                 "frac_of_hbm_8TBps": big_bytes / (ms_big * 1e-3) / 8e12}
            del codes_big, out_big
        # a yardstick, not part of the product: the vendor GEMM (torch.matmul -> hipBLASLt / rocBLAS) on the layer's plain
        # products.  It cannot take codes as its row operand, so the K-hat / V-hat product is given rebuilt rows.
        if "vendor" in extras and dt == "bf16":
            vg = {}
            tv = view["n_before"] if cfg.causal else tn
            dq_, dkv_ = cfg.n_q_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim
            for name, (m_, n_, k_) in {"q_k_v_of_local_rows": (tq, dq_ + 2 * dkv_, D), "k_v_of_rebuilt_rows": (tv, 2 * dkv_, D),
                                       "output_projection": (tq, D, dq_)}.items():
                if m_ == 0:
                    continue
                a_ = torch.randn((m_, k_), device=dev, dtype=torch.float32).to(torch.bfloat16)
                b_ = torch.randn((n_, k_), device=dev, dtype=torch.float32).to(torch.bfloat16)
                ms = timed(lambda: torch.matmul(a_, b_.t()), 50, warm=10)
                vg[name] = {"m_n_k": [m_, n_, k_], "us": ms * 1e3, "tflops": 2.0 * m_ * n_ * k_ / (ms * 1e-3) / 1e12}
                del a_, b_
            result["vendor_gemm_yardstick"] = {**vg, "what": "torch.matmul in bf16 on the same shapes, for context: the layer's projection "
                                               "launch does the first two products (from codes, with the encode alongside) in one launch"}
        # (3) last, because it heats the chip: what the matrix cores of this machine deliver with nothing else in the loop, next to the published peak
        if "probe" in extras and dt == "bf16":
            n_blocks, iters = 1024, 2000
            probe_out = torch.empty(n_blocks * 512, dtype=torch.float32, device=dev)
            ms = timed(lambda: B.astra_probe_mfma_bf16(probe_out, n_blocks, iters), 5, warm=3)
            tf = n_blocks * 8 * iters * 4 * 32768.0 / (ms * 1e-3) / 1e12
            result["mfma_probe"] = {"tflops": tf, "frac_of_published_peak": tf / peak,
                                    "dominant_kernel_frac_of_probe": achieved / tf,
                                    "what": "astra_probe_mfma_bf16: 32x32x16 bf16 MFMAs on register operands only"}
            del probe_out

    if not args.no_cpu_baseline:
        import oracle
        codes_nl_host = codes_nl.cpu().numpy()
        if K > 256:
            codes_nl_host = codes_nl_host.view(np.uint16)
        oracle.num_threads()            # load outside the timed part
        # whole layer calls of the same workload and rank, repeated until about 10 s of CPU work have been timed
        # (at most 8 calls); the oracle is the checker as it stands, never tuned for this
        n_calls, c0 = 0, time.perf_counter()
        while n_calls < 8 and (n_calls == 0 or time.perf_counter() - c0 < 10.0):
            oracle.layer_forward(view["x_local"], codes_nl_host.astype(np.int32), data["codebook"], data["wq"], data["wk"],
                                 data["wv"], data["wo"], n_q_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads, n_cls=cfg.n_cls,
                                 causal=cfg.causal, n_before=view["n_before"])
            n_calls += 1
        c1 = time.perf_counter()
        result["cpu_baseline"] = {"value": n_calls * tq / (c1 - c0), "unit": "tokens/s", "cores": oracle.num_threads(),
                                  "kind": "oracle", "sample": f"{n_calls} whole layer calls of the same workload ({tq} local rows each), "
                                  f"{c1 - c0:.2f} s, fp64 C/OpenMP oracle"}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
