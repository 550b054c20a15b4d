#!/usr/bin/env python3
"""Benchmark of the quantized vector-sparse hot path on one MI355X.

The headline figure (`value`) is the metric's own kernel: the L8-R8 SpMM at 4096 x 4096, V = 8, 90 % of the
vectors zero, N = 256, in effective TOPS = 2 * nnz * N / time, timed with events on the launch stream over
back-to-back launches.  `roofline` describes that kernel.

A *step* is one pass of every kernel row of the path at that shape: SpMM L8-R8 / L8-R4 / L4-R4 / L16-R8 with
N = 256, SDDMM L8-R8 / L4-R4 with K = 256, and the quantized sparse-attention layer (8 heads, L = 4096, d_k = 64,
Q/K/V as a QKV projection writes them, (L, heads, d_k): SDDMM -> softmax -> int8 -> SpMM).  --steps / --warmup count
such steps; their time is `ms_per_step`, their aggregate rate `step.aggregate_tops`, and `roofline_step_dominant`
describes the kernel that takes the largest share of it.  The step is replayed as one HIP graph so that host
launch latency is not what is measured (`--eager` launches the kernels one by one instead).

Inputs are seeded synthetic data already resident in HBM; the sparse operands were converted to the device format
beforehand (the paper builds its format offline as well).

Other modes, each printing ONE JSON object: --sweep (the SpMM / SDDMM grids, for the SpMM with the gather form,
the LDS-resident form and the automatic choice side by side), --skew (panels of log-normal length), --shapes
(matrices with few panels: the automatic kernel variant against every pinned one).

`cpu_baseline` is the CPU oracle timed on this host.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X HBM3E, published
I8_MFMA_PEAK_TOPS = 5000.0  # MI355X dense int8, published
COUNTER_PROFILE = os.path.join(ROOT, "profiles", "bench_step_counters.txt")


def measured_traffic(library_version: str):
    """HBM-side bytes per launch of the step's kernels, from the stored counter summary (FETCH_SIZE + WRITE_SIZE of
    two rocprofv3 --pmc runs of this benchmark, each scaled by what the same counter reads for a plain 64 MiB copy).
    Counters cannot be read from inside the benchmark, so the figures are only as fresh as that file: when it names
    another build of the library than the one running, nothing is returned."""
    try:
        with open(COUNTER_PROFILE) as f:
            text = f.read()
    except OSError:
        return {}, "no counter summary stored"
    m = re.search(r"^library:\s*(.+?)\s*$", text, re.M)
    if not m or m.group(1) != library_version:
        return {}, f"counter summary is of build '{m.group(1) if m else '?'}', running '{library_version}'"
    out = {}
    for m in re.finditer(r"^traffic\s+(\S+)\s+fetch_bytes=(\d+)\s+write_bytes=(\d+)", text, re.M):
        if m.group(1) != "-":
            out[m.group(1)] = out.get(m.group(1), 0) + int(m.group(2)) + int(m.group(3))
    return out, "profiles/bench_step_counters.txt"


M = K = 4096
V = 8
SPARSITY = 0.9
N_SPMM = 256
KD_SDDMM = 256
HEADS, L_ATT, DK = 8, 4096, 64


def build_problem():
    """Seeded inputs of one step, on the host."""
    from paper_2209_06979_amd import workloads as wl
    prob = {}
    for i, prec in enumerate(["L8R8", "L8R4", "L4R4", "L16R8"]):
        prob["spmm_" + prec] = wl.spmm_case(M, K, N_SPMM, V, SPARSITY, prec, wl.seed_for(2, 10 * i))
    for i, prec in enumerate(["L8R8", "L4R4"]):
        prob["sddmm_" + prec] = wl.sddmm_case(M, K, KD_SDDMM, V, SPARSITY, prec, wl.seed_for(3, 10 * i))
    att = wl.attention_case(HEADS, L_ATT, DK, V, SPARSITY, wl.seed_for(5))
    att["s_p"] = np.float32(1.0 / 127.0)
    prob["attention"] = att
    return prob


def quantize_on_gpu(mc, torch, x, bits=8):
    """The layer's input quantisation done by the library itself (mc_absmax + mc_quantize): fp32 host
    array -> (integer codes as a host array, packed two per byte for bits=4; fp32 scale)."""
    xd = torch.from_numpy(np.ascontiguousarray(x)).cuda()
    amax = float(mc.absmax(xd).cpu()[0])
    s = np.float32(np.float64(amax) / (127.0 if bits == 8 else 7.0))
    return mc.quantize(xd, float(s), bits).cpu().numpy(), s


def spmm_alg_bytes(nvec, P, lbits, rbits, N):
    return nvec * V * lbits // 8 + 4 * nvec + 8 * P + K * N * rbits // 8 + 4 * M * N


def sddmm_alg_bytes(nvec, P, bits, Kd):
    return 2 * M * Kd * bits // 8 + 4 * nvec + 8 * P + 4 * nvec * V


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--eager", action="store_true", help="launch kernel by kernel instead of replaying a HIP graph")
    ap.add_argument("--steps-per-graph", type=int, default=10,
                    help="steps captured in one HIP graph (the graph is replayed steps/this many times)")
    ap.add_argument("--reps", type=int, default=200, help="back-to-back launches for the per-kernel timings")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--only", default="", help="comma-separated kernel names: run only these in the step")
    ap.add_argument("--attention-layout", choices=["token", "head"], default="token",
                    help="Q/K/V buffers token-major (L, heads, dk) as a projection writes them, or head-major (heads, L, dk)")
    ap.add_argument("--attention-mode", type=int, default=0,
                    help="0: automatic (the fused kernel); 1: scores+softmax kernel, then the SpMM; 6: separate SDDMM / "
                         "softmax / SpMM kernels (for profiling them)")
    ap.add_argument("--no-per-kernel", action="store_true", help="skip the per-kernel timing runs (counter collection)")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the measurements beside the step: cold-cache and gather-only timings of the headline "
                         "SpMM and the wider precisions that are not part of the step")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the step: time every point of the SpMM grid (V x sparsity x N x precision, 162 points, "
                         "plus L16-R8; gather form, LDS-resident form and the automatic choice) and of the SDDMM grid "
                         "(Kd x sparsity x precision) at 4096 x 4096 and print one JSON object with the table")
    ap.add_argument("--skew", action="store_true",
                    help="instead of the step: SpMM and SDDMM on 4096 x 4096 patterns whose panel lengths are log-normal "
                         "(sigma 0 / 0.5 / 1 / 1.5, same mean as the headline), with and without work items")
    ap.add_argument("--shapes", action="store_true",
                    help="instead of the step: matrices with few panels or short panels; the automatic kernel variant "
                         "against every pinned tile / wave variant")
    ap.add_argument("--table", action="store_true",
                    help="with --sweep / --skew / --shapes: print a plain-text table instead of the JSON object")
    ap.add_argument("--point", default="",
                    help="instead of the step: one SpMM configuration 'prec:V:sparsity:N:form' (form: gather, lds, merged, merged-lds or auto) at "
                         "4096 x 4096, launched --steps times one by one (for counter and trace collection), e.g. L8R8:2:0.5:512:lds")
    ap.add_argument("--phases", action="store_true",
                    help="instead of the step: the headline L8-R8 SpMM run through the instrumented copy of its kernel "
                         "(mc_probe_spmm_phases); prints when its waves reach each stage of the kernel")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one plain 64 MiB device copy, the known-size kernel that scales FETCH_SIZE / WRITE_SIZE")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2209_06979_amd import binding as mc
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.sweep or args.skew or args.shapes or args.phases:
        result = (run_sweep(mc, torch) if args.sweep else run_skew(mc, torch) if args.skew else
                  run_shapes(mc, torch) if args.shapes else run_phases(mc, torch))
        print(as_table(result) if args.table else json.dumps(result))
        return
    if args.point:
        print(json.dumps(run_point(mc, torch, args.point, args.steps, args.warmup, args.calib_copy)))
        return

    prob = build_problem()
    for n in ("q", "k", "v"):
        prob["attention"][n + "8"], prob["attention"]["s_" + n] = quantize_on_gpu(mc, torch, prob["attention"][n])
    t0 = time.perf_counter()
    kernels = []  # name, launch(), ops, algorithmic bytes, device kernel name

    def up(a):
        return torch.from_numpy(np.ascontiguousarray(a)).to(dev)

    keep = []
    for prec in ["L8R8", "L8R4", "L4R4", "L16R8"]:
        c = prob["spmm_" + prec]
        A = mc.SparseMatrix(M, K, V, c["row_ptr"], c["col_idx"], c["values"], mc.LHS_BITS[prec])
        B = up(c["B"])
        C = torch.empty((M, N_SPMM), dtype=torch.int32, device=dev)
        keep += [A, B, C]
        nvec = A.nvec
        kernels.append(dict(
            name="spmm_" + prec, launch=(lambda A=A, B=B, C=C, prec=prec: mc.spmm(A, B, prec, out=C)),
            ops=2 * nvec * V * N_SPMM,
            bytes=spmm_alg_bytes(nvec, M // V, mc.LHS_BITS[prec], mc.RHS_BITS[prec], N_SPMM)))
    for prec in ["L8R8", "L4R4"]:
        c = prob["sddmm_" + prec]
        mask = mc.SparseMatrix(M, K, V, c["row_ptr"], c["col_idx"])
        Q, Km = up(c["Q"]), up(c["Kmat"])
        S = torch.empty(mask.nvec * V, dtype=torch.int32, device=dev)
        keep += [mask, Q, Km, S]
        kernels.append(dict(
            name="sddmm_" + prec, launch=(lambda Q=Q, Km=Km, mask=mask, S=S, prec=prec: mc.sddmm(Q, Km, mask, prec, out=S)),
            ops=2 * mask.nvec * V * KD_SDDMM,
            bytes=sddmm_alg_bytes(mask.nvec, M // V, mc.LHS_BITS[prec], KD_SDDMM)))
    att = prob["attention"]
    amask = mc.SparseMatrix(L_ATT, L_ATT, V, att["row_ptr"], att["col_idx"])
    # --attention-layout token: buffer (L, heads, dk) as a QKV projection writes it, viewed (heads, L, dk)
    def token_major(a):
        if args.attention_layout == "head":
            return up(a)
        return up(np.ascontiguousarray(np.transpose(a, (1, 0, 2)))).permute(1, 0, 2)
    q8, k8, v8 = token_major(att["q8"]), token_major(att["k8"]), token_major(att["v8"])
    if args.attention_layout == "head":
        O = torch.empty((HEADS, L_ATT, DK), dtype=torch.float32, device=dev)
    else:
        O = torch.empty((L_ATT, HEADS, DK), dtype=torch.float32, device=dev).permute(1, 0, 2)
    ws = torch.empty(mc.attention_workspace_bytes(HEADS, amask), dtype=torch.uint8, device=dev)
    keep += [amask, q8, k8, v8, O, ws]
    nnz_att = amask.nvec * V
    # compulsory traffic of the layer: Q, K, V in, O out, the mask pattern once.  (Scores and
    # codes never reach HBM in the fused kernel, so they are not algorithmic bytes.)
    att_bytes = HEADS * (3 * L_ATT * DK + 4 * L_ATT * DK) + 4 * amask.nvec + 8 * (L_ATT // V)
    kernels.append(dict(
        name="attention", launch=(lambda: mc.sparse_attention(q8, k8, v8, amask, att["s_q"], att["s_k"], att["s_v"],
                                                              att["s_p"], out=O, workspace=ws)),
        ops=HEADS * 2 * (2 * nnz_att * DK), bytes=att_bytes))
    torch.cuda.synchronize()
    format_build_s = time.perf_counter() - t0

    mc.set_attention_mode(args.attention_mode)   # (this thread's default; the step's calls pass no options)
    if args.only:
        names = set(args.only.split(","))
        kernels = [k for k in kernels if k["name"] in names]

    def step():
        for k in kernels:
            k["launch"]()

    stream = torch.cuda.Stream()
    graph = None
    with torch.cuda.stream(stream):
        step()                       # first touch outside capture
        stream.synchronize()
        spg = 1
        if not args.eager:
            # several steps per graph: one graph launch costs the host and the command
            # processor ~15 us, which is not what is being measured
            spg = max(1, min(args.steps_per_graph, args.steps))
            while args.steps % spg:
                spg -= 1
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                for _ in range(spg):
                    step()
        run = graph.replay if graph is not None else step
        for _ in range((args.warmup + spg - 1) // spg):
            run()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps // spg):
            run()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0

        if args.calib_copy:
            src = torch.empty(64 * 1024 * 1024, dtype=torch.uint8, device=dev)
            dst = torch.empty_like(src)
            dst.copy_(src)
            stream.synchronize()
        # per-kernel timings: back-to-back launches between two events on the launch stream
        for k in ([] if args.no_per_kernel else kernels):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=stream):
                for _ in range(args.reps):
                    k["launch"]()
            g.replay()
            stream.synchronize()
            samples = []
            for _ in range(5):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                g.replay()
                e1.record(stream)
                e1.synchronize()
                samples.append(e0.elapsed_time(e1) * 1e3 / args.reps)   # microseconds per launch
            k["us"] = float(np.median(samples))
            del g
        extras = None if (args.no_extras or args.only or args.attention_mode) else measure_extras(mc, torch, prob, stream, args.reps, up)
    ms_per_step = elapsed / args.steps * 1e3
    total_ops = sum(k["ops"] for k in kernels)
    aggregate = total_ops / (elapsed / args.steps) / 1e12

    version = mc.lib.mc_version().decode()
    traffic, traffic_source = measured_traffic(version)
    if args.attention_layout != "token" or args.attention_mode:
        traffic.pop("attention", None)
    for k in kernels:
        k.setdefault("us", float("nan"))

    def hbm_roofline(k):
        achieved = k["bytes"] / (k["us"] * 1e-6) / 1e9
        return dict(bound="hbm", kernel=k["name"], achieved=round(achieved, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=round(achieved / HBM_PEAK_GBS, 4), traffic=traffic.get(k["name"]), traffic_source=traffic_source,
                    us_per_launch=round(k["us"], 2), algorithmic_bytes=int(k["bytes"]))

    timed = [k for k in kernels if k["us"] == k["us"]]
    head = next((k for k in timed if k["name"] == "spmm_L8R8"), None)
    roofline = roofline_dom = None
    value = None
    if head is not None:
        value = head["ops"] / head["us"] / 1e6
        roofline = hbm_roofline(head)
        if extras is not None:
            # beside the HBM bound: warm, B lives in L2 and the kernel is bound by moving the gathered rows from
            # L2 into LDS; cold, every operand comes from HBM
            h = extras["headline"]
            roofline.update(cold_us=h["cold_us"], cold_frac=h["cold_hbm_frac"], gathered_bytes=h["gathered_bytes"],
                            gather_peak_tbs_measured=extras["gather_peak_tbs"]["rows_128B"],
                            frac_of_gather_peak=h["frac_of_gather_peak"],
                            i8_mfma_frac_of_published=round(value / I8_MFMA_PEAK_TOPS, 4),
                            i8_mfma_frac_of_measured=round(value / extras["mfma_i8_peak"]["measured_tops"], 4))
    if timed:
        dom = max(timed, key=lambda k: k["us"])
        roofline_dom = hbm_roofline(dom)
        roofline_dom["share_of_step"] = round(dom["us"] / sum(k["us"] for k in timed), 3)
        if extras is not None and dom["name"] == "attention":
            # the practical bound of that kernel: its K and V rows (64 bytes each, padded slots included) at the
            # gather rate measured above (token-major: the rows of two neighbouring heads are fetched as one
            # 128-byte piece)
            gb = HEADS * 2 * amask.nslots * DK
            pk = extras["gather_peak_tbs"]["rows_128B" if args.attention_layout == "token" else "rows_64B"]
            roofline_dom["gathered_bytes"] = int(gb)
            roofline_dom["gather_peak_tbs_measured"] = pk
            roofline_dom["frac_of_gather_peak"] = round(gb / pk / 1e6 / dom["us"], 3)
    per_kernel = {k["name"]: dict(us=round(k["us"], 2), eff_tops=round(k["ops"] / k["us"] / 1e6, 1),
                                  alg_gbs=round(k["bytes"] / k["us"] / 1e3, 1),
                                  hbm_frac=round(k["bytes"] / k["us"] / 1e3 / HBM_PEAK_GBS, 4),
                                  i8_mfma_frac=round(k["ops"] / k["us"] / 1e6 / I8_MFMA_PEAK_TOPS, 4),
                                  traffic=traffic.get(k["name"]))
                  for k in timed}

    cpu = None
    if not args.no_cpu:
        cpu = cpu_baseline(prob)

    out = {
        "metric": "SpMM/SDDMM effective TOPS (2\u00b7nnz\u00b7N/s), 90% sparse, V=8, L8-R8; % roofline",
        "value": (round(value, 2) if value is not None else None), "unit": "TOPS", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": "SpMM L8-R8, A 4096x4096 V=8 s=0.9 (209,920 vectors), B 4096x256 int8, C int32",
                   "value_is": "2*nnz*N / time of that kernel, events on the launch stream around "
                               f"{args.reps} back-to-back launches, median of 5",
                   "step": "4096x4096 V=8 s=0.9: SpMM L8-R8/L8-R4/L4-R4/L16-R8 N=256 + SDDMM L8-R8/L4-R4 K=256 "
                           "+ sparse attention 8 heads L=4096 dk=64 (ms_per_step is one such step)",
                   "launch": "eager" if args.eager else f"hip_graph x{spg} steps", "kernels_in_step": [k["name"] for k in kernels],
                   "library": version,
                   **({"attention_mode": args.attention_mode} if args.attention_mode else {})},
        "step": {"ms": round(ms_per_step, 4), "aggregate_tops": round(aggregate, 2), "ops": int(total_ops)},
        "sddmm_l8r8_tops": (per_kernel.get("sddmm_L8R8") or {}).get("eff_tops"),
        "headline_spmm_l8r8": dict(per_kernel.get("spmm_L8R8") or {}, **((extras or {}).get("headline") or {})),
        "headline_at_16x_rows": (extras or {}).get("headline_at_16x_rows"),
        "mfma_i8_peak": (extras or {}).get("mfma_i8_peak"),
        "launch_floor_us": (extras or {}).get("launch_floor_us"),
        "cold_cache_us": (extras or {}).get("cold_us"),
        "gather_peak_tbs_measured": (extras or {}).get("gather_peak_tbs"),
        "beyond_the_step": (extras or {}).get("wider_precisions"),
        "layer_at_inference_shapes": (extras or {}).get("layer_at_inference_shapes"),
        "spmm_design_steps": (extras or {}).get("spmm_design_steps"),
        "quantisation_streaming": (extras or {}).get("quantisation_streaming"),
        "per_kernel": per_kernel,
        "format_build_s": round(format_build_s, 3),
        "roofline": roofline,
        "roofline_step_dominant": roofline_dom,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


def run_sweep(mc, torch):
    """The grids of the SpMM and SDDMM precision sweeps (Section 5.2 figures' shapes: vector lengths, sparsities,
    widths of the dense operand, precisions) on seeded synthetic 4096 x 4096 patterns, warm caches.  Every SpMM point
    is timed on the operand as given -- rows of B gathered per stored vector (`gather_us`), K-blocks of B resident in
    LDS (`lds_us`, null where that form does not exist: two-plane right operands, more than 63 K-blocks) -- on its
    merged copy (`merged_gather_us`, `merged_lds_us`: consecutive panels sharing one panel of 16 or 8 rows; null
    where there is nothing to merge) and as the library picks by itself (`us`, `form`, `merged`);
    `auto_over_best` = us / the fastest of the pinned forms."""
    from paper_2209_06979_amd import workloads as wl
    stream = torch.cuda.Stream()
    spmm, sddmm = [], []
    gather_only, lds_forced = mc.Options(spmm_slab=-1, spmm_merge=-1), mc.Options(spmm_slab=1, spmm_merge=-1)
    m_gather, m_lds, build_all = mc.Options(spmm_slab=-1, spmm_merge=1), mc.Options(spmm_slab=1, spmm_merge=1), mc.Options(spmm_slab=1, spmm_merge=1)
    with torch.cuda.stream(stream):
        for prec in ("L8R8", "L8R4", "L4R4", "L16R8"):
            for Vv in (2, 4, 8):
                for s in (0.5, 0.7, 0.8, 0.9, 0.95, 0.98):
                    for N in (128, 256, 512):
                        if prec == "L16R8" and (Vv != 8 or N != 256):
                            continue     # the mixed-precision configuration: V = 8, N = 256
                        c = wl.spmm_case(M, K, N, Vv, s, prec, wl.seed_for(2, 1))
                        A = mc.SparseMatrix(M, K, Vv, c["row_ptr"], c["col_idx"], c["values"], mc.LHS_BITS[prec])
                        mc.set_thread_options(build_all)       # the creating thread's options: build the K-blocked and merged copies anyway
                        Af = mc.SparseMatrix(M, K, Vv, c["row_ptr"], c["col_idx"], c["values"], mc.LHS_BITS[prec])
                        mc.set_thread_options(None)
                        B = torch.from_numpy(c["B"]).cuda()
                        C = torch.empty((M, N), dtype=torch.int32, device="cuda")
                        us = time_graph(torch, stream, [lambda: mc.spmm(A, B, prec, out=C)] * 50, rounds=3, warm_ms=25.0)
                        g_us = time_graph(torch, stream, [lambda: mc.spmm(A, B, prec, out=C, options=gather_only)] * 50, rounds=3)
                        l_us = None
                        if mc.spmm_form(Af, N, prec, lds_forced) == "lds":
                            l_us = time_graph(torch, stream, [lambda: mc.spmm(Af, B, prec, out=C, options=lds_forced)] * 50, rounds=3)
                        mg_us = ml_us = None
                        if Af.merge_group:
                            mg_us = time_graph(torch, stream, [lambda: mc.spmm(Af, B, prec, out=C, options=m_gather)] * 50, rounds=3)
                            if mc.spmm_form(Af, N, prec, m_lds) == "lds":
                                ml_us = time_graph(torch, stream, [lambda: mc.spmm(Af, B, prec, out=C, options=m_lds)] * 50, rounds=3)
                        gathered = A.nvec * N * mc.RHS_BITS[prec] / 8
                        r2 = lambda x: round(x, 2) if x is not None else None
                        spmm.append(dict(prec=prec, V=Vv, s=s, N=N, us=round(us, 2), form=mc.spmm_form(A, N, prec),
                                         merged=int(mc.spmm_on_merged(A, N, prec)),
                                         gather_us=round(g_us, 2), lds_us=r2(l_us), merged_gather_us=r2(mg_us), merged_lds_us=r2(ml_us),
                                         auto_over_best=round(us / min(x for x in (g_us, l_us, mg_us, ml_us) if x is not None), 3),
                                         nvec=A.nvec, merged_nvec=(Af.merged_nvec if Af.merge_group else None),
                                         eff_tops=round(2 * A.nvec * Vv * N / us / 1e6, 1),
                                         gather_tbs=round(gathered / g_us / 1e6, 2)))
                        A.close()
                        Af.close()
        for prec in ("L8R8", "L4R4", "L16R16"):
            for Kd in (64, 128, 256):
                for s in (0.7, 0.9, 0.95):
                    c = wl.sddmm_case(M, K, Kd, V, s, prec, wl.seed_for(3, 1))
                    m = mc.SparseMatrix(M, K, V, c["row_ptr"], c["col_idx"])
                    Q, Km = torch.from_numpy(c["Q"]).cuda(), torch.from_numpy(c["Kmat"]).cuda()
                    S = torch.empty(m.nvec * V, dtype=torch.int32, device="cuda")
                    us = time_graph(torch, stream, [lambda: mc.sddmm(Q, Km, m, prec, out=S)] * 50, rounds=3, warm_ms=25.0)
                    gathered = m.nvec * Kd * mc.LHS_BITS[prec] / 8
                    sddmm.append(dict(prec=prec, Kd=Kd, s=s, us=round(us, 2), eff_tops=round(2 * m.nvec * V * Kd / us / 1e6, 1),
                                      gather_tbs=round(gathered / us / 1e6, 2)))
                    m.close()
    return {"sweep": "4096x4096, warm caches, 50 back-to-back launches per point (median of 3)",
            "library": mc.lib.mc_version().decode(), "spmm": spmm, "sddmm": sddmm}


def as_table(result):
    """The result of --sweep / --skew / --shapes as aligned text columns (one table per list of rows)."""
    lines = []
    for key, val in result.items():
        if not (isinstance(val, list) and val and isinstance(val[0], dict)):
            lines.append(f"{key}: {val}")
            continue
        cols = [c for c in val[0] if not isinstance(val[0][c], dict)]
        width = {c: max(len(c), *(len(str(r.get(c))) for r in val)) for c in cols}
        lines += ["", f"[{key}]", "  ".join(c.rjust(width[c]) for c in cols)]
        lines += ["  ".join(str(r.get(c)).rjust(width[c]) for c in cols) for r in val]
    return "\n".join(lines)


def run_point(mc, torch, spec, steps, warmup, calib_copy):
    """One SpMM configuration launched eagerly, for a profiler to look at."""
    from paper_2209_06979_amd import workloads as wl
    prec, Vv, s, N, form = spec.split(":")
    Vv, s, N = int(Vv), float(s), int(N)
    o = {"gather": mc.Options(spmm_slab=-1, spmm_merge=-1), "lds": mc.Options(spmm_slab=1, spmm_merge=-1),
         "merged": mc.Options(spmm_slab=-1, spmm_merge=1), "merged-lds": mc.Options(spmm_slab=1, spmm_merge=1), "auto": None}[form]
    c = wl.spmm_case(M, K, N, Vv, s, prec, wl.seed_for(2, 1))
    if form != "auto":
        mc.set_thread_options(o)
    A = mc.SparseMatrix(M, K, Vv, c["row_ptr"], c["col_idx"], c["values"], mc.LHS_BITS[prec])
    mc.set_thread_options(None)
    B = torch.from_numpy(c["B"]).cuda()
    C = torch.empty((M, N), dtype=torch.int32, device="cuda")
    if calib_copy:
        src = torch.empty(64 * 1024 * 1024, dtype=torch.uint8, device="cuda")
        torch.empty_like(src).copy_(src)
    for _ in range(warmup):
        mc.spmm(A, B, prec, out=C, options=o)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        mc.spmm(A, B, prec, out=C, options=o)
    torch.cuda.synchronize()
    return dict(point=spec, form_run=mc.spmm_form(A, N, prec, o), on_merged_copy=mc.spmm_on_merged(A, N, prec, o), launches=steps,
                us_per_launch_eager=round((time.perf_counter() - t0) / steps * 1e6, 2), nvec=A.nvec,
                gathered_bytes=int(A.nvec * N * mc.RHS_BITS[prec] // 8), library=mc.lib.mc_version().decode())


def run_phases(mc, torch):
    """Where the time of the headline SpMM goes: the same kernel with ten clock readings per wave (mc_probe_spmm_phases),
    launched back to back like the timed kernel; the readings of the last launches, relative to the first wave's start."""
    from paper_2209_06979_amd import workloads as wl
    c = wl.spmm_case(M, K, 256, V, SPARSITY, "L8R8", wl.seed_for(2, 1))
    A = mc.SparseMatrix(M, K, V, c["row_ptr"], c["col_idx"], c["values"], 8)
    B = torch.from_numpy(c["B"]).cuda()
    ref = mc.spmm(A, B, "L8R8", options=mc.Options(spmm_merge=-1, spmm_slab=-1))
    stream = torch.cuda.Stream()
    names = ["wave started", "kernel arguments and panel pointers arrived", "column indices and A operands arrived",
             "rows of the first chunk landed", "all chunks in the accumulators", "partial tile written",
             "workgroup barrier passed", "output pieces summed", "stores issued", "stores acknowledged"]
    samples = []
    with torch.cuda.stream(stream):
        plain_us = time_graph(torch, stream, [lambda: mc.spmm(A, B, "L8R8", out=ref)] * 100, rounds=3, warm_ms=25.0)
        out, trace = mc.probe_spmm_phases(A, B)
        probe_us = time_graph(torch, stream, [lambda: mc.probe_spmm_phases(A, B, out=out, trace=trace)] * 100, rounds=3)
        for _ in range(5):
            for _ in range(20):
                mc.probe_spmm_phases(A, B, out=out, trace=trace)
            stream.synchronize()
            samples.append(trace.cpu().numpy().astype(np.int64) * 0.01)      # 100 MHz ticks -> microseconds
    assert torch.equal(out, ref), "the instrumented kernel's product differs"
    rows = []
    spans = [float((t[:, 9].max() - t[:, 0].min())) for t in samples]
    t = samples[int(np.argsort(spans)[len(spans) // 2])]                       # the launch with the median span
    rel = t - t[:, 0].min()
    for k, n in enumerate(names):
        col = rel[:, k]
        rows.append(dict(stage=n, first=round(float(col.min()), 2), p10=round(float(np.percentile(col, 10)), 2),
                         median=round(float(np.median(col)), 2), p90=round(float(np.percentile(col, 90)), 2),
                         last=round(float(col.max()), 2),
                         median_since_previous_stage=(round(float(np.median(t[:, k] - t[:, k - 1])), 2) if k else 0.0)))
    A.close()
    return {"phases": "SpMM L8-R8 4096x4096 V=8 s=0.9 N=256, kernel spmm_kernel<128,2,8,8,false,2> with time stamps; microseconds "
                      "after the first wave of the launch started; one launch (the median of 5 by span) of 2048 waves",
            "library": mc.lib.mc_version().decode(), "us_per_launch_plain_kernel": round(plain_us, 2),
            "us_per_launch_instrumented_kernel": round(probe_us, 2),
            "span_first_start_to_last_store_us": [round(x, 2) for x in sorted(spans)], "waves": rows}


def lognormal_counts(P, mean, sigma, Kcols, rng):
    """Vectors per panel: log-normal with the given sigma of the logarithm, rescaled to the given mean."""
    if sigma == 0:
        return np.full(P, mean)
    c = rng.lognormal(0.0, sigma, P)
    return np.clip(np.rint(c / c.mean() * mean), 0, Kcols).astype(np.int64)


def run_skew(mc, torch):
    """Panels of very unequal length (a few rows of an attention mask attend to almost everything): vectors per panel
    log-normal around the headline's 410, SpMM L8-R8 N = 256 and SDDMM L8-R8 K = 256 at 4096 x 4096, with the long
    panels cut into work items (automatic) and without."""
    from paper_2209_06979_amd import workloads as wl
    stream = torch.cuda.Stream()
    P = M // V
    rng = np.random.default_rng(3)
    whole = mc.Options(spmm_splitting=-1)
    rows = []
    with torch.cuda.stream(stream):
        for sigma in (0.0, 0.5, 1.0, 1.5):
            counts = lognormal_counts(P, 410, sigma, K, rng)
            rp, ci = wl.ragged_pattern(M, K, V, counts, 11)
            nvec = len(ci)
            A = mc.SparseMatrix(M, K, V, rp, ci, wl.uniform_int8((nvec, V), 12), 8)
            B = torch.from_numpy(wl.uniform_int8((K, N_SPMM), 13)).cuda()
            C = torch.empty((M, N_SPMM), dtype=torch.int32, device="cuda")
            Q = torch.from_numpy(wl.uniform_int8((M, KD_SDDMM), 14)).cuda()
            Km = torch.from_numpy(wl.uniform_int8((K, KD_SDDMM), 15)).cuda()
            S = torch.empty(nvec * V, dtype=torch.int32, device="cuda")
            row = dict(sigma=sigma, nvec=nvec, longest_panel=int(counts.max()), longest_over_mean=round(float(counts.max()) / 410, 1))
            row["spmm_us"] = round(time_graph(torch, stream, [lambda: mc.spmm(A, B, "L8R8", out=C)] * 50, rounds=3, warm_ms=25.0), 2)
            row["spmm_whole_panels_us"] = round(time_graph(torch, stream, [lambda: mc.spmm(A, B, "L8R8", out=C, options=whole)] * 50, rounds=3), 2)
            Am = mc.SparseMatrix(M, K, V, rp, ci)      # the pattern alone (a mask is cut into shorter work items than an operand)
            row["sddmm_us"] = round(time_graph(torch, stream, [lambda: mc.sddmm(Q, Km, Am, "L8R8", out=S)] * 50, rounds=3), 2)
            row["sddmm_whole_panels_us"] = round(time_graph(torch, stream, [lambda: mc.sddmm(Q, Km, Am, "L8R8", out=S, options=whole)] * 50, rounds=3), 2)
            # the attention layer, 8 heads (timing only: one random tensor serves as Q, K and V): the fused kernel runs
            # the panels of such a mask class by class (1, 2, 4, 8 waves per panel); the kernel pipeline for comparison
            for dk in (64, 128):
                x = torch.randint(-127, 128, (L_ATT, HEADS, dk), dtype=torch.int8, device="cuda").permute(1, 0, 2)
                O = torch.empty((L_ATT, HEADS, dk), dtype=torch.float32, device="cuda").permute(1, 0, 2)
                for key, o in ((f"attention_dk{dk}_us", mc.Options()), (f"attention_dk{dk}_kernel_pipeline_us", mc.Options(attention_mode=1))):
                    ws = torch.empty(max(16, mc.attention_workspace_needed(HEADS, dk, Am, 8, o)), dtype=torch.uint8, device="cuda")
                    row[key] = round(time_graph(torch, stream, [lambda: mc.sparse_attention(x, x, x, Am, 0.02, 0.02, 0.02, 1 / 127, out=O,
                                                                                            workspace=ws, options=o)] * 20, rounds=3), 2)
            row["spmm_eff_tops"] = round(2 * nvec * V * N_SPMM / row["spmm_us"] / 1e6, 1)
            row["sddmm_eff_tops"] = round(2 * nvec * V * KD_SDDMM / row["sddmm_us"] / 1e6, 1)
            rows.append(row)
            A.close()
            Am.close()
    return {"skew": "4096x4096 V=8, vectors per panel log-normal (mean 410), L8-R8, N = K_d = 256, attention with 8 heads, "
                    "warm caches, 50 (attention: 20) back-to-back launches (median of 3)",
            "library": mc.lib.mc_version().decode(), "rows": rows}


def run_shapes(mc, torch):
    """Matrices with few or short panels (a launch has far fewer panels than the chip has wave slots): the kernel
    variant the library picks from the shape against every tile width x wave count it could be pinned to."""
    from paper_2209_06979_amd import workloads as wl
    import itertools
    stream = torch.cuda.Stream()
    shapes = [(256, 2304, 512, 0.7), (256, 2304, 512, 0.9), (512, 512, 128, 0.8), (1024, 1024, 256, 0.9), (256, 4096, 256, 0.9),
              (512, 4096, 512, 0.9), (1024, 4096, 256, 0.7), (2048, 2048, 256, 0.9), (256, 1024, 128, 0.5), (128, 4096, 512, 0.5),
              (64, 4096, 512, 0.9), (4096, 512, 128, 0.9), (512, 8192, 256, 0.95), (2048, 4096, 128, 0.98), (128, 2304, 256, 0.7)]
    rows = []
    with torch.cuda.stream(stream):
        for prec in ("L8R8", "L8R4", "L16R8"):
            for Ms, Ks, N, sp in shapes:
                c = wl.spmm_case(Ms, Ks, N, V, sp, prec, 1)
                A = mc.SparseMatrix(Ms, Ks, V, c["row_ptr"], c["col_idx"], c["values"], mc.LHS_BITS[prec])
                B = torch.from_numpy(c["B"]).cuda()
                C = torch.empty((Ms, N), dtype=torch.int32, device="cuda")
                row_bytes = N * mc.RHS_BITS[prec] // 8
                time_graph(torch, stream, [lambda: mc.spmm(A, B, prec, out=C)] * 50, rounds=1, warm_ms=25.0)
                pinned = {}
                for tile, waves in itertools.product((64, 128, 256), (1, 2, 4, 8)):
                    if tile > row_bytes or (tile == 256 and mc.RHS_BITS[prec] == 4):
                        continue
                    o = mc.Options(spmm_row_tile_bytes=tile, spmm_waves=waves)
                    try:
                        pinned[f"{tile}x{waves}"] = round(time_graph(torch, stream, [lambda: mc.spmm(A, B, prec, out=C, options=o)] * 50, rounds=3), 2)
                    except mc.MagicubeError:
                        pass     # a variant that does not exist for this precision
                auto = time_graph(torch, stream, [lambda: mc.spmm(A, B, prec, out=C)] * 50, rounds=3)
                best = min(pinned, key=pinned.get)
                rows.append(dict(prec=prec, M=Ms, K=Ks, N=N, s=sp, panels=Ms // V, auto_us=round(auto, 2), form=mc.spmm_form(A, N, prec),
                                 best_pinned=best, best_pinned_us=pinned[best], auto_over_best=round(auto / pinned[best], 2),
                                 pinned_us=pinned))
                A.close()
    worst = max(r["auto_over_best"] for r in rows)
    within5 = sum(r["auto_over_best"] <= 1.05 for r in rows)
    return {"shapes": "SpMM, V=8, warm caches, 50 back-to-back launches (median of 3); pinned = tile bytes x waves",
            "library": mc.lib.mc_version().decode(), "points": len(rows), "within_5_percent_of_best": within5,
            "worst_auto_over_best": worst, "rows": rows}


def time_graph(torch, stream, launches, rounds=5, warm_ms=0.0):
    """Microseconds per launch: the launches captured once into a HIP graph, replayed between two
    events on the launch stream; median over `rounds` replays.  warm_ms: replay for that long first (after host
    work such as a format build the clocks have dropped, which a single replay of a short graph does not undo)."""
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=stream):
        for f in launches:
            f()
    g.replay()
    stream.synchronize()
    t0 = time.perf_counter()
    while (time.perf_counter() - t0) * 1e3 < warm_ms:
        g.replay()
        stream.synchronize()
    samples = []
    for _ in range(rounds):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        g.replay()
        e1.record(stream)
        e1.synchronize()
        samples.append(e0.elapsed_time(e1) * 1e3 / len(launches))
    return float(np.median(samples))


def measure_extras(mc, torch, prob, stream, reps, up):
    """Measurements beside the step (called on the launch stream).

    headline: the L8-R8 SpMM (a) with cold caches -- 80 copies of all its operands (about 620 MB,
    more than L2 plus the 256 MB memory-side cache) visited in turn, so every launch finds its
    operands in HBM only; (b) its gather alone (mc_probe_gather, same indices and launch shape).
    wider_precisions: the emulated precisions and layer variants that are not rows of the step.
    """
    from paper_2209_06979_amd import workloads as wl
    out = {}
    c = prob["spmm_L8R8"]
    nsets = 80
    sets = []
    for _ in range(nsets):
        A = mc.SparseMatrix(M, K, V, c["row_ptr"], c["col_idx"], c["values"], 8)
        sets.append((A, up(c["B"]), torch.empty((M, N_SPMM), dtype=torch.int32, device="cuda")))
    cold = time_graph(torch, stream, [(lambda A=A, B=B, C=C: mc.spmm(A, B, "L8R8", out=C)) for A, B, C in sets])
    A, B, C = sets[0]
    sink = mc.probe_gather(A, B, "L8R8")
    gather = time_graph(torch, stream, [lambda: mc.probe_gather(A, B, "L8R8", sink=sink)] * reps)
    warm = time_graph(torch, stream, [lambda: mc.spmm(A, B, "L8R8", out=C)] * reps)
    nvec = A.nvec
    alg = spmm_alg_bytes(nvec, M // V, 8, 8, N_SPMM)
    out["headline"] = dict(cold_us=round(cold, 2), cold_alg_gbs=round(alg / cold / 1e3, 1),
                           cold_hbm_frac=round(alg / cold / 1e3 / HBM_PEAK_GBS, 4),
                           gather_only_us=round(gather, 2), time_over_gather_only=round(warm / gather, 2),
                           gathered_bytes=int(nvec * N_SPMM),
                           gather_only_tbs=round(nvec * N_SPMM / gather / 1e6, 2))
    for A, _, _ in sets:
        A.close()
    del sets

    # Cold caches for the other kernels of the step as well: as many independent copies of the
    # operands as it takes to exceed 600 MB, visited in turn.
    cold_all = {"spmm_L8R8": round(cold, 2)}
    def cold_time(make, footprint_bytes):
        n = int(600e6 // footprint_bytes) + 2
        made = [make() for _ in range(n)]
        us = time_graph(torch, stream, [m[0] for m in made])
        for m in made:
            for h in m[1]:
                h.close()
        return round(us, 2)
    for prec in ("L8R4", "L4R4", "L16R8"):
        cc = prob["spmm_" + prec]
        def make(cc=cc, prec=prec):
            A = mc.SparseMatrix(M, K, V, cc["row_ptr"], cc["col_idx"], cc["values"], mc.LHS_BITS[prec])
            B, C = up(cc["B"]), torch.empty((M, N_SPMM), dtype=torch.int32, device="cuda")
            return (lambda: mc.spmm(A, B, prec, out=C)), [A]
        cold_all["spmm_" + prec] = cold_time(make, spmm_alg_bytes(nvec, M // V, mc.LHS_BITS[prec], mc.RHS_BITS[prec], N_SPMM))
    for prec in ("L8R8", "L4R4"):
        cc = prob["sddmm_" + prec]
        def make(cc=cc, prec=prec):
            mk = mc.SparseMatrix(M, K, V, cc["row_ptr"], cc["col_idx"])
            Q, Km = up(cc["Q"]), up(cc["Kmat"])
            S = torch.empty(mk.nvec * V, dtype=torch.int32, device="cuda")
            return (lambda: mc.sddmm(Q, Km, mk, prec, out=S)), [mk]
        cold_all["sddmm_" + prec] = cold_time(make, sddmm_alg_bytes(nvec, M // V, mc.LHS_BITS[prec], KD_SDDMM))
    att = prob["attention"]
    def make_att():
        mk = mc.SparseMatrix(L_ATT, L_ATT, V, att["row_ptr"], att["col_idx"])
        tm = lambda a: up(np.ascontiguousarray(np.transpose(a, (1, 0, 2)))).permute(1, 0, 2)
        q, k, v = tm(att["q8"]), tm(att["k8"]), tm(att["v8"])
        O = torch.empty((L_ATT, HEADS, DK), dtype=torch.float32, device="cuda").permute(1, 0, 2)
        ws = torch.empty(mc.attention_workspace_bytes(HEADS, mk), dtype=torch.uint8, device="cuda")
        return (lambda: mc.sparse_attention(q, k, v, mk, att["s_q"], att["s_k"], att["s_v"], att["s_p"], out=O, workspace=ws)), [mk]
    cold_all["attention"] = cold_time(make_att, HEADS * 7 * L_ATT * DK)
    out["cold_us"] = cold_all

    # What the memory system sustains for this access pattern: the gather alone on 32x the panels
    # (launch and tail amortised), rows of 64 bytes (the attention kernel's K / V rows) and of 128
    # bytes (the SpMM's row pieces), from a table that stays in L2 like B, K and V do.
    peak = {}
    for rb in (64, 128):
        cg = wl.spmm_case(32 * M, K, rb, V, SPARSITY, "L8R8", wl.seed_for(2, 900 + rb))
        Ag = mc.SparseMatrix(32 * M, K, V, cg["row_ptr"], cg["col_idx"], cg["values"], 8)
        Bg = up(cg["B"])
        sg = mc.probe_gather(Ag, Bg, "L8R8")
        best = None
        for waves in (1, 2, 4):       # the best launch shape counts
            mc.set_spmm_variant(rb, waves)
            us = time_graph(torch, stream, [lambda: mc.probe_gather(Ag, Bg, "L8R8", sink=sg)] * 20)
            best = us if best is None else min(best, us)
        mc.set_spmm_variant(0, 0)
        peak[rb] = Ag.nvec * rb / best / 1e6   # TB/s
        Ag.close()
    out["gather_peak_tbs"] = {"rows_64B": round(peak[64], 2), "rows_128B": round(peak[128], 2)}
    # The headline SpMM with 16 times the rows (65,536 x 4096, same sparsity, V and N): a launch of many rounds of
    # workgroups, where start-up, the chain of dependent first loads and the tail no longer count.
    cb = wl.spmm_case(16 * M, K, N_SPMM, V, SPARSITY, "L8R8", wl.seed_for(2, 950))
    Ab = mc.SparseMatrix(16 * M, K, V, cb["row_ptr"], cb["col_idx"], cb["values"], 8)
    Bb, Cb = up(cb["B"]), torch.empty((16 * M, N_SPMM), dtype=torch.int32, device="cuda")
    usb = time_graph(torch, stream, [lambda: mc.spmm(Ab, Bb, "L8R8", out=Cb)] * 10)
    algb = Ab.nvec * V + 4 * Ab.nvec + 8 * (16 * M // V) + K * N_SPMM + 4 * 16 * M * N_SPMM
    out["headline_at_16x_rows"] = dict(us=round(usb, 2), eff_tops=round(2 * Ab.nvec * V * N_SPMM / usb / 1e6, 1),
                                       alg_gbs=round(algb / usb / 1e3, 1), hbm_frac=round(algb / usb / 1e3 / HBM_PEAK_GBS, 4),
                                       gather_tbs=round(Ab.nvec * N_SPMM / usb / 1e6, 2),
                                       frac_of_gather_peak=round(Ab.nvec * N_SPMM / usb / 1e6 / peak[128], 3))
    Ab.close()
    del Bb, Cb
    out["headline"]["frac_of_gather_peak"] = round(nvec * N_SPMM / peak[128] / 1e6 / warm, 3)

    # The matrix unit alone: 1024 workgroups x 4 waves x 2000 x 8 MFMAs (16x16x64 int8, 32768 operations each) on
    # registers, no memory traffic: what this device sustains, beside the published peak.
    wg, iters = 1024, 2000
    sink = mc.probe_mfma(wg, iters)
    us = min(time_graph(torch, stream, [lambda: mc.probe_mfma(wg, iters, sink=sink)] * 3) for _ in range(3))
    # one wave per SIMD (256 workgroups of 4 waves): the first wave's own count of shader-clock cycles and of ticks
    # of the constant 100 MHz clock over its loop tell cycles per MFMA and the clock under this load apart
    sink1 = mc.probe_mfma(256, iters)
    us1 = min(time_graph(torch, stream, [lambda: mc.probe_mfma(256, iters, sink=sink1)] * 3) for _ in range(3))
    cyc, ticks = (int(v) for v in sink1[:2].cpu())
    out["mfma_i8_peak"] = dict(measured_tops=round(wg * 4 * iters * 8 * 32768 / us / 1e6, 1), published_tops=I8_MFMA_PEAK_TOPS,
                               us=round(us, 1), instructions=wg * 4 * iters * 8,
                               one_wave_per_simd=dict(tops=round(256 * 4 * iters * 8 * 32768 / us1 / 1e6, 1),
                                                      shader_cycles_per_mfma=round(cyc / (iters * 8), 2),
                                                      shader_clock_ghz=round(cyc / max(ticks, 1) * 0.1, 3)))
    # four waves per SIMD keep the matrix unit busy: cycles it spends per instruction at the clock just measured
    out["mfma_i8_peak"]["shader_cycles_per_mfma_of_a_busy_simd"] = round(
        out["mfma_i8_peak"]["one_wave_per_simd"]["shader_clock_ghz"] * 1e3 * us / (wg * 4 * iters * 8 / 1024), 2)
    # What one kernel launch costs inside a graph whatever it does: one workgroup, one MFMA round.
    s1 = mc.probe_mfma(1, 1)
    out["launch_floor_us"] = round(time_graph(torch, stream, [lambda: mc.probe_mfma(1, 1, sink=s1)] * reps), 2)

    wide = {}
    for i, prec in enumerate(["L16R16", "L16R4", "L12R4"]):
        cc = wl.spmm_case(M, K, N_SPMM, V, SPARSITY, prec, wl.seed_for(2, 100 + 10 * i))
        A = mc.SparseMatrix(M, K, V, cc["row_ptr"], cc["col_idx"], cc["values"], mc.LHS_BITS[prec])
        B = up(cc["B"])
        C = torch.empty((M, N_SPMM), dtype=torch.int32, device="cuda")
        us = time_graph(torch, stream, [lambda: mc.spmm(A, B, prec, out=C)] * reps)
        ops = 2 * A.nvec * V * N_SPMM
        b = spmm_alg_bytes(A.nvec, M // V, 16, mc.RHS_BITS[prec], N_SPMM)
        wide["spmm_" + prec] = dict(us=round(us, 2), eff_tops=round(ops / us / 1e6, 1), alg_gbs=round(b / us / 1e3, 1))
        A.close()
    cc = wl.sddmm_case(M, K, KD_SDDMM, V, SPARSITY, "L16R16", wl.seed_for(3, 100))
    mask = mc.SparseMatrix(M, K, V, cc["row_ptr"], cc["col_idx"])
    Q, Km = up(cc["Q"]), up(cc["Kmat"])
    S = torch.empty(mask.nvec * V, dtype=torch.int32, device="cuda")
    us = time_graph(torch, stream, [lambda: mc.sddmm(Q, Km, mask, "L16R16", out=S)] * reps)
    ops = 2 * mask.nvec * V * KD_SDDMM
    wide["sddmm_L16R16"] = dict(us=round(us, 2), eff_tops=round(ops / us / 1e6, 1),
                                alg_gbs=round(sddmm_alg_bytes(mask.nvec, M // V, 16, KD_SDDMM) / us / 1e3, 1))
    mask.close()
    att = prob["attention"]
    amask = mc.SparseMatrix(L_ATT, L_ATT, V, att["row_ptr"], att["col_idx"])
    O = torch.empty((HEADS, L_ATT, DK), dtype=torch.float32, device="cuda")
    for name, p_bits, qkv_bits in (("attention_16b8b", 16, 8), ("attention_8b4b", 8, 4)):
        if qkv_bits == 4:
            (q, s_q), (k, s_k), (v, s_v) = (quantize_on_gpu(mc, torch, att[n], 4) for n in "qkv")
        else:
            q, k, v, s_q, s_k, s_v = att["q8"], att["k8"], att["v8"], att["s_q"], att["s_k"], att["s_v"]
        q, k, v = up(q), up(k), up(v)
        ws = torch.empty(mc.attention_workspace_bytes(HEADS, amask, p_bits), dtype=torch.uint8, device="cuda")
        s_p = np.float32(1.0 / (32639.0 if p_bits == 16 else 127.0))
        us = time_graph(torch, stream, [lambda: mc.sparse_attention(q, k, v, amask, s_q, s_k, s_v, s_p, out=O, workspace=ws,
                                                                    p_bits=p_bits, qkv_bits=qkv_bits)] * reps)
        ops = HEADS * 2 * (2 * amask.nvec * V * DK)
        wide[name] = dict(us=round(us, 2), eff_tops=round(ops / us / 1e6, 1))
    # the paper's output type: fp16 written by the fused dequantisation (the step's rows write int32 / fp32)
    tmaj = lambda x: up(np.ascontiguousarray(np.transpose(x, (1, 0, 2)))).permute(1, 0, 2)
    q, k, v = tmaj(att["q8"]), tmaj(att["k8"]), tmaj(att["v8"])
    O16 = torch.empty((L_ATT, HEADS, DK), dtype=torch.float16, device="cuda").permute(1, 0, 2)
    ws = torch.empty(mc.attention_workspace_bytes(HEADS, amask), dtype=torch.uint8, device="cuda")
    us = time_graph(torch, stream, [lambda: mc.sparse_attention(q, k, v, amask, att["s_q"], att["s_k"], att["s_v"], att["s_p"],
                                                                out=O16, workspace=ws, out_dtype=torch.float16)] * reps)
    wide["attention_8b8b_fp16_out"] = dict(us=round(us, 2), eff_tops=round(HEADS * 2 * (2 * amask.nvec * V * DK) / us / 1e6, 1))
    # the general path (any head dimension up to 256 bytes per row, long panels): scores and softmax in one kernel
    # that writes the codes in the SpMM's operand format, then the SpMM; and the older form of three kernels with
    # the scores in HBM between them (what remains for still wider rows or longer panels)
    O32 = torch.empty((L_ATT, HEADS, DK), dtype=torch.float32, device="cuda").permute(1, 0, 2)
    for name, mode in (("attention_8b8b_scores_softmax_then_spmm", 1), ("attention_8b8b_three_kernels", 6)):
        o = mc.Options(attention_mode=mode)
        wsm = torch.empty(max(16, mc.attention_workspace_needed(HEADS, DK, amask, 8, o)), dtype=torch.uint8, device="cuda")
        us = time_graph(torch, stream, [lambda: mc.sparse_attention(q, k, v, amask, att["s_q"], att["s_k"], att["s_v"], att["s_p"],
                                                                    out=O32, workspace=wsm, options=o)] * reps)
        wide[name] = dict(us=round(us, 2), eff_tops=round(HEADS * 2 * (2 * amask.nvec * V * DK) / us / 1e6, 1),
                          workspace_bytes=int(wsm.numel()))
    # the softmax step on its own (8 heads of scores in, int8 codes out; 5 bytes per stored score)
    nsc = amask.nvec * V
    Ssm = torch.randint(-60000, 60000, (HEADS, nsc), dtype=torch.int32, device="cuda")
    csm = torch.empty((HEADS, nsc), dtype=torch.int8, device="cuda")
    us = time_graph(torch, stream, [lambda: mc.sparse_softmax(amask, Ssm, 2.5e-4, 127.0, out=csm)] * reps)
    wide["sparse_softmax_8_heads"] = dict(us=round(us, 2), gbs=round(HEADS * nsc * 5 / us / 1e3, 1),
                                          hbm_frac=round(HEADS * nsc * 5 / us / 1e3 / HBM_PEAK_GBS, 3))
    del Ssm, csm
    # the same layer with head dimension 128 (rows of 128 bytes): the fused kernel and the three kernels
    x128, s128 = quantize_on_gpu(mc, torch, wl.normal_fp32((HEADS, L_ATT, 128), wl.seed_for(5, 9)))
    q128 = tmaj(x128) # serves as Q, K and V: timing only
    O128 = torch.empty((L_ATT, HEADS, 128), dtype=torch.float32, device="cuda").permute(1, 0, 2)
    for name, mode in (("attention_8b8b_dk128", 0), ("attention_8b8b_dk128_scores_softmax_then_spmm", 1),
                       ("attention_8b8b_dk128_three_kernels", 6)):
        o = mc.Options(attention_mode=mode)
        wsm = torch.empty(max(16, mc.attention_workspace_needed(HEADS, 128, amask, 8, o)), dtype=torch.uint8, device="cuda")
        us = time_graph(torch, stream, [lambda: mc.sparse_attention(q128, q128, q128, amask, s128, s128, s128, att["s_p"],
                                                                    out=O128, workspace=wsm, options=o)] * reps)
        wide[name] = dict(us=round(us, 2), eff_tops=round(HEADS * 2 * (2 * amask.nvec * V * 128) / us / 1e6, 1))
    # head dimensions below the fused kernel's tile of 64 or 128 (rows with fewer 16-byte pieces than the tile), and one
    # above every tile (160: the kernel pipeline is what runs)
    for dkx in (32, 96, 160):
        xx, sx = quantize_on_gpu(mc, torch, wl.normal_fp32((HEADS, L_ATT, dkx), wl.seed_for(5, 10 + dkx)))
        qx = tmaj(xx)
        Ox = torch.empty((L_ATT, HEADS, dkx), dtype=torch.float32, device="cuda").permute(1, 0, 2)
        wsm = torch.empty(max(16, mc.attention_workspace_needed(HEADS, dkx, amask, 8)), dtype=torch.uint8, device="cuda")
        us = time_graph(torch, stream, [lambda: mc.sparse_attention(qx, qx, qx, amask, sx, sx, sx, att["s_p"],
                                                                    out=Ox, workspace=wsm)] * reps)
        wide[f"attention_8b8b_dk{dkx}"] = dict(us=round(us, 2), eff_tops=round(HEADS * 2 * (2 * amask.nvec * V * dkx) / us / 1e6, 1))
    amask.close()
    cc = prob["spmm_L8R8"]
    A = mc.SparseMatrix(M, K, V, cc["row_ptr"], cc["col_idx"], cc["values"], 8)
    B, C16 = up(cc["B"]), torch.empty((M, N_SPMM), dtype=torch.float16, device="cuda")
    us = time_graph(torch, stream, [lambda: mc.spmm_dequant(A, B, "L8R8", 1e-4, torch.float16, out=C16)] * reps)
    wide["spmm_L8R8_fp16_out"] = dict(us=round(us, 2), eff_tops=round(2 * A.nvec * V * N_SPMM / us / 1e6, 1))
    # What the pieces of the SpMM design are worth (the counterpart of the ablation in Section 5.1, on the
    # headline matrix and on a matrix of that section's shape): one wave per panel on 64-byte row tiles with
    # one chunk in flight; then the tile and wave count chosen from the shape; then two chunks in flight.
    C32 = torch.empty((M, N_SPMM), dtype=torch.int32, device="cuda")
    ca = wl.spmm_case(256, 2304, 512, V, 0.7, "L8R8", wl.seed_for(2, 900))
    A2 = mc.SparseMatrix(256, 2304, V, ca["row_ptr"], ca["col_idx"], ca["values"], 8)
    B2, C2 = up(ca["B"]), torch.empty((256, 512), dtype=torch.int32, device="cuda")
    ablation = {}
    for name, (Ax, Bx, Cx) in (("headline_4096x4096_s0.9_N256", (A, B, C32)), ("section5.1_shape_256x2304_s0.7_N512", (A2, B2, C2))):
        row = {}
        for step, (tile, waves, stages) in (("plain", (64, 1, 1)), ("tile_and_waves_chosen", (0, 0, 1)), ("two_chunks_in_flight", (0, 0, 2))):
            o = mc.Options(spmm_row_tile_bytes=tile, spmm_waves=waves, spmm_stages=stages, spmm_slab=-1, spmm_merge=-1)
            row[step + "_us"] = round(time_graph(torch, stream, [lambda: mc.spmm(Ax, Bx, "L8R8", out=Cx, options=o)] * reps), 2)
        row["automatic_us"] = round(time_graph(torch, stream, [lambda: mc.spmm(Ax, Bx, "L8R8", out=Cx)] * reps), 2)
        row["automatic_form"] = mc.spmm_form(Ax, Bx.shape[1], "L8R8")
        ablation[name] = row
    out["spmm_design_steps"] = ablation
    A2.close()
    A.close()
    cc = prob["sddmm_L8R8"]
    mask = mc.SparseMatrix(M, K, V, cc["row_ptr"], cc["col_idx"])
    Q, Km = up(cc["Q"]), up(cc["Kmat"])
    S16 = torch.empty(mask.nvec * V, dtype=torch.float16, device="cuda")
    us = time_graph(torch, stream, [lambda: mc.sddmm_dequant(Q, Km, mask, "L8R8", 1e-4, torch.float16, out=S16)] * reps)
    wide["sddmm_L8R8_fp16_out"] = dict(us=round(us, 2), eff_tops=round(2 * mask.nvec * V * KD_SDDMM / us / 1e6, 1))
    mask.close()
    out["wider_precisions"] = wide

    # The layer at the shapes of the paper's end-to-end latency figure (Section 5.3: 4 / 8 heads, sequence
    # 4096 / 8192, batch 2 / 8, sparsity 0.9 / 0.95, head dimension 64), one launch per batch, tensors as
    # (batch, head, token, d) and in the (batch, token, head, d) order a QKV projection writes.
    shapes = {}
    for L, heads, batch, sp in ((4096, 8, 8, 0.9), (8192, 4, 8, 0.9), (8192, 4, 2, 0.95)):
        c = wl.attention_case(1, L, DK, V, sp, wl.seed_for(5, L + heads + batch))
        m = mc.SparseMatrix(L, L, V, c["row_ptr"], c["col_idx"])
        x = wl.normal_fp32((batch, heads, L, DK), wl.seed_for(5, 7))
        for layout in ("head", "token"):
            if layout == "token":
                O = torch.empty((batch, L, heads, DK), dtype=torch.float32, device="cuda").permute(0, 2, 1, 3)
            else:
                O = torch.empty((batch, heads, L, DK), dtype=torch.float32, device="cuda")
            for name, p_bits, qkv_bits in (("8b-8b", 8, 8), ("16b-8b", 16, 8), ("8b-4b", 8, 4)):
                xq, sx = quantize_on_gpu(mc, torch, x, qkv_bits)
                # the same tensor serves as Q, K and V: timing only
                q = up(np.ascontiguousarray(np.transpose(xq, (0, 2, 1, 3)))).permute(0, 2, 1, 3) if layout == "token" else up(xq)
                ws = torch.empty(mc.attention_workspace_bytes(heads, m, p_bits), dtype=torch.uint8, device="cuda")
                s_p = np.float32(1.0 / (32639.0 if p_bits == 16 else 127.0))
                us = time_graph(torch, stream, [lambda: mc.sparse_attention(q, q, q, m, sx, sx, sx, s_p, out=O, workspace=ws,
                                                                            p_bits=p_bits, qkv_bits=qkv_bits)] * 20)
                ops = batch * heads * 2 * (2 * m.nvec * V * DK)
                shapes[f"L{L}_h{heads}_b{batch}_s{sp}_{name}_{layout}-major"] = dict(us=round(us, 1), eff_tops=round(ops / us / 1e6, 1))
        m.close()
    out["layer_at_inference_shapes"] = shapes

    # The layer's first step, quantisation of fp32 projections (a pure streaming kernel): a batch
    # of 64 layers' worth of one tensor, 128 Mi elements, far beyond every cache.
    xs = torch.empty(64 * HEADS * L_ATT * DK, dtype=torch.float32, device="cuda").normal_()
    qs = torch.empty(xs.numel(), dtype=torch.int8, device="cuda")
    mx = torch.empty(1, dtype=torch.float32, device="cuda")
    quant = {}
    for name, fn, nbytes in (("absmax", lambda: mc.absmax(xs, out=mx), 4 * xs.numel()),
                             ("quantize_int8", lambda: mc.quantize(xs, 0.03, 8, out=qs), 5 * xs.numel())):
        us = time_graph(torch, stream, [fn] * 5)
        quant[name] = dict(us=round(us, 1), gbs=round(nbytes / us / 1e3, 1), hbm_frac=round(nbytes / us / 1e3 / HBM_PEAK_GBS, 3))
    out["quantisation_streaming"] = quant
    del xs, qs
    return out


def cpu_baseline(prob):
    """The CPU oracle on the headline operation (the L8-R8 SpMM of `value`), repeated for about ten seconds on all
    host cores the oracle's OpenMP runtime uses, best pass; beside it one pass of the operations of a whole step
    and the headline on one core."""
    import oracle
    c = prob["spmm_L8R8"]
    head_ops = 2 * len(c["col_idx"]) * V * N_SPMM
    best, passes, t_all = None, 0, time.perf_counter()
    while passes < 3 or (time.perf_counter() - t_all < 10.0 and passes < 400):
        t0 = time.perf_counter()
        oracle.spmm(M, K, V, c["row_ptr"], c["col_idx"], c["values"], c["B"], "L8R8")
        dt = time.perf_counter() - t0
        best = dt if best is None else min(best, dt)
        passes += 1
    step_ops = 0
    t0 = time.perf_counter()
    for prec in ["L8R8", "L8R4", "L4R4", "L16R8"]:
        cc = prob["spmm_" + prec]
        oracle.spmm(M, K, V, cc["row_ptr"], cc["col_idx"], cc["values"], cc["B"], prec)
        step_ops += 2 * len(cc["col_idx"]) * V * N_SPMM
    for prec in ["L8R8", "L4R4"]:
        cc = prob["sddmm_" + prec]
        oracle.sddmm(M, K, V, cc["row_ptr"], cc["col_idx"], cc["Q"], cc["Kmat"], prec)
        step_ops += 2 * len(cc["col_idx"]) * V * KD_SDDMM
    a = prob["attention"]
    oracle.attention(a["q8"], a["k8"], a["v8"], a["row_ptr"], a["col_idx"], V, a["s_q"], a["s_k"], a["s_v"], a["s_p"])
    step_ops += HEADS * 2 * (2 * len(a["col_idx"]) * V * DK)
    step_s = time.perf_counter() - t0
    nthreads = oracle.num_threads()
    oracle.set_num_threads(1)
    try:
        t0 = time.perf_counter()
        oracle.spmm(M, K, V, c["row_ptr"], c["col_idx"], c["values"], c["B"], "L8R8")
        single = time.perf_counter() - t0
    finally:
        oracle.set_num_threads(nthreads)
    return dict(value=round(head_ops / best / 1e12, 5), unit="TOPS", cores=nthreads, kind="oracle",
                seconds_per_pass=round(best, 4), passes=passes,
                whole_step_tops=round(step_ops / step_s / 1e12, 5), whole_step_seconds=round(step_s, 3),
                headline_spmm_one_core_tops=round(head_ops / single / 1e12, 5),
                sample=f"the headline L8-R8 SpMM (4096x4096, V=8, s=0.9, N=256) as the oracle computes it, {passes} passes "
                       "in about 10 s, best pass, including the oracle's dense / int32 operand preparation")


if __name__ == "__main__":
    main()
