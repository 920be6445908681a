#!/usr/bin/env python3
"""Benchmark of the MEFT sparse-adapter layer on one MI355X.

A step is one pass of the whole hot path -- meft_route, meft_sparse_fwd, meft_sparse_bwd -- over
one batch of seeded synthetic input that is already resident in HBM.  The metric is
tokens/s = T / (t_route + t_fwd + t_bwd) for one layer.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config llama7b_bf16] [--no-cpu-baseline]

How the kernels are priced (per launch; T tokens, hidden size d, C = top_e * block_size candidates and
top_k selected neurons per token, P = T * top_k (token, neuron) pairs, U touched neurons, s bytes per element):
  * router and key-score contractions (Eq. 5, Eq. 6): matrix-core bound; flops are the method's own count,
    2 T n_blocks d and 2 T C d (Section 3.3), against the published dense bf16 peak;
  * the stages after the selection (Eq. 4 and the backward of Section 3.1): the method's own arithmetic is
    2 P d flop per stage, far below any matrix-core bound, so they are priced against HBM: `compulsory_bytes`
    = what has to cross HBM once whatever the kernel design (the operand rows read once, the result rows written
    once).  The block-dense kernels reach those stages' results through contractions over all C candidates;
    that padded count appears as `dense_equiv_TFLOP/s` and is never a roofline fraction;
  * `hbm_GB/s` = the kernel's real HBM traffic from the rocprofv3 FETCH_SIZE / WRITE_SIZE summary committed under
    profiles/ for the workload (source named in `roofline.traffic`), over the launch time measured here.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 MFMA, published
FP32_VALU_PEAK_TFLOPS = 157.3
TARGET_SCORE_GEMM_FRAC = 0.50   # scoring GEMMs: fraction of the bf16 matrix-core peak
TARGET_HBM_FRAC = 0.60          # gather / scatter stages: fraction of the HBM peak


def kernel_models(cfg, n_touched):
    """Per launch of each kernel: {"bound", "flop" (the method's own), "bytes" (compulsory HBM bytes),
    "dense_flop" (block-dense kernels: the padded contraction they execute)}."""
    s = 2 if cfg.dtype == "bf16" else 4
    T, d, k, C, B, N = cfg.T, cfg.d, cfg.top_k, cfg.C, cfg.n_blocks, cfg.N
    P = T * k
    U = n_touched
    act = T * d * s          # one activation-sized matrix: h, dOut, out, dh
    rows = U * d * s         # the touched rows of K, V, dK or dV
    pair = 2.0 * P * d       # flops of one stage after the selection
    dense = 2.0 * T * C * d
    m = {
        "router_gemm": dict(bound="mfma", flop=2.0 * T * B * d, bytes=act + B * d * s + T * B * 4),
        "score_gemm": dict(bound="mfma", flop=dense, bytes=act + N * d * s),
        "topk_select": dict(bound="hbm", flop=0.0, bytes=T * C * 4.0 + P * 8.0),
        # per-pair kernels: each pair moves one row per gathered matrix (no reuse across pairs is assumed)
        "gather_fwd": dict(bound="hbm", flop=pair, bytes=P * d * s + act + P * 8.0),
        "gather_bwd": dict(bound="hbm", flop=2 * pair, bytes=2.0 * P * d * s + 2.0 * act + P * 12.0),
        "seg_reduce": dict(bound="hbm", flop=2 * pair, bytes=2.0 * P * d * s + P * 12.0 + 2.0 * rows),
        # block-dense kernels: compulsory = operand rows once + result rows once
        "value_gemm": dict(bound="hbm", flop=pair, bytes=rows + P * 8.0 + act, dense_flop=dense),
        "dact_gemm": dict(bound="hbm", flop=pair, bytes=act + rows + P * 8.0, dense_flop=dense),
        "dh_gemm": dict(bound="hbm", flop=pair, bytes=rows + P * 4.0 + act, dense_flop=dense),
        "dV_gemm": dict(bound="hbm", flop=pair, bytes=act + P * 8.0 + rows, dense_flop=dense),
        "dK_gemm": dict(bound="hbm", flop=pair, bytes=act + P * 8.0 + rows, dense_flop=dense),
        # the sum of a token's per-block partial rows is part of the value / dh stage: its compulsory bytes are
        # already counted there (the partial rows themselves are traffic the design adds)
        "reduce_parts": dict(bound="hbm", flop=0.0, bytes=0.0),
    }
    # whole step: h, dOut, K, V read once; out, dh and the touched rows of dK, dV written once; idx / act both ways
    m["_step"] = dict(bound="hbm", flop=2.0 * T * B * d + dense + 5 * pair,
                      bytes=2.0 * act + 2.0 * N * d * s + 2.0 * act + 2.0 * rows + 2.0 * P * 8.0)
    return m


# profiler name of the kernel behind each stage label (the rocprofv3 summaries list kernels by symbol)
STAGE_SYMBOL = {
    "router_gemm": "gemm_mfma_kernel<ProbRouter, true>", "score_gemm": "gemm_mfma_kernel<ProbTokKC<0>, true>",
    "dact_gemm": "gemm_mfma_kernel<ProbTokKC<1>, true>", "value_gemm": "gemm_mfma_kernel<ProbTokNC, true>",
    "dh_gemm": "gemm_mfma_kernel<ProbTokNC, true>",
    # dV / dK: the tile height is chosen per shape (256 rows where the block fills them, else 128)
    "dV_gemm": ("gemm_mfma_kernel<ProbNeuTN<256>, true>", "gemm_mfma_kernel<ProbNeuTN<128>, true>"),
    "dK_gemm": ("gemm_mfma_kernel<ProbNeuTN<256>, true>", "gemm_mfma_kernel<ProbNeuTN<128>, true>"),
    "topk_select": ("topk_select_reg_kernel<16, true>", "topk_select_reg_kernel<32, true>", "topk_select_reg_kernel<4, true>"),
    "reduce_parts": "reduce_parts_kernel<2>",
}
GATHER_SCATTER = ("value_gemm", "dact_gemm", "dh_gemm", "dV_gemm", "dK_gemm", "gather_fwd", "gather_bwd", "seg_reduce")


def profiled_traffic(workload, stage):
    """HBM bytes per launch (read + written) of a stage's kernel, from the rocprofv3 FETCH_SIZE / WRITE_SIZE
    summary committed under profiles/ for this workload; None when there is no such summary."""
    path = os.path.join(ROOT, "profiles", f"{workload}_all_kernels.md")
    sym = STAGE_SYMBOL.get(stage)
    if sym is None or not os.path.exists(path):
        return None
    syms = (sym,) if isinstance(sym, str) else sym
    for line in open(path):
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) == 6 and cells[0] in syms:
            try:
                return {"read_bytes": float(cells[4]) * 1e6, "written_bytes": float(cells[5]) * 1e6,
                        "source": f"profiles/{workload}_all_kernels.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE)"}
            except ValueError:
                return None
    return None


def time_layer(layer, B, steps, warmup):
    """ms per step over `steps` steps after `warmup`, and the per-kernel averages of the same steps run once more
    with every kernel bracketed by HIP events on the launch stream."""
    import torch
    for _ in range(warmup):
        layer.step()
    torch.cuda.synchronize()
    w0 = time.perf_counter()
    for _ in range(steps):
        layer.step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - w0) * 1e3 / steps
    B.meft_profile_enable(True)
    for _ in range(steps):
        layer.step()
    torch.cuda.synchronize()
    prof = B.meft_profile_read()
    B.meft_profile_enable(False)
    kern = {name: ms / n for name, n, ms in prof}          # average ms per launch
    per_step = {name: ms / steps for name, n, ms in prof}
    return ms_per_step, kern, per_step


def price(cfg, models, name, launch_ms):
    """Roofline figures of one kernel launch."""
    m = models[name]
    d_s = launch_ms * 1e-3
    out = {}
    if m["bound"] == "mfma":
        peak = MFMA_BF16_PEAK_TFLOPS if cfg.dtype == "bf16" else FP32_VALU_PEAK_TFLOPS
        out["TFLOP/s"] = round(m["flop"] / d_s / 1e12, 2)
        out["frac_of_peak"] = round(m["flop"] / d_s / 1e12 / peak, 4)
    else:
        if m["flop"]:
            out["method_GFLOP"] = round(m["flop"] / 1e9, 2)
            out["method_TFLOP/s"] = round(m["flop"] / d_s / 1e12, 2)
        if m["bytes"]:
            out["compulsory_MB"] = round(m["bytes"] / 1e6, 1)
            out["compulsory_GB/s"] = round(m["bytes"] / d_s / 1e9, 1)
            out["frac_hbm_compulsory"] = round(m["bytes"] / d_s / 1e9 / HBM_PEAK_GBS, 4)
    if "dense_flop" in m:
        out["dense_equiv_TFLOP/s"] = round(m["dense_flop"] / d_s / 1e12, 2)
    tr = profiled_traffic(cfg.name, name)
    if tr is not None:
        gbs = (tr["read_bytes"] + tr["written_bytes"]) / d_s / 1e9
        out["hbm_GB/s"] = round(gbs, 1)
        out["frac_hbm_traffic"] = round(gbs / HBM_PEAK_GBS, 4)
    return out


def load_stats(layer):
    loads = layer.block_loads()
    return {"max": int(loads.max()), "mean": round(float(loads.mean()), 1), "min": int(loads.min()),
            "blocks_in_use": int((loads > 0).sum())}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="llama7b_bf16")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-tokens", type=int, default=8192)
    ap.add_argument("--verify", action="store_true", help="check structural invariants of one step first")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the measurements beside the headline metric (optimizer step, batch-union variant, the "
                         "other configurations); used for kernel profiles of the headline path alone")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (sharding the layer by token over several GPUs is described, "
              "not built). Run with --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2406_04984_amd import binding as B
    from paper_2406_04984_amd import synth
    from paper_2406_04984_amd.harness import DeviceLayer

    cfg = synth.CONFIGS[args.config]
    t0 = time.time()
    t = synth.make_inputs(cfg)
    layer = DeviceLayer(t, B)
    torch.cuda.synchronize()
    gen_s = time.time() - t0

    if args.verify:
        # one step checked against invariants that hold at any size, before anything is timed
        layer.fill_grad_sentinel()
        layer.step()
        torch.cuda.synchronize()
        nt = int(layer.n_touched.item())
        uniq = torch.unique(layer.idx)
        assert nt == uniq.numel() and torch.equal(layer.touched[:nt].long(), uniq), "touched != unique(idx)"
        assert bool((layer.idx[:, 1:] > layer.idx[:, :-1]).all()), "idx rows not strictly ascending"
        assert bool(torch.isfinite(layer.out.float()).all()) and bool(torch.isfinite(layer.dh.float()).all())
    ms_per_step, kern, per_step = time_layer(layer, B, args.steps, args.warmup)
    tokens_per_s = cfg.T / (ms_per_step * 1e-3)
    n_touched = int(layer.n_touched.item())

    # spread of single steps (the same K steps once more, each bracketed by events on the launch stream)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for a, b in evs:
        a.record()
        layer.step()
        b.record()
    torch.cuda.synchronize()
    single = sorted(a.elapsed_time(b) for a, b in evs)
    step_stats = {"median_ms": round(single[len(single) // 2], 4), "min_ms": round(single[0], 4),
                  "max_ms": round(single[-1], 4)}

    # streaming-copy probe: 1 GiB read + 1 GiB written per launch
    probe_bytes = 1 << 30
    pa = torch.empty((probe_bytes,), dtype=torch.uint8, device="cuda")
    pb = torch.empty((probe_bytes,), dtype=torch.uint8, device="cuda")
    for _ in range(2):
        B.meft_probe_copy(pb, pa, probe_bytes)
    B.meft_profile_enable(True)
    for _ in range(5):
        B.meft_probe_copy(pb, pa, probe_bytes)
    torch.cuda.synchronize()
    copy_ms = B.meft_profile_read()[0][2] / 5
    B.meft_profile_enable(False)
    copy_gbs = 2.0 * probe_bytes / (copy_ms * 1e-3) / 1e9
    del pa, pb

    # matrix-instruction probe: 1024 workgroups x 4 waves x 8 * 4096 instructions of 32768 flop (about 2.4 ms)
    probe_wgs, probe_iters = 1024, 4096
    pm = torch.empty((probe_wgs * 256,), dtype=torch.float32, device="cuda")
    for _ in range(2):
        B.meft_probe_mfma(pm, probe_wgs, probe_iters)
    B.meft_profile_enable(True)
    for _ in range(5):
        B.meft_probe_mfma(pm, probe_wgs, probe_iters)
    torch.cuda.synchronize()
    mfma_ms = B.meft_profile_read()[0][2] / 5
    B.meft_profile_enable(False)
    mfma_tflops = probe_wgs * 4 * 8.0 * probe_iters * 32768 / (mfma_ms * 1e-3) / 1e12
    del pm

    models = kernel_models(cfg, n_touched)
    priced = [k for k in per_step if k in models and (models[k]["bytes"] if models[k]["bound"] == "hbm" else models[k]["flop"])]
    dominant = max(priced, key=lambda k: per_step[k])
    m = models[dominant]
    dur_s = kern[dominant] * 1e-3
    if m["bound"] == "hbm":
        achieved, peak, runit, bound = m["bytes"] / dur_s / 1e9, HBM_PEAK_GBS, "GB/s", "hbm"
    else:
        achieved, runit = m["flop"] / dur_s / 1e12, "TFLOP/s"
        bound, peak = ("mfma", MFMA_BF16_PEAK_TFLOPS) if cfg.dtype == "bf16" else ("alu", FP32_VALU_PEAK_TFLOPS)
    roofline = {"kernel": dominant, "bound": bound, "achieved": round(achieved, 2), "peak": peak,
                "unit": runit, "frac": round(achieved / peak, 4),
                "traffic": profiled_traffic(cfg.name, dominant), "avg_launch_ms": round(kern[dominant], 4),
                "algorithmic": ("compulsory HBM bytes per launch: operand rows read once, result rows written once"
                                if bound == "hbm" else "the method's own flop count per launch"),
                "algorithmic_amount": m["bytes"] if bound == "hbm" else m["flop"]}
    tr = roofline["traffic"]
    if tr is not None and bound == "hbm":
        roofline["traffic_over_algorithmic"] = round((tr["read_bytes"] + tr["written_bytes"]) / m["bytes"], 3)
    # beside the published peak: what this machine's own probes reach (a loop of matrix instructions, a streaming copy)
    roofline["frac_of_measured_peak"] = round(achieved / (copy_gbs if bound == "hbm" else mfma_tflops), 4)
    if cfg.host_kv:
        # keys/values in pinned host memory: the step is bound by the host link.  Bytes: every block in use of K and
        # V goes host->device in the forward (and again in the backward unless the staged copies are kept), the
        # touched rows of dK and dV go back.
        used = int(torch.unique(layer.block_idx).numel())
        link_bytes = (2.0 if cfg.keep_staged else 4.0) * used * cfg.block_size * cfg.d * 2 + 2.0 * n_touched * cfg.d * 2
        gbs = link_bytes / (ms_per_step * 1e-3) / 1e9
        roofline = {"kernel": "host link: hipMemcpyAsync of K, V blocks + rows_to_host", "bound": "host_link",
                    "achieved": round(gbs, 2), "peak": 64.0, "unit": "GB/s", "frac": round(gbs / 64.0, 4),
                    "traffic": None, "note": "PCIe 5.0 x16, 64 GB/s per direction; whole-step bytes over step time"}
    stages = {}
    for name, ms in per_step.items():
        entry = {"ms_per_step": round(ms, 4)}
        if name in models:
            entry.update(price(cfg, models, name, kern[name]))
        stages[name] = entry
    step_model = models["_step"]
    whole_step = {"compulsory_MB": round(step_model["bytes"] / 1e6, 1),
                  "compulsory_GB/s": round(step_model["bytes"] / (ms_per_step * 1e-3) / 1e9, 1),
                  "frac_hbm_compulsory": round(step_model["bytes"] / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                  "method_GFLOP": round(step_model["flop"] / 1e9, 1),
                  "non_gemm_ms": round(sum(v for k_, v in per_step.items() if not k_.endswith("_gemm")), 4)}

    # the two fractions the task names as targets, on this run's kernel times
    targets = {}
    if "score_gemm" in kern and cfg.dtype == "bf16":
        fr = models["score_gemm"]["flop"] / (kern["score_gemm"] * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS
        targets["score_gemm_frac_of_mfma_peak"] = {"value": round(fr, 4), "target": TARGET_SCORE_GEMM_FRAC,
                                                   "met": bool(fr >= TARGET_SCORE_GEMM_FRAC)}
    gs = [n for n in GATHER_SCATTER if n in kern]
    if gs:
        comp = sum(models[n]["bytes"] for n in gs) / (sum(kern[n] for n in gs) * 1e-3) / 1e9 / HBM_PEAK_GBS
        targets["gather_scatter_frac_of_hbm_peak_compulsory_bytes"] = {
            "value": round(comp, 4), "target": TARGET_HBM_FRAC, "met": bool(comp >= TARGET_HBM_FRAC), "stages": gs}
        trs = [profiled_traffic(cfg.name, n) for n in gs]
        if all(x is not None for x in trs):
            real = sum(x["read_bytes"] + x["written_bytes"] for x in trs) / (sum(kern[n] for n in gs) * 1e-3) / 1e9
            targets["gather_scatter_frac_of_hbm_peak_counter_traffic"] = {
                "value": round(real / HBM_PEAK_GBS, 4), "target": TARGET_HBM_FRAC,
                "met": bool(real / HBM_PEAK_GBS >= TARGET_HBM_FRAC)}

    loads = load_stats(layer)

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import oracle
        n = min(cfg.T, args.cpu_sample_tokens)
        hs, gs_ = t.h[:n], t.dOut[:n]
        c0 = time.perf_counter()
        r = oracle.route(hs, t.Wg, cfg.top_e, t.bias)
        f = oracle.forward(hs, t.K, t.V, r.block_idx, cfg.block_size, cfg.top_k)
        rows = np.unique(f.idx)
        oracle.backward(hs, t.K, t.V, f.idx, f.score, gs_, cfg.block_size, rows=rows)
        c_s = time.perf_counter() - c0
        cpu = {"value": round(n / c_s, 2), "unit": "tokens/s", "cores": oracle.threads(), "kind": "oracle",
               "sample": f"first {n} of {cfg.T} tokens of {cfg.name}: route+fwd+bwd in {c_s:.2f} s, fp64, "
                         f"gradient rows of the {rows.size} neurons those tokens touch"}
        del r, f

    # Outside the headline metric: the optimizer step on the touched rows (row-sparse Adam with fp32 weights and
    # moments), timed per parameter matrix with HIP events; pure HBM traffic, reported against the HBM peak.
    extra = {}
    if not cfg.host_kv and not args.no_extras:
        esz = 2 if cfg.dtype == "bf16" else 4
        state = [torch.zeros(cfg.N, cfg.d, device="cuda") for _ in range(2)]
        master = layer.K.float()
        shape = layer.shape
        B.meft_profile_enable(True)
        reps = 5
        for i in range(reps):
            B.meft_adam_rows(shape, B.MeftAdam(1e-4, 0.9, 0.999, 1e-8, i + 1), layer.K, layer.dK, state[0], state[1],
                             master, layer.touched, layer.n_touched)
        torch.cuda.synchronize()
        ms = dict((n_, t_ / c_) for n_, c_, t_ in B.meft_profile_read()).get("adam_rows")
        B.meft_profile_enable(False)
        del state, master
        if ms:
            per_elem = esz + esz + 8 + 8 + 8      # gradient read, weight written, fp32 weight / m / v read and written
            nbytes = float(n_touched) * cfg.d * per_elem
            gbs = nbytes / (ms * 1e-3) / 1e9
            extra["adam_rows"] = {"ms_per_matrix": round(ms, 4), "rows": n_touched, "bytes_per_element": per_elem,
                                  "GB/s": round(gbs, 1), "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4)}

    # Host-resident keys and values: three layers' forwards one after the other, then with each layer's transfer
    # requested before the previous layer's forward is enqueued (the same inputs in every layer, a workspace each).
    if cfg.host_kv and not args.no_extras:
        n_layers = 3
        wss = [layer.ws] + [torch.empty_like(layer.ws) for _ in range(n_layers - 1)]
        pre = B.make_shape(cfg.T, cfg.d, cfg.n_blocks, cfg.block_size, cfg.top_e, cfg.top_k, cfg.dtype,
                           flags=B.MEFT_FLAG_HOST_KV | B.MEFT_FLAG_PRESTAGED)

        def fwd_plain(ws):
            B.meft_sparse_fwd(layer.shape, layer.h, layer.K, layer.V, layer.block_idx, layer.out, layer.idx, layer.act, ws)

        layer.route()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for ws in wss:
            fwd_plain(ws)
        torch.cuda.synchronize()
        seq_ms = (time.perf_counter() - t0) * 1e3 / n_layers
        t0 = time.perf_counter()
        B.meft_hostkv_stage(layer.shape, layer.block_idx, layer.K, layer.V, wss[0])
        for i, ws in enumerate(wss):
            if i + 1 < n_layers:
                B.meft_hostkv_stage(layer.shape, layer.block_idx, layer.K, layer.V, wss[i + 1])
            B.meft_sparse_fwd(pre, layer.h, layer.K, layer.V, layer.block_idx, layer.out, layer.idx, layer.act, ws)
        torch.cuda.synchronize()
        pipe_ms = (time.perf_counter() - t0) * 1e3 / n_layers
        extra["layer_pipeline"] = {"layers": n_layers, "fwd_ms_per_layer_one_after_the_other": round(seq_ms, 3),
                                   "fwd_ms_per_layer_pipelined": round(pipe_ms, 3)}
        del wss

    # The batch-union evaluation of Algorithm 1 on the same inputs and selections: every token over all of S.
    ubytes = B.meft_union_workspace_bytes(layer.shape)
    if ubytes > 0 and not cfg.host_kv and not args.no_extras:
        uws = torch.empty((ubytes,), dtype=torch.uint8, device="cuda")
        S = torch.empty_like(layer.touched)
        n_S = torch.zeros_like(layer.n_touched)
        uout = torch.empty_like(layer.out)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        for rep in range(2):   # the second repetition is the timed one
            ev[0].record()
            B.meft_union_fwd(layer.shape, layer.h, layer.K, layer.V, layer.idx, uout, S, n_S, uws)
            ev[1].record()
            B.meft_union_bwd(layer.shape, layer.h, layer.K, layer.V, S, n_S, layer.dOut, layer.dh, layer.dK, layer.dV,
                             uws)
            ev[2].record()
            torch.cuda.synchronize()
        nS = int(n_S.item())
        f_ms, b_ms = ev[0].elapsed_time(ev[1]), ev[1].elapsed_time(ev[2])
        flop = 2.0 * cfg.T * nS * cfg.d
        extra["union_variant"] = {"S": nS, "fwd_ms": round(f_ms, 3), "bwd_ms": round(b_ms, 3),
                                  "tokens/s": round(cfg.T / ((f_ms + b_ms) * 1e-3), 1),
                                  "fwd_TFLOP/s": round(2 * flop / (f_ms * 1e-3) / 1e12, 1),
                                  "bwd_TFLOP/s": round(5 * flop / (b_ms * 1e-3) / 1e12, 1),
                                  "note": "fwd = 2 contractions of 2*T*|S|*d flop, bwd = 5 (activations recomputed)"}
        del uws, uout

    # The benchmark's other device-resident configurations, in brief: step time, the dominant kernel with its
    # compulsory-bytes fraction, the scoring GEMM's fraction of the matrix-core peak, the realised block loads.
    other = {}
    if not args.no_extras and args.config == "llama7b_bf16":
        del layer, t
        torch.cuda.empty_cache()
        for name in ("small_bf16", "wide_bf16"):
            c2 = synth.CONFIGS[name]
            t2 = synth.make_inputs(c2)
            l2 = DeviceLayer(t2, B)
            ms2, kern2, per2 = time_layer(l2, B, max(5, args.steps // 2), max(3, args.warmup // 2))
            mod2 = kernel_models(c2, int(l2.n_touched.item()))
            dom2 = max((k for k in per2 if k in mod2 and (mod2[k]["bytes"] or mod2[k]["flop"])), key=lambda k: per2[k])
            entry = {"ms_per_step": round(ms2, 4), "tokens/s": round(c2.T / (ms2 * 1e-3), 1),
                     "dominant_kernel": dom2, "dominant": price(c2, mod2, dom2, kern2[dom2]),
                     "whole_step_frac_hbm_compulsory": round(mod2["_step"]["bytes"] / (ms2 * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                     "tokens_per_block": load_stats(l2),
                     "stage_ms": {k_: round(v, 4) for k_, v in per2.items()}}
            if "score_gemm" in kern2:
                entry["score_gemm"] = price(c2, mod2, "score_gemm", kern2["score_gemm"])
            other[name] = entry
            del l2, t2
            torch.cuda.empty_cache()

    line = {
        "metric": "sparse-adapter fwd+bwd tokens/sec per layer",
        "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "single_step": step_stats,
        "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "T": cfg.T, "d": cfg.d, "N": cfg.N, "n_blocks": cfg.n_blocks,
                   "block_size": cfg.block_size, "top_e": cfg.top_e, "top_k": cfg.top_k,
                   "inputs_resident_in_hbm": True, "input_generation_s": round(gen_s, 1)},
        "roofline": roofline, "cpu_baseline": cpu, "targets": targets, "whole_step": whole_step,
        "tokens_per_block": loads, "n_touched": n_touched, "stages": stages,
        "measured_copy_GB/s": round(copy_gbs, 1), "measured_mfma_TFLOP/s": round(mfma_tflops, 1),
        # 256 compute units x 4 matrix cores x 1024 flop per clock (a 32x32x16 bf16 instruction takes 32 clocks)
        "matrix_clock_GHz_implied_by_probe": round(mfma_tflops * 1e12 / (256 * 4 * 1024) / 1e9, 2),
        "other_configs": other, "beyond_the_metric": extra,
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
