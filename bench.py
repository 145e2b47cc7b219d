"""Benchmark of the V:N:M hot path on one MI355X.

Workload: the seven linear layers of one Llama-2-7B block at prefill (4096 tokens), pruned to 64:2:5,
synthetic weights and activations (see synth_inputs.py).  One step is one pass of the whole path over
that block: for every layer vnm_prune_compress (Section 3 pruning + Appendix A conversion, including
the matrix-core copy), vnm_spmm, vnm_decompress.  All inputs are resident in HBM before timing.

Prints ONE JSON line.  `value` is dense-equivalent TFLOP/s of the whole step (2*T*out*in summed over
the layers, divided by the step time, pruning and decompression included).  The `spmm` object holds
what the sparse product alone achieves and its speedup over the dense fp16 GEMM of the same shapes
(torch.matmul, i.e. hipBLASLt/rocBLAS); `roofline` prices the dominant kernel, vnm_spmm, by its
algorithmic flops on kept weights against the fp16 dense MFMA peak; `cpu_baseline` times the CPU
oracle on a bounded sample of the same workload.
"""

from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP16_DENSE_TFLOPS = 2500.0     # MI355X published dense fp16 MFMA peak


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama2_7b", choices=["llama2_7b", "deit_small", "deit_base", "single", "sweep"],
                    help="sweep: times vnm_spmm and vnm_prune_compress against the dense fp16 GEMM over the "
                         "V x M x tokens grid on the two large Llama shapes and runs the (V, M) selection on it")
    ap.add_argument("--V", type=int, default=None)
    ap.add_argument("--M", type=int, default=None)
    ap.add_argument("--tokens", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--spmm-only", action="store_true", help="time vnm_spmm alone (profiling aid)")
    ap.add_argument("--hot-path-only", action="store_true",
                    help="skip the sections after the timed region that run other kernels or other shapes "
                         "(RIA, fused layer, permutation search, few tokens): per-kernel profiler averages "
                         "then cover the timed workload only")
    return ap.parse_args()


def get_layers(args):
    import synth_inputs as syn
    if args.workload == "llama2_7b":
        kw = {}
        if args.V: kw["V"] = args.V
        if args.M: kw["M"] = args.M
        if args.tokens: kw["tokens"] = args.tokens
        return syn.config_llama2_7b(**kw)
    if args.workload == "deit_small":
        return syn.config_deit_small(args.V or 64, args.M or 5)
    if args.workload == "deit_base":
        return syn.config_deit_base(args.V or 64, args.M or 8)
    return syn.config_single_gemm()


def run_sweep(args):
    """V x M x tokens sweep (not the default workload): one JSON line with the table and, per token
    count, the (V, M) the two-phase sifting of Section 4.1 selects for a few speedup thresholds.
    A point's speedup is dense GEMM time / vnm_spmm time summed over the two layer shapes."""
    import torch
    import paper_2410_16135_amd as vnm
    import synth_inputs as syn
    dev = torch.device("cuda:0")

    def timed(f, n):
        for _ in range(3):
            f()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(n):
            f()
        b.record(); torch.cuda.synchronize()
        return a.elapsed_time(b) / n
    layers = syn.config_sweep()
    rows, cache = [], {}
    for L in layers:
        key = (L.out, L.inn)
        if key not in cache:
            W, _ = syn.layer_tensors(L, tokens=1)
            cache[key] = torch.from_numpy(W).to(dev)
        Wd = cache[key]
        _, X = syn.layer_tensors(L)
        Xd = torch.from_numpy(X).to(dev)
        Y = torch.empty((L.tokens, L.out), dtype=torch.float16, device=dev)
        c = vnm.vnm_prune_compress(Wd, L.V, L.M)
        n = max(args.steps, 5)
        t_sp = timed(lambda: vnm.vnm_spmm(Xd, c, Y=Y), n)
        t_de = timed(lambda: torch.matmul(Xd, Wd.t(), out=Y), n)
        t_pr = timed(lambda: vnm.vnm_prune_compress(Wd, L.V, L.M, out=c), 5)
        rows.append({"layer": L.name.split("_")[0], "out": L.out, "in": L.inn, "V": L.V, "M": L.M, "tokens": L.tokens,
                     "spmm_ms": round(t_sp, 4), "dense_fp16_ms": round(t_de, 4), "speedup": round(t_de / t_sp, 3),
                     "prune_compress_ms": round(t_pr, 4)})
    selection = {}
    for T in sorted({r["tokens"] for r in rows}):
        cands = []
        for V in sorted({r["V"] for r in rows}):
            for M in sorted({r["M"] for r in rows}):
                pts = [r for r in rows if r["tokens"] == T and r["V"] == V and r["M"] == M]
                cands.append((V, M, sum(r["dense_fp16_ms"] for r in pts) / sum(r["spmm_ms"] for r in pts)))
        sel = {}
        for s_thr in (1.0, 1.25, 1.5, 2.0, 2.5):
            i = vnm.vnm_select_vm(cands, s_thr)
            sel[str(s_thr)] = None if i < 0 else {"V": cands[i][0], "M": cands[i][1], "speedup": round(cands[i][2], 3),
                                                  "ln_K": vnm.vnm_mask_diversity_log(cands[i][0], cands[i][1])}
        selection[str(T)] = sel
    print(json.dumps({"metric": "V:N:M SpMM speedup vs dense fp16 GEMM, sweep", "unit": "x", "n_gpus": 1,
                      "data": "synthetic", "config": {"workload": "sweep V x M x tokens on 11008x4096 and 4096x11008"},
                      "points": rows, "selected_vm_by_threshold": selection}))


def L0_is_default(layers):
    L = layers[0]
    return L.V == 64 and L.M == 5 and L.tokens == 4096


def cpu_baseline(layers):
    """The oracle as it stands on the host cores: the whole path (prune + compress, decompress,
    masked-dense fp64 product) on every layer of the step, all tokens while that stays within
    about 10-30 s of host work (the Llama-shaped step takes under 10 s), else a token slice."""
    import numpy as np
    import synth_inputs as syn
    from oracle import vnm_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    dt, flops = 0.0, 0.0
    Tp = min(4096, layers[0].tokens)
    for layer in layers:
        W, X = syn.layer_tensors(layer, tokens=Tp)
        t0 = time.perf_counter()
        values, meta, colidx, mask = orc.compress(W, layer.V, layer.M)
        Wd = orc.decompress(values, meta, colidx, layer.out, layer.inn, layer.V, layer.M)
        Y = orc.matmul_ref(X, Wd)
        dt += time.perf_counter() - t0
        flops += 2.0 * Tp * layer.out * layer.inn
    L0 = layers[0]
    # the same on one thread, first layer only, 256 tokens (a few seconds)
    single = None
    try:
        from threadpoolctl import threadpool_limits
        T1 = min(256, L0.tokens)
        W, X = syn.layer_tensors(L0, tokens=T1)
        with threadpool_limits(limits=1):
            t0 = time.perf_counter()
            values, meta, colidx, mask = orc.compress(W, L0.V, L0.M)
            Wd = orc.decompress(values, meta, colidx, L0.out, L0.inn, L0.V, L0.M)
            Y = orc.matmul_ref(X, Wd)
            dt1 = time.perf_counter() - t0
        single = {"value": 2.0 * T1 * L0.out * L0.inn / dt1 / 1e12, "cores": 1, "seconds": dt1,
                  "sample": f"layer {L0.name} only, {T1} of {L0.tokens} tokens"}
    except Exception:
        pass
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s dense-equivalent", "cores": int(threads), "single_core": single,
            "kind": "oracle", "seconds": dt,
            "sample": f"all {len(layers)} layers of the step at {L0.V}:2:{L0.M}, whole path (prune+compress, "
                      f"decompress, fp64 masked-dense product), {Tp} of {L0.tokens} tokens"
                      + ("" if Tp == L0.tokens else "; the pruning part does not shrink with the token cut, "
                                                    "so the full-size figure is higher")}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU; run with --gpus 1 (no collectives or sharding exist here)",
              file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    import paper_2410_16135_amd as vnm
    import synth_inputs as syn

    if args.workload == "sweep":
        run_sweep(args)
        return
    dev = torch.device("cuda:0")
    layers = get_layers(args)
    # ---- resident inputs and preallocated outputs
    state = []
    x_cache = {}
    for L in layers:
        W, X = syn.layer_tensors(L)
        Wd = torch.from_numpy(W).to(dev)
        key = (L.inn, L.tokens, L.seed)
        Xd = torch.from_numpy(X).to(dev)
        c = vnm.vnm_prune_compress(Wd, L.V, L.M)                 # allocates the outputs once
        Y = torch.empty((L.tokens, L.out), dtype=torch.float16, device=dev)
        Wout = torch.empty_like(Wd)
        state.append((L, Wd, Xd, c, Y, Wout))
    ws_bytes = max(vnm.vnm_spmm_workspace_bytes(L.tokens, c) for (L, _, _, c, _, _) in state)
    staged = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)    # vnm_spmm's workspace, shared by all layers
    torch.cuda.synchronize()

    def ev():
        return torch.cuda.Event(enable_timing=True)

    def run_step(record, full):
        """One step.  record: list that receives (layer, events) or None.  full: events around every
        call (the untimed breakdown pass); otherwise only around the product kernel."""
        for (L, Wd, Xd, c, Y, Wout) in state:
            e = [ev() for _ in range(5)] if record is not None else None
            if not args.spmm_only:
                if e and full: e[0].record()
                vnm.vnm_prune_compress(Wd, L.V, L.M, out=c)
            if e and full: e[1].record()
            # vnm_spmm = staging pass + product kernel; issued as its two halves so that the
            # product kernel can be timed on its own (same kernels, same work as vnm_spmm)
            # (up to 32 tokens vnm_spmm is a single few-token kernel without a staging pass: it is
            # then called as such, and its whole time counts as the product)
            if L.tokens > 32:
                vnm.vnm_stage_x(Xd, L.M, staged=staged)
            if e: e[4].record()
            if L.tokens > 32:
                vnm.vnm_spmm_staged(staged, L.tokens, c, Y=Y)
            else:
                vnm.vnm_spmm(Xd, c, Y=Y, workspace=staged)
            if e: e[2].record()
            if not args.spmm_only:
                vnm.vnm_decompress(c, W_out=Wout)
                if e and full: e[3].record()
            if e: record.append((L, e))

    for _ in range(args.warmup):
        run_step(None, False)
    torch.cuda.synchronize()
    records = []
    t_begin = ev(); t_end = ev()
    wall0 = time.perf_counter()
    t_begin.record()
    for _ in range(args.steps):
        run_step(records, False)
    t_end.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - wall0
    step_ms = t_begin.elapsed_time(t_end) / args.steps
    # breakdown pass (after the timed region, not part of `value`): events around every call
    records_full = []
    for _ in range(max(3, min(args.steps, 10))):
        run_step(records_full, True)
    torch.cuda.synchronize()

    # ---- product-kernel times from the events inside the timed region; the other calls' times
    # from the breakdown pass
    per = {}
    for (L, e) in records:
        d = per.setdefault(L.name, {"prune_compress_ms": 0.0, "spmm_ms": 0.0, "decompress_ms": 0.0,
                                    "stage_ms": 0.0, "product_ms": 0.0, "n": 0, "nf": 0})
        d["product_ms"] += e[4].elapsed_time(e[2])
        d["n"] += 1
    for (L, e) in records_full:
        d = per[L.name]
        if not args.spmm_only:
            d["prune_compress_ms"] += e[0].elapsed_time(e[1])
            d["decompress_ms"] += e[2].elapsed_time(e[3])
        d["stage_ms"] += e[1].elapsed_time(e[4])
        d["nf"] += 1
    for d in per.values():
        d["product_ms"] /= d["n"]
        for k in ("prune_compress_ms", "decompress_ms", "stage_ms"):
            d[k] /= d["nf"]
        d["spmm_ms"] = d["stage_ms"] + d["product_ms"]

    # ---- dense fp16 baseline (same shapes, fp16 in / fp32 accumulate / fp16 out), timed the way the
    # sparse product is: one GEMM per layer and step, the layers in turn, so that every launch finds its
    # weight in HBM (a loop over one layer would re-read a weight that stays in the 256 MB last-level cache)
    dense_ms = {L.name: 0.0 for L in layers}
    n = max(10, args.steps)
    evs = []
    for it in range(3 + n):                      # all enqueued back to back, like the timed steps above
        for (L, Wd, Xd, c, Y, Wout) in state:
            e0, e1 = ev(), ev()
            e0.record()
            torch.matmul(Xd, Wd.t(), out=Y)
            e1.record()
            if it >= 3:
                evs.append((L, e0, e1))
    torch.cuda.synchronize()
    for (L, e0, e1) in evs:
        dense_ms[L.name] += e0.elapsed_time(e1) / n

    # one plain device-to-device copy of known size, so that profiler byte counters (FETCH_SIZE /
    # WRITE_SIZE) collected over this same command can be scaled against it
    L_c, Wd_c, _, _, _, Wout_c = state[0]
    Wout_c.copy_(Wd_c)
    torch.cuda.synchronize()
    calib_bytes = Wd_c.numel() * Wd_c.element_size()

    dense_equiv = sum(2.0 * L.tokens * L.out * L.inn for L in layers)
    kept = 0.0
    layer_rows = []
    for L in layers:
        s = vnm.vnm_query_sizes(L.out, L.inn, L.V, L.M)
        k = 2.0 * L.tokens * L.out * (2 * s.col_blocks)
        kept += k
        p = per[L.name]
        layer_rows.append({
            "layer": L.name, "out": L.out, "in": L.inn, "tokens": L.tokens,
            "spmm_ms": round(p["spmm_ms"], 4), "stage_ms": round(p["stage_ms"], 4),
            "product_ms": round(p["product_ms"], 4), "dense_fp16_ms": round(dense_ms[L.name], 4),
            "speedup_vs_dense_fp16": round(dense_ms[L.name] / p["spmm_ms"], 3),
            "spmm_dense_equiv_tflops": round(2.0 * L.tokens * L.out * L.inn / p["spmm_ms"] / 1e9, 1),
            "spmm_kept_tflops": round(k / p["spmm_ms"] / 1e9, 1),
            "prune_compress_ms": round(p["prune_compress_ms"], 4), "decompress_ms": round(p["decompress_ms"], 4)})
    spmm_ms = sum(per[L.name]["spmm_ms"] for L in layers)
    product_ms = sum(per[L.name]["product_ms"] for L in layers)
    stage_ms = sum(per[L.name]["stage_ms"] for L in layers)
    # HBM-side bytes per launch of the product kernel, mean over the 7 launches of a step, from the
    # rocprofv3 FETCH_SIZE / WRITE_SIZE runs summarised in profiles/ (scaled by the calibration
    # copy); known only for the default workload
    default_wl = (args.workload == "llama2_7b" and L0_is_default(layers))
    traffic = 347.1e6 if default_wl else None
    # matrix-core and LDS counters of the same kernel from the same profile (rocprofv3 --pmc, SQ block)
    counters = {"mfma_busy_percent": 42.4, "lds_active_percent_of_cu_busy": 47.1,
                "lds_bank_conflict_percent_of_lds_active": 31.6, "hbm_side_tb_per_s": 2.99,
                "source": "profiles/bench_llama2_7b_64-2-5_T4096.md"} if default_wl else None
    dense_total = sum(dense_ms[L.name] for L in layers)
    L0 = layers[0]
    result = {
        "metric": "V:N:M SpMM dense-equiv TFLOP/s + speedup vs dense fp16 GEMM at 64:2:5",
        "value": dense_equiv / step_ms / 1e9,
        "unit": "TFLOP/s dense-equivalent, whole path (prune+compress, spmm, decompress)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": step_ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"{args.workload} linear layers at {L0.V}:2:{L0.M}, tokens {L0.tokens}, "
                               f"{len(layers)} layers per step", "V": L0.V, "N": 2, "M": L0.M,
                   "tokens": L0.tokens, "spmm_only": bool(args.spmm_only)},
        "spmm": {"ms_per_step": spmm_ms, "stage_x_ms_per_step": stage_ms, "product_ms_per_step": product_ms, "dense_equiv_tflops": dense_equiv / spmm_ms / 1e9,
                 "kept_weight_tflops": kept / spmm_ms / 1e9,
                 "dense_equiv_frac_of_fp16_peak": dense_equiv / spmm_ms / 1e9 / PEAK_FP16_DENSE_TFLOPS,
                 "dense_fp16_gemm_ms": dense_total, "speedup_vs_dense_fp16": dense_total / spmm_ms,
                 "dense_baseline": "torch.matmul fp16 (hipBLASLt/rocBLAS), fp32 accumulate, fp16 out"},
        "roofline": {"bound": "mfma", "kernel": "spmm_smfmac_kernel",
                     "achieved": kept / product_ms / 1e9, "peak": PEAK_FP16_DENSE_TFLOPS, "unit": "TFLOP/s",
                     "frac": kept / product_ms / 1e9 / PEAK_FP16_DENSE_TFLOPS, "traffic": traffic,
                     "launches_per_step": len(layers), "avg_launch_us": product_ms / len(layers) * 1e3,
                     "flops_per_launch": kept / len(layers),
                     "dense_equiv_tflops": dense_equiv / product_ms / 1e9, "counters": counters,
                     "note": "per launch, mean over the launches of a step (one per layer): flops on kept weights "
                             "2*T*out*2*col_blocks / launch duration from HIP events around the product kernel "
                             "inside the timed region; peak = published dense fp16 MFMA rate; traffic = HBM-side "
                             "bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE scaled by a plain copy)"},
        "layers": layer_rows,
        "paper_context": "paper reports only end-to-end model speedups on RTX 3090 (Llama2-7B 64:2:5: 1.49x at "
                         "batch 1, 1.14x at batch 16; Appendix E) -- context, not a target",
        "host_wall_s": wall,
        "calibration_copy": {"bytes_read": calib_bytes, "bytes_written": calib_bytes,
                             "what": "one torch copy_ of the first layer's W after the timed region"},
    }
    if L0.tokens <= 32:
        # few tokens: the product is a stream of the packed weight, bound by HBM, not by the matrix cores
        packed_bytes = float(sum(c.packed.numel() for (_, _, _, c, _, _) in state))
        result["roofline"] = {
            "bound": "hbm", "kernel": "spmm_skinny_kernel / spmm_skinny_resident_kernel (+ splitk_reduce_kernel)",
            "achieved": packed_bytes / product_ms / 1e6, "peak": 8000.0, "unit": "GB/s",
            "frac": packed_bytes / product_ms / 1e6 / 8000.0, "traffic": None,
            "launches_per_step": len(layers), "avg_launch_us": product_ms / len(layers) * 1e3,
            "bytes_per_launch": packed_bytes / len(layers),
            "note": "per call of vnm_spmm, mean over the layers of a step: bytes of the packed weight (read once) / "
                    "duration from HIP events around the call inside the timed region; peak = published HBM rate"}
    if not args.spmm_only and not args.hot_path_only:
        # next row after the hot path (not part of `value`): RIA scores (Eq. 1) and pruning driven
        # by them, on the first layer; and the few-token product (decode) on the same layer
        L, Wd, Xd, c, Y, Wout = state[0]
        act = Xd.float().pow(2).sum(dim=0).sqrt().pow(0.5).contiguous()
        S = vnm.vnm_ria_scores(Wd, act)
        cs = vnm.vnm_prune_compress_scored(Wd, S, L.V, L.M)
        X16 = Xd[:16].contiguous()
        Y16 = torch.empty((16, L.out), dtype=torch.float16, device=dev)

        def timed(f, n=10, warm=1):
            for _ in range(warm):
                f()
            torch.cuda.synchronize()
            a, b = ev(), ev()
            a.record()
            for _ in range(n):
                f()
            b.record(); torch.cuda.synchronize()
            return a.elapsed_time(b) / n
        w_bytes = L.out * L.inn * 2
        t_ria = timed(lambda: vnm.vnm_ria_scores(Wd, act, S=S))
        t_ps = timed(lambda: vnm.vnm_prune_compress_scored(Wd, S, L.V, L.M, out=cs))
        t_16 = timed(lambda: vnm.vnm_spmm(X16, c, Y=Y16), n=30)
        t_16d = timed(lambda: torch.matmul(X16, Wd.t(), out=Y16), n=30)
        # fused layer of Section 4.2, Eq. 6: bias and run-time channel permutations around the product
        g = torch.Generator(device="cpu").manual_seed(7)
        p_in = torch.randperm(L.inn, generator=g).to(torch.int32).to(dev)
        p_out = torch.randperm(L.out, generator=g).to(torch.int32).to(dev)
        bias = torch.randn(L.out, generator=g).to(torch.float16).to(dev)
        # timed through the C ABI with the arguments marshalled once (the Python wrapper's per-call
        # overhead is of the order of these kernels' run time); 300 warm-up calls each: after a lighter phase the
        # first milliseconds of a heavy kernel run at a lower clock
        lib = vnm.load_library()
        nb = ctypes.c_int64(0)
        lib.vnm_spmm_fused_workspace_bytes(L.tokens, L.out, L.inn, L.V, 2, L.M, 1, ctypes.byref(nb))
        ws = torch.empty(nb.value, dtype=torch.uint8, device=dev)
        st = torch.cuda.current_stream().cuda_stream

        def fused(b, pi, po):
            args = (Xd.data_ptr(), L.tokens, Xd.stride(0), c.values.data_ptr(), c.meta.data_ptr(), c.colidx.data_ptr(),
                    c.packed.data_ptr(), L.out, L.inn, L.V, 2, L.M, b.data_ptr() if b is not None else None,
                    pi.data_ptr() if pi is not None else None, po.data_ptr() if po is not None else None,
                    Y.data_ptr(), Y.stride(0), 0, 0, ws.data_ptr(), ws.numel(), st)

            def run():
                rc = lib.vnm_spmm_fused(*args)
                assert rc == 0, rc
            return run
        t_plain = timed(fused(None, None, None), n=50, warm=300)
        t_bias = timed(fused(bias, None, None), n=50, warm=300)
        t_pin = timed(fused(bias, p_in, None), n=50, warm=300)
        t_all = timed(fused(bias, p_in, p_out), n=50, warm=300)
        result["fused_layer"] = {
            "layer": L.name, "spmm_ms": t_plain, "with_bias_ms": t_bias, "with_bias_perm_in_ms": t_pin,
            "with_bias_perm_in_perm_out_ms": t_all,
            "note": "vnm_spmm_fused on the first layer, HIP-event means; permutations folded into the "
                    "neighbouring layers cost nothing, these are the run-time fallbacks"}
        # mask refresh of the LoRA stage with dynamic masks (Eq. 10): merge B A into W, RIA scores, pruning
        r_lora = 16
        gB = torch.Generator(device="cpu").manual_seed(11)
        Bl = (torch.randn(L.out, r_lora, generator=gB) * 0.02).to(dev)
        Al = (torch.randn(r_lora, L.inn, generator=gB) * 0.02).to(dev)
        Wm = torch.empty_like(Wd)
        t_merge = timed(lambda: vnm.vnm_lora_merge(Wd, Bl, Al, 2.0, W_merged=Wm), n=20, warm=50)

        def refresh():
            vnm.vnm_lora_merge(Wd, Bl, Al, 2.0, W_merged=Wm)
            vnm.vnm_ria_scores(Wm, act, S=S)
            vnm.vnm_prune_compress_scored(Wm, S, L.V, L.M, out=cs)
        t_refresh = timed(refresh, n=20, warm=20)
        result["mask_refresh"] = {
            "layer": L.name, "lora_rank": r_lora, "merge_ms": t_merge, "merge_gbps": 2 * w_bytes / t_merge / 1e6,
            "merge_ria_prune_ms": t_refresh,
            "note": "vnm_lora_merge alone, and merge + RIA scores + pruning from scores (one mask update of one "
                    "layer); HIP-event means"}
        vnm.vnm_ria_scores(Wd, act, S=S)          # the search below uses the scores of the unmerged weight
        # channel-permutation search (Eqs. 7-9) on the first layer's RIA scores, one alternation
        sc = float(2 ** 30) / float(S.max().item())
        t0 = time.time()
        _, _, hist = vnm.vnm_permutation_search(S, L.V, L.M, sc, iterations=1)
        result["permutation_search"] = {
            "layer": L.name, "iterations": 1, "seconds": time.time() - t0,
            "objective": [int(h) for h in hist],
            "retained_gain_percent": 100.0 * float(hist[-1] - hist[0]) / float(hist[0]),
            "note": "wall time incl. the host assignment solver (5 problems of 819 x 819, 64 of 64 x 64), "
                    "which takes most of it; device kernels about 25 ms"}
        result["beyond_hot_path"] = {
            "layer": L.name, "ria_scores_ms": t_ria, "prune_compress_scored_ms": t_ps,
            "ria_scores_gbps": (2 * w_bytes + 2 * w_bytes) / t_ria / 1e6,
            "prune_compress_scored_gbps": (w_bytes + 2 * w_bytes) / t_ps / 1e6,
            "spmm_16_tokens_ms": t_16, "dense_16_tokens_ms": t_16d,
            "note": "HIP-event means including launch gaps; bytes counted: RIA reads W twice and writes fp32 "
                    "scores; scored pruning reads W and the scores"}
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(layers)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
