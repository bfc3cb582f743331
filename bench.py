#!/usr/bin/env python3
"""Benchmark of the HDQT matmul path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--s S]

One step = the three matmuls of a training step of one layer (forward, input
gradient, weight gradient), each with its two Hadamard-domain quantizations,
its tiled integer matmul and its dequantization, on synthetic inputs already
resident in HBM.  Prints ONE JSON line:

  value       effective int TOPS of the whole step = 3 * 2MKN / step time
  roofline    the kernel that takes most of the step, priced against HBM
  cpu_baseline the CPU oracle timed on a bounded row slice of the same layer

Per-kernel durations are taken with HIP events recorded by the library around
every launch of the timed region (hdqt_profile_enable), on the launch stream.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "effective int TOPS of HDQT backward GEMMs (% int8 MFMA peak); FWHT-quant GB/s"
HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E
# HBM bytes per launch (fetch + write) of the default workload's kernels, from the
# rocprofv3 FETCH_SIZE / WRITE_SIZE runs summarised in
# profiles/bench_resnet_k1152_hbm_traffic.md (per-launch average over the tensors a
# kernel family runs on); bench.py cannot collect counters itself.
TRAFFIC_SOURCE = "profiles/bench_resnet_k1152_hbm_traffic.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, not measured in this run)"
VALU_SOURCE = "profiles/bench_resnet_k1152_valu_issue.md (rocprofv3 --pmc SQ_INSTS_VALU, not measured in this run)"
MEASURED_TRAFFIC = {
    "fwht_dual_absmax_batch": 336.4e6, "fwht_dual_quant_batch": 422.8e6,
    "gemm_i4_fwd": 74.6e6, "gemm_i4_bwd_input": 307.4e6, "gemm_i4_bwd_weight": 61.7e6,
}
# The kernels' sources as they were when those counters were collected: a SHA-256 over the
# files below, in this order.  The bench line says whether they have changed since (then the
# counter figures describe older kernels; re-collect them and update this value).
PROFILED_SOURCES = ("common.hpp", "lane_ops.hpp", "quantize_dual.hip", "gemm_fast.hip", "gemm.hip")
PROFILED_SOURCES_SHA256 = "d61d623a3722afde237781d0878c8f455e0c1fd4b64411869ecbec48fe330c32"


def profiled_sources_sha256():
    import hashlib
    h = hashlib.sha256()
    for f in PROFILED_SOURCES:
        with open(os.path.join(ROOT, "paper_2310_03675_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


INT8_MFMA_PEAK_TOPS = 5000.0    # MI355X dense int8
# Wave-wide vector-ALU instructions per launch of the two quantizer kernels on this workload
# (rocprofv3 --pmc SQ_INSTS_VALU, profiles/bench_resnet_k1152_valu_issue.md), and the chip's
# issue peak: one such instruction per SIMD every four cycles, 256 CUs x 4 SIMDs x 2.4 GHz / 4.
MEASURED_VALU_INSTS = {"fwht_dual_absmax_batch": 20.73e6, "fwht_dual_quant_batch": 39.24e6}
VALU_ISSUE_PEAK = 256 * 4 * 2.4e9 / 4

WORKLOADS = {
    # name: (constructor kwargs, Hadamard block)
    "resnet_k1152": dict(kind="resnet", batch=256, cin=128, cout=128, hw=16, n=64),
    "resnet_k576": dict(kind="resnet", batch=256, cin=64, cout=64, hw=32, n=64),
    "har": dict(kind="har", n=32),
    "fc": dict(kind="fc", n=16),
}


def make_layer(name, seed=0):
    from paper_2310_03675_amd import workloads
    w = WORKLOADS[name]
    if w["kind"] == "resnet":
        return workloads.resnet_conv_layer(w["batch"], w["cin"], w["cout"], w["hw"], seed=seed), w["n"]
    if w["kind"] == "har":
        return workloads.har_conv_layer(seed=seed), w["n"]
    return workloads.fc_layer(seed=seed), w["n"]


def step_params(B, kind, n, s, a=8, b=4):
    """G stochastic in both backward matmuls, everything else nearest."""
    NE, ST = B.ROUND_NEAREST, B.ROUND_STOCHASTIC
    tid = lambda role: {"X": 0, "W": 1, "G": 2}[role] + 4 * kind
    if kind == B.GEMM_FWD:
        A, Bq = B.Operand(b, NE, 1.0, tid("X")), B.Operand(b, NE, 1.0, tid("W"))
    elif kind == B.GEMM_BWD_INPUT:
        A, Bq = B.Operand(b, ST, 1.0, tid("G")), B.Operand(b, NE, 1.0, tid("W"))
    else:
        A, Bq = B.Operand(b, NE, 1.0, tid("X")), B.Operand(b, ST, 1.0, tid("G"))
    return B.Params(had_block=n, acc_bits=a, s=s, seed=0, A=A, B=Bq)


def cpu_baseline(layer, n, s, rows):
    """The oracle, as it stands, on the first `rows` rows of the layer (all three
    matmuls).  -> dict for the JSON line."""
    from oracle import capi
    X = layer.X[:rows].numpy()
    G = layer.G[:rows].numpy()
    W = layer.W.numpy()
    M, K, N = rows, layer.K, layer.N
    NE, ST = capi.ROUND_NEAREST, capi.ROUND_STOCHASTIC
    runs = [
        (capi.FWD, X, W, capi.Operand(4, NE, 1.0, 0), capi.Operand(4, NE, 1.0, 1)),
        (capi.BWD_INPUT, G, W, capi.Operand(4, ST, 1.0, 6), capi.Operand(4, NE, 1.0, 5)),
        (capi.BWD_WEIGHT, X, G, capi.Operand(4, NE, 1.0, 8), capi.Operand(4, ST, 1.0, 10)),
    ]
    capi.lib()
    t0 = time.perf_counter()
    for kind, P, Q, opA, opB in runs:
        capi.gemm(kind, P, Q, M, K, N, capi.Params(n, 8, s, 0, opA, opB), want_codes=False)
    dt = time.perf_counter() - t0
    ops = 3 * 2.0 * M * K * N
    return {"value": ops / dt / 1e12, "unit": "TOPS", "cores": capi.num_threads(), "kind": "oracle",
            "sample": f"first {rows} of {layer.M} rows of the layer, fwd + bwd_input + bwd_weight, "
                      f"{dt:.1f} s wall"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="resnet_k1152", choices=sorted(WORKLOADS))
    ap.add_argument("--s", type=int, default=32, help="tile length along the contraction")
    ap.add_argument("--acc-bits", type=int, default=8)
    ap.add_argument("--cpu-rows", type=int, default=65536, help="rows of the oracle's sample")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--dist-steps", type=int, default=100,
                    help="steps timed one by one (HIP events around each) for the median / min and the cold variant")
    ap.add_argument("--no-others", action="store_true",
                    help="skip the step lines of the other layer workloads ('other_workloads')")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step into a HIP graph and time its replays (measured: no faster than "
                         "launching from the host, the step is bound by its kernels)")
    ap.add_argument("--no-large-quantize", action="store_true",
                    help="skip the 1 GiB hdqt_quantize measurement ('quantize_1GiB')")
    ap.add_argument("--no-square", action="store_true",
                    help="skip the 4096^3 matmul measurement ('gemm_square_4096')")
    ap.add_argument("--no-conv", action="store_true",
                    help="skip the activation-source variant of the step ('conv_step')")
    ap.add_argument("--no-sweep", action="store_true",
                    help="skip the sweep of input and accumulator widths on the same layer")
    ap.add_argument("--no-resnet18", action="store_true",
                    help="skip the 21 layer shapes of a ResNet-18 step ('resnet18_batch128')")
    ap.add_argument("--no-fallbacks", action="store_true",
                    help="skip the timings of the paths behind the fast kernels' shape limits ('fallback_paths')")
    ap.add_argument("--no-requant", action="store_true",
                    help="skip the forward matmul under the second reading of the accumulator "
                         "(hdqt_gemm_requant, 'requant_fwd')")
    ap.add_argument("--requant", action="store_true", help="(accepted, the leg runs by default)")
    ap.add_argument("--separate", action="store_true",
                    help="run the step as the three per-matmul entry points instead of hdqt_layer_step")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (counter calibration for rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2310_03675_amd import binding as B

    B.load()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    layer, n = make_layer(args.workload)
    M, K, N = layer.M, layer.K, layer.N
    X, W, G = (t.to(dev) for t in (layer.X, layer.W, layer.G))
    kinds = [B.GEMM_FWD, B.GEMM_BWD_INPUT, B.GEMM_BWD_WEIGHT]
    prm = {k: step_params(B, k, n, args.s, args.acc_bits) for k in kinds}
    srcs = {B.GEMM_FWD: (X, W), B.GEMM_BWD_INPUT: (G, W), B.GEMM_BWD_WEIGHT: (X, G)}
    outs = {k: torch.empty(B.out_shape(k, M, K, N), dtype=torch.float32, device=dev) for k in kinds}
    if args.separate:
        ws_bytes = max(B.workspace_size(k, M, K, N, prm[k]) for k in kinds)
    else:
        ws_bytes = B.layer_step_workspace_size(M, K, N, *(prm[k] for k in kinds))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    step_out = tuple(outs[k] for k in kinds)

    def step():
        # (enqueued on torch's current stream: the capture stream while a graph is recorded)
        if args.separate:
            for k in kinds:
                B.gemm(k, srcs[k][0], srcs[k][1], M, K, N, prm[k], out=outs[k], workspace=ws)
        else:
            # Z, dX, dW bit-identical to the three calls above; X and G are read once
            # per quantization pass for both of their Hadamard domains
            B.layer_step(X, W, G, prm[kinds[0]], prm[kinds[1]], prm[kinds[2]], out=step_out,
                         workspace=ws)

    # One step is a fixed sequence of kernel launches (no host decisions, no memsets, no
    # allocation), so it can be captured once into a HIP graph and replayed; the replayed
    # step must reproduce the eagerly launched one bit for bit.
    run, launch = step, "eager"
    if args.graph:
        step()
        torch.cuda.synchronize()
        eager = [o.clone() for o in step_out]
        try:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                step()
            for _ in range(2):
                for o in step_out:
                    o.fill_(float("nan"))
                graph.replay()
                torch.cuda.synchronize()
                assert all(torch.equal(o, e) for o, e in zip(step_out, eager)), "graph replay differs"
            run, launch = graph.replay, "hip graph replay"
        except Exception as exc:            # capture unsupported: keep launching from the host
            print(f"bench.py: graph capture failed ({exc}); launching eagerly", file=sys.stderr)
            torch.cuda.synchronize()
        del eager

    if args.calib_copy:
        a = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        c = torch.empty_like(a)
        c.copy_(a)
        torch.cuda.synchronize()
        del a, c

    # ---- timed region: K steps, no instrumentation
    for _ in range(args.warmup):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    # ---- the distribution: --dist-steps steps timed one by one (an event pair around each, on
    # the stream the step is launched on), warm (back to back) and cold (a 512 MiB device fill
    # between steps, twice the 256 MB memory-side cache: nothing of the inputs, the workspace or
    # the previous step's outputs is left in any cache)
    def timed_one_by_one(count, flush):
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(count)]
        for a, b_ in ev:
            if flush is not None:
                flush.fill_(1)
            a.record()
            run()
            b_.record()
        torch.cuda.synchronize()
        ts = sorted(a.elapsed_time(b_) for a, b_ in ev)
        return {"steps": count, "median_ms": ts[len(ts) // 2], "min_ms": ts[0], "max_ms": ts[-1],
                "mean_ms": sum(ts) / len(ts)}
    step_dist = None
    if args.dist_steps > 0:
        step_dist = {"warm": timed_one_by_one(args.dist_steps, None)}
        flush_buf = torch.empty(512 << 20, dtype=torch.uint8, device=dev)
        step_dist["cold"] = timed_one_by_one(min(args.dist_steps, 100), flush_buf)
        step_dist["cold"]["flush"] = "512 MiB device fill before every step"
        del flush_buf

    # ---- the same K steps again with the library's per-kernel HIP events switched on
    # (two events per launch on the launch stream; they cost a few microseconds per
    # launch, which is why the figure above is taken without them)
    B.profile_enable(True)
    B.profile_collect()
    t1 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt_events = time.perf_counter() - t1
    B.profile_enable(False)
    kern = B.profile_collect()

    ms_per_step = dt / args.steps * 1e3
    ops_step = 3 * 2.0 * M * K * N
    value = ops_step / (dt / args.steps) / 1e12

    # ---- per-kernel table.  Algorithmic bytes / operations of one step, per kernel:
    #   absmax pass: 4 B read per element; quantize pass: 4 B read + 0.5 B written per axis;
    #   matmul: packed operands read once (0.5 B per code) + fp32 output written once,
    #   2*M*K*N operations each.
    elems = {"X": M * K, "W": K * N, "G": M * N}
    if args.separate:
        seen = {"fwht_row": ["X", "G", "W"],      # axis 1: X (fwd), G and W (bwd_input)
                "fwht_col": ["W", "X", "G"]}      # axis 0: W (fwd), X and G (bwd_weight)
    else:
        seen = {"fwht_dua": ["X", "W", "G"]}      # both axes of each tensor from one read per pass
    gemm_bytes = {"fwd": 0.5 * (M * K + K * N) + 4.0 * M * N,
                  "bwd_input": 0.5 * (M * N + K * N) + 4.0 * M * K,
                  "bwd_weight": 0.5 * (M * K + M * N) + 4.0 * K * N}
    measured = MEASURED_TRAFFIC if (args.workload == "resnet_k1152" and args.s == 32
                                    and args.acc_bits == 8 and not args.separate) else {}
    kernels, roof_all = {}, {}
    for name, (l, tot) in kern.items():
        avg_s = tot / l * 1e-3
        per_step = l / args.steps
        kernels[name] = {"launches_per_step": per_step, "avg_us": avg_s * 1e6,
                         "us_per_step": tot / args.steps * 1e3}
        fam = name[:8]
        if fam in seen:
            absmax = "absmax" in name
            per_elem = 4.0 if absmax else 4.0 + (1.0 if fam == "fwht_dua" else 0.5)
            # hdqt_layer_step names the tensor of each two-axis launch (..._X, _W, _G); one
            # launch finds the maxima of all three tensors, one writes the codes of X and W
            if name[-2:] in ("_X", "_W", "_G"):
                tensors = [name[-1]]
            elif name.endswith("_batch"):
                # G's codes come from the same launch unless it ran on its own
                tensors = ["X", "W"] if (not absmax and "fwht_dual_quant_G" in kern) else ["X", "W", "G"]
            else:
                tensors = seen[fam]
            bytes_launch = per_elem * sum(elems[t] for t in tensors) / per_step
            gbps = bytes_launch / avg_s / 1e9
            roof_all[name] = {"bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                              "frac": gbps / HBM_PEAK_GBPS, "traffic": measured.get(name),
                              "algorithmic_bytes_per_launch": bytes_launch}
            if measured and name in MEASURED_VALU_INSTS:
                # the same kernel against the vector ALU's instruction issue rate: pass 2 is
                # limited by it as much as by memory
                rate = MEASURED_VALU_INSTS[name] / avg_s
                roof_all[name]["valu_issue"] = {"wave_instructions_per_launch": MEASURED_VALU_INSTS[name],
                                                "achieved": rate / 1e9, "peak": VALU_ISSUE_PEAK / 1e9,
                                                "unit": "G wave-instructions/s", "frac": rate / VALU_ISSUE_PEAK}
        elif name.startswith("gemm_i4_"):
            which = name[len("gemm_i4_"):]
            tops = ops_step / 3 / avg_s / 1e12
            gbps = gemm_bytes[which] / avg_s / 1e9
            f_mfma, f_hbm = tops / INT8_MFMA_PEAK_TOPS, gbps / HBM_PEAK_GBPS
            # the roofline that binds is the one the kernel sits closer to
            if f_hbm >= f_mfma:
                roof_all[name] = {"bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                                  "frac": f_hbm, "traffic": measured.get(name),
                                  "algorithmic_bytes_per_launch": gemm_bytes[which], "mfma_TOPs": tops}
            else:
                roof_all[name] = {"bound": "mfma", "achieved": tops, "peak": INT8_MFMA_PEAK_TOPS,
                                  "unit": "TOP/s", "frac": f_mfma, "traffic": measured.get(name),
                                  "algorithmic_ops_per_launch": ops_step / 3, "hbm_GBps": gbps}
    try:
        counters_stale = profiled_sources_sha256() != PROFILED_SOURCES_SHA256
    except OSError:
        counters_stale = None          # sources not shipped next to the library
    if counters_stale:
        print("bench.py: the kernels' sources have changed since the rocprofv3 counters in profiles/ were "
              "collected; 'traffic' and 'valu_issue' describe the older kernels", file=sys.stderr)
    for r_ in roof_all.values():
        if r_.get("traffic") is not None:
            r_["traffic_source"] = TRAFFIC_SOURCE
            r_["traffic_sources_changed_since_profile"] = counters_stale
        if "valu_issue" in r_:
            r_["valu_issue"]["source"] = VALU_SOURCE
    dominant = max(roof_all, key=lambda k: kern[k][1])
    roofline = dict(roof_all[dominant], kernel=dominant)
    gemm_ms = sum(tot for name, (l, tot) in kern.items() if name.startswith("gemm") or name == "reduce_splits")
    gemm_tops = ops_step * args.steps / (gemm_ms * 1e-3) / 1e12 if gemm_ms else None
    quant_ms = sum(tot for name, (l, tot) in kern.items() if name.startswith("fwht"))
    quant_bytes = args.steps * sum(
        (4.0 + 4.0 + (1.0 if fam == "fwht_dua" else 0.5)) * elems[t] for fam, ts in seen.items() for t in ts)
    line = {
        "metric": METRIC, "value": value, "unit": "TOPS", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {layer.name} (M={M}, K={K}, N={N}), one training "
                               f"step = fwd + bwd_input + bwd_weight",
                   "entry": "3 x hdqt_gemm_*" if args.separate else "hdqt_layer_step",
                   "launch": launch,
                   "had_block": n, "input_bits": 4, "acc_bits": args.acc_bits, "s": args.s,
                   "rounding": "G stochastic, X and W nearest"},
        "roofline": roofline,
        "gemm": {"tops": gemm_tops, "frac_of_int8_mfma_peak": (gemm_tops or 0) / INT8_MFMA_PEAK_TOPS,
                 "us_per_step": gemm_ms / args.steps * 1e3},
        "fwht_quant_GBps": quant_bytes / (quant_ms * 1e-3) / 1e9 if quant_ms else None,
        "ms_per_step_with_kernel_events": dt_events / args.steps * 1e3,
        "step_time_distribution": step_dist,
        "kernels": kernels,
        "roofline_all": roof_all,
    }
    if not args.no_large_quantize:
        # The quantizer alone on a tensor far larger than any cache (1 GiB, b = 4, nearest):
        # per-pass HBM rate of hdqt_quantize, algorithmic bytes 4 B per element for pass 1 and
        # 4.5 B for pass 2.  Legs: contraction along a row (axis 1) and along a column (axis 0,
        # the transposing write), Hadamard block 64 (registers and lane exchanges only) and
        # 256 (axis 1: more lane stages; axis 0: the strip's 256 rows held whole in registers).
        big = torch.randn((16384, 16384), device=dev)
        op = B.Operand(4, B.ROUND_NEAREST, 1.0, 0)
        elems_big = 16384.0 * 16384.0
        line["quantize_1GiB"] = {}
        for axis_q, n_q in ((1, 64), (0, 64), (1, 256), (0, 256)):
            B.quantize(big, axis_q, n_q, op, 0)
            torch.cuda.synchronize()
            B.profile_enable(True)
            B.profile_collect()
            for _ in range(5):
                B.quantize(big, axis_q, n_q, op, 0)
            torch.cuda.synchronize()
            B.profile_enable(False)
            kq = B.profile_collect()
            k1 = [k_ for k_ in kq if k_.endswith("absmax")]
            k2 = [k_ for k_ in kq if k_.endswith("quant")]
            p1 = sum(kq[k_][1] for k_ in k1) / 5 * 1e-3
            p2 = sum(kq[k_][1] for k_ in k2) / 5 * 1e-3
            leg = {
                "kernels": sorted(kq),
                "pass1_GBps": 4.0 * elems_big / p1 / 1e9, "pass1_frac_of_hbm_peak": 4.0 * elems_big / p1 / 1e9 / HBM_PEAK_GBPS,
                "pass2_GBps": 4.5 * elems_big / p2 / 1e9, "pass2_frac_of_hbm_peak": 4.5 * elems_big / p2 / 1e9 / HBM_PEAK_GBPS,
                "both_GBps": 8.5 * elems_big / (p1 + p2) / 1e9}
            line["quantize_1GiB"][f"axis{axis_q}_n{n_q}"] = leg
        # (the figures of the first leg at the top level too, where earlier runs had them)
        line["quantize_1GiB"].update({k_: v_ for k_, v_ in line["quantize_1GiB"]["axis1_n64"].items() if k_ != "kernels"})
        # what a plain device-to-device copy of the same tensor reaches on this machine (PyTorch's
        # copy kernel, read + write): the streaming ceiling the fractions above can be held against
        dst_big = torch.empty_like(big)
        dst_big.copy_(big)
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record()
        for _ in range(5):
            dst_big.copy_(big)
        ev1.record()
        torch.cuda.synchronize()
        copy_gbps = 2.0 * 4.0 * elems_big / (ev0.elapsed_time(ev1) / 5 * 1e-3) / 1e9
        line["quantize_1GiB"]["device_copy_1GiB_GBps"] = copy_gbps
        for leg_ in ("axis1_n64", "axis0_n64", "axis1_n256", "axis0_n256"):
            line["quantize_1GiB"][leg_]["both_frac_of_device_copy"] = line["quantize_1GiB"][leg_]["both_GBps"] / copy_gbps
        del big, dst_big
    if not args.no_square:
        # The matrix pipe's own rate and the shader clock under that load, for three kinds of
        # operands (hdqt_probe_matrix_clock: independent MFMAs on fragments held in registers,
        # nothing else running): the rooflines above are priced at the published 2.4 GHz peak,
        # the chip's power management sets the clock by what the operands make the pipe switch.
        line["matrix_clock_probe"] = {}
        gen_p = torch.Generator(device="cpu").manual_seed(7)
        codes_p = torch.clamp(torch.round(torch.randn(8192, generator=gen_p) * 1.5), -8, 7).to(torch.int8)
        for kind_p, frag_p in (("zeros", torch.zeros(8192, dtype=torch.uint8)),
                               ("codes_times_16", (codes_p * 16).view(torch.uint8)),
                               ("random_bytes", torch.randint(0, 256, (8192,), generator=gen_p, dtype=torch.uint8))):
            line["matrix_clock_probe"][kind_p] = {f"{w_}_waves_per_simd": B.probe_matrix_clock(frag_p.to(dev), waves_per_simd=w_)
                                                  for w_ in (2, 4)}
        # The integer matmul alone where the matrix pipe is the roofline: 4096^3 on the codes
        # of the square sweep's operands (N(0,1) with 1 % outliers at +-20, Hadamard block 64,
        # 4-bit nearest), 8-bit accumulators, tiles of 32 and 64.
        from paper_2310_03675_amd import workloads
        sq = workloads.square_layer(4096, seed=0)
        opn = B.Operand(4, B.ROUND_NEAREST, 1.0, 0)
        qa, sa = B.quantize(sq.X.to(dev), 1, 64, opn, 0)
        qb, sb = B.quantize(sq.W.to(dev), 0, 64, opn, 0)
        o_sq = torch.empty((4096, 4096), dtype=torch.float32, device=dev)
        ws_sq = torch.empty(max(B.load().hdqt_gemm_codes_workspace_size(4096, 4096, 4096, 32), 256),
                            dtype=torch.uint8, device=dev)
        line["gemm_square_4096"] = {}
        for s_sq in (32, 64):
            for _ in range(3):
                B.gemm_codes(qa, qb, 4, 4, sa, sb, 4096, 64, 8, s_sq, want_acc=False, out=o_sq, workspace=ws_sq)
            torch.cuda.synchronize()
            B.profile_enable(True)
            B.profile_collect()
            for _ in range(10):
                B.gemm_codes(qa, qb, 4, 4, sa, sb, 4096, 64, 8, s_sq, want_acc=False, out=o_sq, workspace=ws_sq)
            torch.cuda.synchronize()
            B.profile_enable(False)
            kg = B.profile_collect()
            us = sum(v[1] for k_, v in kg.items() if k_.startswith("gemm") or k_ == "reduce_splits") * 1e3 / 10
            tops = 2.0 * 4096.0 ** 3 / us / 1e6
            line["gemm_square_4096"][f"s{s_sq}"] = {
                "us": us, "bound": "mfma", "achieved": tops, "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s",
                "frac": tops / INT8_MFMA_PEAK_TOPS}
        del sq, qa, qb, o_sq, ws_sq
        # and 8192^3, where the loop, not the tile boundaries, is what is measured:
        # tiles of 64 with 8-bit accumulators and tiles of 256 with 16-bit ones
        sq = workloads.square_layer(8192, seed=0)
        qa, sa = B.quantize(sq.X.to(dev), 1, 64, opn, 0)
        qb, sb = B.quantize(sq.W.to(dev), 0, 64, opn, 0)
        o_sq = torch.empty((8192, 8192), dtype=torch.float32, device=dev)
        line["gemm_square_8192"] = {}
        for s_sq, a_sq in ((64, 8), (256, 16)):
            for _ in range(2):
                B.gemm_codes(qa, qb, 4, 4, sa, sb, 8192, 64, a_sq, s_sq, want_acc=False, out=o_sq)
            torch.cuda.synchronize()
            B.profile_enable(True)
            B.profile_collect()
            for _ in range(5):
                B.gemm_codes(qa, qb, 4, 4, sa, sb, 8192, 64, a_sq, s_sq, want_acc=False, out=o_sq)
            torch.cuda.synchronize()
            B.profile_enable(False)
            kg = B.profile_collect()
            us = sum(v[1] for k_, v in kg.items() if k_.startswith("gemm")) * 1e3 / 5
            tops = 2.0 * 8192.0 ** 3 / us / 1e6
            line["gemm_square_8192"][f"s{s_sq}_a{a_sq}"] = {
                "us": us, "bound": "mfma", "achieved": tops, "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s",
                "frac": tops / INT8_MFMA_PEAK_TOPS}
        del sq, qa, qb, o_sq
        # The input gradient with its output narrowed to bfloat16 (hdqt_gemm_codes_bf16 on the
        # layer's own codes): the fp32 matmul is bound by the 4*M*K bytes it writes, this one
        # writes half of them.  Not part of `value`: the step hands fp32 on, as the paper does.
        opg = B.Operand(4, B.ROUND_STOCHASTIC, 1.0, 6)
        qg, sg = B.quantize(G, 1, n, opg, 0)
        qw, sw = B.quantize(W, 1, n, opn, 0)
        line["bwd_input_bf16"] = {}
        for tag, bf in (("fp32", False), ("bf16", True)):
            o_dx = torch.empty((M, K), dtype=torch.bfloat16 if bf else torch.float32, device=dev)
            for _ in range(3):
                B.gemm_codes(qg, qw, 4, 4, sg, sw, N, n, args.acc_bits, args.s, want_acc=False, out=o_dx, bf16=bf)
            torch.cuda.synchronize()
            B.profile_enable(True)
            B.profile_collect()
            for _ in range(10):
                B.gemm_codes(qg, qw, 4, 4, sg, sw, N, n, args.acc_bits, args.s, want_acc=False, out=o_dx, bf16=bf)
            torch.cuda.synchronize()
            B.profile_enable(False)
            kg = B.profile_collect()
            us = sum(v[1] for k_, v in kg.items() if k_.startswith("gemm")) * 1e3 / 10
            nbytes = 0.5 * (M * N + K * N) + (2.0 if bf else 4.0) * M * K
            line["bwd_input_bf16"][tag] = {"us": us, "bound": "hbm", "achieved": nbytes / us / 1e3,
                                           "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                                           "frac": nbytes / us / 1e3 / HBM_PEAK_GBPS,
                                           "algorithmic_bytes_per_launch": nbytes}
            del o_dx
        # The input gradient behind a rectifier (hdqt_gemm_bwd_input_masked's kernel): dX written
        # where the layer's input is positive, zero elsewhere; reads X once more (4*M*K bytes)
        # where a framework's own pass over dX reads dX and X and writes dX again.
        try:
            ws_m = torch.empty(B.workspace_size(B.GEMM_BWD_INPUT, M, K, N, prm[B.GEMM_BWD_INPUT]), dtype=torch.uint8, device=dev)
            o_dx = torch.empty((M, K), dtype=torch.float32, device=dev)
            f_m = lambda: B.gemm(B.GEMM_BWD_INPUT, G, W, M, K, N, prm[B.GEMM_BWD_INPUT], out=o_dx, workspace=ws_m, mask=X)
            for _ in range(3):
                f_m()
            torch.cuda.synchronize()
            B.profile_enable(True)
            B.profile_collect()
            for _ in range(10):
                f_m()
            torch.cuda.synchronize()
            B.profile_enable(False)
            kg = B.profile_collect()
            us = sum(v[1] for k_, v in kg.items() if k_.startswith("gemm") or k_ == "relu_mask") * 1e3 / 10
            nbytes = 0.5 * (M * N + K * N) + 8.0 * M * K
            line["bwd_input_bf16"]["relu_masked_fp32"] = {
                "us": us, "bound": "hbm", "achieved": nbytes / us / 1e3, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": nbytes / us / 1e3 / HBM_PEAK_GBPS, "algorithmic_bytes_per_launch": nbytes}
            del ws_m, o_dx
        except B.HdqtError as exc:
            line["bwd_input_bf16"]["relu_masked_fp32"] = {"skipped": str(exc)}
        if layer.act is not None:
            # and with the gradient folded back onto the convolution's input inside the matmul
            # (hdqt_gemm_codes_fold): what is written is the activation's gradient, kh*kw times
            # smaller than the gradient of the im2col matrix
            kh_, kw_ = layer.window
            shape_ = tuple(layer.act.shape)
            try:
                o_act = torch.empty(shape_, dtype=torch.float32, device=dev)
                for _ in range(3):
                    B.gemm_codes_fold(qg, qw, 4, 4, sg, sw, shape_, kh_, kw_, n, args.acc_bits, args.s, out=o_act)
                torch.cuda.synchronize()
                B.profile_enable(True)
                B.profile_collect()
                for _ in range(10):
                    B.gemm_codes_fold(qg, qw, 4, 4, sg, sw, shape_, kh_, kw_, n, args.acc_bits, args.s, out=o_act)
                torch.cuda.synchronize()
                B.profile_enable(False)
                kg = B.profile_collect()
                us = sum(v[1] for k_, v in kg.items() if k_.startswith("gemm")) * 1e3 / 10
                nbytes = 0.5 * (M * N + K * N) + 4.0 * o_act.numel()
                line["bwd_input_bf16"]["folded_fp32"] = {
                    "us": us, "bound": "hbm", "achieved": nbytes / us / 1e3, "peak": HBM_PEAK_GBPS,
                    "unit": "GB/s", "frac": nbytes / us / 1e3 / HBM_PEAK_GBPS,
                    "algorithmic_bytes_per_launch": nbytes}
                del o_act
            except B.HdqtError as exc:
                line["bwd_input_bf16"]["folded_fp32"] = {"skipped": str(exc)}
        del qg, qw
    if layer.act is not None and not args.no_conv and not args.separate:
        # The same step with X given as the convolution's input (hdqt_conv_step): the quantizer
        # reads the activation, kh*kw times smaller than its im2col matrix, and the outputs
        # are bit for bit those of the step above.  Not `value`: the benchmark's workload
        # hands the matrix over; this is what a convolution layer can call instead.
        act_d = layer.act.to(dev)
        kh_, kw_ = layer.window
        try:
            ws_c = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
            conv = lambda: B.conv_step(act_d, kh_, kw_, W, G, prm[kinds[0]], prm[kinds[1]], prm[kinds[2]],
                                       out=step_out, workspace=ws_c)
            ref = [o.clone() for o in step_out]
            conv()
            torch.cuda.synchronize()
            same = all(torch.equal(o, r) for o, r in zip(step_out, ref))
            for _ in range(args.warmup):
                conv()
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for _ in range(args.steps):
                conv()
            torch.cuda.synchronize()
            dt_c = (time.perf_counter() - t1) / args.steps
            B.profile_enable(True)
            B.profile_collect()
            for _ in range(args.steps):
                conv()
            torch.cuda.synchronize()
            B.profile_enable(False)
            kc = B.profile_collect()
            line["conv_step"] = {
                "entry": "hdqt_conv_step", "ms_per_step": dt_c * 1e3, "TOPS": ops_step / dt_c / 1e12,
                "outputs_equal_layer_step": same,
                "activation_bytes": 4.0 * act_d.numel(), "im2col_matrix_bytes": 4.0 * M * K,
                "kernels_us": {n_: tot / l * 1e3 for n_, (l, tot) in kc.items()}}
            # the whole layer from its input to its input's gradient: hdqt_conv_fwd + hdqt_conv_bwd
            # (the gradient folded back inside the matmul), against what the matrix path needs
            # around it: PyTorch's unfold before and fold after
            try:
                pf_, pi_, pw_ = prm[kinds[0]], prm[kinds[1]], prm[kinds[2]]
                def whole():
                    _, sv = B.conv_fwd(act_d, kh_, kw_, W, pf_, pw_)
                    B.conv_bwd(G, W, sv, tuple(act_d.shape), kh_, kw_, pi_, pw_)
                def glue():
                    xs = torch.nn.functional.unfold(act_d, (kh_, kw_), padding=((kh_ - 1) // 2, (kw_ - 1) // 2))
                    xs = xs.transpose(1, 2).reshape(M, K).contiguous()
                    torch.nn.functional.fold(step_out[1].reshape(act_d.shape[0], -1, K).transpose(1, 2),
                                             output_size=tuple(act_d.shape[2:]), kernel_size=(kh_, kw_),
                                             padding=((kh_ - 1) // 2, (kw_ - 1) // 2))
                for name_, fn_ in (("conv_fwd_plus_conv_bwd_ms", whole), ("pytorch_unfold_plus_fold_ms", glue)):
                    for _ in range(3):
                        fn_()
                    torch.cuda.synchronize()
                    t1 = time.perf_counter()
                    for _ in range(10):
                        fn_()
                    torch.cuda.synchronize()
                    line["conv_step"][name_] = (time.perf_counter() - t1) / 10 * 1e3
            except B.HdqtError as exc:
                line["conv_step"]["conv_bwd"] = f"skipped: {exc}"
            del ws_c, ref
        except B.HdqtError as exc:          # geometry the activation-source kernels do not take
            line["conv_step"] = {"skipped": str(exc)}
        del act_d
    if not args.no_sweep and not args.separate:
        # The same step over the input and accumulator widths of the paper's Fig. 4 (inputs of
        # 3 to 8 bits, accumulators of 8 to 32): wall time per step and the rate at the
        # headline metric's operation count.  Not `value`: that is the 4-bit / 8-bit point.
        line["width_sweep"] = {"unit": "ms_per_step", "s": args.s}
        for b_in, a_acc in ((3, 8), (4, 8), (4, 10), (4, 12), (4, 16), (5, 12), (6, 12), (6, 16), (8, 16), (8, 32)):
            prm_w = [step_params(B, k, n, args.s, a_acc, b_in) for k in kinds]
            ws_w = torch.empty(B.layer_step_workspace_size(M, K, N, *prm_w), dtype=torch.uint8, device=dev)
            for _ in range(3):
                B.layer_step(X, W, G, *prm_w, out=step_out, workspace=ws_w)
            torch.cuda.synchronize()
            t_w = time.perf_counter()
            for _ in range(10):
                B.layer_step(X, W, G, *prm_w, out=step_out, workspace=ws_w)
            torch.cuda.synchronize()
            ms_w = (time.perf_counter() - t_w) / 10 * 1e3
            line["width_sweep"][f"b{b_in}_a{a_acc}"] = {"ms": ms_w, "TOPS": 3 * 2.0 * M * K * N / (ms_w * 1e-3) / 1e12}
            del ws_w
    if not args.no_requant and not args.separate:
        k = kinds[0]
        need = B.load().hdqt_gemm_requant_workspace_size(k, M, K, N, prm[k].c())
        ws2 = torch.empty(need, dtype=torch.uint8, device=dev)
        for _ in range(2):
            B.gemm_requant(k, X, W, M, K, N, prm[k], workspace=ws2)
        torch.cuda.synchronize()
        B.profile_enable(True)
        B.profile_collect()
        t2 = time.perf_counter()
        for _ in range(20):
            B.gemm_requant(k, X, W, M, K, N, prm[k], workspace=ws2)
        torch.cuda.synchronize()
        dt2 = (time.perf_counter() - t2) / 20
        B.profile_enable(False)
        kern2 = B.profile_collect()
        tiles = (K + args.s - 1) // args.s
        kus = {n_: tot / l * 1e3 for n_, (l, tot) in kern2.items()}
        line["requant_fwd"] = {
            # the whole call from the fp32 tensors (quantization of X and W included), and the
            # matmul's own launches: pass 1 (tile maxima), pass 2 (quantize and add the tile sums)
            "ms": dt2 * 1e3, "tiles": tiles, "workspace_bytes": need,
            "tile_sums_materialised_bytes": 0 if need < 4.0 * tiles * M * N else 4.0 * tiles * M * N,
            "kernels_us": kus,
            "matmul_us": sum(v for n_, v in kus.items() if n_.startswith("requant") or n_ == "reduce"),
            "matmul_TOPs_two_passes": 2 * 2.0 * M * K * N / (sum(v for n_, v in kus.items() if n_.startswith("requant")) * 1e-6) / 1e12}
        del ws2
    if not args.no_others and not args.separate:
        # One step of the other layer workloads (not `value`): the HAR-style 1-D convolution layer
        # and the 32 x 32 ResNet layer, each with its own Hadamard block, tile length = block
        # for the first (as its configuration says) and the headline's tile length for the second.
        line["other_workloads"] = {}
        for name_o, s_o in (("har", 32), ("resnet_k576", args.s)):
            lay_o, n_o = make_layer(name_o)
            Mo, Ko, No = lay_o.M, lay_o.K, lay_o.N
            Xo, Wo, Go = (t.to(dev) for t in (lay_o.X, lay_o.W, lay_o.G))
            prm_o = [step_params(B, k, n_o, s_o, args.acc_bits) for k in kinds]
            ws_o = torch.empty(B.layer_step_workspace_size(Mo, Ko, No, *prm_o), dtype=torch.uint8, device=dev)
            out_o = tuple(torch.empty(B.out_shape(k, Mo, Ko, No), dtype=torch.float32, device=dev) for k in kinds)
            f_o = lambda: B.layer_step(Xo, Wo, Go, *prm_o, out=out_o, workspace=ws_o)
            for _ in range(args.warmup):
                f_o()
            torch.cuda.synchronize()
            t_o = time.perf_counter()
            for _ in range(args.steps):
                f_o()
            torch.cuda.synchronize()
            dt_o = (time.perf_counter() - t_o) / args.steps
            B.profile_enable(True)
            B.profile_collect()
            for _ in range(args.steps):
                f_o()
            torch.cuda.synchronize()
            B.profile_enable(False)
            k_o = B.profile_collect()
            line["other_workloads"][name_o] = {
                "workload": f"{lay_o.name} (M={Mo}, K={Ko}, N={No})", "had_block": n_o, "s": s_o,
                "ms_per_step": dt_o * 1e3, "TOPS": 3 * 2.0 * Mo * Ko * No / dt_o / 1e12,
                "algorithmic_bytes_per_step": 8.0 * (Mo * Ko + Ko * No + Mo * No) + 2.0 * (Mo * Ko + Ko * No + Mo * No)
                                              + 4.0 * (Mo * No + Mo * Ko + Ko * No),
                "kernels_us": {n_: tot / l * 1e3 for n_, (l, tot) in k_o.items()}}
            del Xo, Wo, Go, ws_o, out_o, lay_o
    if not args.no_resnet18 and not args.separate:
        # The 21 matmul layers of a CIFAR-width ResNet-18 at batch 128, each as one hdqt_layer_step
        # on synthetic tensors of its shape (ReLU-like activations, Kaiming weights, small Gaussian
        # gradients; the first layer's input gradient, which training does not need, is left out):
        # time per layer shape, and the whole network's matmul time per training step (not `value`).
        from paper_2310_03675_amd import workloads as wl18
        per_shape, net_ms, net_ops = {}, 0.0, 0.0
        table = wl18.resnet18_layer_table(128)
        for name_l, Ml, Kl, Nl in table:
            key = f"{Ml}x{Kl}x{Nl}"
            with_dx = name_l != "stem"
            if key not in per_shape:
                g18 = torch.Generator(device="cpu").manual_seed(18 + len(per_shape))
                Xl = torch.relu(torch.randn((Ml, Kl), generator=g18)).to(dev)
                Wl = (torch.randn((Kl, Nl), generator=g18) * (2.0 / Kl) ** 0.5).to(dev)
                Gl = (torch.randn((Ml, Nl), generator=g18) * 1e-2).to(dev)
                p18 = [step_params(B, k, 64, args.s, args.acc_bits) for k in kinds]
                p_in = p18[kinds.index(B.GEMM_BWD_INPUT)] if with_dx else None
                p_fw, p_bw = p18[kinds.index(B.GEMM_FWD)], p18[kinds.index(B.GEMM_BWD_WEIGHT)]
                Zl, dXl, dWl, wsl = B.layer_step(Xl, Wl, Gl, p_fw, p_in, p_bw)
                f18 = lambda: B.layer_step(Xl, Wl, Gl, p_fw, p_in, p_bw, out=(Zl, dXl, dWl), workspace=wsl)
                for _ in range(3):
                    f18()
                torch.cuda.synchronize()
                t18 = time.perf_counter()
                for _ in range(20):
                    f18()
                torch.cuda.synchronize()
                ms18 = (time.perf_counter() - t18) / 20 * 1e3
                ops18 = (3 if with_dx else 2) * 2.0 * Ml * Kl * Nl
                per_shape[key] = {"ms_per_step": ms18, "TOPS": ops18 / (ms18 * 1e-3) / 1e12, "layers": 0,
                                  "matmuls": 3 if with_dx else 2}
                del Xl, Wl, Gl, Zl, dXl, dWl, wsl
            per_shape[key]["layers"] += 1
            net_ms += per_shape[key]["ms_per_step"]
            net_ops += per_shape[key]["TOPS"] * per_shape[key]["ms_per_step"] * 1e9
        line["resnet18_batch128"] = {"layers": len(table), "matmul_ms_per_training_step": net_ms,
                                     "GOP_per_training_step": net_ops / 1e9,
                                     "TOPS": net_ops / (net_ms * 1e-3) / 1e12, "per_shape": per_shape}
    if not args.no_fallbacks and not args.separate:
        # The paths behind the fast kernels' shape limits, each on the benchmark layer's forward
        # operands changed just enough to leave the fast path (not `value`; these paths have
        # parity tests and otherwise no figure anywhere).
        def timed(fn, reps=10):
            fn()
            torch.cuda.synchronize()
            B.profile_enable(True)
            B.profile_collect()
            t_f = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            dt_f = (time.perf_counter() - t_f) / reps
            B.profile_enable(False)
            return dt_f, {n_: tot / l * 1e3 for n_, (l, tot) in B.profile_collect().items()}
        fb = {}
        pf = prm[kinds[0]]
        # contraction lengths that are no multiple of 32: a multiple of 8 still runs the matrix-core
        # kernel (the rows' last 16-byte unit is padded with zeros on its way to LDS), anything else
        # the generic tiled kernel
        for key, Kf in (("fwd_K_multiple_of_8_not_32", K - 8), ("fwd_K_not_multiple_of_8", K - 4)):
            Xf, Wf = X[:, :Kf].contiguous(), W[:Kf].contiguous()
            dt_f, k_f = timed(lambda: B.gemm(kinds[0], Xf, Wf, M, Kf, N, pf))
            fb[key] = {"shape": [M, Kf, N], "ms": dt_f * 1e3, "kernels_us": k_f, "TOPS": 2.0 * M * Kf * N / dt_f / 1e12}
        # 4-bit activations against 8-bit weights: packed codes on one side, a byte per code on the other
        pm = B.Params(had_block=n, acc_bits=16, s=args.s, seed=pf.seed, A=pf.A,
                      B=B.Operand(8, pf.B.round, pf.B.clip, pf.B.tensor_id))
        dt_f, k_f = timed(lambda: B.gemm(kinds[0], X, W, M, K, N, pm))
        fb["fwd_mixed_4bit_8bit"] = {"shape": [M, K, N], "ms": dt_f * 1e3, "kernels_us": k_f,
                                    "TOPS": 2.0 * M * K * N / dt_f / 1e12}
        # axis-0 quantization of a tensor whose column count is no multiple of 4 (generic column kernel)
        Xq = X[:, :K - 2].contiguous()
        dt_f, k_f = timed(lambda: B.quantize(Xq, 0, n, pf.A, 0))
        fb["quantize_axis0_cols_not_multiple_of_4"] = {
            "shape": [M, K - 2], "ms": dt_f * 1e3, "kernels_us": k_f,
            "GBps": 8.5 * M * (K - 2) / dt_f / 1e9}
        # a step with Hadamard blocks of 128: beyond the two-axis kernels, each axis of each tensor
        # is a pass of the single-axis kernels
        prm_f = [step_params(B, k, 128, args.s, args.acc_bits) for k in kinds]
        ws_f = torch.empty(B.layer_step_workspace_size(M, K, N, *prm_f), dtype=torch.uint8, device=dev)
        dt_f, k_f = timed(lambda: B.layer_step(X, W, G, *prm_f, out=step_out, workspace=ws_f))
        fb["step_had_block_128"] = {"ms": dt_f * 1e3, "kernels_us": k_f, "TOPS": ops_step / dt_f / 1e12}
        line["fallback_paths"] = fb
        del Xf, Wf, Xq, ws_f
        # The matmul's test of its tiles (tiles of 32, 8-bit accumulators: a tile whose sums
        # provably stay in range is not clamped) depends on the codes, not on the shape: the
        # forward product's launch on the layer's own codes, where nearly every tile passes,
        # and on codes drawn uniformly from the whole range, where none does and the
        # workgroups give the test up.  Same shape, same kernel instance.
        if args.s == 32 and args.acc_bits == 8:
            qx, sx = B.quantize(X, 1, n, pf.A, 0)
            qw, sw = B.quantize(W, 0, n, pf.B, 0)
            g_t = torch.Generator(device=dev)
            g_t.manual_seed(1234)
            ux = torch.randint(0, 256, qx.shape, dtype=torch.uint8, device=dev, generator=g_t)
            uw = torch.randint(0, 256, qw.shape, dtype=torch.uint8, device=dev, generator=g_t)
            o_t = torch.empty((M, N), dtype=torch.float32, device=dev)
            ws_t = torch.empty(max(B.load().hdqt_gemm_codes_workspace_size(M, N, K, args.s), 256),
                               dtype=torch.uint8, device=dev)
            tt = {}
            for key, (a_, b_) in (("fwd_layer_codes", (qx, qw)), ("fwd_codes_uniform_over_the_range", (ux, uw))):
                _, k_f = timed(lambda: B.gemm_codes(a_, b_, 4, 4, sx, sw, K, n, 8, args.s, want_acc=False,
                                                    out=o_t, workspace=ws_t))
                tt[key + "_us"] = sum(v for n_, v in k_f.items() if n_.startswith("gemm"))
            line["tile_test"] = tt
            del qx, qw, ux, uw, o_t, ws_t
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(layer, n, args.s, min(args.cpu_rows, M))
    print(json.dumps(line))


if __name__ == "__main__":
    main()
