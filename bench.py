#!/usr/bin/env python3
"""Benchmark of the compensated W3A16 expert linear on one MI355X.

Headline workload (config c1): the Mixtral-8x7B-shaped expert up-projection at decode,
X fp16 [16 x 4096], W [14336 x 4096] 3-bit group-64 with a rank-32 compensator.  One "step" is
one milo_w3lr_gemm call.  The weight is rotated through >= 24 distinct copies (> 2x the 256 MB
Infinity Cache) so that every step streams its weight from HBM ("cold" protocol); the steps are
captured in a HIP graph so that Python call overhead does not throttle a microsecond-scale kernel.
value = (packed blob: codes, scales, zero-points; + U + V bytes) / time per step.

Prints ONE JSON line.  --extra adds M = 1 / 4, cache-resident ("hot") numbers, the prefill GEMM
(c2) and the two MoE layers (c3, c4) to an "extra" object.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_FP16_PEAK_TFLOPS = 2500.0


def measured_traffic():
    """HBM bytes per launch of the decode kernel on this workload, from the rocprofv3 --pmc runs
    summarised in profiles/ (FETCH_SIZE + WRITE_SIZE, scaled by a plain copy); None if absent."""
    path = os.path.join(ROOT, "profiles", "w3lr_decode_kernel_c1_pmc.md")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return int(float(line.split(":", 1)[1].strip()))
    except OSError:
        pass
    return None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=240)
    ap.add_argument("--warmup", type=int, default=48)
    ap.add_argument("--copies", type=int, default=24)
    ap.add_argument("--extra", action="store_true", help="also measure M=1/4, hot, c2, c3, c4")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--only-c2", action="store_true",
                    help="run only the c2 prefill GEMM (for counter runs of the tiled kernel)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 256 MiB elementwise copy kernel 20 times (counter "
                         "calibration for --pmc runs)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0,
                    help="CPU time to spend on the oracle baseline")
    return ap.parse_args()


def time_steps(fn_step, n_steps, period, warmup):
    """Time exactly n_steps calls of fn_step(i) (i cycles through `period` variants) inside HIP
    graphs: one graph of `period` steps replayed, plus one for the remainder.  Returns ms total."""
    import torch
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(stream):
        for i in range(min(period, 4)):
            fn_step(i)
    torch.cuda.current_stream().wait_stream(stream)
    torch.cuda.synchronize()

    def capture(count):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for i in range(count):
                fn_step(i)
        return g

    g_full = capture(period)
    rem = n_steps % period
    g_rem = capture(rem) if rem else None
    for _ in range(max(1, warmup // period)):
        g_full.replay()
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    start.record()
    for _ in range(n_steps // period):
        g_full.replay()
    if g_rem is not None:
        g_rem.replay()
    stop.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    return start.elapsed_time(stop), wall_ms


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (--gpus 1); collectives and sharding "
              "are not part of it.", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2504_02658_amd import api, compress, workloads as wl

    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")

    if args.calibrate_copy:
        # A plain elementwise copy kernel of known size (reads 256 MiB, writes 256 MiB per launch):
        # what FETCH_SIZE / WRITE_SIZE read for it gives the counters' scale.
        src = torch.zeros(64 << 20, dtype=torch.int32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(20):
            torch.add(src, 1, out=dst)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes": 256 << 20, "launches": 20}))
        return

    def build_linear(case):
        W = torch.from_numpy(wl.gen_weight(case.N, case.K, case.seed, case.outlier_frac,
                                           case.outlier_gain)).to(dev)
        pw = compress.fit_compensator(W, api.pack_w3(W), case.r, seed=case.seed)
        return W, pw

    if args.only_c2:
        c2 = wl.C2
        _, pw2 = build_linear(c2)
        X2 = torch.from_numpy(wl.gen_activations(c2.M, c2.K, c2.seed)).to(dev)
        Y2 = torch.empty((c2.M, c2.N), dtype=torch.float16, device=dev)
        ws2 = api.new_workspace(api.gemm_workspace_bytes(c2.M, c2.N, c2.K, c2.r), dev)
        ms, _ = time_steps(lambda i: api.w3lr_gemm(X2, pw2, out=Y2, workspace=ws2), 50, 10, 10)
        ms /= 50
        f2 = 2.0 * c2.M * (c2.N * c2.K + c2.r * (c2.N + c2.K))
        print(json.dumps({"c2_prefill": {"us": round(ms * 1e3, 2), "TFLOPs": round(f2 / ms / 1e9, 1),
                                         "flops_per_call": f2}}))
        return

    case = wl.C1[16]
    W, pw = build_linear(case)
    copies = [pw] + [compress.clone_weight(pw) for _ in range(args.copies - 1)]
    wbytes = pw.weight_bytes()
    code_bytes = pw.q3.numel()           # codes, scales and zero-points

    def decode_bench(M, weights, steps, warmup):
        X = torch.from_numpy(wl.gen_activations(M, case.K, case.seed)).to(dev)
        Y = torch.empty((M, case.N), dtype=torch.float16, device=dev)
        ws = api.new_workspace(api.gemm_workspace_bytes(M, case.N, case.K, case.r), dev)
        step = lambda i: api.w3lr_gemm(X, weights[i % len(weights)], out=Y, workspace=ws)
        ev_ms, wall_ms = time_steps(step, steps, len(weights), warmup)
        return ev_ms / steps, wall_ms / steps

    ms_step, wall_step = decode_bench(16, copies, args.steps, args.warmup)
    gbs = wbytes / (ms_step * 1e-3) / 1e9
    flops = 2.0 * 16 * (case.N * case.K + case.r * (case.N + case.K))

    result = {
        "metric": "W3+low-rank GEMM HBM GB/s (M<=16)",
        "value": round(gbs, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_step, 6),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16",
        "data": "synthetic",
        "config": {"workload": "c1: Mixtral-8x7B expert up-projection at decode, M=16, N=14336, "
                               "K=4096, W3 g64 asym + rank-32 fp16 compensator, "
                               f"{args.copies} weight copies rotated (cold HBM)",
                   "M": 16, "N": case.N, "K": case.K, "r": case.r, "copies": args.copies},
        "us_per_call": round(ms_step * 1e3, 3),
        "tflops": round(flops / (ms_step * 1e-3) / 1e12, 3),
        "roofline": {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": measured_traffic(),
                     "kernel": "w3lr_decode_kernel",
                     "bytes_per_launch": wbytes, "weight_only_bytes": code_bytes,
                     "weight_only_frac": round(code_bytes / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
    }

    if args.extra:
        extra = {}
        for M in (1, 4):
            ms, _ = decode_bench(M, copies, args.steps, args.warmup)
            extra[f"c1_M{M}_cold"] = {"us": round(ms * 1e3, 3),
                                      "GBps": round(wbytes / (ms * 1e-3) / 1e9, 1)}
        ms, _ = decode_bench(16, copies[:1] * 24, args.steps, args.warmup)
        extra["c1_M16_hot"] = {"us": round(ms * 1e3, 3), "GBps": round(wbytes / (ms * 1e-3) / 1e9, 1)}
        del copies[1:]
        torch.cuda.empty_cache()

        # c0: the small parity configuration (launch-latency bound; reported in microseconds only)
        c0 = wl.C0
        W0, pw0 = build_linear(c0)
        del W0
        X0 = torch.from_numpy(wl.gen_activations(c0.M, c0.K, c0.seed)).to(dev)
        Y0 = torch.empty((c0.M, c0.N), dtype=torch.float16, device=dev)
        ws0 = api.new_workspace(api.gemm_workspace_bytes(c0.M, c0.N, c0.K, c0.r), dev)
        ms, _ = time_steps(lambda i: api.w3lr_gemm(X0, pw0, out=Y0, workspace=ws0), 240, 24, 48)
        extra["c0_small"] = {"us": round(ms / 240 * 1e3, 3)}
        del pw0, X0, Y0, ws0

        # c2: prefill GEMM
        c2 = wl.C2
        W2, pw2 = build_linear(c2)
        del W2
        X2 = torch.from_numpy(wl.gen_activations(c2.M, c2.K, c2.seed)).to(dev)
        Y2 = torch.empty((c2.M, c2.N), dtype=torch.float16, device=dev)
        ws2 = api.new_workspace(api.gemm_workspace_bytes(c2.M, c2.N, c2.K, c2.r), dev)
        ms, _ = time_steps(lambda i: api.w3lr_gemm(X2, pw2, out=Y2, workspace=ws2), 50, 10, 10)
        ms /= 50
        f2 = 2.0 * c2.M * (c2.N * c2.K + c2.r * (c2.N + c2.K))
        extra["c2_prefill"] = {"us": round(ms * 1e3, 2), "TFLOPs": round(f2 / ms / 1e9, 1),
                               "frac_mfma_peak": round(f2 / ms / 1e9 / MFMA_FP16_PEAK_TFLOPS, 4)}
        del pw2, X2, Y2, ws2
        torch.cuda.empty_cache()

        # c3 / c4: MoE layers (weights drawn on the GPU with the same distribution)
        for mc in (wl.C3, wl.C4):
            gen = torch.Generator(device=dev)
            gen.manual_seed(mc.seed)
            ranks = wl.expert_ranks(mc)
            experts = []
            for e in range(mc.E + mc.n_shared):
                trip = []
                for (N, K) in ((mc.F, mc.H), (mc.F, mc.H), (mc.H, mc.F)):
                    We = torch.randn((N, K), generator=gen, device=dev, dtype=torch.float32) * wl.WEIGHT_STD
                    trip.append(compress.fit_compensator(We, api.pack_w3(We), ranks[e], seed=e))
                    del We
                experts.append(tuple(trip))
            layer = api.MoELayer(experts, mc.H, mc.F)
            Xm = torch.from_numpy(wl.moe_activations(mc)).to(dev)
            ids_np, gates_np = wl.moe_routing(mc)
            ids, gates = torch.from_numpy(ids_np).to(dev), torch.from_numpy(gates_np).to(dev)
            Ym = torch.empty((mc.T, mc.H), dtype=torch.float16, device=dev)
            wsm = api.new_workspace(layer.workspace_bytes(mc.T, ids.shape[1]), dev)
            ms, _ = time_steps(lambda i: layer.forward(Xm, ids, gates, out=Ym, workspace=wsm), 30, 10, 10)
            ms /= 30
            pairs = np.bincount(ids_np.reshape(-1), minlength=mc.E + mc.n_shared)
            fl = sum(2.0 * int(pairs[e]) * (3 * mc.H * mc.F + 3 * ranks[e] * (mc.H + mc.F))
                     for e in range(mc.E + mc.n_shared))
            extra[mc.name] = {"us_per_layer": round(ms * 1e3, 1), "TFLOPs": round(fl / ms / 1e9, 1),
                              "frac_mfma_peak": round(fl / ms / 1e9 / MFMA_FP16_PEAK_TFLOPS, 4)}
            if mc is wl.C3:
                # the same layer at a decode-sized batch (16 tokens): every expert's weights are
                # streamed for a handful of rows, so the figure of merit is HBM bytes per second
                import dataclasses
                md = dataclasses.replace(mc, T=16)
                Xd = torch.from_numpy(wl.moe_activations(md)).to(dev)
                idd_np, gd_np = wl.moe_routing(md)
                idd, gd = torch.from_numpy(idd_np).to(dev), torch.from_numpy(gd_np).to(dev)
                Yd = torch.empty((md.T, md.H), dtype=torch.float16, device=dev)
                wsd = api.new_workspace(layer.workspace_bytes(md.T, idd.shape[1]), dev)
                msd, _ = time_steps(lambda i: layer.forward(Xd, idd, gd, out=Yd, workspace=wsd), 30, 10, 10)
                msd /= 30
                used = sorted(set(idd_np.reshape(-1).tolist()))
                wb = sum(3 * md.H * md.F * 7 / 16 + 3 * 2 * ranks[e] * (md.H + md.F) for e in used)
                extra["c3_shape_16_tokens"] = {"us_per_layer": round(msd * 1e3, 1), "experts_used": len(used),
                                               "weight_MB": round(wb / 1e6, 1),
                                               "GBps": round(wb / (msd * 1e-3) / 1e9, 1),
                                               "frac_hbm_peak": round(wb / (msd * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
                del Xd, Yd, wsd
            del layer, experts, Xm, Ym, wsm
            torch.cuda.empty_cache()
        # Context: what library kernels reach on this machine (not this repository's code): a plain
        # device-to-device copy of 1 GiB (bytes read + written) and a dense fp16 GEMM of 8192^3.
        def eager_ms(fn, n):
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(n):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / n
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        ms = eager_ms(lambda: dst.copy_(src), 20)
        copy_gbs = 2.0 * (1 << 30) / (ms * 1e-3) / 1e9
        del src, dst
        A = torch.randn((8192, 8192), device=dev, dtype=torch.float16)
        B = torch.randn((8192, 8192), device=dev, dtype=torch.float16)
        ms = eager_ms(lambda: torch.matmul(A, B), 10)
        gemm_tf = 2.0 * 8192 ** 3 / (ms * 1e-3) / 1e12
        del A, B
        torch.cuda.empty_cache()
        # ... and a copy of exactly the bytes one c1 launch reads (26.9 MB, sources rotated like the
        # weight copies, 24 copies per graph): what a kernel launch of that size costs on this machine
        small = [torch.empty(wbytes, dtype=torch.uint8, device=dev).random_(0, 255) for _ in range(24)]
        small_dst = torch.empty(wbytes, dtype=torch.uint8, device=dev)
        ms, _ = time_steps(lambda i: small_dst.copy_(small[i % 24]), 240, 24, 48)
        small_us = ms / 240 * 1e3
        del small, small_dst
        torch.cuda.empty_cache()
        extra["achievable_context"] = {"torch_copy_1GiB_GBps": round(copy_gbs, 1),
                                       "torch_fp16_gemm_8192_TFLOPs": round(gemm_tf, 1),
                                       "torch_copy_of_c1_bytes_us": round(small_us, 2)}
        result["extra"] = extra

    if not args.no_cpu_baseline:
        # The fp64 oracle on the host cores, on the same c1 workload (full calls at M = 16):
        # dequantize + X W_dq^T + (X V^T) U^T.  A reported baseline, not a target.
        import oracle
        try:
            from threadpoolctl import threadpool_info
            blas_threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            blas_threads = os.cpu_count()
        Wh = W.cpu().numpy()
        q, s, z = oracle.quantize_rtn(Wh)
        U = pw.U.cpu().numpy()
        V = pw.V.cpu().numpy()
        Xh = wl.gen_activations(16, case.K, case.seed)
        calls, t0 = 0, time.perf_counter()
        while True:
            oracle.w3lr_linear(Xh, q, s, z, U, V)
            calls += 1
            total = time.perf_counter() - t0
            if total >= args.cpu_seconds or calls >= 1000:
                break
        result["cpu_baseline"] = {"value": round(wbytes * calls / total / 1e9, 4), "unit": "GB/s",
                                  "cores": int(blas_threads), "kind": "oracle",
                                  "sample": f"{calls} full c1 calls at M=16 (fp64 dequantize + GEMM "
                                            f"+ low-rank term) in {total:.1f} s, mean rate",
                                  "seconds_per_call": round(total / calls, 4)}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
