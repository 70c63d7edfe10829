#!/usr/bin/env python3
"""Benchmark of the compensated W3A16 expert linear on one MI355X.

Headline workload (config c1): the Mixtral-8x7B-shaped expert up-projection at decode,
X fp16 [16 x 4096], W [14336 x 4096] 3-bit group-64 with a rank-32 compensator.  One "step" is
one milo_w3lr_gemm call.  The weight is rotated through >= 24 distinct copies (> 2x the 256 MB
Infinity Cache) so that every step streams its weight from HBM ("cold" protocol); the steps are
captured in a HIP graph so that Python call overhead does not throttle a microsecond-scale kernel.
value = (packed blob: codes, scales, zero-points; + U + V bytes) / time per step.

Prints ONE JSON line.  Besides the headline it carries, under "extra", the other workloads of the
metric, each with its own roofline object: c1 at M = 1 and 4, Mixtral's down projection at decode,
the small configuration c0, the prefill GEMM c2 and the two MoE layers c3 and c4 (plus c3's shape at
a decode-sized batch), c1 with the INT3 compensator, the symmetric weight and bf16 activations, the time the compressor (Algorithm 1, offline) takes for one weight of c1's
shape, and what a library copy and a library fp16 GEMM reach on the same box (context).  --only NAME[,NAME...] restricts the run to some legs (for profiler runs).
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
MIN_TIMED_MS = 20.0             # a timed region shorter than this is repeated until it is not
LEGS = ("c1", "c1_small_m", "c1_variants", "w2_decode", "c0", "c2", "c3", "c4", "compress", "context")


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
    ap.add_argument("--only", type=str, default="",
                    help="comma-separated legs to run (of: %s); default all" % ", ".join(LEGS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 256 MiB elementwise copy kernel 20 times (counter "
                         "calibration for --pmc runs)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0,
                    help="CPU time to spend on the oracle baseline")
    return ap.parse_args()


def time_steps(fn_step, n_steps, period, warmup):
    """Time n_steps calls of fn_step(i) (i cycles through `period` variants) captured in HIP graphs
    (one graph of `period` steps, one for the remainder) with HIP events on the launching stream.
    A block of n_steps that takes less than MIN_TIMED_MS is repeated, so that the timed region never
    is a single short replay.  Returns (ms per step, steps timed)."""
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

    full, rem = divmod(n_steps, period)
    g_full = capture(period) if full else None
    g_rem = capture(rem) if rem else None

    def block():
        for _ in range(full):
            g_full.replay()
        if g_rem is not None:
            g_rem.replay()

    done = 0
    while done < max(warmup, 1):
        block()
        done += n_steps
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    total_ms, timed, reps = 0.0, 0, 1
    while True:
        start.record()
        for _ in range(reps):
            block()
        stop.record()
        torch.cuda.synchronize()
        total_ms += start.elapsed_time(stop)
        timed += reps * n_steps
        if total_ms >= MIN_TIMED_MS or timed >= 200000:
            break
        per = total_ms / timed
        reps = max(1, int((MIN_TIMED_MS - total_ms) / (per * n_steps)) + 1)
    return total_ms / timed, timed


def fit_compensator(W, pw, r, niter=2, oversample=10, seed=0):
    """Workload preparation (not part of the library): rank-r compensator of a packed weight, with
    the residual E = W - W_dq from the library's own dequantization kernel and U = U^_r sqrt(S_r),
    V = sqrt(S_r) V^_r (Section 3.2.3, Eq. UV) from the randomized SVD the paper's implementation
    uses (appendix "Implementation": torch.svd_lowrank)."""
    import torch
    from paper_2504_02658_amd import api
    if r == 0:
        return pw
    E = W - api.dequant_w3(pw).float()
    gen_state = torch.random.get_rng_state()
    torch.manual_seed(seed)
    try:
        Uh, S, Vh = torch.svd_lowrank(E, q=min(r + oversample, min(E.shape)), niter=niter)
    finally:
        torch.random.set_rng_state(gen_state)
    rs = torch.sqrt(S[:r])
    U = (Uh[:, :r] * rs[None, :]).to(torch.float16).contiguous()
    V = (rs[:, None] * Vh[:, :r].T).to(torch.float16).contiguous()
    return pw.with_compensator(U, V)


def clone_weight(pw):
    """A byte-identical copy at new addresses (to rotate weights through HBM)."""
    from paper_2504_02658_amd import api
    return api.PackedWeight(pw.N, pw.K, pw.q3.clone(),
                            None if pw.U is None else pw.U.clone(),
                            None if pw.V is None else pw.V.clone(), flags=pw.flags, r=pw.r if pw.U is not None else None)


def hbm_roofline(nbytes, ms, kernel, **more):
    gbs = nbytes / (ms * 1e-3) / 1e9
    d = {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
         "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": None, "kernel": kernel, "bytes_per_launch": int(nbytes)}
    d.update(more)
    return d


def mfma_roofline(flops, ms, kernel, **more):
    tf = flops / (ms * 1e-3) / 1e12
    d = {"bound": "mfma", "achieved": round(tf, 1), "peak": MFMA_FP16_PEAK_TFLOPS, "unit": "TFLOP/s",
         "frac": round(tf / MFMA_FP16_PEAK_TFLOPS, 4), "traffic": None, "kernel": kernel, "flops_per_step": flops}
    d.update(more)
    return d


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (--gpus 1); collectives and sharding "
              "are not part of it.", file=sys.stderr)
        sys.exit(2)
    legs = set(LEGS) if not args.only else set(x.strip() for x in args.only.split(",") if x.strip())
    unknown = legs - set(LEGS)
    if unknown:
        print("bench.py: unknown legs %s (known: %s)" % (sorted(unknown), ", ".join(LEGS)), file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2504_02658_amd import api, workloads as wl

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
        pw = fit_compensator(W, api.pack_w3(W), case.r, seed=case.seed)
        return W, pw

    def gemm_leg(M, K, N, r, weights, steps, warmup, dtype=torch.float16):
        X = torch.from_numpy(wl.gen_activations(M, K, 1001)).to(dev).to(dtype)
        Y = torch.empty((M, N), dtype=dtype, device=dev)
        ws = api.new_workspace(api.gemm_workspace_bytes(M, N, K, r), dev)
        step = lambda i: api.w3lr_gemm(X, weights[i % len(weights)], out=Y, workspace=ws)
        ms, timed = time_steps(step, steps, len(weights), warmup)
        assert api.workspace_status(ws) == 0, "a wait inside a GEMM kernel gave up"
        return ms, timed

    result, extra = None, {}
    case = wl.C1[16]
    W1 = pw1 = copies = None
    if legs & {"c1", "c1_small_m", "c1_variants"} or not args.no_cpu_baseline:
        W1, pw1 = build_linear(case)
    if legs & {"c1", "c1_small_m"}:
        copies = [pw1] + [clone_weight(pw1) for _ in range(args.copies - 1)]
    wbytes = pw1.weight_bytes() if pw1 is not None else 0
    code_bytes = pw1.q3.numel() if pw1 is not None else 0

    if "c1" in legs:
        ms_step, timed = gemm_leg(16, case.K, case.N, case.r, copies, args.steps, args.warmup)
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
            "timed_steps": timed,
            "us_per_call": round(ms_step * 1e3, 3),
            "tflops": round(flops / (ms_step * 1e-3) / 1e12, 3),
            "roofline": hbm_roofline(wbytes, ms_step, "w3lr_decode_kernel", traffic=measured_traffic(),
                                     weight_only_bytes=code_bytes,
                                     weight_only_frac=round(code_bytes / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)),
        }
    else:
        result = {"metric": "W3+low-rank GEMM HBM GB/s (M<=16)", "value": None, "unit": "GB/s", "n_gpus": 1,
                  "steps": args.steps, "warmup": args.warmup, "note": "headline leg not run (--only)"}

    if "c1_small_m" in legs:
        for M in (1, 4):
            ms, _ = gemm_leg(M, case.K, case.N, case.r, copies, args.steps, args.warmup)
            extra[f"c1_M{M}_cold"] = {"us": round(ms * 1e3, 3),
                                      "roofline": hbm_roofline(wbytes, ms, "w3lr_decode_kernel")}
        ms, _ = gemm_leg(16, case.K, case.N, case.r, copies[:1] * 24, args.steps, args.warmup)
        extra["c1_M16_hot"] = {"us": round(ms * 1e3, 3), "note": "one weight copy, cache resident; not an HBM figure"}
    if copies is not None:
        del copies[1:]
        copies = None
        torch.cuda.empty_cache()

    if "c1_variants" in legs:
        # the same call with the other forms of the weight (Section 3.2.3 INT3 compensator, Section 3.3
        # symmetric conversion) and with bf16 activations; same cold protocol
        def variant(name, pw, dtype=torch.float16, note=""):
            cps = [pw] + [clone_weight(pw) for _ in range(args.copies - 1)]
            ms, _ = gemm_leg(16, case.K, case.N, case.r, cps, args.steps, args.warmup, dtype)
            extra[name] = {"us": round(ms * 1e3, 3), "note": note,
                           "roofline": hbm_roofline(pw.weight_bytes(), ms, "w3lr_decode_kernel")}
            del cps
            torch.cuda.empty_cache()

        u3, v3 = api.pack_lr3(pw1.U.float(), pw1.V.float())
        variant("c1_M16_int3_compensator", pw1.with_int3_compensator(u3, v3, case.r),
                note="U, V as INT3 blobs (3.5 bit per element instead of 16)")
        pws = fit_compensator(W1, api.pack_w3(W1, symmetric=True), case.r, seed=case.seed)
        variant("c1_M16_symmetric", pws, note="symmetric quantizer, zero-point-free conversion")
        pwb = api.PackedWeight(pw1.N, pw1.K, pw1.q3, pw1.U.to(torch.bfloat16), pw1.V.to(torch.bfloat16))
        variant("c1_M16_bf16", pwb, dtype=torch.bfloat16, note="bf16 activations, compensator and output")
        del u3, v3, pws, pwb

    if "w2_decode" in legs:
        # Mixtral's down projection at decode (the other expert GEMM shape of Section 4): long K
        wc = wl.LinearCase("w2_decode", M=16, N=4096, K=14336, r=32, seed=1005)
        _, pww = build_linear(wc)
        wcopies = [pww] + [clone_weight(pww) for _ in range(args.copies - 1)]
        ms, _ = gemm_leg(16, wc.K, wc.N, wc.r, wcopies, args.steps, args.warmup)
        extra["w2_decode_M16_cold"] = {"us": round(ms * 1e3, 3), "N": wc.N, "K": wc.K, "r": wc.r,
                                       "roofline": hbm_roofline(pww.weight_bytes(), ms, "w3lr_decode_kernel")}
        del wcopies, pww
        torch.cuda.empty_cache()

    if "c0" in legs:
        # c0: the small parity configuration (launch-latency bound; reported in microseconds only)
        c0 = wl.C0
        _, pw0 = build_linear(c0)
        ms, _ = gemm_leg(c0.M, c0.K, c0.N, c0.r, [pw0] * 24, 240, 48)
        extra["c0_small"] = {"us": round(ms * 1e3, 3)}
        del pw0

    if "c2" in legs:
        c2 = wl.C2
        _, pw2 = build_linear(c2)
        ms, _ = gemm_leg(c2.M, c2.K, c2.N, c2.r, [pw2] * 10, 50, 10)
        f2 = 2.0 * c2.M * (c2.N * c2.K + c2.r * (c2.N + c2.K))
        extra["c2_prefill"] = {"us": round(ms * 1e3, 2),
                               "roofline": mfma_roofline(f2, ms, "w3lr_tiled_kernel<1,4,0> (+ splitk_sum_kernel)")}
        del pw2
        torch.cuda.empty_cache()

    # c3 / c4: MoE layers (weights drawn on the GPU with the same distribution as the numpy recipe)
    for leg, mc in (("c3", wl.C3), ("c4", wl.C4)):
        if leg not in legs:
            continue
        gen = torch.Generator(device=dev)
        gen.manual_seed(mc.seed)
        ranks = wl.expert_ranks(mc)
        experts = []
        for e in range(mc.E + mc.n_shared):
            trip = []
            for (N, K) in ((mc.F, mc.H), (mc.F, mc.H), (mc.H, mc.F)):
                We = torch.randn((N, K), generator=gen, device=dev, dtype=torch.float32) * wl.WEIGHT_STD
                trip.append(fit_compensator(We, api.pack_w3(We), ranks[e], seed=e))
                del We
            experts.append(tuple(trip))
        layer = api.MoELayer(experts, mc.H, mc.F)

        def moe_leg(mcase):
            Xm = torch.from_numpy(wl.moe_activations(mcase)).to(dev)
            ids_np, gates_np = wl.moe_routing(mcase)
            ids, gates = torch.from_numpy(ids_np).to(dev), torch.from_numpy(gates_np).to(dev)
            Ym = torch.empty((mcase.T, mcase.H), dtype=torch.float16, device=dev)
            wsm = api.new_workspace(layer.workspace_bytes(mcase.T, ids.shape[1]), dev)
            ms, _ = time_steps(lambda i: layer.forward(Xm, ids, gates, out=Ym, workspace=wsm), 30, 10, 10)
            assert layer.routing_status() == 0, "the MoE layer reported an error"
            return ms, ids_np

        ms, ids_np = moe_leg(mc)
        pairs = np.bincount(ids_np.reshape(-1), minlength=mc.E + mc.n_shared)
        fl = sum(2.0 * int(pairs[e]) * (3 * mc.H * mc.F + 3 * ranks[e] * (mc.H + mc.F))
                 for e in range(mc.E + mc.n_shared))
        extra[mc.name] = {"us_per_layer": round(ms * 1e3, 1), "tokens": mc.T,
                          "roofline": mfma_roofline(fl, ms, "w3lr_tiled_kernel<2,4,1> + <1,4,2> (+ route, order, combine)")}
        if mc is wl.C3:
            # the same layer at a decode-sized batch (16 tokens): every routed expert's weights are
            # streamed for a handful of rows, so the figure of merit is HBM bytes per second
            import dataclasses
            md = dataclasses.replace(mc, T=16)
            msd, idd_np = moe_leg(md)
            used = sorted(set(idd_np.reshape(-1).tolist()))
            wb = sum(3 * md.H * md.F * 7 / 16 + 3 * 2 * ranks[e] * (md.H + md.F) for e in used)
            extra["c3_shape_16_tokens"] = {"us_per_layer": round(msd * 1e3, 1), "experts_used": len(used),
                                           "roofline": hbm_roofline(wb, msd, "grouped W3 kernels of the MoE layer")}
        del layer, experts
        torch.cuda.empty_cache()

    if "compress" in legs:
        # Algorithm 1 for one weight of c1's shape: 20 iterations (the paper's early stop), stop rule off
        # so that the work is fixed; wall clock around the call, which synchronizes by itself
        cc = wl.C1[16]
        Wc = torch.from_numpy(wl.gen_weight_lowrank(cc.N, cc.K, cc.seed, outlier_frac=0.01)).to(dev)
        api.compress_w3lr(Wc, cc.r, iters=2, tol=-1.0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        _, _, _, eps_c = api.compress_w3lr(Wc, cc.r, iters=20, tol=-1.0)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        extra["compress_c1_weight"] = {"seconds": round(dt, 3), "iters": len(eps_c), "N": cc.N, "K": cc.K, "r": cc.r,
                                       "eps_first": round(eps_c[0], 4), "eps_last": round(eps_c[-1], 4)}
        del Wc
        torch.cuda.empty_cache()

    if "context" in legs:
        # What library kernels (not this repository's code) reach on the same box: a device-to-device
        # copy and a dense fp16 GEMM.  Context for the two rooflines, not a target and not a baseline.
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        ms, _ = time_steps(lambda i: dst.copy_(src), 10, 1, 3)
        A = torch.randn((8192, 8192), device=dev, dtype=torch.float16)
        B = torch.randn((8192, 8192), device=dev, dtype=torch.float16)
        C = torch.empty((8192, 8192), device=dev, dtype=torch.float16)
        msg, _ = time_steps(lambda i: torch.matmul(A, B, out=C), 10, 1, 3)
        extra["achievable_context"] = {
            "note": "library kernels on this box, for context: torch device copy of 1 GiB (bytes read + written) "
                    "and torch.matmul 8192^3 fp16 with random operands",
            "copy_TBps": round(2 * (1 << 30) / (ms * 1e-3) / 1e12, 2),
            "dense_fp16_gemm_TFLOPs": round(2 * 8192.0 ** 3 / (msg * 1e-3) / 1e12, 1)}
        del src, dst, A, B, C
        torch.cuda.empty_cache()

    if extra:
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
        Wh = W1.cpu().numpy()
        q, s, z = oracle.quantize_rtn(Wh)
        U = pw1.U.cpu().numpy()
        V = pw1.V.cpu().numpy()
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
