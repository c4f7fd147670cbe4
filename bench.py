#!/usr/bin/env python3
"""Benchmark of the whole hot path on one MI355X.

One step = grf_sample (walks + CSR of Phi_hat), grf_form_buckets (column lists + buckets) and
grf_gather_buckets (gather, contraction, normalisation) on the headline workload: 32768 points in
16 Gaussian clusters, symmetrised 16-NN graph, 32 walks per node, p_halt = 0.2, f of length 16,
batch 1, 8 heads, d = 64, fp32.  Inputs are resident in HBM before the timed region.

Prints ONE JSON line.  `value` is tokens/s/head = N*B*H / step time.  `roofline` is for the gather
kernel (the dominant one): algorithmic bytes per launch over its mean duration between HIP events
recorded on the launch stream inside the timed region.  `cpu_baseline` times the CPU checker on one
head of the same workload on this machine's host cores.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth

# Bytes moved between L2 and the fabric per gather launch, from rocprofv3 --pmc runs of this file
# (FETCH_SIZE x 2.000 + WRITE_SIZE x 1.000, factors from --copy-calibration under the same
# counters).  A stored measurement, not recomputed here; absent workloads report null.
MEASURED_TRAFFIC_BYTES = {"cloud_32k": 322188156585, "vit_grid": 23538457990, "cloud_8k": 224494242686, "cloud_128k": 2542783367655}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cloud_32k")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the CPU checker timing (profiling runs)")
    ap.add_argument("--dynamic-only", action="store_true",
                    help="only the dynamic point-cloud section (graph construction + walks + asymmetric attention), for profiling")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain device-to-device copy of 1 GiB three times (scale for the HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2410_03462_amd import binding as grf
    from paper_2410_03462_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 2
    grf.lib()
    dev = "cuda:0"
    torch.cuda.set_device(0)

    if args.copy_calibration:
        nbytes = 1 << 30
        src = torch.full((nbytes // 4,), 1.0, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": True, "bytes_read_per_copy": nbytes, "bytes_written_per_copy": nbytes, "copies": 3}))
        return 0

    wl = synth.workload(args.workload)
    N, B, H, d = wl.graph.n, wl.B, wl.H, wl.d
    g = grf.DeviceGraph.from_host(wl.graph, dev)
    Q, K, V = wl.qkv()
    to_dev = (lambda x: torch.from_numpy(x).to(dev).to(torch.bfloat16)) if wl.dtype == "bf16" else (lambda x: torch.from_numpy(x).to(dev))
    Qd, Kd, Vd = to_dev(Q), to_dev(K), to_dev(V)

    stream = torch.cuda.current_stream()

    def dynamic_section(aout):
        # dynamic point clouds (Sec. 4 / App. C): the graph is rebuilt every step, so graph construction is on the path.
        # (i) the workload's own graph (symmetrised k-NN, kernel weights) rebuilt on the GPU;
        # (ii) the paper's setting: neighbour lists of length 3, 27 walks of exactly 3 hops, asymmetric GRFs.
        dynamic = None
        tokens = N * B * H
        if "points" in wl.notes:
            pts = torch.from_numpy(wl.notes["points"].astype(np.float32)).to(dev)
            kk, kern = wl.notes["k"], wl.notes["kernel"]
            from scipy.spatial import cKDTree
            sub = wl.notes["points"][:: max(1, N // 4096)]
            sigma = float(np.median(cKDTree(wl.notes["points"]).query(sub, k=kk + 1)[0][:, 1:]))    # scale only; not timed
            kws = torch.empty(grf.grf_knn_graph_workspace_bytes(N, max(kk, 3)), dtype=torch.uint8, device=dev)

            def timed(fn):
                for _ in range(args.warmup):
                    fn()
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                for _ in range(args.steps):
                    fn()
                e1.record(stream)
                torch.cuda.synchronize()
                return e0.elapsed_time(e1) / args.steps

            knn_ms = timed(lambda: grf.grf_knn_graph(pts, kk, True, kern, sigma, workspace=kws))
            f3 = np.array([[1.0, 0.6, 0.3, 0.15]], dtype=np.float32)
            g3 = grf.grf_knn_graph(pts, 3, False, "inv_degree", workspace=kws)
            phi3 = grf.grf_sample(g3, f3, 0.0, 27, wl.walk_seed)

            def dynamic_step():
                gg = grf.grf_knn_graph(pts, 3, False, "inv_degree", workspace=kws)
                grf.grf_sample(gg, f3, 0.0, 27, wl.walk_seed, out=phi3)
                grf.grf_asymmetric_masked_attention(Qd, Kd, Vd, phi3, out=aout)

            knn3_ms = timed(lambda: grf.grf_knn_graph(pts, 3, False, "inv_degree", workspace=kws))
            dyn_ms = timed(dynamic_step)

            # the same step without host synchronisation (counts stay on the device, buffers sized by their bounds),
            # captured once into a HIP graph and replayed
            f3_dev = torch.from_numpy(f3).to(dev)
            g_buf = grf.grf_knn_graph(pts, 3, False, "inv_degree", workspace=kws, sync=False)
            phi_buf = grf.grf_sample_async(g_buf, f3_dev, 0.0, 27, wl.walk_seed)
            sws = torch.empty(1024, dtype=torch.uint8, device=dev)

            def async_step():
                grf.grf_knn_graph(pts, 3, False, "inv_degree", workspace=kws, out=g_buf, sync=False)
                grf.grf_sample_async(g_buf, f3_dev, 0.0, 27, wl.walk_seed, out=phi_buf, workspace=sws)
                grf.grf_asymmetric_masked_attention(Qd, Kd, Vd, phi_buf, out=aout)

            async_step()
            torch.cuda.synchronize()
            side = torch.cuda.Stream()
            side.wait_stream(stream)
            hip_graph = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                with torch.cuda.graph(hip_graph, stream=side):
                    async_step()
            torch.cuda.synchronize()
            replay_ms = timed(hip_graph.replay)
            dynamic = {
                "knn_graph_ms": round(knn_ms, 4), "knn_graph": "k=%d, symmetrised, %s kernel, row-normalised" % (kk, kern),
                "knn_points_per_s": round(N / (knn_ms * 1e-3), 1),
                "paper_setting": {"graph": "k=3 neighbour lists", "walks": "27 per node, 3 hops, no halting", "estimator": "asymmetric GRFs",
                                  "knn_graph_ms": round(knn3_ms, 4), "step_ms": round(dyn_ms, 4), "phi_nnz": phi3.nnz,
                                  "tokens_per_s_per_head": round(tokens / (dyn_ms * 1e-3), 1),
                                  "hip_graph_replay_step_ms": round(replay_ms, 4),
                                  "hip_graph_replay_tokens_per_s_per_head": round(tokens / (replay_ms * 1e-3), 1),
                                  "step": "grf_knn_graph + grf_sample + grf_asymmetric_masked_attention"},
            }
        return dynamic

    if args.dynamic_only:
        print(json.dumps({"workload": wl.name, "dynamic_point_cloud": dynamic_section(torch.empty((B, H, N, d), dtype=torch.float32, device=dev))}))
        return 0

    # buffers sized once, outside the timed region
    phi = grf.grf_sample(g, wl.f, wl.p_halt, wl.n_walks, wl.walk_seed)
    nnz = phi.nnz
    rec = grf.grf_bucket_record_floats(d)
    buckets = torch.empty((B * H, N, rec), dtype=torch.float32, device=dev)
    ws = torch.empty(grf.grf_buckets_workspace_bytes(N, nnz, phi.n_f), dtype=torch.uint8, device=dev)
    out = torch.empty((B, H, N, d), dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream()

    def step(events=None):
        if events: events[0].record(stream)
        grf.grf_sample(g, wl.f, wl.p_halt, wl.n_walks, wl.walk_seed, out=phi)
        if events: events[1].record(stream)
        grf.grf_form_buckets(Kd, Vd, phi, out=buckets, workspace=ws)
        if events: events[2].record(stream)
        grf.grf_gather_buckets(Qd, phi, buckets, out=out)
        if events: events[3].record(stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(events[k])
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    sample_ms = float(np.mean([e[0].elapsed_time(e[1]) for e in events]))
    buckets_ms = float(np.mean([e[1].elapsed_time(e[2]) for e in events]))
    gather_ms = float(np.mean([e[2].elapsed_time(e[3]) for e in events]))
    tokens = N * B * H
    value = tokens / (ms_per_step * 1e-3)

    # algorithmic bytes of one gather launch: per slice, every entry of Phi_hat pulls one bucket
    # record and its (col, val) pair; Q is read and out written once
    gather_bytes = B * H * (nnz * (rec * 4 + 8) + 2 * N * d * 4)
    achieved = gather_bytes / (gather_ms * 1e-3) / 1e9
    # what a plain device-to-device copy of 1 GiB sustains on this machine (read + write bytes), for scale
    cp_src = torch.empty(1 << 28, dtype=torch.float32, device=dev)
    cp_dst = torch.empty_like(cp_src)
    cp_dst.copy_(cp_src)
    torch.cuda.synchronize()
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record(stream)
    for _ in range(5):
        cp_dst.copy_(cp_src)
    c1.record(stream)
    torch.cuda.synchronize()
    copy_gbs = 5 * 2 * cp_src.numel() * 4 / (c0.elapsed_time(c1) * 1e-3) / 1e9
    del cp_src, cp_dst
    roofline = {"kernel": "gather_kernel", "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": MEASURED_TRAFFIC_BYTES.get(args.workload),
                "algorithmic_bytes_per_launch": gather_bytes, "avg_launch_ms": round(gather_ms, 4),
                "copy_1GiB_GBs": round(copy_gbs, 1), "frac_of_copy": round(achieved / copy_gbs, 4)}

    # the bucket-fused variant of the attention call on the same inputs: its own numbers, never `value`
    fws = torch.empty(grf.grf_fused_attention_workspace_bytes(B, H, N, d, nnz, phi.n_f), dtype=torch.uint8, device=dev)
    fout = torch.empty_like(out)

    def fused_step(events=None):
        if events: events[0].record(stream)
        grf.grf_sample(g, wl.f, wl.p_halt, wl.n_walks, wl.walk_seed, out=phi)
        if events: events[1].record(stream)
        grf.grf_masked_linear_attention_fused(Qd, Kd, Vd, phi, workspace=fws, out=fout)
        if events: events[2].record(stream)

    for _ in range(args.warmup):
        fused_step()
    torch.cuda.synchronize()
    fevents = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    f0 = time.perf_counter()
    for k in range(args.steps):
        fused_step(fevents[k])
    torch.cuda.synchronize()
    f1 = time.perf_counter()
    fused_ms_per_step = (f1 - f0) * 1e3 / args.steps
    fused_attn_ms = float(np.mean([e[1].elapsed_time(e[2]) for e in fevents]))
    # two contractions per entry of Phi_hat: S_l += a v^T and P = qw S_l, 2*d*d flops each
    fused_flops = 4.0 * nnz * d * d * B * H
    fused = {
        "entry_point": "grf_masked_linear_attention_fused",
        "ms_per_step": round(fused_ms_per_step, 4),
        "tokens_per_s_per_head": round(tokens / (fused_ms_per_step * 1e-3), 1),
        "attention_ms": round(fused_attn_ms, 4),
        "attention_only_tokens_per_s_per_head": round(tokens / (fused_attn_ms * 1e-3), 1),
        "roofline": {"bound": "mfma", "unit": "TFLOP/s", "peak": 157.3,
                     "achieved_whole_call": round(fused_flops / (fused_attn_ms * 1e-3) / 1e12, 2),
                     "flops_per_call": fused_flops,
                     "note": "whole attention call (column lists + fused buckets + row reduce); per-kernel times in profiles/"},
    }
    elem = 2 if wl.dtype == "bf16" else 4
    if d == 64:
        # at d = 64 the bucket kernels run on the bf16 matrix instructions (fp32 operands in two or three bf16 pieces) and
        # are bound by the rows read and the partial rows written and read back, not by the matrix pipe
        fused_bytes = float(nnz) * B * H * (3 * d * elem + 2 * (d + 1) * 4)
        fused["roofline"] = {"bound": "hbm", "unit": "GB/s", "peak": HBM_PEAK_GBS,
                             "achieved_whole_call": round(fused_bytes / (fused_attn_ms * 1e-3) / 1e9, 1),
                             "bytes_per_call": fused_bytes, "useful_flops_per_call": fused_flops,
                             "useful_TFLOPs_whole_call": round(fused_flops / (fused_attn_ms * 1e-3) / 1e12, 2),
                             "note": "whole attention call; bytes = per entry of Phi_hat and slice three input rows, the partial "
                                     "row written by the bucket kernel and read by the row reduce; re-read input rows are partly "
                                     "served by L2 / Infinity Cache; per-kernel times in profiles/"}

    # asymmetric GRFs (App. D): the same sampled matrix used directly as the mask estimate
    aout = torch.empty_like(out)
    for _ in range(args.warmup):
        grf.grf_asymmetric_masked_attention(Qd, Kd, Vd, phi, out=aout)
    torch.cuda.synchronize()
    a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a0.record(stream)
    for _ in range(args.steps):
        grf.grf_asymmetric_masked_attention(Qd, Kd, Vd, phi, out=aout)
    a1.record(stream)
    torch.cuda.synchronize()
    asym_ms = a0.elapsed_time(a1) / args.steps
    elem = 2 if wl.dtype == "bf16" else 4
    asym_bytes = B * H * (nnz * (2 * d * elem + 8) + N * d * (elem + 4))     # k_j, v_j, (col, val) per entry; q_i in, out_i out
    asymmetric = {
        "entry_point": "grf_asymmetric_masked_attention",
        "attention_ms": round(asym_ms, 4),
        "attention_only_tokens_per_s_per_head": round(tokens / (asym_ms * 1e-3), 1),
        "roofline": {"bound": "hbm", "unit": "GB/s", "peak": HBM_PEAK_GBS,
                     "achieved": round(asym_bytes / (asym_ms * 1e-3) / 1e9, 1),
                     "frac": round(asym_bytes / (asym_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                     "algorithmic_bytes_per_launch": asym_bytes,
                     "note": "K and V of one head (16.8 MB) are re-read from L2 / Infinity Cache, so the algorithmic rate may exceed the HBM peak"},
    }

    # gradients (training with learnable f): backward of the attention call and of the sampler, on the fused
    # forward's saved out and den; six MFMA contractions of 2*nnz*d*d flops per slice
    _, _, fden = grf.grf_masked_linear_attention_fused(Qd, Kd, Vd, phi, workspace=fws, return_num_den=True, out=fout)
    d_out = torch.randn((B, H, N, d), dtype=torch.float32, device=dev, generator=torch.Generator(device=dev).manual_seed(0))
    bws = torch.empty(grf.grf_attention_backward_workspace_bytes(B, H, N, d, nnz, phi.n_f), dtype=torch.uint8, device=dev)

    def backward_step():
        grads = grf.grf_masked_linear_attention_backward(Qd, Kd, Vd, phi, fout, fden, d_out, workspace=bws)
        return grf.grf_sample_backward(g, wl.f_len, wl.p_halt, wl.n_walks, wl.walk_seed, phi, grads[3])

    for _ in range(args.warmup):
        backward_step()
    torch.cuda.synchronize()
    b0, b1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    b0.record(stream)
    for _ in range(args.steps):
        backward_step()
    b1.record(stream)
    torch.cuda.synchronize()
    bwd_ms = b0.elapsed_time(b1) / args.steps
    bwd_flops = 12.0 * nnz * d * d * B * H
    backward = {
        "entry_points": "grf_masked_linear_attention_backward + grf_sample_backward",
        "ms": round(bwd_ms, 4),
        "tokens_per_s_per_head": round(tokens / (bwd_ms * 1e-3), 1),
        "roofline": {"bound": "mfma", "unit": "TFLOP/s", "peak": 157.3,
                     "achieved_whole_call": round(bwd_flops / (bwd_ms * 1e-3) / 1e12, 2), "flops_per_call": bwd_flops,
                     "note": "whole backward (seed, column lists, three bucket passes with their row reductions, dphi, df)"},
    }
    if d == 64:
        # three passes, each reading two input rows and one fp32 seed row per entry of Phi_hat and slice, writing one
        # fp32 partial row and reading it back in the row reduction
        bwd_bytes = float(nnz) * B * H * 3 * (2 * d * elem + d * 4 + 2 * d * 4)
        backward["roofline"] = {"bound": "hbm", "unit": "GB/s", "peak": HBM_PEAK_GBS,
                                "achieved_whole_call": round(bwd_bytes / (bwd_ms * 1e-3) / 1e9, 1),
                                "bytes_per_call": bwd_bytes, "useful_flops_per_call": bwd_flops,
                                "useful_TFLOPs_whole_call": round(bwd_flops / (bwd_ms * 1e-3) / 1e12, 2),
                                "note": "whole backward (seed, column lists, three bucket passes on the bf16 matrix instructions "
                                        "with their row reductions, dphi, df); re-read input rows are partly served by L2 / "
                                        "Infinity Cache; per-kernel times in profiles/"}

    dynamic = dynamic_section(aout)

    result = {
        "metric": "GRF-masked linear attention tokens/s/head at N=%d" % N,
        "value": round(value, 1), "unit": "tokens/s/head",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if wl.dtype == "f32" else "bf16 in, f32 accumulate", "data": "synthetic",
        "config": {"workload": wl.name, "N": N, "batch": B, "heads": H, "d": d, "m": d, "n_walks": wl.n_walks,
                   "p_halt": wl.p_halt, "f_len": wl.f_len, "graph_edges": wl.graph.nnz, "phi_nnz": nnz,
                   "feature_map": "relu", "step": "grf_sample + grf_form_buckets + grf_gather_buckets"},
        "stage_ms": {"sample": round(sample_ms, 4), "buckets": round(buckets_ms, 4), "gather": round(gather_ms, 4)},
        "attention_only_tokens_per_s_per_head": round(tokens / ((buckets_ms + gather_ms) * 1e-3), 1),
        "roofline": roofline,
        "fused_variant": fused,
        "asymmetric_variant": asymmetric,
        "backward": backward,
        "dynamic_point_cloud": dynamic,
    }

    if not args.no_cpu_baseline:
        from oracle import grf_oracle
        grf_oracle.build()
        c0 = time.perf_counter()
        rp, col, val = grf_oracle.sample(wl.graph, wl.f, wl.p_halt, wl.n_walks, wl.walk_seed)
        c1 = time.perf_counter()
        v0 = val[0]
        S, z = grf_oracle.buckets(K[0, 0], V[0, 0], rp, col, v0)
        num, den = grf_oracle.gather(Q[0, 0], rp, col, v0, S, z)
        c2 = time.perf_counter()
        t_sample, t_head = c1 - c0, c2 - c1
        cpu_step = t_sample + B * H * t_head
        # cross-check of the same head against the GPU output while the numbers are at hand
        gpu_head = out[0, 0].cpu().numpy().astype(np.float64)
        with np.errstate(divide="ignore", invalid="ignore"):
            ref_head = num / den[:, None]
        ok = np.isfinite(ref_head).all(axis=1) & (np.abs(den) > 1e-3 * np.abs(den).max())
        result["cpu_baseline"] = {
            "value": round(tokens / cpu_step, 2), "unit": "tokens/s/head", "cores": 1, "kind": "oracle",
            "sample": "sampling of all %d rows (%.2f s) + buckets and gather of 1 of the %d (batch, head) slices (%.2f s), "
                      "single thread; value = N*B*H / (t_sample + B*H*t_slice)" % (N, t_sample, B * H, t_head),
            "seconds_measured": round(t_sample + t_head, 2),
            "gpu_vs_oracle_out_maxabs_on_head0": float(np.abs(gpu_head[ok] - ref_head[ok]).max()),
        }

        # second line: the same checker, one thread per (batch, head) slice (the C routines release the interpreter lock)
        from concurrent.futures import ThreadPoolExecutor
        threads = min(B * H, 16)

        def one_slice(bh):
            b_, h_ = divmod(bh, H)
            vv = val[h_ if val.shape[0] > 1 else 0]
            S_, z_ = grf_oracle.buckets(K[b_, h_], V[b_, h_], rp, col, vv)
            grf_oracle.gather(Q[b_, h_], rp, col, vv, S_, z_)

        n_par = min(B * H, threads)
        p0 = time.perf_counter()
        with ThreadPoolExecutor(max_workers=threads) as pool:
            list(pool.map(one_slice, range(n_par)))
        p1 = time.perf_counter()
        par_step = t_sample + (p1 - p0) * (B * H) / n_par
        result["cpu_baseline"]["parallel"] = {"value": round(tokens / par_step, 2), "unit": "tokens/s/head", "cores": threads,
                                              "sample": "%d slices on %d threads in %.2f s, scaled to %d slices, plus the sampling time" % (n_par, threads, p1 - p0, B * H)}

    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
