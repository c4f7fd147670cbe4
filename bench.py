#!/usr/bin/env python3
"""Benchmark of the whole hot path on one MI355X.

One step = grf_sample (walks + CSR of Phi_hat), grf_form_buckets (column lists + buckets) and
grf_gather_buckets (gather, contraction, normalisation) on the headline workload: 32768 points in
16 Gaussian clusters, symmetrised 16-NN graph, 32 walks per node, p_halt = 0.2, f of length 16,
batch 1, 8 heads, d = 64, fp32.  Inputs are resident in HBM before the timed region.

Prints ONE JSON line.  `value` is tokens/s/head = N*B*H / step time (wall clock over the timed steps, sampler
included).  `attention_call` is the metric's own definition: the median device time of grf_masked_linear_attention
alone; `sampler` reports the walks in hops per second.  `roofline` is for the gather kernel (the dominant one):
algorithmic bytes per launch over its mean duration between HIP events recorded on the launch stream inside the timed
region; its `traffic` and the byte counts of the variants' rooflines come from profiles/hbm_traffic_per_launch.md.
`cpu_baseline` times the CPU checker on one head of the same workload on this machine's host cores.
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

# Bytes moved between L2 and the fabric per launch, counted by rocprofv3 --pmc runs of this file (FETCH_SIZE and
# WRITE_SIZE, scaled by what the same counters read for a plain copy): a stored measurement, read from the table that
# those runs produced, not recomputed here; kernels or workloads that the table does not hold report null.
TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic_per_launch.md")


def counted_traffic(workload, kernel_prefixes):
    """Sum over the table's rows of `workload` whose kernel name starts with one of `kernel_prefixes` of the bytes per
    launch (rows: | workload | kernel | read bytes | written bytes | total bytes |), or None."""
    total, found = 0, False
    try:
        for line in open(TRAFFIC_TABLE):
            cells = [c.strip() for c in line.strip().strip("|").split("|")]
            if len(cells) == 5 and cells[0] == workload and any(cells[1].startswith(k) for k in kernel_prefixes):
                total += int(cells[4]); found = True
    except OSError:
        return None
    return total if found else None


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
    traffic = counted_traffic(args.workload, ["grf::gather_kernel"])
    roofline = {"kernel": "gather_kernel", "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                "algorithmic_bytes_per_launch": gather_bytes, "avg_launch_ms": round(gather_ms, 4),
                "copy_1GiB_GBs": round(copy_gbs, 1), "frac_of_copy": round(achieved / copy_gbs, 4)}
    if traffic is not None:      # the counted bytes over the same time: the counter-based fraction of the HBM peak
        roofline["frac_counted"] = round(traffic / (gather_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
    if traffic is not None and traffic < 0.9 * gather_bytes:
        # a workload whose bucket records of one slice fit L2 re-reads them there: the algorithmic bytes are then a
        # cache rate, and the HBM fraction is the one of the bytes that were counted beyond L2
        counted = traffic / (gather_ms * 1e-3) / 1e9
        roofline.update({"achieved": round(counted, 1), "frac": round(counted / HBM_PEAK_GBS, 4),
                         "frac_of_copy": round(counted / copy_gbs, 4), "bytes": "counted beyond L2 (traffic)",
                         "requested_GBs": round(achieved, 1),
                         "note": "records re-read within a slice are served by L2; requested_GBs is the algorithmic rate"})

    def event_times(fn, steps=None, warmup=None):
        """Per-call device times of fn (ms): HIP events on the launch stream around each of `steps` calls."""
        steps = args.steps if steps is None else steps
        for _ in range(args.warmup if warmup is None else warmup):
            fn()
        torch.cuda.synchronize()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        for a, b in ev:
            a.record(stream); fn(); b.record(stream)
        torch.cuda.synchronize()
        return np.array([a.elapsed_time(b) for a, b in ev])

    def rate(nbytes, ms):
        return round(nbytes / (ms * 1e-3) / 1e9, 1)

    elem = 2 if wl.dtype == "bf16" else 4

    # ---- the attention call alone (column lists + buckets + gather), the quantity the metric is defined on: median of
    # the per-call device times
    aws = torch.empty(grf.grf_attention_workspace_bytes(B, H, N, d, nnz, phi.n_f), dtype=torch.uint8, device=dev)
    att = event_times(lambda: grf.grf_masked_linear_attention(Qd, Kd, Vd, phi, workspace=aws, out=out))
    del aws
    attention_call = {"entry_point": "grf_masked_linear_attention", "calls": int(att.size),
                      "median_ms": round(float(np.median(att)), 4), "mean_ms": round(float(att.mean()), 4),
                      "tokens_per_s_per_head": round(tokens / (float(np.median(att)) * 1e-3), 1)}

    # ---- the sampler: walk hops per second.  Hops are counted exactly from the trajectories (every entry >= 0 beyond a
    # walk's start is one hop); the call simulates every walk twice (count pass, fill pass).
    traj = grf.grf_sample_walks(g, wl.p_halt, wl.n_walks, wl.f_len, wl.walk_seed)
    hops = int((traj[:, :, 1:] >= 0).sum().item())
    del traj
    smp = event_times(lambda: grf.grf_sample(g, wl.f, wl.p_halt, wl.n_walks, wl.walk_seed, out=phi))
    sample_med = float(np.median(smp))
    # bound from the vector ALU: per hop and walk about 20 32-bit multiplies (Philox, two per round, ten rounds per two
    # hops; a quarter-rate instruction) and 45 full-rate integer/float instructions = 125 lane slots; 256 compute units x 4
    # SIMDs x 16 lanes x 2.4 GHz = 39.3e12 lane slots/s; two passes
    alu_hops_per_s = 39.3e12 / 125 / 2
    sampler = {"entry_point": "grf_sample", "median_ms": round(sample_med, 4), "hops": hops, "walks": N * wl.n_walks,
               "hops_per_s": round(hops / (sample_med * 1e-3), 1),
               "alu_bound_hops_per_s": round(alu_hops_per_s, 1), "frac_of_alu_bound": round(hops / (sample_med * 1e-3) / alu_hops_per_s, 4),
               "note": "bound by vector-instruction issue at low lane use (profiles/sampler_counters_cloud_32k.md): the walks of a node "
                       "hop in lock step, a wavefront executes every hop and Philox block while few of its lanes still walk, and the "
                       "kernel runs twice; includes the one host synchronisation that returns nnz"}

    # ---- the bucket-fused variant of the attention call on the same inputs: its own numbers, never `value`
    fws = torch.empty(grf.grf_fused_attention_workspace_bytes(B, H, N, d, nnz, phi.n_f), dtype=torch.uint8, device=dev)
    fout = torch.empty_like(out)
    fus = event_times(lambda: grf.grf_masked_linear_attention_fused(Qd, Kd, Vd, phi, workspace=fws, out=fout))
    fused_attn_ms = float(np.median(fus))
    prepared = grf.grf_phi_prepare(phi)
    prep_bytes = grf.grf_phi_prepare_bytes(N, nnz, phi.n_f)
    fus_p = event_times(lambda: grf.grf_masked_linear_attention_fused(Qd, Kd, Vd, phi, workspace=fws[prep_bytes:], out=fout, prepared=prepared))
    prep_ms = float(np.median(event_times(lambda: grf.grf_phi_prepare(phi, out=prepared))))
    # two contractions per entry of Phi_hat: S_l += a v^T and P = qw S_l, 2*d*d flops each
    fused_flops = 4.0 * nnz * d * d * B * H
    # compulsory HBM bytes of the call: Q, K, V read once, out written once, one partial row per entry of Phi_hat and slice
    # written by the bucket kernels and read back by the row reduction, Phi_hat and its column lists read per slice
    fused_compulsory = B * H * (3 * N * d * elem + N * d * 4 + 2 * nnz * (d + 1) * 4 + nnz * 16)
    fused_counted = counted_traffic(args.workload, ["grf::fused_bucket", "grf::gram_bucket_kernel<float, 3", "grf::gram_bucket_kernel<grf::bf16_t, 3", "grf::fused_reduce"])
    fused_bytes = fused_counted if fused_counted is not None else fused_compulsory
    fused = {
        "entry_point": "grf_masked_linear_attention_fused",
        "attention_ms": round(fused_attn_ms, 4), "attention_mean_ms": round(float(fus.mean()), 4),
        "attention_only_tokens_per_s_per_head": round(tokens / (fused_attn_ms * 1e-3), 1),
        "prepared": {"entry_point": "grf_masked_linear_attention_fused_prepared", "attention_ms": round(float(np.median(fus_p)), 4),
                     "attention_only_tokens_per_s_per_head": round(tokens / (float(np.median(fus_p)) * 1e-3), 1),
                     "grf_phi_prepare_ms": round(prep_ms, 4)},
        "roofline": {"bound": "hbm", "unit": "GB/s", "peak": HBM_PEAK_GBS,
                     "achieved": rate(fused_bytes, fused_attn_ms), "frac": round(rate(fused_bytes, fused_attn_ms) / HBM_PEAK_GBS, 4),
                     "bytes": "counted (profiles/hbm_traffic_per_launch.md: bucket kernels + row reduction)" if fused_counted is not None else "compulsory",
                     "bytes_per_call": fused_bytes, "compulsory_bytes_per_call": fused_compulsory,
                     "useful_flops_per_call": fused_flops, "useful_TFLOPs": round(fused_flops / (fused_attn_ms * 1e-3) / 1e12, 2),
                     "note": "whole call over the time of the whole call; rows of Q, K, V re-read per entry of Phi_hat are served by L2 / Infinity "
                             "Cache and are not HBM traffic; per-kernel times in profiles/"},
    }

    # ---- asymmetric GRFs (App. D): the same sampled matrix used directly as the mask estimate
    aout = torch.empty_like(out)
    asy = event_times(lambda: grf.grf_asymmetric_masked_attention(Qd, Kd, Vd, phi, out=aout))
    asym_ms = float(np.median(asy))
    asym_requested = B * H * (nnz * (2 * d * elem + 8) + N * d * (elem + 4))     # k_j, v_j, (col, val) per entry; q_i in, out_i out
    asym_compulsory = B * H * (3 * N * d * elem + N * d * 4 + nnz * 8)            # every tensor once
    asym_counted = counted_traffic(args.workload, ["grf::asymmetric_kernel"])
    asym_bytes = asym_counted if asym_counted is not None else asym_compulsory
    asymmetric = {
        "entry_point": "grf_asymmetric_masked_attention",
        "attention_ms": round(asym_ms, 4),
        "attention_only_tokens_per_s_per_head": round(tokens / (asym_ms * 1e-3), 1),
        "roofline": {"bound": "hbm", "unit": "GB/s", "peak": HBM_PEAK_GBS,
                     "achieved": rate(asym_bytes, asym_ms), "frac": round(rate(asym_bytes, asym_ms) / HBM_PEAK_GBS, 4),
                     "bytes": "counted (profiles/hbm_traffic_per_launch.md)" if asym_counted is not None else "compulsory",
                     "bytes_per_launch": asym_bytes, "compulsory_bytes_per_launch": asym_compulsory,
                     "requested_bytes_per_launch": asym_requested, "requested_GBs": rate(asym_requested, asym_ms),
                     "note": "requested = rows of K and V per entry of Phi_hat, most of which L2 serves (one head's K and V are 16.8 MB at the "
                             "headline size): a cache rate, not part of the HBM fraction"},
    }

    # ---- gradients (training with learnable f): backward of the attention call and of the sampler, on the fused
    # forward's saved out and den; six contractions of 2*nnz*d*d flops per slice
    _, _, fden = grf.grf_masked_linear_attention_fused(Qd, Kd, Vd, phi, workspace=fws, return_num_den=True, out=fout)
    d_out = torch.randn((B, H, N, d), dtype=torch.float32, device=dev, generator=torch.Generator(device=dev).manual_seed(0))
    bws = torch.empty(grf.grf_attention_backward_workspace_bytes(B, H, N, d, nnz, phi.n_f), dtype=torch.uint8, device=dev)

    def backward_step(prep=None):
        if prep is None:
            grads = grf.grf_masked_linear_attention_backward(Qd, Kd, Vd, phi, fout, fden, d_out, workspace=bws)
        else:
            grads = grf.grf_masked_linear_attention_backward(Qd, Kd, Vd, phi, fout, fden, d_out, workspace=bws[prep_bytes:], prepared=prep)
        return grf.grf_sample_backward(g, wl.f_len, wl.p_halt, wl.n_walks, wl.walk_seed, phi, grads[3])

    bwd = event_times(backward_step)
    bwd_p = event_times(lambda: backward_step(prepared))
    bwd_ms = float(np.median(bwd))
    bwd_flops = 12.0 * nnz * d * d * B * H
    # three passes, each writing one fp32 partial row per entry of Phi_hat and slice and reading it back; Q, K, V, out, den,
    # d_out read and dQ, dK, dV written once; the seed rows written and read per pass
    bwd_compulsory = B * H * (3 * 2 * nnz * d * 4 + 4 * nnz * 4 + 3 * N * d * elem + 5 * N * d * 4 + 4 * N * (d + 1) * 4 + nnz * 16)
    bwd_counted = counted_traffic(args.workload, ["grf::backward_", "grf::gram_bucket_kernel<float, 0", "grf::gram_bucket_kernel<float, 1", "grf::gram_bucket_kernel<float, 2",
                                                  "grf::gram_bucket_kernel<grf::bf16_t, 0", "grf::gram_bucket_kernel<grf::bf16_t, 1", "grf::gram_bucket_kernel<grf::bf16_t, 2",
                                                  "grf::dphi_accumulate", "grf::rows_kernel<2", "grf::df_reduce"])
    bwd_bytes = bwd_counted if bwd_counted is not None else bwd_compulsory
    backward = {
        "entry_points": "grf_masked_linear_attention_backward + grf_sample_backward",
        "ms": round(bwd_ms, 4), "mean_ms": round(float(bwd.mean()), 4),
        "tokens_per_s_per_head": round(tokens / (bwd_ms * 1e-3), 1),
        "prepared": {"entry_points": "grf_masked_linear_attention_backward_prepared + grf_sample_backward", "ms": round(float(np.median(bwd_p)), 4)},
        "roofline": {"bound": "hbm", "unit": "GB/s", "peak": HBM_PEAK_GBS,
                     "achieved": rate(bwd_bytes, bwd_ms), "frac": round(rate(bwd_bytes, bwd_ms) / HBM_PEAK_GBS, 4),
                     "bytes": "counted (profiles/hbm_traffic_per_launch.md: all kernels of both calls)" if bwd_counted is not None else "compulsory",
                     "bytes_per_call": bwd_bytes, "compulsory_bytes_per_call": bwd_compulsory,
                     "useful_flops_per_call": bwd_flops, "useful_TFLOPs": round(bwd_flops / (bwd_ms * 1e-3) / 1e12, 2),
                     "note": "whole backward (seed, column lists, three bucket passes with their row reductions, dphi, df) over its whole time; "
                             "per-kernel times in profiles/"},
    }

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
        "attention_call": attention_call,
        "sampler": sampler,
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
