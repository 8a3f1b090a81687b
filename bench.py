"""Benchmark of one decode step (the whole hot path over one batch of synthetic input).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3_62b] [--no-graph]

Prints ONE JSON line.  `value` is the achieved algorithmic HBM rate of the whole
step (int8 weight bytes + KV bytes read, per second) with every input already
resident in HBM; `ms_per_step` is the decode latency.  `roofline` covers the
dominant kernel (the fused input projection), timed with HIP events on the
stream it runs on, in a second pass of the same K steps so that the events do
not perturb `value`.  `cpu_baseline` times the fp64 oracle on a bounded sample
of the same workload on this machine's host cores.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X HBM3E, published


def cpu_baseline(w, stack_rows=4, seconds_budget=20.0):
    """The oracle as it stands on `stack_rows` batch rows through as many layers
    as fit the time budget; rows and layers scale the cost linearly."""
    import numpy as np
    import torch
    import oracle
    from workloads import synth
    from workloads import configs as C

    R = min(stack_rows, w.batch)
    desc = oracle.make_desc(w)
    pos_all = synth.positions(w, "cpu").numpy()
    pos = pos_all[:R]
    x = oracle.bf16_bits_to_f64_fast(
        synth.hidden_state(w, "cuda").cpu().view(torch.int16).numpy().view(np.uint16)[:R])
    spent, layers_done = 0.0, 0
    for l in range(w.n_layers):
        wts = {n: t.cpu() for n, t in synth.layer_weights(w, l, "cuda").items()}
        k, v = synth.kv_layer(w, l, "cuda", batch=R)
        kc = k.cpu().view(torch.int16).numpy().view(np.uint16).copy()
        vc = v.cpu().view(torch.int16).numpy().view(np.uint16).copy()
        t0 = time.perf_counter()
        oracle.decode_layer(desc, wts, kc, vc, pos, x, w.l_ctx)
        spent += time.perf_counter() - t0
        layers_done += 1
        if spent >= seconds_budget:
            break
    est_step_s = spent * (w.batch / R) * (w.n_layers / layers_done)
    bytes_step = C.algorithmic_bytes(w, pos_all.tolist())
    return {
        "value": bytes_step / est_step_s / 1e9,
        "unit": "GB/s",
        "cores": oracle.num_threads(),
        "kind": "oracle",
        "ms_per_step_extrapolated": est_step_s * 1e3,
        "sample": (f"{R} of {w.batch} batch rows through {layers_done} of {w.n_layers} layers in "
                   f"{spent:.1f} s of oracle time, scaled linearly in rows and layers (extrapolated)"),
    }


# HBM bytes one launch of the input projection moves, from the rocprofv3 FETCH_SIZE / WRITE_SIZE passes
# summarised in profiles/hbm_traffic_pmc_c3_62b_layer.txt (counters scaled by a plain 1 GiB copy):
# (306898.5 * 2.0 + 29696.0 * 1.0) KiB.  Other workloads: not measured.
TRAFFIC_BYTES_PER_LAUNCH = {"c3_62b": int((306898.5 * 2.0 + 29696.0) * 1024)}


def time_workload(w, steps, warmup):
    """Graph-replay time of one decode step of workload `w` (all inputs resident)."""
    import torch
    from workloads import configs as C
    from paper_2211_05102_amd import harness
    st = harness.DeviceStack(w)
    positions = st.positions.cpu().tolist()
    bytes_step = C.algorithmic_bytes(w, positions)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        st.dec.graph_capture(st.packed, st.k_cache, st.v_cache, st.x_in, st.positions, w.l_ctx,
                             st.x_out, st.workspace, stream)
        for _ in range(warmup):
            st.dec.graph_replay(stream)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            st.dec.graph_replay(stream)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / steps
        st.dec.check_async(st.workspace, stream)
    st.dec.graph_release()
    del st
    torch.cuda.empty_cache()
    gbps = bytes_step / dt / 1e9
    return {"ms_per_step": dt * 1e3, "GB/s": gbps, "hbm_peak_frac": gbps / HBM_PEAK_GBPS,
            "tokens_per_s": w.batch / dt}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c3_62b")
    ap.add_argument("--layers", type=int, default=0,
                    help="run a shorter stack of the same layer shape (kernel tuning; not the headline workload)")
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--gemm-wg-in", type=int, default=0)
    ap.add_argument("--gemm-wg-out", type=int, default=0)
    ap.add_argument("--attn-bps", type=int, default=0)
    ap.add_argument("--act-digits", type=int, default=0)
    ap.add_argument("--all-configs", action="store_true",
                    help="also time the other named workloads (graph replay, 5 steps each) and add them to the "
                         "JSON line as per_config; the headline value stays the --workload one")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three plain 1 GiB device copies (reference for scaling rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters in the --pmc passes)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus must be 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from workloads import WORKLOADS
    from workloads import configs as C
    from paper_2211_05102_amd import harness

    w = WORKLOADS[args.workload]
    if args.layers:
        w = w.with_(n_layers=args.layers, name=f"{w.name}[{args.layers} layers]")
    t_setup = time.perf_counter()
    st = harness.DeviceStack(w)
    for name, val in (("gemm_workgroups_in", args.gemm_wg_in), ("gemm_workgroups_out", args.gemm_wg_out),
                      ("attn_blocks_per_split", args.attn_bps), ("act_digits", args.act_digits)):
        if val:
            st.dec.set_option(name, val)
    torch.cuda.synchronize()
    t_setup = time.perf_counter() - t_setup
    positions = st.positions.cpu().tolist()
    bytes_step = C.algorithmic_bytes(w, positions)
    flops_step = C.algorithmic_flops(w, positions)

    stream = torch.cuda.Stream()
    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(3)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    use_graph = not args.no_graph
    with torch.cuda.stream(stream):
        if use_graph:
            st.dec.graph_capture(st.packed, st.k_cache, st.v_cache, st.x_in, st.positions, w.l_ctx,
                                 st.x_out, st.workspace, stream)

        def one_step():
            if use_graph:
                st.dec.graph_replay(stream)
            else:
                st.step(stream)

        for _ in range(args.warmup):
            one_step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            one_step()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        st.dec.check_async(st.workspace, stream)

        # second pass: the same K steps, eager launches, events around the dominant kernel
        st.dec.set_option("profile_kernel", 1)
        for _ in range(args.steps):
            st.step(stream)
        torch.cuda.synchronize()
        k_ms, k_launches = st.dec.profile_read()
        per_kernel = {}
        for code, kname in ((2, "attention"), (3, "qgemm_out"), (4, "epi_in"), (5, "epi_out")):
            st.dec.set_option("profile_kernel", code)
            for _ in range(max(2, args.steps // 4)):
                st.step(stream)
            torch.cuda.synchronize()
            ms, n = st.dec.profile_read()
            per_kernel[kname] = {"avg_us": 1e3 * ms / max(n, 1), "launches": n}
        st.dec.set_option("profile_kernel", 0)

    ms_per_step = elapsed * 1e3 / args.steps
    gbps = bytes_step / (elapsed / args.steps) / 1e9
    k_avg_s = k_ms * 1e-3 / max(k_launches, 1)
    k_bytes = w.d_model * w.n_in  # int8 weight bytes the input projection streams per launch
    k_gbps = k_bytes / k_avg_s / 1e9
    per_kernel["qgemm_in"] = {"avg_us": k_avg_s * 1e6, "launches": k_launches}

    out = {
        "metric": "decode_achieved_hbm_bandwidth_int8_mqa",
        "value": gbps,
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "tokens_per_s": w.batch / (ms_per_step * 1e-3),
        "hbm_peak_frac": gbps / HBM_PEAK_GBPS,
        "algorithmic_bytes_per_step": bytes_step,
        "algorithmic_flops_per_step": flops_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int8",  # int8 x int8 -> int32 MFMA on block fixed-point activations; fp32 folds and softmax
        "data": "synthetic",
        "config": {"workload": w.name, "n_layers": w.n_layers, "d_model": w.d_model,
                   "n_heads": w.n_heads, "d_head": w.d_head, "d_ff": w.d_ff, "batch": w.batch,
                   "kv_len": w.l_ctx, "positions": w.positions, "weights": "int8 per-channel",
                   "launch": "hipGraph replay" if use_graph else "eager", "setup_s": round(t_setup, 1)},
        "roofline": {"bound": "hbm", "kernel": "qgemm_kernel (fused input projection)",
                     "achieved": k_gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": k_gbps / HBM_PEAK_GBPS, "traffic": TRAFFIC_BYTES_PER_LAUNCH.get(args.workload),
                     "bytes_per_launch": k_bytes, "avg_launch_us": k_avg_s * 1e6},
        "kernels": per_kernel,
    }
    del st
    torch.cuda.empty_cache()
    if args.all_configs:
        out["per_config"] = {w.name: {"ms_per_step": ms_per_step, "GB/s": gbps, "hbm_peak_frac": gbps / HBM_PEAK_GBPS}}
        for name in ("c1_tiny", "c2_8b", "c4_540b_shard8", "c5_62b_long"):
            if name == args.workload:
                continue
            out["per_config"][name] = time_workload(WORKLOADS[name], steps=5, warmup=2)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
