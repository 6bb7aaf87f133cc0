#!/usr/bin/env python3
"""Benchmark of the decomposed CLIP contrastive loss (fwd+bwd) on one MI355X.

One step = the whole hot path for every simulated rank of the workload: for r = 0..N-1 one
disco_loss_fwd_bwd call (two logit blocks, row softmax cross-entropy, the four gradient
contractions, d/ds) accumulated on device into the same gI/gT/loss/gs, which stands in for
the all_reduce of Eq. 7.  Inputs are synthetic (synth/features.py), resident in HBM before timing.

Prints ONE JSON line.  `value` = pairs per second = B / t_step (equal to b / t_rank, the "samples/s
per rank share" of the metric).  `roofline` is for the dominant kernel (the logit-tile kernel),
timed live with HIP events recorded by the library between its stages.
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_FP32_TFLOPS = 157.3      # MI355X fp32, matrix and (packed) vector alike

# The paper's own figure where it reports this metric on this workload (context: another machine).  Table 4:
# loss computation 1.6 ms + loss back-propagation 2.8 ms per iteration and GPU at 512 pairs per GPU of a
# 32,768 batch (64 A100, mixed precision) = 512 / 4.4 ms pairs per second per rank share.
PAPER_SAMPLES_PER_S = {"b32k_n64": 512 / 4.4e-3}
PATH_NAMES = {1: "naive", 2: "materialized", 3: "fused", 4: "symmetric"}

# HBM bytes per launch of the dominant kernel, from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs whose
# summaries are profiles/<workload>_hbm_traffic.txt (counters cannot be read from inside this process; the fetch
# part varies by about a quarter from run to run with what the last-level cache still holds).  Workloads and
# paths without such a summary report null on purpose.
MEASURED_TRAFFIC_BYTES = {("b32k_n8", "materialized", "logit_tiles"): 8.962e8,
                          ("b196k_n64", "materialized", "logit_tiles"): 3.509e9,
                          ("b64k_d768_n8", "materialized", "logit_tiles"): 4.590e9,
                          ("full_n1", "symmetric", "logit_tiles_row_and_column_sums"): 3.930e9}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="b32k_n8")
    ap.add_argument("--path", default="auto", choices=["auto", "naive", "materialized", "fused", "symmetric"])
    ap.add_argument("--ranks", default="all", help="'all' (every simulated rank per step) or one rank index")
    ap.add_argument("--features", default="config", choices=["config", "f32"],
                    help="'f32': hand the workload's features over in fp32 whatever its dtype (they then take the fp32 path)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true", help="capture one step (all rank calls) in a graph and time its replays")
    ap.add_argument("--op", default="loss", choices=["loss", "prep", "mfma-peak"],
                    help="'loss': the hot path (default, the headline line); 'prep': the feature normalisation "
                         "forward + backward on both feature matrices of the workload (HBM-bound, reported in GB/s)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 1 GiB device copy three times (to calibrate FETCH_SIZE / WRITE_SIZE) and exit")
    return ap.parse_args()


class HipEvents:
    """hipEvent_t handles created through the HIP runtime already loaded by torch."""

    def __init__(self, n, only=None):
        """n handles; with `only` (a set of indices) the other entries stay NULL and the library skips them."""
        # (events released to device scope: a default event has the stream write the L2 back for the host at
        # every record)
        self.hip = ctypes.CDLL("libamdhip64.so.7") if _loaded("libamdhip64.so.7") else ctypes.CDLL("libamdhip64.so")
        self.n = n
        self.arr = (ctypes.c_void_p * n)()
        for i in range(n):
            if only is not None and i not in only:
                continue
            ev = ctypes.c_void_p()
            assert self.hip.hipEventCreateWithFlags(ctypes.byref(ev), ctypes.c_uint(0x40000000)) == 0
            self.arr[i] = ev

    def elapsed_ms(self, a, b):
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), ctypes.c_void_p(self.arr[a]), ctypes.c_void_p(self.arr[b]))
        assert rc == 0, rc
        return ms.value


def _loaded(name):
    try:
        with open("/proc/self/maps") as f:
            return any(name in line for line in f)
    except OSError:
        return False


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; the N ranks of the workload are simulated on it "
              "(--gpus must be 1)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    if args.copy_calibration:
        a = torch.ones(1 << 28, dtype=torch.int32, device="cuda:0")
        b = torch.zeros_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes": a.numel() * 4, "copies": 3}))
        return

    import paper_2304_08480_amd as dl
    from synth import CONFIGS, make_config_inputs

    if args.op == "prep":
        return bench_prep(args, dl, CONFIGS[args.config], np, torch)
    if args.op == "mfma-peak":
        return bench_mfma_peak(args, dl, np, torch)

    cfg = CONFIGS[args.config]
    B, d, N, b, s = cfg.B, cfg.d, cfg.N, cfg.b, cfg.s
    path = {"auto": dl.DISCO_PATH_AUTO, "naive": dl.DISCO_PATH_NAIVE, "materialized": dl.DISCO_PATH_MATERIALIZED,
            "fused": dl.DISCO_PATH_FUSED, "symmetric": dl.DISCO_PATH_SYMMETRIC}[args.path]
    I, T, Ib, Tb = make_config_inputs(cfg)
    dev = torch.device("cuda:0")
    feat_dtype = "f32" if args.features == "f32" else cfg.dtype
    if feat_dtype == "bf16":
        Id = torch.from_numpy(Ib.view(np.int16)).to(dev)
        Td = torch.from_numpy(Tb.view(np.int16)).to(dev)
        dt = dl.DISCO_BF16
    else:
        Id, Td, dt = torch.from_numpy(I).to(dev), torch.from_numpy(T).to(dev), dl.DISCO_F32
    resolved = dl.disco_resolve_path(B, d, N, dt, path)
    assert resolved > 0, dl.disco_status_string(-resolved)
    ws_bytes = dl.disco_workspace_bytes(B, d, N, dt, path)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    loss = torch.zeros(1, device=dev)
    gs = torch.zeros(1, device=dev)
    gI = torch.zeros(B, d, device=dev)
    gT = torch.zeros(B, d, device=dev)
    ranks = list(range(N)) if args.ranks == "all" else [int(args.ranks)]
    stream = torch.cuda.current_stream()

    def step():
        for n, r in enumerate(ranks):
            dl.disco_loss_fwd_bwd(Id, Td, B, d, r, N, s, dt, path, 1 if n > 0 else 0, loss, gI, gT, gs, ws, ws_bytes, stream)

    nstages = {dl.DISCO_PATH_MATERIALIZED: 6, dl.DISCO_PATH_SYMMETRIC: 7}.get(resolved, 5)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    run_step = step
    if args.graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            dl_stream = torch.cuda.current_stream()
            for n, r in enumerate(ranks):
                dl.disco_loss_fwd_bwd(Id, Td, B, d, r, N, s, dt, path, 1 if n > 0 else 0, loss, gI, gT, gs, ws, ws_bytes, dl_stream)
        run_step = graph.replay
        run_step()
        torch.cuda.synchronize()

    # timed region: exactly `steps` steps, no stage events (they cost about 2 % between kernels); one event
    # between steps gives the per-step times for the median and the minimum
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    torch.cuda.synchronize()
    wall0 = time.perf_counter()
    marks[0].record(stream)
    for k in range(args.steps):
        run_step()
        marks[k + 1].record(stream)
    torch.cuda.synchronize()
    wall1 = time.perf_counter()
    total_ms = marks[0].elapsed_time(marks[-1])
    step_ms = sorted(marks[k].elapsed_time(marks[k + 1]) for k in range(args.steps))

    # stage intervals: the same steps again with the library recording HIP events between its stages on the
    # stream it launches on.  Every rank call gets an event set of its own and nothing synchronises until all calls
    # of `stage_steps` steps are enqueued, so that the kernels run in the same back-to-back stream (same clocks) as
    # in the timed region; averaged over every rank call.  An event between two kernels keeps the second from being
    # set up under the first one's tail: the intervals add up to 5-8 % more than a call takes without them.  They are
    # therefore scaled by (time of a call without events) / (their sum), which brings each within a few per cent of
    # the kernel durations that rocprofv3 --kernel-trace reports for the same stream (profiles/).
    dom_stage = {dl.DISCO_PATH_MATERIALIZED: 1, dl.DISCO_PATH_SYMMETRIC: 1, dl.DISCO_PATH_FUSED: 3}.get(resolved)
    stage_steps = min(args.steps, 3)
    sets = [HipEvents(nstages + 1) for _ in range(stage_steps * len(ranks))]
    k = 0
    for _ in range(stage_steps):
        for n, r in enumerate(ranks):
            dl.disco_set_stage_events(sets[k].arr, sets[k].n)
            dl.disco_loss_fwd_bwd(Id, Td, B, d, r, N, s, dt, path, 1 if n > 0 else 0, loss, gI, gT, gs, ws, ws_bytes, stream)
            k += 1
    torch.cuda.synchronize()
    dl.disco_set_stage_events(None, 0)
    stage_raw = np.zeros(nstages)
    for e in sets:
        stage_raw += np.array([e.elapsed_ms(i, i + 1) for i in range(nstages)])
    stage_raw /= len(sets)
    stage_avg = stage_raw * ((total_ms / args.steps / len(ranks)) / stage_raw.sum())
    if dom_stage is None:
        dom_stage = int(np.argmax(stage_avg))

    ms_per_step = total_ms / args.steps
    calls_per_step = len(ranks)
    ms_per_rank = ms_per_step / calls_per_step
    pairs_per_step = b * calls_per_step
    value = pairs_per_step / (ms_per_step * 1e-3)
    # algorithmic flops of one call: 12 b B d for a rank's two blocks; the non-decomposed loss (N = 1) needs one
    # similarity matrix for both directions, 6 B^2 d.  Executed: what the path that ran multiplies.
    alg_flops_rank = 6.0 * B * B * d if N == 1 else 12.0 * b * B * d
    exec_flops_rank = {dl.DISCO_PATH_SYMMETRIC: 6.0, dl.DISCO_PATH_FUSED: 16.0}.get(resolved, 12.0) * b * B * d
    tflops_alg = alg_flops_rank / (ms_per_rank * 1e-3) / 1e12
    tflops_exec = exec_flops_rank / (ms_per_rank * 1e-3) / 1e12

    if resolved == dl.DISCO_PATH_MATERIALIZED:
        names = ["prep", "logit_tiles", "merge_transpose", "key_grad_gemm", "query_split_gemm", "finalize_scalars"]
        dom = 1
        dom_flops = 4.0 * b * B * d                 # both blocks: 2 * (2 b B d)
        peak, bound, unit = PEAK_BF16_TFLOPS, "mfma", "TFLOP/s"
        dtype = "bf16"
    elif resolved == dl.DISCO_PATH_SYMMETRIC:
        names = ["prep", "logit_tiles_row_and_column_sums", "merge_transpose", "combine", "key_grad_gemm", "query_split_gemm",
                 "finalize_scalars"]
        dom = 1
        dom_flops = 2.0 * B * B * d                 # one similarity matrix
        peak, bound, unit = PEAK_BF16_TFLOPS, "mfma", "TFLOP/s"
        dtype = "bf16"
    elif resolved == dl.DISCO_PATH_FUSED:
        names = ["prep", "streaming_forward", "merge_transpose", "panel_recompute_and_gemms", "finalize_scalars"]
        dom = 3
        dom_flops = 12.0 * b * B * d                # recompute (4) + key side (4) + query side (4), both blocks
        peak, bound, unit = PEAK_BF16_TFLOPS, "mfma", "TFLOP/s"
        dtype = "bf16"
    else:
        names = ["similarity", "row_softmax", "scalars", "key_grad", "query_grad"]
        dom = dom_stage
        dom_flops = 4.0 * b * B * d
        # fp32 features run on the fp32 matrix instruction, bf16 features partly on the vector ALUs: the published
        # peak is the same number for both
        peak, bound, unit = PEAK_FP32_TFLOPS, ("mfma" if feat_dtype != "bf16" else "alu"), "TFLOP/s"
        dtype = "f32"
    dom_ms = float(stage_avg[dom])
    achieved = dom_flops / (dom_ms * 1e-3) / 1e12
    roofline = {
        "bound": bound, "kernel": names[dom], "achieved": round(achieved, 2), "peak": peak, "unit": unit,
        "frac": round(achieved / peak, 4),
        "traffic": MEASURED_TRAFFIC_BYTES.get((cfg.name, PATH_NAMES[resolved], names[dom])),
        "avg_launch_ms": round(dom_ms, 4), "flops_per_launch": dom_flops,
        "stages_ms": {n: round(float(v), 4) for n, v in zip(names, stage_avg)},
        "stage_event_overhead": round(float(stage_raw.sum() / stage_avg.sum()) - 1.0, 4),
    }

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import clip_oracle as oc
        t0 = time.perf_counter()
        n_cpu = 0
        for r in ranks:                       # the oracle as it stands, one rank at a time, for about 10-30 s
            ref = oc.disco_rank(I, T, s, r, N)
            n_cpu += 1
            if time.perf_counter() - t0 > 12.0:
                break
        t_cpu = time.perf_counter() - t0
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count()
        cpu = {"value": round(n_cpu * b / t_cpu, 2), "unit": "samples/s", "cores": cores, "kind": "oracle",
               "sample": f"float64 oracle, {n_cpu} rank call(s) of the workload ({b} pairs x {B} keys each), {t_cpu:.2f} s"}

    out = {
        "metric": "contrastive loss fwd+bwd samples/s per rank share",
        "value": round(value, 1), "unit": "samples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": (round(value / PAPER_SAMPLES_PER_S[cfg.name], 2) if cfg.name in PAPER_SAMPLES_PER_S else None),
        "dtype": dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "B": B, "d": d, "N_simulated_ranks": N, "b": b, "s": round(s, 6),
                   "features": feat_dtype, "ranks_per_step": calls_per_step, "path": PATH_NAMES[resolved],
                   "launch": "graph replay" if args.graph else "eager",
                   "workspace_bytes": ws_bytes},
        "ms_per_step_median": round(step_ms[len(step_ms) // 2], 4), "ms_per_step_min": round(step_ms[0], 4),
        "ms_per_rank_call": round(ms_per_rank, 4),
        "tflops_algorithmic": round(tflops_alg, 2), "tflops_executed": round(tflops_exec, 2),
        "frac_of_bf16_mfma_peak_algorithmic": round(tflops_alg / PEAK_BF16_TFLOPS, 4),
        "wall_ms_per_step": round((wall1 - wall0) * 1e3 / args.steps, 4),
        "loss": float(loss.item()),
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


def bench_mfma_peak(args, dl, np, torch):
    """What the matrix cores sustain with every compute unit issuing bf16 MFMAs from registers and nothing else
    (no memory traffic), after `warmup` launches of about 5 ms each, and the shader clock meanwhile.  This is the
    ceiling the clock management leaves under the published 2.5 PFLOP/s; the tile kernels work against it."""
    dev = torch.device("cuda:0")
    cus = torch.cuda.get_device_properties(dev).multi_processor_count
    sink = torch.zeros(1, device=dev)
    clocks = torch.zeros(2, dtype=torch.int64, device=dev)
    stream = torch.cuda.current_stream()
    iters = 40000                                   # x 8 MFMAs x 32768 flop per wave
    rows = []
    for varied, wgs in ((0, cus), (1, cus // 4), (1, cus)):   # quiet operands; then data-like ones on a quarter and on all of the chip
        for _ in range(max(args.warmup, 20)):
            dl.disco_mfma_probe(wgs, iters, varied, sink, clocks, stream)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record(stream)
        for _ in range(args.steps):
            dl.disco_mfma_probe(wgs, iters, varied, sink, clocks, stream)
        b.record(stream)
        torch.cuda.synchronize()
        ms = a.elapsed_time(b) / args.steps
        c = clocks.cpu().numpy()
        flops = wgs * 8 * iters * 8 * 32768.0
        rows.append({"operands": "sign, exponent and mantissa vary" if varied else "mantissa varies only", "workgroups": wgs,
                     "ms_per_launch": round(ms, 4), "tflops": round(flops / (ms * 1e-3) / 1e12, 1),
                     "shader_clock_mhz": round(100.0 * float(c[0]) / float(c[1]), 1)})
    full = rows[-1]
    out = {"metric": "bf16 MFMA issue rate, registers only, all compute units", "value": full["tflops"], "unit": "TFLOP/s",
           "n_gpus": 1, "steps": args.steps, "warmup": max(args.warmup, 20), "ms_per_step": full["ms_per_launch"],
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": "mfma-peak", "compute_units": cus, "waves_per_simd": 2, "mfma": "v_mfma_f32_32x32x16_bf16"},
           "runs": rows,
           "roofline": {"bound": "mfma", "kernel": "k_mfma_probe", "achieved": full["tflops"], "peak": PEAK_BF16_TFLOPS,
                        "unit": "TFLOP/s", "frac": round(full["tflops"] / PEAK_BF16_TFLOPS, 4), "traffic": None},
           "cpu_baseline": None}
    print(json.dumps(out))


def bench_prep(args, dl, cfg, np, torch):
    """Row L2 normalisation of raw fp32 features to bf16 (forward) and the projection of the fp32 feature
    gradients back through it (backward), for both matrices of the workload.  Algorithmic bytes per element:
    forward 4 read + 2 written, backward 4 + 4 read + 4 written (plus 4 per row for the norms)."""
    B, d = cfg.B, cfg.d
    dev = torch.device("cuda:0")
    g = torch.Generator(device="cpu").manual_seed(cfg.seed)
    X = [torch.randn(B, d, generator=g).mul_(2.0).to(dev) for _ in range(2)]
    G = [torch.randn(B, d, generator=g).mul_(1e-5).to(dev) for _ in range(2)]
    U = [torch.empty((B, d), dtype=torch.int16, device=dev) for _ in range(2)]
    inv = [torch.empty(B, device=dev) for _ in range(2)]
    DX = [torch.empty((B, d), device=dev) for _ in range(2)]
    stream = torch.cuda.current_stream()

    def fwd():
        for z in range(2):
            dl.disco_normalize_fwd(X[z], B, d, dl.DISCO_F32, U[z], dl.DISCO_BF16, inv[z], stream)

    def bwd():
        for z in range(2):
            dl.disco_normalize_bwd(G[z], X[z], dl.DISCO_F32, inv[z], B, d, DX[z], stream)

    def timed(f):
        for _ in range(args.warmup):
            f()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record(stream)
        for _ in range(args.steps):
            f()
        b.record(stream)
        torch.cuda.synchronize()
        return a.elapsed_time(b) / args.steps

    t_f, t_b = timed(fwd), timed(bwd)
    by_f = 2 * (B * d * 6 + B * 4)
    by_b = 2 * (B * d * 12 + B * 4)
    gbs = (by_f + by_b) / ((t_f + t_b) * 1e-3) / 1e9
    out = {
        "metric": "feature normalisation fwd+bwd, both matrices", "value": round(gbs, 1), "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(t_f + t_b, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": cfg.name, "B": B, "d": d, "in": "f32", "out": "bf16"},
        "forward_ms": round(t_f, 4), "backward_ms": round(t_b, 4),
        "roofline": {"bound": "hbm", "kernel": "normalize_fwd + normalize_bwd", "achieved": round(gbs, 1), "peak": 8000.0,
                     "unit": "GB/s", "frac": round(gbs / 8000.0, 4), "traffic": None,
                     "forward_GBps": round(by_f / (t_f * 1e-3) / 1e9, 1), "backward_GBps": round(by_b / (t_b * 1e-3) / 1e9, 1)},
        "cpu_baseline": None,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
