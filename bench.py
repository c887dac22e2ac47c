#!/usr/bin/env python3
"""Benchmark of the DRACO encode/decode hot path on one MI355X.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config i]

A step is one pass of the whole hot path over one batch of synthetic gradient
slabs already resident in HBM: the encoder of all P nodes (G -> Z), then the
parameter-server decoder on the received messages R (Z with the workload's
adversarial rows), through the synchronous C-ABI entry points (sum left on the
device, mask and status on the host).  The metric is the benchmark contract's
"decoded gradient GB/s consumed": P*d*4 bytes per step divided by the step
time.  One JSON line is printed; it also carries the roofline of the dominant
kernel (HIP-event durations recorded by the library on the launch stream) and
the CPU oracle timed on a bounded sample on this machine's host cores.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak
KIND_NAMES = ["encode", "vote", "project", "recombine"]

# HBM bytes per launch divided by the algorithmic bytes, from rocprofv3 --pmc
# FETCH_SIZE / WRITE_SIZE runs of this file, each counter scaled by what it
# reads for the library's plain copy kernel (fetch x2.0000, write x0.9995);
# the figures are in profiles/<workload>_kernels.md.
MEASURED_TRAFFIC_RATIO = {
    "rep_P45_s2_d11.2M": {"encode": 0.9998, "vote": 1.0000},
    "cyc_P45_s3_d25.6M": {"encode": 0.9999, "project": 1.0022, "recombine": 1.0000},
}


def algorithmic_bytes(w, mlen, n_honest, wide=False):
    """Bytes each kernel must move per launch (every input read once, every output written once).
    On the wide wire every message float is two fp32 words."""
    P, d, h = w.P, w.d, mlen // 2   # h: complex entries per message = entries of f
    words = 2 if wide else 1
    return {
        "encode": (P * d + words * P * mlen) * 4,
        "vote": (P * d + d) * 4,
        "project": (words * P * mlen + h) * 4,
        "recombine": (words * n_honest * mlen + d) * 4,
    }


def cpu_baseline(w):
    """The oracle as it stands, on a slice of the same workload sized for ~10-30 s."""
    import numpy as np
    import psutil
    import torch

    from oracle import draco_oracle as o
    from paper_1803_09877_amd import synth

    d_s = min(w.d, 8_000_000 if w.code == "cyc" else 16_000_000)
    ws = synth.scaled(w, d_s)
    G = synth.make_gradients(ws.P, d_s, ws.sigma, ws.seed, device="cpu")[:, :d_s].numpy()
    f = synth.make_projection((d_s + 1) // 2, ws.seed).numpy()
    proc = psutil.Process()
    c0 = proc.cpu_times()
    t_enc = t_dec = 0.0
    reps = 0
    while reps < 20 and (reps == 0 or t_enc + t_dec < 10.0):      # about 10 s of oracle work
        t0 = time.perf_counter()
        if ws.code == "rep":
            Z = o.encode_repetition(G, ws.s).astype(np.float32)
        else:
            Z = o.encode_cyclic(G, ws.s).astype(np.float32)
        t_enc += time.perf_counter() - t0
        R = torch.from_numpy(Z)
        synth.apply_attacks(R, Z.shape[1], ws.adversaries(), ws.seed)
        if ws.decode:
            t1 = time.perf_counter()
            if ws.code == "rep":
                _, mask, st = o.decode_repetition(R.numpy(), ws.s)
            else:
                _, mask, st = o.decode_cyclic(R.numpy(), f, ws.s, d_s)
            t_dec += time.perf_counter() - t1
            assert st == 0 and sorted(np.flatnonzero(mask)) == sorted(j for j, _ in ws.adversaries())
        reps += 1
    c1 = proc.cpu_times()
    wall = t_enc + t_dec
    busy = (c1.user + c1.system) - (c0.user + c0.system)
    return {
        "value": reps * ws.P * d_s * 4 / wall / 1e9,
        "unit": "GB/s",
        "cores": max(1, round(busy / max(wall, 1e-9))),
        "cores_available": len(os.sched_getaffinity(0)),
        "kind": "oracle",
        "sample": f"same recipe at d={d_s} (of {w.d}), P={ws.P}, s={ws.s}, {reps} passes; "
                  f"per pass encode {t_enc / reps:.2f} s + decode {t_dec / reps:.2f} s",
        "encode_s": t_enc / reps,
        "decode_s": t_dec / reps,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=1, help="index into the five benchmark workloads (default 1)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--wide", action="store_true", help="cyclic workloads on the two-word (hi+lo) wire")
    ap.add_argument("--unpacked", action="store_true",
                    help="cyclic workloads on the unpacked wire (d complex entries per message)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the P nodes are message slabs in one GPU's HBM); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_1803_09877_amd import binding as B
    from paper_1803_09877_amd import synth
    from paper_1803_09877_amd.runner import Case

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    w = synth.WORKLOADS[args.config]
    c = Case(w, "cuda:0", wide=args.wide, unpacked=args.unpacked)
    c.encode()
    c.receive()
    torch.cuda.synchronize()
    n_honest = w.P - len(c.adversaries)
    if w.decode:
        mask, status = c.decode()
        assert status == 0 and np.array_equal(mask, c.expected_mask()), "decode did not find the planted adversaries"

    # copy-kernel ceiling of this GPU on the same slabs (R -> Z, which the next encode overwrites)
    ld = c.ld_m
    row_len = c.mlen // 4 * 4

    def copy_once():
        B.draco_copy_probe(c.R, c.Z, w.P, row_len, ld)

    for _ in range(2):
        copy_once()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(5):
        copy_once()
    ev1.record()
    torch.cuda.synchronize()
    copy_gbps = 2 * 4 * w.P * row_len * 5 / (ev0.elapsed_time(ev1) * 1e-3) / 1e9

    for _ in range(args.warmup):
        c.step()
    c.plan.set_timing(args.steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        c.step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    kernel_times = [c.plan.kernel_time(kind) for kind in range(len(KIND_NAMES))]

    # The same step through the stream-ordered entry points (mask and status stay on the
    # device, read once after the K steps), eagerly and as one captured HIP graph per step.
    extra = {}
    if w.decode:
        mask_dev = torch.zeros(4, dtype=torch.int64, device=c.device)
        status_dev = torch.zeros(1, dtype=torch.int32, device=c.device)

        def async_step():
            c.encode()
            if w.code == "rep":
                c.plan.decode_repetition_async(c.R, c.u, mask_dev, status_dev)
            elif args.wide:
                c.plan.decode_cyclic_wide_async(c.R, c.Rlo, c.f, c.u, mask_dev, status_dev)
            else:
                c.plan.decode_cyclic_async(c.R, c.f, c.u, mask_dev, status_dev)

        if w.code == "rep" or w.s <= 16:
            c.plan.set_timing(0)
            for _ in range(args.warmup):
                async_step()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                async_step()
            torch.cuda.synchronize()
            extra["async_ms_per_step"] = (time.perf_counter() - t0) / args.steps * 1e3
            assert int(status_dev.item()) == 0
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                with torch.cuda.graph(graph, stream=side):
                    async_step()
            torch.cuda.synchronize()
            for _ in range(args.warmup):
                graph.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                graph.replay()
            torch.cuda.synchronize()
            extra["graph_ms_per_step"] = (time.perf_counter() - t0) / args.steps * 1e3
            assert int(status_dev.item()) == 0
            words = B.mask_to_bool(mask_dev.cpu().numpy().view(np.uint64), w.P)
            assert np.array_equal(words, c.expected_mask())

    abytes = algorithmic_bytes(w, c.mlen, n_honest, args.wide)
    kernels = {}
    for kind, name in enumerate(KIND_NAMES):
        total_ms, n = kernel_times[kind]
        if n:
            avg = total_ms / n
            kernels[name] = {"avg_ms": avg, "launches": n, "algorithmic_bytes": abytes[name],
                             "GBps": abytes[name] / avg / 1e6, "frac_hbm_peak": abytes[name] / avg / 1e6 / HBM_PEAK_GBS}
    dominant = max(kernels, key=lambda k: kernels[k]["avg_ms"])
    roof = {"bound": "hbm", "kernel": dominant, "achieved": kernels[dominant]["GBps"], "peak": HBM_PEAK_GBS,
            "unit": "GB/s", "frac": kernels[dominant]["GBps"] / HBM_PEAK_GBS, "traffic": None}
    ratio = None if (args.wide or args.unpacked) else MEASURED_TRAFFIC_RATIO.get(w.name, {}).get(dominant)
    if ratio is not None:
        roof["traffic"] = ratio * kernels[dominant]["algorithmic_bytes"]

    consumed = w.P * w.d * 4
    out = {
        "metric": "decoded gradient GB/s consumed (P x d fp32)",
        "value": consumed / (ms_per_step * 1e-3) / 1e9,
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if w.code == "rep" else "f64",
        "data": "synthetic",
        "config": {"workload": w.name + ("+wide_wire" if args.wide else "") + ("+unpacked_wire" if args.unpacked else ""), "code": w.code, "P": w.P, "s": w.s,
                   "d": w.d, "wire_words": 2 if args.wide else 1,
                   "adversaries": [[int(j), a] for j, a in c.adversaries],
                   "step": "encode(all nodes) + decode" if w.decode else "encode(all nodes)"},
        "pct_hbm_peak_consumed": consumed / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS * 100,
        "copy_kernel_ceiling_GBps": copy_gbps,
        "roofline": roof,
        "kernels": kernels,
        "stream_ordered": extra,
    }
    c.close()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
