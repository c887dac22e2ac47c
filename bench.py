#!/usr/bin/env python3
"""Benchmark of the DRACO encode/decode hot path on one MI355X.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config i] [--wire auto|one|wide8|wide16|wide|unpacked]

A step is one pass of the whole hot path over one batch of synthetic gradient
slabs already resident in HBM: the encoder of all P nodes (G -> Z), then the
parameter-server decoder on the received messages R (Z with the workload's
adversarial rows), through the synchronous C-ABI entry points (sum left on the
device, mask and status on the host).  The headline workload is the largest
one, the cyclic code at P = 45, s = 3, d = 25.6 M with full encode and decode,
on the narrowest wire that meets the 1e-4 bar END TO END there (an fp32 word plus an
8-bit code of its rounding residual per float, 5 bytes: that leaves 1.2e-6; one fp32 word
leaves 3e-4).  The metric is the benchmark contract's "decoded gradient
GB/s consumed": P*d*4 bytes per step divided by the step time.

One JSON line is printed.  Beside the headline it carries
  * `roofline`: the dominant kernel's algorithmic bytes over its HIP-event duration
    (events recorded by the library on the launch stream) against 8 TB/s;
  * `cpu_baseline`: the CPU oracle timed on a bounded sample on this machine's cores;
  * `configs`: one record per benchmark configuration (and the headline's shape on the 6-byte,
    8-byte and one-word wires, and the paper-shaped row) with per-kernel avg / median / min, encode-only and decode-only
    "consumed" GB/s, the end-to-end error against the true gradient sum, and the oracle's
    seconds.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak
KIND_NAMES = ["encode", "vote", "project", "recombine", "locate"]
# kernel-name fragments of each kind in the rocprofv3 summaries under profiles/
KIND_KERNEL = {"encode": "encode_", "vote": "decode_rep", "project": "cyc_project_kernel", "recombine": "cyc_recombine"}
TOL_END_TO_END = {"rep": 1e-5, "cyc": 1e-4}
# two-word wires: format of the second word, and fp32 words per message float
WIRE_SECOND = {"wide": "f32", "wide16": "bf16", "wide8": "i8"}
WIRE_WORDS = {"one": 1.0, "wide": 2.0, "wide16": 1.5, "wide8": 1.25, "unpacked": 1.0}
WIRE_TEXT = {"one": "one fp32 word", "wide": "two fp32 words (hi+lo)", "wide16": "fp32 word + bfloat16 word (hi+lo)",
             "wide8": "fp32 word + 8-bit residual code (hi+lo)", "unpacked": "unpacked complex, one word"}


def algorithmic_bytes(w, mlen, n_honest, words):
    """Bytes each kernel must move per launch (every input read once, every output written
    once); `words` = fp32 words per message float (2 on the wide wire, 1.5 with a bfloat16
    second word, 1.25 with an 8-bit one); the encoder reads
    B = m*P per-sample rows."""
    P, d, h = w.P, w.d, mlen // 2   # h: complex entries per message = entries of f
    return {
        "encode": int((w.m * P * d + words * P * mlen) * 4),
        "vote": (P * d + d) * 4,
        "project": int((words * P * mlen + h) * 4),
        "recombine": int((words * n_honest * mlen + d) * 4),
    }


def measured_traffic(workload, kind):
    """HBM bytes per launch of one kernel kind from the committed rocprofv3 --pmc summary of
    this workload (FETCH_SIZE and WRITE_SIZE scaled by the copy kernel), or None."""
    path = os.path.join(ROOT, "profiles", f"{workload}_kernels.md")
    frag = KIND_KERNEL.get(kind)
    if frag is None or not os.path.exists(path):
        return None
    in_table = False
    for line in open(path):
        if line.startswith("## "):
            in_table = line.startswith("## HBM traffic")
        elif in_table and line.startswith("| `") and frag in line and "reduce" not in line:
            cells = [c.strip() for c in line.strip().strip("|").split("|")]
            try:
                return float(cells[5])           # "scaled total B"
            except (IndexError, ValueError):
                return None
    return None


def thread_settings():
    out = {k: os.environ.get(k) for k in ("OMP_NUM_THREADS", "OPENBLAS_NUM_THREADS", "MKL_NUM_THREADS")}
    try:
        from threadpoolctl import threadpool_info
        out["pools"] = [{"api": p.get("user_api"), "lib": p.get("internal_api"), "threads": p.get("num_threads")}
                        for p in threadpool_info()]
    except Exception:
        pass
    return out


def oracle_time(w, wire, budget_s, d_cap):
    """The oracle as it stands on a slice of the same recipe (first d_s coordinates, all P
    nodes), repeated until about budget_s seconds of work are done."""
    import numpy as np
    import psutil
    import torch

    from oracle import draco_oracle as o
    from paper_1803_09877_amd import synth

    d_s = min(w.d, d_cap)
    ws = synth.scaled(w, d_s)
    S = synth.make_gradients(ws.P * ws.m, d_s, ws.sigma, ws.seed, device="cpu")[:, :d_s].numpy()
    unpacked = wire == "unpacked"
    f = synth.make_projection(d_s if unpacked else (d_s + 1) // 2, ws.seed).numpy()
    proc = psutil.Process()
    c0 = proc.cpu_times()
    t_enc = t_dec = 0.0
    reps = 0
    while reps < 20 and (reps == 0 or t_enc + t_dec < budget_s):
        t0 = time.perf_counter()
        G = S if ws.m == 1 else S.astype(np.float64).reshape(ws.P, ws.m, d_s).sum(1)
        if ws.code == "rep":
            Z = o.encode_repetition(G, ws.s)
        elif unpacked:
            Z = o.encode_cyclic_unpacked(G, ws.s)
        else:
            Z = o.encode_cyclic(G, ws.s)
        t_enc += time.perf_counter() - t0
        # the wire: one fp32 word, or the oracle's two-word wire (48 or 32 bits of the fp64 message)
        if wire in WIRE_SECOND:
            hi, lo = o.two_word_wire(Z, WIRE_SECOND[wire])
            R = torch.from_numpy(hi.astype(np.float64) + lo.astype(np.float64))
        else:
            R = torch.from_numpy(Z.astype(np.float32))
        synth.apply_attacks(R, Z.shape[1], ws.adversaries(), ws.seed)
        if ws.decode:
            t1 = time.perf_counter()
            if ws.code == "rep":
                _, mask, st = o.decode_repetition(R.numpy(), ws.s)
            elif unpacked:
                _, mask, st, _ = o.decode_cyclic_unpacked(R.numpy(), f, ws.s)
            else:
                _, mask, st = o.decode_cyclic(R.numpy(), f, ws.s, d_s, tau_h={"wide": o.TAU_H_WIDE, "wide16": o.TAU_H_BF16, "wide8": o.TAU_H_I8}.get(wire, o.TAU_H))
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
        "sample": f"same recipe, first {d_s} of {w.d} coordinates, P={ws.P}, s={ws.s}, B={ws.P * ws.m}, {reps} passes; "
                  f"per pass encode {t_enc / reps:.2f} s + decode {t_dec / reps:.2f} s",
        "encode_s": t_enc / reps,
        "decode_s": t_dec / reps,
        "threads": thread_settings(),
    }


def pick_wire(w, wire):
    """auto: the narrowest wire that meets 1e-4 end to end -- one fp32 word, or, where the entries
    of W reach 1e4 and more (from P = 32 on) and one word cannot, fp32 + an 8-bit residual code."""
    if w.code == "rep":
        return "one"
    if wire != "auto":
        return wire
    return "wide8" if w.P >= 32 else "one"


def stats(ms):
    import numpy as np
    a = np.asarray(ms, dtype=np.float64) * 1e3
    return {"avg_us": float(a.mean()), "median_us": float(np.median(a)), "min_us": float(a.min()), "launches": int(a.size)}


def measure(w, wire, steps, warmup, headline):
    """One workload on the GPU -> record.  Wall-clock loops are bracketed by synchronisations."""
    import numpy as np
    import torch

    from paper_1803_09877_amd import binding as B
    from paper_1803_09877_amd.runner import Case

    wide, unpacked = wire in WIRE_SECOND, wire == "unpacked"
    words = WIRE_WORDS[wire]
    c = Case(w, "cuda:0", wide=WIRE_SECOND.get(wire, False), unpacked=unpacked)
    name = w.name + {"one": "+one_word_wire", "wide": "+wide_wire", "wide16": "+wide16_wire", "wide8": "+wide8_wire",
                     "unpacked": "+unpacked_wire"}[wire] \
        if (w.code == "cyc" and wire != pick_wire(w, "auto")) else w.name
    rec = {"workload": name, "code": w.code, "P": w.P, "s": w.s, "d": w.d, "B": w.P * w.m,
           "wire": WIRE_TEXT[wire] if w.code == "cyc" else "fp32", "wire_words": words,
           "adversaries": [[int(j), a] for j, a in c.adversaries],
           "step": "encode(all nodes) + decode" if w.decode else "encode(all nodes)"}
    c.encode()
    c.receive()
    torch.cuda.synchronize()
    n_honest = w.P - len(c.adversaries)
    if w.decode:
        mask, status = c.decode()
        assert status == 0 and np.array_equal(mask, c.expected_mask()), "decode did not find the planted adversaries"
        # Definition 2 end to end: the decoded sum against the true gradient sum (fp64 on the GPU)
        ref = c.G[:, :w.d].double().sum(0)
        err = float((c.u[:w.d].double() - ref).norm() / ref.norm())
        rec["end_to_end_rel_l2"] = err
        rec["end_to_end_in_tolerance"] = bool(err <= TOL_END_TO_END[w.code])
        del ref

    def timed(fn, k):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(k):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / k * 1e3

    if headline:      # copy-kernel ceiling of this GPU on the same slabs (R -> Z, which the next encode overwrites)
        row_len = c.mlen // 4 * 4
        for _ in range(2):
            B.draco_copy_probe(c.R, c.Z, w.P, row_len, c.ld_m)
        ms = timed(lambda: B.draco_copy_probe(c.R, c.Z, w.P, row_len, c.ld_m), 5)
        rec["copy_kernel_ceiling_GBps"] = 2 * 4 * w.P * row_len / (ms * 1e-3) / 1e9

    for _ in range(warmup):
        c.step()
    rec["ms_per_step"] = timed(c.step, steps)
    # the same steps again with an event pair around every kernel (the events cost a few
    # microseconds per step, so they stay out of the step time above)
    c.plan.set_timing(steps)
    timed(c.step, steps)
    times = {name_: c.plan.kernel_times(kind) for kind, name_ in enumerate(KIND_NAMES)}
    c.plan.set_timing(0)

    consumed = w.P * w.d * 4
    rec["consumed_GBps"] = consumed / (rec["ms_per_step"] * 1e-3) / 1e9
    enc_ms = timed(c.encode, steps)
    rec["encode_only"] = {"ms": enc_ms, "GBps_of_messages_out": consumed / (enc_ms * 1e-3) / 1e9}
    if w.decode:
        dec_ms = timed(c.decode, steps)
        rec["decode_only"] = {"ms": dec_ms, "GBps_consumed": consumed / (dec_ms * 1e-3) / 1e9}

    abytes = algorithmic_bytes(w, c.mlen, n_honest, words)
    kernels = {}
    for kname, ms in times.items():
        if len(ms) == 0:
            continue
        k = stats(ms)
        if kname in abytes:
            k["algorithmic_bytes"] = abytes[kname]
            k["GBps"] = abytes[kname] / (k["avg_us"] * 1e-6) / 1e9
            k["frac_hbm_peak"] = k["GBps"] / HBM_PEAK_GBS
            k["frac_hbm_peak_min"] = abytes[kname] / (k["min_us"] * 1e-6) / 1e9 / HBM_PEAK_GBS
        kernels[kname] = k
    rec["kernels"] = kernels

    # The same step through the stream-ordered entry points (mask and status stay on the
    # device, read once after the K steps), eagerly and as one captured HIP graph per step.
    if headline and w.decode and (w.code == "rep" or w.s <= 16):
        mask_dev = torch.zeros(4, dtype=torch.int64, device=c.device)
        status_dev = torch.zeros(1, dtype=torch.int32, device=c.device)

        def async_step():
            c.encode()
            if w.code == "rep":
                c.plan.decode_repetition_async(c.R, c.u, mask_dev, status_dev)
            elif wide:
                c.plan.decode_cyclic_wide_async(c.R, c.Rlo, c.f, c.u, mask_dev, status_dev)
            else:
                c.plan.decode_cyclic_async(c.R, c.f, c.u, mask_dev, status_dev)

        extra = {}
        for _ in range(warmup):
            async_step()
        extra["async_ms_per_step"] = timed(async_step, steps)
        assert int(status_dev.item()) == 0
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                async_step()
        torch.cuda.synchronize()
        for _ in range(warmup):
            graph.replay()
        extra["graph_ms_per_step"] = timed(graph.replay, steps)
        assert int(status_dev.item()) == 0
        words_ = B.mask_to_bool(mask_dev.cpu().numpy().view(np.uint64), w.P)
        assert np.array_equal(words_, c.expected_mask())
        rec["stream_ordered"] = extra
    c.close()
    del c
    torch.cuda.empty_cache()
    return rec


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=4,
                    help="headline workload: index into the benchmark's configurations (default 4: cyclic, P=45, "
                         "s=3, d=25.6M, encode+decode); 5 = the paper-shaped row (P=45, s=5, B=180)")
    ap.add_argument("--wire", choices=["auto", "one", "wide", "wide16", "wide8", "unpacked"], default="auto",
                    help="cyclic message format (auto: two words where one cannot meet 1e-4 end to end)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-configs", action="store_true", help="skip the per-configuration records")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the P nodes are message slabs in one GPU's HBM); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_1803_09877_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    w = synth.WORKLOADS[args.config]
    wire = pick_wire(w, args.wire)
    head = measure(w, wire, args.steps, args.warmup, headline=True)

    kernels = head["kernels"]
    dominant = max((k for k in kernels if "GBps" in kernels[k]), key=lambda k: kernels[k]["avg_us"])
    roof = {"bound": "hbm", "kernel": dominant, "achieved": kernels[dominant]["GBps"], "peak": HBM_PEAK_GBS,
            "unit": "GB/s", "frac": round(kernels[dominant]["GBps"] / HBM_PEAK_GBS, 4),
            "traffic": measured_traffic(head["workload"], dominant)}
    out = {
        "metric": "decoded gradient GB/s consumed (P x d fp32)",
        "value": head["consumed_GBps"],
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if w.code == "rep" else "f64",
        "data": "synthetic",
        "config": {k: head[k] for k in ("workload", "code", "P", "s", "d", "B", "wire", "wire_words", "adversaries", "step")},
        "pct_hbm_peak_consumed": head["consumed_GBps"] / HBM_PEAK_GBS * 100,
        "copy_kernel_ceiling_GBps": head.get("copy_kernel_ceiling_GBps"),
        "end_to_end_rel_l2": head.get("end_to_end_rel_l2"),
        "end_to_end_in_tolerance": head.get("end_to_end_in_tolerance"),
        "roofline": roof,
        "kernels": kernels,
        "encode_only": head.get("encode_only"),
        "decode_only": head.get("decode_only"),
        "stream_ordered": head.get("stream_ordered", {}),
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = oracle_time(w, wire, 10.0, 8_000_000 if w.code == "cyc" else 16_000_000)

    if not args.no_configs:
        # every benchmark configuration on its default wire, then the headline's shape with a bfloat16
        # and an fp32 second word and on one word (reported: out of tolerance end to end), then the
        # paper-shaped row
        plan = [(i, "auto") for i in range(5)] + [(4, "wide16"), (4, "wide"), (4, "one"), (5, "auto")]
        recs = []
        for i, wr in plan:
            wi = synth.WORKLOADS[i]
            wri = pick_wire(wi, wr)
            if i == args.config and wri == wire:
                r = {k: v for k, v in head.items() if k not in ("stream_ordered", "copy_kernel_ceiling_GBps")}
                r["oracle"] = out.get("cpu_baseline")
            else:
                r = measure(wi, wri, max(5, args.steps // 3), 2, headline=False)
                if not args.no_cpu_baseline:
                    r["oracle"] = oracle_time(wi, wri, 0.0, 2_000_000 if wi.code == "cyc" else 11_200_000)
            r["config_index"] = i
            recs.append(r)
        out["configs"] = recs
        out["paper_context"] = ("the paper's own timings for this path (46 EC2 m4 CPU instances, P=45, B=180, s=5; "
                                "Tables 5-7): encode 0.2-13.6 s, decode 3.0-12.5 s per iteration")
    print(json.dumps(out))


if __name__ == "__main__":
    main()
