"""bench.py's bookkeeping, without a GPU: the algorithmic bytes it prices the kernels with and
the HBM traffic it reads back from the committed rocprofv3 summaries."""
import importlib.util
import os

import pytest

from paper_1803_09877_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
spec = importlib.util.spec_from_file_location("bench", os.path.join(ROOT, "bench.py"))
bench = importlib.util.module_from_spec(spec)
spec.loader.exec_module(bench)


def test_algorithmic_bytes_count_every_input_and_output_once():
    w = synth.WORKLOADS[4]                                   # cyclic, P = 45, s = 3, d = 25.6 M
    mlen = 2 * ((w.d + 1) // 2)
    one = bench.algorithmic_bytes(w, mlen, w.P - 3, 1)
    two = bench.algorithmic_bytes(w, mlen, w.P - 3, 2)
    slab = w.P * w.d * 4
    assert one["encode"] == 2 * slab and two["encode"] == 3 * slab           # G in, one or two message words out
    assert one["project"] == slab + (mlen // 2) * 4                             # every message once, f once
    assert two["recombine"] == 2 * (w.P - 3) * w.d * 4 + w.d * 4                # honest rows only, the sum out
    rep = synth.WORKLOADS[1]
    assert bench.algorithmic_bytes(rep, rep.d, rep.P, 1)["vote"] == (rep.P + 1) * rep.d * 4
    paper = synth.WORKLOADS[5]                                                  # B = 4 P sample rows read
    assert bench.algorithmic_bytes(paper, mlen, paper.P - 5, 2)["encode"] == (4 + 2) * slab
    half = bench.algorithmic_bytes(w, mlen, w.P - 3, 1.5)                       # fp32 word + bfloat16 word
    assert half["encode"] == 2 * slab + slab // 2 and half["project"] == slab + slab // 2 + (mlen // 2) * 4
    quarter = bench.algorithmic_bytes(w, mlen, w.P - 3, 1.25)                   # fp32 word + 8-bit code
    assert quarter["encode"] == 2 * slab + slab // 4 and quarter["recombine"] == (w.P - 3) * w.d * 5 + w.d * 4
    assert all(isinstance(v, int) for v in list(half.values()) + list(quarter.values()))


def test_wire_choice_follows_the_end_to_end_tolerance():
    assert bench.pick_wire(synth.WORKLOADS[1], "auto") == "one"               # repetition: plain fp32
    assert bench.pick_wire(synth.WORKLOADS[2], "auto") == "one"               # P = 15: one word meets 1e-4
    assert bench.pick_wire(synth.WORKLOADS[4], "auto") == "wide8"             # P = 45: it does not; 5 bytes do
    assert bench.pick_wire(synth.WORKLOADS[4], "one") == "one"


@pytest.mark.parametrize("workload,kind,idx,words", [
    ("cyc_P45_s3_d25.6M", "encode", 4, 1.25), ("cyc_P45_s3_d25.6M", "project", 4, 1.25),
    ("cyc_P45_s3_d25.6M", "recombine", 4, 1.25), ("cyc_P45_s3_d25.6M+wide16_wire", "encode", 4, 1.5),
    ("cyc_P45_s3_d25.6M+wide_wire", "encode", 4, 2),
    ("cyc_P45_s3_d25.6M+one_word_wire", "encode", 4, 1), ("rep_P45_s2_d11.2M", "vote", 1, 1),
])
def test_traffic_is_read_from_the_committed_profile(workload, kind, idx, words):
    """The figure bench.py prints as roofline.traffic comes from profiles/<workload>_kernels.md
    (FETCH_SIZE + WRITE_SIZE scaled by the copy kernel) and sits within 1 % of the algorithmic bytes."""
    w = synth.WORKLOADS[idx]
    mlen = 2 * ((w.d + 1) // 2) if w.code == "cyc" else w.d
    got = bench.measured_traffic(workload, kind)
    assert got is not None
    want = bench.algorithmic_bytes(w, mlen, w.P - len(w.attacks), words)[kind]
    assert abs(got / want - 1.0) < 0.01
    assert bench.measured_traffic("no_such_workload", kind) is None
    assert bench.measured_traffic(workload, "locate") is None
