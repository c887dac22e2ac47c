"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py
times (same Case object, same entry points).

The oracle cannot run whole 4.6 GB slabs in seconds, so:
  * encode and the repetition vote are coordinate-local: the oracle recomputes
    windows of coordinates (the head, an unaligned middle stretch and the ragged
    tail) and they are compared element by element;
  * the cyclic locator needs every coordinate: the oracle's projection f R is
    accumulated chunk by chunk over the whole received slab, its phi gives the
    mask (compared bit for bit) and its b recombines the same windows;
  * properties that hold at any size are checked on the whole slab on the GPU
    (bit-identical repetition copies, finite output, untouched padding)."""
import numpy as np
import pytest
import torch

from oracle import draco_oracle as o
from paper_1803_09877_amd import synth
from paper_1803_09877_amd.runner import Case

pytestmark = pytest.mark.gpu


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def windows(d, code):
    """(start, stop) float ranges: head, a middle stretch at an even start that is
    not a multiple of 4 (odd length for the repetition code; the cyclic code's
    complex pairs must stay whole inside a window), and the ragged tail."""
    mid = (d // 2) // 4 * 4 + 1026
    return [(0, 4096), (mid, mid + (3001 if code == "rep" else 3002)), (max(0, (d - 2500) // 2 * 2), d)]


CHUNK = 1 << 20          # coordinates per oracle call in the whole-slab checks (even: complex pairs stay whole)


class RowErrors:
    """Accumulates, per row, the squared error and squared reference over chunks, and checks each
    chunk element by element against a bound relative to the chunk's largest reference entry."""

    def __init__(self, rows):
        self.num = np.zeros(rows)
        self.den = np.zeros(rows)

    def add(self, got, ref, elem_rel, what):
        got = np.asarray(got, dtype=np.float64)
        ref = np.asarray(ref, dtype=np.float64)
        diff = got - ref
        self.num += (diff * diff).sum(axis=-1)
        self.den += (ref * ref).sum(axis=-1)
        bound = elem_rel * np.max(np.abs(ref), axis=-1, initial=0.0)
        worst = np.max(np.abs(diff), axis=-1, initial=0.0)
        assert np.all(worst <= bound), (what, float(np.max(worst - bound)))

    def rel_l2(self):
        return np.sqrt(self.num / np.maximum(self.den, 1e-300))


def whole_slab_check(c, wide=False):
    """Oracle over EVERY coordinate, chunk by chunk: encoder rows, locator (the projection is
    accumulated over the whole received slab), and the decoded sum.  wide: False, or the
    second word's format on the two-word wire ("f32" / "bf16" / "i8")."""
    assert wide in (False, "f32", "bf16", "i8")
    # what hi + lo may differ from the fp64 message by, relative to the chunk's largest entry:
    # the two sides' fp64 W and sums (1e-14), plus the 32-bit wires' own rounding (2^-33, 2^-32)
    wire_elem = {"f32": 2.0 ** -43, "bf16": 2.0 ** -33 + 2.0 ** -43, "i8": 2.0 ** -31.98 + 2.0 ** -43}.get(wide)
    wire_row = {"f32": 1e-12, "bf16": 2.0 ** -33, "i8": 2.0 ** -32}.get(wide)

    def second_word(hi_t, lo_t):
        """fp64 values of a second-word slab chunk next to its first words."""
        if wide == "i8":
            return o.residual_from_code8(hi_t.cpu().numpy(), lo_t.cpu().numpy())
        return lo_t.double().cpu().numpy()

    sum_tol = 1e-6 if wide else 1e-4
    w = c.w
    P, s, d = w.P, w.s, w.d
    mask_gpu, status = c.last_decode if w.decode else (None, 0)
    enc = RowErrors(P)
    msg_ulps = (2 * w.r if w.code == "rep" else 2) * 2.0 ** -24
    gamma = np.zeros(P, dtype=np.complex128)
    f = c.f.cpu().numpy() if w.code == "cyc" else None
    tau = {"f32": o.TAU_H_WIDE, "bf16": o.TAU_H_BF16, "i8": o.TAU_H_I8}.get(wide, o.TAU_H)
    dec = RowErrors(1)
    mask_or = np.zeros(P, dtype=bool)

    def received(a, b):
        R = c.R[:, a:b].cpu().numpy()
        return R.astype(np.float64) + second_word(c.R[:, a:b], c.Rlo[:, a:b]) if wide else R

    for a in range(0, d, CHUNK):
        b = min(d, a + CHUNK)
        G = c.G[:, a:b].cpu().numpy()
        if w.code == "rep":
            Zo = o.encode_repetition(G, s)
            enc.add(c.Z[:, a:b].cpu().numpy(), Zo, msg_ulps, ("encode", a))
        else:
            Zo = o.encode_cyclic(G, s)
            mb = a + Zo.shape[1]
            if wide:       # hi + lo carries the fp64 message to 48 (32) bits
                Zw = c.Z[:, a:mb].double().cpu().numpy() + second_word(c.Z[:, a:mb], c.Zlo[:, a:mb])
                enc.add(Zw, Zo, wire_elem, ("encode", a))
            else:
                enc.add(c.Z[:, a:mb].cpu().numpy(), Zo, msg_ulps, ("encode", a))
        if not w.decode:
            continue
        if w.code == "rep":
            uo, mo, so = o.decode_repetition(received(a, b), s)
            assert so == 0
            mask_or |= mo
            dec.add(c.u[a:b].cpu().numpy()[None], uo[None], 1e-5, ("vote", a))
        else:
            mb = min(c.mlen, (b + 1) // 2 * 2)
            gamma += o.project(o.wire_to_complex(received(a, mb)), f[a // 2:mb // 2])
    assert np.all(enc.rel_l2() <= (wire_row if wide else 1e-6)), enc.rel_l2().max()
    if not w.decode:
        return
    if w.code == "rep":
        assert np.array_equal(mask_or, mask_gpu)
        assert dec.rel_l2()[0] <= 1e-5
        return
    mo, _, so = o.phi_from_projection(gamma, s, tau)
    assert so == 0 == status and np.array_equal(mo, mask_gpu)
    bo = o.solve_b(P, s, [j for j in range(P) if not mo[j]], "min_norm")
    honest = [j for j in range(P) if not mo[j]]
    for a in range(0, d, CHUNK):
        b = min(d, a + CHUNK)
        mb = min(c.mlen, (b + 1) // 2 * 2)
        Rc = o.wire_to_complex(received(a, mb))
        uh = np.zeros(Rc.shape[1], dtype=np.complex128)
        for j in honest:
            uh += bo[j] * Rc[j]
        dec.add(c.u[a:b].cpu().numpy()[None], o.unpack_complex(uh, b - a)[None], sum_tol, ("recombine", a))
    assert dec.rel_l2()[0] <= sum_tol, dec.rel_l2()


def true_sum_error(c):
    """Definition 2: the decoded sum against the adversary-free gradient sum (fp64 on the GPU)."""
    ref = c.G[:, :c.w.d].double().sum(0)
    return float((c.u[:c.w.d].double() - ref).norm() / ref.norm())


@pytest.mark.parametrize("idx", [1, 2, 3, 4])
def test_full_size_workload(idx):
    """Benchmark configurations 1-4 on the one-word wire: three windows as a fast pre-check, then
    the oracle over every coordinate of Z and u (masks bit-exact, sums within tolerance of the
    oracle decoding the same received messages, element-wise bounds on every chunk)."""
    w = synth.WORKLOADS[idx]
    print(f"full-size {w.name}: P={w.P} s={w.s} d={w.d} seed={w.seed}", flush=True)
    c = Case(w)
    try:
        c.encode()
        torch.cuda.synchronize()
        # ---- encoder, windows --------------------------------------------------
        for a, b in windows(w.d, w.code):
            G = c.G[:, a:b].cpu().numpy()
            if w.code == "rep":
                Zo = o.encode_repetition(G, w.s)
                Zg = c.Z[:, a:b].cpu().numpy()
            else:
                Zo = o.encode_cyclic(G, w.s)                     # a is even: pairs (2i, 2i+1) stay together
                Zg = c.Z[:, a:a + Zo.shape[1]].cpu().numpy()
            for j in range(w.P):
                assert rel_l2(Zg[j], Zo[j]) <= 1e-6, (a, b, j)
        if w.code == "rep":                                       # whole slab: copies bit-identical
            r = w.r
            Zi = c.Z[:, :c.mlen].view(torch.int32)
            for j in range(w.P):
                if j % r:
                    assert torch.equal(Zi[j], Zi[j - j % r]), j
        assert torch.isfinite(c.Z[:, :c.mlen]).all()
        c.last_decode = None
        if w.decode:
            c.receive()
            c.u.fill_(float("nan"))
            mask, status = c.decode()
            torch.cuda.synchronize()
            c.last_decode = (mask, status)
            assert status == 0
            assert np.array_equal(mask, c.expected_mask())
            assert torch.isfinite(c.u[:w.d]).all()
            if c.u.numel() > w.d:
                assert torch.isnan(c.u[w.d:]).all()
        whole_slab_check(c)
        if w.decode:
            err = true_sum_error(c)
            print(f"   end-to-end rel-L2 vs true sum: {err:.3e}", flush=True)
            if w.code == "rep":
                assert err <= 1e-5                        # Definition 2, Theorem 2
            elif w.P == 15:
                assert err <= 1e-4                        # Definition 2 within the cyclic bar
            # P = 45 on one fp32 word: see test_one_word_wire_at_p45_misses_the_bar_end_to_end
    finally:
        c.close()


@pytest.mark.xfail(strict=True, reason="one fp32 word per message float cannot carry the cyclic code at P = 45 "
                   "to 1e-4 end to end: |W| reaches 2.6e4 and the rounding of z is amplified to ~3e-4; "
                   "the two-word wire is the path that meets the bar there")
def test_one_word_wire_at_p45_misses_the_bar_end_to_end():
    """Recorded, not hidden: the one-word wire's end-to-end error at (45, 3, 25.6 M) is out of
    tolerance (it is in tolerance stage by stage against the oracle on the same messages)."""
    w = synth.WORKLOADS[4]
    c = Case(w)
    try:
        c.encode()
        c.receive()
        mask, status = c.decode()
        assert status == 0 and np.array_equal(mask, c.expected_mask())
        err = true_sum_error(c)
        print(f"   one-word wire, end-to-end rel-L2 vs true sum: {err:.3e}", flush=True)
        assert err <= 1e-4
    finally:
        c.close()


@pytest.mark.parametrize("second,e2e", [("i8", 5e-6), ("bf16", 2e-6), ("f32", 1e-6)])
def test_full_size_cyclic_wide_wire_end_to_end(second, e2e):
    """Configuration 4 (P=45, s=3, d=25.6M) on the two-word wire -- with the 8-bit second
    word the path the benchmark's headline runs: mask exact, every coordinate of hi+lo and of u
    against the oracle, and the decoded sum within 5e-6 (2e-6 with a bfloat16, 1e-6 with an fp32
    second word) of the TRUE gradient sum (the one-word wire's floor is 3e-4)."""
    w = synth.WORKLOADS[4]
    print(f"full-size wide {w.name} second word {second}", flush=True)
    c = Case(w, wide=second)
    try:
        c.encode()
        c.receive()
        c.u.fill_(float("nan"))
        mask, status = c.decode()
        torch.cuda.synchronize()
        assert status == 0 and np.array_equal(mask, c.expected_mask())
        c.last_decode = (mask, status)
        whole_slab_check(c, wide=second)
        err = true_sum_error(c)
        print(f"   end-to-end rel-L2 vs true sum (wide wire, {second}): {err:.3e}", flush=True)
        assert err <= e2e
        # the messages as sent: the projection's own rounding over 12.8 M terms must stay below
        # the wide wire's (much tighter) zero threshold, or honest nodes would be flagged
        for _ in range(2):                                        # second call: speculative single pass
            mask, status = c.plan.decode_cyclic_wide(c.Z, c.Zlo, c.f, c.u)
            torch.cuda.synchronize()
            assert status == 0 and not mask.any()
            assert true_sum_error(c) <= e2e
    finally:
        c.close()


@pytest.mark.parametrize("second,e2e", [("i8", 2e-5), ("bf16", 1e-5), ("f32", 1e-6)])
def test_full_size_paper_shaped_workload(second, e2e):
    """P = 45, s = 5, B = 180 (the paper's timing setup) at d = 25.6 M on the two-word wire: the
    per-sample rows are summed inside the encoder; mask exact, Definition 2 end to end."""
    w = synth.WORKLOADS[5]
    print(f"full-size paper-shaped {w.name} second word {second}", flush=True)
    c = Case(w, wide=second)
    try:
        c.encode()
        c.receive()
        c.u.fill_(float("nan"))
        mask, status = c.decode()
        torch.cuda.synchronize()
        assert status == 0 and np.array_equal(mask, c.expected_mask())
        d, m = w.d, w.m
        for a, b in windows(d, "cyc"):
            units = c.G[:, a:b].double().reshape(w.P, m, b - a).sum(1).cpu().numpy()
            Zo = o.encode_cyclic(units, w.s)
            Zhi = c.Z[:, a:a + Zo.shape[1]].cpu().numpy()
            Zlo = c.Zlo[:, a:a + Zo.shape[1]]
            Zw = Zhi.astype(np.float64) + (o.residual_from_code8(Zhi, Zlo.cpu().numpy()) if second == "i8"
                                           else Zlo.double().cpu().numpy())
            for j in range(w.P):
                assert rel_l2(Zw[j], Zo[j]) <= {"f32": 1e-12, "bf16": 2.0 ** -33, "i8": 2.0 ** -32}[second], (a, j)
        err = true_sum_error(c)
        print(f"   end-to-end rel-L2 vs true sum: {err:.3e}", flush=True)
        assert err <= e2e
    finally:
        c.close()


def test_full_size_cyclic_unpacked_wire():
    """Config 4 (P=45, s=3, d=25.6M) on the unpacked wire (messages of d complex entries,
    9.2 GB): encoder windows against the oracle's Z = G W, the mask against the oracle's
    phi on the whole-slab projection, recombined windows against the oracle's b."""
    w = synth.WORKLOADS[4]
    print(f"full-size unpacked {w.name}", flush=True)
    c = Case(w, unpacked=True)
    try:
        d = w.d
        c.encode()
        torch.cuda.synchronize()
        wins = [(0, 2048), (d // 2 + 1025, d // 2 + 1025 + 1501), (d - 1201, d)]
        for a, b in wins:
            Zo = o.encode_cyclic_unpacked(c.G[:, a:b].cpu().numpy(), w.s)
            Zg = c.Z[:, 2 * a:2 * b].cpu().numpy()
            for j in range(w.P):
                assert rel_l2(Zg[j], Zo[j]) <= 1e-6, (a, b, j)
        assert torch.isfinite(c.Z[:, :c.mlen]).all()
        c.receive()
        c.u.fill_(float("nan"))
        mask, status = c.decode()
        torch.cuda.synchronize()
        assert status == 0 and np.array_equal(mask, c.expected_mask())
        assert torch.isfinite(c.u[:d]).all()
        f = c.f.cpu().numpy()
        gamma = np.zeros(w.P, dtype=np.complex128)
        step = 1 << 20
        for a in range(0, d, step):
            b = min(d, a + step)
            gamma += o.project(o.wire_to_complex(c.R[:, 2 * a:2 * b].cpu().numpy()), f[a:b])
        mo, _, so = o.phi_from_projection(gamma, w.s)
        assert so == 0 and np.array_equal(mo, mask)
        bo = o.solve_b(w.P, w.s, [j for j in range(w.P) if not mo[j]], "min_norm")
        for a, b in wins:
            Rc = o.wire_to_complex(c.R[:, 2 * a:2 * b].cpu().numpy())
            uh = np.zeros(b - a, dtype=np.complex128)
            for j in range(w.P):
                if not mo[j]:
                    uh += bo[j] * Rc[j]
            assert rel_l2(c.u[a:b].cpu().numpy(), uh.real) <= 1e-4
        ref = c.G[:, :d].double().sum(0)
        err = float((c.u[:d].double() - ref).norm() / ref.norm())
        print(f"   end-to-end rel-L2 vs true sum (unpacked wire): {err:.3e}", flush=True)
        assert err <= 1e-3
    finally:
        c.close()


@pytest.mark.parametrize("code,P,s,d,attacks,placement,sigma", [
    ("rep", 45, 2, 11_173_001, ("signflip", "signflip"), "distinct_groups", 1e-2),   # ResNet-18's count + 1: odd, ragged
    ("cyc", 15, 2, 4_000_001, ("offset", "offset"), "any", 1.0),
    ("cyc", 45, 3, 1_000_003, ("noise", "signflip", "noise"), "adjacent_pair", 1e-2),
])
def test_odd_and_unaligned_lengths_at_scale(code, P, s, d, attacks, placement, sigma):
    """Gradient lengths that are odd and not a multiple of 4: the tail workgroup takes the
    guarded path while every other one takes the unchecked path."""
    w = synth.Workload(name=f"{code}_odd_{d}", code=code, P=P, s=s, d=d, sigma=sigma, attacks=attacks,
                       placement=placement, seed=synth.SEED_BASE + 77)
    print(f"odd-length {w.name}", flush=True)
    c = Case(w)
    try:
        c.Z.fill_(float("nan"))
        c.encode()
        c.receive()
        c.u.fill_(float("nan"))
        mask, status = c.decode()
        torch.cuda.synchronize()
        assert status == 0 and np.array_equal(mask, c.expected_mask())
        assert torch.isfinite(c.Z[:, :c.mlen]).all() and torch.isfinite(c.u[:d]).all()
        if c.ld_m > c.mlen:
            assert torch.isnan(c.Z[:, c.mlen:]).all()                # padding never written
        if c.u.numel() > d:
            assert torch.isnan(c.u[d:]).all()
        a = (d - 3000) // 2 * 2                                     # the ragged tail, element by element
        G = c.G[:, a:d].cpu().numpy()
        if code == "rep":
            Zo = o.encode_repetition(G, s)
            Zg = c.Z[:, a:d].cpu().numpy()
            uo, mo, so = o.decode_repetition(c.R[:, a:d].cpu().numpy(), s)
            assert np.array_equal(mo, mask)
        else:
            Zo = o.encode_cyclic(G, s)
            Zg = c.Z[:, a:c.mlen].cpu().numpy()
            Rc = o.wire_to_complex(c.R[:, a:c.mlen].cpu().numpy())
            bo = o.solve_b(P, s, [j for j in range(P) if not mask[j]], "min_norm")
            uo = o.unpack_complex(sum(bo[j] * Rc[j] for j in range(P) if not mask[j]), d - a)
        for j in range(P):
            assert rel_l2(Zg[j], Zo[j]) <= 1e-6, j
        assert rel_l2(c.u[a:d].cpu().numpy(), uo) <= (1e-5 if code == "rep" else 1e-4)
    finally:
        c.close()


@pytest.mark.parametrize("code", ["rep", "cyc"])
def test_dimension_beyond_two_to_the_31(code):
    """d = 2^31 + 5003 (odd): every float offset inside a row, and every byte offset, needs
    64 bits.  P = 3, s = 1 keeps the three slabs at 26 GB each.  Windows at the head, across
    the 2^31 boundary and at the ragged tail against the oracle; Definition 2 over the
    whole vector, accumulated on the GPU in fp64 chunk by chunk."""
    d = (1 << 31) + 5003
    w = synth.Workload(name=f"{code}_huge", code=code, P=3, s=1, d=d, sigma=1.0, attacks=("signflip",),
                       placement="any", seed=synth.SEED_BASE + 77)
    print(f"huge-d {code}: d={d}", flush=True)
    c = Case(w)
    try:
        c.encode()
        c.receive()
        c.u.fill_(float("nan"))
        mask, status = c.decode()
        torch.cuda.synchronize()
        assert status == 0 and np.array_equal(mask, c.expected_mask())
        wins = [(0, 2048), ((1 << 31) - 1030, (1 << 31) + 1030), (d - 1501 - (d - 1501) % 2, d)]
        U = [j for j in range(3) if not mask[j]]
        for a, b in wins:
            G = c.G[:, a:b].cpu().numpy()
            if code == "rep":
                Zo = o.encode_repetition(G, 1)
                Zg = c.Z[:, a:b].cpu().numpy()
                uo, mo, so = o.decode_repetition(c.R[:, a:b].cpu().numpy(), 1)
                assert so == 0 and np.array_equal(mo, mask)
                tol = 1e-5
            else:
                Zo = o.encode_cyclic(G, 1)
                Zg = c.Z[:, a:a + Zo.shape[1]].cpu().numpy()
                Rc = o.wire_to_complex(c.R[:, a:a + Zo.shape[1]].cpu().numpy())
                bo = o.solve_b(3, 1, U, "min_norm")
                uo = o.unpack_complex(sum(bo[j] * Rc[j] for j in U), b - a)
                tol = 1e-4
            for j in range(3):
                assert rel_l2(Zg[j], Zo[j]) <= 1e-6, (a, b, j)
            assert rel_l2(c.u[a:b].cpu().numpy(), uo) <= tol, (a, b)
        num = den = 0.0
        step = 1 << 28
        for a in range(0, d, step):
            b = min(d, a + step)
            ref = c.G[:, a:b].double().sum(0)
            num += float((c.u[a:b].double() - ref).pow(2).sum())
            den += float(ref.pow(2).sum())
        assert np.isfinite(num) and (num / den) ** 0.5 <= 1e-6
        if c.u.numel() > d:
            assert torch.isnan(c.u[d:]).all()
    finally:
        c.close()


def _time_ms(fn, reps=5):
    fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


@pytest.mark.parametrize("code", ["rep", "cyc"])
def test_encode_and_decode_time_is_linear_in_d_and_P(code):
    """The paper's complexity claims (Remark after Theorem 1; proofs of Theorems 2 and 4): the
    encoders cost O((2s+1) d) per node and the decoders O(P d): doubling d, or tripling P,
    multiplies the time by about that factor."""
    s = 2
    base = dict(code=code, s=s, sigma=1.0, attacks=(), placement="any", seed=synth.SEED_BASE + 5)
    times = {}
    for P, d in [(15, 8_000_000), (15, 16_000_000), (45, 8_000_000)]:
        c = Case(synth.Workload(name=f"lin_{P}_{d}", P=P, d=d, **base))
        try:
            c.encode()
            c.receive()
            times[(P, d)] = (_time_ms(c.encode), _time_ms(lambda: c.decode()))
        finally:
            c.close()
    for k in (0, 1):
        rd = times[(15, 16_000_000)][k] / times[(15, 8_000_000)][k]
        rp = times[(45, 8_000_000)][k] / times[(15, 8_000_000)][k]
        print(f"   {code} {'encode' if k == 0 else 'decode'}: x{rd:.2f} for 2x d, x{rp:.2f} for 3x P", flush=True)
        # the decoders carry a fixed cost (one wavefront of small algebra, one host sync)
        assert 1.4 <= rd <= 2.6
        assert 1.7 <= rp <= 4.0
