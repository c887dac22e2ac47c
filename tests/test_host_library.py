"""CPU-side checks of the C-ABI library (no GPU): it loads, exports what the
header declares, validates arguments, and its host algebra (code matrices, the
locator phi, the recombination vector b) agrees with the oracle and with the
identities the paper fixes.  No kernel is launched here."""
import itertools
import os
import re

import numpy as np
import pytest
import torch

from oracle import draco_oracle as o
from paper_1803_09877_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    L = B.lib()
    for header_name, exports in (("draco.h", B.EXPORTS), ("draco_bench.h", B.BENCH_EXPORTS)):
        header = open(os.path.join(ROOT, "include", header_name)).read()
        declared = set(re.findall(r"\b(draco_[a-z_]+)\s*\(", header))
        assert declared == set(exports), header_name
        for name in declared:
            assert hasattr(L, name), name


@pytest.mark.parametrize("code,P,s,d", [
    (0, 10, 1, 8), (0, 4, 2, 8), (1, 4, 2, 8), (1, 0, 0, 8), (0, 5, -1, 8), (2, 3, 1, 8), (1, 5, 1, 0), (1, 300, 1, 8), (0, 3, 1, 2**32)])
def test_plan_create_rejects_bad_parameters(code, P, s, d):
    with pytest.raises(B.DracoError) as e:
        B.Plan(code, P, s, d)
    assert e.value.status == B.EINVAL


def test_strerror_and_message_len():
    assert B.lib().draco_strerror(0) == b"ok"
    assert b"syndromes" in B.lib().draco_strerror(B.LOCATE_FAILED)
    assert B.Plan(B.CODE_REPETITION, 6, 1, 11).message_len == 11
    assert B.Plan(B.CODE_CYCLIC, 6, 1, 11).message_len == 12
    assert B.Plan(B.CODE_CYCLIC, 6, 1, 12).message_len == 12


def test_wire_selection():
    plan = B.Plan(B.CODE_CYCLIC, 6, 1, 11)
    assert plan.message_len == 12
    plan.set_wire(B.WIRE_UNPACKED)
    assert plan.message_len == 22
    assert plan.projection_vector(3).shape == (11,)
    plan.set_wire(B.WIRE_PACKED)
    assert plan.message_len == 12
    for bad in (2, -1):
        with pytest.raises(B.DracoError) as e:
            plan.set_wire(bad)
        assert e.value.status == B.EINVAL
    with pytest.raises(B.DracoError) as e:
        B.Plan(B.CODE_REPETITION, 6, 1, 11).set_wire(B.WIRE_UNPACKED)
    assert e.value.status == B.EINVAL


@pytest.mark.parametrize("P,s", [(3, 1), (15, 1), (15, 2), (45, 2), (15, 7), (6, 0)])
def test_repetition_plan_matches_oracle(P, s):
    plan = B.Plan(B.CODE_REPETITION, P, s, 16)
    A = o.assign_repetition(P, s)
    assert np.array_equal(plan.assign(), A)
    assert np.array_equal(plan.weights(), A.T.astype(complex))


@pytest.mark.parametrize("P,s", [(4, 1), (5, 1), (7, 2), (7, 3), (9, 4), (15, 2), (15, 7), (45, 3), (45, 5), (6, 0), (64, 10)])
def test_cyclic_plan_matches_oracle(P, s):
    plan = B.Plan(B.CODE_CYCLIC, P, s, 16)
    assert np.array_equal(plan.assign(), o.assign_cyclic(P, s))
    W = plan.weights()
    Wo = o.cyclic_weights(P, s)
    assert np.all((W != 0) == (Wo != 0))
    assert np.abs(W - Wo).max() <= 1e-12 * np.abs(Wo).max()
    # Lemma 4 directly on the library's numbers: rows of W are orthogonal to C_R
    CR = o.idft_matrix(P)[P - 2 * s:]
    if s > 0:
        assert np.abs(W @ CR.conj().T).max() <= 1e-12 * np.abs(W).max() * P


@pytest.mark.parametrize("P,s", [(4, 1), (5, 1), (7, 2), (7, 3), (8, 3), (9, 4)])
def test_locator_every_adversary_subset(P, s):
    """Same enumeration as the oracle's Lemma 2 pin: t = f N and V = the liars."""
    plan = B.Plan(B.CODE_CYCLIC, P, s, 24)
    rng = np.random.default_rng(P * 13 + s)
    G = rng.standard_normal((P, 24)).astype(np.float32)
    Zc = o.encode_cyclic_complex(o.pack_complex(G), s)
    f = (rng.standard_normal(12) + 1).astype(np.float32)
    for a in range(0, s + 1):
        for V in itertools.combinations(range(P), a):
            N = np.zeros_like(Zc)
            for j in V:
                N[j] = rng.standard_normal(12) * 10 + 1j * rng.standard_normal(12)
            gamma = o.project(Zc + N, f)
            mask, t, st = plan.cyclic_locate(gamma)
            assert st == B.OK
            assert sorted(np.flatnonzero(mask)) == sorted(V)
            omask, ot, ost = o.phi_from_projection(gamma, s)
            assert np.array_equal(mask, omask) and ost == o.OK
            if a:
                fN = o.project(N, f)
                assert np.allclose(t, fN, atol=1e-8 * np.abs(fN).max())


def test_locator_with_the_wide_wires_threshold():
    P, s = 9, 3
    plan = B.Plan(B.CODE_CYCLIC, P, s, 32)
    rng = np.random.default_rng(21)
    G = rng.standard_normal((P, 32)).astype(np.float32)
    Zc = o.encode_cyclic_complex(o.pack_complex(G), s)
    f = (rng.standard_normal(16) + 1).astype(np.float32)
    scale = np.median(np.abs(Zc))
    for V in [(), (4,), (0, 8), (2, 3, 7)]:
        Rc = Zc.copy()
        for j in V:
            Rc[j] += (rng.standard_normal(16) + 1j * rng.standard_normal(16)) * 1e-7 * scale
        gamma = o.project(Rc, f)
        mask, _, st = plan.cyclic_locate(gamma, tau=B.TAU_WIDE)
        omask, _, ost = o.phi_from_projection(gamma, s, o.TAU_H_WIDE)
        assert st == B.OK == ost and np.array_equal(mask, omask)
        assert sorted(np.flatnonzero(mask)) == sorted(V)
        loose, _, _ = plan.cyclic_locate(gamma)
        assert not loose.any()
    assert B.TAU == o.TAU_H and B.TAU_WIDE == o.TAU_H_WIDE
    for bad in (0.0, 1.0, -1.0, float("nan")):
        with pytest.raises(B.DracoError):
            plan.cyclic_locate(np.ones(P, dtype=complex), tau=bad)


def test_locator_reports_too_many_adversaries_and_nonfinite():
    P, s = 9, 2
    plan = B.Plan(B.CODE_CYCLIC, P, s, 40)
    rng = np.random.default_rng(3)
    G = rng.standard_normal((P, 40)).astype(np.float32)
    Zc = o.encode_cyclic_complex(o.pack_complex(G), s)
    for j in (0, 3, 6):
        Zc[j] = rng.standard_normal(20) * 100
    gamma = o.project(Zc, np.ones(20))
    mask, _, st = plan.cyclic_locate(gamma)
    omask, _, ost = o.phi_from_projection(gamma, s)
    assert st == B.LOCATE_FAILED and ost == o.LOCATE_FAILED
    assert np.array_equal(mask, omask)
    gamma[1] = np.nan                                   # a fourth bad node, this one not even finite
    mask, _, st = plan.cyclic_locate(gamma)
    omask, _, ost = o.phi_from_projection(gamma, s)
    assert st == B.LOCATE_FAILED == ost and mask[1] and np.array_equal(mask, omask)


def test_locator_flags_nonfinite_projections_and_still_locates():
    P, s = 9, 2
    plan = B.Plan(B.CODE_CYCLIC, P, s, 40)
    rng = np.random.default_rng(4)
    G = rng.standard_normal((P, 40)).astype(np.float32)
    Zc = o.encode_cyclic_complex(o.pack_complex(G), s)
    f = np.ones(20)
    for V, broken in [((2,), (2,)), ((2, 6), (6,)), ((0, 8), (0, 8))]:
        Rc = Zc.copy()
        for j in V:
            Rc[j] = rng.standard_normal(20) * 50
        gamma = o.project(Rc, f)
        for j in broken:
            gamma[j] = np.inf if j % 2 else np.nan
        mask, _, st = plan.cyclic_locate(gamma)
        omask, _, ost = o.phi_from_projection(gamma, s)
        assert st == B.OK == ost
        assert sorted(np.flatnonzero(mask)) == sorted(V) == sorted(np.flatnonzero(omask))


@pytest.mark.parametrize("tau", [B.TAU, B.TAU_I8, B.TAU_BF16, B.TAU_WIDE])
def test_locator_sets_enormous_projections_aside(tau):
    """Lies of 1e2 .. 1e30 times an honest message, on every wire's threshold: the library's host
    locator and the oracle's flag the same nodes (the enormous ones are set aside like broken ones
    once phi has failed); a small lie behind an enormous one is found; more than s enormous lies fail."""
    P, s, h = 15, 2, 200
    plan = B.Plan(B.CODE_CYCLIC, P, s, 2 * h)
    rng = np.random.default_rng(12)
    G = rng.standard_normal((P, 2 * h)).astype(np.float32)
    Zc = o.encode_cyclic_complex(o.pack_complex(G), s)
    f = 1.0 + rng.standard_normal(h)
    scale = np.abs(Zc).max()
    for mag in (1e2, 1e6, 1e10, 1e14, 1e20, 1e30):
        for V in ((3,), (3, 4), (0, 14), (6, 11)):
            Rc = Zc.copy()
            Rc[V[0]] = (rng.standard_normal(h) + 1j * rng.standard_normal(h)) * mag * scale
            if len(V) > 1:
                Rc[V[1]] += 10.0 * scale * rng.standard_normal(h)          # an ordinary lie behind it
            gamma = o.project(Rc, f)
            mask, _, st = plan.cyclic_locate(gamma, tau=tau)
            omask, _, ost = o.phi_from_projection(gamma, s, tau)
            assert st == B.OK == ost, (mag, V)
            assert sorted(np.flatnonzero(mask)) == sorted(V) == sorted(np.flatnonzero(omask)), (mag, V)
    Rc = Zc.copy()
    for j in (1, 5, 9):
        Rc[j] *= 1e28
    gamma = o.project(Rc, f)
    mask, _, st = plan.cyclic_locate(gamma, tau=tau)
    _, _, ost = o.phi_from_projection(gamma, s, tau)
    assert st == B.LOCATE_FAILED == ost


@pytest.mark.parametrize("P,s", [(4, 1), (7, 2), (9, 4)])
def test_recombination_vector_every_honest_set(P, s):
    plan = B.Plan(B.CODE_CYCLIC, P, s, 8)
    W = o.cyclic_weights(P, s)
    for a in range(0, 2 * s + 1):
        for V in itertools.combinations(range(P), a):
            mask = np.zeros(P, dtype=bool)
            mask[list(V)] = True
            b = plan.cyclic_recombination_vector(mask)
            assert np.all(b[mask] == 0)
            assert np.abs(W @ b - 1).max() <= 1e-11                      # Lemma 1
            bo = o.solve_b(P, s, [j for j in range(P) if not mask[j]], "min_norm")
            assert np.abs(b - bo).max() <= 1e-9
    mask = np.zeros(P, dtype=bool)
    mask[:2 * s + 1] = True
    with pytest.raises(B.DracoError):
        plan.cyclic_recombination_vector(mask)


@pytest.mark.parametrize("V", [(), (7,), (3, 4, 5), (0, 44, 20), (10, 11, 30), (43, 44, 0)])
def test_recombination_vector_P45(V):
    P, s = 45, 3
    plan = B.Plan(B.CODE_CYCLIC, P, s, 8)
    W = o.cyclic_weights(P, s)
    mask = np.zeros(P, dtype=bool)
    mask[list(V)] = True
    b = plan.cyclic_recombination_vector(mask)
    assert np.abs(W @ b - 1).max() <= 1e-9
    bo = o.solve_b(P, s, [j for j in range(P) if not mask[j]], "min_norm")
    assert np.linalg.norm(b) <= np.linalg.norm(bo) * (1 + 1e-9)
    assert np.abs(b - bo).max() <= 1e-7


def test_fp32_wire_locator_matches_oracle_on_workload_shapes():
    """Masks from the library's phi and the oracle's phi on fp32-wire projections
    at the benchmark's (P, s), with the attack mixes the workloads use."""
    rng = np.random.default_rng(11)
    for P, s, sigma, advs in [
        (15, 2, 1.0, [(3, "offset"), (9, "offset")]),
        (45, 3, 1e-2, [(3, "noise"), (4, "signflip"), (20, "noise")]),
        (45, 3, 1e-2, [(44, "signflip"), (0, "noise")]),
        (45, 3, 1e-2, []),
    ]:
        d = 20_000
        G = (rng.standard_normal((P, d)) * sigma).astype(np.float32)
        R = o.encode_cyclic(G, s).astype(np.float32)
        for j, kind in advs:
            if kind == "noise":
                R[j] = (rng.standard_normal(R.shape[1]) * 100).astype(np.float32)
            elif kind == "signflip":
                R[j] *= np.float32(-100)
            else:
                R[j] += np.float32(1e3)
        f = (rng.standard_normal(d // 2) + 1).astype(np.float32)
        gamma = o.project(o.wire_to_complex(R), f)
        plan = B.Plan(B.CODE_CYCLIC, P, s, d)
        mask, _, st = plan.cyclic_locate(gamma)
        omask, _, ost = o.phi_from_projection(gamma, s)
        assert st == B.OK and ost == o.OK
        assert np.array_equal(mask, omask)
        assert sorted(np.flatnonzero(mask)) == sorted(j for j, _ in advs)


@pytest.mark.parametrize("seed", [0, 1, 0x9E3779B97F4A7C15, 2**64 - 1])
def test_generated_projection_vector_matches_the_oracles_generator(seed):
    """The library's counter-based f and the oracle's own implementation of the same
    definition: identical fp32 values up to the last bit of libm's log/cos (at most one
    fp32 ulp, on a vanishing fraction of entries)."""
    d = 20_001
    plan = B.Plan(B.CODE_CYCLIC, 5, 1, d)
    f = plan.projection_vector(seed)
    fo = o.projection_vector((d + 1) // 2, seed)
    assert f.shape == fo.shape == (10_001,)
    ulp = np.abs(f.view(np.int32).astype(np.int64) - fo.view(np.int32).astype(np.int64))
    assert ulp.max() <= 1 and (ulp != 0).mean() <= 1e-3
    plan2 = B.Plan(B.CODE_CYCLIC, 5, 1, 64)            # entry i does not depend on d
    assert np.array_equal(plan2.projection_vector(seed), f[:32])
    with pytest.raises(B.DracoError):
        B.Plan(B.CODE_REPETITION, 3, 1, 8).projection_vector(seed)


@pytest.mark.skipif(torch.cuda.is_available(), reason="checks the no-GPU failure mode")
def test_device_entry_points_fail_loudly_without_a_gpu():
    plan = B.Plan(B.CODE_REPETITION, 3, 1, 8)
    with pytest.raises(B.DracoError) as e:
        plan.prepare()
    assert e.value.status == B.EHIP


def test_thresholds_and_formats_agree_across_header_binding_and_oracle():
    """The zero thresholds and second-word formats are numbers shared by the header, the binding and
    the oracle (each writes them out itself): read the header's macros and enumerators and compare."""
    import re
    text = open(os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "draco.h")).read()

    def macro(name):
        m = re.search(r"#define\s+%s\s+\(([^)]*)\)" % name, text)
        assert m, name
        return float(eval(m.group(1), {"__builtins__": {}}))

    assert macro("DRACO_TAU") == B.TAU == o.TAU_H
    assert macro("DRACO_TAU_WIDE") == B.TAU_WIDE == o.TAU_H_WIDE
    assert macro("DRACO_TAU_BF16") == B.TAU_BF16 == o.TAU_H_BF16
    assert macro("DRACO_TAU_I8") == B.TAU_I8 == o.TAU_H_I8
    for name, value in (("DRACO_SECOND_WORD_F32", B.SECOND_WORD_F32), ("DRACO_SECOND_WORD_BF16", B.SECOND_WORD_BF16),
                        ("DRACO_SECOND_WORD_I8", B.SECOND_WORD_I8)):
        m = re.search(r"%s\s*=\s*(\d+)" % name, text)
        assert m and int(m.group(1)) == value, name
    # the host locator's notion of an enormous projection is the oracle's
    P, s = 9, 2
    plan = B.Plan(B.CODE_CYCLIC, P, s, 40)
    rng = np.random.default_rng(1)
    gamma = rng.standard_normal(P) + 1j * rng.standard_normal(P)
    for factor in (o.ENORMOUS * 0.5, o.ENORMOUS * 4, 1e12, 1e25):
        g = gamma.copy()
        g[4] *= factor
        g[7] += 3.0
        mask, _, st = plan.cyclic_locate(g)
        omask, _, ost = o.phi_from_projection(g, s)
        assert st == ost and np.array_equal(mask, omask), factor
