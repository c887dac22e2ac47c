"""Pins for the cyclic-code half of the CPU oracle (no GPU).

Expected values come from the paper and from mathematics, not from the oracle:
Definition 2 / Theorem 4 by exhaustive enumeration of adversary subsets, the
caption of Fig. 1 (4 gradients, r = 3, any 2 updates, 6 pairs), Lemma 1
(support of W, 1_P in the column span), Lemma 4 (clean messages have zero
syndrome), the identity t = f N from the proof of Lemma 2, a locator written
from the definition, the Lagrange closed form of b, unitarity of the IDFT
matrix, and the s = 0 special case (plain sum)."""
import itertools
import os

import numpy as np
import pytest

from oracle import draco_oracle as o

TINY = [(4, 1), (5, 1), (7, 2), (7, 3), (8, 3), (9, 4)]


def _grads(P, d, seed, sigma=1.0):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((P, d)) * sigma).astype(np.float32)


def _f(h, seed):
    rng = np.random.default_rng(seed + 99)
    return (rng.standard_normal(h) + 1.0).astype(np.float32)


def _attack64(R, j, kind, rng):
    """Edits of an fp64 wire message row (interleaved re/im)."""
    if kind == "noise":
        R[j] = rng.standard_normal(R.shape[1]) * 100
    elif kind == "signflip":
        R[j] = -100.0 * R[j]
    elif kind == "offset":
        R[j] = R[j] + 1e3
    elif kind == "constant":
        R[j] = -100.0
    elif kind == "one_coord":
        R[j, int(rng.integers(R.shape[1]))] += 1.0
    else:
        raise ValueError(kind)


# ------------------------------------------------------------------ plan ----
@pytest.mark.parametrize("P,s", TINY + [(15, 2), (15, 7), (45, 3)])
def test_assignment_is_the_unit_shift_circle(P, s):
    A = o.assign_cyclic(P, s)
    r = 2 * s + 1
    assert int(A.sum()) == P * r                               # Definition 1
    assert (A.sum(0) == r).all() and (A.sum(1) == r).all()     # every gradient held r times
    for j in range(P):
        assert sorted(np.flatnonzero(A[j])) == sorted((j + t) % P for t in range(r))
    assert len({tuple(row) for row in A}) == P or r == P       # P distinct sequences on the circle


@pytest.mark.parametrize("P", [1, 2, 3, 4, 7, 15, 45])
def test_idft_matrix_is_unitary_and_symmetric(P):
    C = o.idft_matrix(P)
    assert np.allclose(C @ C.conj().T, np.eye(P), atol=1e-13)
    assert np.allclose(C, C.T)
    # it IS numpy's inverse FFT up to the 1/sqrt(P) convention
    x = np.random.default_rng(P).standard_normal(P) + 1j * np.random.default_rng(P + 1).standard_normal(P)
    assert np.allclose(C @ x, np.fft.ifft(x) * np.sqrt(P), atol=1e-12)


@pytest.mark.parametrize("P,s", TINY + [(15, 2), (15, 7), (6, 0)])
def test_weights_solve_equals_closed_form(P, s):
    """q_j is unique (Sec. 3): the paper's linear solve and the product formula
    must be the same matrix."""
    W1 = o.cyclic_weights_solve(P, s)
    W2 = o.cyclic_weights(P, s)
    assert np.allclose(W1, W2, rtol=0, atol=1e-11 * np.abs(W2).max())


def test_weights_solve_equals_closed_form_P45():
    W1 = o.cyclic_weights_solve(45, 3)
    W2 = o.cyclic_weights(45, 3)
    assert np.abs(W1 - W2).max() <= 1e-8 * np.abs(W2).max()    # the solve loses digits here


@pytest.mark.parametrize("P,s", TINY + [(15, 2), (45, 3), (45, 5)])
def test_lemma1_support_and_lemma4_zero_syndrome(P, s):
    W = o.cyclic_weights(P, s)
    A = o.assign_cyclic(P, s)
    # Z = G W: row k multiplies gradient k, so W[k][j] != 0 only if node j holds k
    assert np.all((W != 0) == (A.T != 0))
    C = o.idft_matrix(P)
    CL, CR = C[:P - 2 * s], C[P - 2 * s:]
    # rows of W lie in the row space of C_L  <=>  W C_R^dagger = 0  (Lemma 4)
    assert np.abs(W @ CR.conj().T).max() <= 1e-13 * np.abs(W).max() * P
    # W = [Q 1] C_L has coefficient 1 on the last row of C_L: W C_L^dagger e_last = 1_P
    coeff = W @ CL.conj().T
    assert np.allclose(coeff[:, -1], 1.0, atol=1e-12 * np.abs(W).max() * P)


@pytest.mark.parametrize("P,s", TINY)
def test_lemma1_ones_in_span_for_every_honest_set(P, s):
    """For EVERY set U of at least P-2s nodes, W_{.,U} b = 1_P is solvable, with
    either choice of b; and 'first' equals the Lagrange closed form
    b_j = sqrt(P) / prod_{m in U, m != j} (w^j - w^m)."""
    W = o.cyclic_weights(P, s)
    x = np.exp(2j * np.pi * np.arange(P) / P)
    for size in range(P - 2 * s, P + 1):
        for U in itertools.combinations(range(P), size):
            for mode in ("first", "min_norm"):
                b = o.solve_b(P, s, list(U), mode)
                assert np.all(b[[j for j in range(P) if j not in U]] == 0)
                assert np.abs(W @ b - 1.0).max() <= 1e-10
            Ub = list(U)[:P - 2 * s]
            lag = np.zeros(P, dtype=complex)
            for j in Ub:
                lag[j] = np.sqrt(P) / np.prod([x[j] - x[m] for m in Ub if m != j])
            assert np.allclose(o.solve_b(P, s, list(U), "first"), lag, atol=1e-10)
            bmin = o.solve_b(P, s, list(U), "min_norm")
            assert np.linalg.norm(bmin) <= np.linalg.norm(lag) * (1 + 1e-9)


def test_lemma1_at_P45_with_clustered_adversaries():
    P, s = 45, 3
    W = o.cyclic_weights(P, s)
    for V in [(), (7,), (3, 4, 5), (0, 44, 20), (10, 11, 30)]:
        U = [j for j in range(P) if j not in V]
        b = o.solve_b(P, s, U, "min_norm")
        assert np.abs(W @ b - 1.0).max() <= 1e-8


# --------------------------------------------------------------- packing ----
@pytest.mark.parametrize("d", [1, 2, 7, 8])
@pytest.mark.parametrize("pairing", ["interleaved", "halves"])
def test_pack_unpack_roundtrip(d, pairing):
    X = np.random.default_rng(d).standard_normal((3, d))
    Xc = o.pack_complex(X, pairing)
    assert Xc.shape == (3, (d + 1) // 2)
    assert np.array_equal(o.unpack_complex(Xc, d, pairing), X)
    if pairing == "halves" and d > 1:                           # the paper's pairing: i with ceil(d/2)+i
        h = (d + 1) // 2
        assert Xc[0, 0] == X[0, 0] + 1j * X[0, h]
    assert np.array_equal(o.wire_to_complex(o.complex_to_wire(Xc)), Xc)


def test_decoded_sum_does_not_depend_on_the_pairing():
    P, s, d = 7, 2, 21
    G = _grads(P, d, 4)
    ref = np.sum(G.astype(np.float64), axis=0)
    for pairing in ("interleaved", "halves"):
        Gc = o.pack_complex(G, pairing)
        Zc = o.encode_cyclic_complex(Gc, s)
        Zc[2] = -100 * Zc[2]
        u_hat, mask, st = o.decode_cyclic_complex(Zc, _f(Gc.shape[1], 1), s)
        assert st == o.OK and list(np.flatnonzero(mask)) == [2]
        assert np.allclose(o.unpack_complex(u_hat, d, pairing), ref, atol=1e-9)


# ----------------------------------------------------------- s = 0 case -----
def test_s0_reduces_to_plain_sum():
    P, d = 6, 40
    G = _grads(P, d, 8)
    W = o.cyclic_weights(P, 0)
    assert np.all((W != 0) == np.eye(P, dtype=bool))            # A = I: one gradient per node
    Z = o.encode_cyclic(G, 0)
    u, mask, st = o.decode_cyclic(Z, _f(d // 2, 0), 0, d)
    assert st == o.OK and not mask.any()
    assert np.allclose(u, np.sum(G.astype(np.float64), axis=0), atol=1e-12)


def test_full_replication_is_a_scaled_sum():
    """P = 2s+1: every node holds every gradient; C_L is the single constant row,
    so every message is (1/sqrt P) * G 1_P."""
    P, s, d = 5, 2, 10
    G = _grads(P, d, 9)
    Zc = o.encode_cyclic_complex(o.pack_complex(G), s)
    ref = o.pack_complex(np.sum(G.astype(np.float64), axis=0)) / np.sqrt(P)
    for j in range(P):
        assert np.allclose(Zc[j], ref, atol=1e-13)


# ------------------------------------------------------------ Fig. 1 --------
def test_fig1_four_point_example(golden_dir):
    """Caption of Fig. 1: with 4 gradients and replication 3 the sum can be
    recovered from ANY 2 of the 4 updates, so one adversary is out-voted by a
    majority over all 6 pairs."""
    gold = {}
    with open(os.path.join(golden_dir, "fig1_four_point_example.txt")) as fh:
        for line in fh:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                gold[k] = int(v)
    P, r = gold["points"], gold["replication"]
    s = gold["adversaries"]
    assert r == 2 * s + 1 and P - 2 * s == gold["sufficient"]
    d = 12
    G = _grads(P, d, 42)
    ref = np.sum(G.astype(np.float64), axis=0)
    Zc = o.encode_cyclic_complex(o.pack_complex(G), s)
    assert int(o.assign_cyclic(P, s).sum()) == P * r
    pairs = list(itertools.combinations(range(P), gold["sufficient"]))
    assert len(pairs) == gold["pairs"]
    # clean: every pair of updates gives the sum
    for U in pairs:
        b = o.solve_b(P, s, list(U), "first")
        u = o.unpack_complex(sum(b[j] * Zc[j] for j in U), d)
        assert np.allclose(u, ref, atol=1e-12)
    # one adversary, each position: exactly the C(3,2) = 3 clean pairs agree, and they hold the sum
    for adv in range(P):
        Rc = Zc.copy()
        Rc[adv] = Rc[adv] * -100.0 + 5.0
        outs = []
        for U in pairs:
            b = o.solve_b(P, s, list(U), "first")
            outs.append(o.unpack_complex(sum(b[j] * Rc[j] for j in U), d))
        good = [np.allclose(u, ref, atol=1e-10) for u in outs]
        assert sum(good) == 3
        assert good == [adv not in U for U in pairs]
        bad = [u for u, g in zip(outs, good) if not g]
        for a, b_ in itertools.combinations(bad, 2):
            assert not np.allclose(a, b_, atol=1e-6)             # the wrong answers do not form a rival majority
        u, mask, st = o.decode_cyclic(o.complex_to_wire(Rc), _f(d // 2, adv), s, d)
        assert st == o.OK and list(np.flatnonzero(mask)) == [adv]
        assert np.allclose(u, ref, atol=1e-10)


# -------------------------------------------------------------- locator -----
@pytest.mark.parametrize("P,s", TINY)
def test_lemma2_t_equals_f_times_N(P, s):
    """Proof of Lemma 2: t = C h = gamma = (f N)^T exactly, for every adversary set."""
    d = 24
    G = _grads(P, d, P + s)
    Zc = o.encode_cyclic_complex(o.pack_complex(G), s)
    f = _f(d // 2, P)
    rng = np.random.default_rng(P * 31 + s)
    for a in range(1, s + 1):
        for V in itertools.combinations(range(P), a):
            N = np.zeros_like(Zc)
            for j in V:
                N[j] = rng.standard_normal(d // 2) * 10 + 1j * rng.standard_normal(d // 2)
            gamma = o.project(Zc + N, f)
            mask, t, st = o.phi_from_projection(gamma, s)
            fN = o.project(N, f)
            assert st == o.OK
            assert np.allclose(t, fN, atol=1e-8 * np.abs(fN).max())
            assert sorted(np.flatnonzero(mask)) == sorted(V)
            # Lemma 4: the syndromes of R are those of N alone
            assert np.allclose(o.syndromes(gamma, s), o.syndromes(fN, s), atol=1e-9 * np.abs(fN).max())
            # and the definition-level locator agrees
            assert np.array_equal(o.phi_bruteforce(gamma, s), mask)


def test_syndromes_are_the_high_dft_bins():
    P, s = 9, 2
    gamma = np.random.default_rng(0).standard_normal(P) + 1j * np.random.default_rng(1).standard_normal(P)
    full = np.fft.fft(gamma) / np.sqrt(P)                       # h = C^dagger gamma
    assert np.allclose(o.syndromes(gamma, s), full[P - 2 * s:], atol=1e-13)


# ------------------------------------------------------ Definition 2 --------
@pytest.mark.parametrize("P,s", TINY)
@pytest.mark.parametrize("kind", ["noise", "signflip", "offset", "constant", "one_coord"])
def test_definition2_every_adversary_subset(P, s, kind):
    """Theorem 4: every adversary set of size <= s, fp64 wire: decode = G 1_P and
    the mask is exactly the set of liars."""
    d = 19                                                       # odd: exercises the zero pad
    G = _grads(P, d, 5 * P + s)
    ref = np.sum(G.astype(np.float64), axis=0)
    Z = o.encode_cyclic(G, s)
    f = _f(Z.shape[1] // 2, P + 7)
    rng = np.random.default_rng(P * 17 + s)
    for a in range(0, s + 1):
        for V in itertools.combinations(range(P), a):
            R = Z.copy()
            for j in V:
                _attack64(R, j, kind, rng)
            for b_mode in ("min_norm", "first"):
                u, mask, st = o.decode_cyclic(R, f, s, d, b_mode)
                assert st == o.OK
                assert sorted(np.flatnonzero(mask)) == sorted(V)
                assert np.linalg.norm(u - ref) <= 1e-9 * np.linalg.norm(ref)


@pytest.mark.parametrize("P,s", [(5, 1), (7, 2), (9, 4)])
def test_definition2_with_nonfinite_messages(P, s):
    """A NaN/Inf message is still one adversarial node: for every adversary subset, with each
    adversary's message made non-finite somewhere, the decoder returns G 1_P and the set."""
    d = 18
    G = _grads(P, d, 3 * P + s)
    ref = np.sum(G.astype(np.float64), axis=0)
    Z = o.encode_cyclic(G, s)
    f = _f(Z.shape[1] // 2, P)
    rng = np.random.default_rng(P)
    for a in range(1, s + 1):
        for V in itertools.combinations(range(P), a):
            R = Z.copy()
            for n, j in enumerate(V):
                if n % 2 == 0:
                    R[j, int(rng.integers(R.shape[1]))] = np.nan if n % 4 == 0 else np.inf
                else:
                    R[j] = -100.0 * R[j]
            with np.errstate(invalid="ignore"):
                u, mask, st = o.decode_cyclic(R, f, s, d)
            assert st == o.OK
            assert sorted(np.flatnonzero(mask)) == sorted(V)
            assert np.linalg.norm(u - ref) <= 1e-9 * np.linalg.norm(ref)


def test_more_than_s_adversaries_is_reported():
    P, s, d = 9, 2, 40
    G = _grads(P, d, 77)
    Z = o.encode_cyclic(G, s)
    rng = np.random.default_rng(5)
    R = Z.copy()
    for j in (0, 3, 6):
        R[j] = rng.standard_normal(R.shape[1]) * 100
    _, _, st = o.decode_cyclic(R, _f(d // 2, 3), s, d)
    assert st == o.LOCATE_FAILED


# ------------------------------------------------- fp32 wire behaviour ------
@pytest.mark.parametrize("P,s,d,sigma,advs,tol", [
    (15, 2, 40_000, 1.0, [(3, "offset"), (9, "offset")], 5e-6),
    (15, 2, 40_000, 1.0, [(3, "offset"), (4, "signflip")], 5e-6),
    (15, 2, 40_000, 1.0, [], 5e-6),
    (45, 3, 40_000, 1e-2, [(3, "noise"), (4, "signflip"), (20, "noise")], 1e-3),
    (45, 3, 40_000, 1e-2, [(44, "signflip"), (0, "noise")], 1e-3),
    (45, 3, 40_000, 1e-2, [], 1e-3),
])
def test_fp32_wire_locates_exactly_and_error_is_the_wire_floor(P, s, d, sigma, advs, tol):
    """With messages rounded to fp32 the clean syndrome is no longer exactly zero;
    the thresholds must still give the exact mask, and the end-to-end error is
    the quantisation floor of the code (grows with max|W|: ~1e-6 at (15,2),
    ~2e-4 at (45,3))."""
    rng = np.random.default_rng(P + s + len(advs))
    G = (rng.standard_normal((P, d)) * sigma).astype(np.float32)
    R = o.encode_cyclic(G, s).astype(np.float32)
    for j, kind in advs:
        if kind == "noise":
            R[j] = (rng.standard_normal(R.shape[1]) * 100).astype(np.float32)
        elif kind == "signflip":
            R[j] = R[j] * np.float32(-100)
        elif kind == "offset":
            R[j] = R[j] + np.float32(1e3)
    f = _f(R.shape[1] // 2, 5)
    u, mask, st = o.decode_cyclic(R, f, s, d)
    assert st == o.OK
    assert sorted(np.flatnonzero(mask)) == sorted(j for j, _ in advs)
    ref = np.sum(G.astype(np.float64), axis=0)
    assert np.linalg.norm(u - ref) <= tol * np.linalg.norm(ref)


def test_planted_mistakes_are_caught():
    """Plausible slips, each planted in a copy of the oracle's steps, must break a pin."""
    P, s, d = 7, 2, 16
    G = _grads(P, d, 3)
    ref = np.sum(G.astype(np.float64), axis=0)
    W = o.cyclic_weights(P, s)
    Gc = o.pack_complex(G)
    # (1) transposed operand: node j using ROW j of W
    Zbad = np.zeros_like(Gc)
    for j in range(P):
        for k in range(P):
            Zbad[j] += W[j, k] * Gc[k]
    U = list(range(P))
    b = o.solve_b(P, s, U)
    assert not np.allclose(o.unpack_complex(sum(b[j] * Zbad[j] for j in U), d), ref, atol=1e-6)
    # (2) conjugate dropped in the syndrome: clean messages no longer have zero syndrome
    Zc = o.encode_cyclic_complex(Gc, s)
    gamma = o.project(Zc, _f(d // 2, 1))
    C = o.idft_matrix(P)
    assert np.abs(o.syndromes(gamma, s)).max() <= 1e-12 * np.abs(gamma).max()
    assert np.abs(C[P - 2 * s:] @ gamma).max() > 1e-3 * np.abs(gamma).max()
    # (3) e_first instead of e_last as the right-hand side for b
    CL = C[:P - 2 * s]
    e0 = np.zeros(P - 2 * s, dtype=complex)
    e0[0] = 1
    b0 = np.linalg.lstsq(CL, e0, rcond=None)[0]
    assert np.abs(W @ b0 - 1).max() > 1e-3


# ------------------------------------------------ phi step 1: the projection f R
def test_project_against_hand_values_and_a_double_loop():
    """phi's first step, gamma'_j = sum_i f_i r_j[i] with f REAL and the message row complex
    (Sec. 3, phi: "f R").  A 3 x 4 case worked by hand, then a random case against an
    explicit double loop.  The mistakes this rules out: conjugating the messages, summing
    over nodes instead of coordinates (f R vs R f^T with the wrong axis), dropping the
    imaginary part, weighting by |f| or f^2."""
    Rc = np.array([[1 + 2j, 0 - 1j, 3 + 0j, -2 + 2j],
                   [0 + 0j, 1 + 1j, -1 - 1j, 4 - 3j],
                   [2 - 1j, 2 + 1j, 0 + 5j, 1 + 0j]])
    f = np.array([1.0, -2.0, 0.5, 3.0])
    # row 0: (1+2j) - 2(0-1j) + 0.5(3) + 3(-2+2j) = (1 + 1.5 - 6) + (2 + 2 + 6)j
    # row 1: 0 - 2(1+1j) + 0.5(-1-1j) + 3(4-3j)   = (-2 - 0.5 + 12) + (-2 - 0.5 - 9)j
    # row 2: (2-1j) - 2(2+1j) + 0.5(5j) + 3(1)    = (2 - 4 + 3) + (-1 - 2 + 2.5)j
    want = np.array([-3.5 + 10j, 9.5 - 11.5j, 1.0 - 0.5j])
    got = o.project(Rc, f)
    assert got.shape == (3,) and got.dtype == np.complex128
    assert np.array_equal(got, want)
    rng = np.random.default_rng(3)
    Rc = rng.standard_normal((5, 7)) + 1j * rng.standard_normal((5, 7))
    f = rng.standard_normal(7) + 1.0
    loop = np.zeros(5, dtype=np.complex128)
    for j in range(5):
        for i in range(7):
            loop[j] += f[i] * Rc[j, i]
    assert np.allclose(o.project(Rc, f), loop, rtol=0, atol=1e-14)
    assert not np.allclose(o.project(Rc, f), np.conj(loop))           # conjugation would show
    # linear in the messages and in f; fp32 inputs are taken up to fp64 exactly
    assert np.allclose(o.project(2 * Rc, f) - o.project(Rc, 2 * f), 0, atol=1e-14)
    R32 = Rc.astype(np.complex64)
    f32 = f.astype(np.float32)
    assert np.array_equal(o.project(R32, f32), o.project(R32.astype(np.complex128), f32.astype(np.float64)))


# ------------------------------------------------ generated projection vector
def test_projection_generator_first_entries_by_hand():
    """Entry 0 for seed 0 worked through with Python integers, step by step, against the
    vectorised-looking loop in the oracle; then the closed form of Box-Muller's radius and
    angle is inverted to recover (u1, u2) from the entry pair construction."""
    M = (1 << 64) - 1
    z = 0x9E3779B97F4A7C15
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M
    z ^= z >> 31
    assert z == 0xE220A8397B1DCDAF                     # splitmix64's published first output for state 0
    u1 = ((z >> 40) + 0.5) / 2 ** 24
    u2 = (((z >> 16) & 0xFFFFFF) + 0.5) / 2 ** 24
    import math
    want = np.float32(1.0 + math.sqrt(-2.0 * math.log(u1)) * math.cos(2.0 * math.pi * u2))
    assert o.projection_vector(1, 0)[0] == want
    # seed enters additively before the finaliser: (seed, i) and (seed + k*gamma, i - k) coincide
    g = 0x9E3779B97F4A7C15
    assert np.array_equal(o.projection_vector(8, 5)[3:], o.projection_vector(5, (5 + 3 * g) & M))


def test_projection_generator_is_standard_normal_about_one():
    """f ~ N(1, I): moments, a Kolmogorov-Smirnov distance against the normal law, no
    correlation between neighbours or between seeds (24-bit uniforms bound |f-1| by 5.8)."""
    from scipy import stats
    n = 200_000
    f = o.projection_vector(n, 7).astype(np.float64)
    g = o.projection_vector(n, 8).astype(np.float64)
    assert abs(f.mean() - 1.0) < 4 / np.sqrt(n)
    assert abs(f.var() - 1.0) < 0.02
    assert stats.kstest(f - 1.0, "norm").statistic < 0.005
    assert abs(np.corrcoef(f[:-1], f[1:])[0, 1]) < 0.01
    assert abs(np.corrcoef(f, g)[0, 1]) < 0.01
    assert np.abs(f - 1.0).max() < 5.9 and np.isfinite(f).all()
    assert len(np.unique(f)) > 0.98 * n


# ------------------------------------------------------------ unpacked wire --
@pytest.mark.parametrize("P,s", TINY)
@pytest.mark.parametrize("kind", ["noise", "signflip", "one_coord"])
def test_unpacked_definition2_every_adversary_subset(P, s, kind):
    """Sec. 3 as stated (Z = G W on the real gradients, d complex entries per message):
    every adversary set of size <= s is located and Re(R_U b) = G 1_P; the imaginary
    part of the recombination is rounding only."""
    d = 11
    G = _grads(P, d, 3 * P + s)
    ref = np.sum(G.astype(np.float64), axis=0)
    Z = o.encode_cyclic_unpacked(G, s)
    assert Z.shape == (P, 2 * d)
    f = _f(d, P + 3)
    rng = np.random.default_rng(P * 19 + s)
    for a in range(0, s + 1):
        for V in itertools.combinations(range(P), a):
            R = Z.copy()
            for j in V:
                _attack64(R, j, kind, rng)
            u, mask, st, resid = o.decode_cyclic_unpacked(R, f, s)
            assert st == o.OK
            assert sorted(np.flatnonzero(mask)) == sorted(V)
            assert np.linalg.norm(u - ref) <= 1e-9 * np.linalg.norm(ref)
            assert resid <= 1e-9 * np.abs(ref).max()


@pytest.mark.parametrize("P,s,d", [(7, 2, 10), (9, 4, 13), (15, 2, 32)])
def test_packing_is_a_linear_recombination_of_the_unpacked_messages(P, s, d):
    """The remark closing Sec. 3: packing coordinates (a, b) into a + ib commutes with the
    linear encoder, so the packed message is z[a] + i z[b] of the unpacked one, entry by
    entry -- for the library's adjacent pairing and for the paper's half-apart pairing."""
    G = _grads(P, d, 77 + P)
    Zu = o.wire_to_complex(o.encode_cyclic_unpacked(G, s))                      # [P][d] complex
    dp = d + (d & 1)
    Zu_pad = np.concatenate([Zu, np.zeros((P, dp - d), dtype=complex)], axis=1)
    Zp = o.wire_to_complex(o.encode_cyclic(G, s, "interleaved"))
    assert np.allclose(Zp, Zu_pad[:, 0::2] + 1j * Zu_pad[:, 1::2], rtol=0, atol=1e-12 * np.abs(Zp).max())
    Zh = o.wire_to_complex(o.encode_cyclic(G, s, "halves"))
    h = (d + 1) // 2
    assert np.allclose(Zh, Zu_pad[:, :h] + 1j * Zu_pad[:, h:], rtol=0, atol=1e-12 * np.abs(Zh).max())


def test_unpacked_messages_of_real_gradients_have_hermitian_structure_in_W_only():
    """An unpacked message is W_{.,j}^T applied to real numbers: its real and imaginary
    parts are the real gradients times Re W and Im W separately."""
    P, s, d = 9, 2, 6
    G = _grads(P, d, 5).astype(np.float64)
    W = o.cyclic_weights(P, s)
    Zc = o.wire_to_complex(o.encode_cyclic_unpacked(G, s))
    assert np.allclose(Zc.real, W.real.T @ G, atol=1e-12 * np.abs(Zc).max())
    assert np.allclose(Zc.imag, W.imag.T @ G, atol=1e-12 * np.abs(Zc).max())


# ------------------------------------------------ threshold of the wide wire --
@pytest.mark.parametrize("P,s", [(5, 1), (7, 2), (9, 4)])
def test_wide_threshold_every_adversary_subset_with_tiny_lies(P, s):
    """Messages carried to 48 bits (hi + lo fp32 words): lies of 1e-7 of the message size,
    every adversary set of size <= s.  With TAU_H_WIDE the set is located and the sum is
    G 1_P; with the one-word TAU_H the lies pass as rounding."""
    d = 16
    G = _grads(P, d, 9 * P + s)
    ref = np.sum(G.astype(np.float64), axis=0)
    Z = o.encode_cyclic(G, s)
    hi = Z.astype(np.float32)
    lo = (Z - hi).astype(np.float32)
    Zw = hi.astype(np.float64) + lo.astype(np.float64)
    f = _f(d // 2, P + 1)
    rng = np.random.default_rng(P + s)
    scale = np.median(np.abs(Zw))
    for a in range(0, s + 1):
        for V in itertools.combinations(range(P), a):
            R = Zw.copy()
            for j in V:
                R[j] += rng.standard_normal(d) * 1e-7 * scale
            u, mask, st = o.decode_cyclic(R, f, s, d, tau_h=o.TAU_H_WIDE)
            assert st == o.OK and sorted(np.flatnonzero(mask)) == sorted(V)
            assert np.linalg.norm(u - ref) <= 1e-11 * np.linalg.norm(ref)
            _, loose, st2 = o.decode_cyclic(R, f, s, d)
            assert st2 == o.OK and not loose.any()


def test_wide_threshold_sits_between_the_floors():
    """Clean syndromes of a 48-bit wire are ~1e-14 of the median projection, those of an fp32
    wire ~5e-8: TAU_H_WIDE lies three orders above the first and far below the second."""
    P, s, d = 45, 3, 40_000
    G = _grads(P, d, 4, 1e-2)
    Z = o.encode_cyclic(G, s)
    hi = Z.astype(np.float32)
    wide = hi.astype(np.float64) + (Z - hi).astype(np.float32).astype(np.float64)
    f = _f(d // 2, 8)
    for R, lo_b, hi_b in ((wide, 0.0, 1e-3 * o.TAU_H_WIDE), (hi.astype(np.float64), 1e3 * o.TAU_H_WIDE, o.TAU_H / 8)):
        gamma = o.project(o.wire_to_complex(R), f)
        floor = np.abs(o.syndromes(gamma, s)).max() / np.median(np.abs(gamma))
        assert lo_b <= floor <= hi_b, floor


# ------------------------------------- two-word wire with a bfloat16 second word --
def test_round_to_bfloat16_hand_values_and_ties():
    """Values whose nearest bfloat16 can be read off: 8 significant bits, ties to even."""
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 2.0 ** -7, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20,
                  -(1.0 + 3 * 2.0 ** -8), 0.0, -0.0, 3.0e38, 1e-30, np.inf, -np.inf], dtype=np.float32)
    want = np.array([1.0, 1.0, 1.0 + 2.0 ** -7, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7,
                     -(1.0 + 2.0 ** -6), 0.0, -0.0, 3.0e38, 1e-30, np.inf, -np.inf], dtype=np.float32)
    got = o.round_to_bfloat16(x)
    assert np.array_equal(got[:8].view(np.uint32), want[:8].view(np.uint32))
    assert (got.view(np.uint32) & 0xFFFF == 0).all()                 # the lower half of every word is clear
    assert np.array_equal(got[10:], want[10:])
    assert abs(float(got[8]) - 3.0e38) <= 2.0 ** -9 * 3.0e38 and abs(float(got[9]) - 1e-30) <= 2.0 ** -9 * 1e-30
    assert np.isnan(o.round_to_bfloat16(np.array([np.nan], dtype=np.float32))).all()


def test_round_to_bfloat16_against_a_library_conversion():
    """torch's CPU conversion to bfloat16 rounds to nearest even as well: bit for bit on random
    fp32 words of every exponent, and rounding twice changes nothing."""
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(5)
    bits = rng.integers(0, 2 ** 32, size=200_000, dtype=np.uint64).astype(np.uint32)
    x = bits.view(np.float32)
    x = x[np.isfinite(x)]
    got = o.round_to_bfloat16(x)
    lib = torch.from_numpy(x.copy()).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(got.view(np.uint32), lib.view(np.uint32))
    assert np.array_equal(o.round_to_bfloat16(got).view(np.uint32), got.view(np.uint32))


def test_two_word_wire_carries_48_and_32_bits():
    """hi + lo is within 2^-48 |z| (fp32 second word) and 2^-33 |z| (bfloat16) of z, element by
    element, and the first word alone within 2^-24 |z|."""
    rng = np.random.default_rng(11)
    z = rng.standard_normal(100_000) * 10.0 ** rng.uniform(-6, 6, 100_000)
    for second, bits in (("f32", 48), ("bf16", 33)):
        hi, lo = o.two_word_wire(z, second)
        assert hi.dtype == lo.dtype == np.float32
        err = np.abs(hi.astype(np.float64) + lo.astype(np.float64) - z)
        assert (err <= 2.0 ** -bits * np.abs(z)).all(), second
        assert (np.abs(hi.astype(np.float64) - z) <= 2.0 ** -24 * np.abs(z)).all()
    assert err.max() > 0                                              # the bfloat16 word does round
    with pytest.raises(ValueError):
        o.two_word_wire(z, "fp8")


def test_bfloat16_second_word_end_to_end_at_p45():
    """(P, s) = (45, 3): W's entries reach 1e4-1e5 and the decoder cancels them, so what the wire
    rounds away comes back amplified.  One fp32 word leaves the decoded sum around 3e-4 from the
    true one -- outside Definition 2's 1e-4 reading -- the bfloat16 second word 2^9 closer."""
    P, s, d = 45, 3, 20_000
    G = _grads(P, d, 21, 1e-2)
    ref = np.sum(G.astype(np.float64), axis=0)
    Z = o.encode_cyclic(G, s)
    f = _f(d // 2, 3)
    errs = {}
    for name, second in (("bf16", "bf16"), ("f32", "f32")):
        hi, lo = o.two_word_wire(Z, second)
        R = hi.astype(np.float64) + lo.astype(np.float64)
        tau = o.TAU_H_BF16 if second == "bf16" else o.TAU_H_WIDE
        u, mask, st = o.decode_cyclic(R, f, s, d, tau_h=tau)
        assert st == o.OK and not mask.any()
        errs[name] = np.linalg.norm(u - ref) / np.linalg.norm(ref)
    u1, mask1, st1 = o.decode_cyclic(Z.astype(np.float32), f, s, d)
    assert st1 == o.OK and not mask1.any()
    errs["one"] = np.linalg.norm(u1 - ref) / np.linalg.norm(ref)
    assert errs["f32"] < 1e-9 < errs["bf16"] < 3e-6 < 1e-4 < errs["one"] < 1e-3, errs
    assert 100 < errs["one"] / errs["bf16"] < 2000, errs             # 2^9 more bits, give or take


@pytest.mark.parametrize("P,s", [(5, 1), (7, 2), (9, 4)])
def test_bfloat16_threshold_every_adversary_subset(P, s):
    """Messages carried to 32 bits: lies of 5e-7 of the message size (the middle of the 2^9 between
    the two thresholds; with 8 coordinates a lie's syndromes scatter over two orders), every
    adversary set of size <= s: located with TAU_H_BF16, passed as rounding by the one-word TAU_H."""
    d = 16
    G = _grads(P, d, 9 * P + s)
    ref = np.sum(G.astype(np.float64), axis=0)
    hi, lo = o.two_word_wire(o.encode_cyclic(G, s), "bf16")
    Zw = hi.astype(np.float64) + lo.astype(np.float64)
    f = _f(d // 2, P + 1)
    rng = np.random.default_rng(P + s)
    scale = np.median(np.abs(Zw))
    for a in range(0, s + 1):
        for V in itertools.combinations(range(P), a):
            R = Zw.copy()
            for j in V:
                R[j] += rng.standard_normal(d) * 5e-7 * scale
            u, mask, st = o.decode_cyclic(R, f, s, d, tau_h=o.TAU_H_BF16)
            assert st == o.OK and sorted(np.flatnonzero(mask)) == sorted(V)
            assert np.linalg.norm(u - ref) <= 1e-7 * np.linalg.norm(ref)
            _, loose, st2 = o.decode_cyclic(R, f, s, d)
            assert st2 == o.OK and not loose.any()


def test_bfloat16_threshold_sits_between_the_floors():
    """Clean syndromes of the 32-bit wire are some 2^-33 of the median projection: TAU_H_BF16 is
    an order above them at the benchmark's shape and far below the one-word wire's floor."""
    P, s, d = 45, 3, 40_000
    G = _grads(P, d, 4, 1e-2)
    Z = o.encode_cyclic(G, s)
    hi, lo = o.two_word_wire(Z, "bf16")
    f = _f(d // 2, 8)
    floors = []
    for R in (hi.astype(np.float64) + lo.astype(np.float64), hi.astype(np.float64)):
        gamma = o.project(o.wire_to_complex(R), f)
        floors.append(np.abs(o.syndromes(gamma, s)).max() / np.median(np.abs(gamma)))
    assert floors[0] <= o.TAU_H_BF16 / 8 and 8 * o.TAU_H_BF16 <= floors[1], floors


# ------------------------------------------ two-word wire with an 8-bit second word --
def test_residual_code8_hand_values():
    """hi = 1 (spacing 2^-23): a residual of a quarter spacing is code 63.5 -> 64 (tie to even),
    half a spacing is 127, its negative -127, nothing is 0; hi = 6 (spacing 2^-21) scales alike;
    a non-finite first word carries no residual."""
    u1, u6 = 2.0 ** -23, 2.0 ** -21
    hi = np.array([1.0, 1.0, 1.0, 1.0, 1.0, 6.0, 6.0, -6.0, np.inf, np.nan, 0.0, 1e-35], dtype=np.float32)
    r = np.array([u1 / 4, u1 / 2, -u1 / 2, 0.0, u1 / 254, u6 / 254 * 10, -u6 / 254 * 100.4, u6 / 254 * 7,
                  1.0, 1.0, 1e-50, 1e-43])
    want = np.array([64, 127, -127, 0, 1, 10, -100, 7, 0, 0, 0, 0], dtype=np.int8)
    got = o.residual_code8(hi, r)
    assert got.dtype == np.int8 and np.array_equal(got, want), got
    back = o.residual_from_code8(hi[:8], got[:8])
    assert np.allclose(back, [64 * u1 / 254, u1 / 2, -u1 / 2, 0, u1 / 254, 10 * u6 / 254, -100 * u6 / 254, 7 * u6 / 254],
                       rtol=1e-15, atol=0)


def test_two_word_wire_with_code8_carries_32_bits():
    """hi + lo within 1/508 of the spacing at hi -- at most 2^-23 |z| / 508, about 2^-32 |z| -- over
    twelve decades; every code is used; powers of two, where the spacing changes, included."""
    rng = np.random.default_rng(12)
    z = rng.standard_normal(200_000) * 10.0 ** rng.uniform(-6, 6, 200_000)
    z[:64] = np.ldexp(1.0, np.arange(-32, 32)) * (1 - 2.0 ** -26)        # just under a power of two: hi rounds up to it
    hi, lo = o.two_word_wire(z, "i8")
    assert hi.dtype == np.float32 and lo.dtype == np.float64
    err = np.abs(hi.astype(np.float64) + lo - z)
    assert (err <= 2.0 ** -23 / 508 * np.abs(z) * (1 + 1e-6)).all()
    assert err.max() > 2.0 ** -36 * np.abs(z).min()
    q = o.residual_code8(hi, z - hi.astype(np.float64))
    assert q.min() == -127 and q.max() == 127 and len(np.unique(q)) == 255
    # the code is the nearest one: no other code is closer to the residual
    u = np.ldexp(1.0, o._ulp_exponent(hi))
    assert (np.abs((z - hi.astype(np.float64)) / u * 254 - q) <= 0.5 + 1e-6).all()


def test_code8_second_word_end_to_end_at_p45():
    """(P, s) = (45, 3): the 5-byte wire leaves the decoded sum within a few 1e-6 of the true one,
    two orders inside the 1e-4 reading of Definition 2 where one fp32 word is outside it; and at the
    paper's (45, 5), where W grows to 1.8e5, still an order inside."""
    for (P, s, bar) in ((45, 3, 5e-6), (45, 5, 2e-5)):
        d = 20_000
        G = _grads(P, d, 21, 1e-2)
        ref = np.sum(G.astype(np.float64), axis=0)
        Z = o.encode_cyclic(G, s)
        f = _f(d // 2, 3)
        hi, lo = o.two_word_wire(Z, "i8")
        u, mask, st = o.decode_cyclic(hi.astype(np.float64) + lo, f, s, d, tau_h=o.TAU_H_I8)
        assert st == o.OK and not mask.any()
        e8 = np.linalg.norm(u - ref) / np.linalg.norm(ref)
        u1, _, _ = o.decode_cyclic(Z.astype(np.float32), f, s, d)
        e1 = np.linalg.norm(u1 - ref) / np.linalg.norm(ref)
        assert e8 < bar < 1e-4 < e1, (P, s, e8, e1)
        assert 50 < e1 / e8 < 1000, (e1, e8)


def test_code8_threshold_sits_between_the_floors():
    """Clean syndromes of the 5-byte wire against TAU_H_I8, as for the other wires."""
    P, s, d = 45, 3, 40_000
    G = _grads(P, d, 4, 1e-2)
    Z = o.encode_cyclic(G, s)
    hi, lo = o.two_word_wire(Z, "i8")
    f = _f(d // 2, 8)
    floors = []
    for R in (hi.astype(np.float64) + lo, hi.astype(np.float64)):
        gamma = o.project(o.wire_to_complex(R), f)
        floors.append(np.abs(o.syndromes(gamma, s)).max() / np.median(np.abs(gamma)))
    assert floors[0] <= o.TAU_H_I8 / 8 and 4 * o.TAU_H_I8 <= floors[1], floors


# ------------------------------------------- structure of W the encoders rely on --
@pytest.mark.parametrize("P,s", [(5, 1), (9, 1), (10, 2), (15, 2), (8, 3), (7, 3), (45, 3), (45, 5), (33, 16)])
def test_weights_factor_into_unit_phases_and_real_taps(P, s):
    """The nodes that do not hold a gradient are consecutive on the circle, so each factor
    w^a - w^b of W's closed form (Sec. 3, the solve for q_j) is a unit phase times a sine and
        W[(j+t) mod P][j] = A_j * rho_t * B_{j+t},   A_j = c e^{i pi D j / P},  B_k = e^{i pi D k / P},
    D = P - 2s - 1, with REAL taps rho_t that do not depend on the node and are symmetric in t.
    Checked on the oracle's own W (the product form and, where it is accurate, the solve)."""
    D, r = P - 2 * s - 1, 2 * s + 1
    mats = [o.cyclic_weights(P, s)] + ([o.cyclic_weights_solve(P, s)] if P <= 15 else [])
    for W in mats:
        c = W[0][0] / abs(W[0][0])
        rho = np.zeros((P, r), dtype=np.complex128)
        for j in range(P):
            for t in range(r):
                rho[j, t] = W[(j + t) % P][j] / (c * np.exp(1j * np.pi * D * j / P) * np.exp(1j * np.pi * D * (j + t) / P))
        scale = np.abs(rho).max()
        tol = 1e-11 if P <= 15 else 1e-8                       # the solve and the long products lose digits at P = 45
        assert np.abs(rho.imag).max() <= tol * scale          # real
        assert np.abs(rho - rho[0]).max() <= tol * scale      # the same taps at every node
        assert np.abs(rho[0].real - rho[0].real[::-1]).max() <= tol * scale   # symmetric window
        assert (rho[0].real > 0).all()
        # and the closed form of a tap: (2^D / sqrt P) * prod over the non-holders of |sin(pi (t - u) / P)|
        want = np.array([2.0 ** D / np.sqrt(P) * np.prod([abs(np.sin(np.pi * (t - u) / P)) for u in range(r, P)])
                         for t in range(r)])
        assert np.allclose(rho[0].real, want, rtol=1e-7 if P > 15 else 1e-10)


# ------------------------------------------------ adversaries that send enormous values --
TAUS = [("one", None, o.TAU_H), ("i8", "i8", o.TAU_H_I8), ("bf16", "bf16", o.TAU_H_BF16), ("f32", "f32", o.TAU_H_WIDE)]


def _received(Z, second):
    if second is None:
        return Z.astype(np.float32).astype(np.float64)
    hi, lo = o.two_word_wire(Z, second)
    return hi.astype(np.float64) + np.asarray(lo, dtype=np.float64)


@pytest.mark.parametrize("P,s,d", [(15, 2, 4_000), (45, 3, 6_000)])
@pytest.mark.parametrize("name,second,tau", TAUS)
def test_enormous_lies_are_located_on_every_wire(P, s, d, name, second, tau):
    """Definition 2 puts no bound on what an adversary sends.  Lies from 1e2 to 1e30 times the size
    of an honest message (up to the edge of fp32) are located and the sum recovered, on every wire's
    threshold: up to about tau * 2^53 by phi as it stands, beyond that because the node is set aside
    like one that sent NaN.  The sum's tolerance is the wire's."""
    G = _grads(P, d, 5, 1e-2)
    ref = np.sum(G.astype(np.float64), axis=0)
    R0 = _received(o.encode_cyclic(G, s), second)
    f = _f(d // 2, 2)
    scale = np.abs(R0).max()
    rng = np.random.default_rng(P)
    tol = 1e-3 if name == "one" else 1e-4
    for mag in (1e2, 1e5, 1e8, 1e11, 1e14, 1e20, 1e30):
        liars = sorted(rng.choice(P, size=s, replace=False).tolist())
        R = R0.copy()
        for k, j in enumerate(liars):                      # one coherent offset, one noise, one reversed message
            if k % 3 == 0:
                R[j] += mag * scale
            elif k % 3 == 1:
                R[j] = rng.standard_normal(R.shape[1]) * mag * scale
            else:
                R[j] *= -mag
        u, mask, st = o.decode_cyclic(R, f, s, d, tau_h=tau)
        assert st == o.OK and sorted(np.flatnonzero(mask)) == liars, (mag, st, np.flatnonzero(mask), liars)
        assert np.linalg.norm(u - ref) <= tol * np.linalg.norm(ref), mag


@pytest.mark.parametrize("name,second,tau", TAUS)
def test_a_small_lie_cannot_hide_behind_an_enormous_one(name, second, tau):
    """Two colluding nodes: one sends 1e25 times an honest message, the other a lie of ordinary size
    (10 times).  The first one's fp64 rounding alone would bury the second's syndromes; with the
    first set aside the second is found."""
    P, s, d = 15, 2, 4_000
    G = _grads(P, d, 6, 1.0)
    ref = np.sum(G.astype(np.float64), axis=0)
    R0 = _received(o.encode_cyclic(G, s), second)
    f = _f(d // 2, 4)
    rng = np.random.default_rng(3)
    for (a, b) in ((2, 9), (7, 8), (14, 0)):
        R = R0.copy()
        R[a] = rng.standard_normal(R.shape[1]) * 1e25 * np.abs(R0).max()
        R[b] += 10.0 * rng.standard_normal(R.shape[1]) * np.abs(R0).max()
        u, mask, st = o.decode_cyclic(R, f, s, d, tau_h=tau)
        assert st == o.OK and sorted(np.flatnonzero(mask)) == sorted((a, b))
        assert np.linalg.norm(u - ref) <= 1e-4 * np.linalg.norm(ref)


def test_a_heavy_tailed_honest_batch_is_not_mistaken_for_lies():
    """Honest gradients may differ in size by many orders (one sample's gradient 3e9 times the
    rest, so that its five holders' projections pass the size at which a node may be set aside):
    large projections alone flag nobody -- nodes are set aside only after phi has failed."""
    P, s, d = 15, 2, 2_000
    G = _grads(P, d, 8, 1.0).astype(np.float64)
    G[4] *= 3e9
    G32 = G.astype(np.float32)
    ref = np.sum(G32.astype(np.float64), axis=0)
    Z = o.encode_cyclic(G32, s)
    f = _f(d // 2, 5)
    gamma = o.project(o.wire_to_complex(Z), f)
    big = np.abs(gamma) > o.ENORMOUS * np.median(np.abs(gamma))
    assert big.sum() > s                                                # holders of that sample: more than s of them
    u, mask, st = o.decode_cyclic(Z, f, s, d)                           # exact messages: nothing to find
    assert st == o.OK and not mask.any()
    assert np.linalg.norm(u - ref) <= 1e-6 * np.linalg.norm(ref)
    R = Z.copy()
    R[11] *= -100.0                                                     # and an ordinary liar among them is still found
    u, mask, st = o.decode_cyclic(R, f, s, d)
    assert st == o.OK and sorted(np.flatnonzero(mask)) == [11]


def test_more_enormous_lies_than_s_still_fail():
    P, s, d = 15, 2, 2_000
    G = _grads(P, d, 9, 1.0)
    R = o.encode_cyclic(G, s).astype(np.float32).astype(np.float64)
    f = _f(d // 2, 6)
    for j in (1, 5, 9):
        R[j] *= 1e28
    u, mask, st = o.decode_cyclic(R, f, s, d)
    assert st == o.LOCATE_FAILED
