"""Pins for the repetition-code half of the CPU oracle (no GPU).

What fixes the expected values here is the paper, not the oracle: Definition 2
(decode equals the plain gradient sum for EVERY adversary set of size <= s,
Theorem 2), the block structure of A^Rep, the redundancy ratio of Definition 1,
the majority property of Algorithm 2 and the s = 0 special case (plain
mini-batch SGD, A = I)."""
import itertools

import numpy as np
import pytest

from oracle import draco_oracle as o


def _grads(P, d, seed, sigma=1.0):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((P, d)) * sigma).astype(np.float32)


def _attack(R, j, kind, rng):
    """Adversarial edits of one fp32 message, including the nasty bit-level ones."""
    if kind == "noise":
        R[j] = (rng.standard_normal(R.shape[1]) * 100).astype(np.float32)
    elif kind == "signflip":
        R[j] = R[j] * np.float32(-100.0)
    elif kind == "constant":
        R[j] = np.float32(-100.0)
    elif kind == "one_ulp":          # a single coordinate off by one ulp
        i = int(rng.integers(R.shape[1]))
        R[j, i] = np.nextafter(R[j, i], np.float32(np.inf))
    elif kind == "nan":
        R[j, int(rng.integers(R.shape[1]))] = np.nan
    elif kind == "neg_zero":         # +0 -> -0 compares equal as floats, not as bits
        R[j, j] = -0.0               # the caller made coordinate j +0 on every node
    else:
        raise ValueError(kind)


@pytest.mark.parametrize("P,s", [(3, 1), (6, 1), (9, 1), (15, 1), (5, 2), (10, 2), (15, 2), (7, 3), (15, 7)])
def test_assignment_matrix_structure(P, s):
    A = o.assign_repetition(P, s)
    r = 2 * s + 1
    assert A.shape == (P, P)
    assert int(A.sum()) == P * r                    # Definition 1: ||A||_0 / P = r
    assert np.array_equal(A, A.T)
    for j in range(P):
        ones = np.flatnonzero(A[j])
        assert len(ones) == r and ones[0] == (j // r) * r and ones[-1] == ones[0] + r - 1


@pytest.mark.parametrize("code,P,s", [("rep", 10, 1), ("rep", 4, 2), ("cyc", 4, 2), ("cyc", 0, 0), ("rep", 5, -1), ("x", 3, 1)])
def test_parameter_conditions_rejected(code, P, s):
    with pytest.raises(ValueError):
        o.check_params(code, P, s)


def test_encode_is_the_group_sum_and_copies_agree():
    P, s, d = 15, 2, 257
    G = _grads(P, d, 1)
    Z = o.encode_repetition(G, s)
    r = 2 * s + 1
    for j in range(P):                              # every node of a group sends the same vector
        assert np.array_equal(Z[j], Z[(j // r) * r])
    # one message per group adds up to the full gradient sum G 1_P
    assert np.allclose(Z[::r].sum(0), G.astype(np.float64).sum(0), rtol=0, atol=1e-12)
    # and each is the sum of exactly its r gradients (textbook routine on the slice)
    for ell in range(P // r):
        assert np.allclose(Z[ell * r], np.add.reduce(G[ell * r:(ell + 1) * r].astype(np.float64), axis=0), atol=1e-13)


def test_s0_is_plain_minibatch_sum():
    G = _grads(6, 100, 2)
    Z = o.encode_repetition(G, 0)
    assert np.array_equal(Z, G.astype(np.float64))          # A = I, E_j returns g_j
    u, mask, st = o.decode_repetition(G, 0)
    assert st == o.OK and not mask.any()
    assert np.allclose(u, np.sum(G.astype(np.float64), axis=0), atol=1e-13)


@pytest.mark.parametrize("n,alphabet,seed", [(n, a, sd) for n in (1, 2, 3, 5, 7, 11) for a in (1, 2, 3) for sd in range(8)])
def test_streaming_vote_finds_the_majority_when_one_exists(n, alphabet, seed):
    rng = np.random.default_rng(1000 * n + 10 * alphabet + seed)
    vals = rng.integers(alphabet, size=n)
    items = [np.array([v, v + 1], dtype=np.uint32) for v in vals]
    naive = o.majority_vote_naive(items)
    got = o.majority_vote_streaming(items)
    counts = np.bincount(vals, minlength=alphabet)
    if counts.max() * 2 > n:                                 # a majority exists: both must name it
        assert naive is not None
        assert vals[got] == np.argmax(counts) == vals[naive]
    else:
        assert naive is None


@pytest.mark.parametrize("P,s", [(3, 1), (6, 1), (9, 1), (5, 2), (10, 2), (7, 3)])
@pytest.mark.parametrize("kind", ["noise", "signflip", "constant", "one_ulp", "nan", "neg_zero"])
def test_definition2_every_adversary_subset(P, s, kind):
    """Theorem 2: for every set of at most s adversarial nodes (also all inside
    one group) the decoder returns G 1_P and names exactly the liars."""
    d = 33
    G = _grads(P, d, 7 * P + s)
    Z32 = o.encode_repetition(G, s).astype(np.float32)       # fp32 wire
    rng = np.random.default_rng(P * 100 + s)
    for a in range(0, s + 1):
        for V in itertools.combinations(range(P), a):
            R = Z32.copy()
            if kind == "neg_zero":
                R[:, :P] = 0.0                              # honest value +0 in the first P coordinates
            for j in V:
                _attack(R, j, kind, rng)
            if kind == "neg_zero" and a == 0:
                continue
            honest = R.copy()
            u, mask, st = o.decode_repetition(R, s)
            assert st == o.OK
            assert sorted(np.flatnonzero(mask)) == sorted(V)
            # the decoded vector is bit-for-bit the sum of one honest copy per group
            r = 2 * s + 1
            expect = np.zeros(d)
            for ell in range(P // r):
                good = [j for j in range(ell * r, (ell + 1) * r) if j not in V][0]
                expect += honest[good].astype(np.float64)
            assert np.array_equal(u, expect)
            if kind != "neg_zero":
                ref = np.sum(G.astype(np.float64), axis=0)   # Definition 2, up to the fp32 wire
                assert np.linalg.norm(u - ref) <= 1e-6 * np.linalg.norm(ref)


def test_fp64_wire_is_exact():
    P, s, d = 9, 1, 50
    G = _grads(P, d, 3)
    Z = o.encode_repetition(G, s)
    R = Z.copy()
    R[4] = -100.0 * R[4]
    u, mask, st = o.decode_repetition(R, s)
    assert st == o.OK and list(np.flatnonzero(mask)) == [4]
    assert np.allclose(u, np.sum(G.astype(np.float64), axis=0), rtol=0, atol=1e-13)


def test_more_than_s_liars_is_reported_or_wins():
    """Outside the contract (more than s adversaries in one group): s+1 distinct
    liars leave no vector held by s+1 nodes -> NO_MAJORITY; s+1 colluding liars
    sending one common vector are the majority and win (Theorem 1: nothing can
    prevent that with r = 2s+1)."""
    P, s, d = 5, 2, 20
    G = _grads(P, d, 5)
    Z32 = o.encode_repetition(G, s).astype(np.float32)
    R = Z32.copy()
    for j in (0, 2, 4):
        R[j] = np.float32(j + 1)
    _, mask, st = o.decode_repetition(R, s)
    assert st == o.NO_MAJORITY
    R = Z32.copy()
    for j in (0, 2, 4):
        R[j] = np.float32(9.0)
    u, mask, st = o.decode_repetition(R, s)
    assert st == o.OK and sorted(np.flatnonzero(mask)) == [1, 3]
    assert np.array_equal(u, np.full(d, 9.0))


def test_planted_mistakes_are_caught():
    """A wrong group boundary or a float (not bitwise) comparison must fail the pins:
    run the checks above against deliberately broken variants."""
    P, s, d = 6, 1, 16
    G = _grads(P, d, 11)
    Z32 = o.encode_repetition(G, s).astype(np.float32)
    # float equality would call -0 == +0 and miss the adversary
    R = Z32.copy()
    R[:, 3] = 0.0
    R[1, 3] = -0.0
    assert np.array_equal(R[0], R[1])                        # equal as floats ...
    _, mask, _ = o.decode_repetition(R, s)
    assert list(np.flatnonzero(mask)) == [1]                 # ... but the oracle sees the bits
    # groups shifted by one node no longer vote among copies of the same sum
    shifted = np.roll(Z32, 1, axis=0)
    _, mask, st = o.decode_repetition(shifted, s)
    assert mask.any()
