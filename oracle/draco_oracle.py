"""CPU oracle for DRACO's encode/decode path (arXiv 1803.09877).

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain reference that the
HIP library is checked against.  It is written from the paper alone, in NumPy
fp64 / complex128, shares no code, table or constant with the HIP path and must
never be imported by it: only tests, the smoke check and the benchmark's
``cpu_baseline`` leg may call it.

Index conventions used throughout (0-based):
  * ``G`` is ``[P][d]``: row k is gradient g_k (the paper's column k of G).
  * ``Z`` / ``R`` are ``[P][len]``: row j is node j's message z_j / r_j.
  * omega = exp(2*pi*i/P);  C[m][j] = omega^(m*j)/sqrt(P)  (Sec. 3, "Cyclic
    Code", the IDFT matrix);  C_L = first P-2s rows, C_R = last 2s rows.

Readings taken where the paper's text is garbled or silent (each is repeated
at the function that uses it):
  * repetition code: P/r groups of r = 2s+1 consecutive nodes (block matrix
    A^Rep); Maj() is taken over whole message vectors with bitwise equality,
    followed by a count that the winner is held by at least s+1 nodes.
  * cyclic code: node j is assigned the 2s+1 cyclically consecutive gradients
    {j, ..., j+2s} mod P; Z = G W, so node j uses column j of W and row k of W
    is supported on the holders of gradient k.
  * complex packing pairs real coordinates; unpacking puts the real and
    imaginary parts back where they came from (it does not add them).
  * "t_j != 0" is decided in floating point: the nodes with the largest |t_j|
    (at most s) that are needed to account for the syndromes.

Pinned by tests/test_oracle_*.py against: Definition 2 by exhaustive
enumeration of adversary subsets, the 4-point example of Fig. 1 (caption),
Lemma 1, Lemma 4 (Orthogonal), the identity t = f N from the proof of Lemma 2,
a brute-force locator, Lagrange closed forms, a projection worked by hand and the
plain sum.  The numeric
coefficients drawn in Fig. 1 itself are not in the text: parity unpinned for
that picture only.
"""
from __future__ import annotations

import itertools

import numpy as np

# Status values returned by the decoders.
OK = 0
NO_MAJORITY = 1      # repetition: some group has no vector held by >= s+1 nodes
LOCATE_FAILED = 2    # cyclic: the locator's answer does not explain the syndromes

# Floating-point reading of "zero" for the syndromes h in phi (Sec. 3), relative
# to rho = median_j |f . r_j|, the size of an honest projection.  An fp32 wire
# leaves clean syndromes near 1e-7 * rho; the smallest attack the benchmark
# workloads make is near 1e-1 * rho.
TAU_H = 32.0 * 2.0 ** -24   # syndromes with max|h_m| <= TAU_H * rho count as zero (32 fp32 ulps)
# The same threshold for messages carried to 48 bits (two fp32 words): their clean syndromes
# sit near 1e-14 * rho, the rounding of the fp64 projection itself.
TAU_H_WIDE = 2.0 ** -36
# And for a two-word wire whose second word is a bfloat16 (32 bits of the message): 32 of its ulps.
TAU_H_BF16 = 32.0 * 2.0 ** -33
# And for an 8-bit second word (a fixed-point residual in units of the first word's ulp, 2^-32 of
# the message at worst): 32 of its ulps.
TAU_H_I8 = 32.0 * 2.0 ** -32


# --------------------------------------------------------------------------
# Argument checks (Theorem 1 and its corollary; "Suppose 2s+1 divides P").
# --------------------------------------------------------------------------
def check_params(code: str, P: int, s: int) -> int:
    """Return r = 2s+1 after checking the conditions the paper puts on (P, s).

    Corollary to Theorem 1: 2s+1 <= P.  Repetition code: 2s+1 divides P.
    """
    if code not in ("rep", "cyc"):
        raise ValueError("code must be 'rep' or 'cyc'")
    if P < 1 or s < 0:
        raise ValueError("need P >= 1 and s >= 0")
    r = 2 * s + 1
    if r > P:
        raise ValueError("need 2s+1 <= P (corollary to Theorem 1)")
    if code == "rep" and P % r != 0:
        raise ValueError("repetition code needs (2s+1) | P")
    return r


# --------------------------------------------------------------------------
# Repetition code (Sec. 3, "Fractional Repetition Code"; Algorithm 2).
# --------------------------------------------------------------------------
def assign_repetition(P: int, s: int) -> np.ndarray:
    """A^Rep: block diagonal with P/r all-ones r x r blocks; A[j][k] = 1 iff
    node j is assigned gradient k."""
    r = check_params("rep", P, s)
    A = np.zeros((P, P), dtype=np.uint8)
    for ell in range(P // r):
        A[ell * r:(ell + 1) * r, ell * r:(ell + 1) * r] = 1
    return A


def encode_repetition(G: np.ndarray, s: int) -> np.ndarray:
    """E^Rep: z_j = Y_j 1_P, the plain sum of the gradients assigned to node j.

    G is [P][d]; returns Z [P][d] in fp64 (the wire rounds it to fp32)."""
    G = np.asarray(G)
    P = G.shape[0]
    A = assign_repetition(P, s).astype(np.float64)
    return A @ G.astype(np.float64)


def _bits(x: np.ndarray) -> np.ndarray:
    """Bit pattern view used for 'equal': fp32 -> uint32, fp64 -> uint64."""
    x = np.ascontiguousarray(x)
    if x.dtype == np.float32:
        return x.view(np.uint32)
    if x.dtype == np.float64:
        return x.view(np.uint64)
    raise TypeError("messages must be float32 or float64")


def majority_vote_streaming(items: list) -> int:
    """Algorithm 2 (streaming majority vote): returns the INDEX of the item it
    ends on.  ``items`` are compared with ``np.array_equal`` on bit patterns."""
    ma = 0
    counter = 0
    for i in range(len(items)):
        if counter == 0:
            ma = i
            counter = 1
        elif np.array_equal(items[ma], items[i]):
            counter += 1
        else:
            counter -= 1
    return ma


def majority_vote_naive(items: list):
    """Quadratic majority by counting: index of an item equal to more than half
    of the items, or None.  Used only to cross-check Algorithm 2."""
    n = len(items)
    for i in range(n):
        c = sum(1 for k in range(n) if np.array_equal(items[i], items[k]))
        if 2 * c > n:
            return i
    return None


def decode_repetition(R: np.ndarray, s: int):
    """D^Rep(R) = sum over the P/r groups of Maj(group's r messages).

    Reading: group ell is nodes ell*r .. ell*r+r-1; Maj compares whole vectors
    bit for bit (so NaN payloads and -0 are ordinary values); Algorithm 2 gives
    the candidate and a count then confirms that at least s+1 nodes hold it
    (Algorithm 2 alone has no such check).  mask[j] = node j's message differs
    from its group's winner.  Returns (u fp64 [d], mask bool [P], status)."""
    R = np.asarray(R)
    P, d = R.shape
    r = check_params("rep", P, s)
    bits = _bits(R)
    u = np.zeros(d, dtype=np.float64)
    mask = np.zeros(P, dtype=bool)
    status = OK
    for ell in range(P // r):
        members = list(range(ell * r, (ell + 1) * r))
        items = [bits[j] for j in members]
        win = majority_vote_streaming(items)
        same = [np.array_equal(items[win], it) for it in items]
        if sum(same) < s + 1:
            status = NO_MAJORITY
        for j, eq in zip(members, same):
            mask[j] = not eq
        u += R[members[win]].astype(np.float64)
    return u, mask, status


# --------------------------------------------------------------------------
# Cyclic code: plan (Sec. 3, "Cyclic Code": A^Cyc, C, C_L, C_R, q_j, W).
# --------------------------------------------------------------------------
def assign_cyclic(P: int, s: int) -> np.ndarray:
    """A^Cyc under the unit-shift reading: node j holds gradients j..j+2s mod P
    (the "P starting positions on a circle" description)."""
    check_params("cyc", P, s)
    A = np.zeros((P, P), dtype=np.uint8)
    for j in range(P):
        for t in range(2 * s + 1):
            A[j, (j + t) % P] = 1
    return A


def idft_matrix(P: int) -> np.ndarray:
    """C[m][j] = exp(2 pi i m j / P) / sqrt(P)."""
    idx = np.arange(P)
    mj = np.outer(idx, idx) % P
    return np.exp(2j * np.pi * mj / P) / np.sqrt(P)


def cyclic_weights_solve(P: int, s: int) -> np.ndarray:
    """W = [Q 1] C_L with each q_k from [q_k 1] . C_L[:, alpha_k] = 0.

    Reading of the row/column roles: Z = G W, so row k of W multiplies gradient
    k and must vanish on alpha_k = the nodes that do NOT hold gradient k
    (|alpha_k| = P-2s-1).  The linear solve is the paper's construction; it is
    the numerically weaker of the two routes for large P (see
    ``cyclic_weights``)."""
    check_params("cyc", P, s)
    A = assign_cyclic(P, s)
    C = idft_matrix(P)
    n = P - 2 * s
    CL = C[:n]
    W = np.zeros((P, P), dtype=np.complex128)
    for k in range(P):
        alpha = [j for j in range(P) if A[j, k] == 0]
        if n - 1 > 0:
            M = CL[:n - 1][:, alpha]            # (n-1) x (n-1)
            rhs = -CL[n - 1, alpha]
            q = np.linalg.solve(M.T, rhs)
        else:
            q = np.zeros(0, dtype=np.complex128)
        row = np.concatenate([q, [1.0]]) @ CL
        row[alpha] = 0.0
        W[k] = row
    return W


def cyclic_weights(P: int, s: int) -> np.ndarray:
    """The same W in closed form.  [q_k 1] C_L restricted to column j is
    (1/sqrt P) * p_k(omega^j) with p_k the MONIC polynomial of degree P-2s-1
    (coefficients q_k, leading 1); the defining equations say p_k vanishes at
    omega^m for every m in alpha_k, and a monic polynomial of that degree with
    P-2s-1 prescribed roots is unique:
        W[k][j] = (1/sqrt P) * prod_{m in alpha_k} (omega^j - omega^m).
    The product has no cancellation, so this is accurate to a few ulp where the
    solve loses digits; tests assert the two agree."""
    check_params("cyc", P, s)
    A = assign_cyclic(P, s)
    x = np.exp(2j * np.pi * np.arange(P) / P)
    W = np.zeros((P, P), dtype=np.complex128)
    for k in range(P):
        alpha = [m for m in range(P) if A[m, k] == 0]
        for j in range(P):
            if A[j, k]:
                W[k, j] = np.prod(x[j] - x[alpha]) / np.sqrt(P)
    return W


# --------------------------------------------------------------------------
# Complex packing (end of Sec. 3).
# --------------------------------------------------------------------------
def pack_complex(X: np.ndarray, pairing: str = "interleaved") -> np.ndarray:
    """Real [.., d] -> complex [.., ceil(d/2)].

    'halves' is the paper's pairing (component i = x_i + 1j * x_{ceil(d/2)+i});
    'interleaved' pairs (x_{2i}, x_{2i+1}) and is the wire layout of the
    library.  A missing last imaginary part (odd d) is 0."""
    X = np.asarray(X, dtype=np.float64)
    d = X.shape[-1]
    h = (d + 1) // 2
    pad = np.zeros(X.shape[:-1] + (2 * h,), dtype=np.float64)
    pad[..., :d] = X
    if pairing == "interleaved":
        return pad[..., 0::2] + 1j * pad[..., 1::2]
    if pairing == "halves":
        return pad[..., :h] + 1j * pad[..., h:]
    raise ValueError(pairing)


def unpack_complex(Xc: np.ndarray, d: int, pairing: str = "interleaved") -> np.ndarray:
    """Inverse of pack_complex: real and imaginary parts go back to the real
    coordinates they were taken from (reading of "sum the real and imaginary
    parts": as written the two halves would be added onto each other, which is
    not G 1_P; the parts are concatenated instead)."""
    Xc = np.asarray(Xc)
    h = Xc.shape[-1]
    out = np.zeros(Xc.shape[:-1] + (2 * h,), dtype=np.float64)
    if pairing == "interleaved":
        out[..., 0::2] = Xc.real
        out[..., 1::2] = Xc.imag
    elif pairing == "halves":
        out[..., :h] = Xc.real
        out[..., h:] = Xc.imag
    else:
        raise ValueError(pairing)
    return out[..., :d]


def wire_to_complex(R: np.ndarray) -> np.ndarray:
    """Message slab as stored on the wire ([P][2h] reals, interleaved re/im)
    -> complex [P][h] in complex128."""
    R = np.asarray(R)
    return R[..., 0::2].astype(np.float64) + 1j * R[..., 1::2].astype(np.float64)


def complex_to_wire(Zc: np.ndarray) -> np.ndarray:
    """complex [P][h] -> fp64 [P][2h] interleaved (rounding to fp32 is the
    caller's business)."""
    out = np.zeros(Zc.shape[:-1] + (2 * Zc.shape[-1],), dtype=np.float64)
    out[..., 0::2] = Zc.real
    out[..., 1::2] = Zc.imag
    return out


def round_to_bfloat16(x: np.ndarray) -> np.ndarray:
    """fp32 values rounded to the nearest bfloat16 (1 sign, 8 exponent, 7 fraction bits: the
    upper half of the fp32 word), ties to the even neighbour; returned as fp32.  NaN stays
    NaN.  The number format is the published one; Sec. 3 leaves a message's format open."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32).astype(np.uint64)
    keep = bits >> 16
    rest = bits & 0xFFFF
    up = (rest > 0x8000) | ((rest == 0x8000) & ((keep & 1) == 1))
    out = ((keep + up.astype(np.uint64)) << 16).astype(np.uint32).view(np.float32)
    return np.where(np.isnan(x), x, out).astype(np.float32)


def _ulp_exponent(hi: np.ndarray) -> np.ndarray:
    """k with 2^k = the spacing of fp32 numbers at hi, from hi's exponent field E: k = max(E, 24) - 150
    (fields below 24, numbers under 2^-103, share the spacing 2^-126: their residuals do not matter)."""
    E = ((np.ascontiguousarray(hi, dtype=np.float32).view(np.uint32) >> 23) & 0xFF).astype(np.int64)
    return np.maximum(E, 24) - 150


def residual_code8(hi: np.ndarray, r: np.ndarray) -> np.ndarray:
    """The rounding residual r = z - hi (|r| <= half the spacing u of fp32 numbers at hi) as an
    8-bit fixed-point code: q = r / u * 254 rounded to the nearest integer, ties to even, so
    q in [-127, 127]; 0 where hi is not finite.  The arithmetic is fp32, as the encoder kernels do
    it: (fp32(r) * 2^-8 / u) * (254 * 2^8), the first product exact, the second rounded once."""
    hi = np.ascontiguousarray(hi, dtype=np.float32)
    r32 = np.asarray(r, dtype=np.float32)
    k = _ulp_exponent(hi)
    with np.errstate(invalid="ignore", over="ignore"):
        t = (r32 * np.ldexp(np.float32(1.0), (-8 - k).astype(np.int32)).astype(np.float32)) * np.float32(65024.0)
        q = np.clip(np.rint(t), -127.0, 127.0)
    q = np.where(np.isfinite(hi) & np.isfinite(q), q, 0.0)
    return q.astype(np.int8)


def residual_from_code8(hi: np.ndarray, q: np.ndarray) -> np.ndarray:
    """What a code of residual_code8 stands for: q * u / 254 (fp64)."""
    return np.asarray(q, dtype=np.float64) * np.ldexp(1.0, _ulp_exponent(hi)) / 254.0


def two_word_wire(Z: np.ndarray, second: str = "f32"):
    """An fp64 message slab as two words per value: hi = fp32(z) and lo = the rounding
    residual z - hi, itself rounded to fp32 ("f32"), to bfloat16 ("bf16"), or to the 8-bit
    code of residual_code8 ("i8").  Returns hi (fp32) and the VALUE the second word stands
    for (fp32; fp64 for "i8", whose values need not be fp32 numbers)."""
    Z = np.asarray(Z, dtype=np.float64)
    with np.errstate(over="ignore"):
        hi = Z.astype(np.float32)
    with np.errstate(invalid="ignore"):
        lo = (Z - hi.astype(np.float64)).astype(np.float32)
    if second == "bf16":
        lo = round_to_bfloat16(lo)
    elif second == "i8":
        lo = residual_from_code8(hi, residual_code8(hi, lo))
    elif second != "f32":
        raise ValueError(second)
    return hi, lo


# --------------------------------------------------------------------------
# Cyclic code: encoder  E^Cyc_j(Y_j) = G W_{.,j}.
# --------------------------------------------------------------------------
def encode_cyclic_complex(Gc: np.ndarray, s: int, W: np.ndarray | None = None) -> np.ndarray:
    """Z = G W on packed gradients: Zc[j] = sum_{k in S_j} W[k][j] * Gc[k],
    S_j the gradients assigned to node j.  Gc is [P][h] complex."""
    Gc = np.asarray(Gc, dtype=np.complex128)
    P = Gc.shape[0]
    if W is None:
        W = cyclic_weights(P, s)
    A = assign_cyclic(P, s)
    Zc = np.zeros_like(Gc)
    for j in range(P):
        for k in range(P):
            if A[j, k]:
                Zc[j] += W[k, j] * Gc[k]
    return Zc


def encode_cyclic(G: np.ndarray, s: int, pairing: str = "interleaved") -> np.ndarray:
    """Real gradients [P][d] -> wire messages [P][2*ceil(d/2)] in fp64
    (interleaved re/im of the complex message)."""
    Gc = pack_complex(G, pairing)
    return complex_to_wire(encode_cyclic_complex(Gc, s))


# --------------------------------------------------------------------------
# Cyclic code: the locator phi (Sec. 3) and a definition-level cross-check.
# --------------------------------------------------------------------------
def projection_vector(h: int, seed: int) -> np.ndarray:
    """The counter-based f ~ N(1, I) of the library's boundary, entry i from (seed, i):
    z = splitmix64's finaliser on seed + (i+1)*0x9E3779B97F4A7C15 (mod 2^64); u1 and u2
    are its top 24 bits and its bits 16..39, each plus 1/2, over 2^24; Box-Muller in fp64,
    f_i = fp32(1 + sqrt(-2 ln u1) cos(2 pi u2)).  Written out here independently of the
    library so that both sides of a parity test can draw the same vector."""
    M = (1 << 64) - 1
    out = np.empty(h, dtype=np.float32)
    for i in range(h):            # plain Python integers: exact 64-bit wrap-around
        z = (seed + (i + 1) * 0x9E3779B97F4A7C15) & M
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M
        z ^= z >> 31
        u1 = ((z >> 40) + 0.5) / 16777216.0
        u2 = (((z >> 16) & 0xFFFFFF) + 0.5) / 16777216.0
        out[i] = np.float32(1.0 + np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2))
    return out


def project(Rc: np.ndarray, f: np.ndarray) -> np.ndarray:
    """gamma'_j = sum_i f_i * r_j[i]  (the row vector f R of phi's first step);
    Rc is [P][h] complex, f is [h] real."""
    return np.asarray(Rc, dtype=np.complex128) @ np.asarray(f, dtype=np.float64)


def syndromes(gamma: np.ndarray, s: int) -> np.ndarray:
    """[h_{P-2s}, ..., h_{P-1}] = (f R) C_R^dagger, in ascending index order:
    h_m = sum_j gamma'_j * conj(C[m][j])."""
    P = gamma.shape[0]
    C = idft_matrix(P)
    return np.conj(C[P - 2 * s:]) @ gamma


def _unexplained(hk: np.ndarray, P: int, s: int, V: list) -> float:
    """Largest syndrome magnitude left after the best fit by errors on V alone
    (Lemma 4: the syndromes of R are those of N, i.e. conj(C_R)[:, V] gamma_V)."""
    if len(V) == 0:
        return float(np.max(np.abs(hk)))
    M = np.conj(idft_matrix(P)[P - 2 * s:])[:, list(V)]
    return float(np.max(np.abs(hk - M @ np.linalg.lstsq(M, hk, rcond=None)[0])))


# A projection more than this many times rho in size is "enormous": its fp64 rounding (2^-53 of
# it), times the error growth of the s-error locator (1e3 - 1e5 at P = 45), comes within reach of
# the zero thresholds.  Lies of a hundred times an honest message stay below it.  See
# phi_from_projection.
ENORMOUS = 2.0 ** 10
# A node that phi HAS located needs setting aside only when the rounding of its projection
# (2^-53 of it, summed over up to 256 nodes) could pass for a syndrome: beyond tau_h * 2^44 * rho.
LOCATED_ENORMOUS_OVER_TAU = 2.0 ** 44


def _phi_attempt(gamma: np.ndarray, s: int, tau_h: float):
    """One pass of phi's steps 2-4 on finite projections -> (located nodes in ranking order, t, found)."""
    P = gamma.shape[0]
    t = np.zeros(P, dtype=np.complex128)
    rho = float(np.median(np.abs(gamma)))
    hk = syndromes(gamma, s)
    if _unexplained(hk, P, s, []) <= tau_h * rho:
        return [], t, True
    h = np.zeros(P, dtype=np.complex128)
    h[P - 2 * s:] = hk
    H = np.empty((s, s), dtype=np.complex128)
    rhs = np.empty(s, dtype=np.complex128)
    for i in range(1, s + 1):
        for k in range(s):
            H[i - 1, k] = h[P - s - i + k]
        rhs[i - 1] = h[P - i]
    Us, sv, Vh = np.linalg.svd(H)
    keep = sv > tau_h * rho
    beta = (Vh.conj().T[:, keep] * (1.0 / sv[keep])) @ (Us.conj().T[keep] @ rhs)
    for ell in range(P - 2 * s):
        acc = 0.0 + 0.0j
        for u in range(s):
            acc += beta[u] * h[(ell + u - s) % P]
        h[ell] = acc
    t = idft_matrix(P) @ h
    order = [int(j) for j in np.argsort(-np.abs(t), kind="stable")[:s]]
    for a in range(1, s + 1):
        if _unexplained(hk, P, s, order[:a]) <= tau_h * rho:
            return order[:a], t, True
    return order, t, False


def phi_from_projection(gamma: np.ndarray, s: int, tau_h: float = TAU_H):
    """phi's steps 2-4 on the P projections gamma' = f R.

    1. h_{P-2s..P-1} from ``syndromes``.
    2. beta from the s x s system whose row i (i = 1..s) reads
         sum_{k=0}^{s-1} beta_k h_{P-s-i+k} = h_{P-i}
       (the printed last row is garbled; this is the row pattern of the first
       rows continued, and the one the proof of Lemma 5 derives).
    3. h_l = sum_u beta_u h_{l+u-s} for l = 0..P-2s-1 (indices mod P).
    4. t = C h;  V = {j : t_j != 0}.
    Floating-point reading.  rho = median |gamma'_j| is the size of an honest
    projection; a syndrome is "zero" when it is below tau_h*rho.  If every
    syndrome is zero there is no adversary.  The s x s system is singular when
    fewer than s nodes lie ("any solution" in the proof of Lemma 2), so it is
    solved in the least-squares sense with singular values below tau_h*rho
    dropped.  "t_j != 0" is decided by need: nodes are ranked by |t_j| and V is
    the shortest leading part of that ranking (at most s nodes) whose errors
    account for the syndromes, i.e. leave them zero after a least-squares fit.
    In exact arithmetic t has exactly |V| non-zeros and this is the same set.
    Returns (mask, t, status); LOCATE_FAILED when no leading part of length
    <= s accounts for the syndromes (more than s liars), with mask = the s
    largest |t_j| as a best effort.

    Messages that are no vectors of R^d, or none that fp64 can weigh: a node
    whose projection is NaN or Inf is flagged outright and its projection taken
    as 0, which leaves an ordinary error f.(-z_j) at a known node for the steps
    above to account for like any other.  A finite projection can still be so
    large that its own fp64 rounding drowns the zero threshold, or swallows a
    smaller lie whole (the adversary may send 1e30).  Call a projection
    enormous when it exceeds ENORMOUS * rho.  After the steps above, the
    located nodes whose projection is enormous and beyond tau_h * 2^44 * rho
    (so large that its rounding could pass for a syndrome) are treated like
    broken ones (flagged, projection 0); if the steps found no set, the top
    layer of the enormous nodes is (those within a factor ENORMOUS of the
    largest).  Then
    the steps run again, provided the flagged nodes stay within s; this
    repeats (lies of 1e30, 1e20 and 1e10 come off one layer at a time) until a
    pass sets nothing aside, whose result stands.  Nodes that phi did not
    locate are never set aside while phi succeeds, so an honest batch with a
    heavy tail flags nobody.  (The paper's n_j are arbitrary reals and its
    arithmetic exact; this is what keeps Definition 2 for them.)
    """
    gamma = np.array(gamma, dtype=np.complex128)
    P = gamma.shape[0]
    mask = np.zeros(P, dtype=bool)
    broken = ~np.isfinite(gamma)
    gamma[broken] = 0.0
    mask |= broken
    if s == 0:
        return mask, np.zeros(P, dtype=np.complex128), (LOCATE_FAILED if broken.any() else OK)
    if int(broken.sum()) > s:
        return mask, np.zeros(P, dtype=np.complex128), LOCATE_FAILED
    while True:          # every pass but the last flags at least one more node: at most s + 1 passes
        located, t, found = _phi_attempt(gamma, s, tau_h)
        rho = float(np.median(np.abs(gamma)))
        size = np.abs(gamma)
        aside = (size > ENORMOUS * rho) & ~mask
        if found:
            among = np.zeros(P, dtype=bool)
            among[located] = True
            aside &= among & (size > LOCATED_ENORMOUS_OVER_TAU * tau_h * rho)
        elif aside.any():
            aside &= size * ENORMOUS > size[aside].max()
        if not aside.any() or int((mask | aside).sum()) > s:
            break
        gamma[aside] = 0.0
        mask |= aside
    mask[located] = True
    return mask, t, (OK if found and int(mask.sum()) <= s else LOCATE_FAILED)


def phi(Rc: np.ndarray, f: np.ndarray, s: int) -> np.ndarray:
    """V = phi(R) as a boolean mask over nodes."""
    return phi_from_projection(project(Rc, f), s)[0]


def phi_bruteforce(gamma: np.ndarray, s: int, tau_h: float = TAU_H) -> np.ndarray:
    """Locator by definition, for tiny P: the smallest node set V (|V| <= s)
    such that the 2s syndromes are those of an error vector supported on V.
    By Lemma 4 the syndromes of R are those of N; columns of C_R restricted to
    at most 2s nodes are independent (Vandermonde), so the set is unique."""
    gamma = np.asarray(gamma, dtype=np.complex128)
    P = gamma.shape[0]
    rho = float(np.median(np.abs(gamma)))
    hk = syndromes(gamma, s)
    CRc = np.conj(idft_matrix(P)[P - 2 * s:])       # h = CRc @ gamma
    for a in range(0, s + 1):
        for V in itertools.combinations(range(P), a):
            if a == 0:
                resid = hk
            else:
                M = CRc[:, list(V)]
                sol = np.linalg.lstsq(M, hk, rcond=None)[0]
                resid = hk - M @ sol
            if float(np.max(np.abs(resid))) <= tau_h * max(rho, np.finfo(float).tiny):
                mask = np.zeros(P, dtype=bool)
                mask[list(V)] = True
                return mask
    return None


# --------------------------------------------------------------------------
# Cyclic code: recombination vector b and the decoder D^Cyc (Algorithm 1).
# --------------------------------------------------------------------------
def solve_b(P: int, s: int, U: list, mode: str = "min_norm") -> np.ndarray:
    """b (length P, zero outside U) with W_{.,U} b = 1_P.

    Route of the proof of Lemma 1: since W = [Q 1] C_L it is enough that
    C_L[:, U] b_U = (0, ..., 0, 1)^T.  'first' uses the first P-2s nodes of U
    exactly as in that proof; 'min_norm' takes the minimum-2-norm solution over
    all of U (any solution gives G 1_P in exact arithmetic; the smallest one
    amplifies wire rounding least)."""
    U = list(U)
    n = P - 2 * s
    if len(U) < n:
        raise ValueError("need at least P-2s honest nodes")
    CL = idft_matrix(P)[:n]
    e = np.zeros(n, dtype=np.complex128)
    e[n - 1] = 1.0
    b = np.zeros(P, dtype=np.complex128)
    if mode == "first":
        Ub = U[:n]
        b[Ub] = np.linalg.solve(CL[:, Ub], e)
    elif mode == "min_norm":
        M = CL[:, U]
        bu = np.linalg.lstsq(M, e, rcond=None)[0]
        # one step of refinement on the residual keeps C_L b = e to rounding
        bu = bu + np.linalg.lstsq(M, e - M @ bu, rcond=None)[0]
        b[U] = bu
    else:
        raise ValueError(mode)
    return b


def decode_cyclic_complex(Rc: np.ndarray, f: np.ndarray, s: int, b_mode: str = "min_norm",
                          tau_h: float = TAU_H):
    """Algorithm 1 on packed messages: V = phi(R); U = complement; b from
    ``solve_b``; u_hat = R_{.,U} b.  Returns (u_hat complex [h], mask, status).
    status LOCATE_FAILED comes from phi (more than s nodes lied); u_hat is
    then not to be trusted."""
    Rc = np.asarray(Rc, dtype=np.complex128)
    P = Rc.shape[0]
    check_params("cyc", P, s)
    gamma = project(Rc, f)
    mask, _, status = phi_from_projection(gamma, s, tau_h)
    U = [j for j in range(P) if not mask[j]]
    if len(U) < P - 2 * s:
        return np.full(Rc.shape[1], np.nan, dtype=np.complex128), mask, LOCATE_FAILED
    b = solve_b(P, s, U, b_mode)
    u_hat = np.zeros(Rc.shape[1], dtype=np.complex128)
    for j in U:
        u_hat += b[j] * Rc[j]
    return u_hat, mask, status


def decode_cyclic(R: np.ndarray, f: np.ndarray, s: int, d: int, b_mode: str = "min_norm",
                  tau_h: float = TAU_H):
    """Wire messages [P][2h] (interleaved re/im) -> (u fp64 [d], mask, status)."""
    u_hat, mask, status = decode_cyclic_complex(wire_to_complex(R), f, s, b_mode, tau_h)
    return unpack_complex(u_hat, d, "interleaved"), mask, status


# --------------------------------------------------------------------------
# Cyclic code on the real gradients directly (Sec. 3 before its closing remark
# on packing): messages carry d complex entries.
# --------------------------------------------------------------------------
def encode_cyclic_unpacked(G: np.ndarray, s: int) -> np.ndarray:
    """Z = G W with the real G [P][d] taken as complex; wire [P][2d] (re/im interleaved)."""
    return complex_to_wire(encode_cyclic_complex(np.asarray(G, dtype=np.float64).astype(np.complex128), s))


def decode_cyclic_unpacked(R: np.ndarray, f: np.ndarray, s: int, b_mode: str = "min_norm"):
    """Wire messages [P][2d] -> (u fp64 [d] = Re(R_{.,U} b), mask, status, residual), f of
    length d.  G 1_P is real, so the imaginary part of the recombination carries only
    rounding; its largest magnitude is returned as `residual` for tests to bound."""
    u_hat, mask, status = decode_cyclic_complex(wire_to_complex(R), f, s, b_mode)
    return u_hat.real.copy(), mask, status, float(np.max(np.abs(u_hat.imag))) if u_hat.size else 0.0


# --------------------------------------------------------------------------
# Parameter server: the model update (Sec. 2, "Distributed Training").
# --------------------------------------------------------------------------
def sgd_update(w: np.ndarray, grad_sum: np.ndarray, gamma: float, batch: int) -> np.ndarray:
    """Mini-batch SGD's step with the recovered gradient sum:
    w_k = w_{k-1} - (gamma / |S_k|) * sum_{i in S_k} g_i, in fp64."""
    w = np.asarray(w, dtype=np.float64)
    return w - (float(gamma) / float(batch)) * np.asarray(grad_sum, dtype=np.float64)
