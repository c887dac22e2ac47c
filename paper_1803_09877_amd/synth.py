"""Seeded synthetic inputs for the DRACO encode/decode path.

This module only MAKES inputs: per-sample gradient slabs, the random projection
vector f, adversary placements and the adversaries' edits of message slabs.  It
holds none of the method's arithmetic (no encoder, no decoder, no code
matrices) and is the one piece shared by the HIP tests, the CPU oracle tests
and the benchmark.  Everything is a torch tensor so the same recipe runs on
the host (oracle-sized cases) and on the GPU (full-sized slabs); the CPU and
GPU generators give different streams for one seed, so a case is always
generated on ONE device and copied to the other side.

Workload recipe (stand-ins for the gradients of the models the paper trains;
no dataset or checkpoint is involved): gradients are i.i.d. N(0, sigma^2)
fp32, one row per unit gradient, B = P rows ("we will assume B = P", Sec. 3).
Attacks act on the fp32 message a node sends (Sec. 4, "Adversarial Attack
Models": reversed gradient -c*g with c = 100, a constant vector, and arbitrary
replacement).
"""
from __future__ import annotations

from dataclasses import dataclass, field

import torch

SEED_BASE = 1803_09877 * 10


def padded_len(n: int, multiple: int = 4) -> int:
    """Row stride (in floats) that keeps every row 16-byte aligned."""
    return (n + multiple - 1) // multiple * multiple


def message_len(code: str, d: int) -> int:
    """Floats per message on the wire: d for the repetition code; for the
    cyclic code the ceil(d/2) complex numbers of the packed message."""
    return d if code == "rep" else 2 * ((d + 1) // 2)


def make_gradients(P: int, d: int, sigma: float, seed: int, device="cpu",
                   ld: int | None = None) -> torch.Tensor:
    """[P][ld] fp32 slab whose first d columns are N(0, sigma^2); padding is 0."""
    ld = padded_len(d) if ld is None else ld
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    out = torch.zeros((P, ld), dtype=torch.float32, device=device)
    for k in range(P):          # row by row: bounded temporary memory
        out[k, :d] = torch.randn(d, generator=g, dtype=torch.float32, device=device) * sigma
    return out


def make_projection(h: int, seed: int, device="cpu") -> torch.Tensor:
    """f ~ N(1, I) of length h (one real per packed complex coordinate), fp32."""
    g = torch.Generator(device=device)
    g.manual_seed(seed ^ 0x5F5F5F)
    return torch.randn(h, generator=g, dtype=torch.float32, device=device) + 1.0


# ---- adversaries' edits: each rewrites row j of a message slab in place ----
def attack_noise(R: torch.Tensor, j: int, n: int, seed: int, std: float = 100.0) -> None:
    """Replace node j's message by N(0, std^2) noise."""
    g = torch.Generator(device=R.device)
    g.manual_seed(seed * 1000003 + j)
    R[j, :n] = torch.randn(n, generator=g, dtype=torch.float32, device=R.device) * std


def attack_signflip(R: torch.Tensor, j: int, n: int, c: float = 100.0) -> None:
    """Reversed-gradient attack: send -c times the prescribed message."""
    R[j, :n] *= -c


def attack_offset(R: torch.Tensor, j: int, n: int, offset: float = 1e3) -> None:
    """Add a constant to every coordinate of the message."""
    R[j, :n] += offset


def attack_constant(R: torch.Tensor, j: int, n: int, kappa: float = -100.0) -> None:
    """Constant adversary: send kappa times the all-ones vector."""
    R[j, :n] = kappa


ATTACKS = {
    "noise": attack_noise,
    "signflip": attack_signflip,
    "offset": attack_offset,
    "constant": attack_constant,
}


def apply_attacks(R: torch.Tensor, n: int, adversaries, seed: int) -> None:
    """adversaries: iterable of (node, attack_name)."""
    for j, name in adversaries:
        if name == "noise":
            attack_noise(R, j, n, seed)
        else:
            ATTACKS[name](R, j, n)


@dataclass
class Workload:
    """One benchmark / parity configuration."""
    name: str
    code: str            # "rep" or "cyc"
    P: int
    s: int
    d: int
    sigma: float
    attacks: tuple       # attack name per adversary
    placement: str       # how the adversarial nodes are drawn
    decode: bool = True
    seed: int = field(default=0)
    m: int = 1           # per-sample gradients per unit gradient: the slab holds B = m*P rows

    @property
    def r(self) -> int:
        return 2 * self.s + 1

    def adversaries(self):
        """Seeded adversary placement -> list of (node, attack_name)."""
        g = torch.Generator()
        g.manual_seed(self.seed + 17)
        P, r, a = self.P, self.r, len(self.attacks)
        if a == 0:
            return []
        if self.placement == "any":
            nodes = torch.randperm(P, generator=g)[:a].tolist()
        elif self.placement == "distinct_groups":
            groups = torch.randperm(P // r, generator=g)[:a].tolist()
            nodes = [gi * r + int(torch.randint(r, (1,), generator=g)) for gi in groups]
        elif self.placement == "adjacent_pair":
            first = int(torch.randint(P, (1,), generator=g))
            nodes = [first, (first + 1) % P]
            while len(nodes) < a:
                c = int(torch.randint(P, (1,), generator=g))
                if all(min((c - n) % P, (n - c) % P) > 1 for n in nodes):
                    nodes.append(c)
        else:
            raise ValueError(self.placement)
        return list(zip(nodes, self.attacks))


def _wl(i, **kw) -> Workload:
    return Workload(seed=SEED_BASE + i, **kw)


# The five configurations the benchmark contract names, in its order, then one shaped like
# the paper's own timing runs (Sec. 4, end-to-end tables: 45 compute nodes, batch B = 180,
# s = 5) at the largest gradient length of the five.
WORKLOADS = [
    _wl(0, name="rep_P15_s1_d10k", code="rep", P=15, s=1, d=10_000, sigma=1.0,
        attacks=("noise",), placement="any"),
    _wl(1, name="rep_P45_s2_d11.2M", code="rep", P=45, s=2, d=11_200_000, sigma=1e-2,
        attacks=("signflip", "signflip"), placement="distinct_groups"),
    _wl(2, name="cyc_P15_s2_d4M", code="cyc", P=15, s=2, d=4_000_000, sigma=1.0,
        attacks=("offset", "offset"), placement="any"),
    _wl(3, name="cyc_encode_P45_s3_d25.6M", code="cyc", P=45, s=3, d=25_600_000, sigma=1e-2,
        attacks=(), placement="any", decode=False),
    _wl(4, name="cyc_P45_s3_d25.6M", code="cyc", P=45, s=3, d=25_600_000, sigma=1e-2,
        attacks=("noise", "signflip", "noise"), placement="adjacent_pair"),
    _wl(5, name="cyc_P45_s5_B180_d25.6M", code="cyc", P=45, s=5, d=25_600_000, sigma=1e-2,
        attacks=("signflip", "constant", "signflip", "constant", "signflip"), placement="any", m=4),
]


def scaled(w: Workload, d: int, name: str | None = None) -> Workload:
    """Same recipe at another gradient length (oracle-sized parity cases)."""
    return Workload(name=name or f"{w.name}@d={d}", code=w.code, P=w.P, s=w.s, d=d,
                    sigma=w.sigma, attacks=w.attacks, placement=w.placement,
                    decode=w.decode, seed=w.seed, m=w.m)
