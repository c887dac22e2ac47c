"""Device-side harness around the library for one workload: allocates the
slabs, fills them from the seeded generators, and calls the C-ABI entry points
through the binding.  Used by the GPU tests, the smoke check and the benchmark.
It holds no arithmetic of the method."""
from __future__ import annotations

import torch

from . import binding as B
from . import synth


class Case:
    """Slabs of one workload resident in HBM.

    G  [B][ld_g]  per-sample gradients, B = m*P rows (m = 1: one unit gradient per row)
    Z  [P][ld_m]  messages as the encoder wrote them
    R  [P][ld_m]  messages as received: Z with the adversaries' edits
    u  [d_pad]    decoded sum
    f  [ceil(d/2)] phi's random projection vector (cyclic code)
    """

    def __init__(self, w: synth.Workload, device: str = "cuda:0", wide=False, unpacked: bool = False):
        """wide: cyclic code with the two-word wire (Zlo / Rlo hold the second word): True or
        "f32" for a float32 second word, "bf16" for a bfloat16 one, "i8" for an 8-bit residual code;
        unpacked: cyclic code with d complex entries per message (f then has d entries)."""
        self.w = w
        assert wide in (False, True, "f32", "bf16", "i8")
        self.lo_dtype = {"bf16": torch.bfloat16, "i8": torch.int8}.get(wide, torch.float32)
        wide = bool(wide)
        self.wide = wide
        self.unpacked = unpacked
        assert not ((wide or unpacked) and w.code != "cyc") and not (wide and unpacked)
        self.device = torch.device(device)
        code = B.CODE_REPETITION if w.code == "rep" else B.CODE_CYCLIC
        self.plan = B.Plan(code, w.P, w.s, w.d)
        if unpacked:
            self.plan.set_wire(B.WIRE_UNPACKED)
        if self.lo_dtype != torch.float32:
            self.plan.set_second_word(B.SECOND_WORD_BF16 if self.lo_dtype == torch.bfloat16 else B.SECOND_WORD_I8)
        self.mlen = self.plan.message_len
        self.ld_g = synth.padded_len(w.d)
        self.ld_m = synth.padded_len(self.mlen)
        self.G = synth.make_gradients(w.P * w.m, w.d, w.sigma, w.seed, device=self.device, ld=self.ld_g)
        self.Z = torch.zeros((w.P, self.ld_m), dtype=torch.float32, device=self.device)
        self.R = None
        self.Zlo = torch.zeros_like(self.Z, dtype=self.lo_dtype) if wide else None
        self.Rlo = None
        self.u = torch.zeros(synth.padded_len(w.d), dtype=torch.float32, device=self.device)
        self.f = None
        if w.code == "cyc":
            self.f = synth.make_projection(self.mlen // 2, w.seed, device=self.device)
        self.adversaries = w.adversaries()
        self.plan.prepare()

    def encode(self, stream=None) -> None:
        if self.w.m > 1:
            if self.wide:
                self.plan.encode_samples_wide(self.G, self.Z, self.Zlo, stream)
            else:
                self.plan.encode_samples(self.G, self.Z, stream)
        elif self.wide:
            self.plan.encode_wide(self.G, self.Z, self.Zlo, stream)
        else:
            self.plan.encode(self.G, self.Z, stream)

    def receive(self) -> None:
        """R <- Z, then the adversaries rewrite their rows (outside the hot path).
        On the wide wire they edit the first word; the second stays as sent."""
        self.R = self.Z.clone()
        if self.wide:
            self.Rlo = self.Zlo.clone()
        synth.apply_attacks(self.R, self.mlen, self.adversaries, self.w.seed)

    def decode(self, stream=None, hostphi: bool = False):
        """-> (mask bool[P], status); the sum lands in self.u[:d].  hostphi selects the
        cyclic decoder whose small linear algebra runs on the host."""
        if self.w.code == "rep":
            return self.plan.decode_repetition(self.R, self.u, stream)
        if self.wide:
            return self.plan.decode_cyclic_wide(self.R, self.Rlo, self.f, self.u, stream)
        if hostphi:
            return self.plan.decode_cyclic_hostphi(self.R, self.f, self.u, stream)
        return self.plan.decode_cyclic(self.R, self.f, self.u, stream)

    def step(self):
        """One pass of the whole hot path: encode all nodes, decode what was received."""
        self.encode()
        if self.w.decode:
            return self.decode()
        return None

    def expected_mask(self):
        import numpy as np
        m = np.zeros(self.w.P, dtype=bool)
        for j, _ in self.adversaries:
            m[j] = True
        return m

    def close(self) -> None:
        self.plan.close()
