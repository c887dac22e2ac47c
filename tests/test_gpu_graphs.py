"""The stream-ordered entry points (encoders and the *_async decoders) enqueue kernels
only -- no allocation, no host wait, no memset node -- so a whole encode + decode step can
be captured into a HIP graph.  Each replay is checked against the eager result, with the
received slab edited and unrelated eager work run between replays."""
import numpy as np
import pytest
import torch

from paper_1803_09877_amd import binding as B
from paper_1803_09877_amd import synth
from paper_1803_09877_amd.runner import Case

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("code,P,s,d,attacks,placement,sigma,wide", [
    ("rep", 45, 2, 300_001, ("signflip", "signflip"), "distinct_groups", 1e-2, False),
    ("cyc", 45, 3, 300_002, ("noise", "signflip", "noise"), "adjacent_pair", 1e-2, False),
    ("cyc", 15, 2, 100_001, ("offset", "offset"), "any", 1.0, False),
    ("cyc", 45, 3, 300_002, ("noise", "signflip", "noise"), "adjacent_pair", 1e-2, "i8"),     # the benchmark's wire
    ("cyc", 33, 2, 100_003, ("signflip", "offset"), "any", 1e-2, "bf16"),
    ("cyc", 15, 2, 100_001, ("offset", "offset"), "any", 1.0, "f32"),
])
def test_graph_replays_match_eager(code, P, s, d, attacks, placement, sigma, wide):
    w = synth.Workload(name=f"graph_{code}", code=code, P=P, s=s, d=d, sigma=sigma, attacks=attacks,
                       placement=placement, seed=synth.SEED_BASE + 404)
    c = Case(w, wide=wide)
    try:
        mask_dev = torch.zeros(4, dtype=torch.int64, device=c.device)
        status_dev = torch.full((1,), -1, dtype=torch.int32, device=c.device)

        def step():
            c.encode()
            if code == "rep":
                c.plan.decode_repetition_async(c.R, c.u, mask_dev, status_dev)
            elif wide:
                c.plan.decode_cyclic_wide_async(c.R, c.Rlo, c.f, c.u, mask_dev, status_dev)
            else:
                c.plan.decode_cyclic_async(c.R, c.f, c.u, mask_dev, status_dev)

        c.encode()
        c.receive()
        step()                                   # warm-up outside capture (one-time kernel attributes)
        torch.cuda.synchronize()

        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                step()
        torch.cuda.synchronize()

        scratch = torch.zeros(1 << 20, device=c.device)
        for it in range(4):
            # new received slab: move the adversaries (honest rows restored from Z)
            c.R.copy_(c.Z)
            if wide:
                c.Rlo.copy_(c.Zlo)
            shift = [((j + 3 * it) % P, a) for j, a in c.adversaries]
            if code == "rep":                     # keep them in distinct groups
                shift = [(((j // w.r + it) % (P // w.r)) * w.r + j % w.r, a) for j, a in c.adversaries]
            synth.apply_attacks(c.R, c.mlen, shift, w.seed + it)
            expect = np.zeros(P, dtype=bool)
            expect[[j for j, _ in shift]] = True
            # eager reference
            c.u.zero_()
            step()
            torch.cuda.synchronize()
            u_ref, m_ref, st_ref = c.u.clone(), mask_dev.clone(), int(status_dev.item())
            assert st_ref == 0 and np.array_equal(B.mask_to_bool(m_ref.cpu().numpy().view(np.uint64), P), expect)
            # unrelated eager work and clobbered outputs, then the replay
            scratch.normal_()
            c.u.fill_(float("nan"))
            mask_dev.fill_(-1)
            status_dev.fill_(-1)
            c.Z.fill_(float("nan"))
            graph.replay()
            torch.cuda.synchronize()
            assert int(status_dev.item()) == 0
            words = (P + 63) // 64                                # only ceil(P/64) mask words are written
            assert torch.equal(mask_dev[:words], m_ref[:words])
            assert torch.equal(c.u[:d], u_ref[:d])
            assert torch.isfinite(c.Z[:, :c.mlen]).all()          # the captured encoder ran too
    finally:
        c.close()
