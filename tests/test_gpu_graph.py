"""The optimizer calls enqueue kernels only (no allocation, no synchronisation, no memset), so a
step can be captured into a HIP graph and replayed; this checks replays against eager execution."""
import numpy as np
import pytest
import torch

from paper_2602_03515_amd import synth

pytestmark = pytest.mark.gpu


def _states(opt, B, n):
    out = []
    for i in range(n):
        for kind in (B.BR_STATE_M, B.BR_STATE_S, B.BR_STATE_L, B.BR_STATE_R, B.BR_STATE_QL, B.BR_STATE_QR):
            if opt.has_state(i, kind):
                out.append(opt.state(i, kind).clone())
    return out


@pytest.mark.parametrize("math", [0, 1, 2])
def test_captured_steps_replay_like_eager_ones(math):
    """Steps 2..5 of one context are replays of two graphs captured once each (accumulate + step;
    for step 4 accumulate + refresh + step, whose step also rebuilds the cached rotated moment as the
    eager one does after a refresh); another context runs the same five steps eagerly.  Between
    replays the process does eager GPU work and synchronises.  The kernels are deterministic, so parameters and state must agree bit for bit.  What a captured call freezes:
    the gradient and parameter pointers and the learning rate (kernel arguments); bias correction is
    off (Algorithm 1), so no argument depends on the step number."""
    from paper_2602_03515_amd import binding as B
    from paper_2602_03515_amd.optimizer import BasisRotationAdam

    shapes = [(200, 136), (1700, 40), (64, 64)]  # 1700 rows: the QR's panels span two workgroups that exchange partial sums
    steps = 5
    rng = np.random.default_rng(5)
    W0 = [rng.standard_normal(s).astype(np.float32) for s in shapes]
    G = [[rng.standard_normal(s).astype(np.float32) * 0.1 for s in shapes] for _ in range(steps)]
    dev = torch.device("cuda:0")
    side = torch.cuda.Stream(device=dev)

    def make():
        params = [torch.from_numpy(w).to(dev) for w in W0]
        grads = [torch.zeros(s, dtype=torch.float32, device=dev) for s in shapes]
        with torch.cuda.stream(side):
            opt = BasisRotationAdam(params, freq=0, lr=1e-2, math=math)
        return params, grads, opt

    def load(grads, t):
        with torch.cuda.stream(side):
            for g, src in zip(grads, G[t]):
                g.copy_(torch.from_numpy(src).to(dev))

    # eager run: refresh before the step at t = 4 (index 3)
    pe, ge, oe = make()
    for t in range(steps):
        load(ge, t)
        with torch.cuda.stream(side):
            oe.accumulate_stats(ge)
            if t == 3:
                oe.refresh_basis()
            oe.apply(ge)
    side.synchronize()

    # captured run: step 1 eager (it builds the cached rotated moment), then graphs
    pg, gg, og = make()
    load(gg, 0)
    with torch.cuda.stream(side):
        og.accumulate_stats(gg)
        og.apply(gg)
    side.synchronize()
    plain, with_refresh = torch.cuda.CUDAGraph(), torch.cuda.CUDAGraph()
    with torch.cuda.graph(plain, stream=side):
        og.accumulate_stats(gg)
        og.apply(gg)
    with torch.cuda.graph(with_refresh, stream=side):
        og.accumulate_stats(gg)
        og.refresh_basis()
        og.apply(gg)
    for t in range(1, steps):
        load(gg, t)
        side.synchronize()
        (with_refresh if t == 3 else plain).replay()
        torch.cuda.synchronize()
        _ = (torch.ones(1 << 16, device=dev) * 2).sum().item()  # the program's own eager work between replays
    torch.cuda.synchronize()
    for a, b in zip(pe, pg):
        assert torch.equal(a, b)
    for a, b in zip(_states(oe, B, len(shapes)), _states(og, B, len(shapes))):
        assert torch.equal(a, b)
    oe.close()
    og.close()
