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


def test_bf16_parameters_first_step_cannot_be_captured_then_replays_match_eager():
    """BF16 parameters keep an FP32 master copy that the first br_step initialises from the parameter.  Baked into
    a graph, that copy would reset the master at every replay, so br_step refuses to capture it (BR_ERR_STATE);
    after one eager step the captured step replays bit for bit like eager steps, the master keeping what it has
    accumulated below one BF16 ulp."""
    from paper_2602_03515_amd import binding as B
    from paper_2602_03515_amd.optimizer import BasisRotationAdam

    shape, steps = (200, 136), 4
    rng = np.random.default_rng(6)
    W0 = torch.from_numpy(rng.standard_normal(shape).astype(np.float32)).to(torch.bfloat16)
    G = [torch.from_numpy((rng.standard_normal(shape) * 0.1).astype(np.float32)).to(torch.bfloat16) for _ in range(steps)]
    dev = torch.device("cuda:0")
    side = torch.cuda.Stream(device=dev)

    def make():
        p = [W0.to(dev).clone()]
        g = [torch.zeros(shape, dtype=torch.bfloat16, device=dev)]
        with torch.cuda.stream(side):
            opt = BasisRotationAdam(p, freq=0, lr=1e-4, grad_dtype=torch.bfloat16)
        return p, g, opt

    pe, ge, oe = make()
    for t in range(steps):
        with torch.cuda.stream(side):
            ge[0].copy_(G[t].to(dev))
            oe.accumulate_stats(ge)
            oe.apply(ge)
    side.synchronize()

    pg, gg, og = make()
    with torch.cuda.stream(side):
        gg[0].copy_(G[0].to(dev))
    side.synchronize()
    refused = torch.cuda.CUDAGraph()
    with torch.cuda.graph(refused, stream=side):
        og.accumulate_stats(gg)
        with pytest.raises(B.BrError) as e:
            og.apply(gg)
    assert e.value.status == B.BR_ERR_STATE and "eagerly" in str(e.value)
    del refused                      # never replayed: it holds step 1's statistics update only
    pg, gg, og = make()              # a fresh context: the refused capture advanced the host-side state of the old one
    with torch.cuda.stream(side):
        gg[0].copy_(G[0].to(dev))
        og.accumulate_stats(gg)
        og.apply(gg)
    side.synchronize()
    plain = torch.cuda.CUDAGraph()
    with torch.cuda.graph(plain, stream=side):
        og.accumulate_stats(gg)
        og.apply(gg)
    for t in range(1, steps):
        with torch.cuda.stream(side):
            gg[0].copy_(G[t].to(dev))
        side.synchronize()
        plain.replay()
        torch.cuda.synchronize()
    assert torch.equal(pe[0], pg[0])
    assert torch.equal(oe.state(0, B.BR_STATE_MASTER), og.state(0, B.BR_STATE_MASTER))
    # lr = 1e-4: single updates are below half a BF16 ulp of O(1) weights; only the master copy keeps them
    assert not torch.equal(oe.state(0, B.BR_STATE_MASTER).to(torch.bfloat16).float(), oe.state(0, B.BR_STATE_MASTER))
    oe.close()
    og.close()
