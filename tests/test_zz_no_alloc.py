"""br_clip_gradients_static (the entry point that allocates nothing) against br_clip_gradients, through
the C ABI: same kernels, the partial sums in the library's own device array instead of the workspace.
Two calls in a row, the second with a smaller input, so that what the first call left in the shared
array cannot leak into the second result."""
import numpy as np
import pytest
import torch

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(300)]


def _case(B, shapes, bf16, scale, seed, max_norm):
    from paper_2602_03515_amd.optimizer import BasisRotationAdam
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    dt = torch.bfloat16 if bf16 else torch.float32
    grads = [(scale * torch.randn(m, n, generator=gen, device=dev)).to(dt).contiguous() for m, n in shapes]
    # existing entry point: context + workspace
    ref = [g.clone() for g in grads]
    params = [torch.zeros(m, n, device=dev, dtype=dt) for m, n in shapes]
    opt = BasisRotationAdam(params, freq=0, lr=1e-3, grad_dtype=dt)
    opt.clip_gradients(ref, max_norm)
    torch.cuda.synchronize()
    ref_result = opt.clip_result().clone()
    opt.close()
    # the entry point under test: descriptors, pointers, caller-owned result; no context, no workspace
    got = [g.clone() for g in grads]
    result = torch.full((2,), -1.0, device=dev)
    descs = B.make_descs([(m, n) for m, n in shapes], param_dtype=B.BR_BF16 if bf16 else B.BR_F32,
                         grad_dtype=B.BR_BF16 if bf16 else B.BR_F32)
    B.br_clip_gradients_static(descs, [g.data_ptr() for g in got], max_norm, result.data_ptr(),
                               torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    # float64 definition on the host, for the norm itself
    norm64 = float(np.sqrt(sum(float((g.double() ** 2).sum()) for g in grads)))
    assert abs(float(result[0]) - norm64) <= 1e-5 * norm64
    # against the existing entry point: the norm is a float sum in a fixed order on both sides (same
    # per-workgroup partials; the launches are grouped alike for these inputs), so a few ulps at most
    assert abs(float(result[0]) - float(ref_result[0])) <= 4 * 2.0 ** -24 * float(ref_result[0])
    assert abs(float(result[1]) - float(ref_result[1])) <= 4 * 2.0 ** -24 * float(ref_result[1])
    clipped = float(ref_result[1]) < 1.0
    for a, b, g in zip(got, ref, grads):
        if not clipped:
            assert torch.equal(a, g) and torch.equal(b, g)
            continue
        # one ulp of the gradient's type where the two factors differ in their last bit
        ulp = 2.0 ** -7 if bf16 else 2.0 ** -22
        diff = (a.double() - b.double()).abs().max()
        assert float(diff) <= ulp * float(b.double().abs().max())
    return clipped


def test_static_clip_matches_workspace_clip_two_calls_in_a_row():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2602_03515_amd import binding as B
    # first call: 70 matrices (two launches of one run plus ragged shapes), clipped
    big = [(96, 130)] * 66 + [(257, 33), (64, 64), (1, 7), (300, 5)]
    assert _case(B, big, bf16=False, scale=0.5, seed=11, max_norm=1.0)
    # second call: a smaller input, not clipped (factor 1: gradients untouched)
    assert not _case(B, [(64, 48), (31, 17)], bf16=False, scale=1e-3, seed=12, max_norm=1.0)
    # third: BF16 gradients, fewer matrices again, clipped
    assert _case(B, [(128, 64), (33, 9), (16, 16)], bf16=True, scale=0.3, seed=13, max_norm=0.5)


def test_static_clip_rejects_bad_arguments_without_launching():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2602_03515_amd import binding as B
    dev = torch.device("cuda:0")
    g = torch.ones(8, 8, device=dev)
    result = torch.zeros(2, device=dev)
    too_many = B.make_descs([(8, 8)] * (B.BR_STATIC_CLIP_MAX_MATS + 1))
    with pytest.raises(B.BrError) as ei:
        B.br_clip_gradients_static(too_many, [g.data_ptr()] * (B.BR_STATIC_CLIP_MAX_MATS + 1), 1.0, result.data_ptr())
    assert ei.value.status == B.BR_ERR_WORKSPACE and "at most" in str(ei.value)
    one = B.make_descs([(8, 8)])
    with pytest.raises(B.BrError) as ei:
        B.br_clip_gradients_static(one, [g.data_ptr()], -1.0, result.data_ptr())
    assert ei.value.status == B.BR_ERR_INVALID_ARG
    with pytest.raises(B.BrError) as ei:
        B.br_clip_gradients_static(one, [g.data_ptr()], 1.0, 0)
    assert ei.value.status == B.BR_ERR_INVALID_ARG
    torch.cuda.synchronize()
    assert torch.equal(g, torch.ones(8, 8, device=dev)) and torch.equal(result, torch.zeros(2, device=dev))
