"""The loss entry point that uses the library's own fixed scratch array instead of a workspace
(for callers that cannot allocate): same results as mae_normpix_loss, bit for bit, on two calls
in a row, the second on a smaller input."""
import numpy as np
import pytest
import torch

import oracle
import paper_2404_00509_amd as mae
from paper_2404_00509_amd import synth
from helpers import ATOL, RTOL, check_grad

pytestmark = pytest.mark.gpu


def _inputs(seed, B, L, D, bf16):
    rng = np.random.default_rng([seed, B, L, D])
    pred = synth.make_pred(seed, B, L, D)
    target = rng.normal(0.0, 1.0, size=(B, L, D)).astype(np.float32)
    mask = (rng.random((B, L)) < 0.75).astype(np.uint8)
    mask[0, 0] = 1
    tp = torch.from_numpy(pred).cuda()
    if bf16:
        tp = tp.to(torch.bfloat16)
    return tp, torch.from_numpy(target).cuda(), torch.from_numpy(mask).cuda(), target, mask


@pytest.mark.parametrize("bf16", [False, True])
def test_static_scratch_matches_workspace_call(bf16):
    # a large grid first (every partial slot of the kernel's launch written), then a small one
    for seed, (B, L, D) in enumerate([(96, 196, 768), (3, 49, 588)]):
        pred, target, mask, target_host, mask_host = _inputs(seed, B, L, D, bf16)
        M = int(mask_host.sum())
        desc = mae.make_loss_desc(pred, target, mask, num_masked=M)
        ws = torch.empty(max(mae.mae_loss_workspace_bytes(desc), 256), dtype=torch.uint8,
                         device="cuda")
        loss_a = torch.full((1,), float("nan"), device="cuda")
        grad_a = torch.full_like(pred, float("nan"))
        mae.mae_normpix_loss(desc, loss_a, grad_a, ws)
        loss_b = torch.full((1,), float("nan"), device="cuda")
        grad_b = torch.full_like(pred, float("nan"))
        mae.mae_normpix_loss_static(desc, loss_b, grad_b)
        torch.cuda.synchronize()
        assert torch.equal(loss_a, loss_b), (B, L, D)
        assert torch.equal(grad_a.view(torch.int16 if bf16 else torch.int32),
                           grad_b.view(torch.int16 if bf16 else torch.int32)), (B, L, D)
        # ... and both against the oracle
        ref_loss, ref_grad, _ = oracle.normpix_loss(pred.float().cpu().numpy(), target_host,
                                                    mask_host, num_masked=M)
        assert abs(loss_b.item() - ref_loss) <= ATOL + RTOL * abs(ref_loss)
        check_grad(grad_b.float().cpu().numpy(), ref_grad, D, M, bf16=bf16, what="static")


def test_static_scratch_loss_only_and_argument_errors():
    pred, target, mask, _, mask_host = _inputs(7, 4, 64, 192, False)
    M = int(mask_host.sum())
    desc = mae.make_loss_desc(pred, target, mask, num_masked=M)
    ws = torch.empty(max(mae.mae_loss_workspace_bytes(desc), 256), dtype=torch.uint8, device="cuda")
    a = torch.zeros(1, device="cuda")
    b = torch.zeros(1, device="cuda")
    mae.mae_normpix_loss(desc, a, None, ws)
    mae.mae_normpix_loss_static(desc, b, None)
    torch.cuda.synchronize()
    assert torch.equal(a, b)
    # straight through the C ABI (the binding would refuse the missing tensor itself)
    import ctypes
    assert mae.load().mae_normpix_loss_static(ctypes.byref(desc), None, None,
                                              None) == mae.binding.MAE_ERR_NULL
    desc.num_masked = -1
    with pytest.raises(mae.MaeError) as e:
        mae.mae_normpix_loss_static(desc, b, None)
    assert e.value.status == mae.binding.MAE_ERR_RANGE


def test_static_scratch_in_a_captured_graph():
    # what the entry point is for: a caller under graph capture.  The first call on a device
    # looks up the array's address, so one call is made before the capture starts.
    pred, target, mask, _, mask_host = _inputs(11, 24, 100, 768, False)
    desc = mae.make_loss_desc(pred, target, mask, num_masked=0)  # divisor counted on the device
    ws = torch.empty(max(mae.mae_loss_workspace_bytes(desc), 256), dtype=torch.uint8, device="cuda")
    loss_ref = torch.zeros(1, device="cuda")
    grad_ref = torch.empty_like(pred)
    mae.mae_normpix_loss(desc, loss_ref, grad_ref, ws)
    loss = torch.zeros(1, device="cuda")
    grad = torch.empty_like(pred)
    mae.mae_normpix_loss_static(desc, loss, grad)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        mae.mae_normpix_loss_static(desc, loss, grad, stream=torch.cuda.current_stream())
    for replay in range(3):
        loss.fill_(float("nan"))
        grad.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(loss, loss_ref), replay
        assert torch.equal(grad.view(torch.int32), grad_ref.view(torch.int32)), replay
        grad_ref.mul_(1.0)  # eager work between replays
        torch.cuda.synchronize()
