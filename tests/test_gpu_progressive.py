"""The paper's progressive schedules through the library: stage switches reuse one set of buffers
(Sec. 5.2 Table 7, Sec. 5.3 Table 9), every stage matches the oracle, and both variants of the
loss (per-patch normalised and plain pixels) match."""
import numpy as np
import pytest
import torch

import oracle
import paper_2404_00509_amd as mae
from paper_2404_00509_amd import synth

from helpers import (ATOL, RTOL, check_grad, check_prep_against_oracle, gpu_loss, prep_to_numpy,
                     to_device)

pytestmark = pytest.mark.gpu

B = 24
PATCH = 16


def _run_stage(dimg, data, bufs, stage_index, out_size, K, seed, batch_index, scale=(0.2, 1.0),
               aug_mode=0, jitter=0.3):
    buf = bufs.stage(stage_index)
    desc = mae.make_prep_desc(*dimg, out_size=out_size, patch=PATCH, num_keep=K, scale=scale,
                              seed=seed, batch_index=batch_index, aug_mode=aug_mode, jitter=jitter)
    assert mae.mae_prep_workspace_bytes(desc) <= buf.workspace.numel()
    for t in (buf.visible, buf.target):
        t.fill_(float("nan"))
    buf.mask.fill_(0xEE)
    buf.ids_restore.fill_(-7)
    mae.mae_prep_batch(desc, buf.visible, buf.mask, buf.ids_restore, buf.ids_keep, buf.target,
                       buf.crop, buf.workspace)
    torch.cuda.synchronize()
    assert mae.mae_prep_status(buf.workspace) == 0
    ref = oracle.prep_batch(*data, out_size=out_size, patch=PATCH, num_keep=K, scale=scale,
                            seed=seed, batch_index=batch_index, aug_mode=aug_mode, jitter=jitter)
    check_prep_against_oracle(prep_to_numpy(buf), ref, what=f"stage{stage_index}")
    return buf, ref


@pytest.mark.parametrize("scheme", [1, 3, 4, 5, 6])
def test_pretrain_schemes_switch_stages_without_reallocation(scheme):
    data = synth.make_images("gradient", B, seed=scheme)
    dimg = to_device(*data)
    stages = [mae.mae_pretrain_stage(scheme, s) for s in (1, 2, 3)]
    assert stages == [oracle.pretrain_stage(scheme, s) for s in (1, 2, 3)]
    bufs = mae.ProgressiveBuffers(B, PATCH, stages)
    max_ld = max(sh[1] * sh[3] for sh in bufs.shapes)
    pred_store = torch.empty(B * max_ld, device="cuda")
    grad_store = torch.empty(B * max_ld, device="cuda")
    torch.cuda.synchronize()
    allocated = torch.cuda.memory_allocated()
    pointers = None
    for i, (res, m) in enumerate(stages):
        L = (res // PATCH) ** 2
        K = mae.mae_num_keep(L, m)
        assert K == oracle.num_keep(L, m) == bufs.shapes[i][2]
        buf, ref = _run_stage(dimg, data, bufs, i, res, K, seed=3, batch_index=10 * scheme + i)
        here = (buf.visible.data_ptr(), buf.target.data_ptr(), buf.mask.data_ptr(),
                buf.ids_restore.data_ptr(), buf.workspace.data_ptr())
        assert pointers is None or here == pointers      # same storage in every stage
        pointers = here

        # both loss variants on this stage's shapes, predictions in reused storage
        D = 3 * PATCH * PATCH
        pred_host = synth.make_pred(scheme, B, L, D)
        pred = pred_store[:B * L * D].view(B, L, D)
        pred.copy_(torch.from_numpy(pred_host))
        M = B * (L - K)
        for norm_pix in (True, False):
            desc = mae.make_loss_desc(pred, buf.target, buf.mask, num_masked=M, norm_pix=norm_pix)
            ws = bufs._workspace  # large enough? checked below
            need = mae.mae_loss_workspace_bytes(desc)
            lws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
            loss = torch.zeros(1, device="cuda")
            grad = grad_store[:B * L * D].view(B, L, D)
            mae.mae_normpix_loss(desc, loss, grad, lws)
            torch.cuda.synchronize()
            if norm_pix:
                ref_loss, ref_grad, _ = oracle.normpix_loss(pred_host, ref["target"], ref["mask"],
                                                            num_masked=M)
            else:
                ref_loss, ref_grad = oracle.pixel_loss(pred_host, ref["target"], ref["mask"],
                                                       num_masked=M)
            assert abs(loss.item() - ref_loss) <= ATOL + RTOL * abs(ref_loss), (norm_pix, i)
            check_grad(grad.cpu().numpy(), ref_grad, D, M, what=f"s{scheme} stage{i}")
            del lws
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() <= allocated + 4096   # only the 1-element loss tensors


@pytest.mark.parametrize("scheme", [mae.MAE_FINETUNE_SCHEME_1, mae.MAE_FINETUNE_SCHEME_3,
                                    mae.MAE_FINETUNE_SCHEME_1_MINUS,
                                    mae.MAE_FINETUNE_SCHEME_1_PLUS])
def test_finetune_schemes_run_with_their_own_scale_range_and_augmentation(scheme):
    """Table 7 through its stage switches: each stage runs at its resolution, with its crop range
    and with the augmentation of its aug column, every patch kept, on buffers allocated once."""
    data = synth.make_images("gradient", B, seed=7)
    dimg = to_device(*data)
    plan = [mae.mae_finetune_stage(scheme, s) for s in (1, 2, 3)]
    for s, (res, lo, hi, aug) in enumerate(plan, start=1):
        ores, sl, sh, oaug = oracle.finetune_stage(scheme, s)
        assert res == ores and lo == np.float32(sl * sl) and hi == np.float32(sh * sh)
        assert aug == oaug
    if scheme == mae.MAE_FINETUNE_SCHEME_1_MINUS:
        assert [a for _, _, _, a in plan] == [mae.MAE_AUG_THREE] * 3
    if scheme == mae.MAE_FINETUNE_SCHEME_1_PLUS:
        assert [a for _, _, _, a in plan] == [mae.MAE_AUG_THREE_PLUS] * 3
    bufs = mae.ProgressiveBuffers(B, PATCH, [(res, 0.0) for res, _, _, _ in plan],
                                  aug_mode=mae.MAE_AUG_THREE_PLUS)
    lengths = [30, 30, 40]
    for epoch in (0, 29, 30, 59, 60, 99):
        stage = mae.mae_stage_of_epoch(epoch, lengths)
        assert stage == oracle.stage_of_epoch(epoch, lengths)
        res, lo, hi, aug = plan[stage - 1]
        L = (res // PATCH) ** 2
        _run_stage(dimg, data, bufs, stage - 1, res, L, seed=5, batch_index=epoch, scale=(lo, hi),
                   aug_mode=aug, jitter=0.3)


@pytest.mark.parametrize("bf16", [False, True])
def test_pixel_loss_variant_shapes(bf16):
    rng = np.random.default_rng(2)
    for (Bn, L, D) in ((2, 9, 768), (3, 7, 588), (1, 5, 147), (2, 3, 3072)):
        target = (rng.standard_normal((Bn, L, D)) * 1.5 + 0.3).astype(np.float32)
        pred = rng.standard_normal((Bn, L, D)).astype(np.float32)
        if bf16:
            pred = torch.from_numpy(pred).to(torch.bfloat16).float().numpy()
        mask = (rng.random((Bn, L)) < 0.7).astype(np.uint8)
        mask[0, 0] = 1
        M = int(mask.sum())
        ref_loss, ref_grad = oracle.pixel_loss(pred, target, mask, num_masked=M, grad_scale=2.0)
        tp = torch.from_numpy(pred).cuda()
        if bf16:
            tp = tp.to(torch.bfloat16)
        desc = mae.make_loss_desc(tp, torch.from_numpy(target).cuda(),
                                  torch.from_numpy(mask).cuda(), num_masked=M, grad_scale=2.0,
                                  norm_pix=False)
        keep = (torch.from_numpy(target).cuda(), torch.from_numpy(mask).cuda())
        desc.target, desc.mask = keep[0].data_ptr(), keep[1].data_ptr()
        ws = torch.empty(max(mae.mae_loss_workspace_bytes(desc), 256), dtype=torch.uint8,
                         device="cuda")
        loss = torch.zeros(1, device="cuda")
        grad = torch.full_like(tp, float("nan"))
        mae.mae_normpix_loss(desc, loss, grad, ws)
        torch.cuda.synchronize()
        assert abs(loss.item() - ref_loss) <= ATOL + RTOL * abs(ref_loss)
        check_grad(grad.float().cpu().numpy(), ref_grad, D, M, grad_scale=2.0, bf16=bf16,
                   what=f"pixel D{D}")
