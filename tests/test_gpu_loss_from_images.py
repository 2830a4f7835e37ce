"""The loss without a stored target (mae_normpix_loss_from_images) against the oracle's chain
(prep, then loss on its target): same tolerances as the two-call path.  mae_prep_batch runs with
target = NULL here, so it also checks that the visible tokens do not depend on the target."""
import numpy as np
import pytest
import torch

import oracle
import paper_2404_00509_amd as mae
from paper_2404_00509_amd import synth

from helpers import (ATOL, RTOL, assert_close_device, check_grad, check_prep_against_oracle,
                     prep_to_numpy, to_device)

pytestmark = pytest.mark.gpu


def _run(dimg, kw, pred, *, file_sizes=None, bf16=False, norm_pix=True, grad_scale=1.0,
         want_grad=True, max_image_side=0, eps=1e-6):
    if file_sizes is None:
        desc = mae.make_prep_desc(*dimg, max_image_side=max_image_side, **kw)
    else:
        desc = mae.make_prep_desc(dimg[0], dimg[1], None, None, file_sizes=file_sizes,
                                  max_image_side=max_image_side, **kw)
    buf = mae.alloc_prep_buffers(desc, want_target=False)
    buf.visible.fill_(float("nan"))
    mae.mae_prep_batch(desc, buf.visible, buf.mask, buf.ids_restore, buf.ids_keep, None, buf.crop,
                       buf.workspace)
    B, L = buf.mask.shape
    M = B * (L - kw["num_keep"])
    ldesc = mae.make_loss_desc(pred, None, buf.mask, num_masked=M, norm_pix=norm_pix,
                               grad_scale=grad_scale, eps=eps)
    ws = torch.empty(max(mae.mae_loss_from_images_workspace_bytes(desc, ldesc), 256),
                     dtype=torch.uint8, device="cuda")
    loss = torch.full((1,), float("nan"), device="cuda")
    grad = torch.full_like(pred, float("nan")) if want_grad else None
    mae.mae_normpix_loss_from_images(desc, buf.workspace, ldesc, loss, grad, ws)
    torch.cuda.synchronize()
    return buf, float(loss.item()), grad, M


def _check(data, kw, pred_host, *, bf16=False, what="", **opt):
    ref = oracle.prep_batch(*data, **kw)
    dimg = to_device(*data)
    pred = torch.from_numpy(pred_host).cuda()
    if bf16:
        pred = pred.to(torch.bfloat16)
        pred_host = pred.float().cpu().numpy()
    buf, loss, grad, M = _run(dimg, kw, pred, **opt)
    norm = opt.get("norm_pix", True)
    scale = opt.get("grad_scale", 1.0)
    if norm:
        ref_loss, ref_grad, _ = oracle.normpix_loss(pred_host, ref["target"], ref["mask"],
                                                    num_masked=M, grad_scale=scale,
                                                    eps=opt.get("eps", 1e-6))
    else:
        ref_loss, ref_grad = oracle.pixel_loss(pred_host, ref["target"], ref["mask"],
                                               num_masked=M, grad_scale=scale)
    got = prep_to_numpy(buf)
    ref_no_target = dict(ref, target=None)
    check_prep_against_oracle(got, ref_no_target, bf16=False, what=what)
    assert abs(loss - ref_loss) <= ATOL + RTOL * abs(ref_loss), (what, loss, ref_loss)
    g = grad.float().cpu().numpy()
    check_grad(g, ref_grad, pred.shape[-1], M, grad_scale=scale, bf16=bf16, what=what)
    vis = ref["mask"] == 0
    assert np.all(g[vis] == 0.0)
    return buf, loss


@pytest.mark.parametrize("name", ["c1", "c2"])
def test_small_configs(name):
    wl = synth.WORKLOADS[name]
    data = synth.make_images(wl.kind, wl.B, seed=0)
    kw = dict(out_size=wl.out_size, patch=wl.patch, num_keep=oracle.num_keep(wl.L, wl.mask_ratio),
              seed=2, batch_index=1)
    _check(data, kw, synth.make_pred(1, wl.B, wl.L, wl.D), what=name)


@pytest.mark.parametrize("S,p,ratio,bf16", [(224, 14, 0.75, True), (224, 14, 0.75, False),
                                            (192, 16, 0.8, True), (64, 32, 0.5, False),
                                            (96, 8, 0.66, False), (256, 16, 0.85, False),
                                            (48, 4, 0.75, False), (96, 12, 0.75, False),
                                            (80, 20, 0.75, True), (96, 24, 0.5, False)])
def test_patch_sizes_ratios_and_bf16(S, p, ratio, bf16):
    B = 12
    data = synth.make_images("gradient", B, seed=3)
    L, D = (S // p) ** 2, 3 * p * p
    kw = dict(out_size=S, patch=p, num_keep=oracle.num_keep(L, ratio), seed=4, batch_index=2)
    _check(data, kw, synth.make_pred(2, B, L, D), bf16=bf16, what=f"S{S} p{p}")


def test_unnormalised_variant_scale_and_loss_only():
    B, S, p = 8, 112, 16
    data = synth.make_images("uniform", B, seed=5)
    L, D = (S // p) ** 2, 3 * p * p
    kw = dict(out_size=S, patch=p, num_keep=oracle.num_keep(L, 0.75), seed=6, batch_index=3)
    pred = synth.make_pred(3, B, L, D)
    _check(data, kw, pred, norm_pix=False, what="un-normalised")
    _check(data, kw, pred, grad_scale=-2.5, eps=1e-3, what="scale and eps")
    # loss only
    ref = oracle.prep_batch(*data, **kw)
    M = B * (L - kw["num_keep"])
    ref_loss, _, _ = oracle.normpix_loss(pred, ref["target"], ref["mask"], num_masked=M)
    _, loss, grad, _ = _run(to_device(*data), kw, torch.from_numpy(pred).cuda(), want_grad=False)
    assert grad is None and abs(loss - ref_loss) <= ATOL + RTOL * abs(ref_loss)


def test_large_images_take_the_unstaged_path_and_flat_patches():
    # sources too large for the staging tile (taps straight from global memory), and flat images
    # (variance zero: the normalised target is 0 / sqrt(eps))
    rng = np.random.default_rng(7)
    imgs = [rng.integers(0, 256, size=(700, 900, 3), dtype=np.uint8),
            np.full((300, 200, 3), 77, np.uint8),
            rng.integers(0, 256, size=(40, 1200, 3), dtype=np.uint8)]
    sizes = np.array([im.size for im in imgs], np.int64)
    offsets = np.zeros(len(imgs), np.int64)
    offsets[1:] = np.cumsum(sizes)[:-1]
    data = (np.concatenate([im.reshape(-1) for im in imgs]), offsets,
            np.array([im.shape[0] for im in imgs], np.int32),
            np.array([im.shape[1] for im in imgs], np.int32))
    S, p = 96, 16
    L, D = (S // p) ** 2, 3 * p * p
    kw = dict(out_size=S, patch=p, num_keep=oracle.num_keep(L, 0.75), seed=8, batch_index=4)
    _check(data, kw, synth.make_pred(4, len(imgs), L, D), what="large and flat")


def test_jpeg_input_and_samples_flagged_invalid():
    B, S = 8, 112
    files, offsets, sizes = synth.make_jpegs("gradient", B, seed=9)
    imgs = [oracle.jpeg_decode(files[o:o + n].tobytes()) for o, n in zip(offsets, sizes)]
    lens = np.array([i.size for i in imgs], np.int64)
    offs = np.zeros(B, np.int64)
    offs[1:] = np.cumsum(lens)[:-1]
    data = (np.concatenate([i.reshape(-1) for i in imgs]), offs,
            np.array([i.shape[0] for i in imgs], np.int32),
            np.array([i.shape[1] for i in imgs], np.int32))
    L, D = (S // 16) ** 2, 768
    kw = dict(out_size=S, patch=16, num_keep=oracle.num_keep(L, 0.75), seed=10, batch_index=5)
    ref = oracle.prep_batch(*data, **kw)
    pred_host = synth.make_pred(5, B, L, D)
    M = B * (L - kw["num_keep"])
    ref_loss, ref_grad, _ = oracle.normpix_loss(pred_host, ref["target"], ref["mask"],
                                                num_masked=M)
    dev = [torch.from_numpy(a).cuda() for a in (files, offsets, sizes)]
    pred = torch.from_numpy(pred_host).cuda()
    buf, loss, grad, _ = _run((dev[0], dev[1]), kw, pred, file_sizes=dev[2])
    assert abs(loss - ref_loss) <= ATOL + RTOL * abs(ref_loss)
    check_grad(grad.cpu().numpy(), ref_grad, D, M, what="jpeg")
    # one file cut inside its tables: flagged, adds nothing to the loss, zero gradient
    bad = files.copy()
    bad[offsets[3] + 30:offsets[3] + 200] = 0
    dev[0] = torch.from_numpy(bad).cuda()
    buf, loss, grad, _ = _run((dev[0], dev[1]), kw, pred, file_sizes=dev[2])
    assert mae.mae_prep_status(buf.workspace) == 1
    assert not buf.mask[3].any()   # the flagged sample takes no part: nothing of it is masked
    without = ref["mask"].copy()
    without[3] = 0           # the sample's patches count as nothing; the divisor stays M
    want, _, _ = oracle.normpix_loss(pred_host, ref["target"], without, num_masked=M,
                                     want_grad=False)
    assert abs(loss - want) <= ATOL + RTOL * abs(want)
    assert bool((grad[3] == 0).all())
    keep = [b for b in range(B) if b != 3]
    check_grad(grad[keep].cpu().numpy(), ref_grad[keep], D, M, what="jpeg next to a bad file")


def test_agrees_with_the_two_call_path_at_full_size():
    """The bench's launch (c4): loss equal to that of mae_prep_batch + mae_normpix_loss to
    rounding, gradients equal element for element on sampled images."""
    wl = synth.WORKLOADS["c4"]
    data = synth.make_images(wl.kind, wl.B, seed=0)
    K = oracle.num_keep(wl.L, wl.mask_ratio)
    kw = dict(out_size=wl.out_size, patch=wl.patch, num_keep=K, seed=0, batch_index=9)
    dimg = to_device(*data)
    gen = torch.Generator(device="cuda").manual_seed(11)
    pred = torch.randn((wl.B, wl.L, wl.D), generator=gen, device="cuda")
    buf, loss, grad, M = _run(dimg, kw, pred)
    desc = mae.make_prep_desc(*dimg, **kw)
    full = mae.alloc_prep_buffers(desc)
    mae.mae_prep_batch(desc, full.visible, full.mask, full.ids_restore, full.ids_keep, full.target,
                       full.crop, full.workspace)
    assert torch.equal(full.visible, buf.visible) and torch.equal(full.mask, buf.mask)
    ldesc = mae.make_loss_desc(pred, full.target, full.mask, num_masked=M)
    ws = torch.empty(max(mae.mae_loss_workspace_bytes(ldesc), 256), dtype=torch.uint8,
                     device="cuda")
    loss2 = torch.zeros(1, device="cuda")
    grad2 = torch.empty_like(pred)
    mae.mae_normpix_loss(ldesc, loss2, grad2, ws)
    torch.cuda.synchronize()
    assert abs(loss - loss2.item()) <= 1e-6 * abs(loss2.item())
    unit = 2.0 / (wl.D * M)
    assert float((grad - grad2).abs().max().item()) / unit <= 2e-5
    # every image against the oracle's chain (its prep, then its loss on its own target)
    oracle_loss = 0.0
    for lo in range(0, wl.B, 256):
        hi = min(lo + 256, wl.B)
        ref = oracle.prep_batch(*data, b_begin=lo, b_end=hi, want_visible=False, **kw)
        part, ref_grad, _ = oracle.normpix_loss(pred[lo:hi].cpu().numpy(), ref["target"],
                                                ref["mask"], num_masked=M)
        oracle_loss += part
        assert_close_device(grad[lo:hi], ref_grad, scale=1.0 / unit, what=f"c4[{lo}:{hi}] grad")
    assert abs(loss - oracle_loss) <= ATOL + RTOL * abs(oracle_loss)


def test_on_a_side_stream_and_in_a_captured_graph():
    """Kernels only (no memset, no copy, no sync): the pair of calls can be captured; every replay
    is checked against the oracle, with eager work in between."""
    wl = synth.WORKLOADS["c1"]
    B = 24
    data = synth.make_images(wl.kind, B, seed=12)
    kw = dict(out_size=wl.out_size, patch=wl.patch, num_keep=oracle.num_keep(wl.L, 0.75), seed=13,
              batch_index=8)
    ref = oracle.prep_batch(*data, **kw)
    pred_host = synth.make_pred(6, B, wl.L, wl.D)
    M = B * (wl.L - kw["num_keep"])
    ref_loss, ref_grad, _ = oracle.normpix_loss(pred_host, ref["target"], ref["mask"],
                                                num_masked=M)
    dimg = to_device(*data)
    pred = torch.from_numpy(pred_host).cuda()
    desc = mae.make_prep_desc(*dimg, **kw)
    buf = mae.alloc_prep_buffers(desc, want_target=False)
    ldesc = mae.make_loss_desc(pred, None, buf.mask, num_masked=M)
    ws = torch.empty(max(mae.mae_loss_from_images_workspace_bytes(desc, ldesc), 256),
                     dtype=torch.uint8, device="cuda")
    loss = torch.zeros(1, device="cuda")
    grad = torch.empty_like(pred)

    def step(stream):
        mae.mae_prep_batch(desc, buf.visible, buf.mask, buf.ids_restore, buf.ids_keep, None,
                           buf.crop, buf.workspace, stream=stream)
        mae.mae_normpix_loss_from_images(desc, buf.workspace, ldesc, loss, grad, ws, stream=stream)

    def check(what):
        torch.cuda.synchronize()
        assert abs(loss.item() - ref_loss) <= ATOL + RTOL * abs(ref_loss), what
        check_grad(grad.cpu().numpy(), ref_grad, wl.D, M, what=what)

    def wipe():
        grad.fill_(float("nan"))
        loss.fill_(-1.0)
        buf.mask.fill_(0xEE)
        torch.cuda.synchronize()

    side = torch.cuda.Stream()
    wipe()
    with torch.cuda.stream(side):
        step(side)
    side.synchronize()
    check("side stream")
    graph = torch.cuda.CUDAGraph()
    wipe()
    with torch.cuda.graph(graph):
        step(torch.cuda.current_stream())
    for replay in range(3):
        wipe()
        graph.replay()
        check(f"graph replay {replay}")
        grad.mul_(1.0)
        torch.cuda.synchronize()
