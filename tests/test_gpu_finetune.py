"""Finetuning augmentation ("3 Aug", "3 Aug+") through mae_prep_batch against the oracle: crop
box, flip and masking order bit-exact, pixels within the fp32 tolerance of the path.  Every image
of a batch draws its own operation, so each batch covers grayscale, solarisation and blur."""
import numpy as np
import pytest
import torch

import oracle
import paper_2404_00509_amd as mae
from paper_2404_00509_amd import synth

from helpers import (ATOL, BF16_RTOL, RTOL, assert_close, assert_close_device,
                     check_prep_against_oracle, gpu_prep, prep_to_numpy)

pytestmark = pytest.mark.gpu


def _ops(seed, batch_index, n, base=0):
    return np.array([oracle.aug_params(seed, batch_index, base + b)[0] for b in range(n)])


@pytest.mark.parametrize("mode", [mae.MAE_AUG_THREE, mae.MAE_AUG_THREE_PLUS])
@pytest.mark.parametrize("scheme,stage", [(1, 1), (3, 2), (3, 3)])
def test_finetune_stages_match_the_oracle(mode, scheme, stage):
    """Table 7: resolutions 160 / 192 / 224 with the scheme's crop range, every patch kept."""
    S, lo, hi, _ = mae.mae_finetune_stage(scheme, stage)
    G = S // 16
    L = G * G
    B = 24
    data = synth.make_images("gradient", B, seed=40 + stage)
    kw = dict(out_size=S, patch=16, num_keep=L, scale=(lo, hi), seed=8, batch_index=stage,
              aug_mode=mode, jitter=0.3)
    ref = oracle.prep_batch(*data, **kw)
    buf, _, _ = gpu_prep(*data, **kw)
    assert mae.mae_prep_status(buf.workspace) == 0
    got = prep_to_numpy(buf)
    check_prep_against_oracle(got, ref, what=f"scheme {scheme} stage {stage} mode {mode}")
    ops = _ops(8, stage, B)
    assert set(ops) == {0, 1, 2}
    if mode == mae.MAE_AUG_THREE:
        # grayscale and solarised images are exact integers before the normalisation: the only
        # error left is the fp32 scale-and-shift
        exact = ops != oracle.OP_BLUR
        assert_close(got["target"][exact], ref["target"][exact], atol=2e-6, rtol=1e-6,
                     what="integer operations")


@pytest.mark.parametrize("mode", [mae.MAE_AUG_THREE, mae.MAE_AUG_THREE_PLUS])
def test_bf16_visible_and_masking_under_the_augmentation(mode):
    # the augmentation also composes with masking: a quarter of the patches kept, bf16 tokens
    S, B = 192, 20
    L = (S // 16) ** 2
    K = oracle.num_keep(L, 0.75)
    data = synth.make_images("gradient", B, seed=50)
    kw = dict(out_size=S, patch=16, num_keep=K, seed=9, batch_index=2, aug_mode=mode, jitter=0.3)
    ref = oracle.prep_batch(*data, **kw)
    buf, _, _ = gpu_prep(*data, bf16=True, **kw)
    check_prep_against_oracle(prep_to_numpy(buf), ref, bf16=True, what=f"bf16 mode {mode}")


def test_jitter_of_strength_zero_is_plain_three_aug():
    S, B = 160, 12
    L = (S // 16) ** 2
    data = synth.make_images("gradient", B, seed=51)
    kw = dict(out_size=S, patch=16, num_keep=L, seed=10, batch_index=0)
    a, _, _ = gpu_prep(*data, aug_mode=mae.MAE_AUG_THREE_PLUS, jitter=0.0, **kw)
    b, _, _ = gpu_prep(*data, aug_mode=mae.MAE_AUG_THREE, **kw)
    # factors are exactly 1: brightness and saturation steps are exact, the contrast step adds
    # (1 - 1) * mean = 0
    assert torch.equal(a.target, b.target) and torch.equal(a.visible, b.visible)
    # and the simple augmentation differs from both (the operation is really applied)
    c, _, _ = gpu_prep(*data, **kw)
    assert not torch.equal(a.target, c.target)
    for t in ("mask", "ids_restore", "ids_keep", "crop"):
        assert torch.equal(getattr(a, t), getattr(c, t)), t


def test_other_patch_sizes_and_resolutions():
    # p = 4 and p = 8 (rows of patches of 12 and 24 bytes), images smaller than the output, an odd
    # grid, and resolutions whose rows of patches the blur splits into two and three column parts
    for S, p, kind in ((32, 4, "uniform"), (64, 8, "uniform"), (112, 16, "uniform"),
                       (240, 16, "gradient"), (256, 16, "gradient"), (160, 32, "gradient")):
        L = (S // p) ** 2
        data = synth.make_images(kind, 16, seed=52)
        kw = dict(out_size=S, patch=p, num_keep=L, seed=11, batch_index=3,
                  aug_mode=mae.MAE_AUG_THREE_PLUS, jitter=0.3)
        ref = oracle.prep_batch(*data, **kw)
        buf, _, _ = gpu_prep(*data, **kw)
        check_prep_against_oracle(prep_to_numpy(buf), ref, what=f"S{S} p{p}")


@pytest.mark.parametrize("mode", [mae.MAE_AUG_THREE, mae.MAE_AUG_THREE_PLUS])
def test_patch_sizes_that_are_even_but_no_multiple_of_four(mode):
    # p = 14 (the other ViT patch size), 6, 10 and 2: a lane then takes two pixels instead of four
    # and the blur stages its bytes in 2-byte pieces
    for S, p, kind in ((224, 14, "gradient"), (196, 14, "gradient"), (60, 6, "uniform"),
                       (100, 10, "gradient"), (32, 2, "uniform")):
        L = (S // p) ** 2
        B = 9 if S > 100 else 16
        data = synth.make_images(kind, B, seed=54)
        kw = dict(out_size=S, patch=p, num_keep=L, seed=12, batch_index=1, aug_mode=mode,
                  jitter=0.3)
        ref = oracle.prep_batch(*data, **kw)
        assert set(_ops(12, 1, B)) == {0, 1, 2}
        buf, _, _ = gpu_prep(*data, **kw)
        assert mae.mae_prep_status(buf.workspace) == 0
        check_prep_against_oracle(prep_to_numpy(buf), ref, what=f"S{S} p{p} mode {mode}")
    # bf16 tokens and masking at p = 14
    S, p, B = 224, 14, 9
    L = (S // p) ** 2
    K = oracle.num_keep(L, 0.75)
    data = synth.make_images("gradient", B, seed=55)
    kw = dict(out_size=S, patch=p, num_keep=K, seed=13, batch_index=2, aug_mode=mode, jitter=0.3)
    ref = oracle.prep_batch(*data, **kw)
    buf, _, _ = gpu_prep(*data, bf16=True, **kw)
    check_prep_against_oracle(prep_to_numpy(buf), ref, bf16=True, what=f"p14 bf16 mode {mode}")


def test_shard_of_a_batch_and_reproducibility():
    S, B = 160, 16
    L = (S // 16) ** 2
    data = synth.make_images("gradient", B, seed=53)
    kw = dict(out_size=S, patch=16, num_keep=L, seed=12, batch_index=5,
              aug_mode=mae.MAE_AUG_THREE_PLUS, jitter=0.3)
    full, _, dimg = gpu_prep(*data, **kw)
    again, _, _ = gpu_prep(*data, device_inputs=dimg, **kw)
    assert torch.equal(full.target, again.target)
    # samples 8..15 as a call of their own: same draws through sample_base
    imgs, offs, hs, ws = data
    sub = (imgs[offs[8]:], (offs[8:] - offs[8]).copy(), hs[8:].copy(), ws[8:].copy())
    part, _, _ = gpu_prep(*sub, sample_base=8, **kw)
    assert torch.equal(part.target, full.target[8:])
    assert torch.equal(part.ids_restore, full.ids_restore[8:])


def test_three_aug_plus_on_a_side_stream_and_in_a_captured_graph():
    # the mode's four launches (two passes each of the resampling and the blur kernel) enqueue
    # kernels only, so the call can be captured; every replay is checked against the oracle
    S, B = 160, 12
    L = (S // 16) ** 2
    data = synth.make_images("gradient", B, seed=61)
    kw = dict(out_size=S, patch=16, num_keep=L, seed=10, batch_index=5,
              aug_mode=mae.MAE_AUG_THREE_PLUS, jitter=0.3)
    ref = oracle.prep_batch(*data, **kw)
    assert set(_ops(10, 5, B)) == {0, 1, 2}
    buf, desc, _ = gpu_prep(*data, **kw)

    def call(stream):
        mae.mae_prep_batch(desc, buf.visible, buf.mask, buf.ids_restore, buf.ids_keep, buf.target,
                           buf.crop, buf.workspace, stream=stream)

    def wipe():
        buf.visible.fill_(float("nan"))
        buf.target.fill_(float("nan"))
        buf.ids_restore.fill_(-1)
        torch.cuda.synchronize()

    side = torch.cuda.Stream()
    wipe()
    with torch.cuda.stream(side):
        call(side)
    side.synchronize()
    check_prep_against_oracle(prep_to_numpy(buf), ref, what="side stream")

    graph = torch.cuda.CUDAGraph()
    wipe()
    with torch.cuda.graph(graph):
        call(torch.cuda.current_stream())
    for replay in range(3):
        wipe()
        graph.replay()
        torch.cuda.synchronize()
        check_prep_against_oracle(prep_to_numpy(buf), ref, what=f"graph replay {replay}")
        buf.target.mul_(1.0)  # eager work between replays
        torch.cuda.synchronize()


@pytest.mark.parametrize("mode", [mae.MAE_AUG_THREE, mae.MAE_AUG_THREE_PLUS])
def test_full_size_batch_every_image(mode):
    """The bench's launch (B = 4096, 224 px, every patch kept): every image against the oracle."""
    wl = synth.WORKLOADS["c4"]
    data = synth.make_images(wl.kind, wl.B, seed=0)
    kw = dict(out_size=wl.out_size, patch=wl.patch, num_keep=wl.L, scale=(0.28 ** 2, 1.0), seed=3,
              batch_index=7, aug_mode=mode, jitter=0.3)
    buf, _, _ = gpu_prep(*data, **kw)
    assert mae.mae_prep_status(buf.workspace) == 0
    for lo in range(0, wl.B, 256):
        hi = min(lo + 256, wl.B)
        ref = oracle.prep_batch(*data, b_begin=lo, b_end=hi, **kw)
        what = f"images {lo}..{hi} mode {mode}"
        for k in ("ids_restore", "ids_keep", "mask"):
            np.testing.assert_array_equal(getattr(buf, k)[lo:hi].cpu().numpy(), ref[k],
                                          err_msg=what + k)
        np.testing.assert_array_equal(buf.crop[lo:hi, :5].cpu().numpy(), ref["crop"], err_msg=what)
        assert_close_device(buf.target[lo:hi], ref["target"], what=what + " target")
        assert_close_device(buf.visible[lo:hi], ref["visible"], what=what + " visible")
    # properties at full size: grayscale images have equal channels, solarised ones stay dark
    mean = torch.tensor(mae.IMAGENET_MEAN, device="cuda")
    std = torch.tensor(mae.IMAGENET_STD, device="cuda")
    if mode == mae.MAE_AUG_THREE:
        ops = torch.from_numpy(_ops(3, 7, wl.B)).cuda()
        px = buf.target.view(wl.B, -1, 3) * std + mean
        gray = px[ops == oracle.OP_GRAY]
        assert (gray - gray[..., :1]).abs().max().item() < 1e-5
        assert px[ops == oracle.OP_SOLARISE].max().item() <= 127 / 255 + 1e-5
