"""Crop decode: mae_prep_batch fed with JPEG files against the oracle's chain (decode the WHOLE
image with the oracle's decoder, then the same pipeline on the decoded pixels).  The decoder's
integer arithmetic is part of its definition, so pixels agree exactly before the resampling and
the outputs agree to the tolerance of the path."""
import numpy as np
import pytest
import torch

import oracle
import paper_2404_00509_amd as mae
from paper_2404_00509_amd import synth

from helpers import check_prep_against_oracle, prep_to_numpy

pytestmark = pytest.mark.gpu


def _decode_all(files, offsets, sizes):
    """Oracle-decoded images in the packed layout of the decoded-input mode."""
    imgs = [oracle.jpeg_decode(files[o:o + n].tobytes()) for o, n in zip(offsets, sizes)]
    hs = np.array([i.shape[0] for i in imgs], np.int32)
    ws = np.array([i.shape[1] for i in imgs], np.int32)
    lens = hs.astype(np.int64) * ws * 3
    offs = np.zeros(len(imgs), np.int64)
    offs[1:] = np.cumsum(lens)[:-1]
    return np.concatenate([i.reshape(-1) for i in imgs]), offs, hs, ws


def _gpu_jpeg_prep(files, offsets, sizes, bf16=False, **kw):
    dev = [torch.from_numpy(a).cuda() for a in (files, offsets, sizes)]
    desc = mae.make_prep_desc(dev[0], dev[1], None, None, file_sizes=dev[2],
                              out_dtype=mae.MAE_BF16 if bf16 else mae.MAE_F32, **kw)
    buf = mae.alloc_prep_buffers(desc)
    buf.visible.fill_(float("nan"))
    buf.target.fill_(float("nan"))
    buf.crop.fill_(-7)
    mae.mae_prep_batch(desc, buf.visible, buf.mask, buf.ids_restore, buf.ids_keep, buf.target,
                       buf.crop, buf.workspace)
    torch.cuda.synchronize()
    return buf, desc


@pytest.mark.parametrize("sub", ["4:2:0", "4:4:4"])
@pytest.mark.parametrize("kind,S", [("gradient", 112), ("uniform", 64)])
def test_crop_decode_matches_full_decode(sub, kind, S):
    B = 16
    files, offsets, sizes = synth.make_jpegs(kind, B, seed=60, subsampling=sub)
    L = (S // 16) ** 2
    kw = dict(out_size=S, patch=16, num_keep=oracle.num_keep(L, 0.75), seed=13, batch_index=1)
    ref = oracle.prep_batch(*_decode_all(files, offsets, sizes), **kw)
    buf, _ = _gpu_jpeg_prep(files, offsets, sizes, **kw)
    assert mae.mae_prep_status(buf.workspace) == 0
    check_prep_against_oracle(prep_to_numpy(buf), ref, what=f"{kind} {sub}")
