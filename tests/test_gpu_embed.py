"""Patch embedding of the visible tokens: the matrix-core kernel behind mae_patch_embed against the
oracle's fp64 triple loop, on the same seeded bf16-representable inputs.

Tolerance.  The products of two bf16 numbers are exact in fp32; what the kernel loses is the fp32
accumulation of D of them plus two fp32 additions.  With u = 2^-24 a sum of D + 2 terms in any
order is within (D + 1) u S of the exact value, S = sum_d |a_d w_d| + |bias| + |pos| (first-order
bound of recursive summation).  fp32 output: that bound (plus its own rounding, 2^-24 |ref|);
bf16 output: additionally one rounding to 8 significant bits, 2^-9 |ref|, checked with 2^-8."""
import numpy as np
import pytest
import torch

import oracle
import paper_2404_00509_amd as mae
from paper_2404_00509_amd import synth

from helpers import gpu_prep

pytestmark = pytest.mark.gpu

U32 = 2.0 ** -24


def _bf16(x):
    """fp32 array -> torch CPU bf16 tensor (round to nearest even)."""
    return torch.from_numpy(np.ascontiguousarray(x, np.float32)).to(torch.bfloat16)


def _inputs(seed, M, D, E, L):
    weight, bias, pos = synth.make_embed_params(seed, D, E, L)
    vis = _bf16(synth.make_visible_rows(seed, M, D))
    return vis, _bf16(weight), bias, pos, synth.make_ids(seed, M, L)


def _reference(vis, w, bias, pos, ids):
    """Oracle result and the magnitude sum S of every output, both [M, E] float64."""
    a = vis.float().numpy()
    wf = w.float().numpy()
    M = a.shape[0]
    ref = oracle.patch_embed(a[None], None if ids is None else ids[None], wf, bias, pos)[0]
    S = np.abs(a).astype(np.float64) @ np.abs(wf).astype(np.float64).T
    if bias is not None:
        S += np.abs(bias)[None]
    if pos is not None:
        S += np.abs(pos[ids])
    assert ref.shape == S.shape == (M, wf.shape[0])
    return ref, S


def _gpu(vis, w, bias, pos, ids, bf16_out, tokens=None, stream=None):
    dev = "cuda"
    dv, dw = vis.to(dev), w.to(dev)
    db = None if bias is None else torch.from_numpy(bias).to(dev)
    dp = None if pos is None else torch.from_numpy(pos).to(dev)
    di = None if ids is None else torch.from_numpy(ids).to(dev)
    desc = mae.make_embed_desc(dv, di, dw, db, dp,
                               out_dtype=mae.MAE_BF16 if bf16_out else mae.MAE_F32)
    if tokens is None:
        tokens = torch.full((dv.shape[0], dw.shape[0]), float("nan"), device=dev,
                            dtype=torch.bfloat16 if bf16_out else torch.float32)
    mae.mae_patch_embed(desc, tokens, stream=stream)
    torch.cuda.synchronize()
    return tokens, (dv, dw, db, dp, di, desc)


def _check(tokens, ref, S, D, bf16_out, what):
    got = tokens.float().cpu().numpy().astype(np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    bound = (D + 1) * U32 * S + (2.0 ** -8 if bf16_out else U32) * np.abs(ref) + 1e-30
    err = np.abs(got - ref)
    bad = ~(err <= bound)  # also catches NaN left by a value that was never written
    if bad.any():
        i = np.unravel_index(np.argmax(np.where(np.isnan(err), np.inf, err - bound)), err.shape)
        raise AssertionError(f"{what}: {int(bad.sum())} of {bad.size} outputs out of tolerance; "
                             f"worst at {i}: gpu {got[i]!r} ref {ref[i]!r} bound {bound[i]:.3e}")


# M, D, E, L: several 256 x 128 tiles with ragged edges in both directions, every kind of last
# slice of D (none, 4, 8, 12, ... values past a multiple of 32), one to five slices
SHAPES = [
    (1176, 768, 768, 196),   # 24 images of the 224-pixel, patch-16 stage at ViT-B width
    (320, 588, 1024, 256),   # patch 14 at ViT-L width: D = 18 * 32 + 12
    (700, 192, 136, 64),     # E a multiple of 8 that ends inside a tile
    (513, 100, 70, 49),      # E not a multiple of 8: element-wise stores
    (257, 36, 129, 16),
    (1, 4, 1, 1),
    (5, 8, 3, 4),
    (64, 32, 128, 196),
    (300, 64, 256, 196),
    (300, 96, 384, 100),
    (256, 3072, 128, 256),   # the longest row the call accepts
]


@pytest.mark.parametrize("M,D,E,L", SHAPES)
@pytest.mark.parametrize("bf16_out", [True, False])
def test_embed_matches_the_oracle(M, D, E, L, bf16_out):
    vis, w, bias, pos, ids = _inputs(7, M, D, E, L)
    ref, S = _reference(vis, w, bias, pos, ids)
    tokens, _ = _gpu(vis, w, bias, pos, ids, bf16_out)
    _check(tokens, ref, S, D, bf16_out, f"M{M} D{D} E{E} L{L}")


@pytest.mark.parametrize("with_bias,with_pos", [(False, False), (True, False), (False, True)])
def test_embed_optional_terms(with_bias, with_pos):
    M, D, E, L = 300, 588, 200, 256
    vis, w, bias, pos, ids = _inputs(8, M, D, E, L)
    bias = bias if with_bias else None
    pos, ids = (pos, ids) if with_pos else (None, None)
    ref, S = _reference(vis, w, bias, pos, ids)
    tokens, _ = _gpu(vis, w, bias, pos, ids, False)
    _check(tokens, ref, S, D, False, f"bias {with_bias} pos {with_pos}")


def test_embed_plain_product_special_cases():
    # weight = rows of the identity: tokens reproduce the inputs exactly (no rounding anywhere)
    M, D = 130, 64
    vis = _bf16(synth.make_visible_rows(9, M, D))
    eye = _bf16(np.eye(D, dtype=np.float32))
    tokens, _ = _gpu(vis, eye, None, None, None, False)
    np.testing.assert_array_equal(tokens.cpu().numpy(), vis.float().numpy())
    # zero weight: tokens = bias + pos[ids], exact in fp32
    _, bias, pos = synth.make_embed_params(9, D, 40, 25)
    ids = synth.make_ids(9, M, 25)
    tokens, _ = _gpu(vis, _bf16(np.zeros((40, D), np.float32)), bias, pos, ids, False)
    np.testing.assert_array_equal(tokens.cpu().numpy(), bias[None] + pos[ids])


def test_embed_clamps_patch_indices_outside_the_grid():
    M, D, E, L = 70, 64, 48, 9
    vis, w, bias, pos, ids = _inputs(10, M, D, E, L)
    wild = ids.copy()
    wild[::3] = -5
    wild[1::3] = L + 1000
    clamped = np.clip(wild, 0, L - 1)
    ref, S = _reference(vis, w, bias, pos, clamped)
    tokens, _ = _gpu(vis, w, bias, pos, wild, False)
    _check(tokens, ref, S, D, False, "clamped ids")


@pytest.mark.parametrize("name", ["c4", "c5"])
def test_embed_full_size_sampled(name):
    """The bench's launch: every visible row of the batch at ViT-B width; the oracle computes a
    sample of rows (first and last tiles, and rows spread over the whole batch)."""
    wl = synth.WORKLOADS[name]
    K = oracle.num_keep(wl.L, wl.mask_ratio)
    M, D, E, L = wl.B * K, wl.D, 768, wl.L
    weight, bias, pos = synth.make_embed_params(11, D, E, L)
    w = _bf16(weight)
    # rows repeat with a period that is no multiple of the tile height, ids do not
    base = _bf16(synth.make_visible_rows(11, 1000, D))
    vis = base.repeat((M + 999) // 1000, 1)[:M].contiguous()
    ids = synth.make_ids(11, M, L)
    rows = np.unique(np.concatenate([np.arange(0, 300), np.arange(M - 300, M),
                                     np.random.default_rng(11).integers(0, M, 400)]))
    ref, S = _reference(vis[rows], w, bias, pos, ids[rows])
    for bf16_out in (True, False):
        tokens, _ = _gpu(vis, w, bias, pos, ids, bf16_out)
        _check(tokens[torch.from_numpy(rows).cuda()], ref, S, D, bf16_out, f"{name} sampled")
        # property at full size: rows with equal inputs and equal patch index give equal outputs
        t = tokens.float()
        same = torch.from_numpy((ids[1000:2000] == ids[:1000])).cuda()
        assert torch.equal(t[:1000][same], t[1000:2000][same])
        assert not torch.isnan(t).any()


def test_embed_after_the_input_pipeline():
    """mae_prep_batch (bf16 visible) feeding mae_patch_embed, against the oracle's chain.  The
    GPU's visible values may differ from the oracle's by one bf16 rounding step, which the
    bound carries: 2^-8 sum |a w| on top of the accumulation bound."""
    wl = synth.WORKLOADS["c1"]
    B = 16
    data = synth.make_images(wl.kind, B, seed=5)
    K = oracle.num_keep(wl.L, wl.mask_ratio)
    kw = dict(out_size=wl.out_size, patch=wl.patch, num_keep=K, seed=3, batch_index=1)
    ref_prep = oracle.prep_batch(*data, **kw)
    buf, _, _ = gpu_prep(*data, bf16=True, **kw)
    np.testing.assert_array_equal(buf.ids_keep.cpu().numpy(), ref_prep["ids_keep"])
    E = 192
    weight, bias, pos = synth.make_embed_params(12, wl.D, E, wl.L)
    w = _bf16(weight)
    vis_ref = _bf16(ref_prep["visible"].reshape(B * K, wl.D))
    ids = ref_prep["ids_keep"].reshape(-1)
    ref, S = _reference(vis_ref, w, bias, pos, ids)
    dev = "cuda"
    tokens = torch.full((B, K, E), float("nan"), device=dev)
    desc = mae.make_embed_desc(buf.visible, buf.ids_keep, w.to(dev),
                               torch.from_numpy(bias).to(dev), torch.from_numpy(pos).to(dev),
                               out_dtype=mae.MAE_F32)
    assert desc.M == B * K and desc.L == wl.L
    mae.mae_patch_embed(desc, tokens)
    torch.cuda.synchronize()
    got = tokens.reshape(B * K, E).cpu().numpy().astype(np.float64)
    bound = ((wl.D + 1) * U32 + 2.0 ** -8) * S + U32 * np.abs(ref)
    assert np.all(np.abs(got - ref) <= bound)
    # and the typical error is far below that worst case
    assert np.median(np.abs(got - ref) / S) < 2.0 ** -12


def test_embed_on_a_side_stream_and_in_a_captured_graph():
    M, D, E, L = 600, 588, 256, 256
    vis, w, bias, pos, ids = _inputs(13, M, D, E, L)
    ref, S = _reference(vis, w, bias, pos, ids)
    tokens, (dv, dw, db, dp, di, desc) = _gpu(vis, w, bias, pos, ids, True)
    _check(tokens, ref, S, D, True, "eager")
    side = torch.cuda.Stream()
    tokens.fill_(float("nan"))
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        mae.mae_patch_embed(desc, tokens, stream=side)
    side.synchronize()
    _check(tokens, ref, S, D, True, "side stream")
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        mae.mae_patch_embed(desc, tokens, stream=torch.cuda.current_stream())
    for replay in range(3):
        tokens.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        _check(tokens, ref, S, D, True, f"graph replay {replay}")
        dv.mul_(1.0)  # eager work between replays
        torch.cuda.synchronize()
