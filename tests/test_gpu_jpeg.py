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

from helpers import assert_close_device, check_neutral_outputs, check_prep_against_oracle, prep_to_numpy

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
    B = 16 if sub == "4:2:0" else 13      # 13: the last group of images is not full
    files, offsets, sizes = synth.make_jpegs(kind, B, seed=60, subsampling=sub)
    L = (S // 16) ** 2
    kw = dict(out_size=S, patch=16, num_keep=oracle.num_keep(L, 0.75), seed=13, batch_index=1)
    ref = oracle.prep_batch(*_decode_all(files, offsets, sizes), **kw)
    buf, _ = _gpu_jpeg_prep(files, offsets, sizes, **kw)
    assert mae.mae_prep_status(buf.workspace) == 0
    check_prep_against_oracle(prep_to_numpy(buf), ref, what=f"{kind} {sub}")


def test_whole_image_and_tiny_crops():
    """Scale range at its ends: the crop is the whole image (every row and column of MCUs is
    decoded), or a few per cent of it (most of the file is skipped)."""
    B, S = 12, 96
    files, offsets, sizes = synth.make_jpegs("gradient", B, seed=61)
    decoded = _decode_all(files, offsets, sizes)
    L = (S // 16) ** 2
    for scale, ratio in (((1.0, 1.0), (1.0, 1.0)), ((0.02, 0.05), (0.75, 4 / 3))):
        kw = dict(out_size=S, patch=16, num_keep=L, scale=scale, ratio=ratio, seed=14,
                  batch_index=2)
        ref = oracle.prep_batch(*decoded, **kw)
        buf, _ = _gpu_jpeg_prep(files, offsets, sizes, **kw)
        check_prep_against_oracle(prep_to_numpy(buf), ref, what=f"scale {scale}")


def test_bf16_tokens_and_finetune_augmentation_from_jpeg():
    B, S = 12, 160
    files, offsets, sizes = synth.make_jpegs("gradient", B, seed=62, quality=75)
    decoded = _decode_all(files, offsets, sizes)
    L = (S // 16) ** 2
    kw = dict(out_size=S, patch=16, num_keep=L, seed=15, batch_index=0,
              aug_mode=mae.MAE_AUG_THREE_PLUS, jitter=0.3)
    ref = oracle.prep_batch(*decoded, **kw)
    buf, _ = _gpu_jpeg_prep(files, offsets, sizes, bf16=True, **kw)
    check_prep_against_oracle(prep_to_numpy(buf), ref, bf16=True, what="jpeg + 3 Aug+")


@pytest.mark.parametrize("quality,optimize", [(50, True), (98, True), (98, False)])
def test_tables_of_the_file_and_other_qualities(quality, optimize):
    """Huffman tables fitted to each image (other code lengths than the standard tables', found
    in the file) and quantisers from coarse to nearly lossless (values of up to 10 bits)."""
    B, S = 12, 96
    files, offsets, sizes = synth.make_jpegs("gradient", B, seed=64, quality=quality,
                                             optimize=optimize)
    L = (S // 16) ** 2
    kw = dict(out_size=S, patch=16, num_keep=oracle.num_keep(L, 0.75), seed=17, batch_index=4)
    ref = oracle.prep_batch(*_decode_all(files, offsets, sizes), **kw)
    buf, _ = _gpu_jpeg_prep(files, offsets, sizes, **kw)
    assert mae.mae_prep_status(buf.workspace) == 0
    check_prep_against_oracle(prep_to_numpy(buf), ref, what=f"quality {quality}")


@pytest.mark.parametrize("rows,blocks", [(0, 0), (2, 0), (0, 3), (0, 1), (3, 0)])
@pytest.mark.parametrize("sub", ["4:2:0", "4:4:4"])
def test_files_whose_rows_are_not_independent(rows, blocks, sub):
    """No restart markers at all (what an encoder writes by default), a restart interval of several
    rows of MCUs, and intervals of a few MCUs that end inside rows: the bytes decoded are the
    oracle's, so every output matches to the path's tolerance."""
    B, S = 14, 96
    kind = "uniform" if blocks == 1 else "gradient"
    files, offsets, sizes = synth.make_jpegs(kind, B, seed=66, subsampling=sub,
                                             restart_rows=rows, restart_blocks=blocks)
    decoded = _decode_all(files, offsets, sizes)
    L = (S // 16) ** 2
    for scale in ((0.2, 1.0), (1.0, 1.0), (0.02, 0.06)):
        kw = dict(out_size=S, patch=16, num_keep=oracle.num_keep(L, 0.75), scale=scale, seed=19,
                  batch_index=6)
        ref = oracle.prep_batch(*decoded, **kw)
        buf, _ = _gpu_jpeg_prep(files, offsets, sizes, **kw)
        assert mae.mae_prep_status(buf.workspace) == 0
        check_prep_against_oracle(prep_to_numpy(buf), ref,
                                  what=f"restart rows {rows} blocks {blocks} {sub} scale {scale}")


def test_a_batch_that_mixes_how_its_files_are_organised():
    import io

    from PIL import Image
    B, S = 12, 112
    imgs = synth.make_images("gradient", B, seed=68)
    variants = [dict(restart_marker_rows=1), dict(), dict(restart_marker_blocks=5),
                dict(restart_marker_rows=4), dict(optimize=True), dict(restart_marker_blocks=2,
                                                                       subsampling="4:4:4")]
    chunks = []
    for b in range(B):
        buf = io.BytesIO()
        args = dict(format="JPEG", quality=85, subsampling="4:2:0")
        args.update(variants[b % len(variants)])
        Image.fromarray(synth.image_view(*imgs, b)).save(buf, **args)
        chunks.append(np.frombuffer(buf.getvalue(), np.uint8))
    sizes = np.array([c.size for c in chunks], np.int32)
    offsets = np.zeros(B, np.int64)
    offsets[1:] = np.cumsum(sizes.astype(np.int64))[:-1]
    files = np.concatenate(chunks)
    L = (S // 16) ** 2
    kw = dict(out_size=S, patch=16, num_keep=oracle.num_keep(L, 0.75), seed=21, batch_index=8)
    ref = oracle.prep_batch(*_decode_all(files, offsets, sizes), **kw)
    buf, _ = _gpu_jpeg_prep(files, offsets, sizes, **kw)
    assert mae.mae_prep_status(buf.workspace) == 0
    check_prep_against_oracle(prep_to_numpy(buf), ref, what="mixed batch")


def test_image_shapes_at_the_limits():
    """Up to 128 rows of MCUs in a file (more rows than a wavefront has lanes), a row of 63 MCUs,
    images smaller than one MCU and with ragged edges, with and without restart markers; an image
    that does not fit the side limit is flagged."""
    import io

    from PIL import Image
    shapes = [(512, 72, "4:4:4", 1), (1024, 48, "4:2:0", 1), (48, 1000, "4:2:0", 1),
              (8, 8, "4:4:4", 1), (5, 7, "4:2:0", 0), (17, 23, "4:2:0", 0), (505, 131, "4:4:4", 0),
              (1040, 64, "4:4:4", 1), (1024, 40, "4:4:4", 1), (1000, 56, "4:4:4", 0)]
    rng = np.random.default_rng(65)
    chunks = []
    for h, w, sub, rst in shapes:
        buf = io.BytesIO()
        kw = dict(restart_marker_rows=1) if rst else {}
        Image.fromarray(synth._one_image("gradient", h, w, rng)).save(
            buf, format="JPEG", quality=90, subsampling=sub, **kw)
        chunks.append(np.frombuffer(buf.getvalue(), np.uint8))
    # and the file written by hand (its own small tables, 162 bytes), after the one that is flagged
    from conftest import read_golden
    hand = next(r[1:] for r in read_golden("jpeg_hand_example.txt") if r[0] == "file")
    chunks.append(np.frombuffer(bytes.fromhex("".join(hand)), np.uint8))
    n = len(chunks)
    sizes = np.array([c.size for c in chunks], np.int32)
    offsets = np.zeros(n, np.int64)
    offsets[1:] = np.cumsum(sizes.astype(np.int64))[:-1]
    files = np.concatenate(chunks)
    S = 64
    L = (S // 16) ** 2
    keep = [b for b in range(n) if b != 7]
    # the oracle gets the hand-written image in place of the file that is too large
    stand_in = [n - 1 if b == 7 else b for b in range(n)]
    decoded = _decode_all(files, offsets[stand_in], sizes[stand_in])
    for scale in ((0.2, 1.0), (1.0, 1.0)):
        kw = dict(out_size=S, patch=16, num_keep=L, scale=scale, seed=18, batch_index=5)
        buf, _ = _gpu_jpeg_prep(files, offsets, sizes, max_image_side=1024, **kw)
        crop = buf.crop.cpu().numpy()
        assert list(np.nonzero(crop[:, 5] == 0)[0]) == [7]        # 1040 rows: beyond the limit
        ref = oracle.prep_batch(*decoded, **kw)
        sel = {k: (v[keep] if v is not None else None) for k, v in ref.items()}
        check_prep_against_oracle(prep_to_numpy(buf, rows=keep), sel, what=f"limits {scale}")


def test_files_the_decoder_does_not_take_are_flagged_and_take_no_part():
    import io

    from PIL import Image
    B, S = 8, 64
    imgs = synth.make_images("uniform", B, seed=63)

    def enc(b, **kw):
        buf = io.BytesIO()
        args = dict(format="JPEG", quality=90, subsampling="4:2:0", restart_marker_rows=1)
        args.update(kw)
        Image.fromarray(synth.image_view(*imgs, b)).save(buf, **args)
        return np.frombuffer(buf.getvalue(), np.uint8)

    good = [enc(b) for b in range(B)]
    gray = io.BytesIO()
    Image.fromarray(synth.image_view(*imgs, 1)).convert("L").save(gray, format="JPEG", quality=90)
    bad = {1: np.frombuffer(gray.getvalue(), np.uint8),   # one component
           3: enc(3, progressive=True),
           4: good[4][:200].copy(),                   # cut inside the tables
           6: enc(6, subsampling="4:2:2")}
    chunks = [bad.get(b, good[b]) for b in range(B)]
    # a file whose entropy-coded data is cut short: decodes (zero bits are supplied), no fault
    chunks[7] = np.concatenate([good[7][:len(good[7]) * 2 // 3], np.array([0xFF, 0xD9], np.uint8)])
    sizes = np.array([c.size for c in chunks], np.int32)
    offsets = np.zeros(B, np.int64)
    offsets[1:] = np.cumsum(sizes.astype(np.int64))[:-1]
    files = np.concatenate(chunks)
    L = (S // 16) ** 2
    kw = dict(out_size=S, patch=16, num_keep=L, seed=16, batch_index=3)
    buf, _ = _gpu_jpeg_prep(files, offsets, sizes, **kw)
    crop = buf.crop.cpu().numpy()
    flagged = sorted(int(b) for b in np.nonzero(crop[:, 5] == 0)[0])
    assert set(bad) <= set(flagged) <= set(bad) | {7}
    assert mae.mae_prep_status(buf.workspace) == len(flagged)
    # the good files give what they give on their own
    keep = [b for b in range(B) if b not in flagged]
    g_sizes = np.array([good[b].size for b in range(B)], np.int32)
    g_offsets = np.zeros(B, np.int64)
    g_offsets[1:] = np.cumsum(g_sizes.astype(np.int64))[:-1]
    ref = oracle.prep_batch(*_decode_all(np.concatenate(good), g_offsets, g_sizes), **kw)
    got = prep_to_numpy(buf, rows=keep)
    sel = {k: (v[keep] if v is not None else None) for k, v in ref.items()}
    check_prep_against_oracle(got, sel, what="good files next to bad ones")
    # flagged samples get the neutral outputs (nothing masked, identity order, zero pixels)
    for b in flagged:
        check_neutral_outputs(buf, b)


def test_files_of_maximum_side_500():
    """The size of the paper's crop-decode benchmark: 24 to 32 rows of MCUs per image, so the four
    images of a wavefront have more rows than it has lanes."""
    B, S = 6, 224
    files, offsets, sizes = synth.make_jpegs("gradient500", B, seed=67)
    L = (S // 16) ** 2
    kw = dict(out_size=S, patch=16, num_keep=oracle.num_keep(L, 0.75), seed=20, batch_index=7)
    ref = oracle.prep_batch(*_decode_all(files, offsets, sizes), **kw)
    buf, _ = _gpu_jpeg_prep(files, offsets, sizes, max_image_side=512, **kw)
    assert mae.mae_prep_status(buf.workspace) == 0
    check_prep_against_oracle(prep_to_numpy(buf), ref, what="side 500")


def test_jpeg_input_on_a_side_stream_and_in_a_captured_graph():
    """The JPEG path enqueues kernels only (header, crop draws, tables, decode, colour, resample,
    augmentation): it can run on any stream and be captured; every replay is checked."""
    B, S = 8, 96
    files, offsets, sizes = synth.make_jpegs("gradient", B, seed=66)
    L = (S // 16) ** 2
    kw = dict(out_size=S, patch=16, num_keep=L, seed=19, batch_index=6,
              aug_mode=mae.MAE_AUG_THREE_PLUS, jitter=0.3)
    ref = oracle.prep_batch(*_decode_all(files, offsets, sizes), **kw)
    dev = [torch.from_numpy(a).cuda() for a in (files, offsets, sizes)]
    desc = mae.make_prep_desc(dev[0], dev[1], None, None, file_sizes=dev[2], **kw)
    buf = mae.alloc_prep_buffers(desc)

    def step(stream):
        mae.mae_prep_batch(desc, buf.visible, buf.mask, buf.ids_restore, buf.ids_keep, buf.target,
                           buf.crop, buf.workspace, stream=stream)

    def wipe():
        buf.visible.fill_(float("nan"))
        buf.target.fill_(float("nan"))
        buf.ids_restore.fill_(-1)
        buf.workspace.zero_()
        torch.cuda.synchronize()

    side = torch.cuda.Stream()
    wipe()
    with torch.cuda.stream(side):
        step(side)
    side.synchronize()
    check_prep_against_oracle(prep_to_numpy(buf), ref, what="side stream")
    graph = torch.cuda.CUDAGraph()
    wipe()
    with torch.cuda.graph(graph):
        step(torch.cuda.current_stream())
    for replay in range(3):
        wipe()
        graph.replay()
        torch.cuda.synchronize()
        check_prep_against_oracle(prep_to_numpy(buf), ref, what=f"graph replay {replay}")
        buf.target.mul_(1.0)          # eager work between replays
        torch.cuda.synchronize()


def test_crop_decode_full_size_every_image():
    """The bench's launch: 4096 files (max side 256, quality 90, 4:2:0) -> 224 px, every image
    against the oracle's path on the oracle-decoded images."""
    from concurrent.futures import ThreadPoolExecutor

    wl = synth.WORKLOADS["c4"]
    files, offsets, sizes = synth.make_jpegs(wl.kind, wl.B, seed=0)
    K = oracle.num_keep(wl.L, wl.mask_ratio)
    kw = dict(out_size=wl.out_size, patch=wl.patch, num_keep=K, seed=5, batch_index=9)
    buf, _ = _gpu_jpeg_prep(files, offsets, sizes, **kw)
    assert mae.mae_prep_status(buf.workspace) == 0
    # whole-file decode by the oracle (the C call releases the interpreter lock)
    blobs = [files[o:o + n].tobytes() for o, n in zip(offsets, sizes)]
    with ThreadPoolExecutor(16) as pool:
        imgs = list(pool.map(oracle.jpeg_decode, blobs))
    lens = np.array([im.size for im in imgs], np.int64)
    offs = np.zeros(wl.B, np.int64)
    offs[1:] = np.cumsum(lens)[:-1]
    decoded = (np.concatenate([im.reshape(-1) for im in imgs]), offs,
               np.array([im.shape[0] for im in imgs], np.int32),
               np.array([im.shape[1] for im in imgs], np.int32))
    for lo in range(0, wl.B, 256):
        hi = min(lo + 256, wl.B)
        ref = oracle.prep_batch(*decoded, b_begin=lo, b_end=hi, **kw)
        what = f"files {lo}..{hi}"
        for k in ("ids_restore", "ids_keep", "mask"):
            np.testing.assert_array_equal(getattr(buf, k)[lo:hi].cpu().numpy(), ref[k],
                                          err_msg=what + k)
        np.testing.assert_array_equal(buf.crop[lo:hi, :5].cpu().numpy(), ref["crop"], err_msg=what)
        assert_close_device(buf.target[lo:hi], ref["target"], what=what + " target")
        assert_close_device(buf.visible[lo:hi], ref["visible"], what=what + " visible")


# ---- the files' row index ------------------------------------------------------------------------
def _row_index(files, offsets, sizes, max_image_side=0):
    """mae_jpeg_index over the files: (index tensor [B, bytes per file], device inputs)."""
    dev = [torch.from_numpy(a).cuda() for a in (files, offsets, sizes)]
    desc = mae.make_prep_desc(dev[0], dev[1], None, None, file_sizes=dev[2], out_size=32, patch=16,
                              num_keep=1, max_image_side=max_image_side)
    index = torch.full((mae.mae_jpeg_index_bytes(desc),), 0xEE, dtype=torch.uint8, device="cuda")
    ws = torch.empty(mae.mae_prep_workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    mae.mae_jpeg_index(desc, index, ws)
    torch.cuda.synchronize()
    return index.view(len(sizes), -1), dev


def _prep_with_index(dev, index, **kw):
    desc = mae.make_prep_desc(dev[0], dev[1], None, None, file_sizes=dev[2], row_index=index, **kw)
    buf = mae.alloc_prep_buffers(desc)
    buf.visible.fill_(float("nan"))
    buf.target.fill_(float("nan"))
    buf.crop.fill_(-7)
    mae.mae_prep_batch(desc, buf.visible, buf.mask, buf.ids_restore, buf.ids_keep, buf.target,
                       buf.crop, buf.workspace)
    torch.cuda.synchronize()
    return buf


@pytest.mark.parametrize("sub", ["4:2:0", "4:4:4"])
def test_row_index_replaces_the_walk_through_the_file(sub):
    """The index of a file (computed once, whatever crops come later) gives the decoder the same
    row starts as walking through the file does: same outputs bit for bit, for files without
    restart markers, with odd intervals and with a marker per row, mixed in one batch, for
    several batches of crops, and for a batch gathered from the indexed files in another order."""
    B, S = 15, 96
    parts = [synth.make_jpegs("gradient", B, seed=70, subsampling=sub, restart_rows=r,
                              restart_blocks=k) for r, k in ((0, 0), (1, 0), (0, 3))]
    pick = np.arange(B) % 3  # file b comes from organisation b mod 3
    blobs = [parts[pick[b]][0][parts[pick[b]][1][b]:parts[pick[b]][1][b] + parts[pick[b]][2][b]]
             for b in range(B)]
    sizes = np.array([len(x) for x in blobs], np.int32)
    offsets = np.zeros(B, np.int64)
    offsets[1:] = np.cumsum((sizes.astype(np.int64) + 7) // 8 * 8)[:-1]
    files = np.zeros(int(offsets[-1] + (sizes[-1] + 7) // 8 * 8), np.uint8)
    for b in range(B):
        files[offsets[b]:offsets[b] + sizes[b]] = blobs[b]
    decoded = _decode_all(files, offsets, sizes)
    index, dev = _row_index(files, offsets, sizes)
    L = (S // 16) ** 2
    for batch_index, scale in ((0, (0.2, 1.0)), (1, (1.0, 1.0)), (2, (0.03, 0.1))):
        kw = dict(out_size=S, patch=16, num_keep=oracle.num_keep(L, 0.75), scale=scale, seed=23,
                  batch_index=batch_index)
        ref = oracle.prep_batch(*decoded, **kw)
        plain, _ = _gpu_jpeg_prep(files, offsets, sizes, **kw)
        got = _prep_with_index(dev, index, **kw)
        assert mae.mae_prep_status(got.workspace) == 0
        check_prep_against_oracle(prep_to_numpy(got), ref, what=f"index, batch {batch_index}")
        assert torch.equal(got.target, plain.target) and torch.equal(got.visible, plain.visible)
    # another batch of the same files: reversed order, index entries gathered like the files
    order = np.arange(B)[::-1].copy()
    sizes2 = sizes[order]
    offsets2 = np.zeros(B, np.int64)
    offsets2[1:] = np.cumsum((sizes2.astype(np.int64) + 7) // 8 * 8)[:-1]
    files2 = np.zeros(int(offsets2[-1] + (sizes2[-1] + 7) // 8 * 8), np.uint8)
    for i, b in enumerate(order):
        files2[offsets2[i]:offsets2[i] + sizes2[i]] = blobs[b]
    dev2 = [torch.from_numpy(a).cuda() for a in (files2, offsets2, sizes2)]
    index2 = index[torch.from_numpy(order).cuda()].contiguous()
    kw = dict(out_size=S, patch=16, num_keep=L, seed=24, batch_index=5)
    ref = oracle.prep_batch(*_decode_all(files2, offsets2, sizes2), **kw)
    got = _prep_with_index(dev2, index2, **kw)
    assert mae.mae_prep_status(got.workspace) == 0
    check_prep_against_oracle(prep_to_numpy(got), ref, what="gathered index")


def test_row_index_entries_are_checked_before_use():
    """The index is the caller's memory.  Entries that cannot belong to their file (zeros, noise,
    the entries of another file) give samples flagged invalid or wrong pixels; the call returns,
    every output is written, and good entries next to them still decode exactly."""
    B, S = 12, 64
    files, offsets, sizes = synth.make_jpegs("gradient", B, seed=71, restart_rows=0)
    decoded = _decode_all(files, offsets, sizes)
    index, dev = _row_index(files, offsets, sizes)
    bad = index.clone()
    bad[1].zero_()                                       # position 0: before the scan data
    rng = np.random.default_rng(5)
    bad[4] = torch.from_numpy(rng.integers(0, 256, bad.shape[1], dtype=np.uint8)).cuda()
    bad[7] = index[8]                                    # another file's row starts
    bad[10].fill_(0xFF)                                  # negative position and bit count
    L = (S // 16) ** 2
    kw = dict(out_size=S, patch=16, num_keep=L, seed=25, batch_index=0)
    ref = oracle.prep_batch(*decoded, **kw)
    got = _prep_with_index(dev, bad.contiguous(), **kw)
    n_bad = mae.mae_prep_status(got.workspace)
    assert 3 <= n_bad <= 4            # only another file's entries may decode (to wrong pixels)
    out = prep_to_numpy(got)
    assert np.isfinite(out["target"]).all() and np.isfinite(out["visible"]).all()
    good = np.array([b for b in range(B) if b not in (1, 4, 7, 10)])
    assert np.all(out["crop"][good, 5] == 1)
    np.testing.assert_array_equal(out["ids_restore"][good], ref["ids_restore"][good])
    assert_close_device(got.target[torch.from_numpy(good).cuda()], ref["target"][good],
                        what="good entries")
    for b in (1, 4, 10):
        check_neutral_outputs(got, b)


def test_row_index_of_files_the_decoder_does_not_take():
    """A file that is not decodable gets an index of unknown rows, and so does every row a file
    does not have; with such an index the sample is flagged exactly as without one."""
    B = 6
    files, offsets, sizes = synth.make_jpegs("gradient", B, seed=72, restart_rows=0)
    files = files.copy()
    files[offsets[2] + 2:offsets[2] + 40] = 0            # the header of file 2 destroyed
    index, dev = _row_index(files, offsets, sizes)
    rows = index.view(B, -1, 32)
    pos = rows[:, :, :4].contiguous().view(torch.int32).view(B, -1).cpu().numpy()
    assert np.all(pos[2] == -1)
    for b in (0, 1, 3, 4, 5):
        h = oracle.jpeg_decode(files[offsets[b]:offsets[b] + sizes[b]].tobytes()).shape[0]
        n_rows = (h + 15) // 16
        assert np.all(pos[b, :n_rows] > 0) and np.all(pos[b, n_rows:] == -1)
        assert np.all(np.diff(pos[b, :n_rows]) > 0)      # rows follow each other in the file
    kw = dict(out_size=64, patch=16, num_keep=4, seed=26, batch_index=0)
    got = _prep_with_index(dev, index, **kw)
    assert mae.mae_prep_status(got.workspace) == 1
    assert prep_to_numpy(got)["crop"][2, 5] == 0


def test_row_index_with_large_files_augmentation_and_the_loss_without_target():
    """The index under the other modes of the call: files of maximum side 500 (two images per
    wavefront in the decode kernel, 64 index rows per file), the finetuning augmentation, and the
    loss that reads the decoded regions again."""
    B, S = 6, 128
    files, offsets, sizes = synth.make_jpegs("gradient500", B, seed=73, restart_rows=0)
    decoded = _decode_all(files, offsets, sizes)
    index, dev = _row_index(files, offsets, sizes, max_image_side=512)
    assert index.shape[1] == 64 * 32
    L = (S // 16) ** 2
    kw = dict(out_size=S, patch=16, num_keep=L, seed=27, batch_index=1, max_image_side=512,
              aug_mode=mae.MAE_AUG_THREE_PLUS, jitter=0.3)
    ref = oracle.prep_batch(*decoded, **{k: v for k, v in kw.items() if k != "max_image_side"})
    got = _prep_with_index(dev, index, **kw)
    assert mae.mae_prep_status(got.workspace) == 0
    check_prep_against_oracle(prep_to_numpy(got), ref, what="index, side 500, 3 Aug+")

    # pretraining step without a stored target on the same files
    K = oracle.num_keep(L, 0.75)
    kw = dict(out_size=S, patch=16, num_keep=K, seed=28, batch_index=2, max_image_side=512)
    ref = oracle.prep_batch(*decoded, **{k: v for k, v in kw.items() if k != "max_image_side"})
    desc = mae.make_prep_desc(dev[0], dev[1], None, None, file_sizes=dev[2], row_index=index, **kw)
    buf = mae.alloc_prep_buffers(desc, want_target=False)
    mae.mae_prep_batch(desc, buf.visible, buf.mask, buf.ids_restore, buf.ids_keep, None, buf.crop,
                       buf.workspace)
    M = B * (L - K)
    pred_host = synth.make_pred(9, B, L, 768)
    pred = torch.from_numpy(pred_host).cuda()
    ldesc = mae.make_loss_desc(pred, None, buf.mask, num_masked=M)
    lws = torch.empty(mae.mae_loss_from_images_workspace_bytes(desc, ldesc), dtype=torch.uint8,
                      device="cuda")
    loss = torch.zeros(1, device="cuda")
    grad = torch.empty_like(pred)
    mae.mae_normpix_loss_from_images(desc, buf.workspace, ldesc, loss, grad, lws)
    torch.cuda.synchronize()
    ref_loss, ref_grad, _ = oracle.normpix_loss(pred_host, ref["target"], ref["mask"], num_masked=M)
    assert abs(loss.item() - ref_loss) <= 1e-5 + 1e-5 * abs(ref_loss)
    from helpers import check_grad
    check_grad(grad.cpu().numpy(), ref_grad, 768, M, what="index + loss from images")
