"""Host-side behaviour of the C ABI that needs no GPU: the library loads, exports every symbol the
public header declares, and rejects bad descriptors before anything is launched."""
import ctypes as C
import os
import re

import pytest
import torch

import oracle
import paper_2404_00509_amd as mae
from paper_2404_00509_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000  # never dereferenced: argument errors are found before any launch


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(mae.LIB_PATH):
        from paper_2404_00509_amd.build import build_hip
        build_hip()
    return mae.load()


def test_library_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "mae_hip.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(mae_[a-z_]+)\s*\(", header))
    assert declared == set(mae.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    assert mae.mae_version() >= 100


def test_error_strings(lib):
    seen = {mae.mae_error_string(s) for s in range(-7, 1)}
    assert len(seen) == 8 and "unknown status" not in seen
    assert mae.mae_error_string(-99) == "unknown status"


def test_num_keep_matches_the_oracle(lib):
    for L in (1, 16, 49, 100, 144, 196, 256):
        for m in (0.0, 0.5, 0.66, 0.75, 0.8, 0.85, 1.0):
            assert mae.mae_num_keep(L, m) == oracle.num_keep(L, m)
    assert mae.mae_num_keep(100, 0.8) == 19
    assert mae.mae_num_keep(0, 0.5) == -1 and mae.mae_num_keep(10, 1.5) == -1


def _prep_desc(**over):
    d = binding.MaePrepDesc()
    d.B = 4
    d.images = d.offsets = d.heights = d.widths = FAKE
    d.images_bytes = 1 << 20
    d.out_size, d.patch, d.num_keep = 224, 16, 49
    d.scale_lo, d.scale_hi, d.ratio_lo, d.ratio_hi, d.flip_p = 0.2, 1.0, 0.75, 4 / 3, 0.5
    d.mean = (C.c_float * 3)(*mae.IMAGENET_MEAN)
    d.std = (C.c_float * 3)(*mae.IMAGENET_STD)
    d.seed, d.batch_index, d.sample_base, d.noise_bits, d.out_dtype = 0, 0, 0, 32, 0
    d.max_image_side = 0
    d.aug_mode, d.jitter = 0, 0.3
    for k, v in over.items():
        if k == "std":
            d.std = (C.c_float * 3)(*v)
        else:
            setattr(d, k, v)
    return d


def _call_prep(lib, d, visible=FAKE, mask=FAKE, ids_restore=FAKE, workspace=FAKE, ws_bytes=1 << 20):
    return lib.mae_prep_batch(C.byref(d), visible, mask, ids_restore, None, None, None, workspace,
                              ws_bytes, None)


@pytest.mark.parametrize("over,status", [
    (dict(images=None), binding.MAE_ERR_NULL),
    (dict(offsets=None), binding.MAE_ERR_NULL),
    (dict(heights=None), binding.MAE_ERR_NULL),
    (dict(widths=None), binding.MAE_ERR_NULL),
    (dict(B=0), binding.MAE_ERR_SHAPE),
    (dict(B=-3), binding.MAE_ERR_SHAPE),
    (dict(B=(1 << 20) + 1), binding.MAE_ERR_RANGE),
    (dict(out_size=230), binding.MAE_ERR_SHAPE),        # not a multiple of the patch
    (dict(out_size=0), binding.MAE_ERR_SHAPE),
    (dict(patch=0), binding.MAE_ERR_SHAPE),
    (dict(num_keep=0), binding.MAE_ERR_SHAPE),
    (dict(num_keep=197), binding.MAE_ERR_SHAPE),
    (dict(out_size=272), binding.MAE_ERR_RANGE),        # 17 x 17 = 289 patches > 256
    (dict(out_size=66, patch=33, num_keep=1), binding.MAE_ERR_RANGE),
    (dict(images_bytes=0), binding.MAE_ERR_RANGE),
    (dict(scale_lo=0.0), binding.MAE_ERR_RANGE),
    (dict(scale_lo=0.9, scale_hi=0.5), binding.MAE_ERR_RANGE),
    (dict(scale_hi=1.5), binding.MAE_ERR_RANGE),
    (dict(ratio_lo=0.0), binding.MAE_ERR_RANGE),
    (dict(ratio_lo=1.2, ratio_hi=1.1), binding.MAE_ERR_RANGE),
    (dict(ratio_lo=0.5), binding.MAE_ERR_RANGE),        # ln below -1/2
    (dict(ratio_hi=2.0), binding.MAE_ERR_RANGE),
    (dict(flip_p=-0.1), binding.MAE_ERR_RANGE),
    (dict(flip_p=1.1), binding.MAE_ERR_RANGE),
    (dict(flip_p=float("nan")), binding.MAE_ERR_RANGE),
    (dict(std=(0.2, 0.0, 0.2)), binding.MAE_ERR_RANGE),
    (dict(noise_bits=0), binding.MAE_ERR_RANGE),
    (dict(noise_bits=33), binding.MAE_ERR_RANGE),
    (dict(sample_base=0xFFFFFFFF), binding.MAE_ERR_RANGE),
    (dict(out_dtype=7), binding.MAE_ERR_DTYPE),
    (dict(max_image_side=-1), binding.MAE_ERR_RANGE),
    (dict(max_image_side=40000), binding.MAE_ERR_RANGE),
    (dict(aug_mode=3), binding.MAE_ERR_RANGE),
    (dict(aug_mode=-1), binding.MAE_ERR_RANGE),
    (dict(aug_mode=2, jitter=-0.1), binding.MAE_ERR_RANGE),
    (dict(aug_mode=2, jitter=float("nan")), binding.MAE_ERR_RANGE),
    (dict(aug_mode=1, out_size=225, patch=15, num_keep=64), binding.MAE_ERR_SHAPE),  # odd patch
])
def test_prep_rejects_bad_descriptors(lib, over, status):
    d = _prep_desc(**over)
    assert _call_prep(lib, d) == status
    assert lib.mae_prep_workspace_bytes(C.byref(d)) == 0


def test_prep_workspace_grows_with_the_augmentation(lib):
    plain = lib.mae_prep_workspace_bytes(C.byref(_prep_desc()))
    assert plain == 256 + 4 * 32
    three = lib.mae_prep_workspace_bytes(C.byref(_prep_desc(aug_mode=1)))
    plus = lib.mae_prep_workspace_bytes(C.byref(_prep_desc(aug_mode=2)))
    # crop records rounded up to 256, the augmentation's draws and taps (64 bytes per sample) likewise,
    # then the 8-bit crops
    assert three == 512 + 256 + 4 * 224 * 224 * 3
    # a double per row of patches and column part: two parts in the blur kernel, one in the
    # resampling kernel
    assert plus == three + 4 * 14 * (2 + 1) * 8
    d = _prep_desc(aug_mode=2)
    assert _call_prep(lib, d, ws_bytes=plus - 1) == binding.MAE_ERR_WORKSPACE


def _jpeg_desc(**over):
    d = _prep_desc(heights=None, widths=None, input_format=binding.MAE_INPUT_JPEG, file_sizes=FAKE)
    for k, v in over.items():
        setattr(d, k, v)
    return d


@pytest.mark.parametrize("over,status", [
    (dict(input_format=2), binding.MAE_ERR_RANGE),
    (dict(input_format=-1), binding.MAE_ERR_RANGE),
    (dict(file_sizes=None), binding.MAE_ERR_NULL),
    (dict(images=FAKE + 4), binding.MAE_ERR_RANGE),     # files are read in aligned 8-byte pieces
    (dict(offsets=None), binding.MAE_ERR_NULL),
])
def test_prep_rejects_bad_jpeg_descriptors(lib, over, status):
    d = _jpeg_desc(**over)
    assert _call_prep(lib, d, ws_bytes=1 << 30) == status
    assert lib.mae_prep_workspace_bytes(C.byref(d)) == 0


def test_jpeg_input_needs_no_sizes_and_a_slot_per_image(lib):
    """Heights and widths come out of the files; the workspace holds, per image, one slot for the
    decoded planes and one for the RGB region, each 3 bytes per pixel of a square whose side is
    max_image_side rounded up to 16 (256 when the caller gives none)."""
    up = lambda v: (v + 255) & ~255
    B = 4
    head = 256 + B * 32
    # file records, heights, widths, region widths, offsets, decoding tables (5488 bytes per image)
    for step in (B * 64, B * 4, B * 4, B * 4, B * 8, B * 5488):
        head = up(head) + step
    for side, slot in ((0, 256), (500, 512), (512, 512), (513, 528)):
        d = _jpeg_desc(max_image_side=side)
        # ... the states at which the crop's rows of MCUs start: 32 bytes per 8 pixels of the side
        tables = up(head) + B * (slot // 8) * 32
        want = up(up(tables) + B * slot * slot * 3) + B * slot * slot * 3
        assert lib.mae_prep_workspace_bytes(C.byref(d)) == want
        assert _call_prep(lib, d, ws_bytes=want - 1) == binding.MAE_ERR_WORKSPACE
    # decoded input with a file-size array is simply decoded input
    assert lib.mae_prep_workspace_bytes(C.byref(_prep_desc(file_sizes=FAKE))) == 256 + B * 32


def test_jpeg_row_index_sizes_and_argument_errors(lib):
    """32 bytes per 8 pixels of the side limit and file; only JPEG descriptors have an index; the
    index call checks its buffers before it touches the device."""
    B = 4
    for side, slot in ((0, 256), (500, 512)):
        d = _jpeg_desc(max_image_side=side)
        assert lib.mae_jpeg_index_bytes(C.byref(d)) == B * (slot // 8) * 32
    assert lib.mae_jpeg_index_bytes(C.byref(_prep_desc())) == 0      # decoded input
    assert lib.mae_jpeg_index_bytes(None) == 0
    d = _jpeg_desc()
    need, ws = lib.mae_jpeg_index_bytes(C.byref(d)), lib.mae_prep_workspace_bytes(C.byref(d))
    call = lambda desc, index=FAKE, nbytes=need, w=FAKE, wbytes=ws: lib.mae_jpeg_index(
        C.byref(desc), index, nbytes, w, wbytes, None)
    assert call(_prep_desc()) == binding.MAE_ERR_RANGE               # decoded input
    assert call(d, index=None) == binding.MAE_ERR_NULL
    assert call(d, w=None) == binding.MAE_ERR_NULL
    assert call(d, index=FAKE + 8) == binding.MAE_ERR_RANGE          # 16-byte alignment
    assert call(d, nbytes=need - 1) == binding.MAE_ERR_WORKSPACE
    assert call(d, wbytes=ws - 1) == binding.MAE_ERR_WORKSPACE
    # the index as an input: JPEG descriptors only, 16-byte aligned
    assert _call_prep(lib, _prep_desc(jpeg_row_index=FAKE)) == binding.MAE_ERR_RANGE
    assert _call_prep(lib, _jpeg_desc(jpeg_row_index=FAKE + 8, jpeg_row_index_bytes=need),
                      ws_bytes=1 << 30) == binding.MAE_ERR_RANGE
    # ... and as large as the descriptor's side limit makes it
    assert _call_prep(lib, _jpeg_desc(jpeg_row_index=FAKE, jpeg_row_index_bytes=need - 1),
                      ws_bytes=1 << 30) == binding.MAE_ERR_WORKSPACE
    assert _call_prep(lib, _jpeg_desc(jpeg_row_index=FAKE, jpeg_row_index_bytes=need,
                                      max_image_side=500), ws_bytes=1 << 32) == binding.MAE_ERR_WORKSPACE


def test_prep_rejects_bad_buffers(lib):
    d = _prep_desc()
    need = lib.mae_prep_workspace_bytes(C.byref(d))
    assert need == 256 + 4 * 32
    assert lib.mae_prep_batch(None, FAKE, FAKE, FAKE, None, None, None, FAKE, 1 << 20,
                              None) == binding.MAE_ERR_NULL
    assert _call_prep(lib, d, visible=None) == binding.MAE_ERR_NULL
    assert _call_prep(lib, d, mask=None) == binding.MAE_ERR_NULL
    assert _call_prep(lib, d, ids_restore=None) == binding.MAE_ERR_NULL
    assert _call_prep(lib, d, visible=FAKE + 4) == binding.MAE_ERR_RANGE        # 16-byte alignment
    assert _call_prep(lib, d, workspace=None) == binding.MAE_ERR_WORKSPACE
    assert _call_prep(lib, d, workspace=FAKE + 64) == binding.MAE_ERR_WORKSPACE  # 256-byte alignment
    assert _call_prep(lib, d, ws_bytes=need - 1) == binding.MAE_ERR_WORKSPACE


def _loss_desc(**over):
    d = binding.MaeLossDesc()
    d.B, d.L, d.D = 2, 196, 768
    d.pred = d.target = d.mask = FAKE
    d.num_masked, d.eps, d.grad_scale, d.pred_dtype = 294, 1e-6, 1.0, 0
    d.norm_pix = 1
    for k, v in over.items():
        setattr(d, k, v)
    return d


@pytest.mark.parametrize("over,status", [
    (dict(pred=None), binding.MAE_ERR_NULL),
    (dict(target=None), binding.MAE_ERR_NULL),
    (dict(mask=None), binding.MAE_ERR_NULL),
    (dict(B=0), binding.MAE_ERR_SHAPE),
    (dict(L=0), binding.MAE_ERR_SHAPE),
    (dict(D=1), binding.MAE_ERR_RANGE),
    (dict(D=4000), binding.MAE_ERR_RANGE),
    (dict(num_masked=-1), binding.MAE_ERR_RANGE),
    (dict(eps=-1.0), binding.MAE_ERR_RANGE),
    (dict(grad_scale=float("inf")), binding.MAE_ERR_RANGE),
    (dict(pred_dtype=2), binding.MAE_ERR_DTYPE),
    (dict(norm_pix=2), binding.MAE_ERR_RANGE),
])
def test_loss_rejects_bad_descriptors(lib, over, status):
    d = _loss_desc(**over)
    assert lib.mae_normpix_loss(C.byref(d), FAKE, FAKE, FAKE, 1 << 20, None) == status
    assert lib.mae_loss_workspace_bytes(C.byref(d)) == 0


def test_loss_rejects_bad_buffers(lib):
    d = _loss_desc()
    need = lib.mae_loss_workspace_bytes(C.byref(d))
    assert need > 0 and need % 8 == 0
    assert lib.mae_normpix_loss(C.byref(d), None, FAKE, FAKE, need, None) == binding.MAE_ERR_NULL
    assert lib.mae_normpix_loss(C.byref(d), FAKE, FAKE + 8, FAKE, need,
                                None) == binding.MAE_ERR_RANGE
    assert lib.mae_normpix_loss(C.byref(d), FAKE, FAKE, None, need,
                                None) == binding.MAE_ERR_WORKSPACE
    assert lib.mae_normpix_loss(C.byref(d), FAKE, FAKE, FAKE, need - 8,
                                None) == binding.MAE_ERR_WORKSPACE
    assert lib.mae_normpix_loss(None, FAKE, FAKE, FAKE, need, None) == binding.MAE_ERR_NULL


def _call_loss_from_images(lib, p, d, prep_ws=FAKE, loss=FAKE, grad=FAKE, ws=FAKE, ws_bytes=1 << 20,
                           prep_bytes=1 << 20):
    return lib.mae_normpix_loss_from_images(C.byref(p), prep_ws, prep_bytes, C.byref(d), loss,
                                            grad, ws, ws_bytes, None)


def test_loss_from_images_validates_both_descriptors(lib):
    p = _prep_desc(B=2)
    d = _loss_desc(target=None)                     # the target is not read
    need = lib.mae_loss_from_images_workspace_bytes(C.byref(p), C.byref(d))
    # a double per image and row of patches, + 128, + the mask's 256 partial counts
    assert need == (2 * 14 + 128) * 8 + 256 * 4
    assert _call_loss_from_images(lib, p, d, ws_bytes=need) == binding.MAE_ERR_NO_DEVICE
    assert _call_loss_from_images(lib, p, d, ws_bytes=need - 1) == binding.MAE_ERR_WORKSPACE
    assert _call_loss_from_images(lib, p, d, prep_ws=None) == binding.MAE_ERR_NULL
    assert _call_loss_from_images(lib, p, d, prep_ws=FAKE + 8) == binding.MAE_ERR_WORKSPACE
    assert _call_loss_from_images(lib, p, d, prep_bytes=256 + 2 * 32 - 1) == binding.MAE_ERR_WORKSPACE
    assert _call_loss_from_images(lib, p, d, loss=None) == binding.MAE_ERR_NULL
    assert _call_loss_from_images(lib, p, d, grad=FAKE + 4) == binding.MAE_ERR_RANGE
    assert _call_loss_from_images(lib, p, d, grad=None, ws_bytes=need) == binding.MAE_ERR_NO_DEVICE
    for bad_p, status in ((_prep_desc(B=3), binding.MAE_ERR_SHAPE),            # other batch
                          (_prep_desc(B=2, out_size=192, num_keep=36), binding.MAE_ERR_SHAPE),
                          (_prep_desc(B=2, aug_mode=1), binding.MAE_ERR_RANGE),   # finetuning mode
                          (_prep_desc(B=2, out_size=0), binding.MAE_ERR_SHAPE)):
        assert _call_loss_from_images(lib, bad_p, d) == status
        assert lib.mae_loss_from_images_workspace_bytes(C.byref(bad_p), C.byref(d)) == 0
    for over, status in ((dict(pred=None), binding.MAE_ERR_NULL), (dict(mask=None), binding.MAE_ERR_NULL),
                         (dict(D=588), binding.MAE_ERR_SHAPE), (dict(num_masked=-1), binding.MAE_ERR_RANGE),
                         (dict(pred_dtype=5), binding.MAE_ERR_DTYPE)):
        assert _call_loss_from_images(lib, p, _loss_desc(target=None, **over)) == status
    # an odd patch size has no 16-byte groups
    odd = _prep_desc(B=2, out_size=225, patch=15, num_keep=56)
    assert _call_loss_from_images(lib, odd, _loss_desc(target=None, L=225, D=675)) == \
        binding.MAE_ERR_SHAPE


def _embed_desc(**over):
    d = binding.MaeEmbedDesc()
    d.M, d.D, d.E, d.L = 196, 768, 768, 196
    d.visible = d.ids_keep = d.weight = d.bias = d.pos = FAKE
    d.out_dtype = binding.MAE_BF16
    for k, v in over.items():
        setattr(d, k, v)
    return d


@pytest.mark.parametrize("over,status", [
    (dict(visible=None), binding.MAE_ERR_NULL),
    (dict(weight=None), binding.MAE_ERR_NULL),
    (dict(ids_keep=None), binding.MAE_ERR_NULL),  # pos is given, so the indices are needed
    (dict(M=0), binding.MAE_ERR_SHAPE),
    (dict(E=0), binding.MAE_ERR_SHAPE),
    (dict(L=0), binding.MAE_ERR_SHAPE),
    (dict(D=0), binding.MAE_ERR_SHAPE),
    (dict(D=27), binding.MAE_ERR_SHAPE),  # 3 x 3 x 3: not a multiple of four values
    (dict(D=3076), binding.MAE_ERR_RANGE),
    (dict(E=8193), binding.MAE_ERR_RANGE),
    (dict(M=(1 << 28) + 1), binding.MAE_ERR_RANGE),
    (dict(out_dtype=2), binding.MAE_ERR_DTYPE),
    (dict(visible=FAKE + 8), binding.MAE_ERR_RANGE),
    (dict(weight=FAKE + 2), binding.MAE_ERR_RANGE),
    (dict(pos=FAKE + 4), binding.MAE_ERR_RANGE),
])
def test_embed_rejects_bad_descriptors(lib, over, status):
    d = _embed_desc(**over)
    assert lib.mae_patch_embed(C.byref(d), FAKE, None) == status


def test_embed_rejects_bad_buffers(lib):
    d = _embed_desc()
    assert lib.mae_patch_embed(C.byref(d), None, None) == binding.MAE_ERR_NULL
    assert lib.mae_patch_embed(C.byref(d), FAKE + 8, None) == binding.MAE_ERR_RANGE
    assert lib.mae_patch_embed(None, FAKE, None) == binding.MAE_ERR_NULL


@pytest.mark.skipif(torch.cuda.is_available(), reason="a GPU is visible")
def test_valid_calls_report_no_device_without_a_gpu(lib):
    # all arguments pass validation; with no device nothing is launched and nothing is read
    assert _call_prep(lib, _prep_desc()) == binding.MAE_ERR_NO_DEVICE
    d = _loss_desc()
    assert lib.mae_normpix_loss(C.byref(d), FAKE, FAKE, FAKE, 1 << 20,
                                None) == binding.MAE_ERR_NO_DEVICE
    e = _embed_desc()
    assert lib.mae_patch_embed(C.byref(e), FAKE, None) == binding.MAE_ERR_NO_DEVICE
    e = _embed_desc(pos=None, ids_keep=None, bias=None)  # both additions are optional
    assert lib.mae_patch_embed(C.byref(e), FAKE, None) == binding.MAE_ERR_NO_DEVICE
    n = C.c_int32(0)
    assert lib.mae_prep_status(FAKE, None, C.byref(n)) == binding.MAE_ERR_NO_DEVICE
    assert lib.mae_prep_status(None, None, C.byref(n)) == binding.MAE_ERR_NULL


def test_binding_does_not_fall_back_when_the_library_is_missing(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "libmae_hip.so"))
    with pytest.raises(FileNotFoundError):
        binding.load()


def test_progressive_tables_match_the_paper(lib, golden):
    for row in golden("progressive_schemes.txt"):
        if row[0] == "pretrain":
            assert mae.mae_pretrain_stage(int(row[1]), int(row[2])) == (int(row[3]), float(row[4]))
        elif row[0] == "finetune":
            scheme = {"1": mae.MAE_FINETUNE_SCHEME_1, "3": mae.MAE_FINETUNE_SCHEME_3,
                      "1-": mae.MAE_FINETUNE_SCHEME_1_MINUS,
                      "1+": mae.MAE_FINETUNE_SCHEME_1_PLUS}[row[1]]
            res, lo, hi, aug = mae.mae_finetune_stage(scheme, int(row[2]))
            assert res == int(row[3])
            assert lo == pytest.approx(float(row[4]) ** 2, rel=1e-6)
            assert hi == pytest.approx(float(row[5]) ** 2, rel=1e-6)
            assert aug == {"3Aug": mae.MAE_AUG_THREE, "3Aug+": mae.MAE_AUG_THREE_PLUS}[row[6]]
        elif row[0] == "lengths":
            lengths = [int(v) for v in row[1:]]
            for epoch in (0, 29, 30, 59, 60, 99, 100, 1000):
                assert mae.mae_stage_of_epoch(epoch, lengths) == oracle.stage_of_epoch(epoch,
                                                                                      lengths)
    for scheme in range(1, 7):
        for stage in (1, 2, 3):
            assert mae.mae_pretrain_stage(scheme, stage) == oracle.pretrain_stage(scheme, stage)
    for bad in ((0, 1), (7, 1), (1, 0), (1, 4)):
        with pytest.raises(mae.MaeError):
            mae.mae_pretrain_stage(*bad)
    with pytest.raises(mae.MaeError):
        mae.mae_finetune_stage(2, 1)
    with pytest.raises(mae.MaeError):
        mae.mae_stage_of_epoch(-1, [1, 2])
    assert mae.mae_stage_of_epoch(0, [0, 0, 5]) == 3


def test_binding_rejects_host_tensors_before_any_call():
    """The library takes raw device pointers: the binding refuses tensors it would misread."""
    import torch

    img = torch.zeros(100, dtype=torch.uint8)
    off = torch.zeros(1, dtype=torch.int64)
    hw = torch.ones(1, dtype=torch.int32)
    with pytest.raises(ValueError, match="device memory"):
        mae.make_prep_desc(img, off, hw, hw, out_size=32, patch=16, num_keep=1)
    with pytest.raises(TypeError, match="torch tensor"):
        mae.make_prep_desc(img.numpy(), off, hw, hw, out_size=32, patch=16, num_keep=1)
    pred = torch.zeros(1, 4, 12)
    with pytest.raises(ValueError, match="device memory"):
        mae.make_loss_desc(pred, pred, torch.zeros(1, 4, dtype=torch.uint8), num_masked=1)
    with pytest.raises(ValueError, match="device memory"):
        mae.make_embed_desc(pred.to(torch.bfloat16), None, pred[0].to(torch.bfloat16))
