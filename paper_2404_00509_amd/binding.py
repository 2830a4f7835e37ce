"""ctypes binding of ``libmae_hip.so`` -- argument marshalling only.

Every step of the path runs in the library's HIP kernels; PyTorch is used for device memory and
for the stream handle.  There is no CPU fallback: if the library is missing, or no GPU is visible,
the calls raise.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmae_hip.so")

MAE_OK = 0
MAE_ERR_NULL, MAE_ERR_SHAPE, MAE_ERR_RANGE, MAE_ERR_DTYPE = -1, -2, -3, -4
MAE_ERR_WORKSPACE, MAE_ERR_NO_DEVICE, MAE_ERR_HIP = -5, -6, -7
MAE_F32, MAE_BF16 = 0, 1
MAE_AUG_SIMPLE, MAE_AUG_THREE, MAE_AUG_THREE_PLUS = 0, 1, 2
MAE_INPUT_DECODED, MAE_INPUT_JPEG = 0, 1
MAE_FINETUNE_SCHEME_1, MAE_FINETUNE_SCHEME_3 = 1, 3
MAE_FINETUNE_SCHEME_1_MINUS, MAE_FINETUNE_SCHEME_1_PLUS = 10, 11

IMAGENET_MEAN = (0.485, 0.456, 0.406)
IMAGENET_STD = (0.229, 0.224, 0.225)

# Entry points declared in include/mae_hip.h.
EXPORTS = ("mae_prep_batch", "mae_prep_workspace_bytes", "mae_prep_status", "mae_num_keep",
           "mae_jpeg_index", "mae_jpeg_index_bytes",
           "mae_normpix_loss", "mae_loss_workspace_bytes", "mae_normpix_loss_static",
           "mae_normpix_loss_from_images",
           "mae_loss_from_images_workspace_bytes", "mae_patch_embed", "mae_pretrain_stage",
           "mae_finetune_stage", "mae_stage_of_epoch", "mae_error_string", "mae_version")


class MaePrepDesc(C.Structure):
    _fields_ = [
        ("B", C.c_int32),
        ("images", C.c_void_p),
        ("images_bytes", C.c_int64),
        ("offsets", C.c_void_p),
        ("heights", C.c_void_p),
        ("widths", C.c_void_p),
        ("out_size", C.c_int32),
        ("patch", C.c_int32),
        ("num_keep", C.c_int32),
        ("scale_lo", C.c_float),
        ("scale_hi", C.c_float),
        ("ratio_lo", C.c_float),
        ("ratio_hi", C.c_float),
        ("flip_p", C.c_float),
        ("mean", C.c_float * 3),
        ("std", C.c_float * 3),
        ("seed", C.c_uint64),
        ("batch_index", C.c_uint64),
        ("sample_base", C.c_uint32),
        ("noise_bits", C.c_int32),
        ("out_dtype", C.c_int32),
        ("max_image_side", C.c_int32),
        ("aug_mode", C.c_int32),
        ("jitter", C.c_float),
        ("input_format", C.c_int32),
        ("file_sizes", C.c_void_p),
        ("jpeg_row_index", C.c_void_p),
        ("jpeg_row_index_bytes", C.c_int64),
    ]


class MaeLossDesc(C.Structure):
    _fields_ = [
        ("B", C.c_int32),
        ("L", C.c_int32),
        ("D", C.c_int32),
        ("pred", C.c_void_p),
        ("target", C.c_void_p),
        ("mask", C.c_void_p),
        ("num_masked", C.c_int64),
        ("eps", C.c_float),
        ("grad_scale", C.c_float),
        ("pred_dtype", C.c_int32),
        ("norm_pix", C.c_int32),
    ]


class MaeEmbedDesc(C.Structure):
    _fields_ = [
        ("M", C.c_int64),
        ("D", C.c_int32),
        ("E", C.c_int32),
        ("L", C.c_int32),
        ("visible", C.c_void_p),
        ("ids_keep", C.c_void_p),
        ("weight", C.c_void_p),
        ("bias", C.c_void_p),
        ("pos", C.c_void_p),
        ("out_dtype", C.c_int32),
    ]


class MaeError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {mae_error_string(status)} (status {status})")


_lib = None


def load():
    """Load the shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2404_00509_amd.build`")
        lib = C.CDLL(LIB_PATH)
        lib.mae_prep_batch.restype = C.c_int
        lib.mae_prep_batch.argtypes = [C.POINTER(MaePrepDesc)] + [C.c_void_p] * 7 + [C.c_size_t,
                                                                                       C.c_void_p]
        lib.mae_prep_workspace_bytes.restype = C.c_size_t
        lib.mae_prep_workspace_bytes.argtypes = [C.POINTER(MaePrepDesc)]
        lib.mae_prep_status.restype = C.c_int
        lib.mae_prep_status.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_int32)]
        lib.mae_jpeg_index_bytes.restype = C.c_size_t
        lib.mae_jpeg_index_bytes.argtypes = [C.POINTER(MaePrepDesc)]
        lib.mae_jpeg_index.restype = C.c_int
        lib.mae_jpeg_index.argtypes = [C.POINTER(MaePrepDesc), C.c_void_p, C.c_size_t, C.c_void_p,
                                       C.c_size_t, C.c_void_p]
        lib.mae_num_keep.restype = C.c_int32
        lib.mae_num_keep.argtypes = [C.c_int32, C.c_double]
        lib.mae_normpix_loss.restype = C.c_int
        lib.mae_normpix_loss.argtypes = [C.POINTER(MaeLossDesc), C.c_void_p, C.c_void_p,
                                         C.c_void_p, C.c_size_t, C.c_void_p]
        lib.mae_loss_workspace_bytes.restype = C.c_size_t
        lib.mae_loss_workspace_bytes.argtypes = [C.POINTER(MaeLossDesc)]
        lib.mae_normpix_loss_static.restype = C.c_int
        lib.mae_normpix_loss_static.argtypes = [C.POINTER(MaeLossDesc), C.c_void_p, C.c_void_p,
                                                C.c_void_p]
        lib.mae_normpix_loss_from_images.restype = C.c_int
        lib.mae_normpix_loss_from_images.argtypes = [
            C.POINTER(MaePrepDesc), C.c_void_p, C.c_size_t, C.POINTER(MaeLossDesc), C.c_void_p,
            C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        lib.mae_loss_from_images_workspace_bytes.restype = C.c_size_t
        lib.mae_loss_from_images_workspace_bytes.argtypes = [C.POINTER(MaePrepDesc),
                                                             C.POINTER(MaeLossDesc)]
        lib.mae_patch_embed.restype = C.c_int
        lib.mae_patch_embed.argtypes = [C.POINTER(MaeEmbedDesc), C.c_void_p, C.c_void_p]
        lib.mae_pretrain_stage.restype = C.c_int
        lib.mae_pretrain_stage.argtypes = [C.c_int32, C.c_int32, C.POINTER(C.c_int32),
                                           C.POINTER(C.c_double)]
        lib.mae_finetune_stage.restype = C.c_int
        lib.mae_finetune_stage.argtypes = [C.c_int32, C.c_int32, C.POINTER(C.c_int32),
                                           C.POINTER(C.c_float), C.POINTER(C.c_float),
                                           C.POINTER(C.c_int32)]
        lib.mae_stage_of_epoch.restype = C.c_int
        lib.mae_stage_of_epoch.argtypes = [C.c_int32, C.POINTER(C.c_int32), C.c_int32]
        lib.mae_error_string.restype = C.c_char_p
        lib.mae_error_string.argtypes = [C.c_int]
        lib.mae_version.restype = C.c_int
        lib.mae_version.argtypes = []
        _lib = lib
    return _lib


def mae_error_string(status: int) -> str:
    return load().mae_error_string(status).decode()


def mae_version() -> int:
    return int(load().mae_version())


def mae_num_keep(L: int, mask_ratio: float) -> int:
    return int(load().mae_num_keep(L, mask_ratio))


def mae_pretrain_stage(scheme: int, stage: int):
    """-> (out_size, mask_ratio) of the paper's pretraining scheme / stage."""
    res, m = C.c_int32(), C.c_double()
    rc = load().mae_pretrain_stage(scheme, stage, C.byref(res), C.byref(m))
    if rc != MAE_OK:
        raise MaeError(rc, "mae_pretrain_stage")
    return res.value, m.value


def mae_finetune_stage(scheme: int, stage: int):
    """-> (out_size, scale_lo, scale_hi, aug_mode): area-fraction bounds and augmentation for
    mae_prep_desc.  scheme: MAE_FINETUNE_SCHEME_1, _3, _1_MINUS, _1_PLUS."""
    res, lo, hi, aug = C.c_int32(), C.c_float(), C.c_float(), C.c_int32()
    rc = load().mae_finetune_stage(scheme, stage, C.byref(res), C.byref(lo), C.byref(hi),
                                   C.byref(aug))
    if rc != MAE_OK:
        raise MaeError(rc, "mae_finetune_stage")
    return res.value, lo.value, hi.value, aug.value


def mae_stage_of_epoch(epoch: int, lengths) -> int:
    arr = (C.c_int32 * len(lengths))(*lengths)
    rc = load().mae_stage_of_epoch(epoch, arr, len(lengths))
    if rc < 0:
        raise MaeError(rc, "mae_stage_of_epoch")
    return rc


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _check(t, name, dtypes=None, numel=None, optional=False):
    """Marshalling checks: the library reads raw device pointers, so a tensor of the wrong type,
    on the host, or with gaps would be read past its end."""
    if t is None:
        if optional:
            return
        raise TypeError(f"{name} is required")
    if not isinstance(t, torch.Tensor):
        raise TypeError(f"{name} must be a torch tensor")
    if not t.is_cuda:
        raise ValueError(f"{name} must live in device memory")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtypes is not None and t.dtype not in (dtypes if isinstance(dtypes, tuple) else (dtypes,)):
        raise TypeError(f"{name} has dtype {t.dtype}, expected {dtypes}")
    if numel is not None and t.numel() < numel:
        raise ValueError(f"{name} holds {t.numel()} elements, {numel} are needed")


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def make_prep_desc(images, offsets, heights, widths, *, out_size, patch, num_keep,
                   scale=(0.2, 1.0), ratio=(3.0 / 4.0, 4.0 / 3.0), flip_p=0.5, mean=IMAGENET_MEAN,
                   std=IMAGENET_STD, seed=0, batch_index=0, sample_base=0, noise_bits=32,
                   out_dtype=MAE_F32, max_image_side=0, aug_mode=0, jitter=0.3,
                   file_sizes=None, row_index=None) -> MaePrepDesc:
    """Decoded input: images / offsets / heights / widths as device tensors.  JPEG input ("crop
    decode"): images = the files back to back, offsets = their starts, file_sizes = their lengths
    (int32); heights and widths are then ignored (pass None).  row_index: what mae_jpeg_index
    wrote for these files with the same max_image_side (uint8 tensor), or None."""
    _check(images, "images", torch.uint8)
    _check(offsets, "offsets", torch.int64)
    if file_sizes is None:
        _check(heights, "heights", torch.int32)
        _check(widths, "widths", torch.int32, numel=heights.numel())
        _check(offsets, "offsets", torch.int64, numel=heights.numel())
    else:
        _check(file_sizes, "file_sizes", torch.int32)
        _check(offsets, "offsets", torch.int64, numel=file_sizes.numel())
    d = MaePrepDesc()
    d.images = images.data_ptr()
    d.images_bytes = int(images.numel())
    d.offsets = offsets.data_ptr()
    if file_sizes is None:
        d.B = int(heights.numel())
        d.heights, d.widths = heights.data_ptr(), widths.data_ptr()
        d.input_format = MAE_INPUT_DECODED
    else:
        d.B = int(file_sizes.numel())
        d.file_sizes = file_sizes.data_ptr()
        d.input_format = MAE_INPUT_JPEG
    d.out_size, d.patch, d.num_keep = out_size, patch, num_keep
    d.scale_lo, d.scale_hi = scale
    d.ratio_lo, d.ratio_hi = ratio
    d.flip_p = flip_p
    d.mean = (C.c_float * 3)(*mean)
    d.std = (C.c_float * 3)(*std)
    d.seed, d.batch_index, d.sample_base = seed, batch_index, sample_base
    d.noise_bits, d.out_dtype = noise_bits, out_dtype
    d.max_image_side = max_image_side
    d.aug_mode, d.jitter = aug_mode, jitter
    if row_index is not None:
        if file_sizes is None:
            raise ValueError("row_index goes with JPEG input (file_sizes)")
        _check(row_index, "row_index", torch.uint8, numel=mae_jpeg_index_bytes(d))
        d.jpeg_row_index = row_index.data_ptr()
        d.jpeg_row_index_bytes = int(row_index.numel())
    return d


def mae_jpeg_index_bytes(desc: MaePrepDesc) -> int:
    return int(load().mae_jpeg_index_bytes(C.byref(desc)))


def mae_jpeg_index(desc: MaePrepDesc, index, workspace, stream=None) -> None:
    """Enqueue the computation of the row index of the descriptor's JPEG files into `index`
    (uint8 device tensor of mae_jpeg_index_bytes(desc) bytes)."""
    _check(index, "index", torch.uint8, numel=mae_jpeg_index_bytes(desc))
    _check(workspace, "workspace")
    rc = load().mae_jpeg_index(C.byref(desc), _ptr(index), index.numel(), _ptr(workspace),
                               workspace.numel() * workspace.element_size(), _stream(stream))
    if rc != MAE_OK:
        raise MaeError(rc, "mae_jpeg_index")


def mae_prep_workspace_bytes(desc: MaePrepDesc) -> int:
    return int(load().mae_prep_workspace_bytes(C.byref(desc)))


def mae_prep_batch(desc: MaePrepDesc, visible, mask, ids_restore, ids_keep=None, target=None,
                   crop_out=None, workspace=None, stream=None) -> None:
    """Enqueue the input pipeline; all tensors are preallocated device tensors."""
    B, p, K = desc.B, max(desc.patch, 1), desc.num_keep
    L, D = (desc.out_size // p) ** 2, 3 * p * p
    _check(visible, "visible", torch.bfloat16 if desc.out_dtype == MAE_BF16 else torch.float32,
           numel=B * K * D)
    _check(mask, "mask", torch.uint8, numel=B * L)
    _check(ids_restore, "ids_restore", torch.int32, numel=B * L)
    _check(ids_keep, "ids_keep", torch.int32, numel=B * K, optional=True)
    _check(target, "target", torch.float32, numel=B * L * D, optional=True)
    _check(crop_out, "crop_out", torch.int32, numel=B * 6, optional=True)
    _check(workspace, "workspace", optional=True)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = load().mae_prep_batch(C.byref(desc), _ptr(visible), _ptr(mask), _ptr(ids_restore),
                               _ptr(ids_keep), _ptr(target), _ptr(crop_out), _ptr(workspace),
                               ws_bytes, _stream(stream))
    if rc != MAE_OK:
        raise MaeError(rc, "mae_prep_batch")


def mae_prep_status(workspace, stream=None) -> int:
    """Synchronises; number of samples the device-side geometry check rejected."""
    n = C.c_int32(-1)
    rc = load().mae_prep_status(_ptr(workspace), _stream(stream), C.byref(n))
    if rc != MAE_OK:
        raise MaeError(rc, "mae_prep_status")
    return n.value


def make_loss_desc(pred, target, mask, *, num_masked, eps=1e-6, grad_scale=1.0,
                   norm_pix=True) -> MaeLossDesc:
    """target may be None for mae_normpix_loss_from_images."""
    _check(pred, "pred", (torch.float32, torch.bfloat16))
    if pred.dim() != 3:
        raise ValueError("pred must have shape [B, L, D]")
    _check(target, "target", torch.float32, numel=pred.numel(), optional=True)
    _check(mask, "mask", torch.uint8, numel=pred.shape[0] * pred.shape[1])
    d = MaeLossDesc()
    d.B, d.L, d.D = (int(v) for v in pred.shape)
    d.pred, d.target, d.mask = pred.data_ptr(), _ptr(target), mask.data_ptr()
    d.num_masked = int(num_masked)
    d.eps, d.grad_scale = eps, grad_scale
    d.pred_dtype = MAE_BF16 if pred.dtype == torch.bfloat16 else MAE_F32
    d.norm_pix = 1 if norm_pix else 0
    return d


def mae_loss_workspace_bytes(desc: MaeLossDesc) -> int:
    return int(load().mae_loss_workspace_bytes(C.byref(desc)))


def _check_loss_outputs(desc, loss, grad):
    _check(loss, "loss", torch.float32, numel=1)
    _check(grad, "grad", torch.bfloat16 if desc.pred_dtype == MAE_BF16 else torch.float32,
           numel=desc.B * desc.L * desc.D, optional=True)


def mae_normpix_loss(desc: MaeLossDesc, loss, grad=None, workspace=None, stream=None) -> None:
    _check_loss_outputs(desc, loss, grad)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = load().mae_normpix_loss(C.byref(desc), _ptr(loss), _ptr(grad), _ptr(workspace), ws_bytes,
                                 _stream(stream))
    if rc != MAE_OK:
        raise MaeError(rc, "mae_normpix_loss")


def mae_normpix_loss_static(desc: MaeLossDesc, loss, grad=None, stream=None) -> None:
    """mae_normpix_loss without a workspace (the library's own fixed scratch array is used)."""
    _check_loss_outputs(desc, loss, grad)
    rc = load().mae_normpix_loss_static(C.byref(desc), _ptr(loss), _ptr(grad), _stream(stream))
    if rc != MAE_OK:
        raise MaeError(rc, "mae_normpix_loss_static")


def mae_loss_from_images_workspace_bytes(prep: MaePrepDesc, desc: MaeLossDesc) -> int:
    return int(load().mae_loss_from_images_workspace_bytes(C.byref(prep), C.byref(desc)))


def mae_normpix_loss_from_images(prep: MaePrepDesc, prep_workspace, desc: MaeLossDesc, loss,
                                 grad=None, workspace=None, stream=None) -> None:
    _check_loss_outputs(desc, loss, grad)
    _check(prep_workspace, "prep_workspace")
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    prep_bytes = prep_workspace.numel() * prep_workspace.element_size()
    rc = load().mae_normpix_loss_from_images(C.byref(prep), _ptr(prep_workspace), prep_bytes,
                                             C.byref(desc), _ptr(loss), _ptr(grad),
                                             _ptr(workspace), ws_bytes, _stream(stream))
    if rc != MAE_OK:
        raise MaeError(rc, "mae_normpix_loss_from_images")


def make_embed_desc(visible, ids_keep, weight, bias=None, pos=None, *,
                    out_dtype=MAE_BF16) -> MaeEmbedDesc:
    """visible [B, K, D] (or [M, D]) bf16, ids_keep [B, K] int32, weight [E, D] bf16,
    bias [E] float32, pos [L, E] float32."""
    _check(visible, "visible", torch.bfloat16)
    _check(weight, "weight", torch.bfloat16)
    if weight.dim() != 2 or weight.shape[1] != visible.shape[-1]:
        raise ValueError("weight must have shape [E, D] with D = visible.shape[-1]")
    rows = visible.numel() // int(visible.shape[-1])
    _check(ids_keep, "ids_keep", torch.int32, numel=rows, optional=pos is None)
    _check(bias, "bias", torch.float32, numel=int(weight.shape[0]), optional=True)
    _check(pos, "pos", torch.float32, optional=True)
    if pos is not None and (pos.dim() != 2 or pos.shape[1] != weight.shape[0]):
        raise ValueError("pos must have shape [L, E]")
    d = MaeEmbedDesc()
    d.D, d.E = int(visible.shape[-1]), int(weight.shape[0])
    d.M = visible.numel() // d.D
    d.L = int(pos.shape[0]) if pos is not None else 1
    d.visible, d.weight = visible.data_ptr(), weight.data_ptr()
    d.ids_keep, d.bias, d.pos = _ptr(ids_keep), _ptr(bias), _ptr(pos)
    d.out_dtype = out_dtype
    return d


def mae_patch_embed(desc: MaeEmbedDesc, tokens, stream=None) -> None:
    _check(tokens, "tokens", torch.bfloat16 if desc.out_dtype == MAE_BF16 else torch.float32,
           numel=desc.M * desc.E)
    rc = load().mae_patch_embed(C.byref(desc), _ptr(tokens), _stream(stream))
    if rc != MAE_OK:
        raise MaeError(rc, "mae_patch_embed")


# ------------------------------------------------------------------------------------------------
# Preallocated buffers for one workload: device memory only, no arithmetic.
# ------------------------------------------------------------------------------------------------
@dataclass
class PrepBuffers:
    visible: torch.Tensor
    mask: torch.Tensor
    ids_restore: torch.Tensor
    ids_keep: torch.Tensor
    target: torch.Tensor
    crop: torch.Tensor
    workspace: torch.Tensor


def alloc_prep_buffers(desc: MaePrepDesc, device="cuda", want_target=True) -> PrepBuffers:
    B, p, K = desc.B, desc.patch, desc.num_keep
    G = desc.out_size // p
    L, D = G * G, 3 * p * p
    vis_dtype = torch.bfloat16 if desc.out_dtype == MAE_BF16 else torch.float32
    ws = max(mae_prep_workspace_bytes(desc), 256)
    return PrepBuffers(
        visible=torch.empty((B, K, D), dtype=vis_dtype, device=device),
        mask=torch.empty((B, L), dtype=torch.uint8, device=device),
        ids_restore=torch.empty((B, L), dtype=torch.int32, device=device),
        ids_keep=torch.empty((B, K), dtype=torch.int32, device=device),
        target=torch.empty((B, L, D), dtype=torch.float32, device=device) if want_target else None,
        crop=torch.empty((B, 6), dtype=torch.int32, device=device),
        workspace=torch.empty(ws, dtype=torch.uint8, device=device),
    )


class ProgressiveBuffers:
    """Device buffers allocated once for the largest stage of a progressive schedule (Sec. 5.2,
    5.3: the resolution and the masking ratio change between stages).  `stage(i)` returns views of
    the same storage shaped for stage i, so a stage switch allocates nothing."""

    def __init__(self, B, patch, stages, device="cuda", bf16=False, want_target=True,
                 aug_mode=MAE_AUG_SIMPLE, max_image_side=0, jpeg=False):
        """aug_mode, max_image_side, jpeg: the most demanding values any stage will be called
        with (they size the workspace)."""
        self.B, self.patch, self.bf16 = B, patch, bf16
        self.shapes = []
        for out_size, mask_ratio in stages:
            G = out_size // patch
            L = G * G
            self.shapes.append((out_size, L, mae_num_keep(L, mask_ratio), 3 * patch * patch))
        max_l = max(s[1] for s in self.shapes)
        max_k = max(s[2] for s in self.shapes)
        D = self.shapes[0][3]
        vis_dtype = torch.bfloat16 if bf16 else torch.float32
        self._visible = torch.empty(B * max_k * D, dtype=vis_dtype, device=device)
        self._mask = torch.empty(B * max_l, dtype=torch.uint8, device=device)
        self._ids_restore = torch.empty(B * max_l, dtype=torch.int32, device=device)
        self._ids_keep = torch.empty(B * max_k, dtype=torch.int32, device=device)
        self._target = (torch.empty(B * max_l * D, dtype=torch.float32, device=device)
                        if want_target else None)
        self._crop = torch.empty((B, 6), dtype=torch.int32, device=device)
        # the workspace of the most demanding stage, as the library sizes it (the pointers of the
        # descriptor are not looked at for that)
        need = 0
        for out_size, _, num_keep, _ in self.shapes:
            d = MaePrepDesc()
            d.B, d.out_size, d.patch, d.num_keep = B, out_size, patch, num_keep
            d.images = d.offsets = d.heights = d.widths = d.file_sizes = 8
            d.images_bytes = 1
            d.scale_lo, d.scale_hi, d.ratio_lo, d.ratio_hi, d.flip_p = 0.2, 1.0, 0.75, 4.0 / 3.0, 0.5
            d.mean = (C.c_float * 3)(*IMAGENET_MEAN)
            d.std = (C.c_float * 3)(*IMAGENET_STD)
            d.noise_bits = 32
            d.out_dtype = MAE_BF16 if bf16 else MAE_F32
            d.max_image_side = max_image_side
            d.aug_mode, d.jitter = aug_mode, 0.3
            d.input_format = MAE_INPUT_JPEG if jpeg else MAE_INPUT_DECODED
            size = mae_prep_workspace_bytes(d)
            if size == 0:
                raise ValueError(f"stage {out_size}px / keep {num_keep} is not a valid descriptor")
            need = max(need, size)
        self._workspace = torch.empty(need, dtype=torch.uint8, device=device)

    def stage(self, i) -> PrepBuffers:
        out_size, L, K, D = self.shapes[i]
        B = self.B
        return PrepBuffers(
            visible=self._visible[:B * K * D].view(B, K, D),
            mask=self._mask[:B * L].view(B, L),
            ids_restore=self._ids_restore[:B * L].view(B, L),
            ids_keep=self._ids_keep[:B * K].view(B, K),
            target=None if self._target is None else self._target[:B * L * D].view(B, L, D),
            crop=self._crop,
            workspace=self._workspace,
        )
