"""ctypes access to the CPU oracle (``mae_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the benchmark's CPU
baseline leg.  The GPU library and its Python binding never import this package, and this package
never imports them.  All arrays are NumPy host arrays.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mae_oracle.c")
_LIB = os.path.join(_HERE, "libmae_oracle.so")

IMAGENET_MEAN = (0.485, 0.456, 0.406)
IMAGENET_STD = (0.229, 0.224, 0.225)


def compile_source(src: str, out: str) -> str:
    """gcc, plain -O2, no contraction, OpenMP over samples / rows only."""
    cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared",
           "-Wall", "-Wextra", "-I", _HERE, "-o", out, src, "-lm"]
    subprocess.run(cmd, check=True, cwd=_HERE)
    return out


def build(force: bool = False) -> str:
    """Compile the oracle if it is missing or older than its source."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        compile_source(_SRC, _LIB)
    return _LIB


class _PrepArgs(C.Structure):
    _fields_ = [
        ("B", C.c_int32),
        ("images", C.c_void_p),
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
        ("noise_bits", C.c_int32),
        ("aug_mode", C.c_int32),
        ("jitter", C.c_float),
        ("images_bytes", C.c_int64),
    ]


_lib = None


def load_library(path: str):
    """Open an oracle shared library and declare its signatures (also used by the tests that
    plant mistakes in a copy of the source)."""
    L = C.CDLL(path)
    L.mae_oracle_mix64.restype = C.c_uint64
    L.mae_oracle_mix64.argtypes = [C.c_uint64]
    L.mae_oracle_draw.restype = C.c_uint64
    L.mae_oracle_draw.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32]
    L.mae_oracle_exp_poly.restype = C.c_double
    L.mae_oracle_exp_poly.argtypes = [C.c_double]
    rrc = [C.c_int32, C.c_int32, C.c_float, C.c_float, C.c_float, C.c_float, C.c_uint64,
           C.c_uint64, C.c_uint32]
    L.mae_oracle_rrc_proposal.restype = None
    L.mae_oracle_rrc_proposal.argtypes = rrc + [C.c_int32, C.c_void_p]
    L.mae_oracle_rrc_params.restype = C.c_int32
    L.mae_oracle_rrc_params.argtypes = rrc + [C.c_void_p]
    L.mae_oracle_flip_bit.restype = C.c_int32
    L.mae_oracle_flip_bit.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, C.c_float]
    L.mae_oracle_resize_taps.restype = None
    L.mae_oracle_resize_taps.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                         C.c_void_p, C.c_void_p]
    L.mae_oracle_crop_resize.restype = None
    L.mae_oracle_crop_resize.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p,
                                         C.c_int32, C.c_int32, C.c_void_p]
    L.mae_oracle_normalise.restype = C.c_double
    L.mae_oracle_normalise.argtypes = [C.c_double, C.c_double, C.c_double]
    L.mae_oracle_patchify.restype = None
    L.mae_oracle_patchify.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
    L.mae_oracle_num_keep.restype = C.c_int32
    L.mae_oracle_num_keep.argtypes = [C.c_int32, C.c_double]
    L.mae_oracle_mask.restype = None
    L.mae_oracle_mask.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, C.c_int32, C.c_int32,
                                  C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
    L.mae_oracle_resize_u8.restype = None
    L.mae_oracle_resize_u8.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_int32,
                                       C.c_int32, C.c_void_p]
    L.mae_oracle_aug_params.restype = None
    L.mae_oracle_aug_params.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, C.c_double,
                                        C.c_void_p, C.c_void_p, C.c_void_p]
    L.mae_oracle_gray.restype = C.c_int32
    L.mae_oracle_gray.argtypes = [C.c_int32] * 3
    L.mae_oracle_solarise.restype = C.c_int32
    L.mae_oracle_solarise.argtypes = [C.c_int32]
    L.mae_oracle_blur_weights.restype = C.c_int32
    L.mae_oracle_blur_weights.argtypes = [C.c_double, C.c_void_p]
    L.mae_oracle_three_aug.restype = None
    L.mae_oracle_three_aug.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_double, C.c_void_p]
    L.mae_oracle_color_jitter.restype = None
    L.mae_oracle_color_jitter.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
    L.mae_oracle_prep_batch.restype = C.c_int32
    L.mae_oracle_prep_batch.argtypes = [C.c_void_p, C.c_int32, C.c_int32] + [C.c_void_p] * 7
    L.mae_oracle_normpix_loss.restype = C.c_int32
    L.mae_oracle_normpix_loss.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                          C.c_void_p, C.c_void_p, C.c_int64, C.c_double,
                                          C.c_double, C.c_void_p, C.c_void_p, C.c_void_p]
    L.mae_oracle_pixel_loss.restype = C.c_int32
    L.mae_oracle_pixel_loss.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                        C.c_void_p, C.c_int64, C.c_double, C.c_void_p, C.c_void_p]
    L.mae_oracle_pretrain_stage.restype = C.c_int32
    L.mae_oracle_pretrain_stage.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    L.mae_oracle_finetune_stage.restype = C.c_int32
    L.mae_oracle_finetune_stage.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                            C.c_void_p, C.c_void_p]
    L.mae_oracle_stage_of_epoch.restype = C.c_int32
    L.mae_oracle_stage_of_epoch.argtypes = [C.c_int32, C.c_void_p, C.c_int32]
    L.mae_oracle_patch_embed.restype = C.c_int32
    L.mae_oracle_patch_embed.argtypes = [C.c_int32] * 5 + [C.c_void_p] * 6
    L.mae_oracle_jpeg_info.restype = C.c_int32
    L.mae_oracle_jpeg_info.argtypes = [C.c_void_p, C.c_int64] + [C.c_void_p] * 5
    L.mae_oracle_jpeg_decode.restype = C.c_int32
    L.mae_oracle_jpeg_decode.argtypes = [C.c_void_p, C.c_int64, C.c_void_p]
    L.mae_oracle_jpeg_decode_ycc.restype = C.c_int32
    L.mae_oracle_jpeg_decode_ycc.argtypes = [C.c_void_p, C.c_int64, C.c_void_p]
    L.mae_oracle_idct8x8.restype = None
    L.mae_oracle_idct8x8.argtypes = [C.c_void_p, C.c_void_p]
    L.mae_oracle_ycc_to_rgb.restype = None
    L.mae_oracle_ycc_to_rgb.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_void_p]
    L.mae_oracle_huff_codes.restype = C.c_int32
    L.mae_oracle_huff_codes.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
    L.mae_oracle_threads.restype = C.c_int32
    L.mae_oracle_threads.argtypes = []
    L.mae_oracle_set_threads.restype = None
    L.mae_oracle_set_threads.argtypes = [C.c_int32]
    return L


def lib():
    global _lib
    if _lib is None:
        _lib = load_library(build())
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


# ---------------------------------------------------------------------------- scalar pieces
def mix64(z: int) -> int:
    return int(lib().mae_oracle_mix64(z & 0xFFFFFFFFFFFFFFFF))


def draw(seed: int, batch_index: int, sample: int, stream: int, ctr: int) -> int:
    return int(lib().mae_oracle_draw(seed, batch_index, sample, stream, ctr))


def exp_poly(x: float) -> float:
    return float(lib().mae_oracle_exp_poly(x))


def rrc_proposal(H, W, scale, ratio, seed, batch_index, sample, attempt):
    out = np.zeros(2, np.int64)
    lib().mae_oracle_rrc_proposal(H, W, scale[0], scale[1], ratio[0], ratio[1], seed, batch_index,
                                  sample, attempt, _p(out))
    return int(out[0]), int(out[1])  # ch, cw


def rrc_params(H, W, scale, ratio, seed, batch_index, sample):
    """-> ((top, left, ch, cw), attempts) ; attempts == 11 means the fallback box."""
    box = np.zeros(4, np.int32)
    n = lib().mae_oracle_rrc_params(H, W, scale[0], scale[1], ratio[0], ratio[1], seed,
                                    batch_index, sample, _p(box))
    return tuple(int(v) for v in box), int(n)


def flip_bit(seed, batch_index, sample, flip_p) -> int:
    return int(lib().mae_oracle_flip_bit(seed, batch_index, sample, flip_p))


def resize_taps(out_size, crop_len, o):
    i0, i1, f = C.c_int32(), C.c_int32(), C.c_double()
    lib().mae_oracle_resize_taps(out_size, crop_len, o, C.byref(i0), C.byref(i1), C.byref(f))
    return i0.value, i1.value, f.value


def crop_resize(img: np.ndarray, box, S: int, flip: int) -> np.ndarray:
    """img [H,W,3] uint8 -> [S,S,3] float64 in pixel units."""
    img = np.ascontiguousarray(img, np.uint8)
    H, W, ch = img.shape
    assert ch == 3
    b = np.asarray(box, np.int32)
    out = np.empty((S, S, 3), np.float64)
    lib().mae_oracle_crop_resize(_p(img), H, W, _p(b), S, int(flip), _p(out))
    return out


def resize_u8(img: np.ndarray, box, S: int, flip: int) -> np.ndarray:
    """img [H,W,3] uint8 -> [S,S,3] uint8: the bilinear value rounded to nearest, ties up."""
    img = np.ascontiguousarray(img, np.uint8)
    H, W, ch = img.shape
    assert ch == 3
    b = np.asarray(box, np.int32)
    out = np.empty((S, S, 3), np.uint8)
    lib().mae_oracle_resize_u8(_p(img), H, W, _p(b), S, int(flip), _p(out))
    return out


AUG_SIMPLE, AUG_THREE, AUG_THREE_PLUS = 0, 1, 2
OP_GRAY, OP_SOLARISE, OP_BLUR = 0, 1, 2


def aug_params(seed, batch_index, sample, jitter=0.3):
    """-> (op, sigma, (brightness, contrast, saturation))."""
    op = C.c_int32()
    sigma = C.c_double()
    bcs = np.empty(3, np.float64)
    lib().mae_oracle_aug_params(seed, batch_index, sample, jitter, C.byref(op), C.byref(sigma),
                                _p(bcs))
    return op.value, sigma.value, tuple(float(v) for v in bcs)


def gray(r: int, g: int, b: int) -> int:
    return int(lib().mae_oracle_gray(r, g, b))


def solarise(v: int) -> int:
    return int(lib().mae_oracle_solarise(v))


def blur_weights(sigma: float) -> np.ndarray:
    w = np.zeros(13, np.float64)
    r = lib().mae_oracle_blur_weights(sigma, _p(w))
    return w[:2 * r + 1].copy()


def three_aug(u8: np.ndarray, op: int, sigma: float = 1.0) -> np.ndarray:
    """u8 [S,S,3] uint8 -> [S,S,3] float64 in pixel units."""
    u8 = np.ascontiguousarray(u8, np.uint8)
    S = u8.shape[0]
    assert u8.shape == (S, S, 3)
    out = np.empty((S, S, 3), np.float64)
    lib().mae_oracle_three_aug(_p(u8), S, op, sigma, _p(out))
    return out


def color_jitter(img: np.ndarray, bcs) -> np.ndarray:
    out = np.ascontiguousarray(img, np.float64).copy()
    S = out.shape[0]
    assert out.shape == (S, S, 3)
    f = np.asarray(bcs, np.float64)
    lib().mae_oracle_color_jitter(_p(out), S, _p(f))
    return out


def normalise(v: float, mean: float, std: float) -> float:
    return float(lib().mae_oracle_normalise(v, mean, std))


def patchify(img: np.ndarray, p: int) -> np.ndarray:
    img = np.ascontiguousarray(img, np.float64)
    S = img.shape[0]
    assert img.shape == (S, S, 3) and S % p == 0
    out = np.empty(((S // p) ** 2, 3 * p * p), np.float64)
    lib().mae_oracle_patchify(_p(img), S, p, _p(out))
    return out


def num_keep(L: int, mask_ratio: float) -> int:
    return int(lib().mae_oracle_num_keep(L, mask_ratio))


def mask(seed, batch_index, sample, L, K, noise_bits=32):
    ids_restore = np.empty(L, np.int32)
    ids_keep = np.empty(K, np.int32)
    m = np.empty(L, np.uint8)
    lib().mae_oracle_mask(seed, batch_index, sample, L, K, noise_bits, _p(ids_restore),
                          _p(ids_keep), _p(m))
    return ids_restore, ids_keep, m


# ---------------------------------------------------------------------------- whole path
def prep_batch(images, offsets, heights, widths, *, out_size, patch, num_keep, scale=(0.2, 1.0),
               ratio=(3.0 / 4.0, 4.0 / 3.0), flip_p=0.5, mean=IMAGENET_MEAN, std=IMAGENET_STD,
               seed=0, batch_index=0, noise_bits=32, b_begin=0, b_end=None, want_target=True,
               want_visible=True, aug_mode=0, jitter=0.3):
    """Run the oracle pipeline on samples [b_begin, b_end).  Returns a dict of NumPy arrays."""
    images = np.ascontiguousarray(images, np.uint8)
    offsets = np.ascontiguousarray(offsets, np.int64)
    heights = np.ascontiguousarray(heights, np.int32)
    widths = np.ascontiguousarray(widths, np.int32)
    B = int(heights.shape[0])
    if b_end is None:
        b_end = B
    n = b_end - b_begin
    G = out_size // patch
    Lp = G * G
    D = 3 * patch * patch
    a = _PrepArgs()
    a.B = B
    a.images, a.offsets = images.ctypes.data, offsets.ctypes.data
    a.heights, a.widths = heights.ctypes.data, widths.ctypes.data
    a.out_size, a.patch, a.num_keep = out_size, patch, num_keep
    a.scale_lo, a.scale_hi = scale
    a.ratio_lo, a.ratio_hi = ratio
    a.flip_p = flip_p
    a.mean = (C.c_float * 3)(*mean)
    a.std = (C.c_float * 3)(*std)
    a.seed, a.batch_index, a.noise_bits = seed, batch_index, noise_bits
    a.aug_mode, a.jitter = aug_mode, jitter
    a.images_bytes = int(images.size)
    out = {
        "visible": np.empty((n, num_keep, D), np.float32) if want_visible else None,
        "mask": np.empty((n, Lp), np.uint8),
        "ids_restore": np.empty((n, Lp), np.int32),
        "ids_keep": np.empty((n, num_keep), np.int32),
        "target": np.empty((n, Lp, D), np.float32) if want_target else None,
        "crop": np.empty((n, 5), np.int32),
        "valid": np.empty((n,), np.uint8),
    }
    rc = lib().mae_oracle_prep_batch(C.byref(a), b_begin, b_end, _p(out["visible"]),
                                     _p(out["mask"]), _p(out["ids_restore"]), _p(out["ids_keep"]),
                                     _p(out["target"]), _p(out["crop"]), _p(out["valid"]))
    if rc != 0:
        raise ValueError("mae_oracle_prep_batch: invalid argument")
    return out


def normpix_loss(pred, target, mask, num_masked=None, eps=1e-6, grad_scale=1.0, want_grad=True,
                 want_that=False):
    """-> (loss float64, grad fp32 [B,L,D] or None, that float64 or None)."""
    pred = np.ascontiguousarray(pred, np.float32)
    target = np.ascontiguousarray(target, np.float32)
    mask = np.ascontiguousarray(mask, np.uint8)
    B, L, D = pred.shape
    assert target.shape == (B, L, D) and mask.shape == (B, L)
    if num_masked is None:
        num_masked = int(mask.astype(np.int64).sum())
    loss = C.c_double()
    grad = np.empty((B, L, D), np.float32) if want_grad else None
    that = np.empty((B, L, D), np.float64) if want_that else None
    rc = lib().mae_oracle_normpix_loss(B, L, D, _p(pred), _p(target), _p(mask), num_masked, eps,
                                       grad_scale, C.byref(loss), _p(grad), _p(that))
    if rc != 0:
        raise ValueError("mae_oracle_normpix_loss: invalid argument")
    return loss.value, grad, that


def pixel_loss(pred, target, mask, num_masked=None, grad_scale=1.0, want_grad=True):
    """Un-normalised variant: -> (loss float64, grad fp32 [B,L,D] or None)."""
    pred = np.ascontiguousarray(pred, np.float32)
    target = np.ascontiguousarray(target, np.float32)
    mask = np.ascontiguousarray(mask, np.uint8)
    B, L, D = pred.shape
    if num_masked is None:
        num_masked = int(mask.astype(np.int64).sum())
    loss = C.c_double()
    grad = np.empty((B, L, D), np.float32) if want_grad else None
    rc = lib().mae_oracle_pixel_loss(B, L, D, _p(pred), _p(target), _p(mask), num_masked,
                                     grad_scale, C.byref(loss), _p(grad))
    if rc != 0:
        raise ValueError("mae_oracle_pixel_loss: invalid argument")
    return loss.value, grad


def pretrain_stage(scheme: int, stage: int):
    """-> (resolution, mask_ratio) of Table 9, or None for an unknown scheme / stage."""
    res, m = C.c_int32(), C.c_double()
    if lib().mae_oracle_pretrain_stage(scheme, stage, C.byref(res), C.byref(m)) != 0:
        return None
    return res.value, m.value


FINETUNE_SCHEMES = {"1": 1, "3": 3, "1-": 10, "1+": 11}


def finetune_stage(scheme: int, stage: int):
    """-> (resolution, sigma_lo, sigma_hi, aug) of Table 7, or None.  scheme 10 / 11 are the
    table's "1-" / "1+"; aug 1 = "3 Aug", 2 = "3 Aug+"."""
    res, lo, hi, aug = C.c_int32(), C.c_double(), C.c_double(), C.c_int32()
    if lib().mae_oracle_finetune_stage(scheme, stage, C.byref(res), C.byref(lo), C.byref(hi),
                                       C.byref(aug)) != 0:
        return None
    return res.value, lo.value, hi.value, aug.value


def stage_of_epoch(epoch: int, lengths) -> int:
    arr = np.ascontiguousarray(lengths, np.int32)
    return int(lib().mae_oracle_stage_of_epoch(epoch, _p(arr), len(arr)))


def patch_embed(visible, ids_keep, weight, bias=None, pos=None):
    """tokens [B,K,E] float64 = visible @ weight.T + bias + pos[ids_keep]."""
    visible = np.ascontiguousarray(visible, np.float32)
    weight = np.ascontiguousarray(weight, np.float32)
    B, K, D = visible.shape
    E = weight.shape[0]
    assert weight.shape == (E, D)
    ids = None if ids_keep is None else np.ascontiguousarray(ids_keep, np.int32)
    b = None if bias is None else np.ascontiguousarray(bias, np.float32)
    p = None if pos is None else np.ascontiguousarray(pos, np.float32)
    L = 1 if p is None else p.shape[0]
    out = np.empty((B, K, E), np.float64)
    rc = lib().mae_oracle_patch_embed(B, K, D, E, L, _p(visible), _p(ids), _p(weight), _p(b),
                                      _p(p), _p(out))
    if rc != 0:
        raise ValueError("mae_oracle_patch_embed: invalid argument")
    return out


def jpeg_info(data: bytes):
    """-> dict(H, W, luma_h, luma_v, restart_interval); raises ValueError on an unsupported file."""
    buf = np.frombuffer(data, np.uint8)
    v = [C.c_int32() for _ in range(5)]
    rc = lib().mae_oracle_jpeg_info(_p(buf), buf.size, *[C.byref(x) for x in v])
    if rc != 0:
        raise ValueError(f"mae_oracle_jpeg_info: {rc}")
    return dict(zip(("H", "W", "luma_h", "luma_v", "restart_interval"), (x.value for x in v)))


def jpeg_decode(data: bytes, ycc: bool = False) -> np.ndarray:
    """Baseline JPEG -> [H, W, 3] uint8 RGB (the whole image); ycc=True: before the colour
    conversion (Y, Cb, Cr per pixel)."""
    info = jpeg_info(data)
    buf = np.frombuffer(data, np.uint8)
    out = np.empty((info["H"], info["W"], 3), np.uint8)
    fn = lib().mae_oracle_jpeg_decode_ycc if ycc else lib().mae_oracle_jpeg_decode
    rc = fn(_p(buf), buf.size, _p(out))
    if rc != 0:
        raise ValueError(f"mae_oracle_jpeg_decode: {rc}")
    return out


def idct8x8(coef) -> np.ndarray:
    """coef [8, 8] int (dequantised, [v][u]) -> [8, 8] uint8 samples ([y][x])."""
    cf = np.ascontiguousarray(coef, np.int32).reshape(64)
    out = np.empty(64, np.uint8)
    lib().mae_oracle_idct8x8(_p(cf), _p(out))
    return out.reshape(8, 8)


def ycc_to_rgb(y: int, cb: int, cr: int):
    out = np.empty(3, np.uint8)
    lib().mae_oracle_ycc_to_rgb(y, cb, cr, _p(out))
    return tuple(int(v) for v in out)


def huff_codes(counts):
    """counts[16] -> list of (code, length) in table order."""
    cnt = np.ascontiguousarray(counts, np.uint8)
    n = int(cnt.sum())
    codes = np.zeros(max(n, 1), np.uint16)
    lengths = np.zeros(max(n, 1), np.uint8)
    m = lib().mae_oracle_huff_codes(_p(cnt), _p(codes), _p(lengths))
    assert m == n
    return [(int(codes[i]), int(lengths[i])) for i in range(n)]


def threads() -> int:
    return int(lib().mae_oracle_threads())


def set_threads(n: int) -> None:
    """Threads for the loops over samples and rows from now on (0 = the default)."""
    lib().mae_oracle_set_threads(int(n))
