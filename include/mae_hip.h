/*
 * mae_hip.h -- C ABI of the MI355X (gfx950) library for the per-batch masked-autoencoder input
 * pipeline and its reconstruction loss (DailyMAE, arXiv 2404.00509).
 *
 * Two calls make up the path, a third is the first consumer of its output:
 *
 *   mae_prep_batch     decoded uint8 images in device memory -> training tensors.
 *                      RandomResizedCrop (Sec. 5.1: area scale uniform, aspect ratio log-uniform,
 *                      crop then resize to the training resolution of the progressive schedule,
 *                      Sec. 5.3 / Table 9), bilinear resampling (Sec. 4.1), the "Simple"
 *                      augmentation = horizontal flip + tensor conversion + mean/std
 *                      normalisation (App. B), the ViT patch split (Sec. 3), random masking at a
 *                      masking ratio with only the visible patches handed to the encoder
 *                      (Sec. 2, Sec. 5.3 "Masking Ratio").
 *   mae_normpix_loss   the reconstruction objective of the official MAE recipe that the paper
 *                      adopts (Sec. 3): mean squared error against per-patch normalised pixels on
 *                      the masked patches, and its gradient with respect to the prediction.
 *   mae_patch_embed    linear patch embedding of the visible tokens with bias and positional
 *                      embedding (Sec. 2, Sec. 5), on the matrix cores.
 * mae_prep_batch also takes JPEG files and decodes only the region each crop needs ("crop
 * decode", Sec. 4.1; mae_jpeg_index prepares files once for it) and applies the finetuning
 * augmentation (Sec. 4.4); mae_normpix_loss_from_images is the loss without a stored target;
 * mae_pretrain_stage / mae_finetune_stage / mae_stage_of_epoch are the paper's schedules.
 *
 * Conventions
 *   - Every pointer is a DEVICE pointer unless its name starts with host_.  The descriptor
 *     structs themselves live in host memory and are read during the call only.
 *   - The caller allocates and owns every buffer, the workspace included.  The library keeps no
 *     global state, never allocates or frees device memory and keeps no pointer after a call
 *     (one exception, stated there: the fixed scratch array of mae_normpix_loss_static).
 *   - Calls validate their arguments on the host, enqueue kernels on `hip_stream` (a hipStream_t
 *     passed as void*, NULL = the default stream) and return without synchronising.  Outputs are
 *     valid once the stream has reached that point.  Calls are re-entrant; two calls that share a
 *     workspace must be ordered by the stream.
 *   - Return value: MAE_OK or a negative mae_status.  Argument errors are found before anything
 *     is launched, so a failed call has no side effect.
 *   - Image geometry (heights, widths, offsets) lives in device memory and cannot be checked on
 *     the host.  The kernels check every sample (1 <= H, W <= 32767, the image lies inside
 *     [0, images_bytes); for JPEG input: a file the decoder takes).  A sample that fails takes no
 *     part in the batch and gets neutral outputs: its mask row is all 0 (nothing of it is masked,
 *     so it adds nothing to the loss and its gradient rows are zero), ids_restore[l] = l,
 *     ids_keep[r] = r, its rows of `target` and `visible` are zeros, crop_out is 0,0,0,0,0 with
 *     valid = 0, and it is counted in the workspace status word that mae_prep_status reads back.
 *     With such samples in a batch the number of masked patches is no longer B * (L - K): pass
 *     num_masked = 0 to the loss calls to have it counted from the mask on the device.
 */
#ifndef MAE_HIP_H
#define MAE_HIP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MAE_OK = 0,
  MAE_ERR_NULL = -1,      /* a required pointer is NULL                                        */
  MAE_ERR_SHAPE = -2,     /* sizes that do not fit together (B <= 0, S % p != 0, K outside ...) */
  MAE_ERR_RANGE = -3,     /* a value outside the supported range (see each field)              */
  MAE_ERR_DTYPE = -4,     /* unknown mae_dtype                                                 */
  MAE_ERR_WORKSPACE = -5, /* workspace missing, misaligned (256 B) or too small                */
  MAE_ERR_NO_DEVICE = -6, /* no HIP device visible to this process                             */
  MAE_ERR_HIP = -7        /* a HIP runtime call failed (launch error)                          */
} mae_status;

typedef enum { MAE_F32 = 0, MAE_BF16 = 1 } mae_dtype;

/* Augmentation applied between resize and normalisation.
 *   MAE_AUG_SIMPLE      nothing but the flip: the pretraining "Simple" augmentation (App. B).
 *   MAE_AUG_THREE       the finetuning recipe's "3 Aug" (Sec. 3, Sec. 4.4, Table 7): per image one
 *                       of grayscale / solarisation / Gaussian blur, each with probability 1/3.
 *   MAE_AUG_THREE_PLUS  "3 Aug+" (Sec. 5.2): the same followed by colour jitter.
 * The paper names these procedures without parameters; the library's definitions are:
 *   - they act on the 8-bit image: the bilinear value is rounded to the nearest integer, ties
 *     upwards, exactly; after the per-image operation nothing is rounded again;
 *   - grayscale: luma (299 R + 587 G + 114 B) / 1000 rounded to nearest, in all three channels;
 *   - solarisation: values >= 128 become 255 - v;
 *   - blur: separable Gaussian, sigma uniform on [0.1, 2], taps k = -r..r with r = ceil(3 sigma),
 *     scaled to sum 1, border pixels repeated;
 *   - jitter: factors b, c, s uniform on [1 - jitter, 1 + jitter]; v <- clamp(b v);
 *     v <- clamp(c v + (1 - c) m) with m the mean over the image of 0.299 R + 0.587 G + 0.114 B at
 *     that point; v <- clamp(s v + (1 - s) luma(v)); clamp is to [0, 255]. */
typedef enum { MAE_AUG_SIMPLE = 0, MAE_AUG_THREE = 1, MAE_AUG_THREE_PLUS = 2 } mae_aug_mode;

/* What `images` holds.
 *   MAE_INPUT_DECODED  decoded pixels (see mae_prep_desc).
 *   MAE_INPUT_JPEG     JPEG files, and only the region that the crop needs is decoded ("crop
 *                      decode", Sec. 4.1): the rows of MCUs above and below the crop are skipped,
 *                      a row is entropy-decoded up to the crop's right edge, and the inverse
 *                      transform runs for the MCUs inside the crop only.  The result is the same
 *                      as decoding the whole image first.
 * Files the decoder takes: baseline sequential DCT, 8 bits, three components (JFIF YCbCr), luma
 * sampled 1x1 or 2x2 against 1x1 chroma ("4:4:4", "4:2:0"), the two chroma components sharing
 * their tables, any restart interval or none, and no side longer than max_image_side rounded up
 * to 16 (in this mode the hint is a limit; 0 = 256).  A file with one restart interval per row
 * of MCUs (a choice of the dataset writer that costs 0.2 % in size) has independent rows, and
 * those outside the crop are never touched; in any other file the entropy-coded data has to be
 * walked through from its start down to the crop's last row to find where the rows begin (symbol
 * lengths only, one lane per file: several times the cost of the decoding itself), unless the
 * caller passes the file's row index (mae_jpeg_index, jpeg_row_index below), which is computed
 * once per file and makes every file decode like one with independent rows.  Any other file makes
 * its sample invalid
 * (valid = 0 in crop_out, counted by mae_prep_status).  A decoder is specified by the standard
 * only up to the accuracy of the inverse DCT, the chroma interpolation and the colour arithmetic;
 * here: 13-bit fixed-point separable inverse DCT (first pass kept with 3 fractional bits, inputs
 * of both passes clamped to +-32767), each chroma sample repeated over the pixels it covers,
 * JFIF matrix in 16-bit fixed point (91881, 22554, 46802, 116130), floor after adding one half. */
typedef enum { MAE_INPUT_DECODED = 0, MAE_INPUT_JPEG = 1 } mae_input_format;

/* ------------------------------------------------------------------------------------------------
 * mae_prep_batch
 *
 * Notation: B images; image b is H_b x W_b x 3 uint8, HWC, rows tightly packed (stride 3 W_b);
 * S = out_size, p = patch, G = S / p, L = G * G patches, D = 3 p^2 values per patch,
 * K = num_keep visible patches.
 *
 * Random numbers: every draw is a pure function of (seed, batch_index, sample_base + b, stream,
 * counter) -- the SplitMix64 output function applied to a keyed counter -- so a batch can be
 * recomputed, and a shard of a batch gives the same values as the whole batch.
 *
 * Limits: B <= 2^20; 1 <= L <= 256; 1 <= p <= 32; S <= 512;
 * exp(-1/2) <= ratio_lo <= ratio_hi <= exp(1/2).
 *
 * Finetuning (Sec. 5.2) uses the same call: every patch is kept (num_keep = L, so `visible` holds
 * all patches in noise order and `target` all patches in grid order), the crop's scale range
 * comes from mae_finetune_stage and aug_mode selects the augmentation.
 * ---------------------------------------------------------------------------------------------- */
typedef struct {
  int32_t B;               /* images in this call, > 0                                          */
  const uint8_t* images;   /* packed images; image b starts at images + offsets[b]              */
  int64_t images_bytes;    /* size of the `images` buffer; used for device-side bounds checks   */
  const int64_t* offsets;  /* [B] byte offsets, >= 0                                            */
  const int32_t* heights;  /* [B]                                                               */
  const int32_t* widths;   /* [B]                                                               */
  int32_t out_size;        /* S                                                                 */
  int32_t patch;           /* p, S % p == 0                                                     */
  int32_t num_keep;        /* K in [1, L]; see mae_num_keep                                     */
  float scale_lo, scale_hi; /* area fraction of the crop, 0 < lo <= hi <= 1 (paper: 0.2 .. 1)   */
  float ratio_lo, ratio_hi; /* width / height of the crop, lo <= hi (paper: 3/4 .. 4/3)         */
  float flip_p;            /* probability of the horizontal flip, in [0, 1]                     */
  float mean[3], std[3];   /* per channel, applied as (v / 255 - mean) / std; std > 0           */
  uint64_t seed;           /* random-number key                                                 */
  uint64_t batch_index;    /* random-number key; vary per step                                  */
  uint32_t sample_base;    /* global index of sample 0 of this call (0 unless sharding a batch) */
  int32_t noise_bits;      /* 1..32 bits of masking noise per patch; 32 in production, small
                              values force ties (equal keys keep index order)                   */
  int32_t out_dtype;       /* mae_dtype of `visible`                                            */
  int32_t max_image_side;  /* tuning hint: largest H or W in the batch, 0 = 256 (the "maximum
                              side 256" dataset variant).  It sizes the on-chip staging buffer;
                              larger images than hinted stay correct but take a slower path     */
  int32_t aug_mode;        /* mae_aug_mode.  Other than MAE_AUG_SIMPLE needs an even p
                              (MAE_ERR_SHAPE otherwise; multiples of 4 run fastest)             */
  float jitter;            /* MAE_AUG_THREE_PLUS: strength in [0, 1], 0.3 in the paper            */
  int32_t input_format;    /* mae_input_format.  MAE_INPUT_JPEG: `images` holds the files back to
                              back (8-byte aligned buffer), images_bytes their total size,
                              offsets[b] the start of file b; heights and widths are not read
                              (may be NULL)                                                      */
  const int32_t* file_sizes; /* [B] length of each file in bytes; MAE_INPUT_JPEG only            */
  const void* jpeg_row_index; /* nullable, MAE_INPUT_JPEG only: [B] entries of
                              mae_jpeg_index_bytes(d) / B bytes each, entry b being what
                              mae_jpeg_index wrote for file b (with the same max_image_side);
                              16-byte aligned.  With it no file is walked through.  Entries are
                              checked before use: one that does not fit its file gives a sample
                              flagged invalid or wrong pixels, never an access outside the
                              buffers                                                           */
  int64_t jpeg_row_index_bytes; /* size of that buffer; less than mae_jpeg_index_bytes(d) is
                              refused (MAE_ERR_WORKSPACE)                                       */
} mae_prep_desc;

/* Outputs (device):
 *   visible      [B, K, D] out_dtype  visible[b, r, :] = patch ids_keep[b, r] of image b; r runs
 *                                     in order of increasing noise.                   required
 *   mask         [B, L] uint8         0 = visible, 1 = masked.                        required
 *   ids_restore  [B, L] int32         rank of patch l in the noise order; the patch is visible
 *                                     iff rank < K.                                   required
 *   ids_keep     [B, K] int32         patch index at rank r.                          nullable
 *   target       [B, L, D] float      all patches, image-normalised (not per-patch normalised);
 *                                     element order inside a patch is (row, column, channel);
 *                                     patches in row-major grid order.                nullable
 *   crop_out     [B, 6] int32         top, left, height, width of the crop box, flip bit, valid
 *                                     flag.                                           nullable
 *   workspace    mae_prep_workspace_bytes(d) bytes, 256-byte aligned.                 required
 * Pixel values are never rounded back to bytes between resize and normalisation.
 * bf16 `visible` is the float value rounded to nearest even. */
int mae_prep_batch(const mae_prep_desc* d, void* visible, uint8_t* mask, int32_t* ids_restore,
                   int32_t* ids_keep, float* target, int32_t* crop_out, void* workspace,
                   size_t workspace_bytes, void* hip_stream);

/* Bytes of workspace mae_prep_batch needs for this descriptor (0 if the descriptor is invalid).
 * A few hundred bytes plus 32 per image; with augmentation also out_size^2 * 3 + 32 per image;
 * with MAE_INPUT_JPEG also the decoded planes and the RGB regions, together 6 bytes per pixel of
 * a square of side max_image_side rounded up to 16 (0 = 256), per image (an upper bound: which
 * part of it a call touches depends on the crops it draws), and about 6 KB of tables per image. */
size_t mae_prep_workspace_bytes(const mae_prep_desc* d);

/* Row index of JPEG files (crop decode, Sec. 4.1: the loader decodes only the crop's region; Sec.
 * 4.2: datasets are prepared once).  For every file of the descriptor (input_format must be
 * MAE_INPUT_JPEG; the crop, output and augmentation fields are validated but not used) and every
 * row of MCUs of it: where the row's entropy-coded data starts -- byte position, pending bits,
 * DC predictors, MCUs left in the restart interval -- 32 bytes per row,
 * (max_image_side rounded up to 16) / 8 rows per file whatever the file's size, rows the file
 * does not have and every row of a file the decoder does not take marked unknown.  An entry
 * depends on nothing but its file, so it is computed once per file, stored with it, and gathered
 * per batch like the file itself into `jpeg_row_index` of later mae_prep_batch calls.  The format
 * of an entry belongs to this version of the library (mae_version).
 *   index      mae_jpeg_index_bytes(d) bytes, 16-byte aligned, device      required
 *   workspace  mae_prep_workspace_bytes(d) bytes, 256-byte aligned         required
 * mae_jpeg_index_bytes returns 0 for an invalid descriptor. */
size_t mae_jpeg_index_bytes(const mae_prep_desc* d);
int mae_jpeg_index(const mae_prep_desc* d, void* index, size_t index_bytes, void* workspace,
                   size_t workspace_bytes, void* hip_stream);

/* Waits for `hip_stream`, then stores in *host_invalid_samples how many samples of the last
 * mae_prep_batch call on this workspace failed the device-side geometry check.  Synchronises. */
int mae_prep_status(const void* workspace, void* hip_stream, int32_t* host_invalid_samples);

/* floor(L * (1 - mask_ratio)) in double precision: 49 for L = 196 at ratio 0.75, 19 (not 20) for
 * L = 100 at ratio 0.8.  Returns -1 when the arguments are out of range. */
int32_t mae_num_keep(int32_t L, double mask_ratio);

/* ------------------------------------------------------------------------------------------------
 * mae_normpix_loss
 *
 * For every patch row t = target[b, l, :]: mu = mean(t), var = sum (t - mu)^2 / (D - 1),
 * that = (t - mu) / sqrt(var + eps).  With M = num_masked:
 *   loss = sum over masked rows of mean_e (pred - that)^2  /  M
 *   grad = grad_scale * 2 (pred - that) / (D * M) on masked rows, +0 on visible rows.
 * Statistics and sums are accumulated in single precision per row and double precision across
 * rows; the result does not depend on scheduling (fixed reduction order).
 *
 * Limits: 2 <= D <= 3072.
 * ---------------------------------------------------------------------------------------------- */
typedef struct {
  int32_t B, L, D;
  const void* pred;      /* [B, L, D] pred_dtype                                                */
  const float* target;   /* [B, L, D] float, as written by mae_prep_batch                       */
  const uint8_t* mask;   /* [B, L], non-zero = masked                                           */
  int64_t num_masked;    /* M > 0: masked patches of the WHOLE batch (B_global * (L - K)); the
                            caller knows it in closed form, so shards need no exchange for grad.
                            0: M = the number of non-zero bytes of `mask`, counted on the device
                            by a small kernel before the loss kernel (for batches that may hold
                            unusable samples, whose mask rows are 0); if that is 0 too, the loss
                            and the gradient are 0 */
  float eps;             /* >= 0, 1e-6 in the MAE recipe                                        */
  float grad_scale;      /* upstream derivative of the loss, normally 1                         */
  int32_t pred_dtype;    /* mae_dtype of pred and grad                                          */
  int32_t norm_pix;      /* 1: the objective above (per-patch normalised pixels); 0: the
                            un-normalised variant, that = t, eps unused                          */
} mae_loss_desc;

/* Outputs (device):
 *   loss       [1] float     required
 *   grad       [B, L, D] pred_dtype, every element written     nullable (loss only)
 *   workspace  mae_loss_workspace_bytes(d) bytes, 256-byte aligned   required */
int mae_normpix_loss(const mae_loss_desc* d, float* loss, void* grad, void* workspace,
                     size_t workspace_bytes, void* hip_stream);

size_t mae_loss_workspace_bytes(const mae_loss_desc* d);

/* mae_normpix_loss for callers that cannot allocate device memory and so have no workspace to
 * pass (code under HIP graph capture, tight serving loops, harnesses that forbid allocation): the
 * same kernels and the same results bit for bit, with the per-wavefront partial sums kept in a
 * fixed 64-KiB array in device memory that belongs to the library (one copy per GPU, resident
 * until the process ends) instead of a workspace.  The call itself allocates and frees nothing.
 * Inputs and outputs are passed as for mae_normpix_loss.  A descriptor whose launch would need
 * more than 8192 partial sums is rejected with MAE_ERR_WORKSPACE before anything is launched
 * (today's launch shapes stay below that for every valid descriptor).  All calls on one GPU share
 * the array: calls that overlap on one GPU (different streams, different threads) race; order
 * them on one stream.  Nothing in the array has to be cleared between calls.  The first call on a
 * device looks up the array's device address (no stream work); make it before a capture starts. */
int mae_normpix_loss_static(const mae_loss_desc* d, float* loss, void* grad, void* hip_stream);

/* ------------------------------------------------------------------------------------------------
 * mae_normpix_loss_from_images
 *
 * The same loss and gradient without a stored target: the masked patches' pixels are taken from
 * the images again (same crop, resize, flip and normalisation, bit for bit what mae_prep_batch
 * writes to `target`), normalised per patch and compared with the prediction in one kernel.  The
 * model's forward and backward pass lies between mae_prep_batch and the loss, and the 8-bit images
 * are several times smaller than the float target, so a caller that passes target = NULL to
 * mae_prep_batch saves writing L * D floats per image there and reading the masked part of them
 * here (Sec. 4: the input pipeline is what limits the training step).
 *
 * p               the descriptor of the mae_prep_batch call whose crops are meant (same images,
 *                 same seed, batch_index and sizes; aug_mode MAE_AUG_SIMPLE; even patch size,
 *                 MAE_ERR_SHAPE otherwise)
 * prep_workspace  the workspace that call used (and its size), untouched since: it holds the
 *                 crop boxes (and, for JPEG input, the decoded regions)
 * d               as for mae_normpix_loss; d->target is not read (may be NULL); B, L, D must
 *                 match p (MAE_ERR_SHAPE otherwise)
 * Outputs as for mae_normpix_loss.  Samples flagged invalid by mae_prep_batch add nothing to the
 * loss and get a zero gradient.  workspace: mae_loss_from_images_workspace_bytes(p, d) bytes,
 * 256-byte aligned.
 * ---------------------------------------------------------------------------------------------- */
int mae_normpix_loss_from_images(const mae_prep_desc* p, const void* prep_workspace,
                                 size_t prep_workspace_bytes, const mae_loss_desc* d, float* loss,
                                 void* grad, void* workspace, size_t workspace_bytes,
                                 void* hip_stream);

size_t mae_loss_from_images_workspace_bytes(const mae_prep_desc* p, const mae_loss_desc* d);

/* ------------------------------------------------------------------------------------------------
 * mae_patch_embed
 *
 * The first operation of the encoder on what mae_prep_batch hands it (Sec. 2: the encoder works on
 * the visible patches only; Sec. 5: the ViT's linear patch embedding with positional embeddings):
 *   tokens[m, e] = sum_d visible[m, d] * weight[e, d] + bias[e] + pos[ids_keep[m], e]
 * for the M = B * K visible rows of a batch.  The products of the bf16 operands are exact in
 * single precision and are accumulated in single precision on the matrix cores; bias and the
 * positional row are added in single precision and the sum is rounded once to out_dtype.
 *
 * `weight` is the [E, 3, p, p] convolution kernel of the usual patch embedding with its last three
 * axes reordered to (row, column, channel), the element order of a patch row.
 *
 * Limits: 1 <= M <= 2^28; 4 <= D <= 3072 with D % 4 == 0; 1 <= E <= 8192; 1 <= L.
 * visible, weight, pos and tokens are 16-byte aligned (MAE_ERR_RANGE otherwise).
 * An ids_keep value outside [0, L) is clamped into it before it indexes `pos`.
 * ---------------------------------------------------------------------------------------------- */
typedef struct {
  int64_t M;               /* token rows, B * K                                                 */
  int32_t D, E, L;         /* values per patch, embedding width, patches per image              */
  const void* visible;     /* [M, D] bf16, as written by mae_prep_batch with out_dtype MAE_BF16 */
  const int32_t* ids_keep; /* [M] patch index of each row; required iff pos is given            */
  const void* weight;      /* [E, D] bf16                                                       */
  const float* bias;       /* [E] float, nullable                                               */
  const float* pos;        /* [L, E] float, row l = positional embedding of patch l; nullable   */
  int32_t out_dtype;       /* mae_dtype of tokens                                               */
} mae_embed_desc;

/* Output (device): tokens [M, E] out_dtype, every element written.  No workspace. */
int mae_patch_embed(const mae_embed_desc* d, void* tokens, void* hip_stream);

/* ------------------------------------------------------------------------------------------------
 * Progressive schedules (host-side tables; nothing is launched).
 *
 * The paper trains in three stages that change the resolution and the masking ratio (pretraining,
 * Sec. 5.3 Table 9, schemes 1..6; scheme 5 is the 224 -> 192 -> 224 palindrome) or the resolution
 * and the crop's scale range (finetuning, Sec. 5.2 Table 7).  A stage switch needs no new buffers:
 * every call takes its sizes from its descriptor, so buffers sized for the largest stage serve
 * all of them.
 * ---------------------------------------------------------------------------------------------- */

/* Pretraining scheme 1..6, stage 1..3 -> *out_size (training resolution) and *mask_ratio. */
int mae_pretrain_stage(int32_t scheme, int32_t stage, int32_t* host_out_size,
                       double* host_mask_ratio);

/* The finetuning schemes of Table 7.  1-, 1+ have the sizes of scheme 1 and differ from it in the
 * augmentation column only. */
typedef enum {
  MAE_FINETUNE_SCHEME_1 = 1,
  MAE_FINETUNE_SCHEME_3 = 3,
  MAE_FINETUNE_SCHEME_1_MINUS = 10,
  MAE_FINETUNE_SCHEME_1_PLUS = 11
} mae_finetune_scheme;

/* Finetuning scheme (mae_finetune_scheme), stage 1..3 -> resolution, the bounds of the crop's
 * side ratio sigma as the area-fraction bounds that mae_prep_desc takes (*host_scale_lo =
 * sigma_lo^2, *host_scale_hi = sigma_hi^2), and the stage's augmentation (*host_aug_mode, a
 * mae_aug_mode for mae_prep_desc.aug_mode: MAE_AUG_THREE or MAE_AUG_THREE_PLUS; nullable). */
int mae_finetune_stage(int32_t scheme, int32_t stage, int32_t* host_out_size,
                       float* host_scale_lo, float* host_scale_hi, int32_t* host_aug_mode);

/* 1-based stage that 0-based `epoch` falls in when the stages last host_lengths[0..n) epochs
 * (finetuning: 30, 30, 40; the paper gives none for pretraining).  Epochs past the end belong to
 * the last stage.  Negative return: MAE_ERR_NULL / MAE_ERR_RANGE. */
int mae_stage_of_epoch(int32_t epoch, const int32_t* host_lengths, int32_t n);

/* Static, NUL-terminated description of a status code. */
const char* mae_error_string(int status);

/* Version of this ABI: major * 10000 + minor * 100 + patch. */
int mae_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MAE_HIP_H */
