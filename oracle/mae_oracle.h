/*
 * CPU oracle for the masked-autoencoder input pipeline (DailyMAE, arXiv 2404.00509).
 *
 * TEST INFRASTRUCTURE ONLY.  This is a slow, plain, scalar implementation whose single purpose is
 * to say what the GPU library must compute.  It shares no source, header, table or helper with the
 * HIP path, and nothing in the product path may call it.  Every pointer is a HOST pointer.
 *
 * Steps, in the order the paper's loader and model apply them:
 *   RandomResizedCrop parameters (Sec. 5.1: area scale uniform, aspect ratio log-uniform, crop a
 *   region then resize it to the output size), the crop + resize itself (Sec. 4.1), the "Simple"
 *   augmentation = horizontal flip + tensor conversion + mean/std normalisation (App. B), the
 *   ViT patch split (Sec. 3, Sec. 5), random masking at a masking ratio with the encoder seeing
 *   only the visible patches (Sec. 2, Sec. 5.3 "Masking Ratio"), and the reconstruction loss of
 *   the official MAE recipe the paper adopts (Sec. 3): mean squared error against per-patch
 *   normalised pixels on the masked patches, with its gradient.
 *
 * The paper leaves rounding, retry, tie-break and random-number details open; the readings taken
 * here are written next to each function.
 *
 * Every function is pinned by tests that do not depend on this file's own arithmetic (closed
 * forms, printed vectors, brute force, library cross-checks); none is "parity unpinned".
 */
#ifndef MAE_ORACLE_H
#define MAE_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- counter-based random numbers (SplitMix64 output function, Steele/Lea/Flood 2014) -------- */
uint64_t mae_oracle_mix64(uint64_t z);
/* (w+1)-th output of a SplitMix64 stream whose state is derived from (seed, batch_index);
 * w = sample<<32 | stream<<24 | ctr.  Streams: 0 scale, 1 log-ratio, 2 top, 3 left (ctr =
 * attempt), 4 flip, 5 mask noise (ctr = patch index). */
uint64_t mae_oracle_draw(uint64_t seed, uint64_t batch_index, uint32_t sample, uint32_t stream,
                         uint32_t ctr);

/* ---- RandomResizedCrop parameters (Sec. 5.1) -------------------------------------------------- */
/* exp(x) as the degree-13 Taylor polynomial in Horner form, fp64, no fused operations. */
double mae_oracle_exp_poly(double x);
/* Proposal of attempt `attempt` (0..9) before the accept test: out = {ch, cw}. */
void mae_oracle_rrc_proposal(int32_t H, int32_t W, float scale_lo, float scale_hi, float ratio_lo,
                             float ratio_hi, uint64_t seed, uint64_t batch_index, uint32_t sample,
                             int32_t attempt, int64_t out_hw[2]);
/* Accepted crop box: box = {top, left, ch, cw}.  Returns the number of attempts used (1..10), or
 * 11 when all ten were rejected and the centred fallback box was taken. */
int32_t mae_oracle_rrc_params(int32_t H, int32_t W, float scale_lo, float scale_hi, float ratio_lo,
                              float ratio_hi, uint64_t seed, uint64_t batch_index, uint32_t sample,
                              int32_t box[4]);

/* ---- flip (App. B) ---------------------------------------------------------------------------- */
int32_t mae_oracle_flip_bit(uint64_t seed, uint64_t batch_index, uint32_t sample, float flip_p);

/* ---- crop + bilinear resize (Sec. 4.1, Sec. 5.1) ---------------------------------------------- */
/* Source taps of output index o when `crop_len` source pixels are resized to `out_size`:
 * half-pixel centres, two taps, clamped to the crop.  f is the exact rational weight of tap i1. */
void mae_oracle_resize_taps(int32_t out_size, int32_t crop_len, int32_t o, int32_t* i0, int32_t* i1,
                            double* f);
/* img: H x W x 3 uint8 (rows tightly packed).  out: S x S x 3 doubles in pixel units (0..255),
 * row-major HWC, already flipped when flip != 0. */
void mae_oracle_crop_resize(const uint8_t* img, int32_t H, int32_t W, const int32_t box[4],
                            int32_t S, int32_t flip, double* out);

/* ---- normalise (App. B) ----------------------------------------------------------------------- */
double mae_oracle_normalise(double v, double mean, double std);

/* ---- patchify (Sec. 3: ViT-B/16 patches) ------------------------------------------------------ */
/* img: S x S x 3 doubles (HWC).  out: L x D doubles, L = (S/p)^2 row-major over patches,
 * D = 3 p^2 with element order (row in patch, column in patch, channel). */
void mae_oracle_patchify(const double* img, int32_t S, int32_t p, double* out);

/* ---- random masking (Sec. 2, Sec. 5.3) -------------------------------------------------------- */
/* floor(L * (1 - mask_ratio)) evaluated in fp64. */
int32_t mae_oracle_num_keep(int32_t L, double mask_ratio);
/* ids_restore[L], ids_keep[K], mask[L] (1 = masked) for one sample.  Rank by counting. */
void mae_oracle_mask(uint64_t seed, uint64_t batch_index, uint32_t sample, int32_t L, int32_t K,
                     int32_t noise_bits, int32_t* ids_restore, int32_t* ids_keep, uint8_t* mask);

/* ---- finetuning augmentation: "3 Aug" and "3 Aug+" (Sec. 3 finetuning recipe, Sec. 4.4 "Data
 * Augmentation", Sec. 5.2 Table 7; the procedure itself is the cited Three Augmentation: one of
 * grayscale / solarisation / Gaussian blur per image, chosen uniformly, optionally followed by
 * colour jitter).  The paper gives no parameters; the readings are written at each function. ---- */
/* The resized crop as an 8-bit image: the bilinear value of mae_oracle_crop_resize rounded to the
 * nearest integer, ties upwards, evaluated in exact integer arithmetic.  out: S x S x 3. */
void mae_oracle_resize_u8(const uint8_t* img, int32_t H, int32_t W, const int32_t box[4], int32_t S,
                          int32_t flip, uint8_t* out);
/* Per-sample draws: op = 0 grayscale, 1 solarise, 2 blur (stream 6); sigma uniform on [0.1, 2]
 * (stream 7); brightness, contrast, saturation factors uniform on [1 - jitter, 1 + jitter]
 * (streams 8, 9, 10). */
void mae_oracle_aug_params(uint64_t seed, uint64_t batch_index, uint32_t sample, double jitter,
                           int32_t* op, double* sigma, double bcs[3]);
/* Luma of an 8-bit pixel with the ITU-R BT.601 weights 0.299, 0.587, 0.114, rounded to the
 * nearest integer in integer arithmetic. */
int32_t mae_oracle_gray(int32_t r, int32_t g, int32_t b);
/* Solarisation with threshold 128: values at or above it are inverted. */
int32_t mae_oracle_solarise(int32_t v);
/* Gaussian taps exp(-k^2 / (2 sigma^2)), k = -radius..radius, radius = ceil(3 sigma), scaled to
 * sum 1.  w must hold 2 * radius + 1 <= 13 values.  Returns the radius. */
int32_t mae_oracle_blur_weights(double sigma, double* w);
/* One of the three operations on an 8-bit S x S x 3 image -> doubles in pixel units.  The blur is
 * the separable Gaussian above with the image's border pixels repeated outwards. */
void mae_oracle_three_aug(const uint8_t* u8, int32_t S, int32_t op, double sigma, double* out);
/* Colour jitter in place on S x S x 3 doubles: brightness (v * b), then contrast (blend with the
 * mean luma of the whole image, weight c), then saturation (blend with the pixel's luma, weight
 * s); every step clamps to [0, 255]. */
void mae_oracle_color_jitter(double* img, int32_t S, const double bcs[3]);

/* ---- the whole input pipeline for samples [b_begin, b_end) of a batch ------------------------- */
typedef struct {
  int32_t B;
  const uint8_t* images;   /* packed HWC uint8; image b starts at images + offsets[b] */
  const int64_t* offsets;  /* [B] */
  const int32_t* heights;  /* [B] */
  const int32_t* widths;   /* [B] */
  int32_t out_size, patch, num_keep;
  float scale_lo, scale_hi, ratio_lo, ratio_hi, flip_p;
  float mean[3], std[3];
  uint64_t seed, batch_index;
  int32_t noise_bits;
  int32_t aug_mode; /* 0 = "Simple" (App. B); 1 = "3 Aug"; 2 = "3 Aug+" = 3 Aug + ColorJitter */
  float jitter;     /* ColorJitter strength (0.3 in Sec. 5.2), used by aug_mode 2 */
  int64_t images_bytes; /* size of `images`, 0 = unknown (then images are not checked against it) */
} mae_oracle_prep_args;

/* Outputs are indexed by (b - b_begin); any may be NULL.  The hash is keyed by the global sample
 * index b, so a slice gives the same values as the full batch.
 *   visible [n,K,D] fp32, target [n,L,D] fp32 (fp64 result rounded once), mask [n,L] uint8,
 *   ids_restore [n,L], ids_keep [n,K], crop [n,5] = top,left,ch,cw,flip, valid [n] uint8.
 * A sample that cannot be read (H or W outside 1..32767, a negative offset, or an image that
 * runs past images_bytes) is left out of training (the paper does not treat unreadable samples;
 * this is the reading taken): valid 0, crop zeros, mask row all 0 (nothing of it is masked, so
 * it adds nothing to the loss), ids_restore[l] = l, ids_keep[r] = r, target and visible rows
 * zero.  The loss's divisor is then the number of 1s in the mask.
 * Returns 0, or -1 on an invalid argument. */
int32_t mae_oracle_prep_batch(const mae_oracle_prep_args* a, int32_t b_begin, int32_t b_end,
                              float* visible, uint8_t* mask, int32_t* ids_restore,
                              int32_t* ids_keep, float* target, int32_t* crop, uint8_t* valid);

/* ---- normalised-pixel loss and gradient (Sec. 3: official MAE objective) ---------------------- */
/* pred, target: [B,L,D] fp32 (target NOT yet per-patch normalised); mask [B,L]; num_masked = the
 * divisor M (masked patches of the whole batch).  loss_out: one double.  grad (nullable): [B,L,D]
 * fp32, the fp64 gradient rounded once; rows with mask 0 are +0.  that (nullable): [B,L,D]
 * doubles, the per-patch normalised target.  Returns 0 or -1. */
int32_t mae_oracle_normpix_loss(int32_t B, int32_t L, int32_t D, const float* pred,
                                const float* target, const uint8_t* mask, int64_t num_masked,
                                double eps, double grad_scale, double* loss_out, float* grad,
                                double* that);
/* Same objective against the image-normalised pixels themselves (no per-patch normalisation):
 * that = target. */
int32_t mae_oracle_pixel_loss(int32_t B, int32_t L, int32_t D, const float* pred,
                              const float* target, const uint8_t* mask, int64_t num_masked,
                              double grad_scale, double* loss_out, float* grad);

/* ---- progressive schedules (Sec. 5.2 Table 7, Sec. 5.3 Table 9) ------------------------------- */
/* Pretraining scheme 1..6, stage 1..3 -> training resolution and masking ratio.  Returns 0, or
 * -1 for an unknown scheme or stage. */
int32_t mae_oracle_pretrain_stage(int32_t scheme, int32_t stage, int32_t* res, double* mask_ratio);
/* Finetuning scheme (1, 3; 10 = the table's "1-", 11 = "1+"), stage 1..3 -> resolution, the bounds
 * sigma-, sigma+ of the crop's side ratio (the crop's area fraction is their square) and the
 * stage's augmentation (aug, nullable: 1 = "3 Aug", 2 = "3 Aug+"). */
int32_t mae_oracle_finetune_stage(int32_t scheme, int32_t stage, int32_t* res, double* sigma_lo,
                                  double* sigma_hi, int32_t* aug);
/* Stage (1-based) that epoch `epoch` (0-based) falls in when the stages last lengths[0..n) epochs;
 * epochs past the end belong to the last stage.  Returns -1 on bad arguments. */
int32_t mae_oracle_stage_of_epoch(int32_t epoch, const int32_t* lengths, int32_t n);

/* ---- patch embedding of the visible tokens (Sec. 2: the encoder sees only the visible patches;
 * Sec. 5: "linear patch embeddings" of the ViT) -------------------------------------------------
 * tokens[b, r, e] = sum_d visible[b, r, d] * weight[e, d] + bias[e] + pos[ids_keep[b, r], e].
 * visible [B,K,D], weight [E,D] (columns in the patch's element order: row, column, channel),
 * bias [E] (nullable), pos [L,E] (nullable; row l = positional embedding of patch l),
 * tokens [B,K,E] doubles.  Returns 0 or -1. */
int32_t mae_oracle_patch_embed(int32_t B, int32_t K, int32_t D, int32_t E, int32_t L,
                               const float* visible, const int32_t* ids_keep, const float* weight,
                               const float* bias, const float* pos, double* tokens);

/* ---- baseline JPEG decoding (Sec. 4.1 "Crop Decode": the loader decodes JPEG files; the paper's
 * contribution is to decode only the region that the crop needs) --------------------------------
 * Plain sequential decoder of what the dataset writer produces: baseline DCT (SOF0), 8 bits, three
 * components (YCbCr, JFIF), luma sampling 1x1 or 2x2 with 1x1 chroma, Huffman tables and
 * quantisation tables as found in the file, optional restart intervals.  Written from the
 * published standard (ITU-T T.81) and JFIF; the choices the standard leaves open are fixed here:
 *   - inverse DCT: separable, 13-bit fixed-point cosines, first pass rounded to 3 fractional
 *     bits, coefficients and first-pass values clamped to +-32767 (mae_oracle_idct8x8);
 *   - chroma upsampling: each chroma sample is repeated over the pixels it covers;
 *   - colour: 16-bit fixed-point JFIF matrix, floor after adding one half (mae_oracle_ycc_to_rgb).
 * The whole image is decoded; cropping is somebody else's business.  Returns 0, or a negative
 * code: -1 bad arguments, -2 not a baseline 3-component JPEG of the supported sampling,
 * -3 truncated or corrupt stream. */
int32_t mae_oracle_jpeg_info(const uint8_t* data, int64_t n, int32_t* H, int32_t* W,
                             int32_t* luma_h, int32_t* luma_v, int32_t* restart_interval);
/* rgb: H x W x 3, rows tightly packed. */
int32_t mae_oracle_jpeg_decode(const uint8_t* data, int64_t n, uint8_t* rgb);
/* The same image before the colour conversion: Y, Cb, Cr per pixel (chroma already repeated). */
int32_t mae_oracle_jpeg_decode_ycc(const uint8_t* data, int64_t n, uint8_t* ycc);
/* Dequantised coefficients in natural (row-major, [v][u]) order -> 64 samples, level-shifted by
 * +128 and clamped to 0..255, row-major. */
void mae_oracle_idct8x8(const int32_t coef[64], uint8_t out[64]);
void mae_oracle_ycc_to_rgb(int32_t y, int32_t cb, int32_t cr, uint8_t rgb[3]);
/* Canonical Huffman codes of a table given as the 16 counts of codes per length (DHT layout):
 * code and length of the i-th symbol in the table's order.  Returns the number of symbols. */
int32_t mae_oracle_huff_codes(const uint8_t counts[16], uint16_t* codes, uint8_t* lengths);

int32_t mae_oracle_threads(void);
/* Threads for the loops over samples and rows from now on (results do not depend on it). */
void mae_oracle_set_threads(int32_t n);

#ifdef __cplusplus
}
#endif
#endif
