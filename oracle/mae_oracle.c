/*
 * CPU oracle for the masked-autoencoder input pipeline.  TEST INFRASTRUCTURE ONLY -- see
 * mae_oracle.h.  Plain scalar C, fp64 arithmetic, no blocking or fusion: each function is the
 * definition of its step written out.  Build with -ffp-contract=off so that the crop-parameter
 * arithmetic is the sequence of correctly rounded +, -, *, /, sqrt that is written here.
 */
#include "mae_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------------------------------------
 * Random numbers.  The paper does not name a generator; the reading taken is a counter-based one
 * so that every draw is a pure function of (seed, batch, sample, stream, counter): the finaliser
 * of SplitMix64 applied to state + (n+1)*golden-gamma is the n-th output of that generator.
 * ---------------------------------------------------------------------------------------------- */
static const uint64_t GOLDEN_GAMMA = 0x9E3779B97F4A7C15ull;

uint64_t mae_oracle_mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

uint64_t mae_oracle_draw(uint64_t seed, uint64_t batch_index, uint32_t sample, uint32_t stream,
                         uint32_t ctr) {
  uint64_t k0 = mae_oracle_mix64(seed + GOLDEN_GAMMA);
  uint64_t k1 = mae_oracle_mix64(k0 + GOLDEN_GAMMA * (batch_index + 1));
  uint64_t w = ((uint64_t)sample << 32) | ((uint64_t)(stream & 0xFFu) << 24) |
               (uint64_t)(ctr & 0xFFFFFFu);
  return mae_oracle_mix64(k1 + GOLDEN_GAMMA * (w + 1));
}

static uint32_t draw_u32(uint64_t seed, uint64_t batch, uint32_t sample, uint32_t stream,
                         uint32_t ctr) {
  return (uint32_t)(mae_oracle_draw(seed, batch, sample, stream, ctr) >> 32);
}

/* uniform in [0,1) with 53 random bits; exact in fp64 */
static double draw_unit(uint64_t seed, uint64_t batch, uint32_t sample, uint32_t stream,
                        uint32_t ctr) {
  uint64_t u53 = mae_oracle_draw(seed, batch, sample, stream, ctr) >> 11;
  return (double)u53 * (1.0 / 9007199254740992.0);
}

/* ------------------------------------------------------------------------------------------------
 * RandomResizedCrop parameters (Sec. 5.1).  The area fraction is uniform on [scale_lo, scale_hi]
 * (the paper's sigma is its square root), the logarithm of the aspect ratio width/height is
 * uniform on [ln ratio_lo, ln ratio_hi].  The paper is silent on rounding, acceptance and the
 * fallback; the reading is the common one: up to ten proposals, sides rounded half-to-even, a
 * proposal is accepted when it fits inside the image, the corner is then uniform over the
 * positions that fit; after ten rejections the largest centred box whose ratio is inside the
 * range is taken.
 * ---------------------------------------------------------------------------------------------- */
double mae_oracle_exp_poly(double x) {
  double e = 1.0;
  for (int k = 13; k >= 1; --k) {
    double xe = x * e;
    double q = xe / (double)k;
    e = 1.0 + q;
  }
  return e;
}

void mae_oracle_rrc_proposal(int32_t H, int32_t W, float scale_lo, float scale_hi, float ratio_lo,
                             float ratio_hi, uint64_t seed, uint64_t batch_index, uint32_t sample,
                             int32_t attempt, int64_t out_hw[2]) {
  double lo = (double)scale_lo, hi = (double)scale_hi;
  double ln_lo = log((double)ratio_lo), ln_hi = log((double)ratio_hi);
  double area = (double)((int64_t)H * (int64_t)W);

  double u_scale = draw_unit(seed, batch_index, sample, 0u, (uint32_t)attempt);
  double u_ratio = draw_unit(seed, batch_index, sample, 1u, (uint32_t)attempt);
  double s = lo + (hi - lo) * u_scale;
  double T = area * s;
  double x = ln_lo + (ln_hi - ln_lo) * u_ratio;
  double r = mae_oracle_exp_poly(x);
  double cw = rint(sqrt(T * r));
  double ch = rint(sqrt(T / r));
  out_hw[0] = (int64_t)ch;
  out_hw[1] = (int64_t)cw;
}

int32_t mae_oracle_rrc_params(int32_t H, int32_t W, float scale_lo, float scale_hi, float ratio_lo,
                              float ratio_hi, uint64_t seed, uint64_t batch_index, uint32_t sample,
                              int32_t box[4]) {
  for (int32_t a = 0; a < 10; ++a) {
    int64_t hw[2];
    mae_oracle_rrc_proposal(H, W, scale_lo, scale_hi, ratio_lo, ratio_hi, seed, batch_index,
                            sample, a, hw);
    int64_t ch = hw[0], cw = hw[1];
    if (cw >= 1 && cw <= W && ch >= 1 && ch <= H) {
      uint64_t ut = draw_u32(seed, batch_index, sample, 2u, (uint32_t)a);
      uint64_t ul = draw_u32(seed, batch_index, sample, 3u, (uint32_t)a);
      /* uniform integer on 0 .. H-ch (resp. 0 .. W-cw): floor(u32 * n / 2^32) */
      int64_t top = (int64_t)((ut * (uint64_t)(H - ch + 1)) >> 32);
      int64_t left = (int64_t)((ul * (uint64_t)(W - cw + 1)) >> 32);
      box[0] = (int32_t)top;
      box[1] = (int32_t)left;
      box[2] = (int32_t)ch;
      box[3] = (int32_t)cw;
      return a + 1;
    }
  }
  /* fallback: centred box, ratio clamped into the range */
  double R = (double)W / (double)H;
  int64_t ch, cw;
  if (R < (double)ratio_lo) {
    cw = W;
    ch = (int64_t)rint((double)W / (double)ratio_lo);
  } else if (R > (double)ratio_hi) {
    ch = H;
    cw = (int64_t)rint((double)H * (double)ratio_hi);
  } else {
    ch = H;
    cw = W;
  }
  if (ch > H) ch = H;
  if (cw > W) cw = W;
  if (ch < 1) ch = 1;
  if (cw < 1) cw = 1;
  box[0] = (int32_t)((H - ch) / 2);
  box[1] = (int32_t)((W - cw) / 2);
  box[2] = (int32_t)ch;
  box[3] = (int32_t)cw;
  return 11;
}

/* ------------------------------------------------------------------------------------------------
 * Horizontal flip (App. B, first part of the "Simple" augmentation): a 24-bit uniform compared
 * with the probability in single precision.
 * ---------------------------------------------------------------------------------------------- */
int32_t mae_oracle_flip_bit(uint64_t seed, uint64_t batch_index, uint32_t sample, float flip_p) {
  uint32_t u24 = draw_u32(seed, batch_index, sample, 4u, 0u) >> 8;
  float u = (float)u24 * (1.0f / 16777216.0f);
  return u < flip_p ? 1 : 0;
}

/* ------------------------------------------------------------------------------------------------
 * Crop + resize (Sec. 4.1: crop, then resize the cropped region to the output size).  Filter is
 * not named in the paper; reading: bilinear, sample positions at pixel centres
 * (src = (o + 1/2) * crop_len / out_size - 1/2), two taps per axis, taps clamped to the crop box,
 * no prefilter, no rounding back to bytes.  The position is kept as the exact rational n / den.
 * ---------------------------------------------------------------------------------------------- */
void mae_oracle_resize_taps(int32_t out_size, int32_t crop_len, int32_t o, int32_t* i0, int32_t* i1,
                            double* f) {
  int64_t n = (2 * (int64_t)o + 1) * (int64_t)crop_len - (int64_t)out_size;
  int64_t den = 2 * (int64_t)out_size;
  if (n <= 0) {
    *i0 = 0;
    *f = 0.0;
  } else {
    *i0 = (int32_t)(n / den);
    *f = (double)(n % den) / (double)den;
  }
  *i1 = (*i0 + 1 < crop_len) ? *i0 + 1 : crop_len - 1;
}

void mae_oracle_crop_resize(const uint8_t* img, int32_t H, int32_t W, const int32_t box[4],
                            int32_t S, int32_t flip, double* out) {
  (void)H;
  int32_t top = box[0], left = box[1], ch = box[2], cw = box[3];
  for (int32_t oy = 0; oy < S; ++oy) {
    int32_t y0, y1;
    double fy;
    mae_oracle_resize_taps(S, ch, oy, &y0, &y1, &fy);
    for (int32_t ox = 0; ox < S; ++ox) {
      /* a flipped output column shows what the mirrored column would have shown */
      int32_t sx = flip ? (S - 1 - ox) : ox;
      int32_t x0, x1;
      double fx;
      mae_oracle_resize_taps(S, cw, sx, &x0, &x1, &fx);
      for (int32_t c = 0; c < 3; ++c) {
        double a00 = img[((int64_t)(top + y0) * W + (left + x0)) * 3 + c];
        double a01 = img[((int64_t)(top + y0) * W + (left + x1)) * 3 + c];
        double a10 = img[((int64_t)(top + y1) * W + (left + x0)) * 3 + c];
        double a11 = img[((int64_t)(top + y1) * W + (left + x1)) * 3 + c];
        double rt = a00 + fx * (a01 - a00);
        double rb = a10 + fx * (a11 - a10);
        out[((int64_t)oy * S + ox) * 3 + c] = rt + fy * (rb - rt);
      }
    }
  }
}

/* ------------------------------------------------------------------------------------------------
 * Normalisation (App. B): byte range to [0,1], then mean / standard deviation per channel.
 * ---------------------------------------------------------------------------------------------- */
double mae_oracle_normalise(double v, double mean, double std) { return (v / 255.0 - mean) / std; }

/* ------------------------------------------------------------------------------------------------
 * Patchify (Sec. 3, ViT-B/16).  Patches in row-major order over the grid; inside a patch the
 * element order is (row, column, channel), which is the order the pixels have in memory.
 * ---------------------------------------------------------------------------------------------- */
void mae_oracle_patchify(const double* img, int32_t S, int32_t p, double* out) {
  int32_t G = S / p;
  int64_t D = 3 * (int64_t)p * p;
  for (int32_t y = 0; y < S; ++y)
    for (int32_t x = 0; x < S; ++x)
      for (int32_t c = 0; c < 3; ++c) {
        int64_t l = (int64_t)(y / p) * G + (x / p);
        int64_t e = ((int64_t)(y % p) * p + (x % p)) * 3 + c;
        out[l * D + e] = img[((int64_t)y * S + x) * 3 + c];
      }
}

/* ------------------------------------------------------------------------------------------------
 * Random masking (Sec. 2: the encoder drops the masked patches; Sec. 5.3: the masking ratio is
 * the fraction of patches that is masked).  One noise key per patch; the K patches with the
 * smallest keys stay visible; equal keys are ordered by patch index.  The rank of a patch is the
 * number of patches that come before it -- written as that count, with no sorting routine.
 * ---------------------------------------------------------------------------------------------- */
int32_t mae_oracle_num_keep(int32_t L, double mask_ratio) {
  return (int32_t)floor((double)L * (1.0 - mask_ratio));
}

void mae_oracle_mask(uint64_t seed, uint64_t batch_index, uint32_t sample, int32_t L, int32_t K,
                     int32_t noise_bits, int32_t* ids_restore, int32_t* ids_keep, uint8_t* mask) {
  uint32_t* key = (uint32_t*)malloc(sizeof(uint32_t) * (size_t)L);
  for (int32_t l = 0; l < L; ++l) {
    uint32_t u = draw_u32(seed, batch_index, sample, 5u, (uint32_t)l);
    key[l] = (noise_bits >= 32) ? u : (u >> (32 - noise_bits));
  }
  for (int32_t l = 0; l < L; ++l) {
    int32_t rank = 0;
    for (int32_t j = 0; j < L; ++j)
      if (key[j] < key[l] || (key[j] == key[l] && j < l)) ++rank;
    if (ids_restore) ids_restore[l] = rank;
    if (mask) mask[l] = (rank >= K) ? 1 : 0;
    if (ids_keep && rank < K) ids_keep[rank] = l;
  }
  free(key);
}

/* ------------------------------------------------------------------------------------------------
 * Finetuning augmentation "3 Aug" / "3 Aug+" (Sec. 3, Sec. 4.4, Table 7).  The paper names the
 * procedure and cites it; it prints no parameter.  Readings: the operations act on the 8-bit
 * image that crop + resize produce (the cited procedure is defined on 8-bit images: a
 * solarisation threshold only means something there), so the resized crop is first rounded to
 * bytes -- exactly, the bilinear value being the rational num / den^2 with den = 2 S.  One of the
 * three operations is drawn per image with equal probability.  After it nothing is rounded
 * again.  "ColorJitter (0.3)" is brightness, contrast and saturation factors uniform on
 * [0.7, 1.3], applied in that order.
 * ---------------------------------------------------------------------------------------------- */
static void taps_exact(int32_t out_size, int32_t crop_len, int32_t o, int32_t* i0, int32_t* i1,
                       int64_t* r) {
  int64_t n = (int64_t)crop_len * (2 * (int64_t)o + 1) - (int64_t)out_size;  /* 2 S src */
  int64_t den = (int64_t)out_size * 2;
  if (n <= 0) {
    *i0 = 0;
    *r = 0;
  } else {
    *i0 = (int32_t)(n / den); /* whole source pixels */
    *r = n % den;
  }
  *i1 = (*i0 < crop_len - 1) ? *i0 + 1 : crop_len - 1;
}

void mae_oracle_resize_u8(const uint8_t* img, int32_t H, int32_t W, const int32_t box[4], int32_t S,
                          int32_t flip, uint8_t* out) {
  (void)H;
  int32_t top = box[0], left = box[1], ch = box[2], cw = box[3];
  int64_t den = 2 * (int64_t)S;
  for (int32_t oy = 0; oy < S; ++oy) {
    int32_t y0, y1;
    int64_t ry;
    taps_exact(S, ch, oy, &y0, &y1, &ry);
    for (int32_t ox = 0; ox < S; ++ox) {
      int32_t sx = flip ? (S - ox - 1) : ox; /* mirrored column */
      int32_t x0, x1;
      int64_t rx;
      taps_exact(S, cw, sx, &x0, &x1, &rx);
      for (int32_t c = 0; c < 3; ++c) {
        int64_t a00 = img[((int64_t)(top + y0) * W + (left + x0)) * 3 + c];
        int64_t a01 = img[((int64_t)(top + y0) * W + (left + x1)) * 3 + c];
        int64_t a10 = img[((int64_t)(top + y1) * W + (left + x0)) * 3 + c];
        int64_t a11 = img[((int64_t)(top + y1) * W + (left + x1)) * 3 + c];
        /* value = num / den^2 */
        int64_t num = (den - ry) * ((den - rx) * a00 + rx * a01) + ry * ((den - rx) * a10 + rx * a11);
        out[((int64_t)oy * S + ox) * 3 + c] = (uint8_t)((2 * num + den * den) / (2 * den * den));
      }
    }
  }
}

void mae_oracle_aug_params(uint64_t seed, uint64_t batch_index, uint32_t sample, double jitter,
                           int32_t* op, double* sigma, double bcs[3]) {
  int32_t k = (int32_t)floor(3.0 * draw_unit(seed, batch_index, sample, 6u, 0u));
  *op = k > 2 ? 2 : k;
  *sigma = 0.1 + 1.9 * draw_unit(seed, batch_index, sample, 7u, 0u);
  for (uint32_t j = 0; j < 3; ++j)
    bcs[j] = 1.0 + jitter * (2.0 * draw_unit(seed, batch_index, sample, 8u + j, 0u) - 1.0);
}

int32_t mae_oracle_gray(int32_t r, int32_t g, int32_t b) {
  return (299 * r + 587 * g + 114 * b + 500) / 1000;
}

int32_t mae_oracle_solarise(int32_t v) { return v >= 128 ? 255 - v : v; }

int32_t mae_oracle_blur_weights(double sigma, double* w) {
  int32_t radius = (int32_t)ceil(3.0 * sigma);
  if (radius < 1) radius = 1;
  double sum = 0.0;
  for (int32_t k = -radius; k <= radius; ++k) {
    w[k + radius] = exp(-(double)(k * k) / (2.0 * sigma * sigma));
    sum += w[k + radius];
  }
  for (int32_t k = 0; k <= 2 * radius; ++k) w[k] /= sum;
  return radius;
}

static int32_t clampi(int32_t v, int32_t lo, int32_t hi) { return v < lo ? lo : (v > hi ? hi : v); }

void mae_oracle_three_aug(const uint8_t* u8, int32_t S, int32_t op, double sigma, double* out) {
  int64_t n = (int64_t)S * S;
  if (op == 0) {
    for (int64_t i = 0; i < n; ++i) {
      double g = (double)mae_oracle_gray(u8[i * 3], u8[i * 3 + 1], u8[i * 3 + 2]);
      out[i * 3] = out[i * 3 + 1] = out[i * 3 + 2] = g;
    }
  } else if (op == 1) {
    for (int64_t i = 0; i < n * 3; ++i) out[i] = (double)mae_oracle_solarise(u8[i]);
  } else {
    double w[13];
    int32_t radius = mae_oracle_blur_weights(sigma, w);
    double* tmp = (double*)malloc(sizeof(double) * (size_t)n * 3);
    /* along y, then along x; border pixels repeated */
    for (int32_t y = 0; y < S; ++y)
      for (int32_t x = 0; x < S; ++x)
        for (int32_t c = 0; c < 3; ++c) {
          double acc = 0.0;
          for (int32_t k = -radius; k <= radius; ++k)
            acc += w[k + radius] * (double)u8[((int64_t)clampi(y + k, 0, S - 1) * S + x) * 3 + c];
          tmp[((int64_t)y * S + x) * 3 + c] = acc;
        }
    for (int32_t y = 0; y < S; ++y)
      for (int32_t x = 0; x < S; ++x)
        for (int32_t c = 0; c < 3; ++c) {
          double acc = 0.0;
          for (int32_t k = -radius; k <= radius; ++k)
            acc += w[k + radius] * tmp[((int64_t)y * S + clampi(x + k, 0, S - 1)) * 3 + c];
          out[((int64_t)y * S + x) * 3 + c] = acc;
        }
    free(tmp);
  }
}

static double clampd(double v) { return v < 0.0 ? 0.0 : (v > 255.0 ? 255.0 : v); }
static double luma(const double* px) { return 0.299 * px[0] + 0.587 * px[1] + 0.114 * px[2]; }

void mae_oracle_color_jitter(double* img, int32_t S, const double bcs[3]) {
  int64_t n = (int64_t)S * S;
  for (int64_t i = 0; i < n * 3; ++i) img[i] = clampd(img[i] * bcs[0]);
  double mean = 0.0;
  for (int64_t i = 0; i < n; ++i) mean += luma(img + i * 3);
  mean /= (double)n;
  for (int64_t i = 0; i < n * 3; ++i) img[i] = clampd(bcs[1] * img[i] + (1.0 - bcs[1]) * mean);
  for (int64_t i = 0; i < n; ++i) {
    double g = luma(img + i * 3);
    for (int32_t c = 0; c < 3; ++c)
      img[i * 3 + c] = clampd(bcs[2] * img[i * 3 + c] + (1.0 - bcs[2]) * g);
  }
}

/* ------------------------------------------------------------------------------------------------
 * Whole input pipeline.
 * ---------------------------------------------------------------------------------------------- */
int32_t mae_oracle_prep_batch(const mae_oracle_prep_args* a, int32_t b_begin, int32_t b_end,
                              float* visible, uint8_t* mask, int32_t* ids_restore,
                              int32_t* ids_keep, float* target, int32_t* crop, uint8_t* valid) {
  if (!a || !a->images || !a->offsets || !a->heights || !a->widths) return -1;
  if (b_begin < 0 || b_end > a->B || b_begin > b_end) return -1;
  int32_t S = a->out_size, p = a->patch, K = a->num_keep;
  if (S < 1 || p < 1 || S % p != 0) return -1;
  int32_t G = S / p, L = G * G;
  int64_t D = 3 * (int64_t)p * p;
  if (K < 1 || K > L) return -1;
  if (a->noise_bits < 1 || a->noise_bits > 32) return -1;
  if (a->aug_mode < 0 || a->aug_mode > 2) return -1;

  int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
  for (int32_t b = b_begin; b < b_end; ++b) {
    int64_t n = b - b_begin;
    int32_t H = a->heights[b], W = a->widths[b];
    const uint8_t* img = a->images + a->offsets[b];

    /* A sample that cannot be read (empty or oversized geometry, or an image that does not lie
     * inside the buffer) takes no part in training: nothing of it is kept or masked, so its mask
     * row is all 0, the patch order is the identity, and its pixels are zeros. */
    int usable = H >= 1 && W >= 1 && H <= 32767 && W <= 32767 && a->offsets[b] >= 0;
    if (usable && a->images_bytes > 0)
      usable = a->offsets[b] + (int64_t)H * W * 3 <= a->images_bytes;
    if (valid) valid[n] = (uint8_t)usable;
    if (!usable) {
      if (crop) memset(crop + n * 5, 0, sizeof(int32_t) * 5);
      for (int32_t l = 0; l < L; ++l) {
        if (ids_restore) ids_restore[n * L + l] = l;
        if (mask) mask[n * L + l] = 0;
        if (ids_keep && l < K) ids_keep[n * K + l] = l;
      }
      if (target) memset(target + n * L * D, 0, sizeof(float) * (size_t)L * (size_t)D);
      if (visible) memset(visible + n * K * D, 0, sizeof(float) * (size_t)K * (size_t)D);
      continue;
    }

    int32_t box[4];
    mae_oracle_rrc_params(H, W, a->scale_lo, a->scale_hi, a->ratio_lo, a->ratio_hi, a->seed,
                          a->batch_index, (uint32_t)b, box);
    int32_t flip = mae_oracle_flip_bit(a->seed, a->batch_index, (uint32_t)b, a->flip_p);
    if (crop) {
      memcpy(crop + n * 5, box, sizeof(box));
      crop[n * 5 + 4] = flip;
    }

    int32_t* restore = (int32_t*)malloc(sizeof(int32_t) * (size_t)L);
    int32_t* keep = (int32_t*)malloc(sizeof(int32_t) * (size_t)K);
    uint8_t* msk = (uint8_t*)malloc((size_t)L);
    mae_oracle_mask(a->seed, a->batch_index, (uint32_t)b, L, K, a->noise_bits, restore, keep, msk);
    if (ids_restore) memcpy(ids_restore + n * L, restore, sizeof(int32_t) * (size_t)L);
    if (ids_keep) memcpy(ids_keep + n * K, keep, sizeof(int32_t) * (size_t)K);
    if (mask) memcpy(mask + n * L, msk, (size_t)L);

    if (visible || target) {
      double* resized = (double*)malloc(sizeof(double) * (size_t)S * S * 3);
      double* patches = (double*)malloc(sizeof(double) * (size_t)L * D);
      if (!resized || !patches) {
        failed = 1;
      } else {
        if (a->aug_mode == 0) {
          mae_oracle_crop_resize(img, H, W, box, S, flip, resized);
        } else {
          uint8_t* u8 = (uint8_t*)malloc((size_t)S * S * 3);
          int32_t op;
          double sigma, bcs[3];
          mae_oracle_resize_u8(img, H, W, box, S, flip, u8);
          mae_oracle_aug_params(a->seed, a->batch_index, (uint32_t)b, (double)a->jitter, &op,
                                &sigma, bcs);
          mae_oracle_three_aug(u8, S, op, sigma, resized);
          if (a->aug_mode == 2) mae_oracle_color_jitter(resized, S, bcs);
          free(u8);
        }
        for (int64_t i = 0; i < (int64_t)S * S; ++i)
          for (int32_t c = 0; c < 3; ++c)
            resized[i * 3 + c] =
                mae_oracle_normalise(resized[i * 3 + c], (double)a->mean[c], (double)a->std[c]);
        mae_oracle_patchify(resized, S, p, patches);
        if (target)
          for (int64_t i = 0; i < (int64_t)L * D; ++i) target[n * L * D + i] = (float)patches[i];
        if (visible)
          for (int32_t r = 0; r < K; ++r)
            for (int64_t e = 0; e < D; ++e)
              visible[(n * K + r) * D + e] = (float)patches[(int64_t)keep[r] * D + e];
      }
      free(resized);
      free(patches);
    }
    free(restore);
    free(keep);
    free(msk);
  }
  return failed ? -1 : 0;
}

/* ------------------------------------------------------------------------------------------------
 * Normalised-pixel reconstruction loss (Sec. 3 adopts the official MAE objective; its formula is
 * not printed in the paper).  For every patch row t[0..D): mu = mean, var = sum (t-mu)^2 / (D-1),
 * that = (t - mu) / sqrt(var + eps).  Row loss = mean over the D elements of (pred - that)^2.
 * loss = sum of the row losses of masked rows / M.  d loss / d pred = 2 (pred - that) / (D M) on
 * masked rows, zero elsewhere; multiplied by the upstream factor grad_scale.
 * ---------------------------------------------------------------------------------------------- */
int32_t mae_oracle_normpix_loss(int32_t B, int32_t L, int32_t D, const float* pred,
                                const float* target, const uint8_t* mask, int64_t num_masked,
                                double eps, double grad_scale, double* loss_out, float* grad,
                                double* that) {
  if (B < 1 || L < 1 || D < 2 || !pred || !target || !mask || !loss_out || num_masked < 1)
    return -1;
  int64_t rows = (int64_t)B * L;
  double M = (double)num_masked;
  double* row_losses = (double*)malloc(sizeof(double) * (size_t)rows);
  if (!row_losses) return -1;
  /* rows are independent; the sum over rows below is taken in row order */
#pragma omp parallel for schedule(static)
  for (int64_t row = 0; row < rows; ++row) {
    const float* t = target + row * D;
    const float* q = pred + row * D;
    double mu = 0.0;
    for (int32_t e = 0; e < D; ++e) mu += (double)t[e];
    mu /= (double)D;
    double ss = 0.0;
    for (int32_t e = 0; e < D; ++e) ss += ((double)t[e] - mu) * ((double)t[e] - mu);
    double var = ss / (double)(D - 1);
    double sd = sqrt(var + eps);
    double row_loss = 0.0;
    for (int32_t e = 0; e < D; ++e) {
      double th = ((double)t[e] - mu) / sd;
      double diff = (double)q[e] - th;
      if (that) that[row * D + e] = th;
      row_loss += diff * diff;
      if (grad)
        grad[row * D + e] =
            mask[row] ? (float)(grad_scale * 2.0 * diff / ((double)D * M)) : 0.0f;
    }
    row_losses[row] = row_loss / (double)D;
  }
  double total = 0.0;
  for (int64_t row = 0; row < rows; ++row)
    if (mask[row]) total += row_losses[row];
  free(row_losses);
  *loss_out = total / M;
  return 0;
}

/* The un-normalised variant of the objective: the target is the image-normalised patch itself. */
int32_t mae_oracle_pixel_loss(int32_t B, int32_t L, int32_t D, const float* pred,
                              const float* target, const uint8_t* mask, int64_t num_masked,
                              double grad_scale, double* loss_out, float* grad) {
  if (B < 1 || L < 1 || D < 1 || !pred || !target || !mask || !loss_out || num_masked < 1)
    return -1;
  int64_t rows = (int64_t)B * L;
  double M = (double)num_masked;
  double total = 0.0;
  for (int64_t row = 0; row < rows; ++row) {
    double row_loss = 0.0;
    for (int32_t e = 0; e < D; ++e) {
      double diff = (double)pred[row * D + e] - (double)target[row * D + e];
      row_loss += diff * diff;
      if (grad)
        grad[row * D + e] =
            mask[row] ? (float)(grad_scale * 2.0 * diff / ((double)D * M)) : 0.0f;
    }
    if (mask[row]) total += row_loss / (double)D;
  }
  *loss_out = total / M;
  return 0;
}

/* ------------------------------------------------------------------------------------------------
 * Progressive schedules.  Sec. 5.3, Table 9: six pretraining schemes of three stages, each stage a
 * training resolution and a masking ratio.  Sec. 5.2, Table 7: finetuning schemes of three stages,
 * each a resolution and the range of the crop's side ratio sigma.
 * ---------------------------------------------------------------------------------------------- */
int32_t mae_oracle_pretrain_stage(int32_t scheme, int32_t stage, int32_t* res, double* mask_ratio) {
  if (scheme < 1 || scheme > 6 || stage < 1 || stage > 3 || !res || !mask_ratio) return -1;
  static const int32_t R[6][3] = {
      {160, 192, 224},  /* 1: resolution and masking ratio both grow            */
      {160, 192, 224},  /* 2: resolution grows, ratio fixed                     */
      {224, 192, 160},  /* 3: resolution shrinks                                */
      {160, 192, 224},  /* 4: resolution grows, ratio grows from the default    */
      {224, 192, 224},  /* 5: palindrome                                        */
      {224, 192, 224},  /* 6: palindrome, harder last stage                     */
  };
  static const double Mr[6][3] = {
      {0.50, 0.66, 0.75}, {0.75, 0.75, 0.75}, {0.75, 0.75, 0.75},
      {0.75, 0.80, 0.85}, {0.75, 0.75, 0.75}, {0.75, 0.75, 0.85},
  };
  *res = R[scheme - 1][stage - 1];
  *mask_ratio = Mr[scheme - 1][stage - 1];
  return 0;
}

int32_t mae_oracle_finetune_stage(int32_t scheme, int32_t stage, int32_t* res, double* sigma_lo,
                                  double* sigma_hi, int32_t* aug) {
  /* scheme: 1, 3, and 10 / 11 for the table's "1-" / "1+" */
  if ((scheme != 1 && scheme != 3 && scheme != 10 && scheme != 11) || stage < 1 || stage > 3 ||
      !res || !sigma_lo || !sigma_hi)
    return -1;
  static const int32_t R[3] = {160, 192, 224};
  static const double hi3[3] = {0.68, 0.84, 1.0};
  *res = R[stage - 1];
  *sigma_lo = 0.28;
  *sigma_hi = scheme == 3 ? hi3[stage - 1] : 1.0;
  /* aug column: 1 = "3 Aug", 2 = "3 Aug+".  Schemes 1 and 3 strengthen it in the last stage;
   * "1-" never does, "1+" uses the stronger one throughout. */
  if (aug) {
    if (scheme == 10) *aug = 1;
    else if (scheme == 11) *aug = 2;
    else *aug = stage == 3 ? 2 : 1;
  }
  return 0;
}

int32_t mae_oracle_stage_of_epoch(int32_t epoch, const int32_t* lengths, int32_t n) {
  if (epoch < 0 || !lengths || n < 1) return -1;
  int64_t end = 0;
  for (int32_t s = 0; s < n; ++s) {
    if (lengths[s] < 0) return -1;
    end += lengths[s];
    if (epoch < end) return s + 1;
  }
  return n;
}

/* ------------------------------------------------------------------------------------------------
 * Patch embedding of the visible tokens: the ViT's linear map of each flattened patch plus the
 * positional embedding of the patch's place in the grid (Sec. 2, Sec. 5).
 * ---------------------------------------------------------------------------------------------- */
int32_t mae_oracle_patch_embed(int32_t B, int32_t K, int32_t D, int32_t E, int32_t L,
                               const float* visible, const int32_t* ids_keep, const float* weight,
                               const float* bias, const float* pos, double* tokens) {
  if (B < 1 || K < 1 || D < 1 || E < 1 || L < 1 || !visible || !weight || !tokens) return -1;
  if (pos && !ids_keep) return -1;
  int bad = 0;
#pragma omp parallel for schedule(static)
  for (int64_t row = 0; row < (int64_t)B * K; ++row) {
    const float* v = visible + row * D;
    int32_t l = ids_keep ? ids_keep[row] : 0;
    if (pos && (l < 0 || l >= L)) {
      bad = 1;
      continue;
    }
    for (int32_t e = 0; e < E; ++e) {
      double acc = 0.0;
      for (int32_t d = 0; d < D; ++d) acc += (double)v[d] * (double)weight[(int64_t)e * D + d];
      if (bias) acc += (double)bias[e];
      if (pos) acc += (double)pos[(int64_t)l * E + e];
      tokens[row * E + e] = acc;
    }
  }
  return bad ? -1 : 0;
}

/* ------------------------------------------------------------------------------------------------
 * Baseline JPEG (ITU-T T.81, JFIF).  Sec. 4.1 of the paper speeds up the loader by decoding only
 * the crop; what a decoder computes is fixed by the standard up to the accuracy of the inverse
 * DCT, the chroma upsampling filter and the colour arithmetic -- those three are fixed in the
 * header of this library.  Everything here is the sequential procedure of the standard's Annex F
 * written out: marker segments, canonical Huffman codes, DC prediction, zero runs, zig-zag.
 * ---------------------------------------------------------------------------------------------- */
static const uint8_t ZIGZAG[64] = {
    0,  1,  8,  16, 9,  2,  3,  10, 17, 24, 32, 25, 18, 11, 4,  5,  12, 19, 26, 33, 40, 48,
    41, 34, 27, 20, 13, 6,  7,  14, 21, 28, 35, 42, 49, 56, 57, 50, 43, 36, 29, 22, 15, 23,
    30, 37, 44, 51, 58, 59, 52, 45, 38, 31, 39, 46, 53, 60, 61, 54, 47, 55, 62, 63};

typedef struct {
  uint8_t counts[16];
  uint8_t symbols[256];
  int32_t nsym;
  int32_t first_code[17]; /* code of the first symbol of each length */
  int32_t first_index[17];
} huff_table;

typedef struct {
  int32_t H, W, ncomp;
  int32_t hs[3], vs[3], tq[3], td[3], ta[3], cid[3];
  uint16_t q[4][64]; /* zig-zag order, as stored */
  int32_t have_q[4];
  huff_table dc[4], ac[4];
  int32_t have_dc[4], have_ac[4];
  int32_t restart;
  int64_t scan; /* offset of the first entropy-coded byte */
} jpeg_header;

static void huff_prepare(huff_table* t) {
  int32_t code = 0, index = 0;
  for (int32_t len = 1; len <= 16; ++len) {
    t->first_code[len] = code;
    t->first_index[len] = index;
    code += t->counts[len - 1];
    index += t->counts[len - 1];
    code <<= 1;
  }
  t->nsym = index;
}

int32_t mae_oracle_huff_codes(const uint8_t counts[16], uint16_t* codes, uint8_t* lengths) {
  int32_t code = 0, i = 0;
  for (int32_t len = 1; len <= 16; ++len) {
    for (int32_t j = 0; j < counts[len - 1]; ++j) {
      codes[i] = (uint16_t)code++;
      lengths[i++] = (uint8_t)len;
    }
    code <<= 1;
  }
  return i;
}

static int32_t be16(const uint8_t* p) { return (p[0] << 8) | p[1]; }

static int32_t jpeg_parse(const uint8_t* d, int64_t n, jpeg_header* h) {
  memset(h, 0, sizeof(*h));
  if (n < 4 || d[0] != 0xFF || d[1] != 0xD8) return -2;
  int64_t pos = 2;
  int32_t have_frame = 0;
  for (;;) {
    if (pos + 4 > n) return -3;
    if (d[pos] != 0xFF) return -3;
    int32_t m = d[pos + 1];
    if (m == 0xFF) { /* fill byte */
      ++pos;
      continue;
    }
    int32_t len = be16(d + pos + 2);
    if (len < 2 || pos + 2 + len > n) return -3;
    const uint8_t* s = d + pos + 4;
    int32_t body = len - 2;
    if (m == 0xDB) { /* quantisation tables */
      int32_t o = 0;
      while (o < body) {
        int32_t pq = s[o] >> 4, tq = s[o] & 15;
        if (pq != 0 || tq > 3 || o + 65 > body) return -2;
        for (int32_t k = 0; k < 64; ++k) h->q[tq][k] = s[o + 1 + k];
        h->have_q[tq] = 1;
        o += 65;
      }
    } else if (m == 0xC0) { /* baseline frame */
      if (body < 6) return -3;
      if (s[0] != 8) return -2;
      h->H = be16(s + 1);
      h->W = be16(s + 3);
      h->ncomp = s[5];
      if (h->ncomp != 3 || body < 6 + 9 || h->H < 1 || h->W < 1) return -2;
      for (int32_t c = 0; c < 3; ++c) {
        h->cid[c] = s[6 + 3 * c];
        h->hs[c] = s[7 + 3 * c] >> 4;
        h->vs[c] = s[7 + 3 * c] & 15;
        h->tq[c] = s[8 + 3 * c];
        if (h->tq[c] > 3) return -2;
      }
      if (h->hs[1] != 1 || h->vs[1] != 1 || h->hs[2] != 1 || h->vs[2] != 1) return -2;
      if (!((h->hs[0] == 1 && h->vs[0] == 1) || (h->hs[0] == 2 && h->vs[0] == 2))) return -2;
      have_frame = 1;
    } else if (m >= 0xC1 && m <= 0xCF && m != 0xC4 && m != 0xC8 && m != 0xCC) {
      return -2; /* any other kind of frame */
    } else if (m == 0xC4) { /* Huffman tables */
      int32_t o = 0;
      while (o < body) {
        if (o + 17 > body) return -3;
        int32_t tc = s[o] >> 4, th = s[o] & 15;
        if (tc > 1 || th > 3) return -2;
        huff_table* t = tc ? &h->ac[th] : &h->dc[th];
        int32_t total = 0;
        for (int32_t i = 0; i < 16; ++i) {
          t->counts[i] = s[o + 1 + i];
          total += t->counts[i];
        }
        if (total > 256 || o + 17 + total > body) return -3;
        for (int32_t i = 0; i < total; ++i) t->symbols[i] = s[o + 17 + i];
        huff_prepare(t);
        if (tc) h->have_ac[th] = 1; else h->have_dc[th] = 1;
        o += 17 + total;
      }
    } else if (m == 0xDD) {
      if (body < 2) return -3;
      h->restart = be16(s);
    } else if (m == 0xDA) { /* start of scan */
      if (!have_frame || body < 1 + 6 + 3 || s[0] != 3) return -2;
      for (int32_t c = 0; c < 3; ++c) {
        if (s[1 + 2 * c] != h->cid[c]) return -2; /* components in frame order */
        h->td[c] = s[2 + 2 * c] >> 4;
        h->ta[c] = s[2 + 2 * c] & 15;
        if (h->td[c] > 3 || h->ta[c] > 3 || !h->have_dc[h->td[c]] || !h->have_ac[h->ta[c]] ||
            !h->have_q[h->tq[c]])
          return -2;
      }
      if (s[7] != 0 || s[8] != 63) return -2; /* sequential: whole spectrum in one scan */
      h->scan = pos + 2 + len;
      return 0;
    } else if (m == 0xD9) {
      return -3;
    }
    pos += 2 + len;
  }
}

int32_t mae_oracle_jpeg_info(const uint8_t* data, int64_t n, int32_t* H, int32_t* W,
                             int32_t* luma_h, int32_t* luma_v, int32_t* restart_interval) {
  if (!data) return -1;
  jpeg_header h;
  int32_t rc = jpeg_parse(data, n, &h);
  if (rc) return rc;
  if (H) *H = h.H;
  if (W) *W = h.W;
  if (luma_h) *luma_h = h.hs[0];
  if (luma_v) *luma_v = h.vs[0];
  if (restart_interval) *restart_interval = h.restart;
  return 0;
}

/* entropy-coded segment reader: bytes after the scan header, 0xFF00 stands for 0xFF, any other
 * marker ends the data (zero bits are supplied beyond it) */
typedef struct {
  const uint8_t* d;
  int64_t n, pos;
  uint32_t acc;
  int32_t nbits;
  int32_t hit_marker;
} bit_reader;

static int32_t next_bit(bit_reader* r) {
  if (r->nbits == 0) {
    uint32_t byte = 0;
    if (!r->hit_marker && r->pos < r->n) {
      byte = r->d[r->pos];
      if (byte == 0xFF) {
        if (r->pos + 1 < r->n && r->d[r->pos + 1] == 0x00) {
          r->pos += 2;
        } else {
          r->hit_marker = 1;
          byte = 0;
        }
      } else {
        r->pos += 1;
      }
    }
    r->acc = byte;
    r->nbits = 8;
  }
  r->nbits -= 1;
  return (int32_t)((r->acc >> r->nbits) & 1u);
}

static int32_t receive(bit_reader* r, int32_t s) {
  int32_t v = 0;
  for (int32_t i = 0; i < s; ++i) v = (v << 1) | next_bit(r);
  return v;
}

static int32_t extend(int32_t v, int32_t s) {
  return (s && v < (1 << (s - 1))) ? v - (1 << s) + 1 : v;
}

static int32_t huff_decode(bit_reader* r, const huff_table* t) {
  int32_t code = 0;
  for (int32_t len = 1; len <= 16; ++len) {
    code = (code << 1) | next_bit(r);
    int32_t k = code - t->first_code[len];
    if (k >= 0 && k < t->counts[len - 1]) return t->symbols[t->first_index[len] + k];
  }
  return -1;
}

static int32_t idct_basis(int32_t x, int32_t u) {
  /* C(u) cos((2x+1) u pi / 16) in 13 fractional bits, C(0) = 1/sqrt(2), C(u>0) = 1 */
  double c = (u == 0) ? sqrt(0.5) : cos((double)((2 * x + 1) * u) * 3.14159265358979323846 / 16.0);
  return (int32_t)lrint(c * 8192.0);
}

static int32_t clamp16(int64_t v) { return v < -32767 ? -32767 : (v > 32767 ? 32767 : (int32_t)v); }
static int64_t floor_shift(int64_t v, int32_t s) { return v >= 0 ? v >> s : -((-v + (1ll << s) - 1) >> s); }

void mae_oracle_idct8x8(const int32_t coef[64], uint8_t out[64]) {
  /* f(x, y) = 1/4 sum_u sum_v C(u) C(v) F(v, u) cos(..x..u) cos(..y..v); coef[v * 8 + u];
   * out[y * 8 + x].  Pass 1 along v (columns), pass 2 along u (rows). */
  int32_t tmp[64];
  for (int32_t y = 0; y < 8; ++y)
    for (int32_t u = 0; u < 8; ++u) {
      int64_t acc = 0;
      for (int32_t v = 0; v < 8; ++v) acc += (int64_t)idct_basis(y, v) * clamp16(coef[v * 8 + u]);
      tmp[y * 8 + u] = clamp16(floor_shift(acc + (1 << 10), 11)); /* 1-D result, 3 more bits */
    }
  for (int32_t y = 0; y < 8; ++y)
    for (int32_t x = 0; x < 8; ++x) {
      int64_t acc = 0;
      for (int32_t u = 0; u < 8; ++u) acc += (int64_t)idct_basis(x, u) * tmp[y * 8 + u];
      int64_t v = floor_shift(acc + (1 << 16), 17) + 128;
      out[y * 8 + x] = (uint8_t)(v < 0 ? 0 : (v > 255 ? 255 : v));
    }
}

void mae_oracle_ycc_to_rgb(int32_t y, int32_t cb, int32_t cr, uint8_t rgb[3]) {
  int64_t b = cb - 128, r = cr - 128;
  int64_t R = y + floor_shift(91881 * r + 32768, 16);
  int64_t G = y - floor_shift(22554 * b + 46802 * r + 32768, 16);
  int64_t B = y + floor_shift(116130 * b + 32768, 16);
  rgb[0] = (uint8_t)(R < 0 ? 0 : (R > 255 ? 255 : R));
  rgb[1] = (uint8_t)(G < 0 ? 0 : (G > 255 ? 255 : G));
  rgb[2] = (uint8_t)(B < 0 ? 0 : (B > 255 ? 255 : B));
}

static int32_t jpeg_decode_any(const uint8_t* data, int64_t n, uint8_t* rgb, int32_t want_ycc);

int32_t mae_oracle_jpeg_decode(const uint8_t* data, int64_t n, uint8_t* rgb) {
  return jpeg_decode_any(data, n, rgb, 0);
}

int32_t mae_oracle_jpeg_decode_ycc(const uint8_t* data, int64_t n, uint8_t* ycc) {
  return jpeg_decode_any(data, n, ycc, 1);
}

static int32_t jpeg_decode_any(const uint8_t* data, int64_t n, uint8_t* rgb, int32_t want_ycc) {
  if (!data || !rgb) return -1;
  jpeg_header h;
  int32_t rc = jpeg_parse(data, n, &h);
  if (rc) return rc;
  int32_t hmax = h.hs[0], vmax = h.vs[0];
  int32_t mcux = (h.W + 8 * hmax - 1) / (8 * hmax), mcuy = (h.H + 8 * vmax - 1) / (8 * vmax);
  /* component planes, whole MCUs */
  uint8_t* plane[3];
  int32_t pw[3], ph[3];
  for (int32_t c = 0; c < 3; ++c) {
    pw[c] = mcux * h.hs[c] * 8;
    ph[c] = mcuy * h.vs[c] * 8;
    plane[c] = (uint8_t*)malloc((size_t)pw[c] * ph[c]);
    if (!plane[c]) return -1;
  }
  bit_reader r = {data, n, h.scan, 0, 0, 0};
  int32_t pred[3] = {0, 0, 0};
  int32_t status = 0;
  int64_t total = (int64_t)mcux * mcuy;
  for (int64_t m = 0; m < total && !status; ++m) {
    if (h.restart && m > 0 && m % h.restart == 0) {
      /* the interval ends on a byte boundary and is followed by RSTn */
      r.nbits = 0;
      if (!(r.pos + 1 < r.n && r.d[r.pos] == 0xFF && r.d[r.pos + 1] >= 0xD0 &&
            r.d[r.pos + 1] <= 0xD7 &&
            r.d[r.pos + 1] == 0xD0 + (int32_t)((m / h.restart - 1) % 8))) {
        status = -3;
        break;
      }
      r.pos += 2;
      r.hit_marker = 0;
      pred[0] = pred[1] = pred[2] = 0;
    }
    int32_t my = (int32_t)(m / mcux), mx = (int32_t)(m % mcux);
    for (int32_t c = 0; c < 3 && !status; ++c)
      for (int32_t bv = 0; bv < h.vs[c] && !status; ++bv)
        for (int32_t bh = 0; bh < h.hs[c] && !status; ++bh) {
          int32_t coef[64];
          memset(coef, 0, sizeof(coef));
          int32_t s = huff_decode(&r, &h.dc[h.td[c]]);
          if (s < 0 || s > 11) {
            status = -3;
            break;
          }
          pred[c] += extend(receive(&r, s), s);
          coef[0] = pred[c] * (int32_t)h.q[h.tq[c]][0];
          for (int32_t k = 1; k < 64;) {
            int32_t rs = huff_decode(&r, &h.ac[h.ta[c]]);
            if (rs < 0) {
              status = -3;
              break;
            }
            int32_t run = rs >> 4, size = rs & 15;
            if (size == 0) {
              if (run != 15) break; /* end of block */
              k += 16;
              continue;
            }
            k += run;
            if (k > 63) {
              status = -3;
              break;
            }
            coef[ZIGZAG[k]] = extend(receive(&r, size), size) * (int32_t)h.q[h.tq[c]][k];
            ++k;
          }
          uint8_t px[64];
          mae_oracle_idct8x8(coef, px);
          int32_t x0 = (mx * h.hs[c] + bh) * 8, y0 = (my * h.vs[c] + bv) * 8;
          for (int32_t y = 0; y < 8; ++y)
            memcpy(plane[c] + (size_t)(y0 + y) * pw[c] + x0, px + 8 * y, 8);
        }
  }
  if (!status) {
    for (int32_t y = 0; y < h.H; ++y)
      for (int32_t x = 0; x < h.W; ++x) {
        int32_t Y = plane[0][(size_t)y * pw[0] + x];
        int32_t cb = plane[1][(size_t)(y * h.vs[1] / vmax) * pw[1] + x * h.hs[1] / hmax];
        int32_t cr = plane[2][(size_t)(y * h.vs[2] / vmax) * pw[2] + x * h.hs[2] / hmax];
        uint8_t* px = rgb + ((size_t)y * h.W + x) * 3;
        if (want_ycc) {
          px[0] = (uint8_t)Y;
          px[1] = (uint8_t)cb;
          px[2] = (uint8_t)cr;
        } else {
          mae_oracle_ycc_to_rgb(Y, cb, cr, px);
        }
      }
  }
  for (int32_t c = 0; c < 3; ++c) free(plane[c]);
  (void)ph;
  return status;
}

int32_t mae_oracle_threads(void) {
#ifdef _OPENMP
  return (int32_t)omp_get_max_threads();
#else
  return 1;
#endif
}

/* Number of threads the loops over samples and rows may use from now on (timing only: results
 * do not depend on it); n < 1 restores the default. */
void mae_oracle_set_threads(int32_t n) {
#ifdef _OPENMP
  omp_set_num_threads(n >= 1 ? n : omp_get_num_procs());
#else
  (void)n;
#endif
}
