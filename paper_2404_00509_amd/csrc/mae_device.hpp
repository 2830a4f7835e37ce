// Shared device-side helpers of the gfx950 kernels: keyed random draws, workgroup remapping for
// the 8 XCDs, packed conversions.  HIP path only.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mae {

constexpr int kWave = 64;         // CDNA wavefront
constexpr int kXcds = 8;          // MI355X: 8 accelerator dies, one L2 each
constexpr int kMaxPatches = 256;  // per image: one wavefront sorts 4 keys per lane

// Per-sample record handed from the parameter kernel to the resampling kernel (workspace).
struct CropRec {
  int32_t top, left, ch, cw;  // crop box inside the image
  int32_t flip;               // 1 = mirror output columns
  int32_t valid;              // 0 = geometry check failed, sample skipped
  int32_t pad0, pad1;
};
static_assert(sizeof(CropRec) == 32, "CropRec is 32 bytes");

// The workspace starts with a 256-byte header, followed by CropRec[B].
constexpr size_t kWorkspaceHeader = 256;
constexpr int32_t kWorkspaceMagic = 0x4D414531;  // "MAE1"
struct WorkspaceHeader {
  int32_t magic;
  int32_t B;  // number of records written by the last call
};

// ---- SplitMix64 output function (Steele, Lea, Flood 2014), used as a keyed counter hash --------
constexpr uint64_t kGamma = 0x9E3779B97F4A7C15ull;

__host__ __device__ inline uint64_t mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

// key1 = state after keying with (seed, batch_index); computed once per call on the host.
__host__ __device__ inline uint64_t batch_key(uint64_t seed, uint64_t batch_index) {
  uint64_t k0 = mix64(seed + kGamma);
  return mix64(k0 + kGamma * (batch_index + 1));
}

enum Stream : uint32_t {
  kScale = 0, kRatio = 1, kTop = 2, kLeft = 3, kFlip = 4, kNoise = 5,
  kAugOp = 6, kBlurSigma = 7, kBrightness = 8, kContrast = 9, kSaturation = 10
};

__device__ inline uint64_t draw(uint64_t key1, uint32_t sample, uint32_t stream, uint32_t ctr) {
  uint64_t w = ((uint64_t)sample << 32) | ((uint64_t)stream << 24) | (uint64_t)ctr;
  return mix64(key1 + kGamma * (w + 1));
}

// uniform in [0, 1) from the top 53 bits of a draw; exact in double precision
__device__ inline double unit53(uint64_t bits) {
  return (double)(bits >> 11) * (1.0 / 9007199254740992.0);
}

// ---- per-sample draws of the finetuning augmentation ("3 Aug" / "3 Aug+", Sec. 5.2 Table 7) -----
// One of grayscale / solarise / Gaussian blur per image with equal probability, the blur's sigma
// uniform on [0.1, 2], and brightness / contrast / saturation factors uniform on 1 +- jitter.
enum AugOp : int32_t { kOpGray = 0, kOpSolarise = 1, kOpBlur = 2 };
struct AugParams {
  int32_t op;
  int32_t radius;  // of the blur: ceil(3 sigma), 1..6
  double sigma;
  float brightness, contrast, saturation;
  float pad;
  // blur images: tap |k| of the kernel exp(-k^2 / (2 sigma^2)) scaled to sum 1, zero beyond the
  // radius (filled in by the parameter kernel, see blur_taps)
  float tap[8];
};
static_assert(sizeof(AugParams) == 64, "one 64-byte record per sample in the workspace");
__device__ inline AugParams aug_params(uint64_t key1, uint32_t sample, float jitter) {
#pragma clang fp contract(off)  // sigma decides the integer radius: no fused multiply-add here
  AugParams ap;
  const int k = (int)floor(3.0 * unit53(draw(key1, sample, kAugOp, 0)));
  ap.op = k > 2 ? 2 : k;
  ap.sigma = 0.1 + 1.9 * unit53(draw(key1, sample, kBlurSigma, 0));
  const int r = (int)ceil(3.0 * ap.sigma);
  ap.radius = r < 1 ? 1 : r;
  const double j = (double)jitter;
  ap.brightness = (float)(1.0 + j * (2.0 * unit53(draw(key1, sample, kBrightness, 0)) - 1.0));
  ap.contrast = (float)(1.0 + j * (2.0 * unit53(draw(key1, sample, kContrast, 0)) - 1.0));
  ap.saturation = (float)(1.0 + j * (2.0 * unit53(draw(key1, sample, kSaturation, 0)) - 1.0));
  ap.pad = 0.0f;
#pragma unroll
  for (int k = 0; k < 8; ++k) ap.tap[k] = 0.0f;
  return ap;
}
// Tap `lane` (0..6) of the blur kernel of an image, by the first lanes of a wavefront together:
// exp(-k^2 / (2 sigma^2)) in double precision, summed over -radius .. radius in index order,
// scaled to sum 1.  Returns zero for lanes beyond the radius.
__device__ inline float blur_taps(const AugParams& ap, int lane) {
  const double k = (double)lane;
  const double e = lane <= ap.radius ? exp(-(k * k) / (2.0 * ap.sigma * ap.sigma)) : 0.0;
  double sum = 0.0;
  for (int j = -6; j <= 6; ++j) sum += __shfl(e, j < 0 ? -j : j, kWave);
  return (float)(e / sum);
}

// ---- the loss's divisor counted on the device ------------------------------------------------------
// A first small kernel leaves n <= kMaxCounts partial counts of the mask's non-zero bytes; every
// wavefront that needs the number of masked patches M adds them up (all lanes get the sum).
constexpr int kMaxCounts = 256;
__device__ inline int64_t sum_counts(const int32_t* counts, int n) {
  const int lane = threadIdx.x % kWave;
  int64_t s = 0;
  for (int i = lane; i < n; i += kWave) s += counts[i];
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) s += __shfl_xor(s, off, kWave);
  return s;
}
// 1 / (D M), and 0 when nothing is masked (the loss is then 0 and no gradient uses the factor)
__device__ inline double inv_count_of(int D, int64_t M) {
  return M > 0 ? 1.0 / ((double)D * (double)M) : 0.0;
}

// ---- workgroup id -> logical tile id, so that consecutive tiles share an XCD (and its L2) ------
// Hardware hands workgroup i to XCD i % 8.  Tiles are split into 8 contiguous ranges, one per XCD.
__device__ inline uint32_t xcd_remap(uint32_t wg, uint32_t n) {
  uint32_t q = n / kXcds, r = n % kXcds;
  uint32_t xcd = wg % kXcds, pos = wg / kXcds;
  return xcd < r ? xcd * (q + 1) + pos : r * (q + 1) + (xcd - r) * q + pos;
}

// ---- float -> bfloat16, round to nearest even (finite inputs) ----------------------------------
__device__ inline uint32_t bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return u >> 16;
}
__device__ inline uint32_t pack_bf16x2(float lo, float hi) {
  return bf16_rne(lo) | (bf16_rne(hi) << 16);
}
__device__ inline float bf16_lo(uint32_t v) { return __uint_as_float(v << 16); }
__device__ inline float bf16_hi(uint32_t v) { return __uint_as_float(v & 0xFFFF0000u); }

}  // namespace mae
