// Crop + bilinear resize (Sec. 4.1, Sec. 5.1) + horizontal flip + mean/std normalisation (App. B)
// + ViT patch split (Sec. 3) + gather of the visible patches (Sec. 2), in one pass: every source
// byte is read from HBM once and every output value is written once, straight into patch order.
//
// One workgroup per (image, row of patches, column part): wide sources are split into column parts
// (whole patches each) so that the staged tile stays small and many workgroups fit a compute unit.
//  * Staging.  The source rows that this patch row taps are brought into LDS as 4-byte RGBx pixel
//    words.  Lane i of a wavefront loads the 16 bytes that hold pixels 4i..4i+3 of a row (one
//    4-byte-aligned global_load_dwordx4; the row's misalignment is taken out with byte-align
//    operations in registers) and writes four pixel words with one ds_write_b128.  All loads of a
//    wavefront (up to seven rows) are issued before the first is consumed, and the tap tables
//    (S horizontal entries, p vertical entries, integer tap positions + fp32 weights) are built
//    while they are in flight.
//  * Compute + store.  A patch is D/4 groups of 16 bytes; wavefront w of the workgroup owns groups
//    64w .. 64w+63 (one per lane) of EVERY patch of the row, so what depends only on the position
//    inside the patch (rows tapped, vertical weights, channel constants, byte selectors) is set
//    up once, and every store instruction covers 1 KiB of contiguous memory.  A group of four
//    consecutive values spans two neighbouring pixels; the taps x and x+1 come from one
//    ds_read2_b32 per row, and one byte-permute per tap row pulls exactly the four bytes needed
//    out of the two pixel words.  Nothing inside the loop reads global memory, so the stores of
//    one patch never have to complete before the next patch is computed.
//  * Variants of the last phase on the same staged tile: the finetuning augmentation as the
//    epilogue (produce_aug: values rounded to bytes in integers, grayscale / solarisation, colour
//    jitter; only the images that drew the blur leave as bytes for the blur kernel); the kept
//    patches only (no target wanted); and the loss itself
//    (produce_loss_wave, produce_loss): the masked patches' values stay in registers, are
//    normalised per patch and compared with the prediction, so that no float target is ever
//    stored or read back.
#include "aug_device.hpp"
#include "mae_device.hpp"
#include "mae_kernels.hpp"

namespace mae {

constexpr int kCropThreads = 256;      // scalar kernel
constexpr int kCropMaxThreads = 1024;  // resampling kernel: 64 threads per 64 groups of a patch
constexpr int kStageRows = 7;  // rows per wavefront whose loads are issued together
constexpr int kCropMaxLds = 64 * 1024;      // dynamic LDS available without opting in to more
constexpr int kCropTileTarget = 40 * 1024;  // LDS per workgroup that still leaves 4 per compute unit

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef u32x4 u32x4_a4 __attribute__((aligned(4)));

// Source taps of output index o when `len` source pixels are resized to S: sample position
// (o + 1/2) len / S - 1/2 kept as the exact fraction n / (2 S); taps clamped to [0, len).
// The integer quotient comes from a float estimate (off by at most one for n < 2^26, quotient
// < 2^15) that is corrected with the exact remainder; inv_den = 1 / (2 S).
// rem is the exact remainder n mod 2 S (the weight of the second tap is rem / (2 S)).
__device__ static inline void resize_taps(int o, int len, int S, float inv_den, int& i0, int& i1,
                                          float& f, int& rem) {
  const int n = (2 * o + 1) * len - S;
  const int den = 2 * S;
  rem = 0;
  if (n <= 0) {
    i0 = 0;
    f = 0.0f;
  } else {
    int q = (int)((float)n * inv_den);
    int r = n - q * den;
    if (r < 0) {
      --q;
      r += den;
    } else if (r >= den) {
      ++q;
      r -= den;
    }
    i0 = q;
    rem = r;
    f = (float)r * inv_den;
  }
  i1 = min(i0 + 1, len - 1);
}
__device__ static inline void resize_taps(int o, int len, int S, float inv_den, int& i0, int& i1,
                                          float& f) {
  int rem;
  resize_taps(o, len, S, inv_den, i0, i1, f, rem);
}

__device__ static inline uint32_t load_rgbx(const uint8_t* p) {
  return (uint32_t)p[0] | ((uint32_t)p[1] << 8) | ((uint32_t)p[2] << 16);
}

// Pixel words at x and x + 1 of one row.  In the tile the word after the last pixel of a row is
// readable (its weight is zero); in global memory the second tap is clamped instead.
template <bool kLds>
__device__ static inline void fetch2(const uint32_t* tile, const uint8_t* base, uint32_t row_off,
                                     int x, int cw, uint32_t& v0, uint32_t& v1) {
  if (kLds) {
    v0 = tile[row_off + x];
    v1 = tile[row_off + x + 1];
  } else {
    v0 = load_rgbx(base + ((size_t)row_off + (size_t)(3 * x)));
    v1 = load_rgbx(base + ((size_t)row_off + (size_t)(3 * min(x + 1, cw - 1))));
  }
}

template <int J>
__device__ static inline float byte_to_float(uint32_t v) {
  return (float)((v >> (8 * J)) & 0xFFu);
}

// 16 bytes at a 4-byte-aligned address; `safe` says that they all lie inside the image buffer.
__device__ static inline u32x4 load16(const uint8_t* p, bool safe, const uint8_t* lo,
                                      const uint8_t* hi) {
  if (safe) return *reinterpret_cast<const u32x4_a4*>(p);
  uint32_t w[4] = {0u, 0u, 0u, 0u};  // first or last bytes of the buffer: take what is inside
  for (int q = 0; q < 16; ++q) {
    if (p + q >= lo && p + q < hi) w[q >> 2] |= (uint32_t)p[q] << (8 * (q & 3));
  }
  return u32x4{w[0], w[1], w[2], w[3]};
}

// 16 loaded bytes, of which the 12 bytes of four pixels start at byte s (0..3) -> 4 RGBx words.
__device__ static inline u32x4 to_pixels(u32x4 d, uint32_t s) {
  const uint32_t e0 = __builtin_amdgcn_alignbyte(d.y, d.x, s);
  const uint32_t e1 = __builtin_amdgcn_alignbyte(d.z, d.y, s);
  const uint32_t e2 = __builtin_amdgcn_alignbyte(d.w, d.z, s);
  return u32x4{e0, __builtin_amdgcn_alignbyte(e1, e0, 3u), __builtin_amdgcn_alignbyte(e2, e1, 2u),
               e2 >> 8};
}

// The compute + store phase of one wavefront: its 64 groups of every patch.  kLds: taps come from
// the staged tile (row offsets in pixel words), otherwise straight from global memory (row offsets
// in bytes; crops too large to stage).  my_rank holds, in lane i, the noise rank of patch i of
// this part (patches gx0 .. gx0 + npatch - 1); cw is the number of source columns from the
// part's first tapped column to the crop's right edge.
// kKeptOnly: no target is wanted, so the masked patches are skipped.
template <bool kLds, bool kBf16, bool kKeptOnly>
__device__ static void produce_patches(const CropArgs& a, const uint32_t* tile, const u32x2* xtab,
                                       const u32x4* ytab, const uint8_t* base, int b, int gy,
                                       int gx0, int npatch, int cw, int my_rank) {
  const int lane = threadIdx.x % kWave;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int p = a.p, D = a.D;
  const int D4 = D >> 2;
  const int pp = p * p;
  const float inv_p = 1.0f / (float)p;
  const float ns0 = a.nscale[0], ns1 = a.nscale[1], ns2 = a.nscale[2];
  const float nb0 = a.nbias[0], nb1 = a.nbias[1], nb2 = a.nbias[2];

  const int e4 = wave * kWave + lane;
  const bool active = e4 < D4;
  const int e = active ? 4 * e4 : 0;
  // elements e .. e+3 belong to pixel qA (channels cA ..) and to the next pixel qB
  const int qA = e / 3;
  const int cA = e - 3 * qA;
  const int qB = min(qA + 1, pp - 1);
  const int pyA = (int)(((float)qA + 0.5f) * inv_p);
  const int pxA = qA - pyA * p;
  const int pyB = (int)(((float)qB + 0.5f) * inv_p);
  const int pxB = qB - pyB * p;
  const u32x4 ya = ytab[pyA], yb = ytab[pyB];
  const uint32_t rowA0 = ya.x, rowA1 = ya.y, rowB0 = yb.x, rowB1 = yb.y;
  const float fyA = __uint_as_float(ya.z), fyB = __uint_as_float(yb.z);
  // byte selectors: A's bytes are 0..2, B's bytes are 4..6 of the 64-bit pair {B, A}
  const uint32_t sel = cA == 0 ? 0x04020100u : (cA == 1 ? 0x05040201u : 0x06050402u);
  const int nA = 3 - cA;  // how many of the four values come from pixel A (1..3)
  float sc[4], bi[4], fy[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    int c = cA + j;
    c = c >= 3 ? c - 3 : c;
    c = c >= 3 ? c - 3 : c;
    sc[j] = c == 0 ? ns0 : (c == 1 ? ns1 : ns2);
    bi[j] = c == 0 ? nb0 : (c == 1 ? nb1 : nb2);
    fy[j] = j == 0 ? fyA : (j == 3 ? fyB : (j < nA ? fyA : fyB));
  }

  for (int gx = 0; gx < npatch; ++gx) {
    const int l = gy * a.G + gx0 + gx;
    const int rank = __builtin_amdgcn_readlane(my_rank, gx);
    if (kKeptOnly && rank >= a.K) continue;
    const u32x2 xa = xtab[gx * p + pxA], xb = xtab[gx * p + pxB];
    const float fxA = __uint_as_float(xa.y), fxB = __uint_as_float(xb.y);
    uint32_t A00, A01, A10, A11, B00, B01, B10, B11;
    fetch2<kLds>(tile, base, rowA0, (int)xa.x, cw, A00, A01);
    fetch2<kLds>(tile, base, rowA1, (int)xa.x, cw, A10, A11);
    fetch2<kLds>(tile, base, rowB0, (int)xb.x, cw, B00, B01);
    fetch2<kLds>(tile, base, rowB1, (int)xb.x, cw, B10, B11);
    const uint32_t P00 = __builtin_amdgcn_perm(B00, A00, sel);
    const uint32_t P01 = __builtin_amdgcn_perm(B01, A01, sel);
    const uint32_t P10 = __builtin_amdgcn_perm(B10, A10, sel);
    const uint32_t P11 = __builtin_amdgcn_perm(B11, A11, sel);

    float out[4];
#define MAE_BLEND(J)                                                                 \
{                                                                                  \
  const float fx = (J) == 0 ? fxA : ((J) == 3 ? fxB : ((J) < nA ? fxA : fxB));     \
  const float a00 = byte_to_float<J>(P00), a01 = byte_to_float<J>(P01);            \
  const float a10 = byte_to_float<J>(P10), a11 = byte_to_float<J>(P11);            \
  const float rt = a00 + fx * (a01 - a00);                                         \
  const float rb = a10 + fx * (a11 - a10);                                         \
  const float v = rt + fy[J] * (rb - rt);                                          \
  out[J] = v * sc[J] + bi[J];                                                      \
}
    MAE_BLEND(0) MAE_BLEND(1) MAE_BLEND(2) MAE_BLEND(3)
#undef MAE_BLEND

    if (active) {
      if (a.target) {
        f32x4* dst = reinterpret_cast<f32x4*>(a.target + ((int64_t)b * a.L + l) * D + e);
        *dst = f32x4{out[0], out[1], out[2], out[3]};
      }
      if (rank < a.K) {
        const int64_t vo = ((int64_t)b * a.K + rank) * D + e;
        if (kBf16) {
          u32x2* dst = reinterpret_cast<u32x2*>(static_cast<uint16_t*>(a.visible) + vo);
          *dst = u32x2{pack_bf16x2(out[0], out[1]), pack_bf16x2(out[2], out[3])};
        } else {
          f32x4* dst = reinterpret_cast<f32x4*>(static_cast<float*>(a.visible) + vo);
          *dst = f32x4{out[0], out[1], out[2], out[3]};
        }
      }
    }
  }
}

// ---- the loss without a stored target ---------------------------------------------------------------
// Same decomposition as produce_patches (a thread owns one 16-byte group position of every patch
// of the part), but the values stay in registers: per patch the workgroup adds them up for the
// mean, then the squared deviations for the variance (two block reductions for all patches of a
// chunk at once), and the masked patches' normalised values meet the prediction: squared error
// into the workgroup's partial sum, gradient written with the same contiguous 16-byte stores.
// Visible patches get a zero gradient and are not resampled.  `masked` holds, in lane i, whether
// patch i of this part is masked.
constexpr int kLossChunk = 8;  // patches whose values a thread holds at once

// (read once, written once: the non-temporal hint keeps them from displacing the source rows)
__device__ static inline f32x4 crop_load_pred4(const void* pred, int64_t elem, bool bf16) {
  if (bf16) {
    const u32x2 raw = __builtin_nontemporal_load(
        reinterpret_cast<const u32x2*>(static_cast<const uint16_t*>(pred) + elem));
    return f32x4{bf16_lo(raw.x), bf16_hi(raw.x), bf16_lo(raw.y), bf16_hi(raw.y)};
  }
  return __builtin_nontemporal_load(
      reinterpret_cast<const f32x4*>(static_cast<const float*>(pred) + elem));
}
__device__ static inline void crop_store_grad4(void* grad, int64_t elem, f32x4 g, bool bf16) {
  if (bf16)
    __builtin_nontemporal_store(u32x2{pack_bf16x2(g.x, g.y), pack_bf16x2(g.z, g.w)},
                                reinterpret_cast<u32x2*>(static_cast<uint16_t*>(grad) + elem));
  else
    __builtin_nontemporal_store(g, reinterpret_cast<f32x4*>(static_cast<float*>(grad) + elem));
}

// grad_scale * 2 / (D M): the host's value, or from the device-side count of masked patches
__device__ static inline float loss_gscale(const CropArgs& a) {
  if (!a.counts) return a.gscale;
  const float g = (float)(a.gscale_num * inv_count_of(a.D, sum_counts(a.counts, a.ncounts)));
  return __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(g)));
}

// Sums of v[0 .. kLossChunk) over the workgroup, lanes by butterfly and wavefronts in index
// order; every thread gets all of them.  red: kLossChunk floats per wavefront.
__device__ static inline void block_sums(float* v, float* red, int lane, int wave, int nwaves) {
#pragma unroll
  for (int j = 0; j < kLossChunk; ++j) {
    float t = v[j];
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) t += __shfl_xor(t, off, kWave);
    v[j] = t;
  }
  __syncthreads();  // the previous round's sums have been read
  if (lane == 0) {
#pragma unroll
    for (int j = 0; j < kLossChunk; ++j) red[wave * kLossChunk + j] = v[j];
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < kLossChunk; ++j) {
    float t = 0.f;
    for (int w = 0; w < nwaves; ++w) t += red[w * kLossChunk + j];
    v[j] = t;
  }
}

template <bool kLds>
__device__ static void produce_loss(const CropArgs& a, const uint32_t* tile, const u32x2* xtab,
                                    const u32x4* ytab, const uint8_t* base, int b, int gy, int gx0,
                                    int npatch, int cw, int masked, float* red, double* red64,
                                    uint32_t tile_id) {
  const int lane = threadIdx.x % kWave;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int nwaves = (int)blockDim.x / kWave;
  const int p = a.p, D = a.D;
  const int D4 = D >> 2;
  const int pp = p * p;
  const float inv_p = 1.0f / (float)p;
  const float ns0 = a.nscale[0], ns1 = a.nscale[1], ns2 = a.nscale[2];
  const float nb0 = a.nbias[0], nb1 = a.nbias[1], nb2 = a.nbias[2];
  const bool bf16 = a.pred_bf16 != 0;

  // position inside the patch: as in produce_patches
  const int e4 = wave * kWave + lane;
  const bool active = e4 < D4;
  const int e = active ? 4 * e4 : 0;
  const int qA = e / 3;
  const int cA = e - 3 * qA;
  const int qB = min(qA + 1, pp - 1);
  const int pyA = (int)(((float)qA + 0.5f) * inv_p);
  const int pxA = qA - pyA * p;
  const int pyB = (int)(((float)qB + 0.5f) * inv_p);
  const int pxB = qB - pyB * p;
  const u32x4 ya = ytab[pyA], yb = ytab[pyB];
  const uint32_t rowA0 = ya.x, rowA1 = ya.y, rowB0 = yb.x, rowB1 = yb.y;
  const float fyA = __uint_as_float(ya.z), fyB = __uint_as_float(yb.z);
  const uint32_t sel = cA == 0 ? 0x04020100u : (cA == 1 ? 0x05040201u : 0x06050402u);
  const int nA = 3 - cA;
  float sc[4], bi[4], fy[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    int c = cA + j;
    c = c >= 3 ? c - 3 : c;
    c = c >= 3 ? c - 3 : c;
    sc[j] = c == 0 ? ns0 : (c == 1 ? ns1 : ns2);
    bi[j] = c == 0 ? nb0 : (c == 1 ? nb1 : nb2);
    fy[j] = j == 0 ? fyA : (j == 3 ? fyB : (j < nA ? fyA : fyB));
  }
  const float inv_d = 1.0f / (float)D, inv_dm1 = 1.0f / (float)(D - 1);
  const f32x4 zero = f32x4{0.f, 0.f, 0.f, 0.f};
  const float gscale = loss_gscale(a);
  double acc = 0.0;

  for (int g0 = 0; g0 < npatch; g0 += kLossChunk) {
    f32x4 val[kLossChunk], q[kLossChunk];
    float s[kLossChunk];
    bool m[kLossChunk];
    // the predictions first: they are on their way while the pixels are resampled
#pragma unroll
    for (int j = 0; j < kLossChunk; ++j) {
      m[j] = g0 + j < npatch && __builtin_amdgcn_readlane(masked, (g0 + j) & (kWave - 1)) != 0;
      q[j] = zero;
      if (m[j] && active)
        q[j] = crop_load_pred4(a.pred, ((int64_t)b * a.L + gy * a.G + gx0 + g0 + j) * D + e, bf16);
    }
#pragma unroll
    for (int j = 0; j < kLossChunk; ++j) {
      val[j] = zero;
      s[j] = 0.f;
      if (!m[j]) continue;
      const int gx = g0 + j;
      const u32x2 xa = xtab[gx * p + pxA], xb = xtab[gx * p + pxB];
      const float fxA = __uint_as_float(xa.y), fxB = __uint_as_float(xb.y);
      uint32_t A00, A01, A10, A11, B00, B01, B10, B11;
      fetch2<kLds>(tile, base, rowA0, (int)xa.x, cw, A00, A01);
      fetch2<kLds>(tile, base, rowA1, (int)xa.x, cw, A10, A11);
      fetch2<kLds>(tile, base, rowB0, (int)xb.x, cw, B00, B01);
      fetch2<kLds>(tile, base, rowB1, (int)xb.x, cw, B10, B11);
      const uint32_t P00 = __builtin_amdgcn_perm(B00, A00, sel);
      const uint32_t P01 = __builtin_amdgcn_perm(B01, A01, sel);
      const uint32_t P10 = __builtin_amdgcn_perm(B10, A10, sel);
      const uint32_t P11 = __builtin_amdgcn_perm(B11, A11, sel);
      float out[4];
#define MAE_BLEND(J)                                                                 \
{                                                                                  \
  const float fx = (J) == 0 ? fxA : ((J) == 3 ? fxB : ((J) < nA ? fxA : fxB));     \
  const float a00 = byte_to_float<J>(P00), a01 = byte_to_float<J>(P01);            \
  const float a10 = byte_to_float<J>(P10), a11 = byte_to_float<J>(P11);            \
  const float rt = a00 + fx * (a01 - a00);                                         \
  const float rb = a10 + fx * (a11 - a10);                                         \
  const float v = rt + fy[J] * (rb - rt);                                          \
  out[J] = v * sc[J] + bi[J];                                                      \
}
      MAE_BLEND(0) MAE_BLEND(1) MAE_BLEND(2) MAE_BLEND(3)
#undef MAE_BLEND
      if (active) {
        val[j] = f32x4{out[0], out[1], out[2], out[3]};
        s[j] = (out[0] + out[1]) + (out[2] + out[3]);
      }
    }
    float rstd[kLossChunk];
#pragma unroll
    for (int j = 0; j < kLossChunk; ++j) rstd[j] = 1.0f;
    if (a.norm_pix) {
      block_sums(s, red, lane, wave, nwaves);
#pragma unroll
      for (int j = 0; j < kLossChunk; ++j) {
        const float mu = s[j] * inv_d;
        val[j] = val[j] - mu;
        s[j] = active ? (val[j].x * val[j].x + val[j].y * val[j].y) +
                            (val[j].z * val[j].z + val[j].w * val[j].w)
                      : 0.f;
      }
      block_sums(s, red, lane, wave, nwaves);
#pragma unroll
      for (int j = 0; j < kLossChunk; ++j) rstd[j] = 1.0f / sqrtf(s[j] * inv_dm1 + a.eps);
    }
    float sq = 0.f;
#pragma unroll
    for (int j = 0; j < kLossChunk; ++j) {
      if (g0 + j >= npatch || !active) continue;
      const int64_t elem = ((int64_t)b * a.L + gy * a.G + gx0 + g0 + j) * D + e;
      f32x4 diff = zero;
      if (m[j]) {
        diff = q[j] - val[j] * rstd[j];
        sq += (diff.x * diff.x + diff.y * diff.y) + (diff.z * diff.z + diff.w * diff.w);
      }
      if (a.grad) crop_store_grad4(a.grad, elem, diff * gscale, bf16);
    }
    acc += (double)sq;
  }
  // the workgroup's share of the loss: lanes by butterfly, wavefronts in index order
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) acc += __shfl_xor(acc, off, kWave);
  __syncthreads();
  if (lane == 0) red64[wave] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    double t = 0.0;
    for (int w = 0; w < nwaves; ++w) t += red64[w];
    a.partials[tile_id] = t;
  }
}

// (The per-group setup and the blend are written out again in each of these functions: behind a
// shared helper the compiler keeps 40 more registers alive, which costs a wavefront per SIMD.)
//
// The same for patches of up to 768 values (NV = groups per lane, D / 4 <= 64 NV): a wavefront
// holds a whole patch, lane i its groups i, i + 64, ..., so the two reductions are wavefront
// butterflies and the wavefronts of the workgroup work through the part's patches independently.
template <bool kLds, int NV>
__device__ static void produce_loss_wave(const CropArgs& a, const uint32_t* tile,
                                         const u32x2* xtab, const u32x4* ytab, const uint8_t* base,
                                         int b, int gy, int gx0, int npatch, int cw, int masked,
                                         double* red64, uint32_t tile_id) {
  const int lane = threadIdx.x % kWave;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int nwaves = (int)blockDim.x / kWave;
  const int p = a.p, D = a.D;
  const int D4 = D >> 2;
  const int pp = p * p;
  const float inv_p = 1.0f / (float)p;
  const bool bf16 = a.pred_bf16 != 0;

  // what depends on the position inside the patch only, per group of the lane
  bool active[NV];
  int e[NV], pxA[NV], pxB[NV], nA[NV];
  uint32_t rowA0[NV], rowA1[NV], rowB0[NV], rowB1[NV], sel[NV];
  float sc[NV][4], bi[NV][4], fy[NV][4];
#pragma unroll
  for (int v = 0; v < NV; ++v) {
    const int e4 = lane + v * kWave;
    active[v] = e4 < D4;
    e[v] = active[v] ? 4 * e4 : 0;
    const int qA = e[v] / 3;
    const int cA = e[v] - 3 * qA;
    const int qB = min(qA + 1, pp - 1);
    const int pyA = (int)(((float)qA + 0.5f) * inv_p);
    pxA[v] = qA - pyA * p;
    const int pyB = (int)(((float)qB + 0.5f) * inv_p);
    pxB[v] = qB - pyB * p;
    const u32x4 ya = ytab[pyA], yb = ytab[pyB];
    rowA0[v] = ya.x;
    rowA1[v] = ya.y;
    rowB0[v] = yb.x;
    rowB1[v] = yb.y;
    const float fyA = __uint_as_float(ya.z), fyB = __uint_as_float(yb.z);
    sel[v] = cA == 0 ? 0x04020100u : (cA == 1 ? 0x05040201u : 0x06050402u);
    nA[v] = 3 - cA;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int c = cA + j;
      c = c >= 3 ? c - 3 : c;
      c = c >= 3 ? c - 3 : c;
      sc[v][j] = a.nscale[c];
      bi[v][j] = a.nbias[c];
      fy[v][j] = j == 0 ? fyA : (j == 3 ? fyB : (j < nA[v] ? fyA : fyB));
    }
  }
  const float inv_d = 1.0f / (float)D, inv_dm1 = 1.0f / (float)(D - 1);
  const f32x4 zero = f32x4{0.f, 0.f, 0.f, 0.f};
  const float gscale = loss_gscale(a);
  double acc = 0.0;

  for (int gx = wave; gx < npatch; gx += nwaves) {
    const int64_t row_elem = ((int64_t)b * a.L + gy * a.G + gx0 + gx) * D;
    if (__builtin_amdgcn_readlane(masked, gx & (kWave - 1)) == 0) {  // visible: zero gradient
      if (a.grad) {
#pragma unroll
        for (int v = 0; v < NV; ++v)
          if (active[v]) crop_store_grad4(a.grad, row_elem + e[v], zero, bf16);
      }
      continue;
    }
    f32x4 q[NV], val[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v)
      q[v] = active[v] ? crop_load_pred4(a.pred, row_elem + e[v], bf16) : zero;
    float s = 0.f;
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      const u32x2 xa = xtab[gx * p + pxA[v]], xb = xtab[gx * p + pxB[v]];
      const float fxA = __uint_as_float(xa.y), fxB = __uint_as_float(xb.y);
      uint32_t A00, A01, A10, A11, B00, B01, B10, B11;
      fetch2<kLds>(tile, base, rowA0[v], (int)xa.x, cw, A00, A01);
      fetch2<kLds>(tile, base, rowA1[v], (int)xa.x, cw, A10, A11);
      fetch2<kLds>(tile, base, rowB0[v], (int)xb.x, cw, B00, B01);
      fetch2<kLds>(tile, base, rowB1[v], (int)xb.x, cw, B10, B11);
      const uint32_t P00 = __builtin_amdgcn_perm(B00, A00, sel[v]);
      const uint32_t P01 = __builtin_amdgcn_perm(B01, A01, sel[v]);
      const uint32_t P10 = __builtin_amdgcn_perm(B10, A10, sel[v]);
      const uint32_t P11 = __builtin_amdgcn_perm(B11, A11, sel[v]);
      float out[4];
#define MAE_BLEND(J)                                                                 \
{                                                                                  \
  const float fx = (J) == 0 ? fxA : ((J) == 3 ? fxB : ((J) < nA[v] ? fxA : fxB));  \
  const float a00 = byte_to_float<J>(P00), a01 = byte_to_float<J>(P01);            \
  const float a10 = byte_to_float<J>(P10), a11 = byte_to_float<J>(P11);            \
  const float rt = a00 + fx * (a01 - a00);                                         \
  const float rb = a10 + fx * (a11 - a10);                                         \
  const float t = rt + fy[v][J] * (rb - rt);                                       \
  out[J] = t * sc[v][J] + bi[v][J];                                                \
}
      MAE_BLEND(0) MAE_BLEND(1) MAE_BLEND(2) MAE_BLEND(3)
#undef MAE_BLEND
      val[v] = active[v] ? f32x4{out[0], out[1], out[2], out[3]} : zero;
      s += (val[v].x + val[v].y) + (val[v].z + val[v].w);
    }
    float rstd = 1.0f;
    if (a.norm_pix) {
#pragma unroll
      for (int off = kWave / 2; off > 0; off >>= 1) s += __shfl_xor(s, off, kWave);
      const float mu = s * inv_d;
      float ss = 0.f;
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        val[v] = val[v] - mu;
        if (active[v])
          ss += (val[v].x * val[v].x + val[v].y * val[v].y) +
                (val[v].z * val[v].z + val[v].w * val[v].w);
      }
#pragma unroll
      for (int off = kWave / 2; off > 0; off >>= 1) ss += __shfl_xor(ss, off, kWave);
      rstd = 1.0f / sqrtf(ss * inv_dm1 + a.eps);
    }
    float sq = 0.f;
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      if (!active[v]) continue;
      const f32x4 diff = q[v] - val[v] * rstd;
      sq += (diff.x * diff.x + diff.y * diff.y) + (diff.z * diff.z + diff.w * diff.w);
      if (a.grad) crop_store_grad4(a.grad, row_elem + e[v], diff * gscale, bf16);
    }
    acc += (double)sq;
  }
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) acc += __shfl_xor(acc, off, kWave);
  if (lane == 0) red64[wave] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    double t = 0.0;
    for (int w = 0; w < nwaves; ++w) t += red64[w];
    a.partials[tile_id] = t;
  }
}

// ---- the finetuning augmentation as the epilogue ("3 Aug", "3 Aug+": Sec. 3, Sec. 4.4, Table 7) ----
// The per-image operation acts on the resized crop rounded to bytes.  Grayscale and solarisation
// are pointwise, so they are applied to the rounded values while these are still in registers and
// the result goes straight to `target` / `visible`; the images that drew the blur only get their
// rounded bytes written (patch order) for the blur kernel.
//
// Grayscale and the jitter's saturation step need whole pixels, so here a lane takes four
// neighbouring pixels of a patch row (12 values) instead of four values -- two pixels when the
// patch size is even but no multiple of four (p = 14) --, and the groups of the part's patches
// are dealt to the lanes in order.  The 64 x 12 values of a wavefront go through a
// wavefront-private strip of LDS so that every store instruction still writes 1 KiB (512 bytes
// with two pixels per lane) of contiguous memory.  Tables: xtab.y = the integer weights den - rx, rx of the two columns as a pair
// of 16-bit values, ytab.z / ytab.w = the weights den - ry, ry of the two rows (den = 2 S).
//
// Rounding.  The bilinear value is num / den^2,
//   top = (den - rx) a00 + rx a01, bot likewise (two-product dot instructions on 16-bit pairs),
//   num = (den - ry) top + ry bot (24-bit multiplies: top, bot < 2^18, the sum < 2^28),
// rounded to the nearest integer, ties upwards: q = floor((num + den^2 / 2) / den^2), all in
// integers.  The quotient is estimated in single precision with the divisor's reciprocal scaled
// by (1 - 2^-21), which makes the estimate too small by at most 2e-4 and never too large, so its
// integer part is q or q - 1 and one comparison of the remainder settles it.
constexpr int kStripFloats = kWave * 12;  // per wavefront

// floor(n / d) for 0 <= n < 2^22 and small d, from the float reciprocal (inv = 1 / d)
__device__ static inline int small_div(int n, float inv) { return (int)(((float)n + 0.5f) * inv); }

// The three channels of the four taps (pixel words w00 w01 / w10 w11) blended and rounded, as
// floats.  wx = (den - rx) | rx << 16; cy, ry = the rows' weights; dd = den^2 < 2^23; inv_dd as
// described above.
// The dot and multiply-add instructions are written out as one block: the three-operand dot with
// a zero addend (the accumulating form would need its destination cleared first) and 24-bit
// multiply-adds (the compiler splits them into multiply + add).  A dot product's result may only
// be read by another kind of instruction three or more instructions later; inside the block every
// result is read five or more instructions after it is written, whatever is scheduled around it.
__device__ static inline void round_blend3(uint32_t w00, uint32_t w01, uint32_t w10, uint32_t w11,
                                           uint32_t wx, int cy, int ry, int dd, float inv_dd,
                                           float* out) {
  // byte C of the two words as a pair of 16-bit values (selector 0x0c gives a zero byte)
  uint32_t t[3], b[3];
#pragma unroll
  for (int c = 0; c < 3; ++c) {
    const uint32_t sel = 0x0c000c00u | ((4u + (uint32_t)c) << 16) | (uint32_t)c;
    t[c] = __builtin_amdgcn_perm(w01, w00, sel);
    b[c] = __builtin_amdgcn_perm(w11, w10, sel);
  }
  int n0, n1, n2, h0, h1, h2;
  asm("v_dot2_i32_i16 %3, %6, %12, 0\n\t"
      "v_dot2_i32_i16 %0, %7, %12, 0\n\t"
      "v_dot2_i32_i16 %4, %8, %12, 0\n\t"
      "v_dot2_i32_i16 %1, %9, %12, 0\n\t"
      "v_dot2_i32_i16 %5, %10, %12, 0\n\t"
      "v_dot2_i32_i16 %2, %11, %12, 0\n\t"
      "v_mad_i32_i24 %3, %13, %3, %15\n\t"
      "v_mad_i32_i24 %0, %14, %0, %3\n\t"
      "v_mad_i32_i24 %4, %13, %4, %15\n\t"
      "v_mad_i32_i24 %1, %14, %1, %4\n\t"
      "v_mad_i32_i24 %5, %13, %5, %15\n\t"
      "v_mad_i32_i24 %2, %14, %2, %5"
      : "=&v"(n0), "=&v"(n1), "=&v"(n2), "=&v"(h0), "=&v"(h1), "=&v"(h2)
      : "v"(t[0]), "v"(b[0]), "v"(t[1]), "v"(b[1]), "v"(t[2]), "v"(b[2]), "v"(wx), "v"(cy),
        "v"(ry), "s"(dd >> 1));
  const int num[3] = {n0, n1, n2};
#pragma unroll
  for (int c = 0; c < 3; ++c) {
    const int q = (int)((float)num[c] * inv_dd);
    int r;
    asm("v_mad_i32_i24 %0, %1, %2, %3" : "=v"(r) : "v"(q), "s"(-dd), "v"(num[c]));
    out[c] = (float)(q + (r >= dd ? 1 : 0));
  }
}

// kPass 0: "3 Aug", or the first pass of "3 Aug+" (kJitter: luma sums only); kPass 1: the second
// pass of "3 Aug+".  `blur`: this image goes to the blur kernel (bytes only; not called in pass 1).
// kPx: neighbouring pixels of a patch row per lane, 4 when p is a multiple of 4, else 2 (p even):
// a lane's values are 3 kPx floats = three pieces of kPx floats (16 or 8 bytes).
template <int kPx>
struct AugPiece;
template <>
struct AugPiece<4> {
  typedef f32x4 type;
};
template <>
struct AugPiece<2> {
  typedef float type __attribute__((ext_vector_type(2)));
};

template <bool kLds, bool kBf16, bool kJitter, int kPass, int kPx>
__device__ static void produce_aug(const CropArgs& a, const uint32_t* tile, const u32x2* xtab,
                                   const u32x4* ytab, const uint8_t* base, int b, int gy, int gx0,
                                   int npatch, int cw, int my_rank, const AugParams& ap, bool blur,
                                   float mean, float* strips, double* red64, uint32_t tile_id) {
  typedef typename AugPiece<kPx>::type piece_t;
  constexpr bool kReduce = kJitter && kPass == 0;
  constexpr int kVals = 3 * kPx;  // values per lane and step
  const int lane = threadIdx.x % kWave;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int p = a.p, D = a.D;
  const int den = 2 * a.S, dd = den * den;
  const float inv_dd = (1.0f / (float)dd) * (1.0f - 1.0f / 2097152.0f);
  const int gpp = (p * p) / kPx;  // groups of kPx pixels per patch
  const float inv_gpp = 1.0f / (float)gpp, inv_p = 1.0f / (float)p;
  const int ngroups = npatch * gpp;
  const int l0 = gy * a.G + gx0;
  const bool gray = ap.op == kOpGray;
  // patches of 16 x 16 or 32 x 32 pixels: the 64 groups of a wavefront's step lie in one patch
  const bool whole = kPx == 4 && (p & 15) == 0;
  const int gsh = __builtin_ctz(gpp), psh = __builtin_ctz(p);  // used when `whole`
  float* strip = strips + wave * (kWave * kVals);
  float lsum = 0.0f;
  // this image's rows of the outputs (uniform over the workgroup)
  float* target_image = a.target ? a.target + (int64_t)b * a.L * D : nullptr;
  uint8_t* u8_image = a.u8_out + (int64_t)b * a.L * D;
  void* visible_image =
      kBf16 ? static_cast<void*>(static_cast<uint16_t*>(a.visible) + (int64_t)b * a.K * D)
            : static_cast<void*>(static_cast<float*>(a.visible) + (int64_t)b * a.K * D);
  // one piece of a patch row of `target` / `visible` (element offsets inside the image)
  auto store_piece = [&](uint32_t target_off, int rank, uint32_t visible_off, piece_t t) {
    if (a.target) *reinterpret_cast<piece_t*>(target_image + target_off) = t;
    if (rank < a.K) {
      if (kBf16) {
        uint16_t* dst = static_cast<uint16_t*>(visible_image) + visible_off;
        if constexpr (kPx == 4)
          *reinterpret_cast<u32x2*>(dst) = u32x2{pack_bf16x2(t[0], t[1]), pack_bf16x2(t[2], t[3])};
        else
          *reinterpret_cast<uint32_t*>(dst) = pack_bf16x2(t[0], t[1]);
      } else {
        *reinterpret_cast<piece_t*>(static_cast<float*>(visible_image) + visible_off) = t;
      }
    }
  };

  // whole wavefronts stay in the loop: the stores are a wavefront's joint work
  for (int i0 = wave * kWave; i0 < ngroups; i0 += (int)blockDim.x) {
    bool have;
    int gx, q, py, px;
    if (whole) {
      have = true;
      gx = i0 >> gsh;  // uniform
      q = 4 * ((i0 & (gpp - 1)) + lane);
      py = q >> psh;
      px = q & (p - 1);
    } else {
      have = i0 + lane < ngroups;
      const int i = have ? i0 + lane : ngroups - 1;
      gx = small_div(i, inv_gpp);
      q = kPx * (i - __mul24(gx, gpp));  // first pixel of the group inside the patch
      py = small_div(q, inv_p);
      px = q - __mul24(py, p);
    }
    const int xt0 = __mul24(gx, p) + px;
    const u32x4 yt = ytab[py];
    const int cy = (int)yt.z, ry = (int)yt.w;

    float v[kVals];
#pragma unroll
    for (int j = 0; j < kPx; ++j) {
      const u32x2 xt = xtab[xt0 + j];
      uint32_t w00, w01, w10, w11;
      fetch2<kLds>(tile, base, yt.x, (int)xt.x, cw, w00, w01);
      fetch2<kLds>(tile, base, yt.y, (int)xt.x, cw, w10, w11);
      round_blend3(w00, w01, w10, w11, xt.y, cy, ry, dd, inv_dd, v + 3 * j);
    }

    if (blur) {  // the blur kernel's input: the rounded values as bytes
      if (have) {
        // offsets inside one image stay below 2^22: 24-bit multiplies, one 64-bit base
        uint8_t* dst = u8_image + (uint32_t)(__mul24(l0 + gx, D) + 3 * q);
        if constexpr (kPx == 4) {
#pragma unroll
          for (int k = 0; k < 3; ++k)
            reinterpret_cast<uint32_t*>(dst)[k] =
                (uint32_t)v[4 * k] | ((uint32_t)v[4 * k + 1] << 8) |
                ((uint32_t)v[4 * k + 2] << 16) | ((uint32_t)v[4 * k + 3] << 24);
        } else {
#pragma unroll
          for (int k = 0; k < 3; ++k)
            reinterpret_cast<uint16_t*>(dst)[k] =
                (uint16_t)((uint32_t)v[2 * k] | ((uint32_t)v[2 * k + 1] << 8));
        }
      }
      continue;
    }

#pragma unroll
    for (int h = 0; h < kPx; ++h) {
      if (gray) {
        // (299 R + 587 G + 114 B) / 1000 rounded to nearest: n + 1/2 is at least 0.0005 away from
        // a multiple of 1000 on either side, far more than the error of the product (n < 2^18)
        const float n =
            fmaf(299.0f, v[3 * h], fmaf(587.0f, v[3 * h + 1], fmaf(114.0f, v[3 * h + 2], 500.5f)));
        float g = floorf(n * 0.001f);
        if (kJitter) {
          // equal channels stay equal under the jitter: one channel's arithmetic, and the
          // saturation step leaves it as it is (the luma weights add up to one)
          g = clamp255(g * ap.brightness);
          if (kReduce) {
            lsum += have ? g : 0.0f;
          } else {
            g = clamp255(ap.contrast * g + (1.0f - ap.contrast) * mean);
          }
        }
        v[3 * h] = v[3 * h + 1] = v[3 * h + 2] = g;
        continue;
      } else {  // solarisation: v >= 128 -> 255 - v, which is the smaller of the two
#pragma unroll
        for (int c = 0; c < 3; ++c)  // (the median with zero of two non-negative numbers)
          v[3 * h + c] = __builtin_amdgcn_fmed3f(v[3 * h + c], 255.0f - v[3 * h + c], 0.0f);
      }
      if (kJitter) {
        const float lum = jitter_pixel<kReduce>(ap, mean, v[3 * h], v[3 * h + 1], v[3 * h + 2]);
        if (kReduce) lsum += have ? lum : 0.0f;
      }
    }
    if (kReduce) continue;

    // normalise, then through the strip: piece k of the strip belongs to group k / 3
    piece_t* mine = reinterpret_cast<piece_t*>(strip + kVals * lane);
    piece_t o[3];
#pragma unroll
    for (int k = 0; k < 3; ++k)
#pragma unroll
      for (int e = 0; e < kPx; ++e) {
        const int idx = kPx * k + e;
        o[k][e] = v[idx] * a.nscale[idx % 3] + a.nbias[idx % 3];
      }
    __builtin_amdgcn_wave_barrier();
    mine[0] = o[0];
    mine[1] = o[1];
    mine[2] = o[2];
    __builtin_amdgcn_wave_barrier();
    if (whole) {
      // one patch, 768 consecutive floats of its row from element 12 (i0 mod gpp) on
      const int gxs = __builtin_amdgcn_readfirstlane(gx);
      const int rank = __builtin_amdgcn_readlane(my_rank, gxs);
      const uint32_t e0 = 12u * (uint32_t)(i0 & (gpp - 1)) + 4u * (uint32_t)lane;
#pragma unroll
      for (int k = 0; k < 3; ++k) {
        const piece_t t = reinterpret_cast<const piece_t*>(strip)[k * kWave + lane];
        const uint32_t eo = e0 + 4u * kWave * k;
        store_piece((uint32_t)((l0 + gxs) * D) + eo, rank, (uint32_t)(rank * D) + eo, t);
      }
      continue;
    }
#pragma unroll
    for (int k = 0; k < 3; ++k) {
      const int piece = k * kWave + lane;
      const int g = i0 + small_div(piece, 1.0f / 3.0f);
      const piece_t t = reinterpret_cast<const piece_t*>(strip)[piece];
      const int pgx = small_div(min(g, ngroups - 1), inv_gpp);
      const int rank = __shfl(my_rank, pgx, kWave);
      if (g >= ngroups) continue;
      // element offset inside the patch row, then inside the image (below 2^20: 24-bit multiplies)
      const int eo = kVals * (g - __mul24(pgx, gpp)) + kPx * (piece - 3 * (g - i0));
      store_piece((uint32_t)(__mul24(l0 + pgx, D) + eo), rank, (uint32_t)(__mul24(rank, D) + eo), t);
    }
  }
  if (kReduce && !blur) {
    // the part's share of the image's luma sum: lanes by butterfly, wavefronts in index order
    double s = (double)lsum;
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) s += __shfl_xor(s, off, kWave);
    if (lane == 0) red64[wave] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
      double t = 0.0;
      const int nwaves = (int)blockDim.x / kWave;
      for (int w = 0; w < nwaves; ++w) t += red64[w];
      a.luma_partials[tile_id] = t;
    }
  }
}

// What a sample that cannot be used gets instead of pixels: zeros in its rows of `target` and, with
// the identity as its patch order, in rows l < K of `visible`; the workgroup of the sample's first
// part also writes the mask row (nothing masked) and the identity order.
__device__ static void neutral_outputs(const CropArgs& a, int b, int gy, int gx0, int npatch,
                                       int part) {
  const int D4 = a.D >> 2;
  const f32x4 zero = f32x4{0.f, 0.f, 0.f, 0.f};
  const int l0 = gy * a.G + gx0;
  for (int i = threadIdx.x; i < npatch * D4; i += (int)blockDim.x) {
    const int gx = i / D4, e = 4 * (i - gx * D4);
    const int l = l0 + gx;
    if (a.target) *reinterpret_cast<f32x4*>(a.target + ((int64_t)b * a.L + l) * a.D + e) = zero;
    if (l < a.K && a.visible) {
      const int64_t vo = ((int64_t)b * a.K + l) * a.D + e;
      if (a.visible_bf16)
        *reinterpret_cast<u32x2*>(static_cast<uint16_t*>(a.visible) + vo) = u32x2{0u, 0u};
      else
        *reinterpret_cast<f32x4*>(static_cast<float*>(a.visible) + vo) = zero;
    }
  }
  if (gy == 0 && part == 0) {
    for (int l = threadIdx.x; l < a.L; l += (int)blockDim.x) {
      if (a.mask_out) a.mask_out[(int64_t)b * a.L + l] = 0;
      if (a.order_out) a.order_out[(int64_t)b * a.L + l] = l;
      if (a.keep_out && l < a.K) a.keep_out[(int64_t)b * a.K + l] = l;
    }
    if (a.crop_out && threadIdx.x < 6) a.crop_out[(int64_t)b * 6 + threadIdx.x] = 0;
  }
}

// Dynamic LDS: [ tile: a.tile_pixels + 4 words | ytab: p x 16 bytes | xtab: a.part_patches p x 8 ].
// kLossMode 1, 2: instead of writing the patches, the loss and its gradient against a.pred
// (1: produce_loss, any patch size; 2: produce_loss_wave, patches of up to 768 values).
// kLossMode -1: the visible tokens only (no target).
// kAug: the finetuning augmentation as the epilogue (produce_aug): 1 = "3 Aug", 2 / 3 = first /
// second pass of "3 Aug+".
// kAugPx: pixels per lane of that epilogue (4 when p is a multiple of 4, else 2).
template <bool kBf16, int kLossMode, int kAug = 0, int kAugPx = 4>
__device__ static inline void crop_band(const CropArgs& a, uint32_t* lds) {
  constexpr bool kLoss = kLossMode > 0;
  constexpr bool kKeptOnly = kLossMode < 0;
  uint32_t* tile = lds;
  u32x4* ytab = reinterpret_cast<u32x4*>(lds + a.tile_pixels + 4);  // row y0, row y1, weight
  u32x2* xtab = reinterpret_cast<u32x2*>(ytab + a.p);                // x0, weight of x0 + 1

  const uint32_t tile_id = xcd_remap(blockIdx.x, gridDim.x);
  const uint32_t row_id = tile_id / (uint32_t)a.col_parts;
  const int part = (int)(tile_id - row_id * (uint32_t)a.col_parts);
  const int b = (int)(row_id / (uint32_t)a.G);
  const int gy = (int)(row_id - (uint32_t)b * (uint32_t)a.G);
  const int gx0 = part * a.G / a.col_parts;  // this part covers patches gx0 .. gx1 - 1
  const int gx1 = (part + 1) * a.G / a.col_parts;
  const int npatch = gx1 - gx0;
  const CropRec rec = reinterpret_cast<const CropRec*>(a.workspace + kWorkspaceHeader)[b];
  if (!rec.valid || npatch <= 0) {
    if constexpr (!kLoss) {
      // an unusable sample takes no part: zero pixels, nothing masked, identity order
      if (!rec.valid && npatch > 0) neutral_outputs(a, b, gy, gx0, npatch, part);
    }
    if constexpr (kLoss) {  // an unusable sample: nothing towards the loss, zero gradient
      if (threadIdx.x == 0) a.partials[tile_id] = 0.0;
      if (a.grad && npatch > 0) {
        const int64_t first = ((int64_t)b * a.L + gy * a.G + gx0) * a.D;
        for (int i = threadIdx.x; i < npatch * (a.D >> 2); i += (int)blockDim.x)
          crop_store_grad4(a.grad, first + 4 * (int64_t)i, f32x4{0.f, 0.f, 0.f, 0.f},
                           a.pred_bf16 != 0);
      }
    }
    return;
  }

  AugParams ap;
  bool blur = false;
  if constexpr (kAug != 0) {
    ap = static_cast<const AugParams*>(a.aug_recs)[b];
    blur = ap.op == kOpBlur;
    // second pass of "3 Aug+": the blur images' bytes are written already
    if (kAug == 3 && blur) return;
  }

  const int S = a.S, p = a.p;
  const int W = a.widths[b];
  const int tid = threadIdx.x;
  const int lane = tid % kWave, wave = tid / kWave;
  const int nwaves = (int)blockDim.x / kWave;

  // rows and columns of the crop that this part taps (taps are monotonic in the output index)
  const float inv_den = 1.0f / (float)(2 * S);
  int ylo, yhi, xlo, xhi, t0, t1;
  float tf;
  resize_taps(gy * p, rec.ch, S, inv_den, ylo, t1, tf);
  resize_taps(gy * p + p - 1, rec.ch, S, inv_den, t0, yhi, tf);
  const int ox_first = gx0 * p, ox_last = gx1 * p - 1;
  resize_taps(rec.flip ? S - 1 - ox_last : ox_first, rec.cw, S, inv_den, xlo, t1, tf);
  resize_taps(rec.flip ? S - 1 - ox_first : ox_last, rec.cw, S, inv_den, t0, xhi, tf);
  const int nrows = yhi - ylo + 1;
  const int ng = (xhi - xlo + 4) >> 2;  // groups of four pixels per staged row
  const int pitch = 4 * ng;             // pixel words per staged row
  const bool use_lds = nrows * pitch <= a.tile_pixels;
  const bool batched = use_lds && ng <= kWave;

  // first tapped pixel of the first tapped row
  const uint8_t* base =
      a.images + a.offsets[b] + ((int64_t)(rec.top + ylo) * W + rec.left + xlo) * 3;
  const int row_bytes = 3 * W;
  const uint8_t* img_end = a.images + a.images_bytes;
  u32x4* tile4 = reinterpret_cast<u32x4*>(tile);

  // noise rank of each patch of this part, one per lane; read back with readlane in the loop
  int my_rank;
  if (kLoss)  // whether the patch is masked
    my_rank = lane < npatch ? (a.mask[(int64_t)b * a.L + gy * a.G + gx0 + lane] != 0 ? 1 : 0) : 0;
  else
    my_rank = lane < npatch ? a.ids_restore[(int64_t)b * a.L + gy * a.G + gx0 + lane] : 0x7fffffff;

  u32x4 d[kStageRows];
  if (batched) {  // these loads stay in flight while the tap tables are built
#pragma unroll
    for (int u = 0; u < kStageRows; ++u) {
      const int r = wave + u * nwaves;
      d[u] = u32x4{0u, 0u, 0u, 0u};
      if (r < nrows && lane < ng) {
        const uint8_t* row = base + (int64_t)r * row_bytes;
        const uint8_t* arow = row - (reinterpret_cast<uintptr_t>(row) & 3u);
        const bool safe = arow >= a.images && arow + 12 * ng + 4 <= img_end;
        d[u] = load16(arow + 12 * lane, safe, a.images, img_end);
      }
    }
  }

  for (int i = tid; i < npatch * p; i += (int)blockDim.x) {
    const int ox = ox_first + i;
    int x0, x1, rem;
    float f;
    resize_taps(rec.flip ? S - 1 - ox : ox, rec.cw, S, inv_den, x0, x1, f, rem);
    // at the right edge both taps are the last pixel: weight 0 makes the second tap irrelevant
    if constexpr (kAug != 0) {  // the two integer weights 2 S - rem, rem as a pair of 16-bit values
      const uint32_t r = x1 == x0 ? 0u : (uint32_t)rem;
      xtab[i] = u32x2{(uint32_t)(x0 - xlo), ((uint32_t)(2 * S) - r) | (r << 16)};
    } else {
      xtab[i] = u32x2{(uint32_t)(x0 - xlo), x1 == x0 ? 0u : __float_as_uint(f)};
    }
  }
  for (int py = tid; py < p; py += (int)blockDim.x) {
    int y0, y1, rem;
    float f;
    resize_taps(gy * p + py, rec.ch, S, inv_den, y0, y1, f, rem);
    const uint32_t stride = use_lds ? (uint32_t)pitch : (uint32_t)row_bytes;
    if constexpr (kAug != 0)  // integer weights of the two rows: 2 S - rem, rem
      ytab[py] = u32x4{(uint32_t)(y0 - ylo) * stride, (uint32_t)(y1 - ylo) * stride,
                       (uint32_t)(2 * S - rem), (uint32_t)rem};
    else
      ytab[py] = u32x4{(uint32_t)(y0 - ylo) * stride, (uint32_t)(y1 - ylo) * stride,
                       __float_as_uint(f), 0u};
  }

  if (batched) {
#pragma unroll
    for (int u = 0; u < kStageRows; ++u) {
      const int r = wave + u * nwaves;
      if (r < nrows && lane < ng) {
        const uint32_t s = (uint32_t)reinterpret_cast<uintptr_t>(base + (int64_t)r * row_bytes) & 3u;
        tile4[r * ng + lane] = to_pixels(d[u], s);
      }
    }
  }
  if (use_lds) {  // rows beyond the first batch, and parts wider than 256 source pixels
    for (int r = batched ? wave + kStageRows * nwaves : wave; r < nrows; r += nwaves) {
      const uint8_t* row = base + (int64_t)r * row_bytes;
      const uint32_t s = (uint32_t)reinterpret_cast<uintptr_t>(row) & 3u;
      const uint8_t* arow = row - s;
      const bool safe = arow >= a.images && arow + 12 * ng + 4 <= img_end;
      for (int g = lane; g < ng; g += kWave)
        tile4[r * ng + g] = to_pixels(load16(arow + 12 * g, safe, a.images, img_end), s);
    }
  }
  __syncthreads();

  if constexpr (kAug != 0) {
    __shared__ double red64[kCropMaxThreads / kWave];
    constexpr bool kJitter = kAug >= 2;
    constexpr int kPass = kAug == 3 ? 1 : 0;
    // the wavefronts' strips follow the tables (16-byte aligned)
    float* strips = reinterpret_cast<float*>(
        lds + ((a.tile_pixels + 4 + 4 * a.p + 2 * a.part_patches * a.p + 3) & ~3));
    float mean = 0.0f;
    if constexpr (kAug == 3) {  // mean luma after the brightness step, from the first pass
      const int slots = a.G * a.col_parts;
      double sum = 0.0;
      for (int g = 0; g < slots; ++g) sum += a.luma_partials[(int64_t)b * slots + g];
      mean = (float)(sum / ((double)S * (double)S));
    }
#define MAE_PRODUCE_AUG(LDS)                                                                      \
  produce_aug<LDS, kBf16, kJitter, kPass, kAugPx>(a, tile, xtab, ytab, base, b, gy, gx0, npatch,  \
                                                  rec.cw - xlo, my_rank, ap, blur, mean, strips,  \
                                                  red64, tile_id)
    if (use_lds) MAE_PRODUCE_AUG(true);
    else MAE_PRODUCE_AUG(false);
#undef MAE_PRODUCE_AUG
  } else if constexpr (kLoss) {
    __shared__ float red[(kCropMaxThreads / kWave) * kLossChunk];
    __shared__ double red64[kCropMaxThreads / kWave];
    if constexpr (kLossMode == 2) {
      const int nv = ((a.D >> 2) + kWave - 1) / kWave;
#define MAE_LOSS_WAVE(LDS, NV)                                                                  \
  produce_loss_wave<LDS, NV>(a, tile, xtab, ytab, base, b, gy, gx0, npatch, rec.cw - xlo, my_rank, \
                             red64, tile_id)
      if (nv == 3 && use_lds) MAE_LOSS_WAVE(true, 3);
      else if (nv == 3) MAE_LOSS_WAVE(false, 3);
      else if (nv == 2 && use_lds) MAE_LOSS_WAVE(true, 2);
      else if (nv == 2) MAE_LOSS_WAVE(false, 2);
      else if (use_lds) MAE_LOSS_WAVE(true, 1);
      else MAE_LOSS_WAVE(false, 1);
#undef MAE_LOSS_WAVE
    } else if (use_lds) {
      produce_loss<true>(a, tile, xtab, ytab, base, b, gy, gx0, npatch, rec.cw - xlo, my_rank, red,
                         red64, tile_id);
    } else {
      produce_loss<false>(a, tile, xtab, ytab, base, b, gy, gx0, npatch, rec.cw - xlo, my_rank,
                          red, red64, tile_id);
    }
  } else if (use_lds) {
    produce_patches<true, kBf16, kKeptOnly>(a, tile, xtab, ytab, base, b, gy, gx0, npatch,
                                                 rec.cw - xlo, my_rank);
  } else {
    produce_patches<false, kBf16, kKeptOnly>(a, tile, xtab, ytab, base, b, gy, gx0, npatch,
                                                  rec.cw - xlo, my_rank);
  }
}

template <bool kBf16>
__global__ __launch_bounds__(kCropMaxThreads) void crop_patch_kernel(CropArgs a) {
  extern __shared__ __attribute__((aligned(16))) uint32_t lds[];
  crop_band<kBf16, 0>(a, lds);
}
// ... when no target is wanted: only the patches that are kept
template <bool kBf16>
__global__ __launch_bounds__(kCropMaxThreads) void crop_kept_kernel(CropArgs a) {
  extern __shared__ __attribute__((aligned(16))) uint32_t lds[];
  crop_band<kBf16, -1>(a, lds);
}

// ... with the finetuning augmentation's pointwise operations as the epilogue
template <bool kBf16, int kAug, int kPx>
__global__ __launch_bounds__(kCropMaxThreads) void crop_aug_kernel(CropArgs a) {
  extern __shared__ __attribute__((aligned(16))) uint32_t lds[];
  crop_band<kBf16, 0, kAug, kPx>(a, lds);
}

// The resampling kernel with the loss as its epilogue: what mae_normpix_loss computes, with the
// masked patches' pixels taken from the images again instead of from a stored target.
__global__ __launch_bounds__(kCropMaxThreads) void crop_loss_kernel(CropArgs a) {
  extern __shared__ __attribute__((aligned(16))) uint32_t lds[];
  crop_band<false, 1>(a, lds);
}
// ... with a wavefront per patch (D <= 768): four wavefronts per workgroup
__global__ __launch_bounds__(4 * kWave) void crop_loss_wave_kernel(CropArgs a) {
  extern __shared__ __attribute__((aligned(16))) uint32_t lds[];
  crop_band<false, 2>(a, lds);
}

// Patch sizes whose 3 p^2 values per patch are not a multiple of four (odd p): one output pixel
// per thread, taps straight from global memory.  Correct for every shape, not tuned further.
template <bool kBf16>
__global__ __launch_bounds__(kCropThreads) void crop_patch_scalar_kernel(CropArgs a) {
  // one output pixel (three values) per thread and pass: the taps are worked out once per pixel
  const int pp = a.p * a.p;
  const int64_t per_image = (int64_t)a.L * pp;
  const int64_t total = (int64_t)a.B * per_image;
  const float inv_den = 1.0f / (float)(2 * a.S);
  for (int64_t idx = (int64_t)blockIdx.x * kCropThreads + threadIdx.x; idx < total;
       idx += (int64_t)gridDim.x * kCropThreads) {
    const int b = (int)(idx / per_image);
    const int rem = (int)(idx - (int64_t)b * per_image);
    const CropRec rec = reinterpret_cast<const CropRec*>(a.workspace + kWorkspaceHeader)[b];
    const int l = rem / pp, q = rem - l * pp;
    const int64_t to = ((int64_t)b * a.L + l) * a.D + 3 * q;  // the pixel's values in `target`
    if (!rec.valid) {  // takes no part: zero pixels, nothing masked, identity order
      const int64_t vo = ((int64_t)b * a.K + l) * a.D + 3 * q;
      for (int c = 0; c < 3; ++c) {
        if (a.target) a.target[to + c] = 0.0f;
        if (l < a.K) {
          if (kBf16) static_cast<uint16_t*>(a.visible)[vo + c] = 0;
          else static_cast<float*>(a.visible)[vo + c] = 0.0f;
        }
      }
      if (q == 0) {
        if (a.mask_out) a.mask_out[(int64_t)b * a.L + l] = 0;
        if (a.order_out) a.order_out[(int64_t)b * a.L + l] = l;
        if (a.keep_out && l < a.K) a.keep_out[(int64_t)b * a.K + l] = l;
        if (a.crop_out && l == 0)
          for (int i = 0; i < 6; ++i) a.crop_out[(int64_t)b * 6 + i] = 0;
      }
      continue;
    }
    const int gy = l / a.G, gx = l - gy * a.G;
    const int py = q / a.p, px = q - py * a.p;
    const int oy = gy * a.p + py, ox = gx * a.p + px;
    int x0, x1, y0, y1;
    float fx, fy;
    resize_taps(rec.flip ? a.S - 1 - ox : ox, rec.cw, a.S, inv_den, x0, x1, fx);
    resize_taps(oy, rec.ch, a.S, inv_den, y0, y1, fy);
    const int W = a.widths[b];
    const uint8_t* img = a.images + a.offsets[b];
    const uint8_t* p00 = img + ((int64_t)(rec.top + y0) * W + rec.left + x0) * 3;
    const uint8_t* p01 = img + ((int64_t)(rec.top + y0) * W + rec.left + x1) * 3;
    const uint8_t* p10 = img + ((int64_t)(rec.top + y1) * W + rec.left + x0) * 3;
    const uint8_t* p11 = img + ((int64_t)(rec.top + y1) * W + rec.left + x1) * 3;
    const int rank = a.ids_restore[(int64_t)b * a.L + l];
    const int64_t vo = ((int64_t)b * a.K + rank) * a.D + 3 * q;
#pragma unroll
    for (int c = 0; c < 3; ++c) {
      const float a00 = p00[c], a01 = p01[c], a10 = p10[c], a11 = p11[c];
      const float rt = a00 + fx * (a01 - a00);
      const float rb = a10 + fx * (a11 - a10);
      const float v = (rt + fy * (rb - rt)) * a.nscale[c] + a.nbias[c];
      if (a.target) a.target[to + c] = v;
      if (rank < a.K) {
        if (kBf16) static_cast<uint16_t*>(a.visible)[vo + c] = (uint16_t)bf16_rne(v);
        else static_cast<float*>(a.visible)[vo + c] = v;
      }
    }
  }
}

// Launch plan of the resampling kernel when no image side exceeds max_side.  A row of patches
// taps at most ceil((p - 1) max_side / S) + 2 source rows; a column part of n patches taps at most
// min(max_side, ceil((n p - 1) max_side / S) + 2) source columns, rounded up to groups of four.  The row is split
// into the fewest parts (whole patches, a power of two) whose tile stays within kCropTileTarget
// bytes, so that several workgroups share a compute unit's LDS.
CropPlan crop_plan(int S, int p, int max_side, int force_parts) {
  const int G = S / p;
  const int64_t rows = ((int64_t)(p - 1) * max_side + S - 1) / S + 2;
  CropPlan plan;
  int parts = 1;
  for (;;) {
    const int n = (G + parts - 1) / parts;  // patches per part
    int64_t cols = ((int64_t)(n * p - 1) * max_side + S - 1) / S + 2;
    if (cols > max_side) cols = max_side;
    cols = (cols + 3) & ~(int64_t)3;
    const int64_t px = rows * cols;
    const int64_t fixed = 16 + 16 * (int64_t)p + 8 * (int64_t)n * p;
    const bool forced = force_parts > 0;
    const bool fits = px * 4 + fixed <= kCropTileTarget;
    if ((forced && parts >= force_parts) || (!forced && fits) || parts * 2 > G) {
      int64_t cap = (kCropMaxLds - fixed) / 4;
      plan.col_parts = parts;
      plan.part_patches = n;
      plan.tile_pixels = (int)((px < cap ? px : cap) & ~(int64_t)3);
      if (plan.tile_pixels < 256) plan.tile_pixels = 256;
      return plan;
    }
    parts *= 2;
  }
}

size_t crop_lds_bytes(const CropArgs& a) {
  return (size_t)(a.tile_pixels + 4) * 4 + (size_t)a.p * 16 + (size_t)a.part_patches * a.p * 8;
}

// First stage of adding the workgroups' partial sums (there are tens of thousands): workgroup w
// adds its contiguous share in a fixed order and leaves one double; the second stage is the
// single-workgroup kernel that finishes the other loss, too.
constexpr int kLossGroups = 128;
__global__ __launch_bounds__(256) void crop_loss_reduce_kernel(const double* partials, int64_t n,
                                                               double* out) {
  __shared__ double red[256];
  const int64_t chunk = (n + kLossGroups - 1) / kLossGroups;
  const int64_t lo = (int64_t)blockIdx.x * chunk, hi = min(n, lo + chunk);
  double s = 0.0;
  for (int64_t i = lo + threadIdx.x; i < hi; i += 256) s += partials[i];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int off = 128; off > 0; off >>= 1) {
    if ((int)threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) out[blockIdx.x] = red[0];
}

// Doubles of workspace: one per workgroup, then kLossGroups for the first stage of their sum.
int64_t crop_loss_partials(const CropArgs& a) {
  return (int64_t)a.B * a.G * a.col_parts + kLossGroups;
}

hipError_t launch_crop_loss(const CropArgs& a, hipStream_t stream) {
  dim3 grid((uint32_t)a.B * (uint32_t)a.G * (uint32_t)a.col_parts);
  const int nv = ((a.D >> 2) + kWave - 1) / kWave;
  // patches of up to 768 values are a wavefront's work each: four wavefronts share a part
  if (nv <= 3)
    hipLaunchKernelGGL(crop_loss_wave_kernel, grid, dim3(4 * kWave), crop_lds_bytes(a), stream, a);
  else
    hipLaunchKernelGGL(crop_loss_kernel, grid, dim3(kWave * nv), crop_lds_bytes(a), stream, a);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return err;
  const int64_t n = (int64_t)grid.x;
  hipLaunchKernelGGL(crop_loss_reduce_kernel, dim3(kLossGroups), dim3(256), 0, stream, a.partials,
                     n, a.partials + n);
  err = hipGetLastError();
  if (err != hipSuccess) return err;
  return launch_loss_finish(a.partials + n, kLossGroups, a.inv_count, a.loss_out, a.counts,
                            a.ncounts, a.D, stream);
}

hipError_t launch_crop_aug(const CropArgs& a, int pass, hipStream_t stream) {
  dim3 grid((uint32_t)a.B * (uint32_t)a.G * (uint32_t)a.col_parts);
  // the groups of four pixels are dealt to the lanes, so any number of wavefronts will do: at
  // most four (their strips share the LDS with the tile)
  const int waves = ((a.D >> 2) + kWave - 1) / kWave;
  dim3 block(kWave * (waves < 4 ? waves : 4));
  const size_t lds = ((crop_lds_bytes(a) + 15) & ~(size_t)15) +
                     (size_t)(block.x / kWave) * kStripFloats * sizeof(float);
  const int aug = a.aug_mode == 1 ? 1 : (pass == 0 ? 2 : 3);
  // four pixels per lane when they tile a patch row, else two (even patch sizes)
#define MAE_AUG_LAUNCH(BF, AUG)                                                          \
  do {                                                                                   \
    if ((a.p & 3) == 0)                                                                  \
      hipLaunchKernelGGL((crop_aug_kernel<BF, AUG, 4>), grid, block, lds, stream, a);    \
    else                                                                                 \
      hipLaunchKernelGGL((crop_aug_kernel<BF, AUG, 2>), grid, block, lds, stream, a);    \
  } while (0)
  if (a.visible_bf16) {
    if (aug == 1) MAE_AUG_LAUNCH(true, 1);
    else if (aug == 2) MAE_AUG_LAUNCH(true, 2);
    else MAE_AUG_LAUNCH(true, 3);
  } else {
    if (aug == 1) MAE_AUG_LAUNCH(false, 1);
    else if (aug == 2) MAE_AUG_LAUNCH(false, 2);
    else MAE_AUG_LAUNCH(false, 3);
  }
#undef MAE_AUG_LAUNCH
  return hipGetLastError();
}

hipError_t launch_crop_patch(const CropArgs& a, hipStream_t stream) {
  if ((a.D & 3) == 0) {
    dim3 grid((uint32_t)a.B * (uint32_t)a.G * (uint32_t)a.col_parts);
    dim3 block(kWave * (((a.D >> 2) + kWave - 1) / kWave));
    const size_t lds = crop_lds_bytes(a);
    if (!a.target && a.visible_bf16) {
      hipLaunchKernelGGL(crop_kept_kernel<true>, grid, block, lds, stream, a);
    } else if (!a.target) {
      hipLaunchKernelGGL(crop_kept_kernel<false>, grid, block, lds, stream, a);
    } else if (a.visible_bf16) {
      hipLaunchKernelGGL(crop_patch_kernel<true>, grid, block, lds, stream, a);
    } else {
      hipLaunchKernelGGL(crop_patch_kernel<false>, grid, block, lds, stream, a);
    }
  } else {
    const int64_t total = (int64_t)a.B * a.L * a.p * a.p;  // output pixels
    int64_t blocks = (total + kCropThreads - 1) / kCropThreads;
    if (blocks > 256 * 64) blocks = 256 * 64;
    dim3 grid((uint32_t)blocks), block(kCropThreads);
    if (a.visible_bf16) {
      hipLaunchKernelGGL(crop_patch_scalar_kernel<true>, grid, block, 0, stream, a);
    } else {
      hipLaunchKernelGGL(crop_patch_scalar_kernel<false>, grid, block, 0, stream, a);
    }
  }
  return hipGetLastError();
}

}  // namespace mae
