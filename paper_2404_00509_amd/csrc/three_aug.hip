// Finetuning augmentation "3 Aug" / "3 Aug+" (Sec. 3 finetuning recipe, Sec. 4.4 "Data
// Augmentation", Sec. 5.2 Table 7): per image one of grayscale / solarisation / Gaussian blur,
// optionally colour jitter (brightness, contrast, saturation), then mean/std normalisation, the
// ViT patch split and the gather of the kept patches.  Input is the 8-bit resized crop that the
// resampling kernel wrote, already in patch order ([B, L, D] bytes, the layout of `target`);
// output is the same `target` / `visible` layout as the pretraining path.
//
// Two kernels, both with one workgroup per (image, row of patches); a workgroup leaves at once
// when its image drew an operation of the other kernel.
//  * aug_point_kernel: grayscale and solarisation are pointwise, so nothing is staged and the band
//    is one linear stream: a lane takes the 12 bytes of four neighbouring pixels of a patch row
//    (one aligned load), applies the operation in integer arithmetic, jitter and normalisation
//    in fp32, and stores the 48 bytes at the same position of `target` (and of `visible` for
//    kept patches).
//  * aug_blur_kernel (bands split into column parts of whole patches): the vertical pass reads
//    the bytes of the 13 image rows around each value from the patch rows in global memory and
//    writes fp32 rows into LDS, six more pixels on either side included; the horizontal pass is
//    folded into the walk over the part in output order: a lane reads the 16 pixels around its
//    four with aligned 16-byte LDS reads and applies all 13 taps (zero beyond the radius).
// The contrast step needs the mean luma of the whole image after the brightness step: with jitter
// on, a first launch of the same kernels (kReduce) only accumulates that sum per band in double
// precision, and the second launch adds the G partial sums of its image in fixed order.
#include "mae_device.hpp"
#include "mae_kernels.hpp"

namespace mae {

constexpr int kAugThreads = 256;
constexpr int kMaxRadius = 6;  // ceil(3 * 2.0)
constexpr int kTaps = 2 * kMaxRadius + 1;

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x3 __attribute__((ext_vector_type(3)));
typedef u32x3 u32x3_a4 __attribute__((aligned(4)));

__device__ static inline float clamp255(float v) { return fminf(fmaxf(v, 0.0f), 255.0f); }
__device__ static inline float luma(float r, float g, float b) {
  return 0.299f * r + 0.587f * g + 0.114f * b;
}

// floor(n / d) for 0 <= n < 2^22 and small d, from the float reciprocal (inv = 1 / d)
__device__ static inline int fast_div(int n, float inv) { return (int)(((float)n + 0.5f) * inv); }

// What every workgroup needs first: its tile, the record of its image, the draws.
struct BandCtx {
  int b, gy;
  bool valid;
  AugParams ap;
};
__device__ static inline BandCtx band_ctx(const AugArgs& a) {
  BandCtx c;
  const uint32_t tile = xcd_remap(blockIdx.x, gridDim.x);
  c.b = (int)(tile / (uint32_t)a.G);
  c.gy = (int)(tile - (uint32_t)c.b * (uint32_t)a.G);
  c.valid = reinterpret_cast<const CropRec*>(a.workspace + kWorkspaceHeader)[c.b].valid != 0;
  c.ap = aug_params(a.key1, a.sample_base + (uint32_t)c.b, a.jitter);
  return c;
}

// Mean luma after the brightness step, from the partial sums of the reduction launch.
__device__ static inline float image_mean(const AugArgs& a, int b) {
  // one slot per (row of patches, column part of the blur kernel); unused slots hold zero
  const int slots = a.G * a.blur_parts;
  double sum = 0.0;
  for (int g = 0; g < slots; ++g) sum += a.partials[(int64_t)b * slots + g];
  return (float)(sum / ((double)a.S * (double)a.S));
}

// Colour jitter of one pixel (fp32).  kReduce: only the brightness step, returns its luma.
template <bool kReduce>
__device__ static inline float jitter_pixel(const AugParams& ap, float mean, float& r, float& g,
                                            float& bl) {
  r = clamp255(r * ap.brightness);
  g = clamp255(g * ap.brightness);
  bl = clamp255(bl * ap.brightness);
  if (kReduce) return luma(r, g, bl);
  const float cm = (1.0f - ap.contrast) * mean;
  r = clamp255(ap.contrast * r + cm);
  g = clamp255(ap.contrast * g + cm);
  bl = clamp255(ap.contrast * bl + cm);
  const float sl = (1.0f - ap.saturation) * luma(r, g, bl);
  r = clamp255(ap.saturation * r + sl);
  g = clamp255(ap.saturation * g + sl);
  bl = clamp255(ap.saturation * bl + sl);
  return 0.0f;
}

// Normalise the 12 values of four pixels and store them to `target` and, for a kept patch, to
// `visible`.  q = index of the first pixel inside the patch (a multiple of 4).
template <bool kBf16>
__device__ static inline void store_group(const AugArgs& a, int b, int l, int q, const float* v) {
  float out[12];
#pragma unroll
  for (int j = 0; j < 12; ++j) out[j] = v[j] * a.nscale[j % 3] + a.nbias[j % 3];
  const int64_t eo = (int64_t)3 * q;  // 48-byte aligned run inside the patch row
  if (a.target) {
    f32x4* dst = reinterpret_cast<f32x4*>(a.target + ((int64_t)b * a.L + l) * a.D + eo);
    dst[0] = f32x4{out[0], out[1], out[2], out[3]};
    dst[1] = f32x4{out[4], out[5], out[6], out[7]};
    dst[2] = f32x4{out[8], out[9], out[10], out[11]};
  }
  const int rank = a.ids_restore[(int64_t)b * a.L + l];
  if (rank < a.K) {
    const int64_t vo = ((int64_t)b * a.K + rank) * a.D + eo;
    if (kBf16) {
      u32x2* dst = reinterpret_cast<u32x2*>(static_cast<uint16_t*>(a.visible) + vo);
      dst[0] = u32x2{pack_bf16x2(out[0], out[1]), pack_bf16x2(out[2], out[3])};
      dst[1] = u32x2{pack_bf16x2(out[4], out[5]), pack_bf16x2(out[6], out[7])};
      dst[2] = u32x2{pack_bf16x2(out[8], out[9]), pack_bf16x2(out[10], out[11])};
    } else {
      f32x4* dst = reinterpret_cast<f32x4*>(static_cast<float*>(a.visible) + vo);
      dst[0] = f32x4{out[0], out[1], out[2], out[3]};
      dst[1] = f32x4{out[4], out[5], out[6], out[7]};
      dst[2] = f32x4{out[8], out[9], out[10], out[11]};
    }
  }
}

// The same for a whole wavefront whose lanes hold consecutive groups (first group `g0`, a multiple
// of 64, of the run of patches that starts with patch l0): the 64 x 12 values go through a wavefront-private strip of LDS so that every store
// instruction writes 1 KiB of contiguous memory instead of 16 bytes out of every 48.
template <bool kBf16>
__device__ static inline void store_groups_wave(const AugArgs& a, int b, int l0, int g0,
                                                int groups_per_patch, float inv_gpp, int ngroups,
                                                float* strip, const float* v, bool have) {
  const int lane = threadIdx.x % kWave;
  f32x4* mine = reinterpret_cast<f32x4*>(strip + 12 * lane);
  f32x4 o[3];
#pragma unroll
  for (int j = 0; j < 3; ++j) {
    float t[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int idx = 4 * j + e;
      t[e] = v[idx] * a.nscale[idx % 3] + a.nbias[idx % 3];
    }
    o[j] = f32x4{t[0], t[1], t[2], t[3]};
  }
  __builtin_amdgcn_wave_barrier();
  if (have) {
    mine[0] = o[0];
    mine[1] = o[1];
    mine[2] = o[2];
  }
  __builtin_amdgcn_wave_barrier();
#pragma unroll
  for (int j = 0; j < 3; ++j) {
    const int piece = j * kWave + lane;      // 16-byte piece of the strip
    const int g = g0 + fast_div(piece, 1.0f / 3.0f);  // the group it belongs to
    if (g >= ngroups) continue;
    const f32x4 t = reinterpret_cast<const f32x4*>(strip)[piece];
    const int gx = fast_div(g, inv_gpp);
    const int l = l0 + gx;
    const int64_t eo = 12 * (int64_t)(g - gx * groups_per_patch) + 4 * (piece - 3 * (g - g0));
    if (a.target)
      *reinterpret_cast<f32x4*>(a.target + ((int64_t)b * a.L + l) * a.D + eo) = t;
    const int rank = a.ids_restore[(int64_t)b * a.L + l];
    if (rank < a.K) {
      const int64_t vo = ((int64_t)b * a.K + rank) * a.D + eo;
      if (kBf16) {
        *reinterpret_cast<u32x2*>(static_cast<uint16_t*>(a.visible) + vo) =
            u32x2{pack_bf16x2(t.x, t.y), pack_bf16x2(t.z, t.w)};
      } else {
        *reinterpret_cast<f32x4*>(static_cast<float*>(a.visible) + vo) = t;
      }
    }
  }
}

// Sum over the workgroup in a fixed order (lanes by butterfly, wavefronts in index order).
template <int kThreads>
__device__ static inline void store_band_sum(const AugArgs& a, int b, int slot, float lsum,
                                             double* red) {
  double s = (double)lsum;
  for (int off = kWave / 2; off > 0; off >>= 1) s += __shfl_xor(s, off);
  const int tid = threadIdx.x;
  if ((tid % kWave) == 0) red[tid / kWave] = s;
  __syncthreads();
  if (tid == 0) {
    double t = 0.0;
    for (int w = 0; w < kThreads / kWave; ++w) t += red[w];
    a.partials[(int64_t)b * a.G * a.blur_parts + slot] = t;
  }
}

// ---- grayscale and solarisation ------------------------------------------------------------------
template <bool kReduce, bool kBf16>
__global__ __launch_bounds__(kAugThreads) void aug_point_kernel(AugArgs a) {
  __shared__ double red[kAugThreads / kWave];
  __shared__ __attribute__((aligned(16))) float strips[kAugThreads * 12];
  const BandCtx c = band_ctx(a);
  if (!c.valid || c.ap.op == kOpBlur) return;
  const int p = a.p, G = a.G;
  const int b = c.b, gy = c.gy;
  const uint8_t* band = a.u8 + ((int64_t)b * a.L + gy * G) * a.D;  // G * D bytes, patch order
  const float mean = (!kReduce && a.mode == 2) ? image_mean(a, b) : 0.0f;
  const bool gray = c.ap.op == kOpGray;
  const int groups_per_patch = (p * p) >> 2;
  const float inv_gpp = 1.0f / (float)groups_per_patch;
  float lsum = 0.0f;
  const int ngroups = G * groups_per_patch;
  float* strip = strips + (threadIdx.x / kWave) * (kWave * 12);
  // whole wavefronts stay in the loop (the stores are a wavefront's joint work)
  for (int i0 = (threadIdx.x / kWave) * kWave; i0 < ngroups; i0 += kAugThreads) {
    const int i = i0 + threadIdx.x % kWave;
    const bool have = i < ngroups;
    const u32x3 w = have ? *reinterpret_cast<const u32x3_a4*>(band + 12 * (int64_t)i)
                         : u32x3{0u, 0u, 0u};
    int by[12];
#pragma unroll
    for (int j = 0; j < 12; ++j) by[j] = (int)((w[j >> 2] >> (8 * (j & 3))) & 0xFFu);
    float v[12];
#pragma unroll
    for (int h = 0; h < 4; ++h) {
      if (gray) {
        const int g = (299 * by[3 * h] + 587 * by[3 * h + 1] + 114 * by[3 * h + 2] + 500) / 1000;
        v[3 * h] = v[3 * h + 1] = v[3 * h + 2] = (float)g;
      } else {
#pragma unroll
        for (int ch = 0; ch < 3; ++ch) {
          const int t = by[3 * h + ch];
          v[3 * h + ch] = (float)(t >= 128 ? 255 - t : t);
        }
      }
      if (a.mode == 2) {
        const float lum = jitter_pixel<kReduce>(c.ap, mean, v[3 * h], v[3 * h + 1], v[3 * h + 2]);
        lsum += have ? lum : 0.0f;
      }
    }
    if (!kReduce)
      store_groups_wave<kBf16>(a, b, gy * G, i0, groups_per_patch, inv_gpp, ngroups, strip, v,
                               have);
  }
  if (kReduce) {
    store_band_sum<kAugThreads>(a, b, gy * a.blur_parts, lsum, red);
    // the slots of the blur kernel's other column parts stay empty for this image
    if (threadIdx.x > 0 && (int)threadIdx.x < a.blur_parts)
      a.partials[((int64_t)b * G + gy) * a.blur_parts + threadIdx.x] = 0.0;
  }
}

// ---- Gaussian blur ---------------------------------------------------------------------------------
// One workgroup per (image, row of patches, column part of whole patches).  Dynamic LDS: p rows of
// 3 (W + 12) floats, W = widest part in pixels: the vertically blurred values of the part's
// columns and of six more pixels on either side (neighbouring columns, or the image's border
// pixel repeated).  The vertical pass reads the 8-bit patch rows straight from global memory:
// always 13 row taps per value (zero weight beyond the radius, rows clamped at the border), so
// that all loads of a value are in flight together.
template <bool kReduce, bool kBf16>
__global__ __launch_bounds__(kAugThreads) void aug_blur_kernel(AugArgs a) {
  extern __shared__ __attribute__((aligned(16))) float vals[];
  __shared__ double wd[kTaps];
  __shared__ float wf[kTaps];  // tap k - 6 at index k; zero beyond the radius
  __shared__ int rowoff[48];   // byte offset of image row y0 - 6 + j inside patch 0 of its grid row
  __shared__ double red[kAugThreads / kWave];
  __shared__ __attribute__((aligned(16))) float strips[kAugThreads * 12];

  const int S = a.S, p = a.p, G = a.G, parts = a.blur_parts;
  const uint32_t tile = xcd_remap(blockIdx.x, gridDim.x);
  const uint32_t band_id = tile / (uint32_t)parts;
  const int part = (int)(tile - band_id * (uint32_t)parts);
  const int b = (int)(band_id / (uint32_t)G);
  const int gy = (int)(band_id - (uint32_t)b * (uint32_t)G);
  const int gx0 = part * G / parts, gx1 = (part + 1) * G / parts;
  const int npatch = gx1 - gx0;
  const bool valid = reinterpret_cast<const CropRec*>(a.workspace + kWorkspaceHeader)[b].valid != 0;
  const AugParams ap = aug_params(a.key1, a.sample_base + (uint32_t)b, a.jitter);
  if (!valid || ap.op != kOpBlur || npatch <= 0) return;

  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int pv = 3 * (a.blur_part_patches * p + 2 * kMaxRadius);  // floats per row, 16-byte multiple
  const int Wp = npatch * p, x_lo = gx0 * p;
  const int prow = 3 * p, prow4 = prow >> 2;  // bytes / words per patch row
  const float inv_prow4 = 1.0f / (float)prow4, inv_p = 1.0f / (float)p;
  const uint8_t* img = a.u8 + (int64_t)b * a.L * a.D;  // patch order
  const int y0 = gy * p;
  const int radius = ap.radius;

  // taps exp(-k^2 / (2 sigma^2)) in double precision, summed in index order, scaled to sum 1
  if (tid < kTaps) {
    const double k = (double)(tid - kMaxRadius);
    wd[tid] = abs(tid - kMaxRadius) <= radius ? exp(-(k * k) / (2.0 * ap.sigma * ap.sigma)) : 0.0;
  }
  if (tid >= kWave && tid < kWave + p + 2 * kMaxRadius) {
    const int j = tid - kWave;
    const int yy = min(max(y0 - kMaxRadius + j, 0), S - 1);
    const int gyy = fast_div(yy, inv_p);
    rowoff[j] = gyy * G * a.D + (yy - gyy * p) * prow;
  }
  __syncthreads();
  if (tid < kTaps) {
    double sum = 0.0;
    for (int k = kMaxRadius - radius; k <= kMaxRadius + radius; ++k) sum += wd[k];
    wf[tid] = (float)(wd[tid] / sum);
  }
  __syncthreads();
  float wt[kTaps];
#pragma unroll
  for (int k = 0; k < kTaps; ++k) wt[k] = wf[k];

  // vertical pass over the part's own columns, four neighbouring values (one word) per step
  const int words = npatch * prow4;
  for (int y = wave; y < p; y += kAugThreads / kWave) {
    for (int d = lane; d < words; d += kWave) {
      const int gxl = fast_div(d, inv_prow4);
      const int64_t col = (int64_t)(gx0 + gxl) * a.D + 4 * (d - gxl * prow4);
      uint32_t w4[kTaps];
#pragma unroll
      for (int k = 0; k < kTaps; ++k)
        w4[k] = *reinterpret_cast<const uint32_t*>(img + rowoff[y + k] + col);
      float acc0 = 0.f, acc1 = 0.f, acc2 = 0.f, acc3 = 0.f;
#pragma unroll
      for (int k = 0; k < kTaps; ++k) {
        acc0 += wt[k] * (float)(w4[k] & 0xFFu);
        acc1 += wt[k] * (float)((w4[k] >> 8) & 0xFFu);
        acc2 += wt[k] * (float)((w4[k] >> 16) & 0xFFu);
        acc3 += wt[k] * (float)(w4[k] >> 24);
      }
      // 18 + 4 d floats into the row: 8-byte aligned
      f32x2* dst = reinterpret_cast<f32x2*>(vals + y * pv + 3 * kMaxRadius + 4 * d);
      dst[0] = f32x2{acc0, acc1};
      dst[1] = f32x2{acc2, acc3};
    }
  }
  // ... and over the six pixels on either side of the part
  for (int i = tid; i < p * 2 * kMaxRadius * 3; i += kAugThreads) {
    const int y = i / (2 * kMaxRadius * 3);
    const int r = i - y * (2 * kMaxRadius * 3);
    const int side = r / (kMaxRadius * 3), t = r - side * (kMaxRadius * 3);
    const int jpx = t / 3, ch = t - 3 * jpx;
    const int x = min(max(side == 0 ? x_lo - kMaxRadius + jpx : x_lo + Wp + jpx, 0), S - 1);
    const int gx = fast_div(x, inv_p);
    const int64_t col = (int64_t)gx * a.D + 3 * (x - gx * p) + ch;
    float acc = 0.f;
#pragma unroll
    for (int k = 0; k < kTaps; ++k) acc += wt[k] * (float)img[rowoff[y + k] + col];
    vals[y * pv + (side == 0 ? t : 3 * (kMaxRadius + Wp) + t)] = acc;
  }
  __syncthreads();

  const float mean = (!kReduce && a.mode == 2) ? image_mean(a, b) : 0.0f;
  const int groups_per_patch = (p * p) >> 2;
  const float inv_gpp = 1.0f / (float)groups_per_patch;
  const int ngroups = npatch * groups_per_patch;
  float* strip = strips + wave * (kWave * 12);
  float lsum = 0.0f;
  for (int i0 = wave * kWave; i0 < ngroups; i0 += kAugThreads) {
    const int i = min(i0 + lane, ngroups - 1);
    const bool have = i0 + lane < ngroups;
    const int gxl = fast_div(i, inv_gpp);
    const int q = 4 * (i - gxl * groups_per_patch);
    const int py = fast_div(q, inv_p), x = gxl * p + (q - py * p);  // pixel inside the part
    // padded pixels x .. x + 15 are the part's pixels x - 6 .. x + 9: 48 floats, 16-byte aligned
    const f32x4* src = reinterpret_cast<const f32x4*>(vals + py * pv + 3 * x);
    float n[48];
#pragma unroll
    for (int j = 0; j < 12; ++j) {
      const f32x4 t = src[j];
      n[4 * j] = t.x;
      n[4 * j + 1] = t.y;
      n[4 * j + 2] = t.z;
      n[4 * j + 3] = t.w;
    }
    float v[12];
#pragma unroll
    for (int h = 0; h < 4; ++h) {
      float r = 0.f, g = 0.f, bl = 0.f;
#pragma unroll
      for (int k = 0; k < kTaps; ++k) {
        r += wt[k] * n[3 * (h + k)];
        g += wt[k] * n[3 * (h + k) + 1];
        bl += wt[k] * n[3 * (h + k) + 2];
      }
      v[3 * h] = r;
      v[3 * h + 1] = g;
      v[3 * h + 2] = bl;
      if (a.mode == 2) {
        const float lum = jitter_pixel<kReduce>(ap, mean, v[3 * h], v[3 * h + 1], v[3 * h + 2]);
        lsum += have ? lum : 0.0f;
      }
    }
    if (!kReduce)
      store_groups_wave<kBf16>(a, b, gy * G + gx0, i0, groups_per_patch, inv_gpp, ngroups, strip,
                               v, have);
  }
  if (kReduce) store_band_sum<kAugThreads>(a, b, (gy * parts + part), lsum, red);
}

// Column parts of the blur kernel: the fewest (whole patches each) whose rows fit 24 KiB of LDS,
// so that four workgroups share a compute unit.
AugPlan three_aug_plan(int S, int p) {
  const int G = S / p;
  AugPlan plan;
  for (int parts = 1;; ++parts) {
    const int n = (G + parts - 1) / parts;
    const size_t lds = (size_t)p * 3 * (n * p + 2 * kMaxRadius) * 4;
    if (lds <= 24 * 1024 || parts >= G) {
      plan.parts = parts;
      plan.part_patches = n;
      plan.lds_bytes = lds;
      return plan;
    }
  }
}

hipError_t launch_three_aug(const AugArgs& a, hipStream_t stream) {
  dim3 grid((uint32_t)a.B * (uint32_t)a.G), block(kAugThreads);
  dim3 bgrid((uint32_t)a.B * (uint32_t)a.G * (uint32_t)a.blur_parts);
  const size_t lds = (size_t)a.p * 3 * (a.blur_part_patches * a.p + 2 * kMaxRadius) * 4;
  if (a.mode == 2) {
    hipLaunchKernelGGL((aug_point_kernel<true, false>), grid, block, 0, stream, a);
    hipLaunchKernelGGL((aug_blur_kernel<true, false>), bgrid, block, lds, stream, a);
  }
  if (a.visible_bf16) {
    hipLaunchKernelGGL((aug_point_kernel<false, true>), grid, block, 0, stream, a);
    hipLaunchKernelGGL((aug_blur_kernel<false, true>), bgrid, block, lds, stream, a);
  } else {
    hipLaunchKernelGGL((aug_point_kernel<false, false>), grid, block, 0, stream, a);
    hipLaunchKernelGGL((aug_blur_kernel<false, false>), bgrid, block, lds, stream, a);
  }
  return hipGetLastError();
}

}  // namespace mae
