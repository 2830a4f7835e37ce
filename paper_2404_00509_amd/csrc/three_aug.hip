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
//  * aug_blur_kernel: the image rows of the band plus `radius` rows above and below (clamped at
//    the image border) are gathered from the patch rows and staged as bytes, the vertical pass
//    writes fp32 rows into LDS with six border pixels repeated on either side, and the
//    horizontal pass is folded into the walk over the band in output order:
//    a lane reads the 16 pixels around its four with aligned 16-byte LDS reads and applies all
//    13 taps (zero beyond the radius).
// The contrast step needs the mean luma of the whole image after the brightness step: with jitter
// on, a first launch of the same kernels (kReduce) only accumulates that sum per band in double
// precision, and the second launch adds the G partial sums of its image in fixed order.
#include "mae_device.hpp"
#include "mae_kernels.hpp"

namespace mae {

constexpr int kAugThreads = 256;    // pointwise kernel
constexpr int kBlurThreads = 1024;  // blur kernel: its LDS allows two workgroups per compute unit,
                                    // so the wavefronts that hide latency have to come from its size
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
  double sum = 0.0;
  for (int g = 0; g < a.G; ++g) sum += a.partials[(int64_t)b * a.G + g];
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
// of 64): the 64 x 12 values go through a wavefront-private strip of LDS so that every store
// instruction writes 1 KiB of contiguous memory instead of 16 bytes out of every 48.
template <bool kBf16>
__device__ static inline void store_groups_wave(const AugArgs& a, int b, int gy, int g0,
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
    const int l = gy * a.G + gx;
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
__device__ static inline void store_band_sum(const AugArgs& a, int b, int gy, float lsum,
                                             double* red) {
  double s = (double)lsum;
  for (int off = kWave / 2; off > 0; off >>= 1) s += __shfl_xor(s, off);
  const int tid = threadIdx.x;
  if ((tid % kWave) == 0) red[tid / kWave] = s;
  __syncthreads();
  if (tid == 0) {
    double t = 0.0;
    for (int w = 0; w < kThreads / kWave; ++w) t += red[w];
    a.partials[(int64_t)b * a.G + gy] = t;
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
      store_groups_wave<kBf16>(a, b, gy, i0, groups_per_patch, inv_gpp, ngroups, strip, v, have);
  }
  if (kReduce) store_band_sum<kAugThreads>(a, b, gy, lsum, red);
}

// ---- Gaussian blur ---------------------------------------------------------------------------------
// Dynamic LDS: [ vals: p rows of 3 (S + 12) floats | staged bytes: (p + 12) rows of 3 S ].
template <bool kReduce, bool kBf16>
__global__ __launch_bounds__(kBlurThreads) void aug_blur_kernel(AugArgs a) {
  extern __shared__ __attribute__((aligned(16))) uint32_t lds[];
  __shared__ double wd[kTaps];
  __shared__ float wf[kTaps];  // tap k - 6 at index k; zero beyond the radius
  __shared__ double red[kBlurThreads / kWave];
  const BandCtx c = band_ctx(a);
  if (!c.valid || c.ap.op != kOpBlur) return;
  const int S = a.S, p = a.p, G = a.G;
  const int b = c.b, gy = c.gy, tid = threadIdx.x;
  const int rv = 3 * S, rv4 = rv >> 2;
  const int pv = 3 * (S + 2 * kMaxRadius);  // floats per padded row; 16-byte multiple
  float* vals = reinterpret_cast<float*>(lds);
  uint32_t* staged = lds + p * pv;
  const uint8_t* img = a.u8 + (int64_t)b * a.L * a.D;  // patch order
  const int y0 = gy * p;
  const int lane = tid % kWave, wave = tid / kWave;
  const int prow4 = (3 * p) >> 2;  // words per patch row
  const float inv_prow4 = 1.0f / (float)prow4, inv_p = 1.0f / (float)p;
  const int radius = c.ap.radius;

  // taps exp(-k^2 / (2 sigma^2)) in double precision, summed in index order, scaled to sum 1
  if (tid < kTaps) {
    const double k = (double)(tid - kMaxRadius);
    wd[tid] = abs(tid - kMaxRadius) <= radius ? exp(-(k * k) / (2.0 * c.ap.sigma * c.ap.sigma))
                                               : 0.0;
  }
  // the band and its halo, border rows repeated
  const int nrows = p + 2 * radius;
  for (int j = wave; j < nrows; j += kBlurThreads / kWave) {
    const int yy = min(max(y0 - radius + j, 0), S - 1);
    const int gyy = fast_div(yy, inv_p), pyy = yy - gyy * p;
    const uint8_t* row = img + (int64_t)gyy * G * a.D + pyy * 3 * p;  // patch 0 of that grid row
    for (int d = lane; d < rv4; d += kWave) {
      const int gx = fast_div(d, inv_prow4);
      staged[j * rv4 + d] =
          reinterpret_cast<const uint32_t*>(row + (int64_t)gx * a.D)[d - gx * prow4];
    }
  }
  __syncthreads();
  if (tid < kTaps) {
    double sum = 0.0;
    for (int k = kMaxRadius - radius; k <= kMaxRadius + radius; ++k) sum += wd[k];
    wf[tid] = (float)(wd[tid] / sum);
  }
  __syncthreads();
  // vertical pass: four neighbouring values (the bytes of one word) per step
  for (int y = wave; y < p; y += kBlurThreads / kWave) {
    for (int d = lane; d < rv4; d += kWave) {
      float acc0 = 0.f, acc1 = 0.f, acc2 = 0.f, acc3 = 0.f;
      for (int k = 0; k <= 2 * radius; ++k) {
        const uint32_t w4 = staged[(y + k) * rv4 + d];
        const float w = wf[kMaxRadius - radius + k];
        acc0 += w * (float)(w4 & 0xFFu);
        acc1 += w * (float)((w4 >> 8) & 0xFFu);
        acc2 += w * (float)((w4 >> 16) & 0xFFu);
        acc3 += w * (float)(w4 >> 24);
      }
      // 18 + 4 d floats into the row: 8-byte aligned
      f32x2* dst = reinterpret_cast<f32x2*>(vals + y * pv + 3 * kMaxRadius + 4 * d);
      dst[0] = f32x2{acc0, acc1};
      dst[1] = f32x2{acc2, acc3};
    }
  }
  __syncthreads();
  // six border pixels repeated on either side of every row
  for (int i = tid; i < p * 2 * kMaxRadius * 3; i += kBlurThreads) {
    const int y = i / (2 * kMaxRadius * 3);
    const int r = i - y * (2 * kMaxRadius * 3);
    const int side = r / (kMaxRadius * 3), t = r - side * (kMaxRadius * 3);
    const int ch = t % 3;
    float* row = vals + y * pv;
    if (side == 0) {
      row[t] = row[3 * kMaxRadius + ch];
    } else {
      row[3 * (kMaxRadius + S) + t] = row[3 * (kMaxRadius + S - 1) + ch];
    }
  }
  __syncthreads();

  const float mean = (!kReduce && a.mode == 2) ? image_mean(a, b) : 0.0f;
  float wt[kTaps];
#pragma unroll
  for (int k = 0; k < kTaps; ++k) wt[k] = wf[k];
  const int groups_per_patch = (p * p) >> 2;
  const float inv_gpp = 1.0f / (float)groups_per_patch;
  float lsum = 0.0f;
  for (int i = tid; i < G * groups_per_patch; i += kBlurThreads) {
    const int gx = fast_div(i, inv_gpp);
    const int q = 4 * (i - gx * groups_per_patch);
    const int py = fast_div(q, inv_p), x = gx * p + (q - py * p);
    // padded pixels x .. x + 15 are image pixels x - 6 .. x + 9: 48 floats, 16-byte aligned
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
      if (a.mode == 2)
        lsum += jitter_pixel<kReduce>(c.ap, mean, v[3 * h], v[3 * h + 1], v[3 * h + 2]);
    }
    if (!kReduce) store_group<kBf16>(a, b, gy * G + gx, q, v);
  }
  if (kReduce) store_band_sum<kBlurThreads>(a, b, gy, lsum, red);
}

size_t three_aug_lds_bytes(int S, int p) {
  return (size_t)p * 3 * (S + 2 * kMaxRadius) * 4 + (size_t)(p + 2 * kMaxRadius) * 3 * S;
}

hipError_t launch_three_aug(const AugArgs& a, hipStream_t stream) {
  dim3 grid((uint32_t)a.B * (uint32_t)a.G), block(kAugThreads), bblock(kBlurThreads);
  const size_t lds = three_aug_lds_bytes(a.S, a.p);
  if (a.mode == 2) {
    hipLaunchKernelGGL((aug_point_kernel<true, false>), grid, block, 0, stream, a);
    hipLaunchKernelGGL((aug_blur_kernel<true, false>), grid, bblock, lds, stream, a);
  }
  if (a.visible_bf16) {
    hipLaunchKernelGGL((aug_point_kernel<false, true>), grid, block, 0, stream, a);
    hipLaunchKernelGGL((aug_blur_kernel<false, true>), grid, bblock, lds, stream, a);
  } else {
    hipLaunchKernelGGL((aug_point_kernel<false, false>), grid, block, 0, stream, a);
    hipLaunchKernelGGL((aug_blur_kernel<false, false>), grid, bblock, lds, stream, a);
  }
  return hipGetLastError();
}

}  // namespace mae
