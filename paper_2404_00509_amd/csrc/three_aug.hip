// Finetuning augmentation "3 Aug" / "3 Aug+" (Sec. 3 finetuning recipe, Sec. 4.4 "Data
// Augmentation", Sec. 5.2 Table 7): per image one of grayscale / solarisation / Gaussian blur,
// optionally colour jitter (brightness, contrast, saturation), then mean/std normalisation, the
// ViT patch split and the gather of the kept patches.  Input is the 8-bit resized crop that the
// resampling kernel wrote (row-major HWC); output is the same `target` / `visible` layout as the
// pretraining path.
//
// One workgroup per (image, row of patches).  The p image rows of the band are first turned into
// fp32 values after the per-image operation, in LDS:
//   grayscale / solarise  pointwise on the bytes (integer arithmetic, exact);
//   blur                  the band plus `radius` rows above and below (clamped at the image
//                         border) is staged as bytes, the vertical pass writes fp32 rows, and the
//                         horizontal pass is folded into the consumer below.
// The consumer walks the band in OUTPUT order, two pixels per lane, so that `target` is written as
// one contiguous run of G * D floats per workgroup; jitter and normalisation are applied on the
// way.  The contrast step needs the mean luma of the whole image after the brightness step:
// with jitter on, a first launch of the same code (kReduce) only accumulates that sum per band in
// double precision, and the second launch adds the G partial sums of its image in fixed order.
#include "mae_device.hpp"
#include "mae_kernels.hpp"

namespace mae {

constexpr int kAugThreads = 256;
constexpr int kMaxRadius = 6;  // ceil(3 * 2.0)

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ static inline float clamp255(float v) { return fminf(fmaxf(v, 0.0f), 255.0f); }
__device__ static inline float luma(float r, float g, float b) {
  return 0.299f * r + 0.587f * g + 0.114f * b;
}

// Dynamic LDS: [ vals: p x 3S floats | staged bytes: (p + 2 kMaxRadius) x 3S ].
template <bool kReduce, bool kBf16>
__global__ __launch_bounds__(kAugThreads) void three_aug_kernel(AugArgs a) {
  extern __shared__ __attribute__((aligned(16))) uint32_t lds[];
  __shared__ double wd[2 * kMaxRadius + 1];
  __shared__ float wf[2 * kMaxRadius + 1];
  __shared__ double red[kAugThreads / kWave];

  const int S = a.S, p = a.p, G = a.G;
  const int rv = 3 * S;    // values (= bytes) per image row; a multiple of 4 because 3 p is
  const int rv4 = rv >> 2;
  float* vals = reinterpret_cast<float*>(lds);
  uint32_t* staged = lds + p * rv;

  const uint32_t tile = xcd_remap(blockIdx.x, gridDim.x);
  const int b = (int)(tile / (uint32_t)G);
  const int gy = (int)(tile - (uint32_t)b * (uint32_t)G);
  const int tid = threadIdx.x;
  const CropRec rec = reinterpret_cast<const CropRec*>(a.workspace + kWorkspaceHeader)[b];
  if (!rec.valid) {
    if (kReduce && tid == 0) a.partials[(int64_t)b * G + gy] = 0.0;
    return;
  }
  const AugParams ap = aug_params(a.key1, a.sample_base + (uint32_t)b, a.jitter);
  const uint8_t* img = a.u8 + (int64_t)b * S * rv;
  const int y0 = gy * p;
  const int radius = ap.radius;

  if (ap.op == kOpBlur) {
    // taps exp(-k^2 / (2 sigma^2)) in double precision, summed in index order, scaled to sum 1
    if (tid <= 2 * radius) {
      const double k = (double)(tid - radius);
      wd[tid] = exp(-(k * k) / (2.0 * ap.sigma * ap.sigma));
    }
    __syncthreads();
    if (tid <= 2 * radius) {
      double sum = 0.0;
      for (int k = 0; k <= 2 * radius; ++k) sum += wd[k];
      wf[tid] = (float)(wd[tid] / sum);
    }
    // the band and its halo, border rows repeated
    const int nrows = p + 2 * radius;
    for (int i = tid; i < nrows * rv4; i += kAugThreads) {
      const int j = i / rv4, d = i - j * rv4;
      const int yy = min(max(y0 - radius + j, 0), S - 1);
      staged[i] = reinterpret_cast<const uint32_t*>(img + (int64_t)yy * rv)[d];
    }
    __syncthreads();
    // vertical pass: four neighbouring values (bytes of one word) per step
    for (int i = tid; i < p * rv4; i += kAugThreads) {
      const int y = i / rv4, d = i - y * rv4;
      float acc0 = 0.f, acc1 = 0.f, acc2 = 0.f, acc3 = 0.f;
      for (int k = 0; k <= 2 * radius; ++k) {
        const uint32_t w4 = staged[(y + k) * rv4 + d];
        const float w = wf[k];
        acc0 += w * (float)(w4 & 0xFFu);
        acc1 += w * (float)((w4 >> 8) & 0xFFu);
        acc2 += w * (float)((w4 >> 16) & 0xFFu);
        acc3 += w * (float)(w4 >> 24);
      }
      reinterpret_cast<f32x4*>(vals)[i] = f32x4{acc0, acc1, acc2, acc3};
    }
  } else {
    for (int i = tid; i < p * S; i += kAugThreads) {
      const int y = i / S, x = i - y * S;
      const uint8_t* px = img + (int64_t)(y0 + y) * rv + 3 * x;
      const int r = px[0], g = px[1], bl = px[2];
      float* dst = vals + y * rv + 3 * x;
      if (ap.op == kOpGray) {
        const float l = (float)((299 * r + 587 * g + 114 * bl + 500) / 1000);
        dst[0] = dst[1] = dst[2] = l;
      } else {
        dst[0] = (float)(r >= 128 ? 255 - r : r);
        dst[1] = (float)(g >= 128 ? 255 - g : g);
        dst[2] = (float)(bl >= 128 ? 255 - bl : bl);
      }
    }
  }
  __syncthreads();

  // mean luma after the brightness step, from the partial sums of the first launch
  float mean = 0.0f;
  if (!kReduce && a.mode == 2) {
    double sum = 0.0;
    for (int g = 0; g < G; ++g) sum += a.partials[(int64_t)b * G + g];
    mean = (float)(sum / ((double)S * (double)S));
  }

  const bool blur = ap.op == kOpBlur;
  const int pairs_per_patch = (p * p) >> 1;
  float lsum = 0.0f;
  for (int i = tid; i < G * pairs_per_patch; i += kAugThreads) {
    const int gx = i / pairs_per_patch;
    const int q = 2 * (i - gx * pairs_per_patch);  // first pixel of the pair inside the patch
    const int py = q / p, x = gx * p + (q - py * p);
    const float* row = vals + py * rv;
    float v[6];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      if (blur) {
        float r = 0.f, g = 0.f, bl = 0.f;
        for (int k = 0; k <= 2 * radius; ++k) {
          const float* t = row + 3 * min(max(x + h + k - radius, 0), S - 1);
          const float w = wf[k];
          r += w * t[0];
          g += w * t[1];
          bl += w * t[2];
        }
        v[3 * h] = r;
        v[3 * h + 1] = g;
        v[3 * h + 2] = bl;
      } else {
        const float* t = row + 3 * (x + h);
        v[3 * h] = t[0];
        v[3 * h + 1] = t[1];
        v[3 * h + 2] = t[2];
      }
      if (a.mode == 2) {
        float r = clamp255(v[3 * h] * ap.brightness);
        float g = clamp255(v[3 * h + 1] * ap.brightness);
        float bl = clamp255(v[3 * h + 2] * ap.brightness);
        if (kReduce) {
          lsum += luma(r, g, bl);
        } else {
          const float cm = (1.0f - ap.contrast) * mean;
          r = clamp255(ap.contrast * r + cm);
          g = clamp255(ap.contrast * g + cm);
          bl = clamp255(ap.contrast * bl + cm);
          const float sl = (1.0f - ap.saturation) * luma(r, g, bl);
          v[3 * h] = clamp255(ap.saturation * r + sl);
          v[3 * h + 1] = clamp255(ap.saturation * g + sl);
          v[3 * h + 2] = clamp255(ap.saturation * bl + sl);
        }
      }
    }
    if (kReduce) continue;

    float out[6];
#pragma unroll
    for (int j = 0; j < 6; ++j) {
      const int c = j % 3;
      out[j] = v[j] * a.nscale[c] + a.nbias[c];
    }
    const int l = gy * G + gx;
    const int64_t eo = (int64_t)3 * q;  // element offset inside the patch; 6 values, 8-byte aligned
    if (a.target) {
      f32x2* dst = reinterpret_cast<f32x2*>(a.target + ((int64_t)b * a.L + l) * a.D + eo);
      dst[0] = f32x2{out[0], out[1]};
      dst[1] = f32x2{out[2], out[3]};
      dst[2] = f32x2{out[4], out[5]};
    }
    const int rank = a.ids_restore[(int64_t)b * a.L + l];
    if (rank < a.K) {
      const int64_t vo = ((int64_t)b * a.K + rank) * a.D + eo;
      if (kBf16) {
        uint32_t* dst = reinterpret_cast<uint32_t*>(static_cast<uint16_t*>(a.visible) + vo);
        dst[0] = pack_bf16x2(out[0], out[1]);
        dst[1] = pack_bf16x2(out[2], out[3]);
        dst[2] = pack_bf16x2(out[4], out[5]);
      } else {
        f32x2* dst = reinterpret_cast<f32x2*>(static_cast<float*>(a.visible) + vo);
        dst[0] = f32x2{out[0], out[1]};
        dst[1] = f32x2{out[2], out[3]};
        dst[2] = f32x2{out[4], out[5]};
      }
    }
  }

  if (kReduce) {
    // fixed order: lanes by butterfly, then the wavefronts in index order
    double s = (double)lsum;
    for (int off = kWave / 2; off > 0; off >>= 1) s += __shfl_xor(s, off);
    if ((tid % kWave) == 0) red[tid / kWave] = s;
    __syncthreads();
    if (tid == 0) {
      double t = 0.0;
      for (int w = 0; w < kAugThreads / kWave; ++w) t += red[w];
      a.partials[(int64_t)b * G + gy] = t;
    }
  }
}

size_t three_aug_lds_bytes(int S, int p) {
  return (size_t)p * 3 * S * 4 + (size_t)(p + 2 * kMaxRadius) * 3 * S;
}

hipError_t launch_three_aug(const AugArgs& a, hipStream_t stream) {
  dim3 grid((uint32_t)a.B * (uint32_t)a.G), block(kAugThreads);
  const size_t lds = three_aug_lds_bytes(a.S, a.p);
  if (a.mode == 2) {
    hipLaunchKernelGGL((three_aug_kernel<true, false>), grid, block, lds, stream, a);
  }
  if (a.visible_bf16) {
    hipLaunchKernelGGL((three_aug_kernel<false, true>), grid, block, lds, stream, a);
  } else {
    hipLaunchKernelGGL((three_aug_kernel<false, false>), grid, block, lds, stream, a);
  }
  return hipGetLastError();
}

}  // namespace mae
