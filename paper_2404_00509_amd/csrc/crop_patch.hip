// Crop + bilinear resize (Sec. 4.1, Sec. 5.1) + horizontal flip + mean/std normalisation (App. B)
// + ViT patch split (Sec. 3) + gather of the visible patches (Sec. 2), in one pass: every source
// byte is read from HBM once and every output value is written once, straight into patch order.
//
// One workgroup per (image, row of patches).  The source rows that this patch row taps are staged
// in LDS as 4-byte RGBx pixels, together with one table of horizontal taps (S entries) and one of
// vertical taps (p entries).  Then each wavefront produces whole patches: lane i writes the i-th
// 16-byte group of the patch, so that every store instruction covers 1 KiB of contiguous memory.
// A group of four consecutive values spans two neighbouring pixels; one byte-permute per tap row
// pulls exactly the four bytes needed out of the two RGBx words.
#include "mae_device.hpp"
#include "mae_kernels.hpp"

namespace mae {

constexpr int kCropThreads = 256;
constexpr int kCropWaves = kCropThreads / kWave;
constexpr int kTilePixels = 8192;  // 32 KiB of staged source pixels per workgroup
constexpr int kMaxOut = 512;       // S
constexpr int kMaxPatch = 32;      // p

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Source taps of output index o when `len` source pixels are resized to S: sample position
// (o + 1/2) len / S - 1/2 kept as the exact fraction n / (2 S); taps clamped to [0, len).
__device__ static inline void resize_taps(int o, int len, int S, int& i0, int& i1, float& f) {
  const int n = (2 * o + 1) * len - S;
  const int den = 2 * S;
  if (n <= 0) {
    i0 = 0;
    f = 0.0f;
  } else {
    i0 = n / den;
    f = (float)(n - i0 * den) / (float)den;
  }
  i1 = min(i0 + 1, len - 1);
}

__device__ static inline uint32_t load_rgbx(const uint8_t* p) {
  return (uint32_t)p[0] | ((uint32_t)p[1] << 8) | ((uint32_t)p[2] << 16);
}

template <bool kLds>
__device__ static inline uint32_t fetch(const uint32_t* tile, const uint8_t* base, int row_off,
                                        int x) {
  if (kLds) return tile[row_off + x];
  return load_rgbx(base + row_off + 3 * x);
}

template <int J>
__device__ static inline float byte_to_float(uint32_t v) {
  return (float)((v >> (8 * J)) & 0xFFu);
}

// The compute + store phase of one workgroup.  kLds: taps come from the staged tile, otherwise
// straight from global memory (crops too large to stage).
template <bool kLds, bool kBf16>
__device__ static void produce_patches(const CropArgs& a, const uint32_t* tile, const u32x2* xtab,
                                       const u32x2* ytab, const uint8_t* base, int row_stride,
                                       int b, int gy, float inv_p) {
  const int lane = threadIdx.x % kWave;
  const int wave = threadIdx.x / kWave;
  const int p = a.p, D = a.D, G = a.G;
  const int D4 = D >> 2;
  const int pp = p * p;

  for (int k0 = 0; k0 < D4; k0 += kWave) {
    const int e4 = k0 + lane;
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
    const u32x2 ya = ytab[pyA], yb = ytab[pyB];
    const int rowA0 = (int)(ya.x & 0xFFFFu) * row_stride, rowA1 = (int)(ya.x >> 16) * row_stride;
    const int rowB0 = (int)(yb.x & 0xFFFFu) * row_stride, rowB1 = (int)(yb.x >> 16) * row_stride;
    const float fyA = __uint_as_float(ya.y), fyB = __uint_as_float(yb.y);
    // byte selectors: A's bytes are 0..2, B's bytes are 4..6 of the 64-bit pair {B, A}
    const uint32_t sel = cA == 0 ? 0x04020100u : (cA == 1 ? 0x05040201u : 0x06050402u);
    const int nA = 3 - cA;  // how many of the four values come from pixel A
    float sc[4], bi[4], fy[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int c = cA + j;
      c = c >= 3 ? c - 3 : c;
      c = c >= 3 ? c - 3 : c;
      sc[j] = c == 0 ? a.nscale[0] : (c == 1 ? a.nscale[1] : a.nscale[2]);
      bi[j] = c == 0 ? a.nbias[0] : (c == 1 ? a.nbias[1] : a.nbias[2]);
      fy[j] = j < nA ? fyA : fyB;
    }

    for (int gx = wave; gx < G; gx += kCropWaves) {
      const int l = gy * G + gx;
      const int rank = a.ids_restore[(int64_t)b * a.L + l];
      const u32x2 xa = xtab[gx * p + pxA], xb = xtab[gx * p + pxB];
      const int xa0 = (int)(xa.x & 0xFFFFu), xa1 = (int)(xa.x >> 16);
      const int xb0 = (int)(xb.x & 0xFFFFu), xb1 = (int)(xb.x >> 16);
      const float fxA = __uint_as_float(xa.y), fxB = __uint_as_float(xb.y);
      const uint32_t A00 = fetch<kLds>(tile, base, rowA0, xa0);
      const uint32_t A01 = fetch<kLds>(tile, base, rowA0, xa1);
      const uint32_t A10 = fetch<kLds>(tile, base, rowA1, xa0);
      const uint32_t A11 = fetch<kLds>(tile, base, rowA1, xa1);
      const uint32_t B00 = fetch<kLds>(tile, base, rowB0, xb0);
      const uint32_t B01 = fetch<kLds>(tile, base, rowB0, xb1);
      const uint32_t B10 = fetch<kLds>(tile, base, rowB1, xb0);
      const uint32_t B11 = fetch<kLds>(tile, base, rowB1, xb1);
      const uint32_t P00 = __builtin_amdgcn_perm(B00, A00, sel);
      const uint32_t P01 = __builtin_amdgcn_perm(B01, A01, sel);
      const uint32_t P10 = __builtin_amdgcn_perm(B10, A10, sel);
      const uint32_t P11 = __builtin_amdgcn_perm(B11, A11, sel);

      float out[4];
#define MAE_BLEND(J)                                                   \
  {                                                                    \
    const float fx = (J) < nA ? fxA : fxB;                             \
    const float a00 = byte_to_float<J>(P00), a01 = byte_to_float<J>(P01); \
    const float a10 = byte_to_float<J>(P10), a11 = byte_to_float<J>(P11); \
    const float rt = a00 + fx * (a01 - a00);                           \
    const float rb = a10 + fx * (a11 - a10);                           \
    const float v = rt + fy[J] * (rb - rt);                            \
    out[J] = v * sc[J] + bi[J];                                        \
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
}

template <bool kBf16>
__global__ __launch_bounds__(kCropThreads) void crop_patch_kernel(CropArgs a) {
  __shared__ uint32_t tile[kTilePixels];
  __shared__ u32x2 xtab[kMaxOut];
  __shared__ u32x2 ytab[kMaxPatch];

  const uint32_t tile_id = xcd_remap(blockIdx.x, gridDim.x);
  const int b = (int)(tile_id / (uint32_t)a.G);
  const int gy = (int)(tile_id - (uint32_t)b * (uint32_t)a.G);
  const CropRec rec = reinterpret_cast<const CropRec*>(a.workspace + kWorkspaceHeader)[b];
  if (!rec.valid) return;

  const int S = a.S, p = a.p;
  const int W = a.widths[b];
  const int tid = threadIdx.x;

  // rows of the crop that this row of patches taps
  int ylo, yhi, t0, t1;
  float tf;
  resize_taps(gy * p, rec.ch, S, ylo, t1, tf);
  resize_taps(gy * p + p - 1, rec.ch, S, t0, yhi, tf);
  const int nrows = yhi - ylo + 1;
  const bool use_lds = nrows * rec.cw <= kTilePixels;

  const uint8_t* base = a.images + a.offsets[b] + ((int64_t)(rec.top + ylo) * W + rec.left) * 3;

  for (int ox = tid; ox < S; ox += kCropThreads) {
    int x0, x1;
    float f;
    resize_taps(rec.flip ? S - 1 - ox : ox, rec.cw, S, x0, x1, f);
    xtab[ox] = u32x2{(uint32_t)x0 | ((uint32_t)x1 << 16), __float_as_uint(f)};
  }
  if (tid < p) {
    int y0, y1;
    float f;
    resize_taps(gy * p + tid, rec.ch, S, y0, y1, f);
    ytab[tid] = u32x2{(uint32_t)(y0 - ylo) | ((uint32_t)(y1 - ylo) << 16), __float_as_uint(f)};
  }

  if (use_lds) {
    const int lane = tid % kWave, wave = tid / kWave;
    for (int yy = wave; yy < nrows; yy += kCropWaves) {
      const uint8_t* src = base + (int64_t)yy * W * 3;
      for (int xx = lane; xx < rec.cw; xx += kWave) tile[yy * rec.cw + xx] = load_rgbx(src + 3 * xx);
    }
  }
  __syncthreads();

  const float inv_p = 1.0f / (float)p;
  if (use_lds) {
    produce_patches<true, kBf16>(a, tile, xtab, ytab, base, rec.cw, b, gy, inv_p);
  } else {
    produce_patches<false, kBf16>(a, tile, xtab, ytab, base, 3 * W, b, gy, inv_p);
  }
}

// Patch sizes whose 3 p^2 values per patch are not a multiple of four (odd p): one value per
// thread, taps straight from global memory.  Correct for every shape, not tuned.
template <bool kBf16>
__global__ __launch_bounds__(kCropThreads) void crop_patch_scalar_kernel(CropArgs a) {
  const int64_t per_image = (int64_t)a.L * a.D;
  const int64_t total = (int64_t)a.B * per_image;
  for (int64_t idx = (int64_t)blockIdx.x * kCropThreads + threadIdx.x; idx < total;
       idx += (int64_t)gridDim.x * kCropThreads) {
    const int b = (int)(idx / per_image);
    const int rem = (int)(idx - (int64_t)b * per_image);
    const CropRec rec = reinterpret_cast<const CropRec*>(a.workspace + kWorkspaceHeader)[b];
    if (!rec.valid) continue;
    const int l = rem / a.D, e = rem - l * a.D;
    const int gy = l / a.G, gx = l - gy * a.G;
    const int q = e / 3, c = e - 3 * q;
    const int py = q / a.p, px = q - py * a.p;
    const int oy = gy * a.p + py, ox = gx * a.p + px;
    int x0, x1, y0, y1;
    float fx, fy;
    resize_taps(rec.flip ? a.S - 1 - ox : ox, rec.cw, a.S, x0, x1, fx);
    resize_taps(oy, rec.ch, a.S, y0, y1, fy);
    const int W = a.widths[b];
    const uint8_t* img = a.images + a.offsets[b];
    const float a00 = img[((int64_t)(rec.top + y0) * W + rec.left + x0) * 3 + c];
    const float a01 = img[((int64_t)(rec.top + y0) * W + rec.left + x1) * 3 + c];
    const float a10 = img[((int64_t)(rec.top + y1) * W + rec.left + x0) * 3 + c];
    const float a11 = img[((int64_t)(rec.top + y1) * W + rec.left + x1) * 3 + c];
    const float rt = a00 + fx * (a01 - a00);
    const float rb = a10 + fx * (a11 - a10);
    const float v = (rt + fy * (rb - rt)) * a.nscale[c] + a.nbias[c];
    if (a.target) a.target[idx] = v;
    const int rank = a.ids_restore[(int64_t)b * a.L + l];
    if (rank < a.K) {
      const int64_t vo = ((int64_t)b * a.K + rank) * a.D + e;
      if (kBf16) {
        static_cast<uint16_t*>(a.visible)[vo] = (uint16_t)bf16_rne(v);
      } else {
        static_cast<float*>(a.visible)[vo] = v;
      }
    }
  }
}

hipError_t launch_crop_patch(const CropArgs& a, hipStream_t stream) {
  if ((a.D & 3) == 0) {
    dim3 grid((uint32_t)a.B * (uint32_t)a.G), block(kCropThreads);
    if (a.visible_bf16) {
      hipLaunchKernelGGL(crop_patch_kernel<true>, grid, block, 0, stream, a);
    } else {
      hipLaunchKernelGGL(crop_patch_kernel<false>, grid, block, 0, stream, a);
    }
  } else {
    const int64_t total = (int64_t)a.B * a.L * a.D;
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
