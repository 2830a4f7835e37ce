// Colour jitter of the finetuning augmentation "3 Aug+" (Sec. 5.2, Table 7), per pixel in single
// precision, shared by the resampling kernel's augmentation epilogue and the blur kernel.
#pragma once

#include "mae_device.hpp"

namespace mae {

__device__ static inline float clamp255(float v) { return fminf(fmaxf(v, 0.0f), 255.0f); }
__device__ static inline float luma(float r, float g, float b) {
  return 0.299f * r + 0.587f * g + 0.114f * b;
}

// Brightness (v * b), contrast (blend with the image's mean luma after the brightness step) and
// saturation (blend with the pixel's luma), each followed by a clamp to [0, 255].
// kReduce: only the brightness step; returns the pixel's luma (what the mean is taken of).
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

}  // namespace mae
