// Per-sample parameters of the input pipeline: RandomResizedCrop box (Sec. 5.1), flip bit
// (App. B) and the random masking order (Sec. 2, Sec. 5.3 "Masking Ratio").
//
// One wavefront per sample.  The crop box needs a handful of fp64 operations, evaluated uniformly
// by all lanes.  The masking order is a sort of L <= 256 (noise, index) keys: 1, 2 or 4 keys per
// lane in registers, ordered by a bitonic network whose exchanges at distance < 64 cross lanes
// and at distance >= 64 stay inside a lane.
#include "mae_device.hpp"
#include "mae_kernels.hpp"

// The crop box must agree bit for bit with a plain evaluation that rounds every fp64 operation
// once, so no multiply-add fusion anywhere in this file.
#pragma clang fp contract(off)

namespace mae {

// exp(x) as the degree-13 Taylor polynomial in Horner form; |x| <= 1/2.
__device__ static double exp_poly(double x) {
  double e = 1.0;
#pragma unroll 1
  for (int k = 13; k >= 1; --k) {
    double xe = x * e;
    double q = xe / (double)k;
    e = 1.0 + q;
  }
  return e;
}

// Nearest integer to sqrt(x), ties to even, for 0 <= x < 2^50.  The square root instruction
// sequence is followed by an exact check against (n -+ 1/2)^2, which is representable.
__device__ static int64_t round_sqrt(double x) {
  double n = rint(sqrt(x));
  const bool even = ((int64_t)n & 1) == 0;
  const double hi = (n + 0.5) * (n + 0.5);
  if (x > hi || (x == hi && !even)) {
    n += 1.0;
  } else if (n >= 1.0) {
    const double lo = (n - 0.5) * (n - 0.5);
    if (x < lo || (x == lo && !even)) n -= 1.0;
  }
  return (int64_t)n;
}

template <int R>
__device__ static void bitonic_sort(uint64_t (&v)[R], int lane) {
  constexpr int N = R * kWave;
#pragma unroll
  for (int k = 2; k <= N; k <<= 1) {
#pragma unroll
    for (int j = k >> 1; j > 0; j >>= 1) {
      if (j >= kWave) {
        // partner is another register of the same lane
        const int dr = j / kWave;
#pragma unroll
        for (int r = 0; r < R; ++r) {
          if ((r & dr) == 0) {
            const int i_hi = r * kWave;  // bit pattern of the register index inside i
            const bool ascending = ((i_hi & k) == 0);
            uint64_t a = v[r], b = v[r | dr];
            bool swap = ascending ? (a > b) : (a < b);
            v[r] = swap ? b : a;
            v[r | dr] = swap ? a : b;
          }
        }
      } else {
#pragma unroll
        for (int r = 0; r < R; ++r) {
          const int i = r * kWave + lane;
          const bool ascending = ((i & k) == 0);
          const bool lower = ((lane & j) == 0);
          uint64_t mine = v[r];
          uint32_t olo = __shfl_xor((uint32_t)mine, j, kWave);
          uint32_t ohi = __shfl_xor((uint32_t)(mine >> 32), j, kWave);
          uint64_t other = ((uint64_t)ohi << 32) | olo;
          bool take_min = (lower == ascending);
          bool other_smaller = other < mine;
          v[r] = (take_min == other_smaller) ? other : mine;
        }
      }
    }
  }
}

template <int R>
__global__ __launch_bounds__(kWave) void params_mask_kernel(ParamArgs a) {
  const int b = blockIdx.x;
  const int lane = threadIdx.x;
  const uint32_t sample = a.sample_base + (uint32_t)b;
  CropRec* rec = reinterpret_cast<CropRec*>(a.workspace + kWorkspaceHeader) + b;

  // ---- geometry check (values are uniform over the wavefront) ---------------------------------
  const int32_t H = a.heights[b];
  const int32_t W = a.widths[b];
  const int64_t off = a.offsets[b];
  bool valid = H >= 1 && W >= 1 && H <= 32767 && W <= 32767 && off >= 0;
  if (valid) valid = off + (int64_t)H * W * 3 <= a.images_bytes;

  int32_t top = 0, left = 0, ch = 0, cw = 0, flip = 0;
  if (valid) {
    // ---- RandomResizedCrop: up to ten proposals, then the centred fallback --------------------
    const double area = (double)((int64_t)H * (int64_t)W);
    bool found = false;
#pragma unroll 1
    for (uint32_t t = 0; t < 10 && !found; ++t) {
      double s = a.scale_lo + a.scale_span * unit53(draw(a.key1, sample, kScale, t));
      double T = area * s;
      double x = a.ln_ratio_lo + a.ln_ratio_span * unit53(draw(a.key1, sample, kRatio, t));
      double r = exp_poly(x);
      int64_t w = round_sqrt(T * r);
      int64_t h = round_sqrt(T / r);
      if (w >= 1 && w <= W && h >= 1 && h <= H) {
        uint64_t ut = draw(a.key1, sample, kTop, t) >> 32;
        uint64_t ul = draw(a.key1, sample, kLeft, t) >> 32;
        top = (int32_t)((ut * (uint64_t)(H - h + 1)) >> 32);
        left = (int32_t)((ul * (uint64_t)(W - w + 1)) >> 32);
        ch = (int32_t)h;
        cw = (int32_t)w;
        found = true;
      }
    }
    if (!found) {
      double R0 = (double)W / (double)H;
      int64_t h, w;
      if (R0 < a.ratio_lo) {
        w = W;
        h = (int64_t)rint((double)W / a.ratio_lo);
      } else if (R0 > a.ratio_hi) {
        h = H;
        w = (int64_t)rint((double)H * a.ratio_hi);
      } else {
        h = H;
        w = W;
      }
      h = h > H ? H : (h < 1 ? 1 : h);
      w = w > W ? W : (w < 1 ? 1 : w);
      ch = (int32_t)h;
      cw = (int32_t)w;
      top = (H - ch) / 2;
      left = (W - cw) / 2;
    }
    // ---- flip: 24-bit uniform against the probability, in single precision --------------------
    uint32_t u24 = (uint32_t)(draw(a.key1, sample, kFlip, 0) >> 32) >> 8;
    flip = ((float)u24 * (1.0f / 16777216.0f) < a.flip_p) ? 1 : 0;
  }

  if (lane == 0) {
    CropRec out;
    out.top = top; out.left = left; out.ch = ch; out.cw = cw;
    out.flip = flip; out.valid = valid ? 1 : 0; out.pad0 = 0; out.pad1 = 0;
    *rec = out;
    if (a.crop_out) {
      int32_t* c = a.crop_out + (int64_t)b * 6;
      c[0] = top; c[1] = left; c[2] = ch; c[3] = cw; c[4] = flip; c[5] = valid ? 1 : 0;
    }
    if (b == 0) {  // header: lets the status query find the records of this call
      WorkspaceHeader* hdr = reinterpret_cast<WorkspaceHeader*>(a.workspace);
      hdr->magic = kWorkspaceMagic;
      hdr->B = a.B;
    }
  }
  // the finetuning augmentation's draws and the blur's taps, once per sample instead of once per
  // workgroup later: every lane makes the same draws, lane k computes tap k
  if (a.aug_out) {
    AugParams ap = aug_params(a.key1, sample, a.jitter);
    const float t = ap.op == kOpBlur ? blur_taps(ap, lane) : 0.0f;
#pragma unroll
    for (int k = 0; k < 7; ++k) ap.tap[k] = __shfl(t, k, kWave);
    if (lane == 0) static_cast<AugParams*>(a.aug_out)[b] = ap;
  }
  if (!valid) return;

  // ---- masking order: sort (noise << 32 | patch index) ----------------------------------------
  const int L = a.L, K = a.K;
  uint64_t v[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int l = r * kWave + lane;
    uint64_t key = ~0ull;  // padding sorts last
    if (l < L) {
      uint32_t noise = (uint32_t)(draw(a.key1, sample, kNoise, (uint32_t)l) >> 32);
      noise >>= (32 - a.noise_bits);
      key = ((uint64_t)noise << 32) | (uint32_t)l;
    }
    v[r] = key;
  }
  bitonic_sort<R>(v, lane);

  const int64_t rowL = (int64_t)b * L, rowK = (int64_t)b * K;
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int rank = r * kWave + lane;
    if (rank < L) {
      const int l = (int)(uint32_t)v[r];
      a.ids_restore[rowL + l] = rank;
      a.mask[rowL + l] = rank >= K ? 1 : 0;
      if (rank < K && a.ids_keep) a.ids_keep[rowK + rank] = l;
    }
  }
}

hipError_t launch_params_mask(const ParamArgs& a, hipStream_t stream) {
  const int R = (a.L + kWave - 1) / kWave;
  dim3 grid(a.B), block(kWave);
  if (R <= 1) {
    hipLaunchKernelGGL(params_mask_kernel<1>, grid, block, 0, stream, a);
  } else if (R == 2) {
    hipLaunchKernelGGL(params_mask_kernel<2>, grid, block, 0, stream, a);
  } else {
    hipLaunchKernelGGL(params_mask_kernel<4>, grid, block, 0, stream, a);
  }
  return hipGetLastError();
}

}  // namespace mae
