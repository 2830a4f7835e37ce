// Gaussian blur of the finetuning augmentation "3 Aug" / "3 Aug+" (Sec. 3 finetuning recipe,
// Sec. 4.4 "Data Augmentation", Sec. 5.2 Table 7).  Per image one of grayscale / solarisation /
// Gaussian blur is drawn; the first two are pointwise and run as the epilogue of the resampling
// kernel, which leaves the rounded 8-bit resized crop of the blur images in patch order
// ([B, L, D] bytes, the layout of `target`).  This kernel blurs them, applies the colour jitter
// of "3 Aug+", normalises and writes `target` / `visible`.
//
// aug_blur_kernel: one workgroup per image, row of patches and column part of whole patches; it
// leaves at once when its image drew another operation.
//  * Staging.  The bytes of the part's rows and of R more rows above and below, over the part's
//    patches and the neighbouring patch on either side, are copied into LDS in image order (all
//    loads of a thread issued before the first is stored).  Rows beyond the image repeat its
//    border row.
//  * Vertical pass.  A thread takes one value column and a run of rows: it converts the bytes it
//    needs once and applies the 2 R + 1 taps to each row of its run; columns beyond the image
//    repeat the border column.  The result (fp32) goes to a second LDS array with R pixels more
//    on either side of the part.
//  * Horizontal pass, folded into the walk over the part in output order: a lane reads the
//    4 + 2 R pixels around its four with aligned 16-byte LDS reads and applies the taps.
// R is the smallest of 2, 4, 6 that holds the image's radius ceil(3 sigma), so that an image with
// a small sigma does not pay for 13 taps.  The taps themselves come with the image's draws from
// the parameter kernel (one record per image) and sit in scalar registers.
// The contrast step needs the mean luma of the whole image after the brightness step: with jitter
// on, a first launch of the same kernel (kReduce) only accumulates that sum per part in double
// precision, and the second launch adds the partial sums of its image in fixed order.
#include "aug_device.hpp"
#include "mae_device.hpp"
#include "mae_kernels.hpp"

namespace mae {

constexpr int kAugThreads = 256;
constexpr int kMaxRadius = 6;  // ceil(3 * 2.0)

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x3 __attribute__((ext_vector_type(3)));
typedef u32x3 u32x3_a4 __attribute__((aligned(4)));

// A lane's kPx neighbouring pixels are 3 kPx floats = three pieces of kPx floats.
template <int kPx>
struct BlurPiece;
template <>
struct BlurPiece<4> {
  typedef f32x4 type;
};
template <>
struct BlurPiece<2> {
  typedef f32x2 type;
};

// floor(n / d) for 0 <= n < 2^22 and small d, from the float reciprocal (inv = 1 / d)
__device__ static inline int fast_div(int n, float inv) { return (int)(((float)n + 0.5f) * inv); }

// Mean luma after the brightness step, from the partial sums of the reduction launch.
__device__ static inline float image_mean(const AugArgs& a, int b) {
  // one slot per (row of patches, column part of the blur kernel); unused slots hold zero
  const int slots = a.G * a.blur_parts;
  double sum = 0.0;
  for (int g = 0; g < slots; ++g) sum += a.partials[(int64_t)b * slots + g];
  return (float)(sum / ((double)a.S * (double)a.S));
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

// ---- Gaussian blur ---------------------------------------------------------------------------------
// Patches staged on either side of the part: enough for the largest radius.
__host__ __device__ static inline int halo_patches(int p) { return (kMaxRadius + p - 1) / p; }

// Copies `rows` image rows (first y_first, clamped into the image) of patches gxa .. gxa + nseg - 1
// from the patch-order bytes `img` into `dst` in image order, in pieces of type T (wseg pieces per
// patch row).  A wavefront takes whole rows, a lane one piece of the row, so that everything that
// depends on the row is the same for all lanes and a piece costs one address addition; a lane
// issues four loads (four rows) before it stores the first.
template <typename T>
__device__ static inline void stage_rows(uint8_t* dst, const uint8_t* img, int rows, int nseg,
                                         int wseg, int y_first, int S, int p, int G, int gxa,
                                         int D) {
  T* out = reinterpret_cast<T*>(dst);
  const int lane = threadIdx.x % kWave;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int pitch = nseg * wseg;
  const float inv_wseg = 1.0f / (float)wseg, inv_p = 1.0f / (float)p;
  constexpr int kBatch = 4, kWaves = kAugThreads / kWave;
  for (int l0 = 0; l0 < pitch; l0 += kWave) {
    const bool have = l0 + lane < pitch;
    const int l = have ? l0 + lane : pitch - 1;
    const int seg = fast_div(l, inv_wseg);
    const uint32_t piece = (uint32_t)(__mul24(gxa + seg, D) + (int)sizeof(T) * (l - seg * wseg));
    for (int j0 = wave; j0 < rows; j0 += kBatch * kWaves) {
      T v[kBatch];
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const int j = min(j0 + u * kWaves, rows - 1);
        const int yy = min(max(y_first + j, 0), S - 1);
        const int gyy = fast_div(yy, inv_p);
        const uint32_t row = (uint32_t)(__mul24(__mul24(gyy, G), D) + (yy - gyy * p) * 3 * p);
        v[u] = *reinterpret_cast<const T*>(img + (row + piece));
      }
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const int j = j0 + u * kWaves;
        if (j < rows && have) out[j * pitch + l] = v[u];
      }
    }
  }
}

// Vertical pass: kRows output rows of one value column per item.
template <int R, int kRows>
__device__ static inline void blur_vertical(const uint8_t* sbytes, float* vbuf, const float* wt,
                                            int p, int S, int x_lo, int xs0, int Wp, int pitchb,
                                            int vpitch) {
  const int ncols = (Wp + 2 * R) * 3;
  const int chunks = p / kRows;
  for (int it = threadIdx.x; it < ncols * chunks; it += kAugThreads) {
    const int yc = fast_div(it, 1.0f / (float)ncols);
    const int vx = it - yc * ncols;
    const int px = fast_div(vx, 1.0f / 3.0f);
    const int c = vx - 3 * px;
    const int xa = min(max(x_lo - R + px, 0), S - 1);  // border column repeated
    // (32-bit offsets, stepped row by row: no multiplication per row)
    uint32_t at = (uint32_t)(__mul24(yc * kRows, pitchb) + (xa - xs0) * 3 + c);
    float in[kRows + 2 * R];
#pragma unroll
    for (int j = 0; j < kRows + 2 * R; ++j) {
      in[j] = (float)sbytes[at];
      at += (uint32_t)pitchb;
    }
#pragma unroll
    for (int y = 0; y < kRows; ++y) {
      float acc = 0.f;
#pragma unroll
      for (int k = 0; k <= 2 * R; ++k) acc += wt[k] * in[y + k];
      vbuf[(yc * kRows + y) * vpitch + vx] = acc;
    }
  }
}

// kPx: pixels per lane in the horizontal pass, 4 when p is a multiple of 4, else 2 (p even).
template <int R, bool kReduce, bool kBf16, int kPx>
__device__ static void blur_part(const AugArgs& a, const AugParams& ap, int b, int gy, int part,
                                 int gx0, int npatch, float* vbuf, uint8_t* scratch,
                                 double* red) {
  typedef typename BlurPiece<kPx>::type piece_t;
  constexpr int kVals = 3 * kPx;
  const int S = a.S, p = a.p, G = a.G;
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int Wp = npatch * p, x_lo = gx0 * p, y0 = gy * p;
  const int hp = halo_patches(p);
  const int gxa = max(gx0 - hp, 0), gxb = min(gx0 + npatch - 1 + hp, G - 1);
  const int nseg = gxb - gxa + 1, xs0 = gxa * p;
  const int pitchb = nseg * 3 * p;  // bytes per staged row
  const int rows = p + 2 * R;
  const float inv_p = 1.0f / (float)p;
  const uint8_t* img = a.u8 + (int64_t)b * a.L * a.D;  // patch order

  // ---- staging: rows y0 - R .. y0 + p - 1 + R (clamped), patches gxa .. gxb ----------------------
  // in pieces of 16 bytes when a patch row is a multiple of that (p = 16, 32), else of 4 bytes,
  // else (p even, no multiple of 4) of 2 bytes
  if constexpr (kPx == 4) {
    if ((p & 15) == 0)
      stage_rows<u32x4>(scratch, img, rows, nseg, (3 * p) >> 4, y0 - R, S, p, G, gxa, a.D);
    else
      stage_rows<uint32_t>(scratch, img, rows, nseg, (3 * p) >> 2, y0 - R, S, p, G, gxa, a.D);
  } else {
    stage_rows<uint16_t>(scratch, img, rows, nseg, (3 * p) >> 1, y0 - R, S, p, G, gxa, a.D);
  }
  // taps -R .. R of this image's kernel as the parameter kernel left them (zero beyond the
  // image's radius); the record is the same for the whole workgroup
  float wt[2 * R + 1];
#pragma unroll
  for (int k = 0; k <= 2 * R; ++k) wt[k] = ap.tap[k < R ? R - k : k - R];
  __syncthreads();

  const int vpitch = (Wp + 2 * R) * 3;  // a multiple of kPx floats
  if constexpr (kPx == 4) {
    if ((p & 7) == 0)
      blur_vertical<R, 8>(scratch, vbuf, wt, p, S, x_lo, xs0, Wp, pitchb, vpitch);
    else
      blur_vertical<R, 4>(scratch, vbuf, wt, p, S, x_lo, xs0, Wp, pitchb, vpitch);
  } else {
    blur_vertical<R, 2>(scratch, vbuf, wt, p, S, x_lo, xs0, Wp, pitchb, vpitch);
  }
  // noise rank of each patch of the part, one per lane (read back with a shuffle at the stores)
  const int l0 = gy * G + gx0;
  const int my_rank = lane < npatch ? a.ids_restore[(int64_t)b * a.L + l0 + lane] : 0x7fffffff;
  __syncthreads();  // the staged bytes are dead from here on: their space serves as the strips

  const float mean = (!kReduce && a.mode == 2) ? image_mean(a, b) : 0.0f;
  const int gpp = (p * p) / kPx;
  const float inv_gpp = 1.0f / (float)gpp;
  const int ngroups = npatch * gpp;
  float* strip = reinterpret_cast<float*>(scratch) + wave * (kWave * kVals);
  float* target_image = a.target ? a.target + (int64_t)b * a.L * a.D : nullptr;
  void* visible_image =
      kBf16 ? static_cast<void*>(static_cast<uint16_t*>(a.visible) + (int64_t)b * a.K * a.D)
            : static_cast<void*>(static_cast<float*>(a.visible) + (int64_t)b * a.K * a.D);
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
  float lsum = 0.0f;
  // patches of 16 x 16 or 32 x 32 pixels: the 64 groups of a wavefront's step lie in one patch
  const bool whole = kPx == 4 && (p & 15) == 0;
  const int gsh = __builtin_ctz(gpp), psh = __builtin_ctz(p);  // used when `whole`
  for (int i0 = wave * kWave; i0 < ngroups; i0 += kAugThreads) {
    bool have;
    int gxl, q, py;
    if (whole) {
      have = true;
      gxl = i0 >> gsh;  // uniform
      q = 4 * ((i0 & (gpp - 1)) + lane);
      py = q >> psh;
    } else {
      have = i0 + lane < ngroups;
      const int i = have ? i0 + lane : ngroups - 1;
      gxl = fast_div(i, inv_gpp);
      q = kPx * (i - gxl * gpp);
      py = fast_div(q, inv_p);
    }
    const int x = gxl * p + (q - py * p);  // pixel inside the part
    // pixels x - R .. x + kPx - 1 + R of the row: (kPx + 2 R) * 3 floats, aligned to a piece
    constexpr int kIn = (kPx + 2 * R) * 3;
    const piece_t* src = reinterpret_cast<const piece_t*>(vbuf + py * vpitch + 3 * x);
    float n[kIn];
#pragma unroll
    for (int j = 0; j < kIn / kPx; ++j) {
      const piece_t t = src[j];
#pragma unroll
      for (int e = 0; e < kPx; ++e) n[kPx * j + e] = t[e];
    }
    float v[kVals];
#pragma unroll
    for (int h = 0; h < kPx; ++h) {
      float r = 0.f, g = 0.f, bl = 0.f;
#pragma unroll
      for (int k = 0; k <= 2 * R; ++k) {
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
    if (kReduce) continue;

    // normalise, then through the wavefront's strip: every store instruction writes 1 KiB (512
    // bytes with two pixels per lane) of contiguous memory; piece k of the strip belongs to
    // group k / 3
    piece_t o[3];
#pragma unroll
    for (int k = 0; k < 3; ++k)
#pragma unroll
      for (int e = 0; e < kPx; ++e) {
        const int idx = kPx * k + e;
        o[k][e] = v[idx] * a.nscale[idx % 3] + a.nbias[idx % 3];
      }
    piece_t* mine = reinterpret_cast<piece_t*>(strip + kVals * lane);
    __builtin_amdgcn_wave_barrier();
    mine[0] = o[0];
    mine[1] = o[1];
    mine[2] = o[2];
    __builtin_amdgcn_wave_barrier();
    if (whole) {
      // one patch, 768 consecutive floats of its row from element 12 (i0 mod gpp) on
      const int gxs = __builtin_amdgcn_readfirstlane(gxl);
      const int rank = __builtin_amdgcn_readlane(my_rank, gxs);
      const uint32_t e0 = 12u * (uint32_t)(i0 & (gpp - 1)) + 4u * (uint32_t)lane;
#pragma unroll
      for (int k = 0; k < 3; ++k) {
        const piece_t t = reinterpret_cast<const piece_t*>(strip)[k * kWave + lane];
        const uint32_t eo = e0 + 4u * kWave * k;
        store_piece((uint32_t)((l0 + gxs) * a.D) + eo, rank, (uint32_t)(rank * a.D) + eo, t);
      }
      continue;
    }
#pragma unroll
    for (int k = 0; k < 3; ++k) {
      const int piece = k * kWave + lane;
      const int g = i0 + fast_div(piece, 1.0f / 3.0f);
      const piece_t t = reinterpret_cast<const piece_t*>(strip)[piece];
      const int pgx = fast_div(min(g, ngroups - 1), inv_gpp);
      const int rank = __shfl(my_rank, pgx, kWave);
      if (g >= ngroups) continue;
      const int eo = kVals * (g - __mul24(pgx, gpp)) + kPx * (piece - 3 * (g - i0));
      store_piece((uint32_t)(__mul24(l0 + pgx, a.D) + eo), rank,
                  (uint32_t)(__mul24(rank, a.D) + eo), t);
    }
  }
  if (kReduce) store_band_sum<kAugThreads>(a, b, gy * a.blur_parts + part, lsum, red);
}

// Dynamic LDS: [ vbuf: p rows of 3 (W + 12) floats, W = widest part in pixels | scratch: the
// staged bytes ((p + 12) rows of the part's patches and their neighbours), later the four
// wavefronts' strips ].
template <bool kReduce, bool kBf16, int kPx>
__global__ __launch_bounds__(kAugThreads) void aug_blur_kernel(AugArgs a) {
  extern __shared__ __attribute__((aligned(16))) float vals[];
  __shared__ double red[kAugThreads / kWave];

  const int p = a.p, G = a.G, parts = a.blur_parts;
  const uint32_t tile = xcd_remap(blockIdx.x, gridDim.x);
  const uint32_t band_id = tile / (uint32_t)parts;
  const int part = (int)(tile - band_id * (uint32_t)parts);
  const int b = (int)(band_id / (uint32_t)G);
  const int gy = (int)(band_id - (uint32_t)b * (uint32_t)G);
  const int gx0 = part * G / parts, gx1 = (part + 1) * G / parts;
  const int npatch = gx1 - gx0;
  const bool valid = reinterpret_cast<const CropRec*>(a.workspace + kWorkspaceHeader)[b].valid != 0;
  if (!valid || npatch <= 0) return;
  const AugParams ap = static_cast<const AugParams*>(a.aug_recs)[b];
  if (ap.op != kOpBlur) return;

  const int radius = ap.radius;
  float* vbuf = vals;
  uint8_t* scratch = reinterpret_cast<uint8_t*>(
      vals + p * 3 * (a.blur_part_patches * p + 2 * kMaxRadius));
  if (radius <= 2)
    blur_part<2, kReduce, kBf16, kPx>(a, ap, b, gy, part, gx0, npatch, vbuf, scratch, red);
  else if (radius <= 4)
    blur_part<4, kReduce, kBf16, kPx>(a, ap, b, gy, part, gx0, npatch, vbuf, scratch, red);
  else
    blur_part<6, kReduce, kBf16, kPx>(a, ap, b, gy, part, gx0, npatch, vbuf, scratch, red);
}

// Bytes of dynamic LDS of the blur kernel for parts of n patches: the vertically blurred rows,
// then the staged bytes (or the four wavefronts' strips, whichever is larger).
static size_t blur_lds_bytes(int p, int n) {
  const size_t vbuf = (size_t)p * 3 * (n * p + 2 * kMaxRadius) * 4;
  const size_t staged = (size_t)(p + 2 * kMaxRadius) * (n + 2 * halo_patches(p)) * 3 * p;
  const size_t strips = (size_t)kAugThreads * 12 * 4;
  return vbuf + (staged > strips ? staged : strips);
}

// Column parts of the blur kernel: the fewest (whole patches each) whose LDS stays within 40 KiB,
// so that four workgroups share a compute unit.
AugPlan three_aug_plan(int S, int p) {
  const int G = S / p;
  AugPlan plan;
  for (int parts = 1;; ++parts) {
    const int n = (G + parts - 1) / parts;
    const size_t lds = blur_lds_bytes(p, n);
    if (lds <= 40 * 1024 || parts >= G) {
      plan.parts = parts;
      plan.part_patches = n;
      plan.lds_bytes = lds;
      return plan;
    }
  }
}

// The blur images of a batch.  reduce: only the luma sums after the brightness step ("3 Aug+").
hipError_t launch_aug_blur(const AugArgs& a, bool reduce, hipStream_t stream) {
  dim3 block(kAugThreads);
  dim3 bgrid((uint32_t)a.B * (uint32_t)a.G * (uint32_t)a.blur_parts);
  const size_t lds = blur_lds_bytes(a.p, a.blur_part_patches);
  // four pixels per lane when they tile a patch row, else two (even patch sizes)
#define MAE_BLUR_LAUNCH(RED, BF)                                                           \
  do {                                                                                     \
    if ((a.p & 3) == 0)                                                                    \
      hipLaunchKernelGGL((aug_blur_kernel<RED, BF, 4>), bgrid, block, lds, stream, a);     \
    else                                                                                   \
      hipLaunchKernelGGL((aug_blur_kernel<RED, BF, 2>), bgrid, block, lds, stream, a);     \
  } while (0)
  if (reduce) MAE_BLUR_LAUNCH(true, false);
  else if (a.visible_bf16) MAE_BLUR_LAUNCH(false, true);
  else MAE_BLUR_LAUNCH(false, false);
#undef MAE_BLUR_LAUNCH
  return hipGetLastError();
}

}  // namespace mae
