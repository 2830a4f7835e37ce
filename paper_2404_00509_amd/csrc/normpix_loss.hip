// Normalised-pixel reconstruction loss and its gradient (the official MAE objective that Sec. 3
// of the paper adopts): per patch row, target statistics -> normalised target -> squared error
// against the prediction on masked rows.
//
// Streaming kernel: one wavefront per pair of adjacent patch rows, the rows held in registers (16-byte loads, lane i
// takes the i-th, (i+64)-th, ... group), two butterfly reductions for mean and variance, gradient
// written with 16-byte stores.  Nothing is read twice, so loads and stores carry the
// non-temporal hint.  Rows are dealt to the wavefronts of the grid round-robin, which keeps the
// rows in flight at any moment inside one small window of each tensor.  Visible rows only get
// zeros written and read nothing.  Each wavefront adds its rows' squared errors in double
// precision and leaves one partial; a second, single-workgroup kernel adds the partials in a
// fixed order, so the loss is reproducible.
#include "mae_device.hpp"
#include "mae_kernels.hpp"

namespace mae {

constexpr int kLossThreads = 256;
constexpr int kLossWaves = kLossThreads / kWave;
constexpr int kComputeUnits = 256;

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ static inline float wave_sum(float v) {
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}

__device__ static inline double wave_sum(double v) {
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}

template <bool kBf16>
__device__ static inline f32x4 load_pred4(const void* pred, int64_t elem) {
  if (kBf16) {
    const u32x2 raw = __builtin_nontemporal_load(
        reinterpret_cast<const u32x2*>(static_cast<const uint16_t*>(pred) + elem));
    return f32x4{bf16_lo(raw.x), bf16_hi(raw.x), bf16_lo(raw.y), bf16_hi(raw.y)};
  }
  return __builtin_nontemporal_load(
      reinterpret_cast<const f32x4*>(static_cast<const float*>(pred) + elem));
}

template <bool kBf16>
__device__ static inline void store_grad4(void* grad, int64_t elem, f32x4 g) {
  if (kBf16) {
    __builtin_nontemporal_store(u32x2{pack_bf16x2(g.x, g.y), pack_bf16x2(g.z, g.w)},
                                reinterpret_cast<u32x2*>(static_cast<uint16_t*>(grad) + elem));
  } else {
    __builtin_nontemporal_store(g, reinterpret_cast<f32x4*>(static_cast<float*>(grad) + elem));
  }
}

// NV = 16-byte groups per lane; D / 4 <= 64 NV.
// kNorm: per-patch normalised target (the recipe's objective); otherwise the target as it is.
// kRowsPerIter: adjacent rows a wavefront handles per pass.
template <int NV, int kRowsPerIter, bool kBf16, bool kNorm>
__global__ __launch_bounds__(kLossThreads) void normpix_loss_kernel(LossArgs a) {
  const int lane = threadIdx.x % kWave;
  const int wave_in_grid = blockIdx.x * kLossWaves + threadIdx.x / kWave;
  const int waves = gridDim.x * kLossWaves;
  const int D = a.D, D4 = a.D >> 2;
  const float inv_d = 1.0f / (float)D;
  const float inv_dm1 = 1.0f / (float)(D - 1);
  double acc = 0.0;
  const float gscale =
      a.counts ? (float)(a.gscale_num * inv_count_of(D, sum_counts(a.counts, a.ncounts))) : a.gscale;

  // kRowsPerIter adjacent rows per pass: all their loads are issued before the first reduction,
  // and each wavefront touches one contiguous span of every tensor.
  for (int64_t row0 = kRowsPerIter * (int64_t)wave_in_grid; row0 < a.rows;
       row0 += kRowsPerIter * (int64_t)waves) {
    f32x4 t[kRowsPerIter][NV], q[kRowsPerIter][NV];
    bool masked[kRowsPerIter];
#pragma unroll
    for (int u = 0; u < kRowsPerIter; ++u) {
      const int64_t row = row0 + u;
      masked[u] = row < a.rows && a.mask[row] != 0;
      const int64_t row_elem = row * D;
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        const int g = lane + v * kWave;
        t[u][v] = f32x4{0.f, 0.f, 0.f, 0.f};
        q[u][v] = t[u][v];
        if (masked[u] && g < D4) {
          t[u][v] = __builtin_nontemporal_load(
              reinterpret_cast<const f32x4*>(a.target + row_elem + 4 * g));
          q[u][v] = load_pred4<kBf16>(a.pred, row_elem + 4 * g);
        }
      }
    }
#pragma unroll
    for (int u = 0; u < kRowsPerIter; ++u) {
      const int64_t row = row0 + u;
      if (row >= a.rows) continue;
      const int64_t row_elem = row * D;
      if (!masked[u]) {  // visible patch: the gradient is zero, nothing was read
        if (a.grad) {
#pragma unroll
          for (int v = 0; v < NV; ++v) {
            const int g = lane + v * kWave;
            if (g < D4) store_grad4<kBf16>(a.grad, row_elem + 4 * g, f32x4{0.f, 0.f, 0.f, 0.f});
          }
        }
        continue;
      }
      float rstd = 1.0f;
      if (kNorm) {
        float s = 0.f;
#pragma unroll
        for (int v = 0; v < NV; ++v) s += (t[u][v].x + t[u][v].y) + (t[u][v].z + t[u][v].w);
        const float mu = wave_sum(s) * inv_d;
        float ss = 0.f;
#pragma unroll
        for (int v = 0; v < NV; ++v) {
          const int g = lane + v * kWave;
          t[u][v] = t[u][v] - mu;
          if (g < D4)
            ss += (t[u][v].x * t[u][v].x + t[u][v].y * t[u][v].y) +
                  (t[u][v].z * t[u][v].z + t[u][v].w * t[u][v].w);
        }
        const float var = wave_sum(ss) * inv_dm1;
        rstd = 1.0f / sqrtf(var + a.eps);
      }
      float sq = 0.f;
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        const int g = lane + v * kWave;
        const f32x4 diff = kNorm ? q[u][v] - t[u][v] * rstd : q[u][v] - t[u][v];
        if (g < D4) {
          sq += (diff.x * diff.x + diff.y * diff.y) + (diff.z * diff.z + diff.w * diff.w);
          if (a.grad) store_grad4<kBf16>(a.grad, row_elem + 4 * g, diff * gscale);
        }
      }
      acc += (double)sq;
    }
  }
  acc = wave_sum(acc);
  if (lane == 0) a.partials[wave_in_grid] = acc;
}

// Rows whose number of 16-byte groups is not a multiple of 64 leave part of a wavefront's last
// load and store per row idle (D = 588: 147 groups, the third instruction moves 19 of 64).  Two
// adjacent rows are contiguous in memory, so here a wavefront takes them as one run of 2 D / 4
// groups, lane i holding groups i, i + 64, ...: every instruction but the run's last is full.
// A group lies in one row (rows are whole groups), the two rows' sums are kept apart, and a
// lane's group takes the statistics of the row it lies in.  NVF = groups per lane.
template <int NVF, bool kBf16, bool kNorm>
__global__ __launch_bounds__(kLossThreads) void normpix_loss_pair_kernel(LossArgs a) {
  const int lane = threadIdx.x % kWave;
  const int wave_in_grid = blockIdx.x * kLossWaves + threadIdx.x / kWave;
  const int waves = gridDim.x * kLossWaves;
  const int D = a.D, D4 = a.D >> 2;
  const float inv_d = 1.0f / (float)D;
  const float inv_dm1 = 1.0f / (float)(D - 1);
  double acc = 0.0;
  const float gscale =
      a.counts ? (float)(a.gscale_num * inv_count_of(D, sum_counts(a.counts, a.ncounts))) : a.gscale;
  const f32x4 zero = f32x4{0.f, 0.f, 0.f, 0.f};

  for (int64_t row0 = 2 * (int64_t)wave_in_grid; row0 < a.rows; row0 += 2 * (int64_t)waves) {
    const bool have1 = row0 + 1 < a.rows;
    const bool m0 = a.mask[row0] != 0, m1 = have1 && a.mask[row0 + 1] != 0;
    const int64_t elem0 = row0 * D;
    f32x4 t[NVF], q[NVF];
    bool second[NVF], live[NVF];
#pragma unroll
    for (int v = 0; v < NVF; ++v) {
      const int g = lane + v * kWave;
      second[v] = g >= D4;
      live[v] = g < (have1 ? 2 * D4 : D4);
      t[v] = zero;
      q[v] = zero;
      if (live[v] && (second[v] ? m1 : m0)) {
        t[v] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(a.target + elem0 + 4 * g));
        q[v] = load_pred4<kBf16>(a.pred, elem0 + 4 * g);
      }
    }
    float rstd0 = 1.0f, rstd1 = 1.0f;
    if (kNorm) {
      float s0 = 0.f, s1 = 0.f;
#pragma unroll
      for (int v = 0; v < NVF; ++v) {
        const float s = (t[v].x + t[v].y) + (t[v].z + t[v].w);  // zero where nothing was loaded
        s0 += second[v] ? 0.f : s;
        s1 += second[v] ? s : 0.f;
      }
      const float mu0 = wave_sum(s0) * inv_d, mu1 = wave_sum(s1) * inv_d;
      float ss0 = 0.f, ss1 = 0.f;
#pragma unroll
      for (int v = 0; v < NVF; ++v) {
        t[v] = t[v] - (second[v] ? mu1 : mu0);
        const float ss = (t[v].x * t[v].x + t[v].y * t[v].y) + (t[v].z * t[v].z + t[v].w * t[v].w);
        const bool counted = live[v] && (second[v] ? m1 : m0);
        ss0 += (counted && !second[v]) ? ss : 0.f;
        ss1 += (counted && second[v]) ? ss : 0.f;
      }
      rstd0 = 1.0f / sqrtf(wave_sum(ss0) * inv_dm1 + a.eps);
      rstd1 = 1.0f / sqrtf(wave_sum(ss1) * inv_dm1 + a.eps);
    }
    float sq = 0.f;
#pragma unroll
    for (int v = 0; v < NVF; ++v) {
      if (!live[v]) continue;
      const int g = lane + v * kWave;
      const bool masked = second[v] ? m1 : m0;
      f32x4 diff = zero;  // visible rows: zero gradient, nothing towards the loss
      if (masked) {
        diff = kNorm ? q[v] - t[v] * (second[v] ? rstd1 : rstd0) : q[v] - t[v];
        sq += (diff.x * diff.x + diff.y * diff.y) + (diff.z * diff.z + diff.w * diff.w);
      }
      if (a.grad) store_grad4<kBf16>(a.grad, elem0 + 4 * g, diff * gscale);
    }
    acc += (double)sq;
  }
  acc = wave_sum(acc);
  if (lane == 0) a.partials[wave_in_grid] = acc;
}

// Any D (not a multiple of four, or too long for registers): three passes over the row.
template <bool kBf16, bool kNorm>
__global__ __launch_bounds__(kLossThreads) void normpix_loss_scalar_kernel(LossArgs a) {
  const int lane = threadIdx.x % kWave;
  const int wave_in_grid = blockIdx.x * kLossWaves + threadIdx.x / kWave;
  const int waves = gridDim.x * kLossWaves;
  const int D = a.D;
  double acc = 0.0;
  const float gscale =
      a.counts ? (float)(a.gscale_num * inv_count_of(D, sum_counts(a.counts, a.ncounts))) : a.gscale;
  for (int64_t row = wave_in_grid; row < a.rows; row += waves) {
    const int64_t row_elem = row * D;
    const float* t = a.target + row_elem;
    if (a.mask[row] == 0) {
      if (a.grad) {
        for (int e = lane; e < D; e += kWave) {
          if (kBf16) static_cast<uint16_t*>(a.grad)[row_elem + e] = 0;
          else static_cast<float*>(a.grad)[row_elem + e] = 0.f;
        }
      }
      continue;
    }
    float mu = 0.f, rstd = 1.0f;
    if (kNorm) {
      float s = 0.f;
      for (int e = lane; e < D; e += kWave) s += t[e];
      mu = wave_sum(s) / (float)D;
      float ss = 0.f;
      for (int e = lane; e < D; e += kWave) ss += (t[e] - mu) * (t[e] - mu);
      const float var = wave_sum(ss) / (float)(D - 1);
      rstd = 1.0f / sqrtf(var + a.eps);
    }
    float sq = 0.f;
    for (int e = lane; e < D; e += kWave) {
      float q;
      if (kBf16) q = __uint_as_float((uint32_t)static_cast<const uint16_t*>(a.pred)[row_elem + e] << 16);
      else q = static_cast<const float*>(a.pred)[row_elem + e];
      const float diff = kNorm ? q - (t[e] - mu) * rstd : q - t[e];
      sq += diff * diff;
      if (a.grad) {
        if (kBf16) static_cast<uint16_t*>(a.grad)[row_elem + e] = (uint16_t)bf16_rne(diff * gscale);
        else static_cast<float*>(a.grad)[row_elem + e] = diff * gscale;
      }
    }
    acc += (double)sq;
  }
  acc = wave_sum(acc);
  if (lane == 0) a.partials[wave_in_grid] = acc;
}

// Adds the per-wavefront partials in a fixed order: thread i takes partials i, i + 256, ...,
// then a tree over the 256 threads.
__global__ __launch_bounds__(kLossThreads) void loss_finish_kernel(const double* partials, int n,
                                                                  double inv_count, float* loss,
                                                                  const int32_t* counts,
                                                                  int ncounts, int D) {
  __shared__ double red[kLossThreads];
  if (counts) inv_count = inv_count_of(D, sum_counts(counts, ncounts));
  double s = 0.0;
  for (int i = threadIdx.x; i < n; i += kLossThreads) s += partials[i];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int off = kLossThreads / 2; off > 0; off >>= 1) {
    if ((int)threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) *loss = (float)(red[0] * inv_count);
}

// Groups per lane of the pair kernel for rows of D values, 0 when pairing saves nothing (a row
// is a whole number of 64-group instructions, or two rows need as many as one row twice) or does
// not fit the registers.
static int pair_groups(int D) {
  const int d4 = D >> 2;
  const int single = (d4 + kWave - 1) / kWave, pair = (2 * d4 + kWave - 1) / kWave;
  return (pair < 2 * single && pair <= 6) ? pair : 0;
}

// Launch shape.  What counts is the amount of row data in flight per compute unit (about 144 KiB
// measured best on MI355X) and that every compute unit gets the same number of workgroups.  Rows
// that bring 6 KiB or more of loads (D = 768 in fp32) go two per pass with 3 workgroups per compute
// unit; shorter rows one per pass with 6, or, when their groups do not fill whole instructions,
// as pairs in one run of groups with 4.
LossShape loss_shape(int64_t rows, int D, bool pred_bf16) {
  LossShape sh;
  const int nv = ((D >> 2) + kWave - 1) / kWave;
  const int64_t load_bytes = (int64_t)D * (pred_bf16 ? 6 : 8);
  const bool vec = (D & 3) == 0 && (D >> 2) <= 12 * kWave;
  sh.rows_per_iter = (vec && nv <= 4 && load_bytes >= 6144) ? 2 : 1;
  // rows as pairs in one run of groups: when that saves a load and a store instruction per pair
  sh.pair_groups = (vec && sh.rows_per_iter == 1) ? pair_groups(D) : 0;
  if (sh.pair_groups) sh.rows_per_iter = 2;
  // workgroups per compute unit (measured best: D = 768 fp32 two rows at 3, D = 588 bf16 pairs
  // at 4, single rows at 6)
  const int per_cu = sh.pair_groups ? 4 : (sh.rows_per_iter == 2 ? 3 : 6);
  const int64_t rows_per_block = (int64_t)kLossWaves * sh.rows_per_iter;
  int64_t blocks = (rows + rows_per_block - 1) / rows_per_block;
  const int64_t cap = (int64_t)kComputeUnits * per_cu;
  if (blocks > cap) blocks = cap;
  if (blocks < 1) blocks = 1;
  sh.waves = (int)blocks * kLossWaves;
  return sh;
}

template <bool kBf16, bool kNorm>
static void launch_vec(const LossArgs& a, dim3 grid, dim3 block, hipStream_t stream) {
  const int nv = ((a.D >> 2) + kWave - 1) / kWave;
  const int nvf = a.pair_groups;
  if (nvf != 0) {
#define MAE_LAUNCH_PAIR(NVF) \
  hipLaunchKernelGGL((normpix_loss_pair_kernel<NVF, kBf16, kNorm>), grid, block, 0, stream, a)
    if (nvf <= 1) MAE_LAUNCH_PAIR(1);
    else if (nvf == 2) MAE_LAUNCH_PAIR(2);
    else if (nvf == 3) MAE_LAUNCH_PAIR(3);
    else if (nvf == 4) MAE_LAUNCH_PAIR(4);
    else if (nvf == 5) MAE_LAUNCH_PAIR(5);
    else MAE_LAUNCH_PAIR(6);
#undef MAE_LAUNCH_PAIR
    return;
  }
#define MAE_LAUNCH(NV, RPI) \
  hipLaunchKernelGGL((normpix_loss_kernel<NV, RPI, kBf16, kNorm>), grid, block, 0, stream, a)
  if (a.rows_per_iter == 2) {
    if (nv <= 1) MAE_LAUNCH(1, 2);
    else if (nv <= 2) MAE_LAUNCH(2, 2);
    else if (nv <= 3) MAE_LAUNCH(3, 2);
    else MAE_LAUNCH(4, 2);
  } else {
    if (nv <= 1) MAE_LAUNCH(1, 1);
    else if (nv <= 2) MAE_LAUNCH(2, 1);
    else if (nv <= 3) MAE_LAUNCH(3, 1);
    else if (nv <= 4) MAE_LAUNCH(4, 1);
    else if (nv <= 6) MAE_LAUNCH(6, 1);
    else if (nv <= 8) MAE_LAUNCH(8, 1);
    else MAE_LAUNCH(12, 1);
  }
#undef MAE_LAUNCH
}

template <bool kBf16, bool kNorm>
static void launch_any(const LossArgs& a, dim3 grid, dim3 block, hipStream_t stream) {
  const bool vec = (a.D & 3) == 0 && (a.D >> 2) <= 12 * kWave;
  if (vec) {
    launch_vec<kBf16, kNorm>(a, grid, block, stream);
  } else {
    hipLaunchKernelGGL((normpix_loss_scalar_kernel<kBf16, kNorm>), grid, block, 0, stream, a);
  }
}

hipError_t launch_loss_finish(const double* partials, int n, double inv_count, float* loss,
                              const int32_t* counts, int ncounts, int D, hipStream_t stream) {
  hipLaunchKernelGGL(loss_finish_kernel, dim3(1), dim3(kLossThreads), 0, stream, partials, n,
                     inv_count, loss, counts, ncounts, D);
  return hipGetLastError();
}

// Non-zero bytes of the mask, one partial count per workgroup (contiguous shares of 64 Ki rows or
// more), for callers that leave the divisor to the device.
constexpr int64_t kCountShare = 65536;
__global__ __launch_bounds__(kLossThreads) void mask_count_kernel(const uint8_t* mask, int64_t rows,
                                                                 int32_t* counts) {
  __shared__ int red[kLossWaves];
  const int64_t share = (rows + gridDim.x - 1) / gridDim.x;
  const int64_t lo = (int64_t)blockIdx.x * share, hi = min(rows, lo + share);
  int c = 0;
  for (int64_t i = lo + threadIdx.x; i < hi; i += kLossThreads) c += mask[i] != 0 ? 1 : 0;
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) c += __shfl_xor(c, off, kWave);
  if (threadIdx.x % kWave == 0) red[threadIdx.x / kWave] = c;
  __syncthreads();
  if (threadIdx.x == 0) {
    int t = 0;
    for (int w = 0; w < kLossWaves; ++w) t += red[w];
    counts[blockIdx.x] = t;
  }
}
int mask_count_blocks(int64_t rows) {
  int64_t n = (rows + kCountShare - 1) / kCountShare;
  return (int)(n < 1 ? 1 : (n > kMaxCounts ? kMaxCounts : n));
}
hipError_t launch_mask_count(const uint8_t* mask, int64_t rows, int32_t* counts,
                             hipStream_t stream) {
  hipLaunchKernelGGL(mask_count_kernel, dim3(mask_count_blocks(rows)), dim3(kLossThreads), 0,
                     stream, mask, rows, counts);
  return hipGetLastError();
}

hipError_t launch_normpix_loss(const LossArgs& a, hipStream_t stream) {
  dim3 grid(a.num_partials / kLossWaves), block(kLossThreads);
  if (a.pred_bf16) {
    if (a.norm_pix) launch_any<true, true>(a, grid, block, stream);
    else launch_any<true, false>(a, grid, block, stream);
  } else {
    if (a.norm_pix) launch_any<false, true>(a, grid, block, stream);
    else launch_any<false, false>(a, grid, block, stream);
  }
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return err;
  hipLaunchKernelGGL(loss_finish_kernel, dim3(1), block, 0, stream, a.partials, a.num_partials,
                     a.inv_count, a.loss, a.counts, a.ncounts, a.D);
  return hipGetLastError();
}

}  // namespace mae
