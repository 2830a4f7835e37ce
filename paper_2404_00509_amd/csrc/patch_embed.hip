// Patch embedding of the visible tokens (Sec. 2: only the visible patches reach the encoder;
// Sec. 5: the ViT's linear patch embedding): tokens = visible x weight^T + bias + pos[ids_keep].
//
// The one dense contraction next to the input pipeline, so it runs on the matrix cores:
// v_mfma_f32_32x32x16_bf16, bf16 operands, fp32 accumulation.  Both operands are K-contiguous
// (visible [M, D], weight [E, D]), which is the layout the instruction wants: a lane supplies 8
// consecutive k of one row.
//
// One workgroup (4 wavefronts as 2 x 2, 128 x 64 each) makes a 256 x 128 tile of the result.  D is
// walked in slices of 32; the two operand slices (256 + 128 rows of 64 bytes = 24 KiB) go from
// global memory straight into LDS (global_load_lds_dwordx4, no trip through registers) into one
// of three stage buffers, two slices ahead of the one being multiplied, and the wavefront waits
// with an explicit vmcnt for exactly the slice it needs.  A staged row is four 16-byte chunks
// whose position is XORed with bits 1..2 of the row number, which spreads the fragment reads
// (ds_read_b128, 32 rows of one chunk column per half wave) over the banks; because a direct load
// always writes lane l to slot l of the wave's 1 KiB window, the swizzle is applied on the global
// side: each lane fetches the chunk that belongs in its slot.  The last, partial slice of a D
// that is no multiple of 32 goes through registers instead, zero-filled past the row's end.
//
// The fragment reads are issued through inline assembly: the compiler does not see them as LDS
// accesses, so it does not make each of them wait for every direct load in flight (which would
// undo the pipeline); the code waits on lgkmcnt itself.
//
// Epilogue: the accumulators go through LDS, 32 rows of the tile at a time, so that the stores to
// `tokens` (and the loads of the positional rows) are 16 bytes per lane and contiguous along a
// row; bias and pos[ids_keep] are added in fp32 before the single rounding to the output type.
// Two workgroups fit a compute unit (212 VGPRs, 75 KiB LDS), so one's epilogue overlaps the
// other's main loop.  Consecutive workgroups of an XCD walk the E direction of one row block
// first: they share the rows of `visible` through that XCD's L2.
#include "mae_device.hpp"
#include "mae_kernels.hpp"

namespace mae {

constexpr int kEmbThreads = 256;
constexpr int kBM = 256, kBN = 128, kBK = 32;
constexpr int kRowChunks = kBK / 8;                       // 4 chunks of 16 bytes per staged row
constexpr int kStageSlots = (kBM + kBN) * kRowChunks;     // 1536 slots of 16 bytes = 24 KiB
constexpr int kLoadsPerWave = kStageSlots / kWave / 4;    // 6 wave-wide loads per stage and wave

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef u32x4 u32x4_a4 __attribute__((aligned(4)));
typedef u32x2 u32x2_a4 __attribute__((aligned(4)));

// Eight consecutive bf16 of a row starting at element k, zero beyond the row's end (D % 4 == 0).
__device__ static inline u32x4 load_chunk(const uint16_t* row, int k, int D) {
  u32x4 v = {0u, 0u, 0u, 0u};
  if (k + 8 <= D) {
    v = *reinterpret_cast<const u32x4_a4*>(row + k);
  } else if (k + 4 <= D) {
    const u32x2 h = *reinterpret_cast<const u32x2_a4*>(row + k);
    v.x = h.x;
    v.y = h.y;
  }
  return v;
}

// 16-byte LDS read the compiler does not see as an LDS access: it would otherwise make every
// read wait for all direct-to-LDS loads in flight, including those of later pipeline stages.
// The caller waits on lgkmcnt itself.
__device__ static inline u32x4 lds_read16(const u32x4* p) {
  u32x4 v;
  const uint32_t addr = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) u32x4*)p;
  asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(addr) : "memory");
  return v;
}

// slot of (row, chunk) inside a staged tile: 64-byte rows, chunk index XORed with bits 1..2 of the
// row so that 8 consecutive rows of one chunk column fall into 8 different 16-byte bank groups
__device__ static inline int slot_of(int row, int chunk) {
  return row * kRowChunks + (chunk ^ ((row >> 1) & (kRowChunks - 1)));
}

template <bool kOutBf16>
__global__ __launch_bounds__(kEmbThreads, 2) void patch_embed_kernel(EmbedArgs a) {
  __shared__ __attribute__((aligned(16))) u32x4 st0[kStageSlots];
  __shared__ __attribute__((aligned(16))) u32x4 st1[kStageSlots];
  __shared__ __attribute__((aligned(16))) u32x4 st2[kStageSlots];
  __shared__ int sIds[kBM];

  const int tid = threadIdx.x;
  const int lane = tid % kWave;
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int wm = wave >> 1, wn = wave & 1;  // 2 x 2 wavefronts, 128 x 64 each
  const int tiles_n = (a.E + kBN - 1) / kBN;
  const int64_t tile = xcd_remap(blockIdx.x, gridDim.x);
  const int64_t m0 = (tile / tiles_n) * kBM;
  const int n0 = (int)(tile % tiles_n) * kBN;
  const int D = a.D;
  const uint16_t* A = static_cast<const uint16_t*>(a.visible);
  const uint16_t* W = static_cast<const uint16_t*>(a.weight);

  for (int r = tid; r < kBM; r += kEmbThreads) {
    const int64_t m = m0 + r;
    int id = (a.ids_keep && m < a.M) ? a.ids_keep[m] : 0;
    sIds[r] = min(max(id, 0), a.L - 1);
  }

  // what this lane brings in per stage: 6 slots; slot s = (wave * 6 + q) * 64 + lane
  const uint16_t* src[kLoadsPerWave];
  int src_chunk[kLoadsPerWave];
#pragma unroll
  for (int q = 0; q < kLoadsPerWave; ++q) {
    const int s = (wave * kLoadsPerWave + q) * kWave + lane;
    const int row = s / kRowChunks;                                  // 0..383: A rows then B rows
    const int chunk = (s % kRowChunks) ^ ((row >> 1) & (kRowChunks - 1));
    src_chunk[q] = chunk;
    if (row < kBM) {
      const int64_t m = min(m0 + row, a.M - 1);                      // rows past the end: any valid row
      src[q] = A + m * D + 8 * chunk;
    } else {
      const int n = min(n0 + row - kBM, a.E - 1);
      src[q] = W + (int64_t)n * D + 8 * chunk;
    }
  }

  const int nk = (D + kBK - 1) / kBK;
#define ISSUE(IT, STAGE)                                                                      \
  {                                                                                           \
    const int k0 = (IT) * kBK;                                                                \
    if (k0 + kBK <= D) {                                                                      \
      _Pragma("unroll") for (int q = 0; q < kLoadsPerWave; ++q) {                            \
        __builtin_amdgcn_global_load_lds(                                                     \
            (const void __attribute__((address_space(1)))*)(src[q] + k0),                     \
            (void __attribute__((address_space(3)))*)(STAGE + (wave * kLoadsPerWave + q) * kWave), \
            16, 0, 0);                                                                        \
      }                                                                                       \
    } else {                                                                                  \
      _Pragma("unroll") for (int q = 0; q < kLoadsPerWave; ++q) {                            \
        STAGE[(wave * kLoadsPerWave + q) * kWave + lane] =                                    \
            load_chunk(src[q] - 8 * src_chunk[q], k0 + 8 * src_chunk[q], D);                  \
      }                                                                                       \
    }                                                                                         \
  }

  f32x16 acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

#define STEP(IT, CUR, NEXT2)                                                                  \
  if ((IT) < nk) {                                                                            \
    if ((IT) + 1 < nk && ((IT) + 2) * kBK <= D) {                                             \
      __builtin_amdgcn_s_waitcnt(0x0F70 | kLoadsPerWave);                                     \
    } else {                                                                                  \
      __builtin_amdgcn_s_waitcnt(0x0F70);                                                     \
    }                                                                                         \
    __builtin_amdgcn_s_barrier();                                                             \
    if ((IT) + 2 < nk) ISSUE((IT) + 2, NEXT2)                                                 \
    const u32x4* sA = CUR;                                                                    \
    const u32x4* sB = CUR + kBM * kRowChunks;                                                 \
    _Pragma("unroll") for (int ks = 0; ks < kBK / 16; ++ks) {                                \
      const int chunk = 2 * ks + (lane >> 5);                                                 \
      bf16x8 fa[4], fb[2];                                                                    \
      _Pragma("unroll") for (int i = 0; i < 4; ++i) fa[i] = __builtin_bit_cast(              \
          bf16x8, lds_read16(sA + slot_of(wm * 128 + i * 32 + (lane & 31), chunk)));          \
      _Pragma("unroll") for (int j = 0; j < 2; ++j) fb[j] = __builtin_bit_cast(              \
          bf16x8, lds_read16(sB + slot_of(wn * 64 + j * 32 + (lane & 31), chunk)));           \
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");                                      \
      _Pragma("unroll") for (int i = 0; i < 4; ++i)                                          \
      _Pragma("unroll") for (int j = 0; j < 2; ++j) acc[i][j] =                              \
          __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);          \
    }                                                                                         \
  }

  if (0 < nk) ISSUE(0, st0)
  if (1 < nk) ISSUE(1, st1)
  __syncthreads();  // sIds
  for (int it = 0; it < nk; it += 3) {
    STEP(it, st0, st2)
    STEP(it + 1, st1, st0)
    STEP(it + 2, st2, st1)
  }
#undef STEP
#undef ISSUE

  // epilogue through LDS, one 32-row band of the tile at a time: fp32 [32][128] = 16 KiB in st0
  float* out_tile = reinterpret_cast<float*>(st0);
#pragma unroll
  for (int band = 0; band < 8; ++band) {
    __syncthreads();  // staged operands (or the previous band) are no longer needed
    if (wm == band / 4) {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int c = wn * 64 + j * 32 + (lane & 31);
        const int n = n0 + c;
        const float bias = (a.bias && n < a.E) ? a.bias[n] : 0.f;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int r = (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
          out_tile[r * kBN + c] = acc[band % 4][j][e] + bias;
        }
      }
    }
    __syncthreads();
    // 32 rows x 16 groups of 8 columns: 2 groups per thread
#pragma unroll
    for (int rep = 0; rep < 2; ++rep) {
      const int idx = tid + rep * kEmbThreads;
      const int r = idx / (kBN / 8), g = idx % (kBN / 8);
      const int tile_row = band * 32 + r;
      const int64_t m = m0 + tile_row;
      const int n = n0 + 8 * g;
      if (m >= a.M || n >= a.E) continue;
      f32x4 v0 = *reinterpret_cast<const f32x4*>(out_tile + r * kBN + 8 * g);
      f32x4 v1 = *reinterpret_cast<const f32x4*>(out_tile + r * kBN + 8 * g + 4);
      float v[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
      const float* pos = a.pos ? a.pos + (int64_t)sIds[tile_row] * a.E + n : nullptr;
      const bool full = n + 8 <= a.E && (a.E & 7) == 0;
      if (full) {
        if (pos) {
          const f32x4 p0 = *reinterpret_cast<const f32x4*>(pos);
          const f32x4 p1 = *reinterpret_cast<const f32x4*>(pos + 4);
          v[0] += p0.x; v[1] += p0.y; v[2] += p0.z; v[3] += p0.w;
          v[4] += p1.x; v[5] += p1.y; v[6] += p1.z; v[7] += p1.w;
        }
        if (kOutBf16) {
          u32x4 o = {pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]),
                     pack_bf16x2(v[6], v[7])};
          *reinterpret_cast<u32x4*>(static_cast<uint16_t*>(a.tokens) + m * a.E + n) = o;
        } else {
          float* dst = static_cast<float*>(a.tokens) + m * a.E + n;
          *reinterpret_cast<f32x4*>(dst) = f32x4{v[0], v[1], v[2], v[3]};
          *reinterpret_cast<f32x4*>(dst + 4) = f32x4{v[4], v[5], v[6], v[7]};
        }
      } else {
        for (int q = 0; q < 8 && n + q < a.E; ++q) {
          const float x = v[q] + (pos ? pos[q] : 0.f);
          if (kOutBf16) static_cast<uint16_t*>(a.tokens)[m * a.E + n + q] = (uint16_t)bf16_rne(x);
          else static_cast<float*>(a.tokens)[m * a.E + n + q] = x;
        }
      }
    }
  }
}

hipError_t launch_patch_embed(const EmbedArgs& a, hipStream_t stream) {
  const int64_t tiles_m = (a.M + kBM - 1) / kBM;
  const int64_t tiles_n = (a.E + kBN - 1) / kBN;
  dim3 grid((uint32_t)(tiles_m * tiles_n)), block(kEmbThreads);
  if (a.out_bf16) {
    hipLaunchKernelGGL(patch_embed_kernel<true>, grid, block, 0, stream, a);
  } else {
    hipLaunchKernelGGL(patch_embed_kernel<false>, grid, block, 0, stream, a);
  }
  return hipGetLastError();
}

}  // namespace mae
