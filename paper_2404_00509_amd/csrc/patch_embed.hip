// Patch embedding of the visible tokens (Sec. 2: only the visible patches reach the encoder;
// Sec. 5: the ViT's linear patch embedding): tokens = visible x weight^T + bias + pos[ids_keep].
//
// The one dense contraction next to the input pipeline, so it runs on the matrix cores:
// v_mfma_f32_32x32x16_bf16, bf16 operands, fp32 accumulation.  Both operands are K-contiguous
// (visible [M, D], weight [E, D]), which is the layout the instruction wants: a lane supplies 8
// consecutive k of one row.
//
// A workgroup of eight wavefronts (2 x 4, 128 x 64 results each) makes a 256 x 256 tile.  D is
// walked in slices of 64 values, so that every row contributes one full 128-byte line per slice:
// half-line requests cost the vector memory pipeline as much as whole lines.  The two operand
// slices (512 rows of 128 bytes = 64 KiB) go from global memory straight into LDS
// (global_load_lds_dwordx4, no trip through registers) into one of two stage buffers while the
// other one is multiplied.  A staged row is eight 16-byte chunks whose position is XORed with
// bits 1..3 of the row number: 16 consecutive rows of one chunk column then fall into 16
// different 16-byte bank groups, which is what a ds_read_b128 of the 64-bank LDS needs to run at
// full rate (fragment reads: 32 rows of one chunk column per half wave).  Because a direct load
// always writes lane l to slot l of the wave's 1 KiB window, the swizzle is applied on the global
// side: each lane fetches the chunk that belongs in its slot.  The last, partial slice of a D
// that is no multiple of 64 goes through registers instead, zero-filled past the row's end.
//
// The fragment reads are issued through inline assembly: the compiler does not see them as LDS
// accesses, so it does not make each of them wait for every direct load in flight (which would
// undo the pipeline); the code waits on lgkmcnt itself and reads one sub-step ahead.
//
// What bounds the kernel is the compute unit's vector memory pipeline (operand slices in, the
// positional rows in, tokens out), not the matrix cores, hence the large tile: it needs the
// fewest operand bytes per result.  The rows of `visible` are first touched here, so their
// latency is that of HBM; every wavefront requests a few lines of later slices into L2 ahead of
// time (one dword per line; the workgroups that share the rows, one per tile along E, split
// them), which shortens the time the staged loads hold the pipeline's miss slots.
//
// Epilogue: each wavefront turns its accumulators into rows through a private strip of LDS, 32
// rows at a time, so that the stores to `tokens` and the loads of the positional rows are
// contiguous along a row (8 values per lane).  The patch indices are fetched at kernel start
// and exchanged between lanes, and the positional rows of the next 32 rows are requested
// before the current ones are transposed.  Bias and pos[ids_keep] are added in fp32 before the
// single rounding to the output type.  Consecutive workgroups of an XCD walk the E direction of
// one row block first: they share the rows of `visible` through that XCD's L2.
#include "mae_device.hpp"
#include "mae_kernels.hpp"

namespace mae {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef u32x4 u32x4_a4 __attribute__((aligned(4)));
typedef u32x2 u32x2_a4 __attribute__((aligned(4)));

constexpr int kBK = 64;            // values of D per pipeline stage: one 128-byte line per row
constexpr int kPrefetch = 3;       // slices of `visible` requested into L2 ahead of staging
constexpr int kRowChunks = 8;      // 16-byte chunks per staged row
constexpr int kEpiPad = 8;         // floats of padding per staged output row

// Eight consecutive bf16 starting at p, of which only `left` lie inside the row (left % 4 == 0).
__device__ static inline u32x4 load_chunk(const uint16_t* p, int left) {
  u32x4 v = {0u, 0u, 0u, 0u};
  if (left >= 8) {
    v = *reinterpret_cast<const u32x4_a4*>(p);
  } else if (left >= 4) {
    const u32x2 h = *reinterpret_cast<const u32x2_a4*>(p);
    v.x = h.x;
    v.y = h.y;
  }
  return v;
}

// 16-byte LDS read the compiler does not see as an LDS access (see the file comment).  The
// caller waits on lgkmcnt itself before it touches the result.
template <int kOff>
__device__ static inline u32x4 lds_read16(uint32_t addr) {
  u32x4 v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(kOff) : "memory");
  return v;
}

// s_waitcnt immediate: vmcnt(n), expcnt and lgkmcnt not waited for
constexpr int waitcnt_vm(int n) { return (n & 0xF) | ((n >> 4) << 14) | 0x0F70; }

template <int TM, int TN, int WGM, int WGN, int STAGES, int OCC, bool kOutBf16>
__global__ __launch_bounds__(64 * WGM * WGN, OCC) void patch_embed_kernel(EmbedArgs a) {
  constexpr int kThreads = 64 * WGM * WGN;
  constexpr int kWaves = WGM * WGN;
  constexpr int BM = 32 * TM * WGM, BN = 32 * TN * WGN;
  constexpr int kSlots = (BM + BN) * kRowChunks;  // 16-byte slots per stage
  constexpr int NL = kSlots / kThreads;           // direct loads per lane and stage
  static_assert(kSlots % kThreads == 0, "stage must divide into wave-wide loads");
  static_assert(NL * (STAGES - 2) <= 63, "vmcnt range");
  constexpr int kStageBytes = kSlots * 16;
  constexpr int kEpiStride = 32 * TN + kEpiPad;           // floats
  constexpr int kEpiWave = 32 * kEpiStride;               // floats per wave
  constexpr int kMainBytes = STAGES * kStageBytes;
  constexpr int kEpiBytes = kWaves * kEpiWave * 4;
  constexpr int kLdsBytes = kMainBytes > kEpiBytes ? kMainBytes : kEpiBytes;
  __shared__ __attribute__((aligned(16))) u32x4 lds[kLdsBytes / 16];

  const int tid = threadIdx.x;
  const int lane = tid % kWave;
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int wm = wave / WGN, wn = wave % WGN;
  const int tiles_n = (a.E + BN - 1) / BN;
  const int64_t tile = xcd_remap(blockIdx.x, gridDim.x);
  const int64_t m0 = (tile / tiles_n) * BM;
  const int n0 = (int)(tile % tiles_n) * BN;
  const int D = a.D;
  const uint16_t* A = static_cast<const uint16_t*>(a.visible);
  const uint16_t* W = static_cast<const uint16_t*>(a.weight);

  // what this lane brings in per stage: slot s = (wave * NL + q) * 64 + lane holds chunk
  // (s % 8) ^ (row / 2 % 8) of row s / 8 (rows of `visible` first, then rows of `weight`)
  const uint16_t* src[NL];
#pragma unroll
  for (int q = 0; q < NL; ++q) {
    const int s = (wave * NL + q) * kWave + lane;
    const int row = s / kRowChunks;
    const int chunk = (s % kRowChunks) ^ ((row >> 1) % kRowChunks);
    if (row < BM) {
      const int64_t m = min(m0 + row, a.M - 1);  // rows past the end: any valid row
      src[q] = A + m * D + 8 * chunk;
    } else {
      const int n = min(n0 + row - BM, a.E - 1);
      src[q] = W + (int64_t)n * D + 8 * chunk;
    }
  }

  auto issue_part = [&](int it, int stage, int q0, int q1) {
    const int k0 = it * kBK;
    u32x4* dst = lds + stage * kSlots + wave * NL * kWave;
    if (k0 + kBK <= D) {
#pragma unroll
      for (int q = 0; q < NL; ++q) {
        if (q < q0 || q >= q1) continue;
        __builtin_amdgcn_global_load_lds(
            (const void __attribute__((address_space(1)))*)(src[q] + k0),
            (void __attribute__((address_space(3)))*)(dst + q * kWave), 16, 0, 0);
      }
    } else if (q0 == 0) {
      // the last, partial slice goes through registers, zero-filled past the row's end
#pragma unroll
      for (int q = 0; q < NL; ++q) {
        const int s = (wave * NL + q) * kWave + lane;
        const int chunk = (s % kRowChunks) ^ ((s / kRowChunks / 2) % kRowChunks);
        dst[q * kWave + lane] = load_chunk(src[q] + k0, D - (k0 + 8 * chunk));
      }
    }
  };
  auto issue = [&](int it, int stage) { issue_part(it, stage, 0, NL); };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // fragment addresses inside a stage (bytes): row (lane % 32) of the wave's first 32-row block,
  // chunk (2 ks + lane / 32) ^ (row / 2 % 8); the row blocks and ks = 0..3 differ by constants
  const uint32_t lds_base =
      (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) u32x4*)lds;
  const uint32_t c0 = (uint32_t)((lane >> 5) ^ ((lane >> 1) & 7)) * 16u;
  const uint32_t a_off = (uint32_t)(wm * 32 * TM + (lane & 31)) * 128u + c0;
  const uint32_t b_off = (uint32_t)(BM + wn * 32 * TN + (lane & 31)) * 128u + c0;

  const int nk = (D + kBK - 1) / kBK;

  // patch index of row (lane % 32) of each of the wave's 32-row bands, for the epilogue
  int idr[TM];
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int64_t m = min(m0 + wm * 32 * TM + i * 32 + (lane & 31), a.M - 1);
    idr[i] = a.pos ? a.ids_keep[m] : 0;  // clamped where it is used: no wait for it here
  }

  // rolling prefetch of `visible` into L2, kPrefetch slices ahead of the staged loads.  The
  // workgroups that share these rows (one per tile along E) each fetch every tiles_n-th row.
  // The destination register is never read; it stays reserved until the loads have returned.
  static_assert(kPrefetch == 0 || STAGES == 2, "prefetch accounting assumes two stages");
  const int jn = (int)(tile % tiles_n);
  const bool wave_pf = kPrefetch > 0 && (wave * kWave * tiles_n + jn) < BM;  // wave-uniform
  const uint16_t* pf_row = A + min(m0 + min(tid * tiles_n + jn, BM - 1), a.M - 1) * D;
  uint32_t pf_dummy = 0;
  auto prefetch = [&](int slice) {
    if (wave_pf) {
      const int k = min(slice * kBK, D - 4);
      asm volatile("global_load_dword %0, %1, off" : "+v"(pf_dummy) : "v"(pf_row + k) : "memory");
    }
  };

#pragma unroll
  for (int s = 0; s < STAGES - 1; ++s)
    if (s < nk) issue(s, s);
#pragma unroll
  for (int s = 1; s <= kPrefetch; ++s) prefetch(s);

  int cur = 0;
  for (int it = 0; it < nk; ++it) {
    // the slice of this iteration has landed; later ones (at most STAGES - 2) may stay in flight
    if (STAGES >= 3 && it + STAGES - 2 < nk && (it + STAGES - 1) * kBK <= D) {
      __builtin_amdgcn_s_waitcnt(waitcnt_vm(NL * (STAGES - 2)));
    } else if (kPrefetch > 0 && wave_pf && (it + 1) * kBK <= D) {
      // only the prefetches issued after this slice's loads may still be in flight
      if (it == 0) __builtin_amdgcn_s_waitcnt(0x0070 | (kPrefetch & 0xF));
      else __builtin_amdgcn_s_waitcnt(0x0070 | 1);
    } else {
      __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) and lgkmcnt(0): staged stores included
    }
    __builtin_amdgcn_s_barrier();
    {
      const int nxt = it + STAGES - 1;
      int st = cur + STAGES - 1;
      if (st >= STAGES) st -= STAGES;
      if (nxt < nk) {
        issue(nxt, st);
        prefetch(nxt + kPrefetch);
      }
    }
    const uint32_t sbase = lds_base + (uint32_t)cur * kStageBytes;
    u32x4 fa[2][TM], fb[2][TN];
    auto read_frags = [&](int ks, int set) {
      const uint32_t va = sbase + (a_off ^ (32u * ks));
      const uint32_t vb = sbase + (b_off ^ (32u * ks));
      if constexpr (TM >= 1) fa[set][0] = lds_read16<0>(va);
      if constexpr (TM >= 2) fa[set][1] = lds_read16<4096>(va);
      if constexpr (TM >= 3) fa[set][2] = lds_read16<8192>(va);
      if constexpr (TM >= 4) fa[set][3] = lds_read16<12288>(va);
      if constexpr (TN >= 1) fb[set][0] = lds_read16<0>(vb);
      if constexpr (TN >= 2) fb[set][1] = lds_read16<4096>(vb);
      if constexpr (TN >= 3) fb[set][2] = lds_read16<8192>(vb);
      if constexpr (TN >= 4) fb[set][3] = lds_read16<12288>(vb);
    };
    read_frags(0, 0);
#pragma unroll
    for (int ks = 0; ks < kBK / 16; ++ks) {
      const int set = ks & 1;
      if (ks + 1 < kBK / 16) {
        read_frags(ks + 1, set ^ 1);
        // the reads of this sub-step are complete when only the TM + TN just issued remain
        if constexpr (TM + TN == 6)
          asm volatile("s_waitcnt lgkmcnt(6)" ::: "memory");
        else if constexpr (TM + TN == 5)
          asm volatile("s_waitcnt lgkmcnt(5)" ::: "memory");
        else if constexpr (TM + TN == 4)
          asm volatile("s_waitcnt lgkmcnt(4)" ::: "memory");
        else
          asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      } else {
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      }
      // tie the fragments to the wait so that no multiply is scheduled above it
#pragma unroll
      for (int i = 0; i < TM; ++i) asm volatile("" : "+v"(fa[set][i]));
#pragma unroll
      for (int j = 0; j < TN; ++j) asm volatile("" : "+v"(fb[set][j]));
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
              __builtin_bit_cast(bf16x8, fa[set][i]), __builtin_bit_cast(bf16x8, fb[set][j]),
              acc[i][j], 0, 0, 0);
    }
    cur = cur + 1 == STAGES ? 0 : cur + 1;
  }

  // ---- epilogue: each wavefront turns its own accumulators into rows through a private strip
  // of LDS (32 rows at a time), adds bias and the positional row, stores 8 values per lane.
  // The positional rows of the next band are requested before the current band is transposed.
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  asm volatile("" ::"v"(pf_dummy));
  __syncthreads();  // every wavefront is done with the staged operands
  float* epi = reinterpret_cast<float*>(lds) + wave * kEpiWave;
  constexpr int kLanesPerRow = 4 * TN;            // 8 columns per lane
  constexpr int kRowsPerRep = kWave / kLanesPerRow;
  constexpr int kReps = 32 / kRowsPerRep;
  const int col8 = (lane % kLanesPerRow) * 8;
  const int n = n0 + wn * 32 * TN + col8;
  const bool vec_ok = (a.E % 8 == 0) && n + 8 <= a.E;
  float bias[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int nb = n0 + wn * 32 * TN + j * 32 + (lane & 31);
    bias[j] = (a.bias && nb < a.E) ? a.bias[nb] : 0.f;
  }
  f32x4 p[2][kReps][2];
  int pid[2][kReps];
  auto load_pos = [&](int i, int buf) {
#pragma unroll
    for (int rep = 0; rep < kReps; ++rep) {
      const int r = rep * kRowsPerRep + lane / kLanesPerRow;
      const int id = min(max(__builtin_amdgcn_ds_bpermute(4 * r, idr[i]), 0), a.L - 1);
      pid[buf][rep] = id;
      p[buf][rep][0] = p[buf][rep][1] = f32x4{0.f, 0.f, 0.f, 0.f};
      if (a.pos && vec_ok) {
        const f32x4* src4 = reinterpret_cast<const f32x4*>(a.pos + (int64_t)id * a.E + n);
        p[buf][rep][0] = src4[0];
        p[buf][rep][1] = src4[1];
      }
    }
  };
  load_pos(0, 0);
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    if (i + 1 < TM) load_pos(i + 1, (i + 1) & 1);
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int r = (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
        epi[r * kEpiStride + j * 32 + (lane & 31)] = acc[i][j][e] + bias[j];
      }
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int rep = 0; rep < kReps; ++rep) {
      const int r = rep * kRowsPerRep + lane / kLanesPerRow;
      const int64_t m = m0 + wm * 32 * TM + i * 32 + r;
      if (m >= a.M || n >= a.E) continue;
      const f32x4 va = *reinterpret_cast<const f32x4*>(epi + r * kEpiStride + col8);
      const f32x4 vb = *reinterpret_cast<const f32x4*>(epi + r * kEpiStride + col8 + 4);
      if (vec_ok) {
        const f32x4 qa = p[i & 1][rep][0], qb = p[i & 1][rep][1];
        const float v[8] = {va.x + qa.x, va.y + qa.y, va.z + qa.z, va.w + qa.w,
                            vb.x + qb.x, vb.y + qb.y, vb.z + qb.z, vb.w + qb.w};
        if (kOutBf16) {
          const u32x4 o = {pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]),
                           pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7])};
          *reinterpret_cast<u32x4*>(static_cast<uint16_t*>(a.tokens) + m * a.E + n) = o;
        } else {
          f32x4* dst = reinterpret_cast<f32x4*>(static_cast<float*>(a.tokens) + m * a.E + n);
          dst[0] = f32x4{v[0], v[1], v[2], v[3]};
          dst[1] = f32x4{v[4], v[5], v[6], v[7]};
        }
      } else {
        const float v[8] = {va.x, va.y, va.z, va.w, vb.x, vb.y, vb.z, vb.w};
        const float* pos = a.pos ? a.pos + (int64_t)pid[i & 1][rep] * a.E + n : nullptr;
        for (int q = 0; q < 8 && n + q < a.E; ++q) {
          const float x = v[q] + (pos ? pos[q] : 0.f);
          if (kOutBf16) static_cast<uint16_t*>(a.tokens)[m * a.E + n + q] = (uint16_t)bf16_rne(x);
          else static_cast<float*>(a.tokens)[m * a.E + n + q] = x;
        }
      }
    }
  }
}

template <int TM, int TN, int WGM, int WGN, int STAGES, int OCC>
static hipError_t launch_cfg(const EmbedArgs& a, hipStream_t stream) {
  constexpr int BM = 32 * TM * WGM, BN = 32 * TN * WGN;
  const int64_t tiles_m = (a.M + BM - 1) / BM;
  const int64_t tiles_n = (a.E + BN - 1) / BN;
  dim3 grid((uint32_t)(tiles_m * tiles_n)), block(64 * WGM * WGN);
  if (a.out_bf16) {
    hipLaunchKernelGGL((patch_embed_kernel<TM, TN, WGM, WGN, STAGES, OCC, true>), grid, block, 0,
                       stream, a);
  } else {
    hipLaunchKernelGGL((patch_embed_kernel<TM, TN, WGM, WGN, STAGES, OCC, false>), grid, block, 0,
                       stream, a);
  }
  return hipGetLastError();
}

hipError_t launch_patch_embed(const EmbedArgs& a, hipStream_t stream) {
  // 256 x 256 tile, eight wavefronts (2 x 4) of 128 x 64, two stages of 64 KiB
  return launch_cfg<4, 2, 2, 4, 2, 1>(a, stream);
}

}  // namespace mae
