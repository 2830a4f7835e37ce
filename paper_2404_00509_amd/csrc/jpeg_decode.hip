// Crop decode (Sec. 4.1 "Crop Decode"): the loader's images are JPEG files, and only the region
// that the random crop needs is decoded.  Baseline sequential DCT (ITU-T T.81), 8 bits, three
// components (JFIF YCbCr), luma sampled 1x1 or 2x2 against 1x1 chroma, tables as found in the file,
// any restart interval.  The rows of MCUs above and below the crop are not transformed, a row is
// entropy-decoded only up to the crop's right edge, and the inverse transform runs only for the
// MCUs inside it.  With one restart interval per row of MCUs (a choice of the dataset writer) the
// rows are independent and those outside the crop are never touched; in any other file the
// entropy-coded data is one chain, and a first kernel walks it (symbol lengths only) down to the
// crop's last row to find where each row starts.
//
//  * jpeg_header_kernel: one lane per file walks the marker segments and leaves a record (size,
//    sampling, restart interval, where the tables and the entropy-coded data start) plus the
//    image's height and width for the crop-parameter kernel.
//  * jpeg_tables_kernel: one wavefront per image builds what the decoder needs and leaves it in
//    the workspace: the Huffman tables (the code ranges of Annex C plus a direct table for codes
//    of up to 10 bits), the quantiser steps in zig-zag order, the crop's rows and columns of
//    MCUs, and, for files with a restart interval per row, the restart markers (16 bytes per lane
//    and step, positions ranked with a prefix sum) = the states at which the rows start.  The
//    crop record is rewritten relative to the decoded region.
//  * jpeg_scan_kernel (other files): one lane per file, two files per wavefront with their
//    tables in LDS, decodes code lengths and DC differences only, handles restart markers where
//    they come, and records the state of the bit reader and the DC predictors at the start of
//    each of the crop's rows of MCUs.
//  * jpeg_decode_kernel: one wavefront per group of four images, their tables copied into LDS;
//    the rows of MCUs that the crops touch are dealt to the lanes, one row per lane.  A lane's
//    file bytes come through its column of a ring in LDS that is fed at the start of every
//    block, where all lanes are at the same instruction; the bit buffer takes four bytes at a
//    time unless one of them is 0xFF.  Per block: DC difference, AC symbols with one table
//    look-up each (code and value bits out of the same 32-bit peek), de-quantisation on
//    insertion, fixed-point separable inverse DCT in LDS, eight 8-byte stores into the image's
//    Y, Cb or Cr plane.
//  * jpeg_colour_kernel: planes -> interleaved RGB rows of the region (repeated chroma,
//    fixed-point JFIF colour matrix), which is what the resampling kernel reads.
//
// The integer arithmetic of the inverse DCT and of the colour conversion is part of the
// definition of the output (a decoder is only specified up to that): 13-bit cosines, first pass
// kept with 3 fractional bits, both passes' inputs clamped to +-32767, floor after adding one half.
//
// Every read of file bytes is clamped into the file, every table index is masked, and every loop
// has a fixed bound, so a corrupt file gives wrong pixels or a sample flagged invalid, nothing else.
#include "mae_device.hpp"
#include "mae_kernels.hpp"

namespace mae {

constexpr int kJpegThreads = 64;  // one wavefront per workgroup
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__constant__ uint8_t kZigzag[64] = {
    0,  1,  8,  16, 9,  2,  3,  10, 17, 24, 32, 25, 18, 11, 4,  5,  12, 19, 26, 33, 40, 48,
    41, 34, 27, 20, 13, 6,  7,  14, 21, 28, 35, 42, 49, 56, 57, 50, 43, 36, 29, 22, 15, 23,
    30, 37, 44, 51, 58, 59, 52, 45, 38, 31, 39, 46, 53, 60, 61, 54, 47, 55, 62, 63};

// C(u) cos((2x+1) u pi / 16) * 2^13 rounded, C(0) = 1/sqrt 2: row x, column u
__constant__ __attribute__((aligned(16))) int16_t kBasis[64] = {
    5793, 8035,  7568,  6811,  5793,  4551,  3135,  1598,   //
    5793, 6811,  3135,  -1598, -5793, -8035, -7568, -4551,  //
    5793, 4551,  -3135, -8035, -5793, 1598,  7568,  6811,   //
    5793, 1598,  -7568, -4551, 5793,  6811,  -3135, -8035,  //
    5793, -1598, -7568, 4551,  5793,  -6811, -3135, 8035,   //
    5793, -4551, -3135, 8035,  -5793, -1598, 7568,  -6811,  //
    5793, -6811, 3135,  1598,  -5793, 8035,  -7568, 4551,   //
    5793, -8035, 7568,  -6811, 5793,  -4551, 3135,  -1598};

__device__ static inline int be16(const uint8_t* p) { return ((int)p[0] << 8) | (int)p[1]; }

// ---- header ----------------------------------------------------------------------------------------
__global__ __launch_bounds__(kJpegThreads) void jpeg_header_kernel(JpegArgs a) {
  const int b = (int)(blockIdx.x * kJpegThreads + threadIdx.x);
  if (b >= a.B) return;
  JpegRec rec;
  memset(&rec, 0, sizeof(rec));
  int H = 1, W = 1;  // what the crop-parameter kernel sees for an unusable file
  const int64_t off = a.offsets[b];
  const int64_t n = (int64_t)a.sizes[b];
  bool ok = off >= 0 && n >= 4 && off + n <= a.files_bytes;
  if (ok) {
    const uint8_t* d = a.files + off;
    ok = d[0] == 0xFF && d[1] == 0xD8;
    int64_t pos = 2;
    bool have_frame = false, have_scan = false;
    int tq[3] = {0, 0, 0}, cid[3] = {0, 0, 0};
    int q_off[4] = {0, 0, 0, 0}, dc_off[4] = {0, 0, 0, 0}, ac_off[4] = {0, 0, 0, 0};
    for (int seg = 0; seg < 64 && ok && !have_scan; ++seg) {
      if (pos + 4 > n || d[pos] != 0xFF) {
        ok = false;
        break;
      }
      const int m = d[pos + 1];
      if (m == 0xFF) {
        ++pos;
        continue;
      }
      const int len = be16(d + pos + 2);
      if (len < 2 || pos + 2 + len > n) {
        ok = false;
        break;
      }
      const uint8_t* s = d + pos + 4;
      const int body = len - 2;
      if (m == 0xDB) {
        for (int o = 0; o + 65 <= body; o += 65) {
          const int pq = s[o] >> 4, t = s[o] & 15;
          if (pq != 0 || t > 3) {
            ok = false;
            break;
          }
          q_off[t] = (int)(pos + 4 + o + 1);
        }
      } else if (m == 0xC0) {
        if (body < 15 || s[0] != 8 || s[5] != 3) {
          ok = false;
          break;
        }
        H = be16(s + 1);
        W = be16(s + 3);
        int hs[3], vs[3];
        for (int c = 0; c < 3; ++c) {
          cid[c] = s[6 + 3 * c];
          hs[c] = s[7 + 3 * c] >> 4;
          vs[c] = s[7 + 3 * c] & 15;
          tq[c] = s[8 + 3 * c] & 3;
        }
        ok = H >= 1 && W >= 1 && hs[1] == 1 && vs[1] == 1 && hs[2] == 1 && vs[2] == 1 &&
             ((hs[0] == 1 && vs[0] == 1) || (hs[0] == 2 && vs[0] == 2));
        rec.hs = hs[0];
        have_frame = true;
      } else if (m >= 0xC1 && m <= 0xCF && m != 0xC4 && m != 0xC8 && m != 0xCC) {
        ok = false;
      } else if (m == 0xC4) {
        int o = 0;
        for (int t = 0; t < 8 && o + 17 <= body; ++t) {
          const int tc = s[o] >> 4, th = s[o] & 15;
          int total = 0;
          for (int i = 0; i < 16; ++i) total += s[o + 1 + i];
          if (tc > 1 || th > 3 || total > 256 || o + 17 + total > body) {
            ok = false;
            break;
          }
          (tc ? ac_off : dc_off)[th] = (int)(pos + 4 + o + 1);
          o += 17 + total;
        }
      } else if (m == 0xDD) {
        rec.restart = body >= 2 ? be16(s) : 0;
      } else if (m == 0xDA) {
        if (!have_frame || body < 10 || s[0] != 3 || s[7] != 0 || s[8] != 63) {
          ok = false;
          break;
        }
        for (int c = 0; c < 3; ++c) {
          const int td = s[2 + 2 * c] >> 4, ta = s[2 + 2 * c] & 15;
          if (s[1 + 2 * c] != cid[c] || td > 3 || ta > 3 || !dc_off[td] || !ac_off[ta] ||
              !q_off[tq[c]])
            ok = false;
          // luma tables first, the two chroma components share theirs in files we accept
          if (c < 2) {
            rec.dc_off[c] = dc_off[td & 3];
            rec.ac_off[c] = ac_off[ta & 3];
            rec.q_off[c] = q_off[tq[c]];
          } else if (dc_off[td & 3] != rec.dc_off[1] || ac_off[ta & 3] != rec.ac_off[1] ||
                     q_off[tq[c]] != rec.q_off[1]) {
            ok = false;
          }
        }
        rec.scan_off = (int)(pos + 2 + len);
        have_scan = true;
      } else if (m == 0xD9) {
        ok = false;
      }
      pos += 2 + len;
    }
    ok = ok && have_scan;
  }
  if (ok) {
    const int mcu = 8 * rec.hs;
    rec.mcux = (W + mcu - 1) / mcu;
    rec.mcuy = (H + mcu - 1) / mcu;
    // the image has to fit its slot of the region buffer
    ok = rec.mcux * mcu <= a.slot_side && rec.mcuy * mcu <= a.slot_side;
  }
  if (!ok) {
    H = 1;
    W = 1;
  }
  rec.H = H;
  rec.W = W;
  rec.size = ok ? (int)n : 0;
  rec.valid = ok ? 1 : 0;
  a.recs[b] = rec;
  a.heights[b] = H;
  a.widths[b] = W;
  a.region_offsets[b] = (int64_t)b * a.slot_side * a.slot_side * 3;
  a.region_widths[b] = 1;
}

// ---- entropy decoding ------------------------------------------------------------------------------
// File bytes reach a lane through its column of a ring in LDS (128 bytes per lane, dword i of lane
// l at ring[i][l], so that every access of a wavefront is free of bank conflicts).  The ring is fed
// at points that all lanes pass together, the start of every block: the 32 bytes loaded at the
// previous such point are written to the ring, and the next 32 are requested if the ring has
// room.  The wait for memory is then one block of decoding long, whichever lanes asked.  A lane
// that runs dry inside a block loads and waits on the spot.
constexpr int kRingBytes = 128;
constexpr int kRingStep = 32;  // bytes per load point: two 16-byte chunks
typedef uint32_t u32x4_a8 __attribute__((ext_vector_type(4), aligned(8)));

struct BitReader {
  const uint8_t* chunks;  // 8-byte aligned start of the file's first chunk (at or before the file)
  int64_t chunks_bytes;   // bytes from there to the end of the buffer of files
  uint32_t* ring;         // this lane's column: dword i at ring[i * kJpegThreads]
  int skew;               // file position pos is byte pos + skew from `chunks`
  int n;                  // file size
  int pos;                // next byte of the file
  int have;               // the ring holds the bytes before this one (from `chunks`, multiple of 32)
  bool pending;           // `next` holds the 32 bytes at `have`, not yet in the ring
  u32x4_a8 next[2];
  uint64_t acc;  // the low nbits bits are the unread ones, oldest on top
  int nbits;
  bool ended;  // a marker was reached: zero bits from here on
};

// The 16 bytes at `base + at` (8-byte aligned) of a buffer of `bytes` bytes; bytes beyond its end
// read as zero.
__device__ static inline u32x4_a8 load_chunk(const uint8_t* base, int64_t bytes, int64_t at) {
  if (__builtin_expect(at + 16 <= bytes, 1)) return *reinterpret_cast<const u32x4_a8*>(base + at);
  // the last bytes of the buffer of files: a rolled loop, this code is inlined in many places
  uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll 1
  for (int j = 0; j < 4; ++j) {
    uint32_t v = 0;
#pragma unroll 1
    for (int i = 0; i < 4; ++i)
      if (at + 4 * j + i < bytes) v |= (uint32_t)base[at + 4 * j + i] << (8 * i);
    w[j] = v;
  }
  return u32x4_a8{w[0], w[1], w[2], w[3]};
}
__device__ static __forceinline__ void request_bytes(BitReader& r) {
  r.next[0] = load_chunk(r.chunks, r.chunks_bytes, r.have);
  r.next[1] = load_chunk(r.chunks, r.chunks_bytes, r.have + 16);
  r.pending = true;
}
__device__ static __forceinline__ void accept_bytes(BitReader& r) {
  const int i = (r.have & (kRingBytes - 1)) >> 2;  // 32 bytes never wrap: both are powers of two
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    r.ring[(i + j) * kJpegThreads] = r.next[0][j];
    r.ring[(i + 4 + j) * kJpegThreads] = r.next[1][j];
  }
  r.have += kRingStep;
  r.pending = false;
}
// The point all lanes pass together (start of a block).
__device__ static __forceinline__ void feed_ring(BitReader& r) {
  if (r.pending) accept_bytes(r);
  // room: the 32 bytes to come replace those 128 bytes back, which must have been read
  if (!r.ended && r.have - (r.pos + r.skew) <= kRingBytes - kRingStep && r.have < r.n + r.skew)
    request_bytes(r);
}
// Makes the `count` <= 4 bytes at file position pos available in the ring.
__device__ static __forceinline__ void need_bytes(BitReader& r, int pos, int count) {
  while (pos + r.skew + count > r.have) {
    if (!r.pending) request_bytes(r);
    accept_bytes(r);
  }
}
__device__ static __forceinline__ void open_reader(BitReader& r, int start) {
  r.pos = start;
  r.have = (start + r.skew) & ~(kRingStep - 1);
  r.pending = false;
  r.acc = 0;
  r.nbits = 0;
  if (!r.ended) {
    need_bytes(r, start, 4);
    request_bytes(r);
  }
}
__device__ static inline uint32_t ring_dword(const BitReader& r, int i) {
  return r.ring[(i & (kRingBytes / 4 - 1)) * kJpegThreads];
}
// Byte `pos` of the file (pos < n).
__device__ static __forceinline__ uint32_t file_byte(BitReader& r, int pos) {
  need_bytes(r, pos, 1);
  const int q = pos + r.skew;
  return (ring_dword(r, q >> 2) >> (8 * (q & 3))) & 0xFFu;
}

// Tops the bit buffer up to at least 33 bits: enough for the longest code (16) together with the
// longest value (15).  0xFF00 stands for a data byte 0xFF; any other marker ends the data of this
// row, and zero bits are supplied from there on.  Four bytes without a 0xFF among them, the usual
// case, go in at once.
// The four bytes at the read position, as they would go into the bit buffer at once; `usable`
// says whether they may (inside the file and the ring, no 0xFF among them).  Reading them early
// costs nothing: the position only moves when the buffer is topped up.
struct NextFour {
  uint32_t bits;   // first byte on top
  bool usable;
  bool in_reach;   // the four bytes are inside the file and in the ring (they may hold a 0xFF)
};
__device__ static inline NextFour next_four(const BitReader& r) {
  const int q = r.pos + r.skew;
  const uint32_t x = __builtin_amdgcn_alignbyte(ring_dword(r, (q >> 2) + 1), ring_dword(r, q >> 2),
                                                (uint32_t)(q & 3));
  const uint32_t inv = ~x;  // a byte 0xFF of x is a zero byte here
  NextFour f;
  f.bits = __builtin_bswap32(x);
  // (no short-circuit: straight-line code lets the reads above overlap the table look-up)
  f.in_reach = (int)!r.ended & (int)(r.pos + 4 <= r.n) & (int)(q + 4 <= r.have);
  f.usable = (int)f.in_reach & (int)(((inv - 0x01010101u) & ~inv & 0x80808080u) == 0u);
  return f;
}
__device__ static __forceinline__ void fill_bytewise(BitReader& r);
__device__ static __forceinline__ void fill(BitReader& r, const NextFour& f) {
  if (r.nbits > 32) return;
  if (f.usable) {
    r.acc = (r.acc << 32) | (uint64_t)f.bits;
    r.nbits += 32;
    r.pos += 4;
    return;
  }
  if (f.in_reach) {
    // a 0xFF among the four: byte by byte out of the register.  0xFF00 is a data byte 0xFF, any
    // other follower a marker; a 0xFF in the last place waits for its follower.
    bool skip = false, stop = false;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t b = (f.bits >> (24 - 8 * i)) & 0xFFu;
      const uint32_t follower = i < 3 ? (f.bits >> (16 - 8 * i)) & 0xFFu : 1u;
      const bool data = !skip && !stop && (b != 0xFFu || (i < 3 && follower == 0u));
      const bool marker = !skip && !stop && b == 0xFFu && i < 3 && follower != 0u;
      stop = stop || (!skip && b == 0xFFu && (i == 3 || follower != 0u));
      r.ended = r.ended || marker;
      const bool stuffed = data && b == 0xFFu;
      if (data) {
        r.acc = (r.acc << 8) | b;
        r.nbits += 8;
        r.pos += stuffed ? 2 : 1;
      }
      skip = stuffed;
    }
    if (r.nbits > 32) return;
  }
  fill_bytewise(r);
}
__device__ static __forceinline__ void fill(BitReader& r) {
  if (r.nbits > 32) return;
  if (!r.ended && r.pos + 4 <= r.n) need_bytes(r, r.pos, 4);
  fill(r, next_four(r));
}
__device__ static __forceinline__ void fill_bytewise(BitReader& r) {
  while (r.nbits <= 32) {
    uint32_t byte = 0;
    if (!r.ended && r.pos < r.n) {
      byte = file_byte(r, r.pos);
      if (byte == 0xFF) {
        if (r.pos + 1 < r.n && file_byte(r, r.pos + 1) == 0x00) {
          r.pos += 2;
        } else {
          r.ended = true;
          byte = 0;
        }
      } else {
        r.pos += 1;
      }
    }
    r.acc = (r.acc << 8) | byte;
    r.nbits += 8;
  }
}
// At a restart boundary: what is left of the interval (the padding of its last byte, fill bytes)
// is dropped, the marker skipped and the reader opened behind it.  Returns false when no restart
// marker follows within a few bytes.
__device__ static __forceinline__ bool restart_reader(BitReader& r) {
  int p = r.pos;  // the reader never loads a marker: it is at or behind this byte
  bool found = false;
  for (int i = 0; i < 16 && !found; ++i) {
    if (p + 1 >= r.n) break;
    if (file_byte(r, p) == 0xFFu && (file_byte(r, p + 1) & 0xF8u) == 0xD0u) found = true;
    else ++p;
  }
  r.ended = !found;
  open_reader(r, found ? p + 2 : r.pos);
  return found;
}

// The next 32 bits (after fill()), the oldest on top.
__device__ static inline uint32_t peek32(const BitReader& r) {
  return (uint32_t)(r.acc >> (r.nbits - 32));
}

// `size` >= 1 value bits that follow a code of `len` bits in `top`, as the signed value they stand
// for (T.81 F.2.2.1: the lower half of the range is the negative numbers).
__device__ static inline int value_bits(uint32_t top, int len, int size) {
  const int v = (int)((top << len) >> (32 - size));
  return v < (1 << (size - 1)) ? v - (1 << size) + 1 : v;
}

// Canonical code (Annex C) in the form the decoder wants.  With every code left-aligned in 16
// bits, the codes of one length are a range, and the ranges follow each other with the length:
// range[l].limit is the end of the range of length l + 1, so the length of the code that starts
// the 16 bits x is one more than the number of limits that x has reached.  range[l].delta turns
// the leading l + 1 bits into the index of the symbol.
struct CodeRange {
  uint32_t limit;
  int32_t delta;
};
struct alignas(16) HuffDc {
  CodeRange range[16];
  uint8_t symbols[16];  // categories 0..11
};
constexpr int kFastBits = 10;
struct alignas(16) HuffAc {
  CodeRange range[16];
  uint8_t symbols[256];
  uint16_t fast[1 << kFastBits];  // per 10-bit prefix: length << 8 | symbol, 0 = a longer code
};

// The code that starts the 16 bits x, looking at lengths above kFrom only: index (length - 1) of
// its length, 16 = none, and through `index` the position of its symbol in the table.
template <int kFrom>
__device__ static inline int find_code(const CodeRange* range, uint32_t x, int& index) {
  int len = kFrom, delta = range[kFrom].delta;
#pragma unroll
  for (int l = kFrom; l < 16; ++l) {
    if (x >= range[l].limit) {
      len = l + 1;
      delta = l + 1 < 16 ? range[l + 1].delta : 0;
    }
  }
  index = delta + (int)(x >> (15 - min(len, 15)));
  return len;
}

// Sum over eight 16-bit values times one row of the basis, two products per instruction; the
// sums stay below 2^31 (the row's absolute values add up to 43284, the values are at most 32767).
typedef short s16x2 __attribute__((ext_vector_type(2)));
__device__ static inline int basis_dot(const s16x2 v[4], int row) {
  const s16x2* basis = reinterpret_cast<const s16x2*>(kBasis) + row * 4;
  int acc = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) acc = __builtin_amdgcn_sdot2(v[i], basis[i], acc, false);
  return acc;
}

// One row of the second pass of the inverse DCT below.
__device__ static inline void idct_row(const int16_t* coef, int y, int out[8]) {
  s16x2 t[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
    t[i] = s16x2{coef[(y * 8 + 2 * i) * kJpegThreads], coef[(y * 8 + 2 * i + 1) * kJpegThreads]};
#pragma unroll
  for (int x = 0; x < 8; ++x)
    out[x] = min(max(((basis_dot(t, x) + (1 << 16)) >> 17) + 128, 0), 255);
}

// Dequantised coefficients (natural order, 16-bit) -> 64 samples, in two passes.  The coefficients
// live in LDS with the lane as the fastest index (element k of this lane at coef[k * 64]): the
// lanes of a wavefront then touch neighbouring addresses instead of one bank.  The first pass
// overwrites each column with its transform (the clamped values fit 16 bits); the second gives
// the samples row by row.
__device__ static inline void idct_columns(int16_t* coef) {
  for (int u = 0; u < 8; ++u) {
    s16x2 c[4];
    int t[8];
#pragma unroll
    for (int i = 0; i < 4; ++i)
      c[i] = s16x2{coef[(2 * i * 8 + u) * kJpegThreads], coef[((2 * i + 1) * 8 + u) * kJpegThreads]};
#pragma unroll
    for (int y = 0; y < 8; ++y)
      t[y] = min(max((basis_dot(c, y) + (1 << 10)) >> 11, -32767), 32767);
#pragma unroll
    for (int y = 0; y < 8; ++y) coef[(y * 8 + u) * kJpegThreads] = (int16_t)t[y];
  }
}

__device__ static inline uint32_t ycc_to_rgbx(int y, int cb, int cr) {
  const int b = cb - 128, r = cr - 128;
  const int R = min(max(y + ((91881 * r + 32768) >> 16), 0), 255);
  const int G = min(max(y - ((22554 * b + 46802 * r + 32768) >> 16), 0), 255);
  const int B = min(max(y + ((116130 * b + 32768) >> 16), 0), 255);
  return (uint32_t)R | ((uint32_t)G << 8) | ((uint32_t)B << 16);
}

// Images per workgroup of the decode kernel (template parameter kGroup: 4, 2 or 1): their rows of
// MCUs share the 64 lanes.  A lane gets at most kGroup rows (an image has at most 64).

// What the wavefront keeps per image of its group.
struct JpegImage {
  HuffDc dc[2];  // luma, chroma
  HuffAc ac[2];
  uint16_t qz[2][64];  // per zig-zag position: natural position << 8 | quantiser step
  int my0, mx0, mx1, nrows, region_w, hs, size, scan_off, live;
  int restart, mcux;  // restart interval in MCUs (0 = none), MCUs per row of the image
  int64_t origin, region_off;
};

// What the table kernel hands to the decode kernel per image (through the workspace).
struct alignas(16) JpegPrepared {
  JpegImage im;
};
static_assert(sizeof(JpegPrepared) % 16 == 0, "copied in 16-byte pieces");

// Where the entropy-coded data of one of the crop's rows of MCUs starts: the bit reader's state
// and the DC predictors at that point (workspace; max_rows of them per image).
struct alignas(16) RowState {
  int32_t pos;        // next byte of the file that goes into the bit buffer; -1 = not known
  int32_t nbits;      // unread bits in acc
  uint64_t acc;
  int16_t pred[3];    // Y, Cb, Cr
  uint16_t rst_left;  // MCUs from here to the next restart marker (unused without an interval)
  int32_t pad;
};
static_assert(sizeof(RowState) == 32, "32 bytes per row");

template <int kGroup>
struct JpegLds {
  JpegPrepared img[kGroup];
  // one block per lane, the lane is the fastest index; row 64 takes the stores of skipped blocks
  int16_t coef[65][kJpegThreads];
  uint32_t ring[kRingBytes / 4][kJpegThreads];  // file bytes on their way to the lanes
};

// Tables, crop geometry and restart-marker positions of image b into slot `im` (whole wavefront).
__device__ static void jpeg_prepare_image(const JpegArgs& a, int b, JpegImage& im) {
  const int lane = threadIdx.x;
  const JpegRec rec = a.recs[b];
  CropRec* crop = reinterpret_cast<CropRec*>(a.workspace + kWorkspaceHeader) + b;
  CropRec cr = *crop;
  RowState* states = reinterpret_cast<RowState*>(a.row_states) + (int64_t)b * a.max_rows;
  __syncthreads();  // everybody has read the record before lane 0 rewrites it
  if (a.whole_image) {
    // index run: the "crop" is the whole image, and every row of the index gets a defined value
    // whatever becomes of the file
    cr.top = 0;
    cr.left = 0;
    cr.ch = rec.H;
    cr.cw = rec.W;
    cr.flip = 0;
    cr.valid = 1;
    RowState none;
    none.pos = -1;
    none.nbits = 0;
    none.acc = 0;
    none.pred[0] = none.pred[1] = none.pred[2] = 0;
    none.rst_left = 0;
    none.pad = 0;
    for (int i = lane; i < a.max_rows; i += kJpegThreads) states[i] = none;
    __syncthreads();
  }
  if (!rec.valid) {
    if (lane == 0) {
      crop->valid = 0;
      if (a.crop_out) a.crop_out[(int64_t)b * 6 + 5] = 0;
      im.live = 0;
      im.nrows = 0;
    }
    return;
  }
  if (!cr.valid) {
    if (lane == 0) {
      im.live = 0;
      im.nrows = 0;
    }
    return;
  }
  const uint8_t* d = a.files + a.offsets[b];
  const int n = rec.size;
  const int mcu = 8 * rec.hs;
  // rows and columns of MCUs that the crop touches
  const int my0 = cr.top / mcu, my1 = min((cr.top + cr.ch - 1) / mcu, rec.mcuy - 1);
  const int mx0 = cr.left / mcu, mx1 = min((cr.left + cr.cw - 1) / mcu, rec.mcux - 1);
  if (lane == 0) {
    im.my0 = my0;
    im.mx0 = mx0;
    im.mx1 = mx1;
    im.nrows = my1 - my0 + 1;
    im.region_w = (mx1 - mx0 + 1) * mcu;
    im.hs = rec.hs;
    im.size = n;
    im.scan_off = rec.scan_off;
    im.restart = rec.restart;
    im.mcux = rec.mcux;
    im.live = 1;
    im.origin = a.offsets[b];
    im.region_off = a.region_offsets[b];
    // region geometry for the colour kernel and the resampling kernel
    a.region_widths[b] = (mx1 - mx0 + 1) * mcu;
    a.recs[b].region_h = (my1 - my0 + 1) * mcu;
    crop->top = cr.top - my0 * mcu;
    crop->left = cr.left - mx0 * mcu;
  }

  // tables: symbols and quantiser steps by all lanes
  for (int t = 0; t < 2; ++t) {
    if (lane < 16) im.dc[t].symbols[lane] = d[min(rec.dc_off[t] + 16 + lane, n - 1)];
    for (int i = lane; i < 256; i += kJpegThreads)
      im.ac[t].symbols[i] = d[min(rec.ac_off[t] + 16 + i, n - 1)];
  }
  for (int i = lane; i < 128; i += kJpegThreads)
    im.qz[i >> 6][i & 63] =
        (uint16_t)(((int)kZigzag[i & 63] << 8) | d[min(rec.q_off[i >> 6] + (i & 63), n - 1)]);
  {  // code ranges: lane = table * 16 + (length - 1); the counts of the shorter lengths come from
     // the lanes before it (first code of a length = twice the end of the length before)
    const int tt = lane >> 4, len = lane & 15;
    const int t = tt & 1;
    const bool is_ac = tt >= 2;
    const int count = d[min((is_ac ? rec.ac_off[t] : rec.dc_off[t]) + len, n - 1)];
    int code = 0, index = 0;
    for (int j = 0; j < 15; ++j) {
      const int cj = __shfl(count, (tt << 4) + j);
      if (j < len) {
        code += cj << (len - j);
        index += cj;
      }
    }
    CodeRange* range = is_ac ? im.ac[t].range : im.dc[t].range;
    range[len].delta = index - code;
    range[len].limit = (uint32_t)(code + count) << (15 - len);
  }
  __syncthreads();
  for (int t = 0; t < 2; ++t) {
    HuffAc& h = im.ac[t];
    // direct table: the code that starts a 10-bit prefix is the one of the first length whose
    // range the prefix (followed by zeros) falls into; none = a longer code
    for (int i = lane; i < (1 << kFastBits); i += kJpegThreads) {
      const uint32_t x = (uint32_t)i << (16 - kFastBits);
      int len = kFastBits;
      for (int l = kFastBits - 1; l >= 0; --l)
        if (x < h.range[l].limit) len = l;
      uint16_t e = 0;
      if (len < kFastBits)
        e = (uint16_t)(((len + 1) << 8) |
                       h.symbols[(h.range[len].delta + (int)(x >> (15 - len))) & 255]);
      h.fast[i] = e;
    }
  }

  // the rows' states: unknown until found below or by the scan kernel
  {
    RowState none;
    none.pos = -1;
    none.nbits = 0;
    none.acc = 0;
    none.pred[0] = none.pred[1] = none.pred[2] = 0;
    none.rst_left = 0;
    none.pad = 0;
    const int nrows = min(my1 - my0 + 1, a.max_rows);
    for (int i = lane; i < nrows; i += kJpegThreads) states[i] = none;
  }
  __syncthreads();  // (these stores are complete before a row's real state is written)
  if (a.row_index) {
    // the states come from the caller's index of the file (row r of the file at entry r).  It is
    // the caller's memory: an entry that does not point into the entropy-coded data or whose bit
    // count is impossible is left unknown, which flags the sample in the decode kernel.
    const RowState* index = reinterpret_cast<const RowState*>(a.row_index) + (int64_t)b * a.max_rows;
    const int nrows = min(my1 - my0 + 1, a.max_rows);
    for (int i = lane; i < nrows; i += kJpegThreads) {
      if (my0 + i >= a.max_rows) continue;
      RowState st = index[my0 + i];
      const bool ok = st.pos >= rec.scan_off && st.pos <= n && st.nbits >= 0 && st.nbits <= 64;
      if (ok) states[i] = st;
    }
    return;
  }
  if (rec.restart != rec.mcux) return;  // rows not independent: the scan kernel finds the states

  // restart markers: marker m (0-based) ends MCU row m; row r starts after marker r - 1.  The
  // file is scanned in aligned 16-byte pieces of the buffer, one per lane and step, the next
  // step's pieces loaded while this step's are examined.
  RowState start;
  start.nbits = 0;
  start.acc = 0;
  start.pred[0] = start.pred[1] = start.pred[2] = 0;
  start.rst_left = (uint16_t)rec.restart;
  start.pad = 0;
  const int64_t origin = a.offsets[b];
  const int64_t first = (origin + rec.scan_off) & ~(int64_t)15;
  const int64_t last = origin + n - 1;  // a marker starts before this byte
  int seen = 0;                         // markers before the current step
  u32x4_a8 cur = load_chunk(a.files, a.files_bytes, first + lane * 16);
  for (int64_t base = first; base < last && seen <= my1; base += kJpegThreads * 16) {
    const int64_t at = base + lane * 16;
    const u32x4_a8 next = load_chunk(a.files, a.files_bytes, at + kJpegThreads * 16);
    // the byte after this piece: the first of the next lane's, or of the next step's
    uint32_t follow = (uint32_t)__shfl_down((int)(cur.x & 0xFFu), 1);
    const uint32_t wrap = (uint32_t)__shfl((int)(next.x & 0xFFu), 0);
    if (lane == kJpegThreads - 1) follow = wrap;
    const int p0 = (int)(at - origin);  // file position of the piece (negative before the file)
    uint32_t mask = 0;                  // bit i: a restart marker starts at byte p0 + i
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const uint32_t b0 = (cur[i >> 2] >> (8 * (i & 3))) & 0xFFu;
      const uint32_t b1 = i < 15 ? (cur[(i + 1) >> 2] >> (8 * ((i + 1) & 3))) & 0xFFu : follow;
      const int pp = p0 + i;
      if (pp >= rec.scan_off && pp + 1 < n && b0 == 0xFFu && (b1 & 0xF8u) == 0xD0u)
        mask |= 1u << i;
    }
    const int cnt = __popc(mask);
    // rank of this lane's first marker among the wavefront's: counts of the lanes before it
    int before = cnt;
    for (int off = 1; off < kWave; off <<= 1) {
      const int t = __shfl_up(before, off);
      if (lane >= off) before += t;
    }
    const int total = __shfl(before, kWave - 1);
    before -= cnt;
    for (int i = 0; i < 16; ++i) {
      if (!((mask >> i) & 1u)) continue;
      // the row that starts after this marker
      const int row = seen + before + __popc(mask & ((1u << i) - 1u)) + 1;
      if (row >= my0 && row <= my1 && row - my0 < a.max_rows) {
        start.pos = p0 + i + 2;
        states[row - my0] = start;
      }
    }
    seen += total;
    cur = next;
  }
  if (my0 == 0 && lane == 0) {
    start.pos = rec.scan_off;
    states[0] = start;
  }
}

// One wavefront per image: tables, crop geometry, row starts -> workspace.  Many of these fit a
// CU at once, which hides the latency of the scattered header reads and of the marker scan.
__global__ __launch_bounds__(kJpegThreads) void jpeg_tables_kernel(JpegArgs a) {
  __shared__ JpegPrepared p;
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  const int b = (int)blockIdx.x;
  for (int i = threadIdx.x; i < (int)(sizeof(JpegPrepared) / 16); i += kJpegThreads)
    reinterpret_cast<u32x4*>(&p)[i] = u32x4{0u, 0u, 0u, 0u};
  __syncthreads();
  jpeg_prepare_image(a, b, p.im);
  __syncthreads();
  u32x4* dst = reinterpret_cast<u32x4*>(a.prepared + (size_t)b * sizeof(JpegPrepared));
  for (int i = threadIdx.x; i < (int)(sizeof(JpegPrepared) / 16); i += kJpegThreads)
    dst[i] = reinterpret_cast<const u32x4*>(&p)[i];
}

// DC difference of the next block (T.81 F.2.2.1).  Returns false for a code that does not exist
// or a category that 8-bit data does not have (the difference is then 0).
__device__ static __forceinline__ bool decode_dc(BitReader& r, const HuffDc& h, int& diff) {
  fill(r);
  const uint32_t top = peek32(r);
  const uint32_t x = top >> 16;
  int index;
  int len = find_code<0>(h.range, x, index);
  int sym = 16;
  if (len < 16) sym = h.symbols[index & 15];
  const bool ok = sym <= 11;
  if (!ok) {
    sym = 0;
    len = -1;
  }
  diff = sym ? value_bits(top, len + 1, sym) : 0;
  r.nbits -= len + 1 + sym;
  return ok;
}

// AC coefficients of a block (F.2.2.2): a symbol is a run of zeros << 4 | size of the value.  The
// usual step -- short code, and the next four bytes ready if the buffer has to be topped up -- is
// straight-line code; everything else takes the one branch.  kStore: de-quantised values go to
// the lane's column of `coef` (natural order; row 64 takes what is skipped); otherwise only the
// symbols' lengths are followed.  Returns false for a code that does not exist or a run past the
// end of the block.
template <bool kStore>
__device__ static __forceinline__ bool decode_ac(BitReader& r, const HuffAc& h, const uint16_t* qz,
                                        int16_t* coef, bool want) {
  bool ok = true;
  fill(r);
  for (int k = 1; k < 64;) {
    const NextFour ahead = next_four(r);  // in flight while the symbol is looked up
    const uint32_t top = peek32(r);
    const int e = h.fast[top >> (32 - kFastBits)];
    int len1 = e >> 8, rs = e & 255;
    const bool top_up = r.nbits - (len1 + (rs & 15)) <= 32;
    if ((int)(e == 0) | ((int)top_up & (int)!ahead.usable)) {
      if (!e) {
        int index;
        const int len = find_code<kFastBits>(h.range, top >> 16, index);
        rs = h.symbols[index & 255];
        len1 = len + 1;
        if (len == 16) {  // no such code: flag the sample and end the block
          ok = false;
          rs = 0;
          len1 = 0;
        }
      }
      r.nbits -= len1 + (rs & 15);
      fill(r, ahead);
    } else {
      r.nbits -= len1 + (rs & 15) - (top_up ? 32 : 0);
      r.acc = top_up ? (r.acc << 32) | (uint64_t)ahead.bits : r.acc;
      r.pos += top_up ? 4 : 0;
    }
    const int run = rs >> 4, size = rs & 15;
    // size 0: sixteen zeros (run 15) or the end of the block
    k += size ? run : (run == 15 ? 16 : 64);
    ok = ok && !(size != 0 && k > 63);
    if (kStore) {  // no branch: what is not to be stored goes to the spare row 64
      const bool store = size != 0 && k <= 63;
      const int zq = qz[k & 63];
      coef[(store && want ? zq >> 8 : 64) * kJpegThreads] = (int16_t)min(
          max(value_bits(top, len1, size ? size : 1) * (zq & 255), -32767), 32767);
    }
    k += size ? 1 : 0;
  }
  return ok;
}

__device__ static __forceinline__ void reader_for(BitReader& r, const JpegArgs& a, const JpegImage& im,
                                         uint32_t* ring) {
  r.skew = (int)(im.origin & 7);
  r.chunks = a.files + (im.origin - r.skew);
  r.chunks_bytes = a.files_bytes - (im.origin - r.skew);
  r.ring = ring;
  r.n = im.size;
}
// Opens the reader in the state recorded for a row.
__device__ static __forceinline__ void open_at(BitReader& r, const RowState& st) {
  open_reader(r, st.pos);
  r.acc = st.acc;
  r.nbits = st.nbits;
}

// ---- files whose rows of MCUs are not independent: where does each of the crop's rows start? ----
// One lane per file, kScanImages files per wavefront (two: a batch then gives every SIMD two
// wavefronts to switch between, and a lane rarely waits for the other's longer block).  The lane walks
// the entropy-coded data from its start: per block the DC difference (the predictors run through
// the whole interval) and the lengths of the AC symbols; at every restart boundary the marker is
// skipped and the predictors cleared.  At the first MCU of each of the crop's rows the reader's
// state goes to the workspace.  The walk ends with the crop's last row.
constexpr int kScanImages = 2;
struct JpegScanLds {
  JpegPrepared img[kScanImages];
  uint32_t ring[kRingBytes / 4][kJpegThreads];
};

__global__ __launch_bounds__(kJpegThreads) void jpeg_scan_kernel(JpegArgs a) {
  __shared__ JpegScanLds s;
  const int lane = threadIdx.x;
  const int b0 = (int)blockIdx.x * kScanImages;
  const int nimg = min(kScanImages, a.B - b0);
  bool need = false;
  if (lane < nimg) {
    const JpegRec rec = a.recs[b0 + lane];
    const CropRec cr = reinterpret_cast<const CropRec*>(a.workspace + kWorkspaceHeader)[b0 + lane];
    need = rec.valid && (cr.valid || a.whole_image) && rec.restart != rec.mcux && !a.row_index;
  }
  if (__builtin_amdgcn_ballot_w64(need) == 0) return;  // every file here has independent rows
  {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const u32x4* src = reinterpret_cast<const u32x4*>(a.prepared + (size_t)b0 * sizeof(JpegPrepared));
    u32x4* dst = reinterpret_cast<u32x4*>(&s.img[0]);
    const int n16 = nimg * (int)(sizeof(JpegPrepared) / 16);
    for (int i = lane; i < n16; i += kJpegThreads) dst[i] = src[i];
  }
  __syncthreads();
  if (!need) return;  // (no barrier below)

  const JpegImage& im = s.img[lane].im;
  const int b = b0 + lane;
  RowState* states = reinterpret_cast<RowState*>(a.row_states) + (int64_t)b * a.max_rows;
  BitReader r;
  reader_for(r, a, im, &s.ring[0][lane]);
  r.ended = false;
  open_reader(r, im.scan_off);
  const int nblk = im.hs * im.hs, per_mcu = nblk + 2;
  const int rows = im.my0 + im.nrows;  // rows of MCUs down to the crop's last
  const int mcux = im.mcux, interval = im.restart;
  int pred[3] = {0, 0, 0};
  int rst_left = interval;
  bool bad = false;
  // one block per iteration (every lane is at the start of a block here); the bounds do not
  // depend on the data
  int row = 0, mx = 0, blk = 0;
  const int64_t blocks = (int64_t)rows * mcux * per_mcu;
  for (int64_t it = 0; it < blocks; ++it) {
    if (blk == 0) {  // first block of an MCU
      if (interval) {
        if (rst_left == 0) {
          bad = bad || !restart_reader(r);
          pred[0] = pred[1] = pred[2] = 0;
          rst_left = interval;
        }
      }
      if (mx == 0 && row >= im.my0 && row - im.my0 < a.max_rows) {
        RowState st;
        st.pos = r.pos;
        st.nbits = r.nbits;
        st.acc = r.acc;
        st.pred[0] = (int16_t)pred[0];
        st.pred[1] = (int16_t)pred[1];
        st.pred[2] = (int16_t)pred[2];
        st.rst_left = (uint16_t)rst_left;
        st.pad = 0;
        if (r.ended) st.pos = -1;  // the data ended before this row
        states[row - im.my0] = st;
      }
      rst_left -= interval ? 1 : 0;
    }
    const int c = blk < nblk ? 0 : blk - nblk + 1;  // component
    const int t = c ? 1 : 0;                        // table set
    feed_ring(r);
    int diff;
    bad = bad || !decode_dc(r, im.dc[t], diff);
    pred[0] += c == 0 ? diff : 0;
    pred[1] += c == 1 ? diff : 0;
    pred[2] += c == 2 ? diff : 0;
    bad = bad || !decode_ac<false>(r, im.ac[t], nullptr, nullptr, false);
    if (++blk == per_mcu) {
      blk = 0;
      if (++mx == mcux) {
        mx = 0;
        ++row;
      }
    }
  }
  if (bad) {
    reinterpret_cast<CropRec*>(a.workspace + kWorkspaceHeader)[b].valid = 0;
    if (a.crop_out) a.crop_out[(int64_t)b * 6 + 5] = 0;
  }
}

template <int kGroup>
__global__ __launch_bounds__(kJpegThreads) void jpeg_decode_kernel(JpegArgs a) {
  __shared__ JpegLds<kGroup> s;
  const int lane = threadIdx.x;
  const int b0 = (int)blockIdx.x * kGroup;
  const int nimg = min(kGroup, a.B - b0);
  {  // the images' tables, as the table kernel left them
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const u32x4* src = reinterpret_cast<const u32x4*>(a.prepared + (size_t)b0 * sizeof(JpegPrepared));
    u32x4* dst = reinterpret_cast<u32x4*>(&s.img[0]);
    const int n16 = nimg * (int)(sizeof(JpegPrepared) / 16);
    for (int i = lane; i < n16; i += kJpegThreads) dst[i] = src[i];
  }
  __syncthreads();

  // the rows of MCUs of the group's images, one after the other, are dealt to the lanes
  int first_task[kGroup + 1];
  first_task[0] = 0;
#pragma unroll
  for (int i = 0; i < kGroup; ++i)
    first_task[i + 1] = first_task[i] + (i < nimg ? min(s.img[i].im.nrows, a.max_rows) : 0);
  const int ntasks = first_task[kGroup];
  int16_t* coef = &s.coef[0][lane];  // element k at coef[k * 64]
#pragma unroll 1
  for (int task = lane; task < ntasks; task += kJpegThreads) {
    int slot = 0, slot_first = 0;
#pragma unroll
    for (int i = 1; i < kGroup; ++i) {
      if (task >= first_task[i]) {
        slot = i;
        slot_first = first_task[i];
      }
    }
    const int row = task - slot_first;  // row of MCUs inside the crop's range
    const JpegImage& im = s.img[slot].im;
    const int b = b0 + slot;
    const RowState st = (reinterpret_cast<const RowState*>(a.row_states) +
                         (int64_t)b * a.max_rows)[row];
    const int hs = im.hs, mcu = 8 * hs;
    const int mx0 = im.mx0, mx1 = im.mx1, region_w = im.region_w;
    // the image's slot of the plane buffer: Y (region_w wide), then Cb and Cr (region_w / hs wide)
    const int chroma_w = region_w / hs;
    uint8_t* plane_y = a.planes + im.region_off;
    uint8_t* plane_cb = plane_y + (int64_t)im.nrows * mcu * region_w;
    uint8_t* plane_cr = plane_cb + (int64_t)im.nrows * 8 * chroma_w;
    const bool found = st.pos >= im.scan_off && st.pos <= im.size;
    BitReader r;
    reader_for(r, a, im, &s.ring[0][lane]);
    r.ended = !found;  // start unknown: zero bits, and the sample is flagged below
    if (found) {
      open_at(r, st);
    } else {
      open_reader(r, im.scan_off);
    }
    int pred_y = st.pred[0], pred_cb = st.pred[1], pred_cr = st.pred[2];
    const int interval = im.restart;
    int rst_left = st.rst_left;
    const int nblk = hs * hs;  // luma blocks per MCU
    bool bad = !found;
    for (int mx = 0; mx <= mx1; ++mx) {
      if (interval) {  // a restart boundary inside the row
        if (mx > 0 && rst_left == 0) {
          bad = bad || !restart_reader(r);
          pred_y = pred_cb = pred_cr = 0;
          rst_left = interval;
        }
        --rst_left;
      }
      const bool want = mx >= mx0;
      const int x0 = (mx - mx0) * mcu, y0 = row * mcu;
      for (int blk = 0; blk < nblk + 2; ++blk) {
        const int c = blk < nblk ? 0 : blk - nblk + 1;  // component
        const int t = c ? 1 : 0;                        // table set
        if (want)
          for (int i = 0; i < 64; ++i) coef[i * kJpegThreads] = 0;
        feed_ring(r);
        int diff;
        bad = bad || !decode_dc(r, im.dc[t], diff);
        pred_y += c == 0 ? diff : 0;
        pred_cb += c == 1 ? diff : 0;
        pred_cr += c == 2 ? diff : 0;
        const int dcv = c == 0 ? pred_y : (c == 1 ? pred_cb : pred_cr);
        const uint16_t* qz = im.qz[t];
        if (want) coef[0] = (int16_t)min(max(dcv * (int)(qz[0] & 255), -32767), 32767);
        bad = bad || !decode_ac<true>(r, im.ac[t], qz, coef, want);
        if (!want) continue;
        idct_columns(coef);
        // the block's rows, eight samples = one 8-byte store each (rows of every plane start on
        // 8-byte boundaries: widths are multiples of 8)
        uint8_t* out;
        int pitch;
        if (c == 0) {
          pitch = region_w;
          out = plane_y + (int64_t)(y0 + (blk / hs) * 8) * region_w + x0 + (blk % hs) * 8;
        } else {
          pitch = chroma_w;
          out = (c == 1 ? plane_cb : plane_cr) + (int64_t)row * 8 * chroma_w + (mx - mx0) * 8;
        }
        for (int y = 0; y < 8; ++y) {
          int v[8];
          idct_row(coef, y, v);
          const uint32_t lo = (uint32_t)v[0] | ((uint32_t)v[1] << 8) | ((uint32_t)v[2] << 16) |
                              ((uint32_t)v[3] << 24);
          const uint32_t hi = (uint32_t)v[4] | ((uint32_t)v[5] << 8) | ((uint32_t)v[6] << 16) |
                              ((uint32_t)v[7] << 24);
          *reinterpret_cast<u32x2*>(out + (int64_t)y * pitch) = u32x2{lo, hi};
        }
      }
    }
    if (bad) {
      reinterpret_cast<CropRec*>(a.workspace + kWorkspaceHeader)[b].valid = 0;
      if (a.crop_out) a.crop_out[(int64_t)b * 6 + 5] = 0;
    }
  }
}

size_t jpeg_prepared_bytes() { return sizeof(JpegPrepared); }
size_t jpeg_row_state_bytes() { return sizeof(RowState); }

hipError_t launch_jpeg_header(const JpegArgs& a, hipStream_t stream) {
  dim3 grid((uint32_t)((a.B + kJpegThreads - 1) / kJpegThreads)), block(kJpegThreads);
  hipLaunchKernelGGL(jpeg_header_kernel, grid, block, 0, stream, a);
  return hipGetLastError();
}

// Planes -> interleaved RGB, the region's rows as the resampling kernel reads them.  One workgroup
// per image and band of rows, four pixels per thread and step; chroma is repeated over hs x hs
// pixels (T.81 A.1.1 leaves upsampling open; repetition is this library's definition).
constexpr int kColourThreads = 256;
constexpr int kColourBand = 32;
__global__ __launch_bounds__(kColourThreads) void jpeg_colour_kernel(JpegArgs a, int bands) {
  const int b = (int)(blockIdx.x / (uint32_t)bands);
  const int band = (int)(blockIdx.x - (uint32_t)b * (uint32_t)bands);
  const JpegRec rec = a.recs[b];
  const int first = band * kColourBand;
  if (!rec.valid || first >= rec.region_h) return;
  const int region_w = a.region_widths[b], hs = rec.hs;
  const int chroma_w = region_w / hs;
  const int64_t off = a.region_offsets[b];
  const uint8_t* plane_y = a.planes + off;
  const uint8_t* plane_cb = plane_y + (int64_t)rec.region_h * region_w;
  const uint8_t* plane_cr = plane_cb + (int64_t)(rec.region_h / hs) * chroma_w;
  uint8_t* region = a.regions + off;
  const int ng = region_w >> 2;
  const int rows = min(kColourBand, rec.region_h - first);
  for (int i = (int)threadIdx.x; i < rows * ng; i += kColourThreads) {
    const int y = first + i / ng, g = i % ng;
    const uint32_t yy = *reinterpret_cast<const uint32_t*>(plane_y + (int64_t)y * region_w + 4 * g);
    uint32_t cb, cr;  // one byte per pixel
    if (hs == 2) {
      const int64_t o = (int64_t)(y >> 1) * chroma_w + 2 * g;
      const uint32_t b2 = *reinterpret_cast<const uint16_t*>(plane_cb + o);
      const uint32_t r2 = *reinterpret_cast<const uint16_t*>(plane_cr + o);
      cb = (b2 & 0xFFu) * 0x0101u | (b2 >> 8) * 0x01010000u;
      cr = (r2 & 0xFFu) * 0x0101u | (r2 >> 8) * 0x01010000u;
    } else {
      const int64_t o = (int64_t)y * chroma_w + 4 * g;
      cb = *reinterpret_cast<const uint32_t*>(plane_cb + o);
      cr = *reinterpret_cast<const uint32_t*>(plane_cr + o);
    }
    uint32_t px[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
      px[j] = ycc_to_rgbx((int)((yy >> (8 * j)) & 0xFFu), (int)((cb >> (8 * j)) & 0xFFu),
                          (int)((cr >> (8 * j)) & 0xFFu));
    // rows of the region start on 4-byte boundaries (their width is a multiple of 8 pixels)
    uint32_t* dst = reinterpret_cast<uint32_t*>(region + ((int64_t)y * region_w + 4 * g) * 3);
    dst[0] = px[0] | (px[1] << 24);
    dst[1] = (px[1] >> 8) | (px[2] << 16);
    dst[2] = (px[2] >> 16) | (px[3] << 8);
  }
}

hipError_t launch_jpeg_index(const JpegArgs& a, hipStream_t stream) {
  dim3 block(kJpegThreads);
  hipLaunchKernelGGL(jpeg_tables_kernel, dim3((uint32_t)a.B), block, 0, stream, a);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return err;
  hipLaunchKernelGGL(jpeg_scan_kernel, dim3((uint32_t)((a.B + kScanImages - 1) / kScanImages)),
                     block, 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_jpeg_decode(const JpegArgs& a, hipStream_t stream) {
  dim3 block(kJpegThreads);
  hipLaunchKernelGGL(jpeg_tables_kernel, dim3((uint32_t)a.B), block, 0, stream, a);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return err;
  // files whose rows are not independent (its wavefronts leave at once where there are none)
  hipLaunchKernelGGL(jpeg_scan_kernel, dim3((uint32_t)((a.B + kScanImages - 1) / kScanImages)),
                     block, 0, stream, a);
  err = hipGetLastError();
  if (err != hipSuccess) return err;
  // as many images per wavefront as fill its lanes with rows of MCUs: an image of the largest
  // side allowed has slot_side / 16 rows of them when its luma is sampled 2x2
  const int rows = a.slot_side / 16;
  const uint32_t B = (uint32_t)a.B;
  if (rows <= 16)
    hipLaunchKernelGGL(jpeg_decode_kernel<4>, dim3((B + 3) / 4), block, 0, stream, a);
  else if (rows <= 32)
    hipLaunchKernelGGL(jpeg_decode_kernel<2>, dim3((B + 1) / 2), block, 0, stream, a);
  else
    hipLaunchKernelGGL(jpeg_decode_kernel<1>, dim3(B), block, 0, stream, a);
  err = hipGetLastError();
  if (err != hipSuccess) return err;
  const int bands = (a.slot_side + kColourBand - 1) / kColourBand;
  hipLaunchKernelGGL(jpeg_colour_kernel, dim3((uint32_t)a.B * (uint32_t)bands),
                     dim3(kColourThreads), 0, stream, a, bands);
  return hipGetLastError();
}

}  // namespace mae
