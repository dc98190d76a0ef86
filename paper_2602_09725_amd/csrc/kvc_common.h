// Internal definitions shared by the host layer and the gfx950 kernels of libkvc.
// Not part of the public interface (that is include/kvc.h).
#pragma once

#include <stdint.h>

#include "kvc.h"

#if defined(__HIPCC__)
#define KVC_HD __host__ __device__ __forceinline__
#else
#define KVC_HD inline
#endif

namespace kvc {

// Division of a 31-bit unsigned dividend by a run-time constant with one
// high multiply, one add and one shift (round-up reciprocal method):
//   s = ceil(log2 d), m = floor(2^32 * (2^s - d) / d) + 1,
//   n / d = (mulhi(m, n) + n) >> s     for 0 <= n < 2^31, 1 <= d < 2^31.
// The kernels index tokens, tile positions and cache slots with it, because
// F, TX and the block size are run-time values and a hardware integer divide
// would cost more ALU work than the dequantization itself.
struct FastDiv {
  uint32_t d, m, s;
};

inline FastDiv make_fastdiv(uint32_t d) {
  FastDiv f;
  f.d = d;
  uint32_t s = 0;
  while ((1ull << s) < d) ++s;
  f.s = s;
  f.m = (uint32_t)((((1ull << s) - d) << 32) / d) + 1u;
  return f;
}

KVC_HD uint32_t fd_mulhi(uint32_t a, uint32_t b) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __umulhi(a, b);
#else
  return (uint32_t)(((uint64_t)a * b) >> 32);
#endif
}

KVC_HD uint32_t fd_div(const FastDiv& f, uint32_t n) { return (fd_mulhi(f.m, n) + n) >> f.s; }

KVC_HD void fd_divmod(const FastDiv& f, uint32_t n, uint32_t& q, uint32_t& r) {
  q = fd_div(f, n);
  r = n - q * f.d;
}

// Derived geometry of a kvc_layout (notation of include/kvc.h).
struct Geo {
  int32_t L, H, D, C, T;
  int32_t th, tw, TX, TY;
  int32_t seg, d1;       // two-level tile: run length d2 (0: row-major retile) and runs per head
  int32_t F, LG, W, Hp;
  int32_t G;             // TX*TY tile positions per frame
  int32_t FG;            // F*G >= T token positions per chunk
  int32_t apt;           // atoms (8 consecutive elements) per token = C/8
  int32_t dtype;
  int32_t mode[2];       // quantization mode of K, V
  int64_t plane;         // Hp*W bytes
  int64_t frame_bytes;   // per chunk
  int64_t meta_floats;   // per chunk
  int64_t meta_off[2];   // float offset of the K / V block inside a chunk's meta
  FastDiv dF, dTX, dtw, dD;
  FastDiv dseg, dh2;     // two-level tile: run length, heads side by side in a tile row
};

// Intra-frame layout (Sec. 3.2.2): first element e of an atom -> (row, column) inside the token's tile.
KVC_HD void tile_pos(const Geo& g, uint32_t e, uint32_t& r, uint32_t& cc) {
  if (g.seg == 0) {
    fd_divmod(g.dtw, e, r, cc);  // row-major reshape of the H*D vector
  } else {
    uint32_t h, d, a, b, c, i;
    fd_divmod(g.dD, e, h, d);
    fd_divmod(g.dh2, h, a, b);   // head = a * h2 + b
    fd_divmod(g.dseg, d, c, i);  // element of the head = c * d2 + i
    r = a * (uint32_t)g.d1 + c;
    cc = b * (uint32_t)g.seg + i;
  }
}

// Fills `g` from a validated layout.  Returns KVC_OK or the reason the kernels
// cannot take it.
kvc_status make_geo(const kvc_layout* lo, Geo* g);

}  // namespace kvc
