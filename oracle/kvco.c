/*
 * kvco.c -- CPU oracle (test infrastructure only, see kvco.h).
 *
 * Every function is the definition written out: one element at a time, one
 * index formula, no blocking or fusion.  Floating point is IEEE binary32 with
 * round-to-nearest-even throughout (the quantizer's precision), no contraction
 * (build with -ffp-contract=off -fno-fast-math).
 */
#include "kvco.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---------------------------------------------------------------- geometry */

static int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

int kvco_check(const kvco_layout* lo) {
  if (!lo) return 1;
  if (lo->L < 1 || lo->H < 1 || lo->D < 1 || lo->T < 1) return 1;
  if (lo->th < 1 || lo->tw < 1 || lo->TX < 1 || lo->TY < 1) return 1;
  if ((int64_t)lo->th * lo->tw != (int64_t)lo->H * lo->D) return 1; /* Sec. 3.2.2: a tile is a reshape of the H*D vector */
  if (lo->seg < 0) return 1;
  if (lo->seg > 0) {
    /* Sec. 3.2.2: head_dim = d1 * d2 and head_num = h1 * h2 with tile = (h1*d1, h2*d2) */
    const int64_t d2 = lo->seg;
    if (lo->D % d2 != 0 || lo->tw % d2 != 0) return 1;
    if (lo->H % (lo->tw / d2) != 0) return 1;
    if ((int64_t)(lo->H / (lo->tw / d2)) * (lo->D / d2) != lo->th) return 1;
  }
  if (lo->dtype != 0 && lo->dtype != 1) return 1;
  if ((lo->k_mode != 0 && lo->k_mode != 1) || (lo->v_mode != 0 && lo->v_mode != 1)) return 1;
  return 0;
}

/* Sec. 3.2.1 step 2: the T tensors of a chunk form T/F groups of F tensors.
 * A frame offers TX*TY tile positions, one per group, so F = ceil(T / (TX*TY)). */
int64_t kvco_frames_per_group(const kvco_layout* lo) {
  return ceil_div(lo->T, (int64_t)lo->TX * lo->TY);
}

static int64_t layer_groups(const kvco_layout* lo) { return ceil_div(lo->L, 3); } /* step 1: three-layer chunks */
static int64_t plane_bytes(const kvco_layout* lo) {
  return ((int64_t)lo->TY * lo->th) * ((int64_t)lo->TX * lo->tw);
}

int64_t kvco_frame_bytes(const kvco_layout* lo) {
  return 2 * layer_groups(lo) * kvco_frames_per_group(lo) * 3 * plane_bytes(lo);
}

static int64_t kind_mode(const kvco_layout* lo, int kind) { return kind == 0 ? lo->k_mode : lo->v_mode; }

static int64_t kind_meta_floats(const kvco_layout* lo, int kind) {
  int64_t pairs = kind_mode(lo, kind) == 0 ? (int64_t)lo->L * lo->H * lo->D  /* per channel */
                                           : (int64_t)lo->L * lo->T * lo->H; /* per (token, head) */
  return 2 * pairs;
}

int64_t kvco_meta_floats(const kvco_layout* lo) { return kind_meta_floats(lo, 0) + kind_meta_floats(lo, 1); }

int64_t kvco_meta_kind_offset(const kvco_layout* lo, int kind) { return kind == 0 ? 0 : kind_meta_floats(lo, 0); }

int64_t kvco_frame_offset(const kvco_layout* lo, int kind, int l, int64_t t, int h, int d) {
  const int64_t F = kvco_frames_per_group(lo);
  const int64_t W = (int64_t)lo->TX * lo->tw;
  /* Sec. 3.2.2: heads in initial order (rule iii), elements of a head in order (rule ii), no mixing of heads
   * (rule i).  seg = 0: the H*D vector of the token reshaped row-major to (th, tw).  seg = d2 > 0: head_num is
   * reshaped to (h1, h2) and head_dim to (d1, d2), and the tile is (h1*d1, h2*d2): head h = a*h2 + b, element
   * d = c*d2 + i  ->  row a*d1 + c, column b*d2 + i (with d1 = 1 or h2 = 1 that is the row-major reshape again). */
  int64_t r, cc;
  if (lo->seg == 0) {
    const int64_t e = (int64_t)h * lo->D + d;
    r = e / lo->tw;
    cc = e % lo->tw;
  } else {
    const int64_t d2 = lo->seg;
    const int64_t d1 = lo->D / d2;
    const int64_t h2 = lo->tw / d2;
    r = (h / h2) * d1 + d / d2;
    cc = (h % h2) * d2 + d % d2;
  }
  /* Sec. 3.2.1 steps 2-3: token t is tensor number t % F of group t / F; the
   * tensors of a group share one tile position in F consecutive frames.  Tile
   * positions are taken in raster order over the TX x TY grid. */
  const int64_t f = t % F;
  const int64_t g = t / F;
  const int64_t ty = g / lo->TX;
  const int64_t tx = g % lo->TX;
  const int64_t y = ty * lo->th + r;
  const int64_t x = tx * lo->tw + cc;
  /* Sec. 3.2.1 step 1 and its last sentence: three layers -> three planes. */
  const int64_t lg = l / 3;
  const int64_t pl = l % 3;
  const int64_t frame = ((int64_t)kind * layer_groups(lo) + lg) * F + f;
  return (frame * 3 + pl) * plane_bytes(lo) + y * W + x;
}

int64_t kvco_meta_offset(const kvco_layout* lo, int kind, int l, int64_t t, int h, int d) {
  int64_t pair;
  if (kind_mode(lo, kind) == 0)
    pair = ((int64_t)l * lo->H + h) * lo->D + d;
  else
    pair = ((int64_t)l * lo->T + t) * lo->H + h;
  return kvco_meta_kind_offset(lo, kind) + 2 * pair;
}

/* ------------------------------------------------------- 16-bit <-> binary32 */

static float widen_f16(uint16_t b) {
  const int s = b >> 15, e = (b >> 10) & 31, m = b & 1023;
  float v;
  if (e == 0)
    v = ldexpf((float)m, -24); /* subnormal: m * 2^-24 */
  else if (e == 31)
    v = m ? NAN : INFINITY;
  else
    v = ldexpf((float)(m + 1024), e - 25); /* (1 + m/1024) * 2^(e-15) */
  return s ? -v : v;
}

static float widen_bf16(uint16_t b) {
  uint32_t u = (uint32_t)b << 16; /* bf16 is the upper half of binary32 */
  float v;
  memcpy(&v, &u, 4);
  return v;
}

/* Round |x| to the nearest multiple of the target format's quantum at x's
 * binade, ties to the even multiple; `mant` explicit mantissa bits, `emin` the
 * smallest normal exponent. */
static double round_to_format(double ax, int mant, int emin) {
  int ex;
  (void)frexp(ax, &ex); /* ax = m * 2^ex, m in [0.5, 1)  =>  floor(log2 ax) = ex - 1 */
  int e = ex - 1;
  if (e < emin) e = emin;
  const double q = ldexp(1.0, e - mant);
  return rint(ax / q) * q; /* division by a power of two is exact; rint is ties-to-even */
}

static uint16_t narrow_f16(float x) {
  const uint16_t s = signbit(x) ? 0x8000u : 0;
  if (isnan(x)) return 0x7e00u;
  const double ax = fabs((double)x);
  if (isinf(x)) return s | 0x7c00u;
  if (ax == 0.0) return s;
  const double v = round_to_format(ax, 10, -14);
  if (v >= 65536.0) return s | 0x7c00u; /* past the largest finite fp16 (65504) */
  if (v == 0.0) return s;
  int ex;
  (void)frexp(v, &ex);
  const int e = ex - 1;
  if (e < -14) return s | (uint16_t)ldexp(v, 24);                 /* subnormal: v / 2^-24 */
  const int m = (int)ldexp(v, 10 - e) - 1024;                      /* v / 2^(e-10) - 1024 */
  return s | (uint16_t)((e + 15) << 10) | (uint16_t)m;
}

static uint16_t narrow_bf16(float x) {
  if (isnan(x)) return 0x7fc0u;
  const uint16_t s = signbit(x) ? 0x8000u : 0;
  if (isinf(x)) return s | 0x7f80u;
  const double ax = fabs((double)x);
  if (ax == 0.0) return s;
  const float v = (float)round_to_format(ax, 7, -126); /* exact: fits bf16, or overflows to +inf */
  uint32_t u;
  memcpy(&u, &v, 4);
  return s | (uint16_t)(u >> 16);
}

float kvco_widen(uint16_t bits, int dtype) { return dtype == 0 ? widen_f16(bits) : widen_bf16(bits); }
uint16_t kvco_narrow(float x, int dtype) { return dtype == 0 ? narrow_f16(x) : narrow_bf16(x); }

/* ----------------------------------------------------------------- quantizer */

void kvco_group_params(const float* xs, int64_t n, float* scale, float* mn_out, float* inv) {
  float mn = xs[0], mx = xs[0];
  for (int64_t i = 1; i < n; ++i) {
    if (xs[i] < mn) mn = xs[i];
    if (xs[i] > mx) mx = xs[i];
  }
  mn = mn + 0.0f; /* -0.0 -> +0.0 so the stored minimum has one bit pattern */
  const float range = mx - mn;
  if (range == 0.0f) {
    *scale = 0.0f;
    *inv = 0.0f;
  } else {
    *scale = range / 255.0f;
    *inv = 255.0f / range;
  }
  *mn_out = mn;
}

uint8_t kvco_quantize(float x, float mn, float inv) {
  const float diff = x - mn;
  const float pos = diff * inv;
  float q = rintf(pos); /* round half to even */
  if (!(q > 0.0f)) q = 0.0f;
  if (q > 255.0f) q = 255.0f;
  return (uint8_t)q;
}

float kvco_dequantize(uint8_t code, float scale, float mn) { return fmaf((float)code, scale, mn); }

/* ---------------------------------------------------------------- pack side */

#ifndef KVCO_BUILD_ID
#define KVCO_BUILD_ID "unknown"
#endif
static const char build_tag[] = "kvco-build-id:" KVCO_BUILD_ID; /* also found by scanning the file */
const char* kvco_build_id(void) { return build_tag + 14; }

int kvco_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

static void pack_unit(const kvco_layout* lo, const uint16_t* src /* (kind,l) slab, token 0 of the chunk */,
                      int64_t token_stride, int64_t n, int kind, int l, uint8_t* fr, float* me) {
  const int mode = (int)kind_mode(lo, kind);
  const int64_t glen = mode == 0 ? n : lo->D;
  float* xs = (float*)malloc(sizeof(float) * (size_t)glen);
  if (mode == 0) {
    for (int h = 0; h < lo->H; ++h)
      for (int d = 0; d < lo->D; ++d) {
        for (int64_t t = 0; t < n; ++t) xs[t] = kvco_widen(src[t * token_stride + (int64_t)h * lo->D + d], lo->dtype);
        float scale, mn, inv;
        kvco_group_params(xs, n, &scale, &mn, &inv);
        const int64_t mo = kvco_meta_offset(lo, kind, l, 0, h, d);
        me[mo] = scale;
        me[mo + 1] = mn;
        for (int64_t t = 0; t < n; ++t) fr[kvco_frame_offset(lo, kind, l, t, h, d)] = kvco_quantize(xs[t], mn, inv);
      }
  } else {
    for (int64_t t = 0; t < n; ++t)
      for (int h = 0; h < lo->H; ++h) {
        for (int d = 0; d < lo->D; ++d) xs[d] = kvco_widen(src[t * token_stride + (int64_t)h * lo->D + d], lo->dtype);
        float scale, mn, inv;
        kvco_group_params(xs, lo->D, &scale, &mn, &inv);
        const int64_t mo = kvco_meta_offset(lo, kind, l, t, h, 0);
        me[mo] = scale;
        me[mo + 1] = mn;
        for (int d = 0; d < lo->D; ++d) fr[kvco_frame_offset(lo, kind, l, t, h, d)] = kvco_quantize(xs[d], mn, inv);
      }
  }
  free(xs);
}

int kvco_pack(const kvco_layout* lo, const uint16_t* kv, int64_t layer_stride, int64_t kv_stride,
              int64_t token_stride, int64_t n_tokens, uint8_t* frames, float* meta) {
  if (kvco_check(lo) || n_tokens < 0) return 1;
  if (n_tokens == 0) return 0;
  if (!kv || !frames || !meta) return 1;
  const int64_t n_chunks = ceil_div(n_tokens, lo->T);
  const int64_t fb = kvco_frame_bytes(lo), mf = kvco_meta_floats(lo);
  /* bytes and pairs that no valid element reaches are zero */
  memset(frames, 0, (size_t)(n_chunks * fb));
  memset(meta, 0, sizeof(float) * (size_t)(n_chunks * mf));
  const int64_t units = n_chunks * 2 * lo->L;
#pragma omp parallel for schedule(dynamic)
  for (int64_t u = 0; u < units; ++u) {
    const int64_t c = u / (2 * lo->L);
    const int kind = (int)((u / lo->L) % 2);
    const int l = (int)(u % lo->L);
    const int64_t first = c * lo->T;
    const int64_t n = n_tokens - first < lo->T ? n_tokens - first : lo->T;
    pack_unit(lo, kv + l * layer_stride + kind * kv_stride + first * token_stride, token_stride, n, kind, l,
              frames + c * fb, meta + c * mf);
  }
  return 0;
}

/* ------------------------------------------------------------- restore side */

static uint16_t restore_element(const kvco_layout* lo, const uint8_t* fr, const float* me, int kind, int l,
                                int64_t t, int h, int d) {
  const uint8_t code = fr[kvco_frame_offset(lo, kind, l, t, h, d)];
  const int64_t mo = kvco_meta_offset(lo, kind, l, t, h, d);
  return kvco_narrow(kvco_dequantize(code, me[mo], me[mo + 1]), lo->dtype);
}

int kvco_restore(const kvco_layout* lo, const uint8_t* frames, const float* meta, int64_t n_tokens,
                 uint16_t* kv_out, int64_t layer_stride, int64_t kv_stride, int64_t token_stride) {
  if (kvco_check(lo) || n_tokens < 0) return 1;
  if (n_tokens == 0) return 0;
  if (!kv_out || !frames || !meta) return 1;
  const int64_t n_chunks = ceil_div(n_tokens, lo->T);
  const int64_t fb = kvco_frame_bytes(lo), mf = kvco_meta_floats(lo);
  const int64_t units = n_chunks * 2 * lo->L;
#pragma omp parallel for schedule(dynamic)
  for (int64_t u = 0; u < units; ++u) {
    const int64_t c = u / (2 * lo->L);
    const int kind = (int)((u / lo->L) % 2);
    const int l = (int)(u % lo->L);
    const int64_t first = c * lo->T;
    const int64_t n = n_tokens - first < lo->T ? n_tokens - first : lo->T;
    for (int64_t t = 0; t < n; ++t)
      for (int h = 0; h < lo->H; ++h)
        for (int d = 0; d < lo->D; ++d)
          kv_out[l * layer_stride + kind * kv_stride + (first + t) * token_stride + (int64_t)h * lo->D + d] =
              restore_element(lo, frames + c * fb, meta + c * mf, kind, l, t, h, d);
  }
  return 0;
}

int kvco_restore_paged(const kvco_layout* lo, const uint8_t* frames, const float* meta, int64_t first_token,
                       int64_t n_tokens, uint16_t* const* layer_cache, int64_t num_blocks, int32_t block_size,
                       const int32_t* block_table, int64_t table_len, uint32_t* err) {
  if (kvco_check(lo) || n_tokens < 0 || first_token < 0 || first_token % lo->T != 0) return 1;
  if (num_blocks < 1 || block_size < 1) return 1;
  if (n_tokens == 0) return 0;
  if (!layer_cache || !block_table || !frames || !meta) return 1;
  if (table_len * block_size < first_token + n_tokens) return 1;
  const int64_t n_chunks = ceil_div(n_tokens, lo->T);
  const int64_t fb = kvco_frame_bytes(lo), mf = kvco_meta_floats(lo);
  const int64_t C = (int64_t)lo->H * lo->D;
  const int64_t units = n_chunks * 2 * lo->L;
  int bad = 0;
#pragma omp parallel for schedule(dynamic) reduction(| : bad)
  for (int64_t u = 0; u < units; ++u) {
    const int64_t c = u / (2 * lo->L);
    const int kind = (int)((u / lo->L) % 2);
    const int l = (int)(u % lo->L);
    const int64_t first = c * lo->T;
    const int64_t n = n_tokens - first < lo->T ? n_tokens - first : lo->T;
    for (int64_t t = 0; t < n; ++t) {
      const int64_t p = first_token + first + t; /* position in the sequence */
      const int64_t phys = block_table[p / block_size];
      if (phys < 0 || phys >= num_blocks) {
        bad |= 1;
        continue;
      }
      uint16_t* slot = layer_cache[l] + (((int64_t)kind * num_blocks + phys) * block_size + p % block_size) * C;
      for (int h = 0; h < lo->H; ++h)
        for (int d = 0; d < lo->D; ++d)
          slot[(int64_t)h * lo->D + d] = restore_element(lo, frames + c * fb, meta + c * mf, kind, l, t, h, d);
    }
  }
  if (err && bad) *err |= 1u;
  return 0;
}

/* One decoded frame -> paged slots (Sec. 3.3.2, frame-wise restoration).  The frame is addressed
 * with the chunk-section formula minus the offset of the frame's first byte. */
int kvco_restore_paged_frame(const kvco_layout* lo, const uint8_t* frame, const float* meta, int kind, int lg, int f,
                             int64_t first_token, int64_t n_tokens, uint16_t* const* layer_cache, int64_t num_blocks,
                             int32_t block_size, const int32_t* block_table, int64_t table_len, uint32_t* err) {
  if (kvco_check(lo) || first_token < 0 || first_token % lo->T != 0) return 1;
  if (n_tokens < 1 || n_tokens > lo->T || num_blocks < 1 || block_size < 1) return 1;
  const int64_t F = kvco_frames_per_group(lo);
  if (kind < 0 || kind > 1 || lg < 0 || lg >= layer_groups(lo) || f < 0 || f >= F) return 1;
  if (!frame || !meta || !layer_cache || !block_table) return 1;
  if (table_len * block_size < first_token + n_tokens) return 1;
  const int64_t C = (int64_t)lo->H * lo->D;
  /* first byte of this frame inside the chunk section: plane 0 of layer 3*lg, token f, element 0 sits at
   * tile position 0 of frame f */
  const int64_t frame_start = kvco_frame_offset(lo, kind, 3 * lg, f, 0, 0);
  int bad = 0;
  for (int pl = 0; pl < 3; ++pl) {
    const int l = 3 * lg + pl;
    if (l >= lo->L) continue;
    for (int64_t t = f; t < n_tokens; t += F) { /* Sec. 3.2.1 step 3: tensor number f of every group */
      const int64_t p = first_token + t;
      const int64_t phys = block_table[p / block_size];
      if (phys < 0 || phys >= num_blocks) {
        bad = 1;
        continue;
      }
      uint16_t* slot = layer_cache[l] + (((int64_t)kind * num_blocks + phys) * block_size + p % block_size) * C;
      for (int h = 0; h < lo->H; ++h)
        for (int d = 0; d < lo->D; ++d) {
          const uint8_t code = frame[kvco_frame_offset(lo, kind, l, t, h, d) - frame_start];
          const int64_t mo = kvco_meta_offset(lo, kind, l, t, h, d);
          slot[(int64_t)h * lo->D + d] = kvco_narrow(kvco_dequantize(code, meta[mo], meta[mo + 1]), lo->dtype);
        }
    }
  }
  if (err && bad) *err |= 1u;
  return 0;
}
