// Pack kernels: group statistics, 8-bit quantization and the codec-friendly
// layout (Sec. 3.2.1 steps 1-3, Sec. 3.2.2, Sec. 4 item (1)).
//
// One launch covers both quantization groupings; a workgroup takes one of two
// bodies according to the grouping of the kind it works on:
//  * per-token groups (one group = the D elements of one head of one token):
//    statistics, quantization and the layout scatter fused in one pass.  A thread
//    holds an atom of 8 consecutive elements; the D/8 lanes of a head reduce
//    min/max with a cross-lane butterfly, so the input is read exactly once.
//  * per-channel groups (one group = one channel over the valid tokens of a
//    chunk): a workgroup owns a strip of channels of one (chunk, kind, layer).
//    A chunk of up to 2048 tokens is loaded once into the registers and the
//    LDS of a 512-thread workgroup that has its CU to itself, reduced to the
//    column min/max (registers + one LDS step across waves) and quantized from
//    where it waits; of longer chunks the last 3072 tokens wait like that and
//    the tokens before them are read twice (statistics, then quantization).
// Both kernels write every byte of their part of the frame section, zero for
// tile positions without a token and for the planes of layers beyond L, so the
// caller never has to clear the buffer.
#include <hip/hip_runtime.h>

#include <atomic>

#include "kvc_device.h"
#include "kvc_launch.h"

namespace kvc {

#ifndef KVC_PACK_U_RESIDENT
#define KVC_PACK_U_RESIDENT 8  // loads in flight per thread of the per-token body beside the resident strips (8 waves per CU)
#endif
#ifndef KVC_PACK_U
#define KVC_PACK_U 4  // ... beside the streamed strips (16 waves per CU)
#endif
#ifndef KVC_PACK_STREAM_U
#define KVC_PACK_STREAM_U 4  // ... of the two-pass per-channel body (next to the 16 it keeps)
#endif
#ifndef KVC_PACK_STREAM_ATOMS
#define KVC_PACK_STREAM_ATOMS 8  // atoms per strip of the two-pass per-channel body
#endif

namespace {

struct GroupParams {
  float scale, mn, inv;
};

// scale / min / reciprocal step of one group from its min and max (all fp32,
// both divisions correctly rounded).
__device__ __forceinline__ GroupParams group_params(float lo, float hi) {
  GroupParams q;
  q.mn = lo == 0.0f ? 0.0f : lo;  // -0.0 -> +0.0
  const float range = hi - q.mn;
  if (range == 0.0f) {
    q.scale = 0.0f;
    q.inv = 0.0f;
  } else {
    q.scale = range / 255.0f;
    q.inv = 255.0f / range;
  }
  return q;
}

// code = clamp(rint((x - mn) * inv), 0, 255), written into byte `sel` of `acc`.
// Subtraction and product are separately rounded (no contraction is possible:
// there is no add after the mul).  v_cvt_pk_u8_f32 rounds to nearest even under
// the default rounding mode and saturates to [0, 255], i.e. it is rint + clamp +
// convert + byte insert in one instruction.
__device__ __forceinline__ uint32_t quantize_into(uint32_t acc, uint32_t sel, float x, float mn, float inv) {
  return __builtin_amdgcn_cvt_pk_u8_f32((x - mn) * inv, sel, acc);
}

// 8 elements -> 8 code bytes with one {mn, inv} for all (per-token groups)
__device__ __forceinline__ u32x2 quantize_atom(const float (&x)[8], float mn, float inv) {
  u32x2 o{0u, 0u};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    o.x = quantize_into(o.x, i, x[i], mn, inv);
    o.y = quantize_into(o.y, i, x[4 + i], mn, inv);
  }
  return o;
}

// 8 elements -> 8 code bytes with one {mn, inv} per element (per-channel groups)
__device__ __forceinline__ u32x2 quantize_atom(const float (&x)[8], const float (&mn)[8], const float (&inv)[8]) {
  u32x2 o{0u, 0u};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    o.x = quantize_into(o.x, i, x[i], mn[i], inv[i]);
    o.y = quantize_into(o.y, i, x[4 + i], mn[4 + i], inv[4 + i]);
  }
  return o;
}

template <int DT>
__device__ __forceinline__ void widen_atom(const u32x4& v, float (&x)[8]) {
  widen_pair<DT>(v.x, x[0], x[1]);
  widen_pair<DT>(v.y, x[2], x[3]);
  widen_pair<DT>(v.z, x[4], x[5]);
  widen_pair<DT>(v.w, x[6], x[7]);
}

// Minimum and maximum of the 8 elements of an atom.  fp16 pairs are compared with
// the packed half-precision min / max (exact), two elements per instruction.
template <int DT>
__device__ __forceinline__ void atom_minmax(const u32x4& v, float& lo, float& hi);
template <>
__device__ __forceinline__ void atom_minmax<KVC_F16>(const u32x4& v, float& lo, float& hi) {
  // (copy the components to scalars first: a bit cast applied directly to a
  // component of a vector reads the wrong dword with this compiler)
  const uint32_t w0 = v.x, w1 = v.y, w2 = v.z, w3 = v.w;
  const f16x2 a = __builtin_bit_cast(f16x2, w0), b = __builtin_bit_cast(f16x2, w1);
  const f16x2 c = __builtin_bit_cast(f16x2, w2), d = __builtin_bit_cast(f16x2, w3);
  const f16x2 mn = __builtin_elementwise_min(__builtin_elementwise_min(a, b), __builtin_elementwise_min(c, d));
  const f16x2 mx = __builtin_elementwise_max(__builtin_elementwise_max(a, b), __builtin_elementwise_max(c, d));
  lo = __builtin_fminf((float)mn.x, (float)mn.y);
  hi = __builtin_fmaxf((float)mx.x, (float)mx.y);
}
template <>
__device__ __forceinline__ void atom_minmax<KVC_BF16>(const u32x4& v, float& lo, float& hi) {
  float x[8];
  widen_atom<KVC_BF16>(v, x);
  lo = hi = x[0];
#pragma unroll
  for (int i = 1; i < 8; ++i) {
    lo = __builtin_fminf(lo, x[i]);
    hi = __builtin_fmaxf(hi, x[i]);
  }
}

// Running per-channel minimum / maximum of the 8 channels of an atom over many
// tokens.  fp16 stays packed (4 + 4 VGPRs, two channels per instruction); bf16
// is widened first (no packed bf16 compare).
template <int DT>
struct ColumnStats;
template <>
struct ColumnStats<KVC_F16> {
  f16x2 lo[4], hi[4];
  __device__ __forceinline__ void init() {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      lo[j] = f16x2{(_Float16)__builtin_inff(), (_Float16)__builtin_inff()};
      hi[j] = f16x2{(_Float16)-__builtin_inff(), (_Float16)-__builtin_inff()};
    }
  }
  __device__ __forceinline__ void add(const u32x4& v) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      lo[j] = __builtin_elementwise_min(lo[j], __builtin_bit_cast(f16x2, w[j]));
      hi[j] = __builtin_elementwise_max(hi[j], __builtin_bit_cast(f16x2, w[j]));
    }
  }
  __device__ __forceinline__ void merge_xor(int m) {  // with the lane m away
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      lo[j] = __builtin_elementwise_min(lo[j], __builtin_bit_cast(f16x2, __shfl_xor(__builtin_bit_cast(uint32_t, lo[j]), m)));
      hi[j] = __builtin_elementwise_max(hi[j], __builtin_bit_cast(f16x2, __shfl_xor(__builtin_bit_cast(uint32_t, hi[j]), m)));
    }
  }
  __device__ __forceinline__ void get(float (&l)[8], float (&h)[8]) const {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      l[2 * j] = (float)lo[j].x;
      l[2 * j + 1] = (float)lo[j].y;
      h[2 * j] = (float)hi[j].x;
      h[2 * j + 1] = (float)hi[j].y;
    }
  }
};
template <>
struct ColumnStats<KVC_BF16> {
  float lo[8], hi[8];
  __device__ __forceinline__ void init() {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      lo[j] = __builtin_inff();
      hi[j] = -__builtin_inff();
    }
  }
  __device__ __forceinline__ void add(const u32x4& v) {
    float x[8];
    widen_atom<KVC_BF16>(v, x);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      lo[j] = __builtin_fminf(lo[j], x[j]);
      hi[j] = __builtin_fmaxf(hi[j], x[j]);
    }
  }
  __device__ __forceinline__ void merge_xor(int m) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      lo[j] = __builtin_fminf(lo[j], __shfl_xor(lo[j], m));
      hi[j] = __builtin_fmaxf(hi[j], __shfl_xor(hi[j], m));
    }
  }
  __device__ __forceinline__ void get(float (&l)[8], float (&h)[8]) const {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      l[j] = lo[j];
      h[j] = hi[j];
    }
  }
};

// Address of the 8 code bytes of atom (row r, column cc already folded into
// fbase) of token position t inside the (chunk, kind, layer) plane sequence.
__device__ __forceinline__ uint8_t* code_addr(const Geo& g, uint8_t* fbase, uint32_t t) {
  uint32_t gi, f, ty, tx;
  fd_divmod(g.dF, t, gi, f);      // Sec. 3.2.1 step 2: group and index inside the group
  fd_divmod(g.dTX, gi, ty, tx);   // tile position of the group, raster order
  return fbase + (int64_t)f * 3 * g.plane + ((int64_t)ty * g.th * g.W + tx * (uint32_t)g.tw);
}

// ------------------------------------------------------------ per-token groups

// min / max over the 16 lanes of a DPP row (every lane gets the result).  Each step pairs a lane
// with one that holds a different part of the row: neighbours, the other pair of the quad, the
// mirrored half row, the mirrored row.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ void head_minmax16(float& lo, float& hi) {
  lo = __builtin_fminf(lo, dpp_move<0xB1>(lo));   // quad_perm [1,0,3,2]
  hi = __builtin_fmaxf(hi, dpp_move<0xB1>(hi));
  lo = __builtin_fminf(lo, dpp_move<0x4E>(lo));   // quad_perm [2,3,0,1]
  hi = __builtin_fmaxf(hi, dpp_move<0x4E>(hi));
  lo = __builtin_fminf(lo, dpp_move<0x141>(lo));  // row_half_mirror
  hi = __builtin_fmaxf(hi, dpp_move<0x141>(hi));
  lo = __builtin_fminf(lo, dpp_move<0x140>(lo));  // row_mirror
  hi = __builtin_fmaxf(hi, dpp_move<0x140>(hi));
}

template <int DT, bool UNIFORM, int U>
__device__ __forceinline__ void pack_token_body(const PackParams& p, uint32_t unit) {
  const Geo& g = p.g;
  uint32_t uu = unit;
  const uint32_t tbi = uu % (uint32_t)p.tbc;
  uu /= (uint32_t)p.tbc;
  const uint32_t l = uu % (uint32_t)g.L;
  uu /= (uint32_t)g.L;
  const uint32_t kind = (uint32_t)p.kinds_tok[uu % (uint32_t)p.n_kinds_tok];
  const uint32_t c = uu / (uint32_t)p.n_kinds_tok;
  if (threadIdx.x >= (uint32_t)(g.apt * p.tpp)) return;  // the block is rounded up to whole waves

  const uint32_t tid = threadIdx.x;
  uint32_t tsub = fd_div(p.dapt, tid);
  const uint32_t ca = tid - tsub * (uint32_t)g.apt;
  if (UNIFORM) tsub = wave_uniform(tsub);
  const uint32_t e = ca * 8u;
  const uint32_t glanes = (uint32_t)g.D / 8u;  // lanes of one group: a power of two <= 64

  const int64_t chunk_first = (int64_t)c * g.T;
  const int64_t left = p.n_tokens - chunk_first;
  const int32_t n = left < (int64_t)g.T ? (int32_t)left : g.T;
  // token positions in the tile rows that can hold a token of this chunk; the rows below are the zero units'
  const int32_t positions = (int32_t)c + 1 == p.n_chunks ? p.positions_last : p.positions_full;
  const int32_t t0 = (int32_t)tbi * p.tb;
  const int32_t t1 = t0 + p.tb < positions ? t0 + p.tb : positions;

  uint32_t r, cc;
  tile_pos(g, e, r, cc);
  const uint32_t lg = l / 3u, pl = l - lg * 3u;
  uint8_t* fbase = p.frames + (int64_t)c * g.frame_bytes + (((int64_t)kind * g.LG + lg) * g.F * 3 + pl) * g.plane +
                   (r * (uint32_t)g.W + cc);
  const uint32_t h = fd_div(g.dD, e);
  float* mrow = p.meta + (int64_t)c * g.meta_floats + g.meta_off[kind] + 2 * ((int64_t)l * g.T * g.H + h);
  const uint16_t* src = p.kv + (int64_t)l * p.ls + (int64_t)kind * p.ks + chunk_first * p.ts + e;
  const bool leader = (ca & (glanes - 1u)) == 0u;

  const int32_t step = p.tpp;
  int32_t tb0 = t0;
  // whole passes of U tokens that all exist: no branches between the loads and the stores
  const int32_t full_end = n < t1 ? n : t1;
  for (; tb0 + U * step <= full_end; tb0 += U * step) {
    u32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int32_t t = tb0 + u * step + (int32_t)tsub;
      v[u] = stream_load<u32x4>(src + (int64_t)t * p.ts);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int32_t t = tb0 + u * step + (int32_t)tsub;
      float lo, hi;
      atom_minmax<DT>(v[u], lo, hi);
      if (glanes == 16u) {  // D = 128: the 16 lanes of a head are one DPP row
        head_minmax16(lo, hi);
      } else {
        for (uint32_t m = 1; m < glanes; m <<= 1) {
          lo = __builtin_fminf(lo, __shfl_xor(lo, (int)m));
          hi = __builtin_fmaxf(hi, __shfl_xor(hi, (int)m));
        }
      }
      const GroupParams q = group_params(lo, hi);
      float x[8];
      widen_atom<DT>(v[u], x);
      const u32x2 o = quantize_atom(x, q.mn, q.inv);
      stream_store<u32x2>(code_addr(g, fbase, (uint32_t)t), o);
      if (leader) *reinterpret_cast<f32x2*>(mrow + 2 * (int64_t)t * g.H) = f32x2{q.scale, q.mn};
    }
  }
  for (; tb0 < t1; tb0 += U * step) {
    u32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int32_t t = tb0 + u * step + (int32_t)tsub;
      v[u] = u32x4{0u, 0u, 0u, 0u};
      if (t < n) v[u] = stream_load<u32x4>(src + (int64_t)t * p.ts);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int32_t t = tb0 + u * step + (int32_t)tsub;
      if (t >= t1) continue;
      uint8_t* dst = code_addr(g, fbase, (uint32_t)t);
      if (t >= n) {  // no token here: zero codes, zero pair
        stream_store<u32x2>(dst, u32x2{0u, 0u});
        if (leader && t < g.T) *reinterpret_cast<f32x2*>(mrow + 2 * (int64_t)t * g.H) = f32x2{0.f, 0.f};
        continue;
      }
      float lo, hi;
      atom_minmax<DT>(v[u], lo, hi);
      for (uint32_t m = 1; m < glanes; m <<= 1) {  // butterfly over the lanes of the head
        lo = __builtin_fminf(lo, __shfl_xor(lo, (int)m));
        hi = __builtin_fmaxf(hi, __shfl_xor(hi, (int)m));
      }
      const GroupParams q = group_params(lo, hi);
      float x[8];
      widen_atom<DT>(v[u], x);
      const u32x2 o = quantize_atom(x, q.mn, q.inv);
      stream_store<u32x2>(dst, o);
      if (leader) *reinterpret_cast<f32x2*>(mrow + 2 * (int64_t)t * g.H) = f32x2{q.scale, q.mn};
    }
  }
  // Pairs of the token positions of this block that the loops did not visit (a short chunk uses fewer tile
  // rows than a full one; every such position is past the chunk's last token): {0, 0}.
  const int32_t m1 = t0 + p.tb < g.T ? t0 + p.tb : g.T;
  for (int32_t t = (t1 > t0 ? t1 : t0) + (int32_t)tsub; t < m1; t += step)
    if (leader) *reinterpret_cast<f32x2*>(mrow + 2 * (int64_t)t * g.H) = f32x2{0.f, 0.f};
}

// ---------------------------------------------------------- per-channel groups

constexpr int kMaxStripAtoms = 16;  // 128 channels

// The workgroup's column statistics (each thread: its 8 channels over the token rows it took) -> the strip's group
// parameters: lanes of a wave that hold the same atom differ by multiples of strip_atoms and are merged first, one
// lane per atom leaves the wave's extremes in LDS, one thread per channel finishes the reduction, derives the
// parameters, writes the channel's {scale, mn} pair, and hands {mn, inv} to all threads through LDS.  Two barriers;
// every thread of the workgroup must come here.
template <int DT>
__device__ __forceinline__ void strip_parameters(const PackParams& p, ColumnStats<DT>& st, uint32_t strip, uint32_t kind,
                                                 uint32_t l, uint32_t c, float (*red_lo)[kMaxStripAtoms * 8],
                                                 float (*red_hi)[kMaxStripAtoms * 8], float (&mnv)[8], float (&inv)[8]) {
  const Geo& g = p.g;
  const uint32_t tid = threadIdx.x;
  const uint32_t sa = (uint32_t)p.strip_atoms;
  const uint32_t a = tid & (sa - 1u);
  for (uint32_t m = sa; m < 64u; m <<= 1) st.merge_xor((int)m);
  float lo[8], hi[8];
  st.get(lo, hi);
  const uint32_t wave = tid >> 6, lane = tid & 63u;
  const uint32_t n_waves = blockDim.x >> 6;
  if (lane < sa) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      red_lo[wave][lane * 8 + i] = lo[i];
      red_hi[wave][lane * 8 + i] = hi[i];
    }
  }
  __syncthreads();
  float* par_mn = &red_lo[n_waves][0];
  float* par_inv = &red_hi[n_waves][0];
  if (tid < sa * 8u) {
    float l0 = red_lo[0][tid], h0 = red_hi[0][tid];
    for (uint32_t w = 1; w < n_waves; ++w) {
      l0 = __builtin_fminf(l0, red_lo[w][tid]);
      h0 = __builtin_fmaxf(h0, red_hi[w][tid]);
    }
    const GroupParams q = group_params(l0, h0);
    par_mn[tid] = q.mn;
    par_inv[tid] = q.inv;
    const uint32_t ch = strip * sa * 8u + tid;
    if (ch < (uint32_t)g.C) {
      float* mp = p.meta + (int64_t)c * g.meta_floats + g.meta_off[kind] + 2 * ((int64_t)l * g.C + ch);
      *reinterpret_cast<f32x2*>(mp) = f32x2{q.scale, q.mn};
    }
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    mnv[i] = par_mn[a * 8 + i];
    inv[i] = par_inv[a * 8 + i];
  }
}

// Streaming variant for chunks too long for the register-resident strip: the strip is read twice, once for the
// column statistics and once to quantize -- except its last (kStreamTailLoads + kStreamStashLoads) * rows tokens
// (3072 with 1024 threads), which wait on chip between the two passes: 16 loads per thread in registers, 8 more in the
// CU's LDS (128 KB of its 160 KB; the workgroup has the CU to itself anyway).  Every thread reads back the LDS words it wrote itself, so the stash needs no barrier.
constexpr int kStreamTailLoads = 16;
constexpr int kStreamStashLoads = 8;

template <int DT>
__device__ __forceinline__ void pack_channel_body(const PackParams& p, uint32_t unit, float (*red_lo)[kMaxStripAtoms * 8],
                                                  float (*red_hi)[kMaxStripAtoms * 8], u32x4* stash) {
  constexpr int U = KVC_PACK_STREAM_U;
  constexpr int NT = kStreamTailLoads, NS = kStreamStashLoads;
  static_assert(NS % U == 0, "the stash is filled in steps of U loads");
  const Geo& g = p.g;
  uint32_t uu = unit;
  const uint32_t strip = uu % (uint32_t)p.n_strips;
  uu /= (uint32_t)p.n_strips;
  const uint32_t l = uu % (uint32_t)g.L;
  uu /= (uint32_t)g.L;
  const uint32_t kind = (uint32_t)p.kinds_ch[uu % (uint32_t)p.n_kinds_ch];
  const uint32_t c = uu / (uint32_t)p.n_kinds_ch;

  const uint32_t tid = threadIdx.x;
  const uint32_t sa = (uint32_t)p.strip_atoms;  // power of two <= 64
  const uint32_t a = tid & (sa - 1u);
  const uint32_t row = tid / sa;
  const uint32_t rows = (uint32_t)p.rows;
  const uint32_t ca = strip * sa + a;
  const bool active = ca < (uint32_t)g.apt;
  const uint32_t e = (active ? ca : 0u) * 8u;  // idle lanes of a ragged last strip shadow atom 0 and never store

  const int64_t chunk_first = (int64_t)c * g.T;
  const int64_t left = p.n_tokens - chunk_first;
  const uint32_t n = left < (int64_t)g.T ? (uint32_t)left : (uint32_t)g.T;
  const uint32_t positions = (uint32_t)((int32_t)c + 1 == p.n_chunks ? p.positions_last : p.positions_full);
  // tokens [0, head_n) are streamed twice; [head_n, tail_0) wait in LDS and [tail_0, n) in registers
  const uint32_t head_n = n > (uint32_t)(NT + NS) * rows ? n - (uint32_t)(NT + NS) * rows : 0u;
  const uint32_t tail_0 = head_n + (uint32_t)NS * rows;
  u32x4* const mine = stash + tid;  // slot i of this thread: mine[i * blockDim.x]

  uint32_t r, cc;
  tile_pos(g, e, r, cc);
  const uint32_t lg = l / 3u, pl = l - lg * 3u;
  uint8_t* fbase = p.frames + (int64_t)c * g.frame_bytes + (((int64_t)kind * g.LG + lg) * g.F * 3 + pl) * g.plane +
                   (r * (uint32_t)g.W + cc);
  const uint16_t* src = p.kv + (int64_t)l * p.ls + (int64_t)kind * p.ks + chunk_first * p.ts + e;

  float mnv[8], inv[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    mnv[i] = 0.f;
    inv[i] = 0.f;
  }
  u32x4 tail[NT];

  if (n > 0) {
    // pass 1: column min / max of the strip over the chunk's valid tokens
    ColumnStats<DT> st;
    st.init();
    for (uint32_t tb0 = 0; tb0 < head_n; tb0 += U * rows) {
      u32x4 v[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint32_t t = tb0 + u * rows + row;
        const uint32_t tc = t < head_n ? t : head_n - 1u;  // a repeated token leaves min / max unchanged
        v[u] = *reinterpret_cast<const u32x4*>(src + (int64_t)tc * p.ts);  // cached: read again in pass 2
      }
#pragma unroll
      for (int u = 0; u < U; ++u) st.add(v[u]);
    }
#pragma unroll
    for (int i0 = 0; i0 < NS; i0 += U) {
      u32x4 v[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint32_t t = head_n + (uint32_t)(i0 + u) * rows + row;
        v[u] = stream_load<u32x4>(src + (int64_t)(t < n ? t : n - 1u) * p.ts);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        st.add(v[u]);
        mine[(uint32_t)(i0 + u) * blockDim.x] = v[u];
      }
    }
#pragma unroll
    for (int i = 0; i < NT; ++i) {
      const uint32_t t = tail_0 + (uint32_t)i * rows + row;
      tail[i] = stream_load<u32x4>(src + (int64_t)(t < n ? t : n - 1u) * p.ts);
    }
#pragma unroll
    for (int i = 0; i < NT; ++i) st.add(tail[i]);
    strip_parameters<DT>(p, st, strip, kind, l, c, red_lo, red_hi, mnv, inv);
  }
  if (!active) return;  // after the barriers: lanes of a ragged last strip store nothing

  // pass 2: quantize and scatter -- the streamed tokens from memory again, ...
  for (uint32_t tb0 = 0; tb0 < head_n; tb0 += U * rows) {
    u32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t t = tb0 + u * rows + row;
      v[u] = u32x4{0u, 0u, 0u, 0u};
      if (t < head_n) v[u] = stream_load<u32x4>(src + (int64_t)t * p.ts);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t t = tb0 + u * rows + row;
      if (t >= head_n) continue;
      float x[8];
      widen_atom<DT>(v[u], x);
      stream_store<u32x2>(code_addr(g, fbase, t), quantize_atom(x, mnv, inv));
    }
  }
  // ... the kept tokens from LDS and from the registers, ...
#pragma unroll
  for (int i = 0; i < NS; ++i) {
    const uint32_t t = head_n + (uint32_t)i * rows + row;
    if (t >= n) continue;
    float x[8];
    widen_atom<DT>(mine[(uint32_t)i * blockDim.x], x);
    stream_store<u32x2>(code_addr(g, fbase, t), quantize_atom(x, mnv, inv));
  }
#pragma unroll
  for (int i = 0; i < NT; ++i) {
    const uint32_t t = tail_0 + (uint32_t)i * rows + row;
    if (t >= n) continue;
    float x[8];
    widen_atom<DT>(tail[i], x);
    stream_store<u32x2>(code_addr(g, fbase, t), quantize_atom(x, mnv, inv));
  }
  // ... and zeros for the tile positions of the used tile rows that hold no token.
  for (uint32_t t = n + row; t < positions; t += rows) stream_store<u32x2>(code_addr(g, fbase, t), u32x2{0u, 0u});
}

// Resident variant: the strip of one (chunk, kind, layer) -- up to kResidentLoads * rows tokens x 128
// channels, 512 KB of fp16 at 512 threads -- is loaded once, reduced, and quantized from where it waits, so
// the input is read from HBM exactly once.  Of a thread's 64 loads 46 wait in its registers (184 VGPRs of the
// 256 a wave gets at two waves per SIMD) and 18 in LDS (144 KB of the CU's 160 KB), each thread reading back
// the words it wrote itself, so the LDS part needs no barrier.  A strip as wide as a 128-byte line of codes is
// what this buys: strips of 64 channels, which fit the registers alone, share every code line with their
// neighbour and write 20 % more bytes than the codes have (with both kinds per channel 1.21 -> 1.18 ms).
constexpr int kResidentThreads = 512;
constexpr int kResidentAtoms = 16;
constexpr int kResidentRegs = 46;  // loads of a thread that wait in registers
constexpr int kResidentLds = 18;   // ... in LDS
constexpr int kResidentLoads = kResidentRegs + kResidentLds;
constexpr int kResidentGroup = 6;  // loads in flight while the LDS slots are filled
static_assert(kResidentLds % kResidentGroup == 0, "the LDS slots are filled a whole group of loads at a time");

template <int DT>
__device__ __forceinline__ void pack_channel_body_resident(const PackParams& p, uint32_t unit,
                                                           float (*red_lo)[kMaxStripAtoms * 8],
                                                           float (*red_hi)[kMaxStripAtoms * 8], u32x4* stash) {
  constexpr int NI = kResidentLoads, NR = kResidentRegs, NS = kResidentLds;
  const Geo& g = p.g;
  uint32_t uu = unit;
  const uint32_t strip = uu % (uint32_t)p.n_strips;
  uu /= (uint32_t)p.n_strips;
  const uint32_t l = uu % (uint32_t)g.L;
  uu /= (uint32_t)g.L;
  const uint32_t kind = (uint32_t)p.kinds_ch[uu % (uint32_t)p.n_kinds_ch];
  const uint32_t c = uu / (uint32_t)p.n_kinds_ch;

  const uint32_t tid = threadIdx.x;
  const uint32_t sa = (uint32_t)p.strip_atoms;
  const uint32_t a = tid & (sa - 1u);
  const uint32_t row = tid / sa;
  const uint32_t rows = (uint32_t)p.rows;
  const uint32_t ca = strip * sa + a;
  const bool active = ca < (uint32_t)g.apt;
  const uint32_t e = (active ? ca : 0u) * 8u;

  const int64_t chunk_first = (int64_t)c * g.T;
  const int64_t left = p.n_tokens - chunk_first;
  const int32_t n = left < (int64_t)g.T ? (int32_t)left : g.T;
  const uint32_t positions = (uint32_t)((int32_t)c + 1 == p.n_chunks ? p.positions_last : p.positions_full);

  uint32_t r, cc;
  tile_pos(g, e, r, cc);
  const uint32_t lg = l / 3u, pl = l - lg * 3u;
  uint8_t* fplane = p.frames + (int64_t)c * g.frame_bytes + (((int64_t)kind * g.LG + lg) * g.F * 3 + pl) * g.plane;
  const uint8_t* srcb = reinterpret_cast<const uint8_t*>(p.kv + (int64_t)l * p.ls + (int64_t)kind * p.ks + chunk_first * p.ts);
  const uint32_t ts2 = (uint32_t)p.ts * 2u;

  u32x4 v[NR];                       // loads NS .. NI-1
  u32x4* const mine = stash + tid;   // load i < NS: mine[i * blockDim.x]
  float mnv[8], inv[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) mnv[i] = inv[i] = 0.f;

  if (n > 0) {
    // byte offsets grow by a constant per pass; rows past the last token repeat it (min / max unchanged)
    const uint32_t last = ((uint32_t)n - 1u) * ts2 + e * 2u, off_row = row * ts2 + e * 2u, off_step = rows * ts2;
    ColumnStats<DT> st;
    st.init();
    // the loads that wait in LDS first, while the registers of the others are still free to carry them
#pragma unroll
    for (int i0 = 0; i0 < NS; i0 += kResidentGroup) {
      u32x4 w[kResidentGroup];
#pragma unroll
      for (int u = 0; u < kResidentGroup; ++u) {
        const uint32_t off = off_row + (uint32_t)(i0 + u) * off_step;
        w[u] = stream_load<u32x4>(srcb + (size_t)(off < last ? off : last));
      }
#pragma unroll
      for (int u = 0; u < kResidentGroup; ++u) {
        st.add(w[u]);
        mine[(uint32_t)(i0 + u) * blockDim.x] = w[u];
      }
    }
#pragma unroll
    for (int i = 0; i < NR; ++i) {
      const uint32_t off = off_row + (uint32_t)(NS + i) * off_step;
      v[i] = stream_load<u32x4>(srcb + (size_t)(off < last ? off : last));
    }
#pragma unroll
    for (int i = 0; i < NR; ++i) st.add(v[i]);
    strip_parameters<DT>(p, st, strip, kind, l, c, red_lo, red_hi, mnv, inv);
  }
  if (!active) return;  // after the barriers: lanes of a ragged last strip store nothing

  // Quantize from the registers; tile positions without a token get zeros.  Token position
  // t -> frame t % F, tile (t / F) % TX of tile row (t / F) / TX; when the rows of a pass
  // are a whole number of tile rows (rows % (F * TX) == 0) the offset grows by a constant per pass.
  const uint32_t frame3 = (uint32_t)(3 * g.plane), trs = (uint32_t)g.th * (uint32_t)g.W;
  const uint32_t lane_off = r * (uint32_t)g.W + cc;
  uint32_t gi0, f0, ty0, tx0;
  fd_divmod(g.dF, row, gi0, f0);
  fd_divmod(g.dTX, gi0, ty0, tx0);
  const uint32_t off0 = f0 * frame3 + ty0 * trs + tx0 * (uint32_t)g.tw + lane_off;
  const uint32_t pass_step = p.pass_step;  // bytes per pass, 0 if not constant
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const uint32_t t = row + (uint32_t)i * rows;
    if (t >= positions) continue;
    u32x2 o{0u, 0u};
    if (t < (uint32_t)n) {
      float x[8];
      if (i < NS)
        widen_atom<DT>(mine[(uint32_t)i * blockDim.x], x);
      else
        widen_atom<DT>(v[i < NS ? 0 : i - NS], x);
      o = quantize_atom(x, mnv, inv);
    }
    uint32_t off = off0 + (uint32_t)i * pass_step;
    if (pass_step == 0u) {
      uint32_t gi, f, ty, tx;
      fd_divmod(g.dF, t, gi, f);
      fd_divmod(g.dTX, gi, ty, tx);
      off = f * frame3 + ty * trs + tx * (uint32_t)g.tw + lane_off;
    }
    stream_store<u32x2>(fplane + (size_t)off, o);
  }
  for (uint32_t t = row + (uint32_t)NI * rows; t < positions; t += rows) {
    uint32_t gi, f, ty, tx;
    fd_divmod(g.dF, t, gi, f);
    fd_divmod(g.dTX, gi, ty, tx);
    stream_store<u32x2>(fplane + (size_t)(f * frame3 + ty * trs + tx * (uint32_t)g.tw + lane_off), u32x2{0u, 0u});
  }
}

// ------------------------------------------------------------------ zero fill

// Frame bytes no token of a chunk can reach are cleared by workgroups of their own with plain
// full-width stores: the planes of layers beyond L, and the tile rows below the last row that
// holds a token (a chunk shorter than the frame's tile grid, a grid larger than the chunk).
constexpr uint32_t kZeroPiece = 64u << 10;  // bytes one workgroup clears

// Clears [dst, dst + bytes); dst is 8-byte aligned and bytes a multiple of 8.
__device__ __forceinline__ void zero_span(uint8_t* dst, uint32_t bytes) {
  const uint32_t tid = threadIdx.x, nt = blockDim.x;
  if ((reinterpret_cast<uintptr_t>(dst) & 8u) != 0u && bytes != 0u) {  // one 8-byte store up to 16-byte alignment
    if (tid == 0) stream_store<u32x2>(dst, u32x2{0u, 0u});
    dst += 8;
    bytes -= 8u;
  }
  const uint32_t n16 = bytes >> 4;
  for (uint32_t i = tid; i < n16; i += nt) stream_store<u32x4>(dst + (size_t)i * 16u, u32x4{0u, 0u, 0u, 0u});
  if ((bytes & 8u) != 0u && tid == 0) stream_store<u32x2>(dst + (size_t)n16 * 16u, u32x2{0u, 0u});
}

__device__ __forceinline__ void pack_zero_body(const PackParams& p, uint32_t z) {
  const Geo& g = p.g;
  const uint32_t F = (uint32_t)g.F, L = (uint32_t)g.L;
  uint32_t c, kind, l3, f, piece, start;
  if (z < p.n_zero_pad) {  // plane of a layer that does not exist: all of it
    piece = z % p.pieces_plane;
    z /= p.pieces_plane;
    f = z % F;
    z /= F;
    const uint32_t npad = 3u * (uint32_t)g.LG - L;
    l3 = L + z % npad;
    z /= npad;
    kind = z & 1u;
    c = z >> 1;
    start = 0u;
  } else {  // plane of a real layer: the tile rows below the chunk's last used row
    z -= p.n_zero_pad;
    uint32_t pieces, positions;
    if (z < p.n_zero_full) {  // chunks that hold T tokens
      pieces = p.pieces_tail_full;
      positions = (uint32_t)p.positions_full;
      c = 0u;
    } else {                   // the last chunk of the call, which may be shorter
      z -= p.n_zero_full;
      pieces = p.pieces_tail_last;
      positions = (uint32_t)p.positions_last;
      c = (uint32_t)p.n_chunks - 1u;
    }
    piece = z % pieces;
    z /= pieces;
    f = z % F;
    z /= F;
    l3 = z % L;
    z /= L;
    kind = z & 1u;
    c += z >> 1;
    start = positions / ((uint32_t)g.TX * F) * (uint32_t)g.th * (uint32_t)g.W;  // used tile rows * bytes per tile row
  }
  const uint32_t plane = (uint32_t)g.plane;
  const uint64_t lo = (uint64_t)start + (uint64_t)piece * kZeroPiece;
  if (lo >= plane) return;
  const uint32_t bytes = plane - (uint32_t)lo < kZeroPiece ? plane - (uint32_t)lo : kZeroPiece;
  uint8_t* dst = p.frames + (int64_t)c * g.frame_bytes +
                 ((((int64_t)kind * g.LG + l3 / 3u) * g.F + f) * 3 + l3 % 3u) * g.plane + (int64_t)lo;
  zero_span(dst, bytes);
}

template <int DT, bool UNIFORM, bool RESIDENT>
__global__ void __launch_bounds__(RESIDENT ? kResidentThreads : 1024) pack_kernel(const PackParams p) {
  // partial column extremes of the waves; the row after them carries the finished {mn} / {inv} of the strip
  constexpr int kWaves = (RESIDENT ? kResidentThreads : 1024) / 64;
  __shared__ float red_lo[kWaves + 1][kMaxStripAtoms * 8];
  __shared__ float red_hi[kWaves + 1][kMaxStripAtoms * 8];
  extern __shared__ u32x4 stash[];  // the loads of the per-channel bodies that wait in LDS, one slot per thread each
  // Workgroups go to the 8 XCDs round-robin.  Each XCD gets one contiguous range
  // of the per-channel units, one of the per-token units and one of the zero-fill
  // units, so neighbouring strips and token blocks share an L2 and every XCD has
  // the same mix of work.
  const uint32_t xcd = blockIdx.x & 7u, idx = blockIdx.x >> 3;
  if (idx < p.ch_per_xcd) {
    const uint32_t unit = xcd * p.ch_per_xcd + idx;
    if (unit < p.n_units_ch) {
      if (RESIDENT)
        pack_channel_body_resident<DT>(p, unit, red_lo, red_hi, stash);
      else
        pack_channel_body<DT>(p, unit, red_lo, red_hi, stash);
    }
  } else if (idx < p.ch_per_xcd + p.tok_per_xcd) {
    const uint32_t unit = xcd * p.tok_per_xcd + (idx - p.ch_per_xcd);
    if (unit < p.n_units_tok) pack_token_body<DT, UNIFORM, RESIDENT ? KVC_PACK_U_RESIDENT : KVC_PACK_U>(p, unit);
  } else {
    const uint32_t unit = xcd * p.zero_per_xcd + (idx - p.ch_per_xcd - p.tok_per_xcd);
    if (unit < p.n_units_zero) pack_zero_body(p, unit);
  }
}

// The per-channel bodies ask for more dynamic LDS than the 64 KB a kernel gets unasked; the limit of a kernel
// is raised once per device (devices beyond the 64 the mask covers: on every launch).
template <int DT, bool UNIFORM, bool RESIDENT>
hipError_t launch_variant(dim3 grid, dim3 block, size_t lds, hipStream_t stream, const PackParams& p) {
  static std::atomic<uint64_t> raised{0};
  const auto fn = pack_kernel<DT, UNIFORM, RESIDENT>;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const uint64_t bit = dev < 64 ? 1ull << dev : 0ull;
  if ((raised.load(std::memory_order_acquire) & bit) == 0) {
    constexpr size_t most = RESIDENT ? (size_t)kResidentLds * kResidentThreads * sizeof(u32x4)
                                     : (size_t)kStreamStashLoads * 1024 * sizeof(u32x4);
    e = hipFuncSetAttribute((const void*)fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)most);
    if (e != hipSuccess) return e;
    raised.fetch_or(bit, std::memory_order_release);
  }
  hipLaunchKernelGGL(fn, grid, block, lds, stream, p);
  return hipGetLastError();
}

}  // namespace

kvc_status plan_pack(PackParams& p, int* threads_out) {
  const Geo& g = p.g;
  p.n_chunks = (int32_t)((p.n_tokens + g.T - 1) / g.T);
  if (g.apt > 1024) return KVC_ERR_UNSUPPORTED;
  p.n_kinds_ch = p.n_kinds_tok = 0;
  for (int kind = 0; kind < 2; ++kind) {
    if (g.mode[kind] == KVC_Q_PER_CHANNEL)
      p.kinds_ch[p.n_kinds_ch++] = kind;
    else
      p.kinds_tok[p.n_kinds_tok++] = kind;
  }
  // per-token part: a whole number of tokens per pass, about 256 threads
  const int glanes = g.D / 8;
  if (p.n_kinds_tok > 0 && (glanes > 64 || (glanes & (glanes - 1)) != 0)) return KVC_ERR_UNSUPPORTED;
  // Per-channel kinds whose chunk fits the resident strip run with 512 threads (the strip then spans 32 token
  // rows x 64 loads = 2048 tokens of 128 channels: 256-byte input rows, 128-byte code rows).
  p.strip_atoms = kResidentAtoms;
  // The resident body forms 32-bit byte offsets for all kResidentLoads x rows token rows of a strip, whatever
  // the chunk length (rows past the last token are clamped afterwards), and inside the chunk's frame section.
  const int64_t resident_rows = (int64_t)kResidentLoads * (kResidentThreads / p.strip_atoms);
  p.resident = p.n_kinds_ch > 0 && g.T <= resident_rows && resident_rows * p.ts * 2 < (1ll << 32) &&
                       g.frame_bytes < (1ll << 32)
                   ? 1
                   : 0;
  // Chunks too long for that read the part of each strip that does not fit on chip twice.  Few, large
  // workgroups (one of 1024 threads per CU) give each strip the whole CU's registers and LDS to wait in, and
  // keep the strips in flight few, so that part of the second read still finds its strip in the last-level
  // cache: 10 240-token chunks pack in 1.37 ms this way against 1.83 ms with 256-thread workgroups.
#ifndef KVC_PACK_STREAM_THREADS
#define KVC_PACK_STREAM_THREADS 1024
#endif
  if (!p.resident) p.strip_atoms = KVC_PACK_STREAM_ATOMS;
  const int want = p.resident ? kResidentThreads : KVC_PACK_STREAM_THREADS;
  p.tpp = g.apt >= want ? 1 : want / g.apt;
  p.dapt = make_fastdiv((uint32_t)g.apt);
  const int threads = p.resident ? kResidentThreads : (g.apt * p.tpp + 63) / 64 * 64;
  // Token positions the bodies walk: those of the tile rows a token of the chunk can fall into.  What lies
  // below is zero and belongs to the zero-fill units, as do the planes of layers beyond L.
  const auto positions = [&](int64_t n) { return (int32_t)(((n + g.F - 1) / g.F + g.TX - 1) / g.TX * g.TX * g.F); };
  const int64_t n_last = p.n_tokens - (int64_t)(p.n_chunks - 1) * g.T;
  p.positions_full = positions(g.T);
  p.positions_last = positions(n_last);
  p.tb = 128;  // token positions per workgroup of the per-token kinds (32: 1.27 ms, 64: 1.18, 128: 1.157, 256: 1.166, 512: 1.20)
  p.tbc = (p.positions_full + p.tb - 1) / p.tb;
  // per-channel part: strips of 8*strip_atoms channels
  p.n_strips = (g.apt + p.strip_atoms - 1) / p.strip_atoms;
  p.rows = threads / p.strip_atoms;
  p.pass_step = p.rows % (g.F * g.TX) == 0 ? (uint32_t)(p.rows / (g.F * g.TX)) * (uint32_t)g.th * (uint32_t)g.W : 0u;
  const int64_t per_kind = (int64_t)p.n_chunks * g.L;
  const int64_t units_ch = per_kind * p.n_kinds_ch * p.n_strips;
  const int64_t units_tok = per_kind * p.n_kinds_tok * p.tbc;
  const auto pieces = [](int64_t bytes) { return (bytes + kZeroPiece - 1) / kZeroPiece; };
  const int64_t tile_row = (int64_t)g.th * g.W;
  p.pieces_plane = (uint32_t)pieces(g.plane);
  p.pieces_tail_full = (uint32_t)pieces(g.plane - p.positions_full / (g.TX * g.F) * tile_row);
  p.pieces_tail_last = (uint32_t)pieces(g.plane - p.positions_last / (g.TX * g.F) * tile_row);
  const int64_t zero_pad = (int64_t)p.n_chunks * 2 * (3 * g.LG - g.L) * g.F * p.pieces_plane;
  const int64_t zero_full = (int64_t)(p.n_chunks - 1) * 2 * g.L * g.F * p.pieces_tail_full;
  const int64_t zero_last = (int64_t)2 * g.L * g.F * p.pieces_tail_last;
  if (units_ch + units_tok + zero_pad + zero_full + zero_last > 0x7fffffff / 8) return KVC_ERR_UNSUPPORTED;
  p.n_units_ch = (uint32_t)units_ch;
  p.n_units_tok = (uint32_t)units_tok;
  p.n_zero_pad = (uint32_t)zero_pad;
  p.n_zero_full = (uint32_t)zero_full;
  p.n_units_zero = (uint32_t)(zero_pad + zero_full + zero_last);
  p.ch_per_xcd = (p.n_units_ch + 7u) / 8u;
  p.tok_per_xcd = (p.n_units_tok + 7u) / 8u;
  p.zero_per_xcd = (p.n_units_zero + 7u) / 8u;
  p.units_per_xcd = p.ch_per_xcd + p.tok_per_xcd + p.zero_per_xcd;
  *threads_out = threads;
  return KVC_OK;
}

kvc_status launch_pack(PackParams p, hipStream_t stream) {
  if (p.n_tokens <= 0) return KVC_OK;
  int threads = 0;
  const kvc_status st = plan_pack(p, &threads);
  if (st != KVC_OK) return st;
  const Geo& g = p.g;
  const dim3 grid(p.units_per_xcd * 8u), block((unsigned)threads);
  const bool uniform = g.apt % 64 == 0;
  const size_t lds = (size_t)(p.resident ? kResidentLds : kStreamStashLoads) * threads * sizeof(u32x4);
  hipError_t err = hipSuccess;
#define KVC_LAUNCH_PACK(DT_, UNI_, RES_) err = launch_variant<DT_, UNI_, RES_>(grid, block, lds, stream, p)
  if (g.dtype == KVC_F16) {
    if (uniform) {
      if (p.resident) KVC_LAUNCH_PACK(KVC_F16, true, true); else KVC_LAUNCH_PACK(KVC_F16, true, false);
    } else {
      if (p.resident) KVC_LAUNCH_PACK(KVC_F16, false, true); else KVC_LAUNCH_PACK(KVC_F16, false, false);
    }
  } else {
    if (uniform) {
      if (p.resident) KVC_LAUNCH_PACK(KVC_BF16, true, true); else KVC_LAUNCH_PACK(KVC_BF16, true, false);
    } else {
      if (p.resident) KVC_LAUNCH_PACK(KVC_BF16, false, true); else KVC_LAUNCH_PACK(KVC_BF16, false, false);
    }
  }
#undef KVC_LAUNCH_PACK
  return err == hipSuccess ? KVC_OK : KVC_ERR_RUNTIME;
}

}  // namespace kvc
